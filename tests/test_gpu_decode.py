"""Token-sharded KV-cache decode: the newest token's query row against every cached kv shard
(Cost Optimizations appendix, "Caching"), element-wise against the oracle, then the merge through
cascade_lse_merge with a one-row plan."""
import numpy as np
import pytest

from cascade_inputs import bf16_bits, make_assignment, round_to_bf16
from oracle import cascade_oracle as orc

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


@pytest.fixture(scope="module")
def cas():
    import torch
    assert torch.cuda.is_available()
    import paper_2507_05228_amd as cas
    cas.load_library()
    return cas


def build_cache(rng, dtype, B, H, Hkv, d, lens, cap, amp=1.0):
    """Random q and per-shard caches; rows past a shard's length hold a large sentinel that must never be read into
    a result."""
    S = lens.shape[1]
    q = amp * rng.standard_normal((B, H, d))
    kc = np.full((B, Hkv, S, cap, d), 777.0)
    vc = np.full((B, Hkv, S, cap, d), -777.0)
    for b in range(B):
        for k in range(S):
            L = lens[b, k]
            kc[b, :, k, :L] = amp * rng.standard_normal((Hkv, L, d))
            vc[b, :, k, :L] = rng.standard_normal((Hkv, L, d))
    if dtype == "bf16":
        q, kc, vc = (round_to_bf16(t.astype(np.float32)).astype(np.float64) for t in (q, kc, vc))
    else:
        q, kc, vc = (t.astype(np.float32).astype(np.float64) for t in (q, kc, vc))
    return q, kc, vc


def run_case(cas, dtype, B, H, Hkv, d, lens, cap, u_mode="unnorm", amp=1.0, seed=0):
    import torch
    rng = np.random.default_rng(seed)
    lens = np.asarray(lens, dtype=np.int32).reshape(B, -1)
    S = lens.shape[1]
    q, kc, vc = build_cache(rng, dtype, B, H, Hkv, d, lens, cap, amp)
    qd, kd, vd = (cas.to_device(t, dtype) for t in (q, kc, vc))
    ld = torch.from_numpy(lens).cuda()
    m = torch.full((B, H, S), 7.0, dtype=torch.float32, device="cuda")
    e = torch.full((B, H, S), 7.0, dtype=torch.float32, device="cuda")
    u = torch.full((B, S, H, d), 7.0, dtype=torch.float32, device="cuda")
    scale = d ** -0.5
    mode = cas.U_UNNORMALISED if u_mode == "unnorm" else cas.U_NORMALISED
    cas.cascade_decode_partial_attn(qd, kd, vd, ld, m, e, u, scale, u_mode=mode)
    torch.cuda.synchronize()
    refs = [orc.decode_partials(q[b], [kc[b, :, k, :lens[b, k]] for k in range(S)],
                                [vc[b, :, k, :lens[b, k]] for k in range(S)], scale) for b in range(B)]
    m_r = np.stack([r[0] for r in refs]); e_r = np.stack([r[1] for r in refs]); u_r = np.stack([r[2] for r in refs])
    mg, eg, ug = (t.cpu().numpy().astype(np.float64) for t in (m, e, u))
    dead = ~np.isfinite(m_r)
    assert np.array_equal(~np.isfinite(mg), dead)
    assert (mg[dead] == -np.inf).all() and (eg[dead] == 0).all()
    tol_stat = 1e-5 if dtype == "f32" else 1e-4
    assert (np.abs(mg[~dead] - m_r[~dead]) / np.maximum(1.0, np.abs(m_r[~dead]))).max() < tol_stat
    assert (np.abs(eg - e_r) / np.maximum(1.0, e_r)).max() < tol_stat
    want_u = u_r if u_mode == "norm" else e_r.transpose(0, 2, 1)[..., None] * u_r
    assert np.abs(ug - want_u).max() / max(np.abs(want_u).max(), 1e-300) < TOL[dtype]
    assert (ug[dead.transpose(0, 2, 1)] == 0).all()
    # merge through the prefill merge with a one-row plan (bf16: the head dims the prefill path is built for)
    if u_mode == "unnorm" and (dtype == "f32" or d in (64, 128)):
        plan = cas.cascade_plan_create(B, 1, S, np.array([0], dtype=np.int32))
        o = torch.empty((B, 1, H * d), dtype=qd.dtype, device="cuda")
        cas.cascade_lse_merge(plan, m.view(B, H, S, 1), e.view(B, H, S, 1), u.view(B, S, H, 1, d), o, H, Hkv, d,
                              row_layout=cas.ROWS_PACKED)
        torch.cuda.synchronize()
        o_ref = np.stack([orc.decode_merge(*r) for r in refs])
        got = o.float().cpu().numpy().astype(np.float64).reshape(B, H * d)
        live = np.isfinite(m_r).any(axis=2)                    # heads with at least one cached key
        if live.any():
            err = np.abs(got - o_ref).reshape(B, H, d)[live].max() / max(np.abs(o_ref).max(), 1e-300)
            assert err < TOL[dtype]
    return mg, eg, ug


@pytest.mark.parametrize("dtype,H,Hkv,d", [
    ("f32", 4, 4, 16), ("f32", 6, 2, 32), ("f32", 8, 1, 64), ("f32", 2, 1, 256), ("f32", 3, 3, 4),
    ("bf16", 8, 2, 128), ("bf16", 4, 4, 64), ("bf16", 8, 1, 128), ("bf16", 4, 2, 64), ("bf16", 6, 2, 128),
    ("bf16", 2, 2, 8), ("bf16", 2, 1, 512), ("bf16", 12, 2, 64),
])
def test_decode_partials_match_oracle(cas, dtype, H, Hkv, d):
    lens = [[37, 0, 128, 1, 64, 100], [5, 128, 0, 0, 77, 3]]       # ragged, empty and full shards
    run_case(cas, dtype, 2, H, Hkv, d, lens, 128, seed=H * d)


@pytest.mark.parametrize("dtype,d", [("f32", 16), ("bf16", 128)])
def test_decode_normalised_mode_and_large_logits(cas, dtype, d):
    run_case(cas, dtype, 1, 4, 2, d, [[50, 9, 300, 17]], 300, u_mode="norm", seed=3)
    run_case(cas, dtype, 1, 4, 2, d, [[50, 9, 300, 17]], 300, u_mode="unnorm", amp=6.0, seed=4)


def test_decode_equals_last_row_of_prefill_partials(cas):
    """Same sequence, same sharding: decode of the newest token == row N-1 of cascade_partial_attn."""
    import torch
    B, H, Hkv, N, d, beta = 1, 8, 2, 300, 128, 5
    rng = np.random.default_rng(5)
    q = round_to_bf16(rng.standard_normal((B, H, N, d)).astype(np.float32))
    k = round_to_bf16(rng.standard_normal((B, Hkv, N, d)).astype(np.float32))
    v = round_to_bf16(rng.standard_normal((B, Hkv, N, d)).astype(np.float32))
    a = make_assignment("ragged", N, beta, 2)
    plan = cas.cascade_plan_create(B, N, beta, a)
    qd, kd, vd = (cas.to_device(t, "bf16") for t in (q, k, v))
    m = torch.empty((B, H, beta, N), dtype=torch.float32, device="cuda")
    e = torch.empty_like(m)
    u = torch.empty((B, beta, H, N, d), dtype=torch.float32, device="cuda")
    ws = cas.new_workspace(cas.cascade_partial_attn_workspace_bytes(plan, qd, H, Hkv, d))
    cas.cascade_partial_attn(plan, qd, kd, vd, m, e, u, H, Hkv, d, d ** -0.5, row_layout=cas.ROWS_ORIGINAL, workspace=ws)
    lists = orc.shard_index_lists(a, beta)
    _, _, inv = orc.shard_plan(a, beta)
    cap = max(len(S) for S in lists)
    kc = np.zeros((B, Hkv, beta, cap, d), dtype=np.float32)
    vc = np.zeros_like(kc)
    for kk, S in enumerate(lists):
        kc[:, :, kk, :len(S)] = k[:, :, S]
        vc[:, :, kk, :len(S)] = v[:, :, S]
    lens = torch.tensor([[len(S) for S in lists]], dtype=torch.int32, device="cuda")
    md = torch.empty((B, H, beta), dtype=torch.float32, device="cuda")
    ed = torch.empty_like(md)
    ud = torch.empty((B, beta, H, d), dtype=torch.float32, device="cuda")
    cas.cascade_decode_partial_attn(cas.to_device(q[:, :, N - 1], "bf16"), cas.to_device(kc, "bf16"),
                                    cas.to_device(vc, "bf16"), lens, md, ed, ud, d ** -0.5)
    torch.cuda.synchronize()
    r = int(inv[N - 1])
    assert torch.allclose(md, m[:, :, :, r], rtol=1e-5, atol=1e-5)
    assert torch.allclose(ed, e[:, :, :, r], rtol=1e-4, atol=1e-5)
    ref_u = u[:, :, :, r]
    assert (ud - ref_u).abs().max() / ref_u.abs().max() < 2e-2


def test_decode_error_paths(cas):
    import torch
    q = torch.zeros(1, 4, 64, dtype=torch.bfloat16, device="cuda")
    kc = torch.zeros(1, 2, 3, 16, 64, dtype=torch.bfloat16, device="cuda")
    lens = torch.zeros(1, 3, dtype=torch.int32, device="cuda")
    m = torch.zeros(1, 4, 3, device="cuda"); u = torch.zeros(1, 3, 4, 64, device="cuda")
    with pytest.raises(cas.CascadeError) as ei:
        cas.cascade_decode_partial_attn(q, kc, kc, lens, m, m.clone(), None, 0.125)
    assert ei.value.status == cas.EINVAL
    kc3 = torch.zeros(1, 3, 3, 16, 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(cas.CascadeError) as ei:                              # H % H_KV != 0
        cas.cascade_decode_partial_attn(q, kc3, kc3, lens, m, m.clone(), u, 0.125)
    assert ei.value.status == cas.ESHAPE
    q48 = torch.zeros(1, 4, 48, dtype=torch.bfloat16, device="cuda")
    kc48 = torch.zeros(1, 2, 3, 16, 48, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(cas.CascadeError) as ei:                              # 48 is not 8 * 2^j
        cas.cascade_decode_partial_attn(q48, kc48, kc48, lens, m, m.clone(), torch.zeros(1, 3, 4, 48, device="cuda"), 0.125)
    assert ei.value.status == cas.EUNSUPPORTED


# ---------------------------------------------------------------- prefill -> cache -> one decode step
def _small_llama(dtype, d):
    from cascade_inputs import CONFIGS
    return CONFIGS["C3"].with_(name=f"decode-llama-{dtype}-{d}", dtype=dtype, d_model=256, n_heads=4, n_kv_heads=2,
                               head_dim=d, d_ff=512, batch=2, seq_len=199, n_shards=5, index=51)


@pytest.mark.parametrize("dtype,d,kind", [("bf16", 64, "perm"), ("bf16", 128, "ragged"), ("f32", 32, "roundrobin")])
def test_prefill_cache_then_decode_step_is_the_last_row_of_the_longer_sequence(cas, dtype, d, kind):
    """Layer forward on the first N tokens, its k, v moved into the per-shard cache, then the token N composed from
    the entry points (norm, q/k/v shard GEMM with rotary at position N, append, per-shard partials, merge, o
    projection + residual, norm, FFN): equals row N of the unsharded layer on N + 1 tokens."""
    import torch
    from cascade_inputs import make_hidden, make_layer_weights
    cfg = _small_llama(dtype, d)
    N, B, beta = cfg.seq_len, cfg.batch, cfg.n_shards
    H, Hkv, D = cfg.n_heads, cfg.n_kv_heads, cfg.d_model
    w = make_layer_weights(cfg)
    h_full = make_hidden(cfg.with_(seq_len=N + 1))                        # [B, N + 1, D]
    a_full = make_assignment(kind, N + 1, beta, 5)
    a, j_new = a_full[:N], int(a_full[N])
    tol = TOL[dtype]

    # prefill of the first N tokens
    plan = cas.cascade_plan_create(B, N, beta, a)
    desc = cas.make_layer_desc(cfg, cas.ATTN_FUSED)
    t = {k: cas.to_device(v, dtype) for k, v in w.items()}
    wts = cas.make_layer_weights(t)
    h_in = cas.to_device(h_full[:, :N], dtype)
    h_out = torch.empty_like(h_in)
    ws = cas.new_workspace(cas.cascade_layer_workspace_bytes(plan, desc))
    cas.cascade_layer_forward(plan, desc, wts, h_in, h_out, ws)
    sizes = np.bincount(a, minlength=beta)
    cap = int(sizes.max()) + 3
    kc = torch.full((B, Hkv, beta, cap, d), 768.0, dtype=h_in.dtype, device="cuda")
    vc = torch.full((B, Hkv, beta, cap, d), -768.0, dtype=h_in.dtype, device="cuda")
    lens = torch.full((B, beta), -1, dtype=torch.int32, device="cuda")
    cas.cascade_layer_kv_to_cache(plan, desc, ws, kc, vc, lens)
    torch.cuda.synchronize()
    assert np.array_equal(lens.cpu().numpy(), np.tile(sizes, (B, 1)))
    # cache content = the oracle's pre-pass k, v of every shard (rotary at the tokens' own positions)
    lists = orc.shard_index_lists(a, beta)
    w64 = {k: v.astype(np.float64) for k, v in w.items()}
    for b in range(B):
        for k, R in enumerate(lists):
            _, k_ref, v_ref = orc.pre_pass(h_full[b, R].astype(np.float64), R, w64, cfg)
            got_k = kc[b, :, k, :len(R)].float().cpu().numpy()
            got_v = vc[b, :, k, :len(R)].float().cpu().numpy()
            assert np.abs(got_k - k_ref).max() < tol * max(np.abs(k_ref).max(), 1)
            assert np.abs(got_v - v_ref).max() < tol * max(np.abs(v_ref).max(), 1)
    assert float(kc[:, :, 0, sizes[0]:].float().min()) == 768.0            # rows past a shard's size untouched

    # token N
    nk = cas.NORM_RMSNORM
    hn = cas.to_device(h_full[:, N], dtype)                               # [B, D]
    x = torch.empty_like(hn)
    cas.cascade_norm(hn, t["norm1_g"], None, x, nk, cfg.eps)
    wqkv = torch.cat([t["wq"], t["wk"], t["wv"]], dim=0).contiguous()
    QW = (H + 2 * Hkv) * d
    qkv = torch.empty(B, QW, dtype=hn.dtype, device="cuda")
    plan_pos = cas.cascade_plan_create(B, 1, 1, np.zeros(1, np.int32), positions=np.array([N], np.int32))
    cas.cascade_shard_gemm(plan_pos, x, wqkv, qkv, epilogue=cas.EPI_ROPE, rope_cols=(H + Hkv) * d, head_dim=d,
                           rope_theta=cfg.rope_theta)
    q = qkv[:, :H * d].reshape(B, H, d).contiguous()
    kc[:, :, j_new, sizes[j_new]] = qkv[:, H * d:(H + Hkv) * d].reshape(B, Hkv, d)
    vc[:, :, j_new, sizes[j_new]] = qkv[:, (H + Hkv) * d:].reshape(B, Hkv, d)
    lens[:, j_new] += 1
    m = torch.empty(B, H, beta, dtype=torch.float32, device="cuda")
    e = torch.empty_like(m)
    u = torch.empty(B, beta, H, d, dtype=torch.float32, device="cuda")
    cas.cascade_decode_partial_attn(q, kc, vc, lens, m, e, u, cfg.scale)
    plan1 = cas.cascade_plan_create(B, 1, beta, np.array([j_new], np.int32))
    o = torch.empty(B, 1, H * d, dtype=hn.dtype, device="cuda")
    cas.cascade_lse_merge(plan1, m.view(B, H, beta, 1), e.view(B, H, beta, 1), u.view(B, beta, H, 1, d), o, H, Hkv, d)
    h1 = torch.empty_like(hn)
    cas.cascade_shard_gemm(None, o.view(B, H * d), t["wo"], h1, residual=hn, epilogue=cas.EPI_RESIDUAL)
    x2 = torch.empty_like(hn)
    cas.cascade_norm(h1, t["norm2_g"], None, x2, nk, cfg.eps)
    act = torch.empty(B, cfg.d_ff, dtype=hn.dtype, device="cuda")
    cas.cascade_shard_gemm(None, x2, t["w_gate"], act, W_up=t["w_up"], epilogue=cas.EPI_SWIGLU)
    out = torch.empty_like(hn)
    cas.cascade_shard_gemm(None, act, t["w_down"], out, residual=h1, epilogue=cas.EPI_RESIDUAL)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    for b in range(B):
        want = orc.layer_direct(h_full[b], w, cfg, rows=np.array([N]))[0]
        assert np.abs(got[b] - want).max() / np.abs(want).max() < tol


def test_cache_from_a_prefill_with_distinct_row_and_kv_shardings(cas):
    """Row shards R (5) and key/value shards S = their 2-split (10): the cache slabs follow S."""
    import torch
    from cascade_inputs import make_hidden, make_layer_weights
    cfg = _small_llama("bf16", 64)
    N, B, alpha = cfg.seq_len, cfg.batch, cfg.n_shards
    a = make_assignment("perm", N, alpha, 8)
    a_kv = orc.m_split_assignment(a, alpha, 2)
    beta = 2 * alpha
    w, h = make_layer_weights(cfg), make_hidden(cfg)
    plan = cas.cascade_plan_create_rs(B, N, alpha, a, beta, a_kv)
    desc = cas.make_layer_desc(cfg, cas.ATTN_FUSED)
    t = {k: cas.to_device(v, "bf16") for k, v in w.items()}
    h_in = cas.to_device(h, "bf16")
    h_out = torch.empty_like(h_in)
    ws = cas.new_workspace(cas.cascade_layer_workspace_bytes(plan, desc))
    cas.cascade_layer_forward(plan, desc, cas.make_layer_weights(t), h_in, h_out, ws)
    sizes = np.bincount(a_kv, minlength=beta)
    cap = int(sizes.max())
    kc = torch.zeros((B, cfg.n_kv_heads, beta, cap, 64), dtype=h_in.dtype, device="cuda")
    vc = torch.zeros_like(kc)
    lens = torch.zeros((B, beta), dtype=torch.int32, device="cuda")
    cas.cascade_layer_kv_to_cache(plan, desc, ws, kc, vc, lens)
    torch.cuda.synchronize()
    assert np.array_equal(lens.cpu().numpy(), np.tile(sizes, (B, 1)))
    w64 = {k: v.astype(np.float64) for k, v in w.items()}
    for b in range(B):
        for k, S in enumerate(orc.shard_index_lists(a_kv, beta)):
            _, k_ref, v_ref = orc.pre_pass(h[b, S].astype(np.float64), S, w64, cfg)
            assert np.abs(kc[b, :, k, :len(S)].float().cpu().numpy() - k_ref).max() < TOL["bf16"] * max(np.abs(k_ref).max(), 1)
            assert np.abs(vc[b, :, k, :len(S)].float().cpu().numpy() - v_ref).max() < TOL["bf16"] * max(np.abs(v_ref).max(), 1)
    # a capacity below the largest shard is refused
    small = torch.zeros((B, cfg.n_kv_heads, beta, cap - 1, 64), dtype=h_in.dtype, device="cuda")
    with pytest.raises(cas.CascadeError) as ei:
        cas.cascade_layer_kv_to_cache(plan, desc, ws, small, small.clone(), lens)
    assert ei.value.status == cas.ESHAPE
