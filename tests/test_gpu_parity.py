"""Parity of the HIP library (through the C-ABI binding) against the float64 CPU oracle on the same
seeded inputs.  Tolerances: max|gpu - ref| / max|ref| per tensor <= 1e-5 (fp32) or 2e-2 (bf16 with
fp32 accumulation); shard maps bit-exact."""
import numpy as np
import pytest

from cascade_inputs import CONFIGS, make_assignment, make_hidden, make_layer_weights, round_to_bf16
from oracle import cascade_oracle as orc

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


@pytest.fixture(scope="module")
def cas():
    import torch
    assert torch.cuda.is_available()
    import paper_2507_05228_amd as cas
    cas.load_library()          # raises if the HIP library is missing: no fallback
    return cas


def rel_err(g, r):
    return float(np.abs(np.asarray(g, dtype=np.float64) - r).max() / max(np.abs(r).max(), 1e-300))


def dev(cas, x, dtype):
    return cas.to_device(x, dtype)


def host(t):
    return t.float().cpu().numpy().astype(np.float64)


def rand(rng, shape, dtype, std=1.0):
    x = (rng.standard_normal(shape) * std).astype(np.float32)
    return round_to_bf16(x) if dtype == "bf16" else x


# ---------------------------------------------------------------------------- plan
@pytest.mark.parametrize("kind,N,beta", [("perm", 128, 4), ("contiguous", 1024, 8), ("roundrobin", 512, 64),
                                         ("ragged", 333, 7), ("ragged", 40, 16), ("perm", 2048, 16)])
def test_plan_maps_bit_exact(cas, kind, N, beta):
    a = make_assignment(kind, N, beta, 5)
    plan = cas.cascade_plan_create(2, N, beta, a)
    off_r, perm_r, inv_r = orc.shard_plan(a, beta)
    perm_h, inv_h, off_h = cas.cascade_plan_maps_host(plan)
    perm_d, inv_d, off_d = (t.cpu().numpy() for t in cas.cascade_plan_maps(plan))
    for got in (perm_h, perm_d):
        assert got.dtype == np.int32 and np.array_equal(got, perm_r)
    for got in (inv_h, inv_d):
        assert np.array_equal(got, inv_r)
    for got in (off_h, off_d):
        assert np.array_equal(got, off_r)


def test_plan_error_paths(cas):
    a = np.zeros(16, dtype=np.int32)
    with pytest.raises(cas.CascadeError) as ei:
        bad = a.copy(); bad[3] = 4
        cas.cascade_plan_create(1, 16, 4, bad)
    assert ei.value.status == cas.EASSIGN
    with pytest.raises(cas.CascadeError) as ei:
        bad = a.copy(); bad[0] = -1
        cas.cascade_plan_create(1, 16, 4, bad)
    assert ei.value.status == cas.EASSIGN
    for args in ((0, 16, 4), (1, 16, 0)):
        with pytest.raises(cas.CascadeError) as ei:
            cas.cascade_plan_create(*args, a)
        assert ei.value.status == cas.EINVAL
    with pytest.raises(cas.CascadeError) as ei:
        cas.cascade_plan_create(1, 16, 4, a, mask_kind=7)
    assert ei.value.status == cas.EINVAL


# ---------------------------------------------------------------------------- shard GEMM
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M_N_K", [(128, 192, 64), (300, 200, 136), (512, 1000, 264), (40, 24, 8)])
def test_shard_gemm_plain(cas, dtype, M_N_K):
    import torch
    M, N, K = M_N_K
    rng = np.random.default_rng(M + N + K)
    x, w = rand(rng, (M, K), dtype), rand(rng, (N, K), dtype, 0.1)
    X, W = dev(cas, x, dtype), dev(cas, w, dtype)
    Y = torch.empty(M, N, dtype=X.dtype, device="cuda")
    cas.cascade_shard_gemm(None, X, W, Y)
    ref = orc.linear(x.astype(np.float64), w.astype(np.float64))
    assert rel_err(host(Y), ref) < TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_shard_gemm_gather_bias_gelu_and_scatter_residual(cas, dtype):
    import torch
    B, N, beta, K, F = 2, 200, 5, 72, 328
    rng = np.random.default_rng(3)
    a = make_assignment("ragged", N, beta, 11)
    plan = cas.cascade_plan_create(B, N, beta, a)
    _, perm, _ = orc.shard_plan(a, beta)
    x = rand(rng, (B * N, K), dtype)
    w1, b1 = rand(rng, (F, K), dtype, 0.2), rand(rng, (F,), dtype, 0.2)
    w2, b2 = rand(rng, (K, F), dtype, 0.1), rand(rng, (K,), dtype, 0.2)
    X, W1, B1, W2, B2 = (dev(cas, t, dtype) for t in (x, w1, b1, w2, b2))
    # gather original rows into packed order, bias + GELU
    H1 = torch.empty(B * N, F, dtype=X.dtype, device="cuda")
    cas.cascade_shard_gemm(plan, X, W1, H1, bias=B1, epilogue=cas.EPI_BIAS | cas.EPI_GELU_ERF,
                           x_rows=cas.ROWS_ORIGINAL)
    rows = np.concatenate([b * N + perm for b in range(B)])
    x64 = x.astype(np.float64)
    ref1 = orc.gelu_erf(orc.linear(x64[rows], w1.astype(np.float64), b1.astype(np.float64)))
    assert rel_err(host(H1), ref1) < TOL[dtype]
    # packed rows in, residual gathered from original order, result scattered back to original order
    Y = torch.zeros(B * N, K, dtype=X.dtype, device="cuda")
    cas.cascade_shard_gemm(plan, H1, W2, Y, bias=B2, residual=X, epilogue=cas.EPI_BIAS | cas.EPI_RESIDUAL,
                           y_rows=cas.ROWS_ORIGINAL, res_rows=cas.ROWS_ORIGINAL)
    h1 = host(H1)
    ref2 = np.empty((B * N, K))
    ref2[rows] = x64[rows] + orc.linear(h1, w2.astype(np.float64), b2.astype(np.float64))
    assert rel_err(host(Y), ref2) < TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_shard_gemm_swiglu_and_tanh(cas, dtype):
    import torch
    M, K, F = 260, 136, 200
    rng = np.random.default_rng(4)
    x, wg, wu = rand(rng, (M, K), dtype), rand(rng, (F, K), dtype, 0.2), rand(rng, (F, K), dtype, 0.2)
    X, WG, WU = (dev(cas, t, dtype) for t in (x, wg, wu))
    Y = torch.empty(M, F, dtype=X.dtype, device="cuda")
    cas.cascade_shard_gemm(None, X, WG, Y, W_up=WU, epilogue=cas.EPI_SWIGLU)
    x64 = x.astype(np.float64)
    ref = orc.silu(orc.linear(x64, wg.astype(np.float64))) * orc.linear(x64, wu.astype(np.float64))
    assert rel_err(host(Y), ref) < TOL[dtype]
    cas.cascade_shard_gemm(None, X, WG, Y, epilogue=cas.EPI_GELU_TANH)
    assert rel_err(host(Y), orc.gelu_tanh(orc.linear(x64, wg.astype(np.float64)))) < TOL[dtype]


# One shape per tile variant of the bf16 MFMA kernels (8 wavefronts at 192 / 224 / 256 columns, one wavefront per
# SIMD at 192 / 224 and for SwiGLU at 224 / 256, the 256x128 ping-pong kernel), chosen with the launcher's own cost
# rule on 256 CUs; ragged M and N, bias + GELU or residual, every output element against the oracle.  The last three
# shapes have 11 and 18 rows of tiles: the tile order then runs in groups of 8 rows of tiles with a shorter last group.
@pytest.mark.parametrize("M,N,swiglu", [(700, 1000, False), (700, 1000, True), (700, 9600, True), (700, 13728, False),
                                        (1000, 12352, False), (1000, 14416, False), (1300, 10804, False),
                                        (2000, 12352, False), (40, 448, True), (1, 1000, True), (3, 5000, False),
                                        (2700, 6000, False), (2700, 9600, True), (4500, 2100, False)])
@pytest.mark.parametrize("epi", ["plain", "bias_gelu", "residual"])
def test_shard_gemm_every_mfma_tile_variant(cas, M, N, swiglu, epi):
    import torch
    if swiglu and epi == "bias_gelu":
        pytest.skip("SwiGLU launches carry no bias or GELU")
    K = 192
    rng = np.random.default_rng(M + N)
    x, w = rand(rng, (M, K), "bf16"), rand(rng, (N, K), "bf16", 0.2)
    x64, w64 = x.astype(np.float64), w.astype(np.float64)
    X, W = dev(cas, x, "bf16"), dev(cas, w, "bf16")
    Y = torch.full((M, N), 7.0, dtype=X.dtype, device="cuda")
    kw, ep = {}, 0
    ref = orc.linear(x64, w64)
    if swiglu:
        wu = rand(rng, (N, K), "bf16", 0.2)
        kw["W_up"] = dev(cas, wu, "bf16")
        ep |= cas.EPI_SWIGLU
        ref = orc.silu(ref) * orc.linear(x64, wu.astype(np.float64))
    if epi == "bias_gelu":
        b = rand(rng, (N,), "bf16", 0.3)
        kw["bias"] = dev(cas, b, "bf16")
        ep |= cas.EPI_BIAS | cas.EPI_GELU_ERF
        ref = orc.gelu_erf(ref + b.astype(np.float64))
    if epi == "residual":
        r = rand(rng, (M, N), "bf16")
        kw["residual"] = dev(cas, r, "bf16")
        ep |= cas.EPI_RESIDUAL
        ref = ref + r.astype(np.float64)
    cas.cascade_shard_gemm(None, X, W, Y, epilogue=ep, **kw)
    assert rel_err(host(Y), ref) < TOL["bf16"]


@pytest.mark.parametrize("epi", ["plain", "bias", "bias_residual"])
def test_shard_gemm_256_wide_tiles_one_wavefront_per_simd(cas, epi):
    """Several rounds of 256 x 256 tiles over a long reduction (the o projection / FFN down of a long prefill):
    the launcher then takes the one-wavefront schedule with 256 accumulator registers.  Ragged M and N."""
    import torch
    M, N, K = 8000, 4000, 2048
    rng = np.random.default_rng(77)
    x, w = rand(rng, (M, K), "bf16"), rand(rng, (N, K), "bf16", 0.05)
    X, W = dev(cas, x, "bf16"), dev(cas, w, "bf16")
    ref = orc.linear(x.astype(np.float64), w.astype(np.float64))
    kw, ep = {}, 0
    if "bias" in epi:
        b = rand(rng, (N,), "bf16", 0.3)
        kw["bias"] = dev(cas, b, "bf16"); ep |= cas.EPI_BIAS
        ref = ref + b.astype(np.float64)
    if "residual" in epi:
        r = rand(rng, (M, N), "bf16")
        kw["residual"] = dev(cas, r, "bf16"); ep |= cas.EPI_RESIDUAL
        ref = ref + r.astype(np.float64)
    Y = torch.full((M, N), 7.0, dtype=X.dtype, device="cuda")
    cas.cascade_shard_gemm(None, X, W, Y, epilogue=ep, **kw)
    assert rel_err(host(Y), ref) < TOL["bf16"]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_shard_gemm_rope_uses_original_positions(cas, dtype):
    import torch
    B, N, beta, K, H, d = 1, 96, 3, 64, 3, 32
    rng = np.random.default_rng(5)
    a = make_assignment("perm", N, beta, 2)
    pos = rng.permutation(4 * N)[:N].astype(np.int32)         # arbitrary positions
    plan = cas.cascade_plan_create(B, N, beta, a, positions=pos)
    _, perm, _ = orc.shard_plan(a, beta)
    x, w = rand(rng, (N, K), dtype), rand(rng, ((H + 1) * d, K), dtype, 0.2)
    X, W = dev(cas, x, dtype), dev(cas, w, dtype)
    Y = torch.empty(N, (H + 1) * d, dtype=X.dtype, device="cuda")
    cas.cascade_shard_gemm(plan, X, W, Y, epilogue=cas.EPI_ROPE, x_rows=cas.ROWS_ORIGINAL, rope_cols=H * d,
                           head_dim=d, rope_theta=10000.0)
    y = orc.linear(x.astype(np.float64)[perm], w.astype(np.float64))
    ref = y.copy()
    for h in range(H):
        ref[:, h * d:(h + 1) * d] = orc.rope(y[:, h * d:(h + 1) * d], pos[perm], 10000.0)
    assert rel_err(host(Y), ref) < TOL[dtype]
    assert rel_err(host(Y)[:, :H * d], y[:, :H * d]) > 0.05       # the rotation did happen


def test_shard_gemm_error_paths(cas):
    import torch
    X = torch.zeros(8, 12, dtype=torch.bfloat16, device="cuda")      # k = 12 is not a multiple of 8
    W = torch.zeros(4, 12, dtype=torch.bfloat16, device="cuda")
    Y = torch.zeros(8, 4, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(cas.CascadeError) as ei:
        cas.cascade_shard_gemm(None, X, W, Y)
    assert ei.value.status == cas.EUNSUPPORTED
    with pytest.raises(cas.CascadeError) as ei:
        cas.cascade_shard_gemm(None, X, W, Y, x_rows=cas.ROWS_ORIGINAL)     # a map needs a plan
    assert ei.value.status == cas.EINVAL
    plan = cas.cascade_plan_create(1, 16, 2, np.zeros(16, dtype=np.int32))
    with pytest.raises(cas.CascadeError) as ei:
        cas.cascade_shard_gemm(plan, X.float(), W.float(), Y.float(), x_rows=cas.ROWS_ORIGINAL)   # 8 rows != 16
    assert ei.value.status == cas.ESHAPE
    with pytest.raises(cas.CascadeError) as ei:
        cas.cascade_shard_gemm(None, X.float(), W.float(), Y.float(), epilogue=cas.EPI_BIAS)       # bias missing
    assert ei.value.status == cas.EINVAL


# ---------------------------------------------------------------------------- partial attention + merge
def attn_case(cas, dtype, B, H, Hkv, N, d, beta, kind, layout, mask_kind="causal", seed=0, positions=None, amp=1.0):
    import torch
    rng = np.random.default_rng(seed)
    q, k, v = (rand(rng, (B, H, N, d), dtype, amp), rand(rng, (B, Hkv, N, d), dtype, amp),
               rand(rng, (B, Hkv, N, d), dtype))
    a = make_assignment(kind, N, beta, seed + 1)
    plan = cas.cascade_plan_create(B, N, beta, a, positions=positions,
                                   mask_kind=cas.MASK_CAUSAL if mask_kind == "causal" else cas.MASK_NONE)
    _, perm, _ = orc.shard_plan(a, beta)
    scale = d ** -0.5
    if layout == "packed":
        qd, kd, vd = (dev(cas, t[:, :, perm], dtype) for t in (q, k, v))
        row_layout = cas.ROWS_PACKED
    else:
        qd, kd, vd = (dev(cas, t, dtype) for t in (q, k, v))
        row_layout = cas.ROWS_ORIGINAL
    m = torch.full((B, H, beta, N), 7.0, dtype=torch.float32, device="cuda")
    e = torch.full((B, H, beta, N), 7.0, dtype=torch.float32, device="cuda")
    u = torch.full((B, beta, H, N, d), 7.0, dtype=torch.float32, device="cuda")
    ws = cas.new_workspace(cas.cascade_partial_attn_workspace_bytes(plan, qd, H, Hkv, d))
    cas.cascade_partial_attn(plan, qd, kd, vd, m, e, u, H, Hkv, d, scale, row_layout=row_layout, workspace=ws)
    refs = [orc.partial_attention_all_pairs(q[b], k[b], v[b], a, beta, positions=positions, scale=scale,
                                            mask_kind=mask_kind) for b in range(B)]
    m_r = np.stack([r[0] for r in refs]); e_r = np.stack([r[1] for r in refs]); u_r = np.stack([r[2] for r in refs])
    return plan, (m, e, u), (m_r, e_r, u_r), perm


def check_partials(dtype, got, ref):
    m, e, u = (host(t) for t in got)
    m_r, e_r, u_r = ref
    dead = ~np.isfinite(m_r)
    assert np.array_equal(~np.isfinite(m), dead)
    assert (m[dead] == -np.inf).all() and (e[dead] == 0).all()
    tol_stat = 1e-5 if dtype == "f32" else 1e-4            # m, e are fp32 functions of exact bf16 inputs
    assert (np.abs(m[~dead] - m_r[~dead]) / np.maximum(1.0, np.abs(m_r[~dead]))).max() < tol_stat
    assert (np.abs(e - e_r) / np.maximum(1.0, e_r)).max() < tol_stat
    lse, lse_r = m[~dead] + np.log(e[~dead]), m_r[~dead] + np.log(e_r[~dead])
    assert (np.abs(lse - lse_r) / np.maximum(1.0, np.abs(lse_r))).max() < tol_stat
    ut_r = e_r.transpose(0, 2, 1, 3)[..., None] * u_r        # u~ = e * u, [B, beta, H, N, d]
    assert rel_err(u, ut_r) < TOL[dtype]
    assert (u[dead.transpose(0, 2, 1, 3)] == 0).all()
    # 1 <= e <= |S_k| (the stability remark's "e <= 1" is a slip).  The kernel's e is the sum relative to its
    # fp32 row maximum, which may sit half an fp32 ulp of the logit (~1e-5 relative at logits in the hundreds,
    # scaled by log2 e) above the exact one, so e may undershoot 1 by that much; m + log e is unaffected.
    assert (e[~dead] >= 1.0 - 2e-5).all()


@pytest.mark.parametrize("dtype,H,Hkv,N,d,beta,kind,layout", [
    ("f32", 4, 4, 128, 16, 4, "perm", "original"),
    ("f32", 4, 2, 100, 24, 5, "ragged", "packed"),
    ("f32", 2, 1, 70, 8, 16, "ragged", "original"),            # some shards empty
    ("bf16", 4, 4, 256, 64, 4, "perm", "original"),
    ("bf16", 8, 2, 384, 128, 3, "perm", "original"),           # GQA 4:1, 128-row shards
    ("bf16", 8, 1, 200, 128, 4, "ragged", "packed"),           # GQA 8:1, ragged tiles
    ("bf16", 2, 1, 300, 64, 7, "ragged", "original"),          # GQA 2:1
    ("bf16", 3, 3, 330, 64, 2, "contiguous", "packed"),        # MHA, shards larger than a tile
    ("bf16", 4, 1, 96, 128, 24, "ragged", "original"),         # tiny shards, some empty
    ("bf16", 4, 2, 512, 128, 8, "roundrobin", "original"),
    ("bf16", 4, 2, 48, 64, 48, "roundrobin", "original"),      # singleton shards: e = 1, u~ = the one visible v
    ("bf16", 4, 2, 130, 128, 1, "contiguous", "packed"),       # one shard: plain causal attention, ragged tail
    ("bf16", 2, 2, 1, 64, 1, "contiguous", "original"),        # a single token
    ("f32", 2, 1, 33, 16, 33, "roundrobin", "packed"),
])
def test_partial_attn_matches_oracle(cas, dtype, H, Hkv, N, d, beta, kind, layout):
    B = 2
    plan, got, ref, _ = attn_case(cas, dtype, B, H, Hkv, N, d, beta, kind, layout, seed=N + d)
    check_partials(dtype, got, ref)


@pytest.mark.parametrize("dtype,d", [("f32", 16), ("bf16", 64), ("bf16", 128)])
def test_partial_attn_no_mask_and_custom_positions(cas, dtype, d):
    plan, got, ref, _ = attn_case(cas, dtype, 1, 4, 2, 160, d, 5, "perm", "original", mask_kind="none", seed=1)
    check_partials(dtype, got, ref)
    pos = np.random.default_rng(9).permutation(1000)[:160].astype(np.int32)
    plan, got, ref, _ = attn_case(cas, dtype, 1, 4, 2, 160, d, 5, "perm", "original", seed=2, positions=pos)
    check_partials(dtype, got, ref)


@pytest.mark.parametrize("d", [64, 128])
def test_partial_attn_unordered_positions_many_tiles_per_shard(cas, d):
    """Positions that do not ascend with the token index, shards of several key/value tiles: the
    visible tiles of a query tile are then not a prefix of the shard in packed order."""
    N = 640
    pos = np.random.default_rng(11).permutation(3 * N)[:N].astype(np.int32)
    plan, got, ref, _ = attn_case(cas, "bf16", 1, 4, 2, N, d, 2, "perm", "packed", seed=5, positions=pos)
    check_partials("bf16", got, ref)
    plan, got, ref, _ = attn_case(cas, "bf16", 1, 2, 2, N, d, 3, "ragged", "original", seed=6, positions=pos)
    check_partials("bf16", got, ref)


# ---------------------------------------------------------------------------- distinct row / key-value shardings
def rs_partitions(cas, N, kind, seed):
    """(row assignment, alpha, kv assignment, beta)."""
    if kind == "msplit":                                      # (c, delta) rows, m-split key/value shards
        a, alpha = cas.cascade_cdelta_assignment(N, 8, 32)
        return a, alpha, cas.cascade_m_split(a, alpha, 2), 2 * alpha
    if kind == "msplit4":
        a, alpha = cas.cascade_cdelta_assignment(N, 4, 8)
        return a, alpha, cas.cascade_m_split(a, alpha, 4), 4 * alpha
    if kind == "coarser":                                     # key/value shards = unions of row shards
        a = make_assignment("perm", N, 6, seed)
        return a, 6, (a // 2).astype(np.int32), 3
    a = make_assignment("ragged", N, 4, seed)                 # unrelated partitions
    return a, 4, make_assignment("perm", N, 5, seed + 1), 5


@pytest.mark.parametrize("kind", ["msplit", "coarser", "unrelated"])
def test_plan_with_two_shardings_maps_bit_exact(cas, kind):
    N = 200
    a, alpha, kv, beta = rs_partitions(cas, N, kind, 3)
    plan = cas.cascade_plan_create_rs(2, N, alpha, a, beta, kv)
    off_r, perm_r, inv_r = orc.shard_plan(a, alpha)
    off_s, perm_s, _ = orc.shard_plan(kv, beta)
    perm, inv, off = cas.cascade_plan_maps_host(plan)
    assert np.array_equal(perm, perm_r) and np.array_equal(inv, inv_r) and np.array_equal(off, off_r)
    n, kperm, koff, k2r = cas.cascade_plan_kv_maps_host(plan)
    assert n == beta and np.array_equal(kperm, perm_s) and np.array_equal(koff, off_s)
    assert np.array_equal(k2r, inv_r[perm_s])
    single = cas.cascade_plan_create(2, N, alpha, a)
    n1, kperm1, koff1, k2r1 = cas.cascade_plan_kv_maps_host(single)      # one partition: kv maps are the row maps
    assert n1 == alpha and np.array_equal(kperm1, perm_r) and np.array_equal(koff1, off_r) and k2r1 is None


@pytest.mark.parametrize("dtype,H,Hkv,N,d,kind,layout", [
    ("f32", 4, 2, 96, 16, "msplit", "original"),
    ("f32", 2, 2, 70, 8, "unrelated", "packed"),
    ("bf16", 4, 2, 512, 128, "msplit", "packed"),             # 4 row shards of 128, 8 kv shards of 64 keys
    ("bf16", 8, 2, 384, 128, "coarser", "original"),          # kv shards of 128 keys span two row shards
    ("bf16", 4, 4, 300, 64, "unrelated", "packed"),
    ("bf16", 4, 1, 256, 64, "msplit4", "original"),
])
def test_partial_attn_with_two_shardings_matches_oracle(cas, dtype, H, Hkv, N, d, kind, layout):
    """Query rows follow the row sharding R, key/value shards the sharding S (Section 5.1, m-split of
    Section 6.4): m, e, u~ per (R-packed row, kv shard), then the merge over the kv shards."""
    import torch
    B = 2
    rng = np.random.default_rng(N + d)
    q, k, v = rand(rng, (B, H, N, d), dtype), rand(rng, (B, Hkv, N, d), dtype), rand(rng, (B, Hkv, N, d), dtype)
    a, alpha, kv, beta = rs_partitions(cas, N, kind, 7)
    plan = cas.cascade_plan_create_rs(B, N, alpha, a, beta, kv)
    _, perm, _ = orc.shard_plan(a, alpha)
    scale = d ** -0.5
    if layout == "packed":
        qd, kd, vd = (dev(cas, t[:, :, perm], dtype) for t in (q, k, v))
        row_layout = cas.ROWS_PACKED
    else:
        qd, kd, vd = (dev(cas, t, dtype) for t in (q, k, v))
        row_layout = cas.ROWS_ORIGINAL
    m = torch.full((B, H, beta, N), 7.0, dtype=torch.float32, device="cuda")
    e = torch.full((B, H, beta, N), 7.0, dtype=torch.float32, device="cuda")
    u = torch.full((B, beta, H, N, d), 7.0, dtype=torch.float32, device="cuda")
    ws = cas.new_workspace(cas.cascade_partial_attn_workspace_bytes(plan, qd, H, Hkv, d))
    cas.cascade_partial_attn(plan, qd, kd, vd, m, e, u, H, Hkv, d, scale, row_layout=row_layout, workspace=ws)
    refs = [orc.partial_attention_rs(q[b], k[b], v[b], a, alpha, kv, beta, scale=scale) for b in range(B)]
    ref = tuple(np.stack([r[i] for r in refs]) for i in range(3))
    check_partials(dtype, (m, e, u), ref)
    # merge over the beta key/value shards: plain attention in R-packed rows
    o = torch.empty((B, N, H * d), dtype=qd.dtype, device="cuda")
    cas.cascade_lse_merge(plan, m, e, u, o, H, Hkv, d, row_layout=cas.ROWS_PACKED)
    o_ref = np.stack([orc.lse_merge_all(*r) for r in refs])
    assert rel_err(host(o), o_ref) < TOL[dtype]


@pytest.mark.parametrize("cfg_name,kind", [("small-llama", "msplit"), ("small-llama", "unrelated"),
                                           ("f32-llama", "coarser"), ("small-gpt", "msplit")])
@pytest.mark.parametrize("mode", ["fused", "materialised"])
def test_layer_forward_with_two_shardings(cas, cfg_name, kind, mode):
    cfg = {"small-llama": SMALL_LLAMA, "f32-llama": F32_LLAMA, "small-gpt": SMALL_GPT}[cfg_name]
    attn_mode = cas.ATTN_FUSED if mode == "fused" else cas.ATTN_MATERIALISED
    a, alpha, kv, beta = rs_partitions(cas, cfg.seq_len, kind, 13)
    w, h = make_layer_weights(cfg), make_hidden(cfg)
    out = cas.layer_forward_numpy(cfg.with_(n_shards=alpha), w, h, a, attn_mode=attn_mode, token_to_kv_shard=kv)
    ref = orc.layer_direct_batch(h, w, cfg)
    assert rel_err(out, ref) < TOL[cfg.dtype]
    if mode == "materialised" and cfg_name == "small-llama" and kind == "msplit":
        ref_rs = np.stack([orc.layer_sharded_rs(h[b], w, cfg, a, alpha, kv, beta) for b in range(cfg.batch)])
        assert rel_err(out, ref_rs) < TOL[cfg.dtype]


@pytest.mark.parametrize("dtype,d", [("f32", 32), ("bf16", 128)])
def test_partial_attn_large_logits_are_stable(cas, dtype, d):
    plan, got, ref, _ = attn_case(cas, dtype, 1, 2, 2, 128, d, 4, "perm", "original", seed=3, amp=6.0)
    assert np.abs(ref[0][np.isfinite(ref[0])]).max() > 100
    check_partials(dtype, got, ref)


@pytest.mark.parametrize("dtype,d,u_mode", [("f32", 16, "norm"), ("bf16", 128, "norm"), ("f32", 20, "unnorm"),
                                            ("bf16", 64, "unnorm")])
def test_lse_merge_matches_oracle_on_oracle_partials(cas, dtype, d, u_mode):
    """The merge alone: its inputs are the ORACLE's partials (fp32-rounded), its output is
    compared with the oracle's merge of the same numbers."""
    import torch
    B, H, Hkv, N, beta = 2, 4, 2, 150, 6
    rng = np.random.default_rng(12)
    q, k, v = rng.standard_normal((B, H, N, d)) * 2, rng.standard_normal((B, Hkv, N, d)) * 2, rng.standard_normal((B, Hkv, N, d))
    a = make_assignment("ragged", N, beta, 4)
    plan = cas.cascade_plan_create(B, N, beta, a)
    _, perm, _ = orc.shard_plan(a, beta)
    parts = [orc.partial_attention_all_pairs(q[b], k[b], v[b], a, beta, scale=d ** -0.5) for b in range(B)]
    m32, e32, u32 = (np.stack([p[i] for p in parts]).astype(np.float32) for i in range(3))
    ref = np.stack([orc.lse_merge_all(m32[b].astype(np.float64), e32[b].astype(np.float64), u32[b].astype(np.float64))
                    for b in range(B)])                                        # [B, N, H*d], packed rows
    u_in = u32 if u_mode == "norm" else (e32.transpose(0, 2, 1, 3)[..., None] * u32).astype(np.float32)
    md, ed, ud = (torch.from_numpy(t).cuda() for t in (m32, e32, u_in))
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    mode = cas.U_NORMALISED if u_mode == "norm" else cas.U_UNNORMALISED
    o = torch.empty(B, N, H * d, dtype=tdt, device="cuda")
    lse = torch.empty(B, H, N, dtype=torch.float32, device="cuda")
    cas.cascade_lse_merge(plan, md, ed, ud, o, H, Hkv, d, row_layout=cas.ROWS_PACKED, u_mode=mode, lse_out=lse)
    tol = 1e-5 if dtype == "f32" else 4e-3          # bf16 here only rounds the output
    assert rel_err(host(o), ref) < tol
    o2 = torch.empty_like(o)
    cas.cascade_lse_merge(plan, md, ed, ud, o2, H, Hkv, d, row_layout=cas.ROWS_ORIGINAL, u_mode=mode)
    assert np.array_equal(host(o2)[:, perm], host(o))                         # scatter is a pure row move
    n = m32.astype(np.float64).max(axis=2)
    wsum = (np.exp(m32.astype(np.float64) - n[:, :, None]) * e32).sum(axis=2)
    assert rel_err(host(lse), n + np.log(wsum)) < 1e-5


def test_partial_then_merge_equals_direct_attention(cas):
    """GPU partials merged on the GPU equal unsharded softmax attention (oracle brute route)."""
    import torch
    for dtype, d in (("f32", 16), ("bf16", 128)):
        B, H, Hkv, N, beta = 1, 4, 2, 192, 6
        plan, got, ref, perm = attn_case(cas, dtype, B, H, Hkv, N, d, beta, "perm", "original", seed=21)
        tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        o = torch.empty(B, N, H * d, dtype=tdt, device="cuda")
        cas.cascade_lse_merge(plan, *got, o, H, Hkv, d, row_layout=cas.ROWS_ORIGINAL)
        ref_o = orc.lse_merge_all(*[r[0] for r in ref])                      # packed rows
        want = np.empty_like(ref_o)
        want[perm] = ref_o
        assert rel_err(host(o)[0], want) < TOL[dtype]


def test_attention_error_paths(cas):
    import torch
    plan = cas.cascade_plan_create(1, 64, 2, np.zeros(64, dtype=np.int32))
    q = torch.zeros(1, 4, 64, 64, dtype=torch.bfloat16, device="cuda")
    kv = torch.zeros(1, 3, 64, 64, dtype=torch.bfloat16, device="cuda")
    m = torch.zeros(1, 4, 2, 64, device="cuda"); u = torch.zeros(1, 2, 4, 64, 64, device="cuda")
    with pytest.raises(cas.CascadeError) as ei:                              # H % H_KV != 0
        cas.cascade_partial_attn(plan, q, kv, kv, m, m.clone(), u, 4, 3, 64, 0.125)
    assert ei.value.status == cas.ESHAPE
    kv = torch.zeros(1, 2, 64, 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(cas.CascadeError) as ei:                              # bf16 path needs its workspace
        cas.cascade_partial_attn(plan, q, kv, kv, m, m.clone(), u, 4, 2, 64, 0.125, workspace=None)
    assert ei.value.status == cas.EWORKSPACE
    q48 = torch.zeros(1, 4, 64, 48, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(cas.CascadeError) as ei:                              # head_dim 48 not built for bf16
        cas.cascade_partial_attn(plan, q48, q48, q48, m, m.clone(), u, 4, 4, 48, 0.125)
    assert ei.value.status == cas.EUNSUPPORTED


# ---------------------------------------------------------------------------- whole layer
SMALL_LLAMA = CONFIGS["C3"].with_(name="small-llama", d_model=512, n_heads=8, n_kv_heads=2, head_dim=128,
                                  d_ff=1024, seq_len=640, n_shards=5, index=31)
SMALL_LLAMA64 = CONFIGS["C3"].with_(name="small-llama64", d_model=256, n_heads=4, n_kv_heads=4, head_dim=64,
                                    d_ff=520, seq_len=300, n_shards=4, index=32, assignment="ragged")
SMALL_GPT = CONFIGS["C2"].with_(name="small-gpt", d_model=256, n_heads=4, n_kv_heads=4, head_dim=64, d_ff=1024,
                                batch=2, seq_len=384, n_shards=3, index=33)
F32_LLAMA = CONFIGS["C3"].with_(name="f32-llama", dtype="f32", d_model=96, n_heads=6, n_kv_heads=2, head_dim=16,
                                d_ff=200, seq_len=150, n_shards=6, index=34, assignment="ragged")


def layer_case(cas, cfg, attn_mode, io_rows=None, seed=None):
    a = make_assignment(cfg.assignment, cfg.seq_len, cfg.n_shards, 77 if seed is None else seed)
    w, h = make_layer_weights(cfg), make_hidden(cfg)
    io = cas.ROWS_ORIGINAL if io_rows is None else io_rows
    out = cas.layer_forward_numpy(cfg, w, h, a, attn_mode=attn_mode, io_rows=io)
    return a, w, h, out


@pytest.mark.parametrize("cfg", [CONFIGS["C1"], F32_LLAMA, SMALL_LLAMA, SMALL_LLAMA64, SMALL_GPT],
                         ids=lambda c: c.name)
@pytest.mark.parametrize("mode", ["fused", "materialised"])
def test_layer_forward_matches_oracle(cas, cfg, mode):
    attn_mode = cas.ATTN_FUSED if mode == "fused" else cas.ATTN_MATERIALISED
    a, w, h, out = layer_case(cas, cfg, attn_mode)
    ref = orc.layer_sharded_batch(h, w, cfg, a, cfg.n_shards)
    assert rel_err(out, ref) < TOL[cfg.dtype]
    direct = orc.layer_direct_batch(h, w, cfg)
    assert rel_err(out, direct) < TOL[cfg.dtype]


ROPE_BIAS = SMALL_LLAMA.with_(name="small-llama-bias", bias=True, norm="layernorm", act="gelu", index=35)
ROPE_POST = SMALL_LLAMA64.with_(name="small-llama64-post", norm_placement="post", index=36)
ROPE_WIDE = SMALL_LLAMA.with_(name="llama-2-tiles", d_model=1024, n_heads=16, n_kv_heads=4, seq_len=520, n_shards=3,
                              index=37)


@pytest.mark.parametrize("cfg", [SMALL_LLAMA, SMALL_LLAMA64, ROPE_BIAS, ROPE_POST, ROPE_WIDE], ids=lambda c: c.name)
@pytest.mark.parametrize("fused_qkv", [False, True], ids=["three-weights", "one-qkv-weight"])
def test_layer_rotary_embedding_paths(cas, cfg, fused_qkv):
    """The rotary embedding runs in the q/k/v projection's epilogue (bf16, pre-norm: one segment when the three
    weights are one matrix, three segments otherwise; with and without a bias) or as a pass of its own
    (post-norm); positions do not ascend with the token index, so a rotation by the row number would show."""
    a = make_assignment(cfg.assignment, cfg.seq_len, cfg.n_shards, 79)
    pos = np.random.default_rng(13).permutation(3 * cfg.seq_len)[:cfg.seq_len].astype(np.int32)
    w, h = make_layer_weights(cfg), make_hidden(cfg)
    out = cas.layer_forward_numpy(cfg, w, h, a, positions=pos, fused_qkv=fused_qkv)
    ref = orc.layer_direct_batch(h, w, cfg, positions=pos)
    assert rel_err(out, ref) < TOL[cfg.dtype]


@pytest.mark.parametrize("mode", ["fused", "materialised"])
def test_layer_forward_with_unordered_positions(cas, mode):
    """Token positions that do not ascend with the token index (rotary angles and the causal mask
    both follow them): shards hold several key/value tiles whose position ranges interleave."""
    cfg = SMALL_LLAMA
    attn_mode = cas.ATTN_FUSED if mode == "fused" else cas.ATTN_MATERIALISED
    a = make_assignment(cfg.assignment, cfg.seq_len, cfg.n_shards, 78)
    pos = np.random.default_rng(12).permutation(2 * cfg.seq_len)[:cfg.seq_len].astype(np.int32)
    w, h = make_layer_weights(cfg), make_hidden(cfg)
    out = cas.layer_forward_numpy(cfg, w, h, a, positions=pos, attn_mode=attn_mode)
    ref = orc.layer_direct_batch(h, w, cfg, positions=pos)
    assert rel_err(out, ref) < TOL[cfg.dtype]


@pytest.mark.parametrize("cfg", [CONFIGS["C1"], SMALL_LLAMA], ids=lambda c: c.name)
def test_layer_partials_match_oracle(cas, cfg):
    a = make_assignment(cfg.assignment, cfg.seq_len, cfg.n_shards, 5)
    w, h = make_layer_weights(cfg), make_hidden(cfg)
    out, (m, e, u) = cas.layer_forward_numpy(cfg, w, h, a, attn_mode=cas.ATTN_MATERIALISED, return_partials=True)
    w64 = {k: v.astype(np.float64) for k, v in w.items()}
    q, k, v = orc.pre_pass(h[0].astype(np.float64), np.arange(cfg.seq_len), w64, cfg)
    m_r, e_r, u_r = orc.partial_attention_all_pairs(q, k, v, a, cfg.n_shards, scale=cfg.scale)
    dead = ~np.isfinite(m_r)
    assert np.array_equal(~np.isfinite(m[0]), dead)
    tol = TOL[cfg.dtype]                      # q, k, v themselves carry the dtype's rounding here
    assert (np.abs(m[0][~dead] - m_r[~dead]) / np.maximum(1.0, np.abs(m_r[~dead]))).max() < tol
    assert (np.abs(e[0] - e_r) / np.maximum(1.0, e_r)).max() < tol
    assert rel_err(u[0], e_r.transpose(1, 0, 2)[..., None] * u_r) < tol


@pytest.mark.parametrize("cfg", [F32_LLAMA, SMALL_LLAMA], ids=lambda c: c.name)
def test_layer_output_invariant_under_resharding_and_io_layout(cas, cfg):
    import torch
    base = layer_case(cas, cfg, cas.ATTN_FUSED, seed=1)[3]
    for seed, beta, kind in [(2, cfg.n_shards, "perm"), (3, 3, "roundrobin"), (4, 1, "contiguous")]:
        c2 = cfg.with_(n_shards=beta, assignment=kind)
        other = layer_case(cas, c2, cas.ATTN_FUSED, seed=seed)[3]
        assert rel_err(other, base) < TOL[cfg.dtype]
    # packed io: feed packed rows, get packed rows
    a = make_assignment(cfg.assignment, cfg.seq_len, cfg.n_shards, 1)
    _, perm, _ = orc.shard_plan(a, cfg.n_shards)
    w, h = make_layer_weights(cfg), make_hidden(cfg)
    out_p = cas.layer_forward_numpy(cfg, w, h[:, perm], a, io_rows=cas.ROWS_PACKED)
    assert np.array_equal(out_p, base[:, perm])


def test_layer_forward_is_deterministic(cas):
    cfg = SMALL_LLAMA
    o1 = layer_case(cas, cfg, cas.ATTN_FUSED)[3]
    o2 = layer_case(cas, cfg, cas.ATTN_FUSED)[3]
    assert np.array_equal(o1, o2)


def test_layer_error_paths(cas):
    import torch
    cfg = SMALL_LLAMA64
    a = make_assignment("perm", cfg.seq_len, cfg.n_shards, 1)
    plan = cas.cascade_plan_create(cfg.batch, cfg.seq_len, cfg.n_shards, a)
    desc = cas.make_layer_desc(cfg)
    tensors = {k: cas.to_device(v, cfg.dtype) for k, v in make_layer_weights(cfg).items()}
    w = cas.make_layer_weights(tensors)
    h = cas.to_device(make_hidden(cfg), cfg.dtype)
    out = torch.empty_like(h)
    need = cas.cascade_layer_workspace_bytes(plan, desc)
    assert need > 0
    with pytest.raises(cas.CascadeError) as ei:
        cas.cascade_layer_forward(plan, desc, w, h, out, cas.new_workspace(need // 2))
    assert ei.value.status == cas.EWORKSPACE
    with pytest.raises(cas.CascadeError) as ei:
        cas.cascade_layer_forward(plan, desc, w, h, h, cas.new_workspace(need))       # in-place not allowed
    assert ei.value.status == cas.EINVAL
    bad = cas.make_layer_desc(cfg.with_(n_heads=5, n_kv_heads=2))
    assert cas.cascade_layer_workspace_bytes(plan, bad) == 0
    with pytest.raises(cas.CascadeError) as ei:
        cas.cascade_layer_forward(plan, bad, w, h, out, cas.new_workspace(need))
    assert ei.value.status == cas.ESHAPE
    bad = cas.make_layer_desc(cfg.with_(head_dim=48))
    with pytest.raises(cas.CascadeError) as ei:
        cas.cascade_layer_forward(plan, bad, w, h, out, cas.new_workspace(need))
    assert ei.value.status == cas.EUNSUPPORTED
    tensors2 = dict(tensors); tensors2.pop("w_gate")
    with pytest.raises(cas.CascadeError) as ei:
        cas.cascade_layer_forward(plan, desc, cas.make_layer_weights(tensors2), h, out, cas.new_workspace(need))
    assert ei.value.status == cas.EINVAL


# ---------------------------------------------------------------------------- post-norm block, layer stack
@pytest.mark.parametrize("cfg_name", ["small-gpt", "small-llama", "f32-llama", "C1"])
@pytest.mark.parametrize("mode", ["fused", "materialised"])
@pytest.mark.parametrize("mask_kind", ["none", "causal"])
def test_post_norm_layer_matches_oracle(cas, cfg_name, mode, mask_kind):
    """The BERT-shaped block: norms after the residual sums, bidirectional (mask none) or causal."""
    base = {"small-gpt": SMALL_GPT, "small-llama": SMALL_LLAMA, "f32-llama": F32_LLAMA, "C1": CONFIGS["C1"]}[cfg_name]
    cfg = base.with_(norm_placement="post")
    attn_mode = cas.ATTN_FUSED if mode == "fused" else cas.ATTN_MATERIALISED
    a = make_assignment(cfg.assignment, cfg.seq_len, cfg.n_shards, 21)
    w, h = make_layer_weights(cfg), make_hidden(cfg)
    mk = cas.MASK_NONE if mask_kind == "none" else cas.MASK_CAUSAL
    out = cas.layer_forward_numpy(cfg, w, h, a, attn_mode=attn_mode, mask_kind=mk)
    ref = orc.layer_direct_batch(h, w, cfg, mask_kind=mask_kind)
    assert rel_err(out, ref) < TOL[cfg.dtype]
    pre = orc.layer_direct_batch(h, w, base, mask_kind=mask_kind)
    assert rel_err(pre, ref) > 2 * TOL[cfg.dtype]             # the placement matters at this tolerance


@pytest.mark.parametrize("cfg_name,n_layers,io", [("small-llama", 3, "original"), ("small-gpt", 2, "original"),
                                                  ("f32-llama", 4, "packed"), ("small-llama", 1, "original")])
def test_layer_stack_matches_oracle_and_single_layer_calls(cas, cfg_name, n_layers, io):
    import torch
    cfg = {"small-gpt": SMALL_GPT.with_(norm_placement="post"), "small-llama": SMALL_LLAMA, "f32-llama": F32_LLAMA}[cfg_name]
    a = make_assignment(cfg.assignment, cfg.seq_len, cfg.n_shards, 23)
    ws_np = [make_layer_weights(cfg.with_(index=50 + l)) for l in range(n_layers)]
    h = make_hidden(cfg)
    io_rows = cas.ROWS_ORIGINAL if io == "original" else cas.ROWS_PACKED
    plan = cas.cascade_plan_create(cfg.batch, cfg.seq_len, cfg.n_shards, a)
    desc = cas.make_layer_desc(cfg, cas.ATTN_FUSED, io_rows)
    tensors = [{k: cas.to_device(v, cfg.dtype) for k, v in w.items()} for w in ws_np]
    wts = [cas.make_layer_weights(t) for t in tensors]
    _, perm, _ = orc.shard_plan(a, cfg.n_shards)
    h_host = h if io == "original" else h[:, perm]
    h_in = cas.to_device(h_host, cfg.dtype)
    h_out = torch.empty_like(h_in)
    ws = cas.new_workspace(cas.cascade_layer_stack_workspace_bytes(plan, desc, n_layers))
    cas.cascade_layer_stack_forward(plan, desc, wts, h_in, h_out, ws)
    torch.cuda.synchronize()
    got = h_out.float().cpu().numpy().astype(np.float64)
    # the same layers one call at a time (every intermediate in the caller's row order): bit-identical
    ws1 = cas.new_workspace(cas.cascade_layer_workspace_bytes(plan, desc))
    cur = h_in
    for wl in wts:
        nxt = torch.empty_like(cur)
        cas.cascade_layer_forward(plan, desc, wl, cur, nxt, ws1)
        cur = nxt
    torch.cuda.synchronize()
    assert torch.equal(cur, h_out)
    ref = np.stack([orc.layer_stack_direct(h[b], ws_np, cfg) for b in range(cfg.batch)])
    ref = ref if io == "original" else ref[:, perm]
    tol = TOL[cfg.dtype] * (1 if cfg.dtype == "f32" else n_layers)      # bf16 roundings accumulate over the layers
    assert rel_err(got, ref) < tol


def test_layer_forward_can_be_captured_in_a_hip_graph_and_replayed(cas):
    """The layer forward allocates nothing and records no memset: a caller can capture it once and replay it.
    Every replay (with eager work and synchronisations in between, and the output cleared first) reproduces the
    eager result bit for bit, also after the input changed in place."""
    import torch
    cfg = SMALL_LLAMA
    a = make_assignment("perm", cfg.seq_len, cfg.n_shards, 3)
    w, h = make_layer_weights(cfg), make_hidden(cfg)
    plan = cas.cascade_plan_create(cfg.batch, cfg.seq_len, cfg.n_shards, a)
    desc = cas.make_layer_desc(cfg, cas.ATTN_FUSED)
    t = {k: cas.to_device(v, cfg.dtype) for k, v in w.items()}
    wts = cas.make_layer_weights(t)
    h_in = cas.to_device(h, cfg.dtype)
    h_out = torch.empty_like(h_in)
    ws = cas.new_workspace(cas.cascade_layer_workspace_bytes(plan, desc))
    step = lambda: cas.cascade_layer_forward(plan, desc, wts, h_in, h_out, ws)
    step()
    torch.cuda.synchronize()
    ref = h_out.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                                     # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    torch.cuda.synchronize()
    for rep in range(3):
        h_out.fill_(7.0)
        junk = torch.randn(256, 256, device="cuda") @ torch.randn(256, 256, device="cuda")   # eager work in between
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(h_out, ref), rep
    h_in.mul_(0.5)                                                 # same buffers, new contents
    step()
    torch.cuda.synchronize()
    ref2 = h_out.clone()
    h_out.fill_(7.0)
    g.replay()
    torch.cuda.synchronize()
    assert torch.equal(h_out, ref2) and not torch.equal(ref2, ref)
