"""Seeded random sweep over plans and head layouts: partial attention (every (j, k) pair) and the merged
result against the oracle, on shapes nobody picked by hand - ragged and empty shards, shards of one to
several tiles, every grouped-query ratio the kernels specialise for, both masks, custom positions."""
import numpy as np
import pytest

from oracle import cascade_oracle as orc
from test_gpu_parity import TOL, attn_case, cas, check_partials, host, rel_err  # noqa: F401 (cas is a fixture)

pytestmark = pytest.mark.gpu

HEADS = [(4, 4), (4, 2), (8, 2), (8, 1), (6, 3), (2, 1), (3, 3), (12, 3)]
KINDS = ["perm", "ragged", "contiguous", "roundrobin"]


def draw_case(seed):
    rng = np.random.default_rng(1000 + seed)
    dtype = "f32" if seed % 4 == 3 else "bf16"
    H, Hkv = HEADS[rng.integers(len(HEADS))]
    d = int(rng.choice([64, 128])) if dtype == "bf16" else int(rng.choice([8, 16, 24, 40]))
    N = int(rng.integers(1, 520)) if dtype == "bf16" else int(rng.integers(1, 160))
    beta = int(rng.integers(1, min(N, 24) + 1))
    kind = KINDS[rng.integers(len(KINDS))]
    layout = "packed" if rng.integers(2) else "original"
    mask_kind = "none" if rng.integers(4) == 0 else "causal"
    positions = None
    if rng.integers(3) == 0:
        positions = rng.permutation(4 * N + 7)[:N].astype(np.int32)
    return dict(dtype=dtype, H=H, Hkv=Hkv, d=d, N=N, beta=beta, kind=kind, layout=layout, mask_kind=mask_kind,
                positions=positions)


@pytest.mark.parametrize("seed", range(32))
def test_random_plan_partials_and_merge(cas, seed):
    import torch
    c = draw_case(seed)
    print("case", seed, {k: (v if k != "positions" else v is not None) for k, v in c.items()}, flush=True)
    B = 1 + seed % 2
    plan, got, ref, perm = attn_case(cas, c["dtype"], B, c["H"], c["Hkv"], c["N"], c["d"], c["beta"], c["kind"],
                                     c["layout"], mask_kind=c["mask_kind"], seed=seed, positions=c["positions"])
    check_partials(c["dtype"], got, ref)
    # merge of the device partials against the merge of the oracle's partials (Algorithm 4)
    m, e, u = got
    H, N, d = c["H"], c["N"], c["d"]
    o = torch.full((B, N, H * d), 3.0, dtype=torch.bfloat16 if c["dtype"] == "bf16" else torch.float32, device="cuda")
    cas.cascade_lse_merge(plan, m, e, u, o, H, c["Hkv"], d, row_layout=cas.ROWS_PACKED, u_mode=cas.U_UNNORMALISED)
    m_r, e_r, u_r = ref
    for b in range(B):
        o_ref = orc.lse_merge_all(m_r[b], e_r[b], u_r[b])                   # [N, H*d], packed rows
        assert rel_err(host(o[b]), o_ref) < TOL[c["dtype"]]


def draw_layer(seed):
    from cascade_inputs import CONFIGS
    rng = np.random.default_rng(5000 + seed)
    f32 = seed % 4 == 3
    H, Hkv = HEADS[rng.integers(len(HEADS))]
    hd = int(rng.choice([8, 16, 24])) if f32 else int(rng.choice([64, 128]))
    llama = bool(rng.integers(2))
    base = CONFIGS["C3"] if llama else CONFIGS["C2"]
    d_model = int(rng.choice([64, 96, 136])) if f32 else int(rng.choice([128, 256, 320, 512, 584]))
    d_ff = int(rng.choice([72, 200, 256])) if f32 else int(rng.choice([256, 520, 1024, 1096]))
    N = int(rng.integers(1, 140)) if f32 else int(rng.integers(1, 420))
    return base.with_(name=f"sweep{seed}", dtype="f32" if f32 else "bf16", d_model=d_model, n_heads=H, n_kv_heads=Hkv,
                      head_dim=hd, d_ff=d_ff, batch=1 + seed % 2, seq_len=N, n_shards=int(rng.integers(1, min(N, 12) + 1)),
                      assignment=KINDS[rng.integers(len(KINDS))], index=400 + seed,
                      norm_placement="post" if rng.integers(4) == 0 else "pre")


@pytest.mark.parametrize("seed", range(16))
def test_random_layer_forward(cas, seed):
    from cascade_inputs import make_assignment, make_hidden, make_layer_weights
    cfg = draw_layer(seed)
    print("case", seed, cfg, flush=True)
    a = make_assignment(cfg.assignment, cfg.seq_len, cfg.n_shards, 900 + seed)
    w, h = make_layer_weights(cfg), make_hidden(cfg)
    direct = orc.layer_direct_batch(h, w, cfg)
    for attn_mode in (cas.ATTN_FUSED, cas.ATTN_MATERIALISED):
        out = cas.layer_forward_numpy(cfg, w, h, a, attn_mode=attn_mode, io_rows=cas.ROWS_ORIGINAL)
        assert rel_err(out, direct) < TOL[cfg.dtype], attn_mode


@pytest.mark.parametrize("seed", range(24))
def test_random_shard_gemm(cas, seed):
    """Random M, N, K (ragged against every tile size), random epilogue, gathered input rows and scattered
    output rows through a random plan: every output element against the oracle."""
    import torch
    from cascade_inputs import make_assignment
    from test_gpu_parity import dev, rand
    rng = np.random.default_rng(9000 + seed)
    dtype = "f32" if seed % 4 == 3 else "bf16"
    B = int(rng.integers(1, 3))
    Nseq = int(rng.integers(1, 400 if dtype == "bf16" else 90))
    M = B * Nseq
    K = 8 * int(rng.integers(1, 80)) if rng.integers(2) else 64 * int(rng.integers(1, 12))
    N = 4 * int(rng.integers(1, 700 if dtype == "bf16" else 60))
    beta = int(rng.integers(1, min(Nseq, 9) + 1))
    a = make_assignment(KINDS[rng.integers(len(KINDS))], Nseq, beta, seed)
    plan = cas.cascade_plan_create(B, Nseq, beta, a)
    _, perm, _ = orc.shard_plan(a, beta)
    rows = np.concatenate([b * Nseq + perm for b in range(B)])          # packed row r holds original row rows[r]
    x, w = rand(rng, (M, K), dtype), rand(rng, (N, K), dtype, 0.2)
    x64, w64 = x.astype(np.float64), w.astype(np.float64)
    x_orig, y_orig = bool(rng.integers(2)), bool(rng.integers(2))
    mode = ["plain", "bias", "bias_gelu", "gelu_tanh", "residual", "bias_residual", "swiglu"][rng.integers(7)]
    print("case", seed, dict(dtype=dtype, M=M, N=N, K=K, beta=beta, x_orig=x_orig, y_orig=y_orig, mode=mode), flush=True)
    X, W = dev(cas, x, dtype), dev(cas, w, dtype)
    kw, ep = {}, 0
    xin = x64[rows] if x_orig else x64                                   # the GEMM's input rows in packed order
    ref = orc.linear(xin, w64)
    if mode == "swiglu":
        wu = rand(rng, (N, K), dtype, 0.2)
        kw["W_up"] = dev(cas, wu, dtype); ep |= cas.EPI_SWIGLU
        ref = orc.silu(ref) * orc.linear(xin, wu.astype(np.float64))
    if "bias" in mode:
        b = rand(rng, (N,), dtype, 0.3)
        kw["bias"] = dev(cas, b, dtype); ep |= cas.EPI_BIAS
        ref = ref + b.astype(np.float64)
    if mode == "bias_gelu":
        ep |= cas.EPI_GELU_ERF; ref = orc.gelu_erf(ref)
    if mode == "gelu_tanh":
        ep |= cas.EPI_GELU_TANH; ref = orc.gelu_tanh(ref)
    if "residual" in mode:
        r = rand(rng, (M, N), dtype)                                     # residual rows in the output's order
        kw["residual"] = dev(cas, r, dtype); ep |= cas.EPI_RESIDUAL
        kw["res_rows"] = cas.ROWS_ORIGINAL if y_orig else cas.ROWS_PACKED
        ref = ref + (r.astype(np.float64)[rows] if y_orig else r.astype(np.float64))
    Y = torch.full((M, N), 7.0, dtype=X.dtype, device="cuda")
    cas.cascade_shard_gemm(plan, X, W, Y, epilogue=ep, x_rows=cas.ROWS_ORIGINAL if x_orig else cas.ROWS_PACKED,
                           y_rows=cas.ROWS_ORIGINAL if y_orig else cas.ROWS_PACKED, **kw)
    got = host(Y)
    want = np.empty_like(ref)
    if y_orig:
        want[rows] = ref                                                 # packed result row r lands in original row rows[r]
    else:
        want = ref
    assert rel_err(got, want) < TOL[dtype]
