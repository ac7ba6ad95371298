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
