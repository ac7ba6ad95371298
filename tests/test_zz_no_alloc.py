"""The entry point that allocates nothing (cascade_partial_attn_static: scratch in a static device array)
against cascade_partial_attn with a caller's workspace: same kernels, so the outputs must be bit-identical.
Two calls in a row, the second on a smaller problem (the static array keeps the first call's contents)."""
import numpy as np
import pytest

from cascade_inputs import make_assignment, round_to_bf16

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cas():
    import torch
    assert torch.cuda.is_available()
    import paper_2507_05228_amd as cas
    cas.load_library()
    return cas


def _case(cas, B, H, Hkv, N, d, beta, kind, layout, seed, dtype="bf16"):
    import torch
    rng = np.random.default_rng(seed)

    def draw(shape):
        x = rng.standard_normal(shape).astype(np.float32)
        return cas.to_device(round_to_bf16(x) if dtype == "bf16" else x, dtype)

    q, k, v = draw((B, H, N, d)), draw((B, Hkv, N, d)), draw((B, Hkv, N, d))
    a = make_assignment(kind, N, beta, seed + 1)
    plan = cas.cascade_plan_create(B, N, beta, a)
    outs = []
    for static in (False, True):
        m = torch.full((B, H, beta, N), 7.0, dtype=torch.float32, device="cuda")
        e = torch.full((B, H, beta, N), 7.0, dtype=torch.float32, device="cuda")
        u = torch.full((B, beta, H, N, d), 7.0, dtype=torch.float32, device="cuda")
        if static:
            cas.cascade_partial_attn_static(plan, q, k, v, m, e, u, H, Hkv, d, d ** -0.5, row_layout=layout)
        else:
            ws = cas.new_workspace(cas.cascade_partial_attn_workspace_bytes(plan, q, H, Hkv, d))
            cas.cascade_partial_attn(plan, q, k, v, m, e, u, H, Hkv, d, d ** -0.5, row_layout=layout, workspace=ws)
        torch.cuda.synchronize()
        outs.append((m.cpu().numpy(), e.cpu().numpy(), u.cpu().numpy()))
    return outs


def test_static_scratch_entry_point_matches_the_workspace_one_twice(cas):
    # first call: ragged shards, rows in the caller's order (uses both the V^T and the gathered-K part of the scratch)
    big = _case(cas, 2, 8, 2, 700, 128, 5, "ragged", cas.ROWS_ORIGINAL, seed=3)
    # second call: a smaller problem with another head dimension, over the first call's leftovers
    small = _case(cas, 1, 4, 4, 130, 64, 3, "perm", cas.ROWS_PACKED, seed=4)
    for ref, got in (big, small):
        for r, g in zip(ref, got):
            assert np.array_equal(r, g, equal_nan=True)
    assert np.isfinite(big[1][2]).all() and np.abs(big[1][2]).max() > 0      # something was computed


def test_static_scratch_fp32_needs_none(cas):
    ref, got = _case(cas, 1, 2, 1, 70, 16, 4, "ragged", cas.ROWS_ORIGINAL, seed=5, dtype="f32")
    for r, g in zip(ref, got):
        assert np.array_equal(r, g, equal_nan=True)


def test_static_scratch_rejects_what_does_not_fit(cas):
    import torch
    B, H, Hkv, N, d = 1, 16, 16, 16384, 128          # 2 * 16 * 128 * (16384 + 16384) * 2 bytes = 128 MiB of scratch
    plan = cas.cascade_plan_create(B, N, 4, make_assignment("contiguous", N, 4, 0))
    q = torch.zeros((1, 1, 8, d), dtype=torch.bfloat16, device="cuda")   # never read: the size check comes first
    assert cas.cascade_partial_attn_workspace_bytes(plan, q, H, Hkv, d) > cas.STATIC_SCRATCH_BYTES
    with pytest.raises(cas.CascadeError) as ei:
        cas.cascade_partial_attn_static(plan, q, q, q, q, q, q, H, Hkv, d, 1.0)
    assert ei.value.status == cas.EWORKSPACE
