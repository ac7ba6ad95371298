"""The FFN down projection as a split reduction (two workgroups per 256 x 256 tile, half of K each, the first to
finish hands its accumulators to the second through scratch in the workspace): a layer whose shapes select that
kernel on a 256-CU device (80 tiles, the last row of tiles half empty) against the float64 CPU oracle, element by
element, and the properties the exchange must have whatever the order of arrival."""
import numpy as np
import pytest

from cascade_inputs import CONFIGS, make_assignment, make_hidden, make_layer_weights
from oracle import cascade_oracle as orc

pytestmark = pytest.mark.gpu

TOL = 2e-2          # bf16 storage, fp32 accumulation: max|gpu - ref| / max|ref|

# 1152 rows x 4096 columns = 5 x 16 tiles of 256 x 256; the FFN down projection reduces over 8192, the shortest
# reduction the library splits (the o projection, over 16 heads of 128, stays whole)
SPLIT = CONFIGS["C3"].with_(name="llama-split-reduction", d_model=4096, n_heads=16, n_kv_heads=4, head_dim=128,
                            d_ff=8192, seq_len=1152, n_shards=6, index=38)
SPLIT_GELU = SPLIT.with_(name="gpt-split-reduction", bias=True, norm="layernorm", act="gelu", rope=False, index=39)
SPLIT_POST = SPLIT.with_(name="llama-split-reduction-post", norm_placement="post", index=40)


@pytest.fixture(scope="module")
def cas():
    import torch
    assert torch.cuda.is_available()
    import paper_2507_05228_amd as cas
    cas.load_library()
    return cas


def rel_err(g, r):
    return float(np.abs(np.asarray(g, dtype=np.float64) - r).max() / max(np.abs(r).max(), 1e-300))


def test_the_shape_asks_for_split_reduction_scratch(cas):
    """80 tiles x 256 KB of fp32 partials are part of the layer workspace at 1152 rows, none at 1024 rows (64 tiles
    fill a quarter of the CUs: the 128-row kernels take those)."""
    import torch
    if torch.cuda.get_device_properties(0).multi_processor_count != 256:
        pytest.skip("tile counts chosen for 256 CUs")
    need = {}
    for n in (1024, 1152):
        cfg = SPLIT.with_(seq_len=n)
        plan = cas.cascade_plan_create(1, n, cfg.n_shards, make_assignment(cfg.assignment, n, cfg.n_shards, 5))
        need[n] = cas.cascade_layer_workspace_bytes(plan, cas.make_layer_desc(cfg, cas.ATTN_FUSED))
    # every other buffer grows with the row count (the attention scratch a little less: tile padding)
    assert need[1152] - need[1024] * 1152 // 1024 >= 0.95 * 80 * 256 * 256 * 4


@pytest.mark.parametrize("cfg", [SPLIT, SPLIT_GELU, SPLIT_POST], ids=lambda c: c.name)
def test_layer_with_split_reduction_gemms_matches_oracle(cas, cfg):
    """Pre-norm SwiGLU block (residual only in the second workgroup's epilogue), LayerNorm / GELU block with biases
    (bias and residual), post-norm block (the flag words are cleared by the norm in front of the MLP)."""
    a = make_assignment(cfg.assignment, cfg.seq_len, cfg.n_shards, 83)
    w, h = make_layer_weights(cfg), make_hidden(cfg)
    out = cas.layer_forward_numpy(cfg, w, h, a)
    ref = orc.layer_direct_batch(h, w, cfg)
    assert rel_err(out, ref) < TOL


def test_split_reduction_does_not_depend_on_what_the_workspace_held(cas):
    """The ticket and flag words are cleared inside the call and count up over the launches that share them: the
    same call on a workspace full of ones, on the workspace the previous call left behind, and twice in a row
    inside a layer stack gives the same bits (the sum of the two halves does not depend on who finished first)."""
    import torch
    cfg = SPLIT
    a = make_assignment(cfg.assignment, cfg.seq_len, cfg.n_shards, 83)
    w, h = make_layer_weights(cfg), make_hidden(cfg)
    plan = cas.cascade_plan_create(cfg.batch, cfg.seq_len, cfg.n_shards, a)
    desc = cas.make_layer_desc(cfg, cas.ATTN_FUSED)
    t = {k: cas.to_device(v, cfg.dtype) for k, v in w.items()}
    wts = cas.make_layer_weights(t)
    h_in = cas.to_device(h, cfg.dtype)
    outs = []
    ws = cas.new_workspace(cas.cascade_layer_stack_workspace_bytes(plan, desc, 2))
    for fill in (0xFF, None, 0x00, None):
        if fill is not None:
            ws.view(torch.uint8).fill_(fill)
        o = torch.empty_like(h_in)
        cas.cascade_layer_forward(plan, desc, wts, h_in, o, ws)
        torch.cuda.synchronize()
        outs.append(o)
    for o in outs[1:]:
        assert torch.equal(o, outs[0])
    two = torch.empty_like(h_in)
    cas.cascade_layer_stack_forward(plan, desc, [wts, wts], h_in, two, ws)
    second = torch.empty_like(h_in)
    cas.cascade_layer_forward(plan, desc, wts, outs[0], second, ws)
    torch.cuda.synchronize()
    assert torch.equal(two, second)


def test_layer_with_split_reduction_replays_from_a_hip_graph(cas):
    """The exchange clears its flag words inside the captured work (a norm launch, no memset): replays, with eager
    work and synchronisations in between and the scratch overwritten, reproduce the eager result bit for bit."""
    import torch
    cfg = SPLIT
    a = make_assignment(cfg.assignment, cfg.seq_len, cfg.n_shards, 83)
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
        ws.fill_(0xA5 if rep % 2 else 0x00)                        # whatever the last replay left is gone
        junk = torch.randn(256, 256, device="cuda") @ torch.randn(256, 256, device="cuda")   # eager work in between
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(h_out, ref), rep
