"""CPU-side checks of the boundary: the shared library loads, exports every symbol the header
declares, and the ctypes mirrors of the descriptor structs have the header's layout.
No compute call is made here (there is no GPU in this environment)."""
import ctypes as C
import numpy as np
import os
import re
import subprocess

import pytest

import paper_2507_05228_amd as cas

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "cascade.h")


def declared_symbols():
    text = open(HEADER).read()
    return sorted(set(re.findall(r"CASCADE_API\s+[\w\s\*]+?\b(cascade_\w+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib_path():
    if not os.path.exists(cas.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return cas.LIB_PATH


def test_header_declares_the_four_ops():
    names = declared_symbols()
    for op in ("cascade_shard_gemm", "cascade_partial_attn", "cascade_lse_merge", "cascade_layer_forward"):
        assert op in names


def test_library_exports_every_declared_symbol(lib_path):
    lib = C.CDLL(lib_path)
    for name in declared_symbols():
        assert hasattr(lib, name), name
    assert sorted(cas.EXPORTS) == declared_symbols()


def test_binding_has_the_same_names():
    for name in ("cascade_plan_create", "cascade_plan_maps", "cascade_shard_gemm", "cascade_partial_attn",
                 "cascade_lse_merge", "cascade_layer_forward", "cascade_layer_workspace_bytes"):
        assert callable(getattr(cas, name))


def test_struct_layouts_match_the_header(tmp_path):
    """Compile a tiny C program against the header and compare sizeof / offsetof with ctypes."""
    src = tmp_path / "layout.c"
    src.write_text(
        '#include <stdio.h>\n#include <stddef.h>\n#include "cascade.h"\n'
        "int main(void){\n"
        'printf("%zu %zu %zu %zu\\n", sizeof(cascade_gemm_desc), sizeof(cascade_attn_desc),'
        " sizeof(cascade_layer_desc), sizeof(cascade_layer_weights));\n"
        'printf("%zu %zu %zu\\n", offsetof(cascade_attn_desc, q_stride_b), offsetof(cascade_layer_desc, io_rows),'
        " offsetof(cascade_layer_weights, norm2_b));\n"
        'printf("%zu\\n", offsetof(cascade_gemm_desc, rope_theta));\n'
        'printf("%zu %zu\\n", sizeof(cascade_lm_head_desc), offsetof(cascade_lm_head_desc, out_rows));\n'
        "return 0;}\n")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    got = [int(t) for t in out]
    want = [C.sizeof(cas.GemmDesc), C.sizeof(cas.AttnDesc), C.sizeof(cas.LayerDesc), C.sizeof(cas.LayerWeights),
            cas.AttnDesc.q_stride_b.offset, cas.LayerDesc.io_rows.offset, cas.LayerWeights.norm2_b.offset,
            cas.GemmDesc.rope_theta.offset, C.sizeof(cas.LmHeadDesc), cas.LmHeadDesc.out_rows.offset]
    assert got == want


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(cas, "_lib", None)
    monkeypatch.setattr(cas, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        cas.load_library()


def test_product_package_does_not_import_the_oracle():
    for dirpath, _, files in os.walk(os.path.join(ROOT, "paper_2507_05228_amd")):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower().replace("no cpu fallback", ""), f
    text = open(os.path.join(ROOT, "oracle", "cascade_oracle.py")).read()
    assert "paper_2507_05228_amd" not in text and "ctypes" not in text


# ---------------------------------------------------------------------------- host-only plan generators
def _read_rx():
    rx = {}
    path = os.path.join(os.path.dirname(__file__), "golden", "msplit_example.txt")
    for line in open(path):
        if line.startswith("RX"):
            key, vals = line.split(":")
            _, i, x = key.split()
            rx[(int(i), int(x))] = [int(t) for t in vals.split()]
    return rx


def test_cdelta_and_m_split_generators_reproduce_the_worked_example():
    """Section 6.4's N = 18 example (alpha = 3, c = 2, delta = 6, m = 2), through the C entry points."""
    a, n = cas.cascade_cdelta_assignment(18, 2, 6)
    assert n == 3
    assert a.tolist() == [0, 0, 1, 1, 2, 2] * 3
    kv = cas.cascade_m_split(a, 3, 2)
    for (i, x), toks in _read_rx().items():
        for t in toks:
            assert kv[t - 1] == 2 * (i - 1) + (x - 1)


@pytest.mark.parametrize("N,c,delta,m", [(18, 2, 6, 2), (256, 8, 64, 4), (50, 3, 10, 3), (32, 1, 8, 1), (100, 4, 30, 5)])
def test_generators_agree_with_the_oracle_bit_for_bit(N, c, delta, m):
    from oracle import cascade_oracle as orc
    a, n = cas.cascade_cdelta_assignment(N, c, delta)
    assert n == -(-delta // c)
    assert np.array_equal(a, orc.cdelta_assignment(N, c, delta))
    assert np.array_equal(cas.cascade_m_split(a, n, m), orc.m_split_assignment(a, n, m))


def test_generator_error_paths():
    with pytest.raises(cas.CascadeError) as ei:
        cas.cascade_cdelta_assignment(16, 0, 4)
    assert ei.value.status == cas.EINVAL
    with pytest.raises(cas.CascadeError) as ei:
        cas.cascade_m_split(np.array([0, 1, 5], dtype=np.int32), 3, 2)
    assert ei.value.status == cas.EASSIGN
    with pytest.raises(cas.CascadeError) as ei:
        cas.cascade_m_split(np.array([0, 1, 2], dtype=np.int32), 3, 0)
    assert ei.value.status == cas.EINVAL


def test_comm_cost_matches_equation_1_and_the_papers_table():
    from oracle import cascade_oracle as orc
    for alpha, beta, F, d, H, Hkv, N in [(16, 16, 2, 128, 32, 8, 2048), (3, 6, 4, 64, 12, 12, 128), (1, 1, 2, 16, 4, 4, 18)]:
        a, b, r = cas.cascade_comm_cost(alpha, beta, F, d, H, Hkv, N)
        total, oa, ob = orc.comm_bytes(beta, F, d, H, Hkv, N)
        assert (a, b) == (oa, ob) and a + b == total == beta * F * (2 * d * H + 2 * d * Hkv + 2 * H) * N
        assert r == 2 * alpha * beta * beta
        assert cas.cascade_comm_cost(alpha, beta, F, d, H, Hkv, N, m_split_scheme=True)[2] == 2 * beta * beta
    # the printed byte table (bf16, N = 128, beta = alpha, summed over layers; 3 decimals)
    models = {"base": dict(H=12, d=64, layers=12), "large": dict(H=16, d=64, layers=24)}
    path = os.path.join(os.path.dirname(__file__), "golden", "comm_table.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        alpha, base_gb, large_gb = line.split()
        for name, want in (("base", float(base_gb)), ("large", float(large_gb))):
            mdl = models[name]
            a, b, _ = cas.cascade_comm_cost(int(alpha), int(alpha), 2, mdl["d"], mdl["H"], mdl["H"], 128)
            assert abs((a + b) * mdl["layers"] / 1e9 - want) <= 0.0006
    with pytest.raises(cas.CascadeError) as ei:
        cas.cascade_comm_cost(0, 4, 2, 64, 8, 8, 128)
    assert ei.value.status == cas.EINVAL


def test_comm_time_matches_equation_2_and_the_oracle():
    """cascade_comm_time with explicit shard sizes (a plan needs a GPU) against the oracle's node-by-node count."""
    from oracle import cascade_oracle as orc
    rng = np.random.default_rng(5)
    for N, alpha, m, F, d, H, Hkv in ((300, 5, 3, 2, 64, 12, 12), (1000, 7, 1, 4, 128, 32, 8), (18, 3, 2, 2, 16, 4, 2)):
        a = rng.integers(0, alpha, size=N)
        kv = orc.m_split_assignment(a, alpha, m)
        R, S = orc.shard_index_lists(a, alpha), orc.shard_index_lists(kv, alpha * m)
        tau, bw = 0.38e-3, 2.5e8
        want = orc.comm_time(R, S, F, d, H, Hkv, tau, bw)
        got = cas.cascade_comm_time(F, d, H, Hkv, tau, bw, n_kv_shards=alpha * m,
                                    max_row_shard=max(len(r) for r in R), max_kv_shard=max(len(s) for s in S))
        assert np.allclose(got, want, rtol=1e-12, atol=0)
    # one shard, no latency: the bytes of Equation 1 over the bandwidth
    a_bytes, b_bytes, _ = cas.cascade_comm_cost(1, 1, 2, 64, 12, 12, 128)
    total, ta, tb = cas.cascade_comm_time(2, 64, 12, 12, 0.0, 1e9, n_kv_shards=1, max_row_shard=128, max_kv_shard=128)
    assert np.isclose(ta * 1e9, a_bytes) and np.isclose(tb * 1e9, b_bytes) and np.isclose(total, ta + tb)
    for bad in (dict(latency_s=-1.0), dict(bandwidth_bytes_per_s=0.0), dict(n_kv_shards=0)):
        kw = dict(latency_s=0.0, bandwidth_bytes_per_s=1e9, n_kv_shards=2, max_row_shard=4, max_kv_shard=4)
        kw.update(bad)
        with pytest.raises(cas.CascadeError) as ei:
            cas.cascade_comm_time(2, 64, 12, 12, **kw)
        assert ei.value.status == cas.EINVAL


def test_unified_workspace_query_needs_no_device_for_the_zero_cases():
    """Operations without a workspace report 0; invalid descriptors report 0 (no plan can exist without a GPU)."""
    assert cas.cascade_workspace_bytes(None, None, cas.OP_SHARD_GEMM) == 0
    assert cas.cascade_workspace_bytes(None, None, cas.OP_LSE_MERGE) == 0
    assert cas.cascade_workspace_bytes(None, None, cas.OP_LAYER_FORWARD) == 0
    assert cas.cascade_workspace_bytes(None, None, 99) == 0
