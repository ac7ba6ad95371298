"""Pins for the float64 oracle: values the paper prints, closed forms, invariants,
brute force with plain Python loops, and library routines (torch CPU, float64) for the
special cases that reduce to them.  None of these call the HIP path."""
import math
import os

import numpy as np
import pytest
import torch

from cascade_inputs import CONFIGS, make_assignment, make_hidden, make_layer_weights
from oracle import cascade_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

TINY_LLAMA = CONFIGS["C3"].with_(name="tiny-llama", dtype="f32", d_model=32, n_heads=4, n_kv_heads=2,
                                 head_dim=8, d_ff=48, batch=1, seq_len=24, n_shards=4, index=11)
TINY_GPT = CONFIGS["C1"].with_(name="tiny-gpt", d_model=24, n_heads=3, n_kv_heads=3, head_dim=8,
                               d_ff=40, batch=1, seq_len=20, n_shards=5, index=12)


def rel_err(a, b):
    return np.abs(a - b).max() / max(np.abs(b).max(), 1e-300)


# ---------------------------------------------------------------- brute force helpers (pure Python)
def brute_attention(q, k, v, pos, scale, causal=True):
    """softmax(scale q k^T + s) v from the definition, Python loops, no max subtraction."""
    H, N, d = q.shape
    rep = H // k.shape[0]
    out = np.zeros((H, N, d))
    for h in range(H):
        g = h // rep
        for x in range(N):
            ws, acc = 0.0, [0.0] * d
            for y in range(N):
                if causal and pos[y] > pos[x]:
                    continue
                a = scale * sum(q[h, x, i] * k[g, y, i] for i in range(d))
                p = math.exp(a)
                ws += p
                for i in range(d):
                    acc[i] += p * v[g, y, i]
            out[h, x] = [t / ws for t in acc]
    return out


def rand_qkv(seed, H, Hkv, N, d, amp=1.0):
    rng = np.random.default_rng(seed)
    return (amp * rng.standard_normal((H, N, d)), amp * rng.standard_normal((Hkv, N, d)),
            rng.standard_normal((Hkv, N, d)))


# ---------------------------------------------------------------- sharding / plan
def test_shard_plan_is_sorted_partition():
    a = make_assignment("ragged", 50, 7, 3)
    offsets, perm, inv = orc.shard_plan(a, 7)
    assert sorted(perm.tolist()) == list(range(50))
    assert (inv[perm] == np.arange(50)).all()
    for j in range(7):
        rows = perm[offsets[j]:offsets[j + 1]]
        assert (a[rows] == j).all()
        assert (np.diff(rows) > 0).all()
    assert offsets[-1] == 50


def test_shard_plan_rejects_bad_ids():
    with pytest.raises(ValueError):
        orc.shard_plan(np.array([0, 3, 1]), 3)
    with pytest.raises(ValueError):
        orc.shard_plan(np.array([0, -1, 1]), 3)


def _read_example():
    R, RX, S = {}, {}, {}
    for line in open(os.path.join(GOLDEN, "msplit_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, vals = line.split(":")
        key = key.split()
        vals = [int(t) for t in vals.split()]
        if key[0] == "R":
            R[int(key[1])] = vals
        elif key[0] == "RX":
            RX[(int(key[1]), int(key[2]))] = vals
        else:
            S[tuple(int(t) for t in key[1:])] = vals
    return R, RX, S


def test_cdelta_and_msplit_match_the_worked_example():
    """Section 6.4 example: alpha=3, c=2, delta=6, N=18, m=2 (paper is 1-based)."""
    R, RX, S = _read_example()
    a = orc.cdelta_assignment(18, c=2, delta=6)
    lists = orc.shard_index_lists(a, 3)
    split = {}
    for i in range(3):
        assert (lists[i] + 1).tolist() == R[i + 1]
        for x, part in enumerate(orc.m_split(lists[i], 2)):
            split[(i + 1, x + 1)] = (part + 1).tolist()
    assert split == RX
    assert len(S) == 21
    for (i, x, j, y), want in S.items():
        assert sorted(set(split[(i, x)]) | set(split[(j, y)])) == want
    # S_{m(i-1)+x} = R_{i,x}: beta = m * alpha shards that still partition [N]
    allv = sorted(t for v in split.values() for t in v)
    assert allv == list(range(1, 19))


def test_cdelta_shard_count_and_gap():
    """alpha = ceil(delta / c) (Section 6) and gap delta - c + 1 = (alpha-1) c + 1 between clusters."""
    for c, delta, N in [(2, 6, 18), (8, 64, 256), (3, 10, 50), (1, 8, 32)]:
        a = orc.cdelta_assignment(N, c, delta)
        alpha = -(-delta // c)
        assert a.max() + 1 == alpha
        R0 = orc.shard_index_lists(a, alpha)[0]
        jumps = np.diff(R0)
        assert set(jumps.tolist()) <= {1, delta - c + 1}
        if delta % c == 0 and len(R0) > c:
            assert delta - c + 1 == (alpha - 1) * c + 1


# ---------------------------------------------------------------- cost model
def test_comm_bytes_reproduces_the_papers_table():
    """Equation 1 with F=2 bytes, N=128, beta=alpha, summed over layers, against the
    printed table (3 decimals)."""
    models = {"base": dict(H=12, Hkv=12, d=64, layers=12), "large": dict(H=16, Hkv=16, d=64, layers=24)}
    rows = [l.split() for l in open(os.path.join(GOLDEN, "comm_table.txt")) if not l.startswith("#")]
    for alpha, base_gb, large_gb in rows:
        for name, want in (("base", float(base_gb)), ("large", float(large_gb))):
            mdl = models[name]
            total, a, b = orc.comm_bytes(int(alpha), 2, mdl["d"], mdl["H"], mdl["Hkv"], 128)
            assert total == a + b
            gb = total * mdl["layers"] / 1e9
            assert abs(gb - want) <= 0.0006, (alpha, name, gb, want)


def test_comm_bytes_halves_closed_form():
    total, a, b = orc.comm_bytes(beta=16, F=2, d=128, H=32, Hkv=8, N=2048)
    assert a == 16 * 2 * 128 * (32 + 16) * 2048
    assert b == 16 * 2 * 130 * 32 * 2048
    assert total == 16 * 2 * (2 * 128 * 32 + 2 * 128 * 8 + 2 * 32) * 2048


def test_comm_time_is_equation_2():
    """Equation 2 (Theoretical Costs): 2 tau + beta F d (H + 2 H_KV) / B * max|R_i| + F (d + 2) H / B * max|S_j|,
    here against the oracle's node-by-node count on ragged partitions with R != S."""
    rng = np.random.default_rng(12)
    for N, alpha, m, F, d, H, Hkv in ((300, 5, 3, 2, 64, 12, 12), (1000, 7, 1, 4, 128, 32, 8), (64, 64, 2, 2, 16, 4, 2)):
        a = rng.integers(0, alpha, size=N)
        kv = orc.m_split_assignment(a, alpha, m)
        R, S = orc.shard_index_lists(a, alpha), orc.shard_index_lists(kv, alpha * m)
        tau, bw = 0.38e-3, 2e9 / 8
        total, t_a, t_b = orc.comm_time(R, S, F, d, H, Hkv, tau, bw)
        beta = alpha * m
        want = (2 * tau + beta * F * d * (H + 2 * Hkv) / bw * max(len(r) for r in R)
                + F * (d + 2) * H / bw * max(len(s) for s in S))
        assert math.isclose(total, want, rel_tol=1e-12)
        assert math.isclose(total, t_a + t_b, rel_tol=1e-15)


def test_comm_time_reduces_to_equation_1_over_bandwidth():
    """Equal shards: every node of a stage sends the same amount, so (stage time - tau) x nodes x B is that
    stage's byte count of Equation 1 (itself pinned by the paper's table); one shard without latency is
    CommBytes / B; the latency enters as 2 tau; more key/value shards never make it faster."""
    N, F, d, H, Hkv, bw = 1024, 2, 64, 12, 12, 3.0e8
    for alpha, m in ((1, 1), (4, 1), (8, 2), (16, 4)):
        a = orc.cdelta_assignment(N, N // alpha // 4 or 1, N // 4 if alpha > 1 else N)
        if alpha == 1:
            a = np.zeros(N, dtype=np.int64)
        assert a.max() + 1 == alpha
        kv = orc.m_split_assignment(a, alpha, m)
        beta = alpha * m
        R, S = orc.shard_index_lists(a, alpha), orc.shard_index_lists(kv, beta)
        assert len({len(r) for r in R}) == 1 and len({len(s) for s in S}) == 1
        total, t_a, t_b = orc.comm_time(R, S, F, d, H, Hkv, 0.0, bw)
        all_bytes, bytes_a, bytes_b = orc.comm_bytes(beta, F, d, H, Hkv, N)
        assert math.isclose(t_a * alpha * bw, bytes_a, rel_tol=1e-12)
        assert math.isclose(t_b * beta * beta * bw, bytes_b, rel_tol=1e-12)
        if beta == 1:
            assert math.isclose(total * bw, all_bytes, rel_tol=1e-12)
        with_tau = orc.comm_time(R, S, F, d, H, Hkv, 1e-3, bw)[0]
        assert math.isclose(with_tau - total, 2e-3, rel_tol=1e-9)
    times = []
    for m in (1, 2, 4, 8):                      # same row shards, finer key/value shards
        a = orc.cdelta_assignment(N, 32, 256)
        S = orc.shard_index_lists(orc.m_split_assignment(a, 8, m), 8 * m)
        times.append(orc.comm_time(orc.shard_index_lists(a, 8), S, F, d, H, Hkv, 0.0, bw)[1])
    assert all(x < y for x, y in zip(times, times[1:]))     # stage A grows with beta


def test_overhead_ops_ratio():
    """Appendix C: overhead / (H N^2 d) = 1/N + 1/d."""
    H, N, d = 32, 2048, 128
    a, b = orc.overhead_ops(H, N, d)
    assert math.isclose((a + b) / (H * N * N * d), 1 / N + 1 / d)


# ---------------------------------------------------------------- per-token pieces vs closed forms / libraries
def test_linear_brute_force():
    rng = np.random.default_rng(0)
    x, w, b = rng.standard_normal((3, 5)), rng.standard_normal((4, 5)), rng.standard_normal(4)
    y = orc.linear(x, w, b)
    for r in range(3):
        for o in range(4):
            assert math.isclose(y[r, o], sum(x[r, i] * w[o, i] for i in range(5)) + b[o], rel_tol=1e-13)


def test_norms_closed_form_and_torch():
    x = np.array([[1.0, 2.0, 3.0, 4.0]])
    # mean 2.5, biased variance 1.25
    y = orc.layer_norm(x, np.ones(4), np.zeros(4), 0.0)
    np.testing.assert_allclose(y[0], (x[0] - 2.5) / math.sqrt(1.25), rtol=1e-14)
    y = orc.rms_norm(x, np.ones(4), 0.0)
    np.testing.assert_allclose(y[0], x[0] / math.sqrt(7.5), rtol=1e-14)
    rng = np.random.default_rng(1)
    x, g, b = rng.standard_normal((6, 16)), rng.standard_normal(16), rng.standard_normal(16)
    t = torch.nn.functional.layer_norm(torch.tensor(x), (16,), torch.tensor(g), torch.tensor(b), 1e-5)
    np.testing.assert_allclose(orc.layer_norm(x, g, b, 1e-5), t.numpy(), rtol=1e-12, atol=1e-14)
    t = torch.nn.functional.rms_norm(torch.tensor(x), (16,), torch.tensor(g), 1e-5)
    np.testing.assert_allclose(orc.rms_norm(x, g, 1e-5), t.numpy(), rtol=1e-12, atol=1e-14)


def test_activations_known_values_and_torch():
    assert orc.gelu_erf(np.array([0.0]))[0] == 0.0
    assert math.isclose(orc.gelu_erf(np.array([1.0]))[0], 0.8413447460685429, rel_tol=1e-14)   # Phi(1)
    assert math.isclose(orc.gelu_erf(np.array([-1.0]))[0], -0.15865525393145707, rel_tol=1e-13)
    assert math.isclose(orc.silu(np.array([1.0]))[0], 1 / (1 + math.exp(-1)), rel_tol=1e-15)
    x = np.linspace(-6, 6, 101)
    tx = torch.tensor(x)
    np.testing.assert_allclose(orc.gelu_erf(x), torch.nn.functional.gelu(tx).numpy(), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(orc.gelu_tanh(x), torch.nn.functional.gelu(tx, approximate="tanh").numpy(),
                               rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(orc.silu(x), torch.nn.functional.silu(tx).numpy(), rtol=1e-12, atol=1e-15)


def test_rope_properties():
    rng = np.random.default_rng(2)
    d, theta = 8, 10000.0
    x = rng.standard_normal((2, 5, d))
    pos = np.array([0, 3, 7, 11, 40])
    y = orc.rope(x, pos, theta)
    np.testing.assert_array_equal(y[:, 0], x[:, 0])                       # position 0: identity
    half = d // 2
    for i in range(half):                                                 # each pair keeps its norm
        np.testing.assert_allclose(y[..., i] ** 2 + y[..., i + half] ** 2,
                                   x[..., i] ** 2 + x[..., i + half] ** 2, rtol=1e-12)
    # d = 2: plain rotation by pos radians (theta**0 = 1)
    v = orc.rope(np.array([[1.0, 0.0]]), np.array([0.5]), 123.0)
    np.testing.assert_allclose(v[0], [math.cos(0.5), math.sin(0.5)], rtol=1e-15)
    # explicit frequency of pair i: theta**(-2i/d)
    one = np.zeros((1, d)); one[0, 1] = 1.0
    r = orc.rope(one, np.array([2.0]), theta)
    ang = 2.0 * theta ** (-2.0 / d)
    np.testing.assert_allclose([r[0, 1], r[0, 1 + half]], [math.cos(ang), math.sin(ang)], rtol=1e-14)
    # relative-position property: <R_p q, R_s k> depends on p - s only
    q, k = rng.standard_normal((1, d)), rng.standard_normal((1, d))
    def dot(p, s):
        return (orc.rope(q, np.array([p]), theta) @ orc.rope(k, np.array([s]), theta).T).item()
    assert math.isclose(dot(9, 4), dot(25, 20), rel_tol=1e-11)
    assert not math.isclose(dot(9, 4), dot(9, 5), rel_tol=1e-3)


# ---------------------------------------------------------------- Algorithm 3 pins
@pytest.mark.parametrize("kind,beta", [("perm", 4), ("contiguous", 3), ("roundrobin", 5), ("ragged", 6), ("roundrobin", 12)])
def test_partials_merge_equals_brute_force_attention(kind, beta):
    H, Hkv, N, d = 4, 2, 12, 3
    q, k, v = rand_qkv(5, H, Hkv, N, d)
    a = make_assignment(kind, N, beta, 9)
    m, e, u = orc.partial_attention_all_pairs(q, k, v, a, beta, scale=0.7)
    o = orc.lse_merge_all(m, e, u)                                  # packed rows
    _, perm, _ = orc.shard_plan(a, beta)
    want = brute_attention(q, k, v, np.arange(N), 0.7)              # (H, N, d) original order
    got = o.reshape(N, H, d).transpose(1, 0, 2)
    np.testing.assert_allclose(got, want[:, perm], rtol=1e-12, atol=1e-14)


def test_pair_identity_exp_a_v_equals_u_e_exp_m():
    """exp(a^{S_j S_k}) v^{S_k} = u * e * exp(m) (proof of the CompNode theorem, Section 6.3),
    right-hand side from the oracle, left-hand side by loops without any stabilisation."""
    H, Hkv, N, d, beta = 2, 1, 10, 3, 3
    q, k, v = rand_qkv(6, H, Hkv, N, d)
    a = make_assignment("perm", N, beta, 4)
    m, e, u = orc.partial_attention_all_pairs(q, k, v, a, beta, scale=1.0)
    lists = orc.shard_index_lists(a, beta)
    _, perm, _ = orc.shard_plan(a, beta)
    for kk, Sk in enumerate(lists):
        for r, x in enumerate(perm):
            for h in range(H):
                vis = [y for y in Sk if y <= x]
                direct = np.zeros(d)
                es = 0.0
                for y in vis:
                    p = math.exp(sum(q[h, x, i] * k[0, y, i] for i in range(d)))
                    direct += p * v[0, y]
                    es += p
                if not vis:
                    assert m[h, kk, r] == -np.inf and e[h, kk, r] == 0.0 and not u[kk, h, r].any()
                    continue
                np.testing.assert_allclose(u[kk, h, r] * e[h, kk, r] * math.exp(m[h, kk, r]), direct, rtol=1e-12)
                assert math.isclose(e[h, kk, r] * math.exp(m[h, kk, r]), es, rel_tol=1e-12)


def test_zero_queries_count_visible_keys_exactly():
    """q = 0: every logit is 0, so m = 0, e = number of visible keys of S_k (an integer),
    and the merged output is the mean of the visible values."""
    H, Hkv, N, d, beta = 2, 2, 16, 4, 4
    _, k, v = rand_qkv(7, H, Hkv, N, d)
    q = np.zeros((H, N, d))
    for kind in ("perm", "roundrobin", "contiguous"):
        a = make_assignment(kind, N, beta, 1)
        lists = orc.shard_index_lists(a, beta)
        _, perm, _ = orc.shard_plan(a, beta)
        m, e, u = orc.partial_attention_all_pairs(q, k, v, a, beta)
        for kk, Sk in enumerate(lists):
            cnt = np.array([(Sk <= x).sum() for x in perm])
            assert (e[:, kk] == cnt[None]).all()
            assert (m[:, kk][:, cnt > 0] == 0).all() and (m[:, kk][:, cnt == 0] == -np.inf).all()
        o = orc.lse_merge_all(m, e, u).reshape(N, H, d)
        for r, x in enumerate(perm):
            np.testing.assert_allclose(o[r], v[:, :x + 1].mean(axis=1), rtol=1e-13)


def test_tile_shapes_of_roundrobin_and_contiguous():
    """Round-robin shards give exactly lower-triangular tiles; contiguous shards give empty
    tiles above the diagonal (every e there is 0)."""
    N, beta, H, d = 12, 3, 1, 2
    q = np.zeros((H, N, d)); k = np.zeros((H, N, d)); v = np.ones((H, N, d))
    m, e, _ = orc.partial_attention_all_pairs(q, k, v, make_assignment("roundrobin", N, beta, 0), beta)
    size = N // beta
    for j in range(beta):
        for kk in range(beta):
            r = np.arange(size)
            want = r + (1 if kk <= j else 0)                  # col c visible iff c < r or (c == r and k <= j)
            assert (e[0, kk, j * size:(j + 1) * size] == want).all()
    m, e, _ = orc.partial_attention_all_pairs(q, k, v, make_assignment("contiguous", N, beta, 0), beta)
    for j in range(beta):
        for kk in range(beta):
            blk = e[0, kk, j * size:(j + 1) * size]
            if kk > j:
                assert (blk == 0).all()
            elif kk < j:
                assert (blk == size).all()
            else:
                assert (blk == np.arange(1, size + 1)).all()


def test_constant_values_give_constant_output():
    H, Hkv, N, d, beta = 2, 1, 14, 3, 4
    q, k, _ = rand_qkv(8, H, Hkv, N, d, amp=3.0)
    v = np.broadcast_to(np.array([1.5, -2.0, 0.25]), (Hkv, N, d)).copy()
    a = make_assignment("ragged", N, beta, 2)
    o = orc.lse_merge_all(*orc.partial_attention_all_pairs(q, k, v, a, beta))
    np.testing.assert_allclose(o.reshape(N, H, d), np.broadcast_to(v[0, 0], (N, H, d)), rtol=1e-13)


def test_stability_bounds():
    """m_k <= n; 1 <= e <= |S_k| on rows with a visible key (the paper's 'e <= 1' is a slip:
    the maximal term contributes exactly 1)."""
    H, Hkv, N, d, beta = 3, 3, 30, 4, 5
    q, k, v = rand_qkv(9, H, Hkv, N, d, amp=6.0)        # logits of a few hundred
    a = make_assignment("perm", N, beta, 5)
    m, e, u = orc.partial_attention_all_pairs(q, k, v, a, beta)
    sizes = np.bincount(a, minlength=beta)
    n = m.max(axis=1)
    assert np.isfinite(n).all()
    for kk in range(beta):
        seen = np.isfinite(m[:, kk])
        assert (e[:, kk][seen] >= 1.0).all() and (e[:, kk][seen] <= sizes[kk]).all()
        assert (e[:, kk][~seen] == 0).all()
        assert (m[:, kk] <= n).all()
    o = orc.lse_merge_all(m, e, u)
    assert np.isfinite(o).all()
    assert np.abs(m[np.isfinite(m)]).max() > 100                   # far beyond fp32 exp range: stabilisation matters
    want = brute_attention(q, k, v, np.arange(N), 1.0)             # unstabilised double-precision exp
    _, perm, _ = orc.shard_plan(a, beta)
    np.testing.assert_allclose(o.reshape(N, H, d).transpose(1, 0, 2), want[:, perm], rtol=1e-9)


def test_one_shard_is_textbook_attention_torch():
    """beta = 1: Algorithm 3 is stable softmax attention and Algorithm 4 is the identity;
    compare with torch's scaled_dot_product_attention in float64."""
    H, Hkv, N, d = 4, 2, 17, 8
    q, k, v = rand_qkv(10, H, Hkv, N, d)
    a = np.zeros(N, dtype=np.int32)
    m, e, u = orc.partial_attention_all_pairs(q, k, v, a, 1, scale=d ** -0.5)
    o = orc.lse_merge_all(m, e, u).reshape(N, H, d).transpose(1, 0, 2)
    np.testing.assert_allclose(o, u[0], rtol=1e-14)
    tq, tk, tv = (torch.tensor(t) for t in (q, np.repeat(k, 2, 0), np.repeat(v, 2, 0)))
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True).numpy()
    np.testing.assert_allclose(o, want, rtol=1e-11, atol=1e-13)
    # and the bidirectional case
    m, e, u = orc.partial_attention_all_pairs(q, k, v, a, 1, scale=d ** -0.5, mask_kind="none")
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).numpy()
    np.testing.assert_allclose(u[0], want, rtol=1e-11, atol=1e-13)


def test_singleton_shards():
    """beta = N: every visible pair has e = 1, u = the value row; merge = plain softmax."""
    H, Hkv, N, d = 2, 2, 9, 3
    q, k, v = rand_qkv(11, H, Hkv, N, d)
    a = np.arange(N, dtype=np.int32)
    m, e, u = orc.partial_attention_all_pairs(q, k, v, a, N)
    for kk in range(N):
        for r in range(N):
            if kk <= r:
                assert (e[:, kk, r] == 1).all()
                np.testing.assert_array_equal(u[kk, :, r], v[:, kk])
            else:
                assert (e[:, kk, r] == 0).all()
    o = orc.lse_merge_all(m, e, u).reshape(N, H, d).transpose(1, 0, 2)
    np.testing.assert_allclose(o, brute_attention(q, k, v, np.arange(N), 1.0), rtol=1e-12)


def test_merge_is_associative():
    """Merging all partials equals merging the merges of any grouping (expsum identity of the
    Post-Pass subsection applied twice)."""
    H, Hkv, N, d, beta = 2, 1, 12, 3, 6
    q, k, v = rand_qkv(12, H, Hkv, N, d, amp=4.0)
    a = make_assignment("roundrobin", N, beta, 0)
    m, e, u = orc.partial_attention_all_pairs(q, k, v, a, beta, mask_kind="none")
    full = orc.post_pass_merge(list(m.transpose(1, 0, 2)), list(e.transpose(1, 0, 2)), list(u))
    groups = [[0, 3], [1, 2, 5], [4]]
    gm, ge, gu = [], [], []
    for g in groups:
        ms, es, us = [m[:, t] for t in g], [e[:, t] for t in g], [u[t] for t in g]
        n = np.max(ms, axis=0)
        w = sum(np.exp(mm - n) * ee for mm, ee in zip(ms, es))
        gm.append(n); ge.append(w); gu.append(orc.post_pass_merge(ms, es, us))
    np.testing.assert_allclose(orc.post_pass_merge(gm, ge, gu), full, rtol=1e-13)


def test_custom_positions_define_the_mask():
    """The mask follows the positions array, not the row number."""
    H, Hkv, N, d, beta = 1, 1, 8, 2, 2
    q, k, v = rand_qkv(13, H, Hkv, N, d)
    pos = np.array([5, 2, 7, 0, 3, 6, 1, 4])
    a = make_assignment("roundrobin", N, beta, 0)
    o = orc.lse_merge_all(*orc.partial_attention_all_pairs(q, k, v, a, beta, positions=pos))
    _, perm, _ = orc.shard_plan(a, beta)
    want = brute_attention(q, k, v, pos, 1.0)
    np.testing.assert_allclose(o.reshape(N, H, d).transpose(1, 0, 2), want[:, perm], rtol=1e-12)


# ---------------------------------------------------------------- whole layer
def brute_layer(h, w, cfg):
    """The pre-norm layer written with Python loops for the contractions (tiny shapes only)."""
    N, D = h.shape
    H, Hkv, d = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim

    def lin(x, W, b):
        out = np.zeros((x.shape[0], W.shape[0]))
        for r in range(x.shape[0]):
            for o in range(W.shape[0]):
                out[r, o] = sum(x[r, i] * W[o, i] for i in range(W.shape[1])) + (0.0 if b is None else b[o])
        return out

    def nrm(x, g, b):
        out = np.zeros_like(x)
        for r in range(x.shape[0]):
            row = x[r]
            if cfg.norm == "layernorm":
                mu = sum(row) / D
                var = sum((t - mu) ** 2 for t in row) / D
                out[r] = [(t - mu) / math.sqrt(var + cfg.eps) * g[i] + b[i] for i, t in enumerate(row)]
            else:
                ms = sum(t * t for t in row) / D
                out[r] = [t / math.sqrt(ms + cfg.eps) * g[i] for i, t in enumerate(row)]
        return out

    def rot(x, p):       # x (d,)
        half = d // 2
        y = x.copy()
        for i in range(half):
            ang = p * cfg.rope_theta ** (-2.0 * i / d)
            y[i] = x[i] * math.cos(ang) - x[i + half] * math.sin(ang)
            y[i + half] = x[i + half] * math.cos(ang) + x[i] * math.sin(ang)
        return y

    post = getattr(cfg, "norm_placement", "pre") == "post"
    x = h if post else nrm(h, w["norm1_g"], w.get("norm1_b"))
    q = lin(x, w["wq"], w.get("bq")).reshape(N, H, d).transpose(1, 0, 2).copy()
    k = lin(x, w["wk"], w.get("bk")).reshape(N, Hkv, d).transpose(1, 0, 2).copy()
    v = lin(x, w["wv"], w.get("bv")).reshape(N, Hkv, d).transpose(1, 0, 2).copy()
    if cfg.rope:
        for t in range(N):
            for hh in range(H):
                q[hh, t] = rot(q[hh, t], t)
            for hh in range(Hkv):
                k[hh, t] = rot(k[hh, t], t)
    o = brute_attention(q, k, v, np.arange(N), cfg.scale).transpose(1, 0, 2).reshape(N, H * d)
    h1 = h + lin(o, w["wo"], w.get("bo"))
    if post:
        h1 = nrm(h1, w["norm1_g"], w.get("norm1_b"))
    x2 = h1 if post else nrm(h1, w["norm2_g"], w.get("norm2_b"))
    if cfg.act == "swiglu":
        g = lin(x2, w["w_gate"], None)
        up = lin(x2, w["w_up"], None)
        act = np.array([[gg / (1 + math.exp(-gg)) * uu for gg, uu in zip(gr, ur)] for gr, ur in zip(g, up)])
        out = h1 + lin(act, w["w_down"], None)
    else:
        up = lin(x2, w["w_up"], w.get("b_up"))
        act = np.array([[0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in row] for row in up])
        out = h1 + lin(act, w["w_down"], w.get("b_down"))
    return nrm(out, w["norm2_g"], w.get("norm2_b")) if post else out


@pytest.mark.parametrize("cfg", [TINY_LLAMA.with_(seq_len=7, d_model=12, n_heads=2, n_kv_heads=1, head_dim=4, d_ff=10),
                                 TINY_GPT.with_(seq_len=6, d_model=10, n_heads=2, n_kv_heads=2, head_dim=4, d_ff=9),
                                 TINY_GPT.with_(seq_len=6, d_model=10, n_heads=2, n_kv_heads=2, head_dim=4, d_ff=9,
                                                norm_placement="post"),
                                 TINY_LLAMA.with_(seq_len=5, d_model=8, n_heads=2, n_kv_heads=2, head_dim=4, d_ff=6,
                                                  norm_placement="post")])
def test_layer_direct_equals_brute_force_layer(cfg):
    w = {k: v.astype(np.float64) * 10 for k, v in make_layer_weights(cfg).items()}   # x10: make every term matter
    for key in ("norm1_g", "norm2_g"):
        w[key] = w[key] / 10
    h = make_hidden(cfg)[0].astype(np.float64)
    np.testing.assert_allclose(orc.layer_direct(h, w, cfg), brute_layer(h, w, cfg), rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("cfg", [TINY_LLAMA, TINY_GPT])
@pytest.mark.parametrize("kind", ["perm", "contiguous", "roundrobin", "ragged", "singleton", "one"])
def test_layer_sharded_equals_layer_direct(cfg, kind):
    w = make_layer_weights(cfg)
    w = {k: v * (8.0 if v.ndim == 2 else 1.0) for k, v in w.items()}       # logits of order 1
    h = make_hidden(cfg)[0]
    N = cfg.seq_len
    if kind == "singleton":
        beta, a = N, np.arange(N, dtype=np.int32)
    elif kind == "one":
        beta, a = 1, np.zeros(N, dtype=np.int32)
    else:
        beta = cfg.n_shards
        a = make_assignment(kind, N, beta, 17)
    direct = orc.layer_direct(h, w, cfg)
    sharded = orc.layer_sharded(h, w, cfg, a, beta)
    assert rel_err(sharded, direct) < 1e-12
    # rows= path computes the same rows
    rows = np.array([0, 5, N - 1])
    assert rel_err(orc.layer_direct(h, w, cfg, rows=rows), direct[rows]) < 1e-13


def test_layer_output_is_invariant_under_resharding():
    cfg = TINY_LLAMA
    w, h = make_layer_weights(cfg), make_hidden(cfg)[0]
    base = orc.layer_sharded(h, w, cfg, make_assignment("perm", cfg.seq_len, 4, 1), 4)
    for seed, beta in [(2, 4), (3, 6), (4, 3)]:
        other = orc.layer_sharded(h, w, cfg, make_assignment("perm", cfg.seq_len, beta, seed), beta)
        assert rel_err(other, base) < 1e-12


def test_layer_bidirectional_mask():
    cfg = TINY_GPT
    w, h = make_layer_weights(cfg), make_hidden(cfg)[0]
    a = make_assignment("perm", cfg.seq_len, cfg.n_shards, 3)
    d1 = orc.layer_direct(h, w, cfg, mask_kind="none")
    d2 = orc.layer_sharded(h, w, cfg, a, cfg.n_shards, mask_kind="none")
    assert rel_err(d2, d1) < 1e-12
    assert rel_err(orc.layer_direct(h, w, cfg), d1) > 1e-6       # the mask matters


def test_partials_from_layer_match_standalone_pairs():
    cfg = TINY_LLAMA
    w, h = make_layer_weights(cfg), make_hidden(cfg)[0]
    a = make_assignment("perm", cfg.seq_len, cfg.n_shards, 8)
    _, partial = orc.layer_sharded(h, w, cfg, a, cfg.n_shards, return_partials=True)
    w64 = {k: v.astype(np.float64) for k, v in w.items()}
    q, k, v = orc.pre_pass(h.astype(np.float64), np.arange(cfg.seq_len), w64, cfg)
    m, e, u = orc.partial_attention_all_pairs(q, k, v, a, cfg.n_shards, scale=cfg.scale)
    offsets, _, _ = orc.shard_plan(a, cfg.n_shards)
    for (j, kk), (mj, ej, uj) in partial.items():
        sl = slice(offsets[j], offsets[j + 1])
        np.testing.assert_allclose(m[:, kk, sl], mj, rtol=1e-12)
        np.testing.assert_allclose(e[:, kk, sl], ej, rtol=1e-12)
        np.testing.assert_allclose(u[kk][:, sl], uj, rtol=1e-11, atol=1e-14)


# ---------------------------------------------------------------- distinct hidden / key-value shardings (R != S)
def test_m_split_assignment_matches_the_worked_example():
    """Section 6.4: S_{m(i-1)+x} = R_{i,x}; with the N = 18 example, token t of R_{i,x} (1-based) must get
    0-based kv shard m (i-1) + (x-1)."""
    _, RX, _ = _read_example()
    a = orc.cdelta_assignment(18, c=2, delta=6)
    kv = orc.m_split_assignment(a, 3, 2)
    want = np.empty(18, dtype=np.int64)
    for (i, x), toks in RX.items():
        for t in toks:
            want[t - 1] = 2 * (i - 1) + (x - 1)
    assert kv.tolist() == want.tolist()
    # each kv shard lies inside one row shard, and the pieces of a row shard interleave
    for s in range(6):
        assert set(a[kv == s].tolist()) == {s // 2}


def _rs_partitions(N, kind, seed):
    if kind == "msplit":                                  # (c, delta) rows, m-split kv shards (the paper's scheme)
        a = orc.cdelta_assignment(N, 2, 8)
        return a, 4, orc.m_split_assignment(a, 4, 2), 8
    if kind == "coarser":                                 # kv shards that are unions of row shards
        a = make_assignment("perm", N, 6, seed)
        return a, 6, (a // 2).astype(np.int32), 3
    a = make_assignment("ragged", N, 4, seed)             # unrelated partitions
    return a, 4, make_assignment("perm", N, 5, seed + 1), 5


@pytest.mark.parametrize("kind", ["msplit", "coarser", "unrelated"])
def test_partials_with_two_shardings_are_the_single_sharding_partials_rerouted(kind):
    """A partial (m, e, u) of query row t against kv shard S_k does not depend on how rows are sharded:
    partial_attention_rs must hold, at R-packed row inv_perm_R[t], what the single-partition routine
    (pinned by brute force above) holds at S-packed row inv_perm_S[t]."""
    H, Hkv, N, d = 4, 2, 24, 8
    q, k, v = rand_qkv(21, H, Hkv, N, d)
    a, alpha, kv, beta = _rs_partitions(N, kind, 5)
    pos = np.random.default_rng(3).permutation(3 * N)[:N]
    m, e, u = orc.partial_attention_rs(q, k, v, a, alpha, kv, beta, positions=pos, scale=0.3)
    m1, e1, u1 = orc.partial_attention_all_pairs(q, k, v, kv, beta, positions=pos, scale=0.3)
    _, _, inv_r = orc.shard_plan(a, alpha)
    _, _, inv_s = orc.shard_plan(kv, beta)
    np.testing.assert_array_equal(m[:, :, inv_r], m1[:, :, inv_s])
    np.testing.assert_array_equal(e[:, :, inv_r], e1[:, :, inv_s])
    np.testing.assert_array_equal(u[:, :, inv_r], u1[:, :, inv_s])
    # and merged over the kv shards they give plain attention, rows in R-packed order
    _, perm_r, _ = orc.shard_plan(a, alpha)
    o = orc.lse_merge_all(m, e, u).reshape(N, H, d).transpose(1, 0, 2)
    want = brute_attention(q, k, v, pos, 0.3)[:, perm_r]
    np.testing.assert_allclose(o, want, rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("cfg", [TINY_LLAMA, TINY_GPT])
@pytest.mark.parametrize("kind", ["msplit", "coarser", "unrelated"])
def test_layer_with_two_shardings_equals_layer_direct(cfg, kind):
    w = make_layer_weights(cfg)
    w = {k: v * (8.0 if v.ndim == 2 else 1.0) for k, v in w.items()}
    h = make_hidden(cfg)[0]
    a, alpha, kv, beta = _rs_partitions(cfg.seq_len, kind, 9)
    direct = orc.layer_direct(h, w, cfg)
    assert rel_err(orc.layer_sharded_rs(h, w, cfg, a, alpha, kv, beta), direct) < 1e-12
    # with S = R it is Algorithm 1 as implemented by layer_sharded
    assert rel_err(orc.layer_sharded_rs(h, w, cfg, a, alpha, a, alpha), orc.layer_sharded(h, w, cfg, a, alpha)) < 1e-13


# ---------------------------------------------------------------- token-sharded KV-cache decode
def _cache_shards(k, v, assign, beta):
    lists = orc.shard_index_lists(assign, beta)
    return [k[:, S] for S in lists], [v[:, S] for S in lists]


def test_decode_merge_is_plain_attention_of_the_last_row():
    """Brute force: the newest token attends every cached token (its own included)."""
    H, Hkv, N, d = 4, 2, 19, 6
    q, k, v = rand_qkv(31, H, Hkv, N, d)
    want = brute_attention(q, k, v, np.arange(N), 0.4)[:, N - 1]            # last row sees all N keys
    for beta, kind, seed in [(1, "perm", 0), (4, "perm", 1), (5, "ragged", 2), (N, "singleton", 0), (8, "ragged", 3)]:
        a = np.arange(N, dtype=np.int32) if kind == "singleton" else make_assignment(kind, N, beta, seed)
        ks, vs = _cache_shards(k, v, a, beta)
        m, e, u = orc.decode_partials(q[:, N - 1], ks, vs, 0.4)
        np.testing.assert_allclose(orc.decode_merge(m, e, u), want.reshape(-1), rtol=1e-11, atol=1e-13)
        assert ((e >= 1.0) | (e == 0.0)).all()
        sizes = np.array([x.shape[1] for x in ks])
        assert (e <= sizes[None, :] + 1e-12).all()
        assert (np.isneginf(m) == (sizes[None, :] == 0)).all()             # empty cache shard: (-inf, 0, 0)
        assert (u[sizes == 0] == 0).all()


def test_decode_partials_are_the_prefill_partials_of_the_last_token():
    """The cached-decode partials of the newest token equal row N-1 of the prefill partials of the
    same sequence under the same sharding (the causal mask hides nothing from the last token)."""
    H, Hkv, N, d, beta = 4, 4, 24, 8, 4
    q, k, v = rand_qkv(32, H, Hkv, N, d)
    a = make_assignment("perm", N, beta, 6)
    m1, e1, u1 = orc.partial_attention_all_pairs(q, k, v, a, beta, scale=0.35)
    _, _, inv = orc.shard_plan(a, beta)
    ks, vs = _cache_shards(k, v, a, beta)
    m, e, u = orc.decode_partials(q[:, N - 1], ks, vs, 0.35)
    r = inv[N - 1]
    np.testing.assert_allclose(m, m1[:, :, r], rtol=1e-13)
    np.testing.assert_allclose(e, e1[:, :, r], rtol=1e-12)
    np.testing.assert_allclose(u, u1[:, :, r], rtol=1e-11, atol=1e-14)


def test_decode_single_key_shards():
    """beta = N: every shard caches one key, so m = scale q.k, e = 1 and u is that key's value row."""
    H, Hkv, N, d = 2, 1, 5, 4
    q, k, v = rand_qkv(33, H, Hkv, N, d)
    ks, vs = _cache_shards(k, v, np.arange(N, dtype=np.int32), N)
    m, e, u = orc.decode_partials(q[:, N - 1], ks, vs, 0.5)
    assert np.allclose(e, 1.0)
    for kk in range(N):
        for h in range(H):
            assert abs(m[h, kk] - 0.5 * float(q[h, N - 1] @ k[0, kk])) < 1e-13
            np.testing.assert_allclose(u[kk, h], v[0, kk], rtol=1e-13)


# ---------------------------------------------------------------- post-norm block, layer stack
@pytest.mark.parametrize("cfg", [TINY_GPT.with_(norm_placement="post"), TINY_LLAMA.with_(norm_placement="post")])
@pytest.mark.parametrize("mask_kind", ["causal", "none"])
def test_post_norm_layer_sharded_equals_direct(cfg, mask_kind):
    """The BERT-shaped block (norm after each residual sum), bidirectional or causal."""
    w = make_layer_weights(cfg)
    w = {k: v * (8.0 if v.ndim == 2 else 1.0) for k, v in w.items()}
    h = make_hidden(cfg)[0]
    a = make_assignment("perm", cfg.seq_len, cfg.n_shards, 4)
    direct = orc.layer_direct(h, w, cfg, mask_kind=mask_kind)
    assert rel_err(orc.layer_sharded(h, w, cfg, a, cfg.n_shards, mask_kind=mask_kind), direct) < 1e-12
    assert rel_err(orc.layer_direct(h, w, cfg.with_(norm_placement="pre"), mask_kind=mask_kind), direct) > 1e-3
    # every output row of a post-norm layer is normalised: zero mean / unit variance before gain and bias
    if cfg.norm == "layernorm":
        z = (direct - w["norm2_b"]) / w["norm2_g"]
        assert np.abs(z.mean(axis=1)).max() < 1e-9 and np.abs(z.var(axis=1) - 1).max() < 1e-3


def test_layer_stack_is_the_composition_of_layers_under_any_sharding():
    cfg = TINY_LLAMA
    ws = [make_layer_weights(cfg.with_(index=40 + l)) for l in range(3)]
    ws = [{k: v * (6.0 if v.ndim == 2 else 1.0) for k, v in w.items()} for w in ws]
    h = make_hidden(cfg)[0]
    want = h.astype(np.float64)
    for w in ws:
        want = orc.layer_direct(want, w, cfg)
    assert rel_err(orc.layer_stack_direct(h, ws, cfg), want) == 0
    for seed, beta in [(1, 4), (2, 6)]:
        a = make_assignment("perm", cfg.seq_len, beta, seed)
        assert rel_err(orc.layer_stack_sharded(h, ws, cfg, a, beta), want) < 1e-11


# ---------------------------------------------------------------- LM head on sharded rows
@pytest.mark.parametrize("cfg", [TINY_LLAMA, TINY_GPT], ids=lambda c: c.name)
def test_lm_head_direct_equals_brute_force(cfg):
    """Closing norm and vocabulary projection from their definitions, Python loops."""
    from cascade_inputs import make_head_weights
    V = 37
    head = make_head_weights(cfg, V)
    head = {k: v * (8.0 if v.ndim == 2 else 1.0) for k, v in head.items()}
    h = make_hidden(cfg)[0].astype(np.float64)
    N, D = h.shape
    want = np.zeros((N, V))
    for t in range(N):
        row = [float(x) for x in h[t]]
        if cfg.norm == "layernorm":
            mu = sum(row) / D
            var = sum((x - mu) ** 2 for x in row) / D
            xn = [(x - mu) / math.sqrt(var + cfg.eps) * float(head["norm_g"][i]) + float(head["norm_b"][i])
                  for i, x in enumerate(row)]
        else:
            ms = sum(x * x for x in row) / D
            xn = [x / math.sqrt(ms + cfg.eps) * float(head["norm_g"][i]) for i, x in enumerate(row)]
        for c in range(V):
            want[t, c] = sum(xn[i] * float(head["w_vocab"][c, i]) for i in range(D))
    assert rel_err(orc.lm_head_direct(h, head, cfg), want) < 1e-13


def test_lm_head_sharded_equals_direct_and_names_the_owner_of_the_last_token():
    from cascade_inputs import make_head_weights
    cfg = TINY_LLAMA
    V = 53
    head = make_head_weights(cfg, V)
    head["w_vocab"] = head["w_vocab"] * 8.0
    h = make_hidden(cfg)[0]
    direct = orc.lm_head_direct(h, head, cfg)
    for kind, beta, seed in [("perm", 4, 1), ("roundrobin", 6, 2), ("ragged", 5, 3), ("contiguous", 3, 4)]:
        a = make_assignment(kind, cfg.seq_len, beta, seed)
        assert rel_err(orc.lm_head_sharded(h, head, cfg, a, beta), direct) < 1e-13  # same rows, row-wise arithmetic
        tok, shard, row = orc.next_token(h, head, cfg, a, beta)
        assert shard == a[cfg.seq_len - 1] and tok == int(np.argmax(direct[-1])) and rel_err(row, direct[-1]) < 1e-13
    # custom positions: the last token is the one with the largest position, wherever it is stored
    pos = np.random.default_rng(5).permutation(cfg.seq_len) * 3 + 2
    a = make_assignment("perm", cfg.seq_len, 4, 6)
    tok, shard, row = orc.next_token(h, head, cfg, a, 4, positions=pos)
    t_last = int(np.argmax(pos))
    assert shard == a[t_last] and tok == int(np.argmax(direct[t_last]))
    # ties go to the lowest index (rows 2 and 7 equal and largest, exactly: one-hot rows pick a coordinate)
    head2 = dict(head)
    w2 = np.zeros((9, cfg.d_model))
    w2[2, 0] = w2[7, 0] = 1.0
    head2["w_vocab"] = w2
    h2 = np.abs(h) + 0.5                                  # coordinate 0 of the normalised row is positive
    tok2, _, row2 = orc.next_token(h2, head2, cfg, a, 4)
    assert tok2 == 2 and row2[2] == row2[7] > 0


def test_lm_head_identity_projection_returns_the_normalised_row():
    """W_vocab = I: the logits are the closing norm's output, whose rows have unit mean square before the gain."""
    from cascade_inputs import make_head_weights
    cfg = TINY_LLAMA
    head = make_head_weights(cfg, cfg.d_model)
    head["w_vocab"] = np.eye(cfg.d_model)
    h = make_hidden(cfg)[0]
    z = orc.lm_head_direct(h, head, cfg) / head["norm_g"].astype(np.float64)
    assert np.abs((z ** 2).mean(axis=1) - 1).max() < 1e-4
