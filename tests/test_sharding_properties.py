"""Properties of the (c, delta)-sharding and the m-split that follow from their definitions
(Section 6: the (c, delta)-sequence definition, the cluster-gap remark of the vocab-matching
paragraph, the m-split of the AttnNode Full Security subsection), checked on randomly drawn
parameters against BOTH generators: the library's C entry points and the oracle's.  Neither
formula is retyped here: the expected sets are built element by element from the definition."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import paper_2507_05228_amd as cas
from oracle import cascade_oracle as orc


def _both(N, c, delta):
    a_lib, n_lib = cas.cascade_cdelta_assignment(N, c, delta)
    a_orc = orc.cdelta_assignment(N, c, delta)
    return [("library", a_lib, n_lib), ("oracle", a_orc, int(a_orc.max()) + 1 if N else 0)]


def _sequence_from_definition(N, start, width, delta):
    """{start .. start+width-1, delta+start .. delta+start+width-1, 2 delta + ...} inside [0, N)."""
    out = []
    base = start
    while base < N:
        for t in range(base, min(base + width, N)):
            out.append(t)
        base += delta
    return out


params = st.tuples(st.integers(1, 400), st.integers(1, 12), st.integers(1, 96)).filter(lambda p: p[1] <= p[2])


@settings(max_examples=150, deadline=None, derandomize=True)
@given(params)
def test_every_shard_is_a_c_delta_sequence_and_the_shards_partition_the_tokens(p):
    N, c, delta = p
    alpha = -(-delta // c)
    for name, a, n in _both(N, c, delta):
        assert len(a) == N
        if name == "library":
            assert n == alpha, name
        seen = np.zeros(N, dtype=int)
        for i in range(alpha):
            width = min(c, delta - i * c)                     # the last shard's clusters may be shorter
            expect = _sequence_from_definition(N, i * c, width, delta)
            got = np.nonzero(a == i)[0].tolist()
            assert got == expect, (name, i)
            seen[got] += 1
        assert (seen == 1).all(), name


@settings(max_examples=100, deadline=None, derandomize=True)
@given(params)
def test_gap_between_the_clusters_of_a_shard(p):
    """From the last index of a cluster to the first of the next one: delta - c + 1 (full clusters)."""
    N, c, delta = p
    for name, a, _ in _both(N, c, delta):
        for i in range(int(a.max()) + 1 if N else 0):
            idx = np.nonzero(a == i)[0]
            jumps = np.diff(idx)
            width = min(c, delta - i * c)
            assert set(jumps.tolist()) <= {1, delta - width + 1}, (name, i)


msplit_params = st.tuples(st.integers(1, 300), st.integers(1, 8), st.integers(1, 64), st.integers(1, 6)).filter(
    lambda p: p[1] <= p[2])


@settings(max_examples=150, deadline=None, derandomize=True)
@given(msplit_params)
def test_m_split_partitions_every_row_shard_into_interleaved_pieces(p):
    N, c, delta, m = p
    a, alpha = cas.cascade_cdelta_assignment(N, c, delta)
    for name, kv in (("library", cas.cascade_m_split(a, alpha, m)), ("oracle", orc.m_split_assignment(a, alpha, m))):
        assert len(kv) == N
        for i in range(alpha):
            R = np.nonzero(a == i)[0]                         # sorted row shard
            pieces = [np.nonzero(kv == m * i + x)[0] for x in range(m)]
            # S_{m i + x} = R_{i,x}: a subset of R_i, the pieces partition it
            assert sorted(np.concatenate(pieces).tolist()) == R.tolist(), (name, i)
            # piece x holds the elements at ranks x, x + m, x + 2m, ... of sorted R_i
            for x in range(m):
                assert pieces[x].tolist() == [R[r] for r in range(x, len(R), m)], (name, i, x)
            sizes = [len(q) for q in pieces]
            assert max(sizes) - min(sizes) <= 1


@settings(max_examples=100, deadline=None, derandomize=True)
@given(st.tuples(st.integers(2, 8), st.integers(2, 8), st.integers(1, 6)))
def test_with_m_equal_c_the_pieces_are_delta_apart_and_no_attn_node_sees_three_neighbours(p):
    """Section 6.4: with m = c (and c dividing delta) the elements of R_{i,x} are delta positions
    apart, and S_j union S_k never holds three consecutive tokens when delta > 2."""
    c, alpha, t = p
    delta = c * alpha
    N = delta * t
    a, n = cas.cascade_cdelta_assignment(N, c, delta)
    assert n == alpha
    kv = cas.cascade_m_split(a, alpha, c)
    beta = c * alpha
    pieces = [np.nonzero(kv == j)[0] for j in range(beta)]
    for q in pieces:
        assert len(q) == t
        assert (np.diff(q) == delta).all()
    for j in range(beta):
        for k in range(j, beta):
            u = np.union1d(pieces[j], pieces[k])
            runs = np.diff(u) == 1
            assert not (runs[:-1] & runs[1:]).any(), (j, k)
