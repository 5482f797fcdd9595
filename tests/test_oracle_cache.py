"""Pins for the oracle's cache draw (paper Section 3.2, Eq. (1); Theorem 1:
drawn without replacement, |C| nodes).

 - a single stream draw lands on node i with probability deg(i)/sum deg
   (chi-square against the closed form of Eq. (1));
 - the cache is successive weighted sampling without replacement: exact
   inclusion probabilities obtained by enumerating every ordered draw sequence
   on a tiny graph are compared with frequencies over many seeds;
 - Section 3.4's p^C = 1-(1-p)^|C| is the inclusion probability of the first
   |C| stream draws: checked empirically and against exact rationals;
 - invariants: |C| distinct nodes, none of degree 0, ascending, bitmap and
   num_draws consistent with the stream, superset of the i.i.d. prefix set.
"""
from fractions import Fraction
from itertools import permutations

import numpy as np
import pytest
from scipy import stats

import oracle
from conftest import random_symmetric_csr


def tiny_graph():
    # 7 nodes, degrees 4,3,3,2,2,2,0 (node 6 isolated); symmetric
    edges = [(0, 1), (0, 2), (0, 3), (0, 4), (1, 2), (1, 5), (2, 3), (4, 5)]
    n = 7
    adj = [[] for _ in range(n)]
    for a, b in edges:
        adj[a].append(b)
        adj[b].append(a)
    indptr = np.zeros(n + 1, dtype=np.int64)
    indices = []
    for i in range(n):
        indptr[i + 1] = indptr[i] + len(adj[i])
        indices += sorted(adj[i])
    return indptr, np.array(indices, dtype=np.int32)


def test_single_draw_is_degree_proportional():
    rng = np.random.default_rng(11)
    indptr, _ = random_symmetric_csr(60, 8, rng, hub_boost=1)
    deg = np.diff(indptr).astype(np.float64)
    N = 120_000
    counts = np.zeros(60)
    for j in range(N):
        counts[oracle.cache_draw_node(indptr, 99, 3, j)] += 1
    assert counts[deg == 0].sum() == 0
    nz = deg > 0
    chi = stats.chisquare(counts[nz], N * deg[nz] / deg.sum())
    assert chi.pvalue > 1e-4, chi


def test_single_draw_uses_row_owner_of_a_uniform_entry():
    # degrees 1,0,3: entries 0 | 1,2,3 -> node 0 w.p. 1/4, node 2 w.p. 3/4, node 1 never
    indptr = np.array([0, 1, 1, 4], dtype=np.int64)
    got = np.bincount([oracle.cache_draw_node(indptr, 5, 0, j) for j in range(40_000)], minlength=3)
    assert got[1] == 0
    assert abs(got[0] / 40_000 - 0.25) < 0.01


def test_cache_stream_keying_and_range_map():
    """Draw j of the cache stream of (seed, epoch): the Philox block with counter (j low, j high, epoch, tag) under the
    key (seed low, seed high) gives r = word1 * 2^32 + word0, the entry is floor(r * nnz / 2^64) and the node is the
    row that owns it.  Pinned against the word-size-generic Philox of test_oracle_philox and Python integers, on
    ragged degrees, stream positions above 2^32, epochs and seeds above 2^32."""
    from test_oracle_philox import philox4_generic, M32, W32
    tag = 0x43414348                                    # the cache stream's counter word
    rng = np.random.default_rng(3)
    deg = rng.integers(0, 50, size=400)
    deg[::7] = 0
    indptr = np.zeros(401, dtype=np.int64)
    indptr[1:] = np.cumsum(deg)
    nnz = int(indptr[-1])
    for seed in (9, (3 << 40) | 77):
        for epoch in (0, 5, (1 << 31) + 3):
            for j in (0, 1, 2, 1000, (1 << 32) + 5, (1 << 40) + 123):
                w = philox4_generic((j & 0xFFFFFFFF, j >> 32, epoch & 0xFFFFFFFF, tag), (seed & 0xFFFFFFFF, seed >> 32), 32, M32, W32)
                r = (w[1] << 32) | w[0]
                e = (r * nnz) >> 64
                node = int(np.searchsorted(indptr, e, side="right")) - 1
                assert oracle.cache_draw_node(indptr, seed, epoch, j) == node, (seed, epoch, j)


def exact_wor_inclusion(p, c):
    """Successive sampling without replacement: P(sequence) = prod p_i/(1 - mass already taken)."""
    n = len(p)
    incl = [Fraction(0)] * n
    support = [i for i in range(n) if p[i] > 0]
    for seq in permutations(support, c):
        pr, used = Fraction(1), Fraction(0)
        for i in seq:
            pr *= p[i] / (1 - used)
            used += p[i]
        for i in seq:
            incl[i] += pr
    return incl


@pytest.mark.parametrize("c", [1, 2, 3])
def test_cache_inclusion_matches_exact_without_replacement(c):
    indptr, _ = tiny_graph()
    deg = np.diff(indptr)
    p = [Fraction(int(d), int(deg.sum())) for d in deg]
    incl = exact_wor_inclusion(p, c)
    assert sum(incl) == c
    T = 20_000
    counts = np.zeros(7)
    for seed in range(T):
        nodes, bitmap, nd = oracle.sample_cache(indptr, seed, 0, c)
        assert len(set(nodes.tolist())) == c
        counts[nodes] += 1
    assert counts[6] == 0
    # per-node binomial z-scores against the exact inclusion probability
    for i in range(6):
        pi = float(incl[i])
        z = (counts[i] - T * pi) / np.sqrt(T * pi * (1 - pi))
        assert abs(z) < 4.5, (i, counts[i] / T, pi)


def test_p_cache_formula_is_the_iid_prefix_inclusion_probability():
    indptr, _ = tiny_graph()
    deg = np.diff(indptr)
    c = 3
    T = 20_000
    counts = np.zeros(7)
    for seed in range(T):
        prefix = {oracle.cache_draw_node(indptr, seed, 1, j) for j in range(c)}
        for i in prefix:
            counts[i] += 1
    for i in range(6):
        p = Fraction(int(deg[i]), int(deg.sum()))
        exact = 1 - (1 - p) ** c
        assert abs(oracle.p_cache(float(p), c) - float(exact)) < 1e-15
        z = (counts[i] - T * float(exact)) / np.sqrt(T * float(exact) * (1 - float(exact)))
        assert abs(z) < 4.5


def test_p_cache_numerics_against_high_precision():
    from decimal import Decimal, getcontext
    getcontext().prec = 60
    for deg_u, nnz, c in [(1, 1_600_000_000, 1_110_000), (20_000, 1_600_000_000, 1_110_000),
                          (37, 39_753_424, 10_000), (6102, 39_753_424, 10_000), (1, 3, 2)]:
        p = Decimal(deg_u) / Decimal(nnz)
        exact = 1 - (1 - p) ** c
        got = oracle.p_cache(deg_u / nnz, c)
        assert abs(Decimal(got) - exact) / exact < Decimal("1e-13")
    # limits: |C| p << 1 -> |C| p ; p = 1 -> 1
    assert abs(oracle.p_cache(1e-12, 1000) / 1e-9 - 1) < 1e-6
    assert oracle.p_cache(1.0, 5) == 1.0


def test_cache_invariants_and_stream_consistency(small_graph):
    indptr, _ = small_graph
    n = len(indptr) - 1
    deg = np.diff(indptr)
    for seed, epoch, c in [(1, 0, 1), (1, 1, 17), (2, 0, 64), (3, 5, 200)]:
        nodes, bitmap, nd = oracle.sample_cache(indptr, seed, epoch, c)
        assert len(nodes) == c and np.all(np.diff(nodes) > 0)
        assert np.all(deg[nodes] > 0)
        bits = np.unpackbits(bitmap.view(np.uint8), bitorder="little")[:n]
        assert np.array_equal(np.flatnonzero(bits), nodes)
        stream = [oracle.cache_draw_node(indptr, seed, epoch, j) for j in range(nd)]
        assert set(stream) == set(nodes.tolist())                 # exactly the distinct nodes of the used prefix
        assert stream[-1] not in stream[:-1]                       # the last used draw brought a new node
        assert set(stream[:c]) <= set(nodes.tolist())              # i.i.d. prefix set is contained
        assert nd >= c


def test_cache_depends_on_seed_and_epoch_only(small_graph):
    indptr, _ = small_graph
    a = oracle.sample_cache(indptr, 10, 0, 40)[0]
    assert np.array_equal(a, oracle.sample_cache(indptr, 10, 0, 40)[0])
    assert not np.array_equal(a, oracle.sample_cache(indptr, 10, 1, 40)[0])
    assert not np.array_equal(a, oracle.sample_cache(indptr, 11, 0, 40)[0])


def test_cache_larger_than_support_is_reported():
    indptr, _ = tiny_graph()     # 6 nodes of positive degree
    assert len(oracle.sample_cache(indptr, 0, 0, 6)[0]) == 6
    with pytest.raises(RuntimeError):
        oracle.sample_cache(indptr, 0, 0, 7, max_draws=10_000)
