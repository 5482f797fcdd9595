"""Pins for the oracle's layer sampler and importance weights (paper Sections
2.1, 3.3, 3.4, 4.1; Algorithm 1 top-down loop).

 - Floyd's subset draw: exhaustive enumeration of every word tuple's outcome
   for small (m, k) gives each k-subset exactly k! times (uniform subsets);
 - sampler invariants: true neighbors, cached at the input layer, no
   duplicates in a row, count = min(k, eligible), ascending CSR position,
   eligible count = brute-force |N(v) & C|;
 - subsets across seeds are uniform (chi-square);
 - weights equal Section 3.4's formulas evaluated with exact rationals;
 - the unbiased variant's expectation over caches and samples equals the
   closed form sum_u x_u * pi_u / p^C_u (pi = exact inclusion probability).
"""
from fractions import Fraction
from itertools import combinations, product
from math import comb, factorial

import numpy as np
import pytest
from scipy import stats

import oracle
from test_oracle_cache import exact_wor_inclusion, tiny_graph


def word_for(t, j):
    """Smallest 32-bit word w with floor(w*(j+1)/2^32) == t."""
    w = -((-t * (1 << 32)) // (j + 1))
    assert (w * (j + 1)) >> 32 == t and 0 <= w < (1 << 32)
    return w


@pytest.mark.parametrize("m,k", [(2, 1), (4, 2), (5, 3), (6, 2), (7, 4), (8, 3), (8, 7)])
def test_floyd_enumeration_gives_each_subset_k_factorial_times(m, k):
    seen = {}
    ranges = [range(m - k + s + 1) for s in range(k)]
    for ts in product(*ranges):
        words = [word_for(t, m - k + s) for s, t in enumerate(ts)]
        ranks = tuple(int(r) for r in oracle.floyd(m, k, words))
        assert list(ranks) == sorted(set(ranks)) and len(ranks) == k and 0 <= ranks[0] and ranks[-1] < m
        seen[ranks] = seen.get(ranks, 0) + 1
    assert len(seen) == comb(m, k)
    assert set(seen.values()) == {factorial(k)}


def test_floyd_word_to_range_map_extremes():
    # word 0 -> 0, word 2^32-1 -> j (never j+1)
    assert list(oracle.floyd(10, 1, [0])) == [0]
    assert list(oracle.floyd(10, 1, [0xFFFFFFFF])) == [9]
    assert list(oracle.floyd(2 ** 31, 1, [0xFFFFFFFF])) == [2 ** 31 - 1]


def brute_force_rows(indptr, indices, bitmap, dst, policy):
    out = []
    for v in dst:
        row = indices[indptr[v]:indptr[v + 1]]
        if policy == oracle.CACHE_ONLY:
            row = [int(u) for u in row if (int(bitmap[int(u) >> 6]) >> (int(u) & 63)) & 1]
        out.append([int(u) for u in row])
    return out


@pytest.mark.parametrize("policy,k", [(oracle.UNIFORM, 1), (oracle.UNIFORM, 5), (oracle.UNIFORM, 15),
                                      (oracle.CACHE_ONLY, 1), (oracle.CACHE_ONLY, 5), (oracle.CACHE_ONLY, 10)])
def test_sampler_invariants(small_graph, policy, k):
    indptr, indices = small_graph
    n = len(indptr) - 1
    nodes, bitmap, _ = oracle.sample_cache(indptr, 3, 0, 60)
    dst = np.random.default_rng(5).permutation(n)[:150].astype(np.int32)
    nbr, w, cnt, elig = oracle.sample_layer(indptr, indices, bitmap, 60, 1234, 2, policy, oracle.W_PRINTED, k, dst)
    rows = brute_force_rows(indptr, indices, bitmap, dst, policy)
    took_subset = False
    for r, v in enumerate(dst):
        e = rows[r]
        assert elig[r] == len(e)
        assert cnt[r] == min(k, len(e))
        got = nbr[r, :cnt[r]].tolist()
        assert all(x == -1 for x in nbr[r, cnt[r]:])
        assert len(set(got)) == len(got)
        pos = [e.index(u) for u in got]                 # members of the eligible list ...
        assert pos == sorted(pos)                       # ... in ascending CSR position
        if len(e) <= k:
            assert got == e
        else:
            took_subset = True
        if policy == oracle.UNIFORM:
            assert np.all(w[r, :cnt[r]] == 1.0)
    assert took_subset


def test_sampler_depends_on_seed_layer_and_node_only(small_graph):
    indptr, indices = small_graph
    _, bitmap, _ = oracle.sample_cache(indptr, 3, 0, 60)
    dst = np.arange(0, 100, dtype=np.int32)
    a = oracle.sample_layer(indptr, indices, bitmap, 60, 7, 2, oracle.UNIFORM, 0, 4, dst)[0]
    b = oracle.sample_layer(indptr, indices, bitmap, 60, 7, 2, oracle.UNIFORM, 0, 4, dst[::-1].copy())[0]
    assert np.array_equal(a, b[::-1])                   # a row's sample does not depend on its position
    c = oracle.sample_layer(indptr, indices, bitmap, 60, 7, 3, oracle.UNIFORM, 0, 4, dst)[0]
    d = oracle.sample_layer(indptr, indices, bitmap, 60, 8, 2, oracle.UNIFORM, 0, 4, dst)[0]
    assert not np.array_equal(a, c) and not np.array_equal(a, d)


@pytest.mark.parametrize("policy", [oracle.UNIFORM, oracle.CACHE_ONLY])
def test_sampled_subsets_are_uniform_across_seeds(policy):
    # star-ish row: node 0 with 6 neighbors, all cached for CACHE_ONLY
    n = 7
    indptr = np.array([0, 6, 7, 8, 9, 10, 11, 12], dtype=np.int64)
    indices = np.array([1, 2, 3, 4, 5, 6, 0, 0, 0, 0, 0, 0], dtype=np.int32)
    bitmap = np.array([0b1111110], dtype=np.uint64)
    k = 3
    subsets = {s: 0 for s in combinations(range(1, 7), k)}
    T = 20_000
    dst = np.array([0], dtype=np.int32)
    for seed in range(T):
        nbr, _, cnt, _ = oracle.sample_layer(indptr, indices, bitmap, 6, seed, 1, policy, 0, k, dst)
        subsets[tuple(nbr[0].tolist())] += 1
    chi = stats.chisquare(list(subsets.values()))
    assert chi.pvalue > 1e-4, chi


@pytest.mark.parametrize("wmode", [oracle.W_PRINTED, oracle.W_UNBIASED])
def test_weights_match_exact_rationals(small_graph, wmode):
    indptr, indices = small_graph
    nnz = int(indptr[-1])
    c = 60
    _, bitmap, _ = oracle.sample_cache(indptr, 3, 0, c)
    dst = np.arange(0, 200, dtype=np.int32)
    k = 3
    nbr, w, cnt, elig = oracle.sample_layer(indptr, indices, bitmap, c, 77, 1, oracle.CACHE_ONLY, wmode, k, dst)
    checked = 0
    for r in range(len(dst)):
        for s in range(cnt[r]):
            u = int(nbr[r, s])
            p = Fraction(int(indptr[u + 1] - indptr[u]), nnz)
            pc = 1 - (1 - p) ** c
            nc = int(elig[r])
            if wmode == oracle.W_PRINTED:
                exact = 1 / (pc * Fraction(k, min(k, nc)))
            else:
                exact = Fraction(nc, min(k, nc)) / pc
            assert abs(float(w[r, s]) - float(exact)) <= 1.2e-7 * float(exact)   # one fp32 rounding
            checked += 1
    assert checked > 100
    # unbiased / printed = N_C * k / min(k, N_C)^2: equal only at N_C == k
    for nc, ratio in [(4, 1.0), (3, 4.0 / 3.0), (8, 2.0), (1, 4.0)]:
        got = oracle.edge_weight(5, 1000, 10, 4, nc, oracle.W_UNBIASED) / oracle.edge_weight(5, 1000, 10, 4, nc, oracle.W_PRINTED)
        assert abs(got - ratio) < 1e-6


def test_unbiased_weights_expectation_closed_form():
    """E over (cache, sample) of sum_e w_e x_e = sum_{u in N(v)} x_u * pi_u / p^C_u, where
    pi_u is the exact inclusion probability of the without-replacement cache (paper's
    expectation identity in Section 3.1 with the true inclusion probability in place of
    p^C would give sum x_u exactly)."""
    indptr, indices = tiny_graph()
    deg = np.diff(indptr)
    nnz = int(deg.sum())
    c, k, v = 3, 1, 0
    p = [Fraction(int(d), nnz) for d in deg]
    pi = exact_wor_inclusion(p, c)
    x = np.array([0.0, 1.0, -2.0, 3.5, 0.25, 0.0, 0.0])
    nb = indices[indptr[v]:indptr[v + 1]]
    expect = sum(float(x[u]) * float(pi[u]) / float(1 - (1 - p[u]) ** c) for u in nb)
    T = 40_000
    dst = np.array([v], dtype=np.int32)
    vals = np.zeros(T)
    for seed in range(T):
        _, bitmap, _ = oracle.sample_cache(indptr, seed, 0, c)
        nbr, w, cnt, _ = oracle.sample_layer(indptr, indices, bitmap, c, 10_000_000 + seed, 1, oracle.CACHE_ONLY,
                                             oracle.W_UNBIASED, k, dst)
        vals[seed] = sum(float(w[0, s]) * x[nbr[0, s]] for s in range(cnt[0]))
    z = (vals.mean() - expect) / (vals.std(ddof=1) / np.sqrt(T))
    assert abs(z) < 4.5, (vals.mean(), expect)


# ---------------------------------------------------------------------------
# CACHE_FIRST (Section 3.3: from the cache first, the shortfall uniformly from the
# rest of the neighborhood)

def _split_row(indptr, indices, bitmap, v):
    row = [int(u) for u in indices[indptr[v]:indptr[v + 1]]]
    cached = [u for u in row if (int(bitmap[u >> 6]) >> (u & 63)) & 1]
    rest = [u for u in row if not (int(bitmap[u >> 6]) >> (u & 63)) & 1]
    return row, cached, rest


@pytest.mark.parametrize("k", [1, 4, 9])
def test_cache_first_invariants_and_reduction_to_the_other_policies(small_graph, k):
    indptr, indices = small_graph
    n = len(indptr) - 1
    c = 60
    _, bitmap, _ = oracle.sample_cache(indptr, 3, 0, c)
    dst = np.random.default_rng(6).permutation(n)[:300].astype(np.int32)
    args = (indptr, indices, bitmap, c, 4321, 2)
    nbr, w, cnt, elig = oracle.sample_layer(*args, oracle.CACHE_FIRST, oracle.W_PRINTED, k, dst)
    nbr_c, w_c, cnt_c, _ = oracle.sample_layer(*args, oracle.CACHE_ONLY, oracle.W_PRINTED, k, dst)
    nbr_u, w_u, cnt_u, _ = oracle.sample_layer(*args, oracle.UNIFORM, oracle.W_PRINTED, k, dst)
    seen = dict(full_cache=0, no_cache=0, mixed_subset=0, mixed_all=0)
    for r, v in enumerate(dst):
        row, cached, rest = _split_row(indptr, indices, bitmap, v)
        assert elig[r] == len(cached)
        assert cnt[r] == min(k, len(row))
        got = nbr[r, :cnt[r]].tolist()
        assert all(x == -1 for x in nbr[r, cnt[r]:]) and len(set(got)) == len(got)
        head = min(k, len(cached))
        # the cached part is exactly what CACHE_ONLY takes, with its weights
        assert got[:head] == nbr_c[r, :cnt_c[r]].tolist() and cnt_c[r] == head
        assert np.array_equal(w[r, :head], w_c[r, :head])
        fill = got[head:]
        assert len(fill) == min(k - head, len(rest))
        pos = [rest.index(u) for u in fill]              # members of N(v) \ C ...
        assert pos == sorted(pos)                        # ... in ascending CSR position
        assert np.all(w[r, head:cnt[r]] == 1.0)
        if len(cached) >= k:
            seen["full_cache"] += 1
            assert not fill
        elif not cached:
            seen["no_cache"] += 1                        # nothing cached: the row's draw is the UNIFORM one
            assert got == nbr_u[r, :cnt_u[r]].tolist() and np.array_equal(w[r], w_u[r])
        elif len(rest) > k - head:
            seen["mixed_subset"] += 1
        else:
            seen["mixed_all"] += 1
            assert fill == rest
    assert seen["no_cache"] > 0 and seen["full_cache"] > 0, seen
    if k > 1:                                            # 0 < N_C < k needs k >= 2
        assert seen["mixed_subset"] > 0, seen


def _star_row():
    # node 0 has neighbors 1..9; 1 and 2 are cached
    n = 10
    indptr = np.array([0, 9] + list(range(10, 19)), dtype=np.int64)
    indices = np.array(list(range(1, 10)) + [0] * 9, dtype=np.int32)
    bitmap = np.array([0b110], dtype=np.uint64)
    return n, indptr, indices, bitmap


def test_cache_first_fill_is_uniform_over_the_uncached_neighbors():
    n, indptr, indices, bitmap = _star_row()
    k = 5                                                 # 2 from the cache, 3 of the 7 others
    subsets = {s: 0 for s in combinations(range(3, 10), 3)}
    T = 35_000
    dst = np.array([0], dtype=np.int32)
    for seed in range(T):
        nbr, _, cnt, elig = oracle.sample_layer(indptr, indices, bitmap, 2, seed, 1, oracle.CACHE_FIRST, 0, k, dst)
        assert cnt[0] == 5 and elig[0] == 2 and nbr[0, :2].tolist() == [1, 2]
        subsets[tuple(nbr[0, 2:].tolist())] += 1
    chi = stats.chisquare(list(subsets.values()))
    assert chi.pvalue > 1e-4, chi


def test_cache_first_fill_uses_its_own_philox_slots():
    """The fill draw of a row with N_C cached neighbors uses slots N_C, N_C+1, ...: with one cached
    neighbor and k = 2 the single fill word is slot 1 of the row, i.e. the word that a UNIFORM row
    draws second."""
    n, indptr, indices, _ = _star_row()
    bitmap = np.array([0b10], dtype=np.uint64)            # only node 1 cached; 8 others
    dst = np.array([0], dtype=np.int32)
    for seed in range(50):
        nbr, _, cnt, _ = oracle.sample_layer(indptr, indices, bitmap, 1, seed, 3, oracle.CACHE_FIRST, 0, 2, dst)
        ctr = (0, 0, 3, 0x4E424853)                       # (node, slot >> 2, layer, tag)
        word = int(oracle.philox4x32_10(ctr, (seed & 0xFFFFFFFF, seed >> 32))[1])
        expect = 2 + ((word * 8) >> 32)                   # rank t of the 8 uncached neighbors 2..9
        assert cnt[0] == 2 and nbr[0].tolist() == [1, expect]


def test_cache_first_unbiased_weights_given_the_cache():
    """Given the cache, sum over fill edges of w*x estimates the sum of x over N(v) \\ C, and
    the fill weight is |N(v) \\ C| / r exactly; the cached part is taken whole (N_C < k)."""
    n, indptr, indices, bitmap = _star_row()
    x = np.array([0.0, 2.0, -1.0, 0.5, 3.0, -2.5, 1.25, 4.0, -0.75, 6.0])
    k = 4                                                 # 2 cached + 2 of 7
    dst = np.array([0], dtype=np.int32)
    T = 30_000
    vals = np.zeros(T)
    for seed in range(T):
        nbr, w, cnt, _ = oracle.sample_layer(indptr, indices, bitmap, 2, seed, 1, oracle.CACHE_FIRST,
                                             oracle.W_UNBIASED, k, dst)
        assert np.all(w[0, 2:4] == np.float32(7.0 / 2.0))
        vals[seed] = float(np.dot(w[0, 2:4].astype(np.float64), x[nbr[0, 2:4]]))
    expect = x[3:].sum()
    z = (vals.mean() - expect) / (vals.std(ddof=1) / np.sqrt(T))
    assert abs(z) < 4.5, (vals.mean(), expect)
    # cached part: N_C / (min(k, N_C) * p^C) = 1 / p^C
    p1 = 1.0 / 18.0
    pc = 1 - (1 - p1) ** 2
    assert abs(float(w[0, 0]) - 1.0 / pc) < 1e-6 / pc


def test_slots_beyond_the_fourth_take_later_philox_blocks():
    """A row with more than four draws uses several Philox blocks: slot s takes word s & 3 of the block whose
    counter is (node, s >> 2, layer, tag) under the key (seed low, seed high).  Pinned against the word-size-generic
    Philox of test_oracle_philox (validated there against numpy's generator) and Floyd's draw written out here:
    one hub row of degree 200, fan-outs 5..16, several nodes, layers and seeds above 2^32.  A swapped counter word,
    a word taken from the wrong block or a block reused for slots 4.. changes the sample."""
    from test_oracle_philox import philox4_generic, M32, W32
    tag = 0x4E424853                                    # the neighbor-draw stream's counter word
    deg = 200
    n = deg + 8
    rows = [np.arange(1, deg + 1) if v in (0, 203, 207) else np.array([], dtype=np.int64) for v in range(n)]
    rows[203] = np.arange(0, deg)                       # other hubs with other neighbor lists
    rows[207] = np.arange(3, deg + 3)
    indptr = np.zeros(n + 1, dtype=np.int64)
    indptr[1:] = np.cumsum([len(r) for r in rows])
    indices = np.concatenate(rows).astype(np.int32)
    for seed in (5, (7 << 32) | 11):
        key = (seed & 0xFFFFFFFF, seed >> 32)
        for layer in (1, 3):
            for k in (5, 8, 10, 15, 16):
                for node in (0, 203, 207):
                    chosen = []
                    for s_ in range(k):
                        word = philox4_generic((node, s_ >> 2, layer, tag), key, 32, M32, W32)[s_ & 3]
                        j = deg - k + s_
                        t = (word * (j + 1)) >> 32
                        chosen.append(j if t in chosen else t)
                    expect = rows[node][sorted(chosen)]
                    nbr, _, cnt, elig = oracle.sample_layer(indptr, indices, None, 0, seed, layer, oracle.UNIFORM, 0, k,
                                                            np.array([node], dtype=np.int32))
                    assert cnt[0] == k and elig[0] == deg
                    assert np.array_equal(nbr[0], expect), (seed, layer, k, node)
