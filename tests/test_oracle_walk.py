"""Pins for the oracle's random-walk cache probability (Section 3.2, second approach:
P^l = (D_l A + I) P^(l-1), P^0 uniform on the training nodes) and for the draws and weights
that use it.  The oracle keeps the vector in integers with floor rounding; here it is checked
against the same recursion in fp64 with scipy's sparse product, against hand-computed values,
and its draws against the probabilities it defines."""
from fractions import Fraction

import numpy as np
import pytest
import scipy.sparse as sp
from scipy import stats

import oracle


def _float_walk(indptr, indices, train, fanouts, sender_scaled=False):
    n = len(indptr) - 1
    A = sp.csr_matrix((np.ones(len(indices)), indices, indptr), shape=(n, n))
    deg = np.diff(indptr).astype(np.float64)
    P = np.zeros(n)
    P[train] = 1.0
    for k in fanouts:
        d = np.where(deg > 0, np.minimum(k, deg) / np.maximum(deg, 1), 0.0)
        P = P + (A @ (d * P) if sender_scaled else d * (A @ P))
    return P


def test_walk_weights_hand_computed_path_graph():
    # 1 - 0 - 2: training node 1, two steps with fan-out 2, 1024 units per training node
    ip = np.array([0, 2, 3, 4], dtype=np.int64)
    ix = np.array([1, 2, 0, 0], dtype=np.int32)
    w, pre = oracle.walk_weights(ip, ix, [1], [2, 2], scale_log2=10)
    # step 1: W0 = 0 + (2/2)*(1024+0), W1 = 1024 + 1*0, W2 = 0 + 1*0; step 2: W0 = 1024 + 1024, W1 = 1024 + 1024, W2 = 1024
    assert w.tolist() == [2048, 2048, 1024]
    assert pre.tolist() == [0, 2048, 4096, 5120]
    # fan-out 1 halves what node 0 (degree 2) receives: floor(1 * 1024 / 2)
    w1, _ = oracle.walk_weights(ip, ix, [1], [1], scale_log2=10)
    assert w1.tolist() == [512, 1024, 0]


def test_walk_weights_match_the_fp64_recursion(small_graph):
    indptr, indices = small_graph
    n = len(indptr) - 1
    train = np.random.default_rng(2).permutation(n)[:40].astype(np.int32)
    fanouts = [15, 10, 5]
    scale = 30
    w, pre = oracle.walk_weights(indptr, indices, train, fanouts, scale_log2=scale)
    ref = _float_walk(indptr, indices, train, fanouts)
    got = w.astype(np.float64) / 2.0 ** scale
    assert np.all(np.abs(got - ref) <= 1e-6 * ref.max())
    assert pre[0] == 0 and np.array_equal(np.diff(pre).astype(np.uint64), w)
    # the receiver's d scales the sum (D A, as printed), not the sender's (A D)
    wrong = _float_walk(indptr, indices, train, fanouts, sender_scaled=True)
    assert np.abs(wrong - ref).max() > 1e-3 * ref.max()
    # the first step uses the fan-out next to the seeds: reversing the list changes the result
    w_rev, _ = oracle.walk_weights(indptr, indices, train, fanouts[::-1], scale_log2=scale)
    ref_rev = _float_walk(indptr, indices, train, fanouts[::-1])
    assert np.all(np.abs(w_rev.astype(np.float64) / 2.0 ** scale - ref_rev) <= 1e-6 * ref_rev.max())
    assert np.abs(ref_rev - ref).max() > 1e-3 * ref.max()


def test_walk_weights_reject_overflow_and_bad_arguments(small_graph):
    indptr, indices = small_graph
    with pytest.raises(OverflowError):
        oracle.walk_weights(indptr, indices, np.arange(200, dtype=np.int32), [60, 60, 60, 60, 60, 60, 60, 60], scale_log2=40)
    with pytest.raises(RuntimeError):
        oracle.walk_weights(indptr, indices, np.array([len(indptr) + 5], dtype=np.int32), [5], scale_log2=10)


def test_cache_draw_follows_the_walk_probability(small_graph):
    indptr, indices = small_graph
    n = len(indptr) - 1
    train = np.arange(0, 25, dtype=np.int32)
    w, pre = oracle.walk_weights(indptr, indices, train, [3, 2], scale_log2=24)
    support = np.flatnonzero(w)
    assert 25 < len(support) < n                       # two steps reach only part of the graph
    T = 60_000
    draws = np.array([oracle.cache_draw_node(pre, 5, 0, j) for j in range(T)])
    assert np.all(w[draws] > 0)                        # a node the walk cannot reach is never drawn
    counts = np.bincount(draws, minlength=n)[support].astype(np.float64)
    expect = w[support].astype(np.float64) / float(pre[-1]) * T
    big = expect >= 5
    obs, exp = counts[big], expect[big]
    if (~big).any():                                   # pool the rare nodes into one cell
        obs, exp = np.append(obs, counts[~big].sum()), np.append(exp, expect[~big].sum())
    chi = stats.chisquare(obs, exp)
    assert chi.pvalue > 1e-4, chi
    nodes, bitmap, _ = oracle.sample_cache(pre, 5, 0, 50)
    assert len(set(nodes.tolist())) == 50 and np.all(w[nodes] > 0)


def test_importance_weights_use_the_walk_probability(small_graph):
    indptr, indices = small_graph
    train = np.arange(0, 60, dtype=np.int32)
    w, pre = oracle.walk_weights(indptr, indices, train, [6, 6, 6], scale_log2=24)
    c, k = 80, 3
    _, bitmap, _ = oracle.sample_cache(pre, 9, 1, c)
    dst = np.arange(0, 300, dtype=np.int32)
    nbr, wt, cnt, elig = oracle.sample_layer(indptr, indices, bitmap, c, 3, 1, oracle.CACHE_ONLY, oracle.W_PRINTED, k, dst,
                                             prob_prefix=pre)
    checked = 0
    for r in range(len(dst)):
        for s in range(cnt[r]):
            u = int(nbr[r, s])
            p = Fraction(int(w[u]), int(pre[-1]))
            pc = 1 - (1 - p) ** c
            exact = 1 / (pc * Fraction(k, min(k, int(elig[r]))))
            assert abs(float(wt[r, s]) - float(exact)) <= 1.2e-7 * float(exact)
            checked += 1
    assert checked > 50
    # with the degree prefix (Eq. (1)) the same call is the default one
    a = oracle.sample_layer(indptr, indices, bitmap, c, 3, 1, oracle.CACHE_ONLY, oracle.W_PRINTED, k, dst, prob_prefix=indptr)
    b = oracle.sample_layer(indptr, indices, bitmap, c, 3, 1, oracle.CACHE_ONLY, oracle.W_PRINTED, k, dst)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
