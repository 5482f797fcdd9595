"""Pins for the oracle's frontier union / relabelling, gather and aggregation
(paper Algorithm 1: set union in the top-down loop, weighted aggregation in the
bottom-up loop; Section 2.2 steps 2-3 for the gather; Section 3.4 for 1/p)."""
from fractions import Fraction

import numpy as np
import scipy.sparse as sp

import oracle


def make_blocks(small_graph, seed=42, fanouts=(6, 4, 3), policies=(0, 0, 1), c=60, wmode=oracle.W_PRINTED):
    indptr, indices = small_graph
    _, bitmap, _ = oracle.sample_cache(indptr, 3, 0, c)
    seeds = np.random.default_rng(seed).permutation(len(indptr) - 1)[:32].astype(np.int32)
    return oracle.sample_blocks(indptr, indices, bitmap, c, seed, seeds, list(fanouts), list(policies), wmode), seeds, bitmap


def test_block_structure_and_round_trip(small_graph):
    indptr, indices = small_graph
    c = 60
    blocks, seeds, bitmap = make_blocks(small_graph)
    L = len(blocks)
    dst = seeds
    for i, b in enumerate(blocks):
        k = (6, 4, 3)[i]
        pol = (0, 0, 1)[i]
        assert np.array_equal(b.dst_nodes, dst)
        R = len(dst)
        # src = dst prefix ++ strictly ascending tail disjoint from dst; all unique
        assert np.array_equal(b.src_nodes[:R], dst)
        tail = b.src_nodes[R:]
        assert np.all(np.diff(tail) > 0)
        assert len(np.intersect1d(tail, dst)) == 0
        assert len(np.unique(b.src_nodes)) == len(b.src_nodes)
        # raw per-row sample reproduced through the relabel map
        nbr, w, cnt, elig = oracle.sample_layer(indptr, indices, bitmap, c, 42, L - i, pol, 0, k, dst)
        assert np.array_equal(np.diff(b.indptr), cnt)
        assert b.indptr[0] == 0
        flat = np.concatenate([nbr[r, :cnt[r]] for r in range(R)]) if R else np.zeros(0, np.int32)
        assert np.array_equal(b.src_nodes[b.indices], flat)
        flat_w = np.concatenate([w[r, :cnt[r]] for r in range(R)])
        assert np.array_equal(b.weights, flat_w)
        # the union is exactly dst U sampled ids (library set routine)
        assert np.array_equal(np.sort(b.src_nodes), np.union1d(dst, flat))
        assert np.array_equal(tail, np.setdiff1d(flat, dst))
        dst = b.src_nodes
    # the input layer's new nodes are all cached
    last = blocks[-1]
    tail = last.src_nodes[last.num_dst:]
    assert np.all((bitmap[tail >> 6] >> (tail & 63).astype(np.uint64)) & np.uint64(1))


def test_block_with_empty_rows_and_no_edges():
    dst = np.array([5, 2, 9], dtype=np.int32)
    nbr = np.full((3, 2), -1, dtype=np.int32)
    w = np.zeros((3, 2), dtype=np.float32)
    cnt = np.zeros(3, dtype=np.int32)
    b = oracle.build_block(dst, 2, nbr, w, cnt, cnt)
    assert b.num_edges == 0 and np.array_equal(b.src_nodes, dst) and np.array_equal(b.indptr, [0, 0, 0, 0])
    nbr[1] = [9, 7]
    cnt[1] = 2
    w[1] = [0.5, 2.0]
    b = oracle.build_block(dst, 2, nbr, w, cnt, cnt)
    assert np.array_equal(b.src_nodes, [5, 2, 9, 7])
    assert np.array_equal(b.indices, [2, 3]) and np.array_equal(b.indptr, [0, 0, 2, 2])
    assert np.array_equal(b.weights, [0.5, 2.0])


def test_gather_equals_fancy_indexing():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((300, 20)).astype(np.float32)
    nodes = rng.integers(0, 300, size=500).astype(np.int32)
    out = oracle.gather(x, nodes)
    assert out.tobytes() == x[nodes].tobytes()
    assert oracle.gather(x, np.zeros(0, np.int32)).shape == (0, 20)


def test_aggregate_equals_sparse_matmul_divided_by_row_count(small_graph):
    blocks, _, _ = make_blocks(small_graph)
    rng = np.random.default_rng(1)
    for b in blocks:
        x = rng.standard_normal((b.num_src, 24)).astype(np.float32)
        out = oracle.aggregate(b.indptr, b.indices, b.weights, x)
        A = sp.csr_matrix((b.weights.astype(np.float64), b.indices, b.indptr), shape=(b.num_dst, b.num_src))
        ref = A @ x.astype(np.float64)
        n_v = np.diff(b.indptr).astype(np.float64)
        ref = np.where(n_v[:, None] > 0, ref / np.maximum(n_v, 1)[:, None], 0.0)
        scale = (abs(A) @ np.abs(x).astype(np.float64)) / np.maximum(n_v, 1)[:, None]
        assert np.all(np.abs(out - ref) <= 1e-7 * scale + 1e-30)
        assert np.all(out[n_v == 0] == 0)


def test_aggregate_order_and_transpose_sensitivity():
    # 2 dst rows, 3 src rows; a wrong index (transposed operand) or a dropped weight changes the result
    indptr = np.array([0, 2, 3], dtype=np.int32)
    indices = np.array([2, 0, 1], dtype=np.int32)
    weights = np.array([2.0, 4.0, 0.5], dtype=np.float32)
    x = np.array([[1.0, 10.0], [2.0, 20.0], [3.0, 30.0]], dtype=np.float32)
    out = oracle.aggregate(indptr, indices, weights, x)
    assert np.array_equal(out, [[(2 * 3 + 4 * 1) / 2, (2 * 30 + 4 * 10) / 2], [0.5 * 2, 0.5 * 20]])


def test_mean_of_printed_weights_closed_form(small_graph):
    """With the printed coefficient and a mean over min(k, N_C) sampled rows,
    out = (1/k) * sum_u x_u / p^C_u (the importance-sampling form quoted for
    layer-wise sampling in Section 2.1); with all-ones features the output is
    the mean of the weights."""
    indptr, indices = small_graph
    nnz = int(indptr[-1])
    c, k = 60, 3
    blocks, _, _ = make_blocks(small_graph, fanouts=(6, k), policies=(0, 1), c=c)
    b = blocks[-1]
    x = np.random.default_rng(2).standard_normal((b.num_src, 5)).astype(np.float32)
    out = oracle.aggregate(b.indptr, b.indices, b.weights, x)
    ones = oracle.aggregate(b.indptr, b.indices, b.weights, np.ones((b.num_src, 1), np.float32))
    for r in range(b.num_dst):
        lo, hi = b.indptr[r], b.indptr[r + 1]
        if hi == lo:
            assert np.all(out[r] == 0)
            continue
        acc = np.zeros(5)
        for e in range(lo, hi):
            u = int(b.src_nodes[b.indices[e]])
            p = Fraction(int(indptr[u + 1] - indptr[u]), nnz)
            pc = float(1 - (1 - p) ** c)
            acc += x[b.indices[e]].astype(np.float64) / pc
        assert np.allclose(out[r], acc / k, rtol=2e-6, atol=1e-6)
        assert abs(ones[r, 0] - b.weights[lo:hi].astype(np.float64).mean()) < 1e-6 * ones[r, 0]


# ---------------------------------------------------------------------------
# the update step h_u = g(W . (h_u, h_N(u)))  (Algorithm 1; GraphSAGE form of Section 2.1)

def test_sage_dense_matches_the_concatenated_matrix_product():
    rng = np.random.default_rng(3)
    rows, f1, f2, hdim = 37, 12, 20, 9
    hs = rng.standard_normal((rows, f1)).astype(np.float32)
    hn = rng.standard_normal((rows, f2)).astype(np.float32)
    w = rng.standard_normal((f1 + f2, hdim)).astype(np.float32)
    b = rng.standard_normal(hdim).astype(np.float32)
    pre = np.concatenate([hs, hn], axis=1).astype(np.float64) @ w.astype(np.float64) + b.astype(np.float64)
    got = oracle.sage_dense(hs, hn, w, b, relu=False)
    assert np.allclose(got, pre, rtol=0, atol=1e-6 * np.abs(pre).max())
    got_relu = oracle.sage_dense(hs, hn, w, b, relu=True)
    assert np.array_equal(got_relu, np.maximum(got, 0.0)) and (got < 0).any()
    # without bias; the self part multiplies the first F1 rows of W, the neighbor part the rest
    only_self = oracle.sage_dense(hs, np.zeros_like(hn), w, None, relu=False)
    assert np.allclose(only_self, hs.astype(np.float64) @ w[:f1].astype(np.float64), atol=1e-5)
    only_neigh = oracle.sage_dense(np.zeros_like(hs), hn, w, None, relu=False)
    assert np.allclose(only_neigh, hn.astype(np.float64) @ w[f1:].astype(np.float64), atol=1e-5)


def test_sage_dense_hand_computed():
    hs = np.array([[1.0, 2.0]], dtype=np.float32)
    hn = np.array([[3.0]], dtype=np.float32)
    w = np.array([[1.0, -1.0], [0.5, 0.0], [2.0, -4.0]], dtype=np.float32)     # rows: self0, self1, neigh0
    b = np.array([0.25, 1.0], dtype=np.float32)
    assert oracle.sage_dense(hs, hn, w, b, relu=False).tolist() == [[8.25, -12.0]]
    assert oracle.sage_dense(hs, hn, w, b, relu=True).tolist() == [[8.25, 0.0]]
