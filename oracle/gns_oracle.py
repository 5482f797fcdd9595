"""ctypes front end of ``gns_oracle.c`` (test infrastructure only).

The arithmetic lives in the C file; this module only marshals numpy arrays and
strings the per-layer calls together in the order of Algorithm 1's top-down
loop (layer L next to the seeds down to layer 1, the input layer).
"""
import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

UNIFORM = 0
CACHE_ONLY = 1
CACHE_FIRST = 2
W_PRINTED = 0
W_UNBIASED = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gns_oracle.c")
_LIB = os.path.join(_HERE, "libgns_oracle.so")
_lib = None


def build_oracle(force=False):
    """Compile the C oracle with gcc (plain -O2, no vectorisation flags)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct)) if a is not None else None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build_oracle()
    L = ctypes.CDLL(_LIB)
    i64, i32, u64, u32 = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64, ctypes.c_uint32
    P = ctypes.POINTER
    L.gns_oracle_philox4x32_10.argtypes = [P(u32), P(u32), P(u32)]
    L.gns_oracle_philox4x32_10.restype = None
    L.gns_oracle_cache_draw_node.argtypes = [i64, P(i64), u64, u64, u64]
    L.gns_oracle_cache_draw_node.restype = i64
    L.gns_oracle_sample_cache.argtypes = [i64, P(i64), u64, u64, i64, i64, P(i32), P(u64)]
    L.gns_oracle_sample_cache.restype = i64
    L.gns_oracle_floyd.argtypes = [i64, i32, P(u32), P(i64)]
    L.gns_oracle_floyd.restype = None
    L.gns_oracle_p_cache.argtypes = [ctypes.c_double, i64]
    L.gns_oracle_p_cache.restype = ctypes.c_double
    L.gns_oracle_edge_weight.argtypes = [i64, i64, i64, i32, i64, i32]
    L.gns_oracle_edge_weight.restype = ctypes.c_float
    L.gns_oracle_sample_layer.argtypes = [i64, P(i64), P(i32), P(u64), i64, u64, i32, i32, i32, i32,
                                          i64, P(i32), P(i32), P(ctypes.c_float), P(i32), P(i32)]
    L.gns_oracle_sample_layer.restype = ctypes.c_int
    L.gns_oracle_sample_layer_p.argtypes = [i64, P(i64), P(i32), P(u64), i64, P(i64), u64, i32, i32, i32, i32,
                                            i64, P(i32), P(i32), P(ctypes.c_float), P(i32), P(i32)]
    L.gns_oracle_sample_layer_p.restype = ctypes.c_int
    L.gns_oracle_walk_weights.argtypes = [i64, P(i64), P(i32), i64, P(i32), i32, P(i32), i32, P(u64), P(i64)]
    L.gns_oracle_walk_weights.restype = ctypes.c_int
    L.gns_oracle_build_block.argtypes = [i64, P(i32), i32, P(i32), P(ctypes.c_float), P(i32),
                                         P(i32), P(i32), P(ctypes.c_float), P(i32)]
    L.gns_oracle_build_block.restype = i64
    L.gns_oracle_gather.argtypes = [i64, P(ctypes.c_float), i64, P(i32), P(ctypes.c_float)]
    L.gns_oracle_gather.restype = None
    L.gns_oracle_aggregate.argtypes = [i64, P(i32), P(i32), P(ctypes.c_float), i64,
                                       P(ctypes.c_float), P(ctypes.c_float)]
    L.gns_oracle_aggregate.restype = None
    L.gns_oracle_sage_dense.argtypes = [i64, i64, P(ctypes.c_float), i64, P(ctypes.c_float), i64, P(ctypes.c_float),
                                        P(ctypes.c_float), i32, P(ctypes.c_float)]
    L.gns_oracle_sage_dense.restype = None
    _lib = L
    return L


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    _load().gns_oracle_philox4x32_10(_p(c, ctypes.c_uint32), _p(k, ctypes.c_uint32), _p(out, ctypes.c_uint32))
    return out


def cache_draw_node(indptr, seed, epoch, j):
    ip = _i64(indptr)
    return int(_load().gns_oracle_cache_draw_node(len(ip) - 1, _p(ip, ctypes.c_int64), seed, epoch, j))


def sample_cache(indptr, seed, epoch, cache_size, max_draws=None):
    """Returns (cache_nodes ascending int32, bitmap uint64, num_draws)."""
    ip = _i64(indptr)
    n = len(ip) - 1
    if max_draws is None:
        max_draws = (1 << 32) - 1
    nodes = np.zeros(cache_size, dtype=np.int32)
    bitmap = np.zeros((n + 63) // 64, dtype=np.uint64)
    nd = _load().gns_oracle_sample_cache(n, _p(ip, ctypes.c_int64), seed, epoch, cache_size, max_draws,
                                         _p(nodes, ctypes.c_int32), _p(bitmap, ctypes.c_uint64))
    if nd < 0:
        raise RuntimeError("oracle sample_cache failed (%d)" % nd)
    return nodes, bitmap, int(nd)


def floyd(m, k, words):
    w = np.ascontiguousarray(words, dtype=np.uint32)
    assert len(w) == k and 0 < k < m
    ranks = np.zeros(k, dtype=np.int64)
    _load().gns_oracle_floyd(m, k, _p(w, ctypes.c_uint32), _p(ranks, ctypes.c_int64))
    return ranks


def p_cache(p_u, cache_size):
    return float(_load().gns_oracle_p_cache(p_u, cache_size))


def edge_weight(deg_u, nnz, cache_size, k, n_c, wmode=W_PRINTED):
    return float(_load().gns_oracle_edge_weight(deg_u, nnz, cache_size, k, n_c, wmode))


def walk_weights(indptr, indices, train_nodes, fanouts, scale_log2=20):
    """Section 3.2's random-walk cache probability in integer units; returns (weights u64[n],
    prefix i64[n+1]).  The prefix plays the role of indptr in sample_cache / sample_layer."""
    ip, ix, tr = _i64(indptr), _i32(indices), _i32(train_nodes)
    fo = _i32(fanouts)
    n = len(ip) - 1
    w = np.zeros(n, dtype=np.uint64)
    pre = np.zeros(n + 1, dtype=np.int64)
    rc = _load().gns_oracle_walk_weights(n, _p(ip, ctypes.c_int64), _p(ix, ctypes.c_int32), len(tr),
                                         _p(tr, ctypes.c_int32), len(fo), _p(fo, ctypes.c_int32), scale_log2,
                                         _p(w, ctypes.c_uint64), _p(pre, ctypes.c_int64))
    if rc == -2:
        raise OverflowError("walk weights do not fit: lower scale_log2")
    if rc != 0:
        raise RuntimeError("oracle walk_weights failed (%d)" % rc)
    return w, pre


def sample_layer(indptr, indices, cache_bitmap, cache_size, seed, layer, policy, wmode, k, dst_nodes,
                 prob_prefix=None):
    """One layer; returns (nbr[R,k], w[R,k], cnt[R], eligible[R]); unused slots are -1 / 0.
    prob_prefix: integer prefix array of the cache probability (default: indptr, Eq. (1))."""
    ip, ix, dst = _i64(indptr), _i32(indices), _i32(dst_nodes)
    pp = ip if prob_prefix is None else _i64(prob_prefix)
    n, R = len(ip) - 1, len(dst)
    nbr = np.full((R, k), -1, dtype=np.int32)
    w = np.zeros((R, k), dtype=np.float32)
    cnt = np.zeros(R, dtype=np.int32)
    elig = np.zeros(R, dtype=np.int32)
    bm = None if cache_bitmap is None else np.ascontiguousarray(cache_bitmap, dtype=np.uint64)
    rc = _load().gns_oracle_sample_layer_p(n, _p(ip, ctypes.c_int64), _p(ix, ctypes.c_int32),
                                           _p(bm, ctypes.c_uint64), cache_size, _p(pp, ctypes.c_int64), seed, layer,
                                           policy, wmode, k, R, _p(dst, ctypes.c_int32), _p(nbr, ctypes.c_int32),
                                           _p(w, ctypes.c_float), _p(cnt, ctypes.c_int32), _p(elig, ctypes.c_int32))
    if rc != 0:
        raise RuntimeError("oracle sample_layer failed (%d)" % rc)
    return nbr, w, cnt, elig


@dataclass
class OracleBlock:
    """One layer's block: a CSR over (dst rows) x (src columns), local ids."""
    indptr: np.ndarray
    indices: np.ndarray
    weights: np.ndarray
    src_nodes: np.ndarray
    dst_nodes: np.ndarray
    row_eligible: np.ndarray

    @property
    def num_dst(self):
        return len(self.dst_nodes)

    @property
    def num_src(self):
        return len(self.src_nodes)

    @property
    def num_edges(self):
        return len(self.indices)


def build_block(dst_nodes, k, nbr, w, cnt, elig):
    dst = _i32(dst_nodes)
    R = len(dst)
    E = int(cnt.sum())
    indptr = np.zeros(R + 1, dtype=np.int32)
    indices = np.zeros(E, dtype=np.int32)
    weights = np.zeros(E, dtype=np.float32)
    src = np.zeros(R + E, dtype=np.int32)
    nbr_c, w_c, cnt_c = _i32(nbr), np.ascontiguousarray(w, dtype=np.float32), _i32(cnt)
    ns = _load().gns_oracle_build_block(R, _p(dst, ctypes.c_int32), k, _p(nbr_c, ctypes.c_int32),
                                        _p(w_c, ctypes.c_float), _p(cnt_c, ctypes.c_int32),
                                        _p(indptr, ctypes.c_int32), _p(indices, ctypes.c_int32),
                                        _p(weights, ctypes.c_float), _p(src, ctypes.c_int32))
    if ns < 0:
        raise RuntimeError("oracle build_block failed")
    return OracleBlock(indptr, indices, weights, src[:ns].copy(), dst, np.asarray(elig, dtype=np.int32))


def sample_blocks(indptr, indices, cache_bitmap, cache_size, seed, seeds, fanouts, policies, wmode=W_PRINTED,
                  prob_prefix=None):
    """Algorithm 1's top-down loop.  fanouts[0]/policies[0] belong to layer L
    (next to the seeds); the paper's layer number of list index i is L - i.
    Returns the list of blocks in the same order."""
    L = len(fanouts)
    dst = _i32(seeds)
    blocks = []
    for i in range(L):
        layer = L - i
        nbr, w, cnt, elig = sample_layer(indptr, indices, cache_bitmap, cache_size, seed, layer,
                                         policies[i], wmode, fanouts[i], dst, prob_prefix=prob_prefix)
        blk = build_block(dst, fanouts[i], nbr, w, cnt, elig)
        blocks.append(blk)
        dst = blk.src_nodes
    return blocks


def gather(x, nodes):
    x = np.ascontiguousarray(x, dtype=np.float32)
    nd = _i32(nodes)
    out = np.zeros((len(nd), x.shape[1]), dtype=np.float32)
    _load().gns_oracle_gather(x.shape[1], _p(x, ctypes.c_float), len(nd), _p(nd, ctypes.c_int32),
                              _p(out, ctypes.c_float))
    return out


def aggregate(indptr, indices, weights, x_src):
    ip, ix = _i32(indptr), _i32(indices)
    w = np.ascontiguousarray(weights, dtype=np.float32)
    xs = np.ascontiguousarray(x_src, dtype=np.float32)
    R, F = len(ip) - 1, xs.shape[1]
    out = np.zeros((R, F), dtype=np.float32)
    _load().gns_oracle_aggregate(R, _p(ip, ctypes.c_int32), _p(ix, ctypes.c_int32), _p(w, ctypes.c_float), F,
                                 _p(xs, ctypes.c_float), _p(out, ctypes.c_float))
    return out


def sage_dense(h_self, h_neigh, w, bias=None, relu=True):
    """out = g(h_self @ W[:F1] + h_neigh @ W[F1:] + bias), fp64 accumulation, fp32 result."""
    hs = np.ascontiguousarray(h_self, dtype=np.float32)
    hn = np.ascontiguousarray(h_neigh, dtype=np.float32)
    ww = np.ascontiguousarray(w, dtype=np.float32)
    rows, f1 = hs.shape
    f2 = hn.shape[1]
    assert hn.shape[0] == rows and ww.shape[0] == f1 + f2
    hdim = ww.shape[1]
    bb = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    out = np.zeros((rows, hdim), dtype=np.float32)
    _load().gns_oracle_sage_dense(rows, f1, _p(hs, ctypes.c_float), f2, _p(hn, ctypes.c_float), hdim,
                                  _p(ww, ctypes.c_float), _p(bb, ctypes.c_float), 1 if relu else 0,
                                  _p(out, ctypes.c_float))
    return out
