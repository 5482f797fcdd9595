#!/usr/bin/env python3
"""Writes tests/golden/oracle_config1_batch.txt: digests of what the CPU oracle computes for
one mini-batch of the tiny workload (config 1).  The paper prints no worked example, so this
fixture does not come from the paper: it freezes the oracle's conventions (Philox keying,
Floyd draw, frontier order, weight formulas), so that an unintended change of the oracle shows
up as a test failure instead of silently moving the target the HIP path is checked against.
Calls only oracle/ and the seeded input generators.  Run from the repository root:
    python tests/golden/make_golden.py
"""
import hashlib
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle                                    # noqa: E402
from paper_2106_06150_amd import synth           # noqa: E402


def digest(a):
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()[:32]


def compute():
    c = synth.CONFIGS[1]
    sd = synth.config_seeds(1)
    g = synth.make_config_graph(1)
    ip, ix = g.indptr.numpy(), g.indices.numpy()
    feat = synth.node_features(c["n"], c["feat"], sd["feat"]).numpy()
    cache_size = int(c["n"] * c["cache_frac"])
    seeds = synth.uniform_seed_batch(c["n"], c["batch"], sd["batch"]).numpy()
    lines = ["graph n=%d nnz=%d indptr=%s indices=%s" % (c["n"], int(ip[-1]), digest(ip.astype(np.int64)), digest(ix))]
    nodes, bitmap, draws = oracle.sample_cache(ip, sd["cache"], 0, cache_size)
    lines.append("cache size=%d draws=%d nodes=%s" % (cache_size, draws, digest(nodes.astype(np.int32))))
    for name, policies, wmode in [("uniform+cache_only/printed", [oracle.UNIFORM, oracle.CACHE_ONLY], oracle.W_PRINTED),
                                  ("cache_first+cache_only/unbiased", [oracle.CACHE_FIRST, oracle.CACHE_ONLY], oracle.W_UNBIASED)]:
        blocks = oracle.sample_blocks(ip, ix, bitmap, cache_size, sd["batch"], seeds, list(c["fanouts"]), policies, wmode)
        for i, b in enumerate(blocks):
            lines.append("%s layer_index=%d dst=%d src=%d edges=%d indptr=%s indices=%s src_nodes=%s weights=%s"
                         % (name, i, b.num_dst, b.num_src, b.num_edges, digest(b.indptr.astype(np.int32)),
                            digest(b.indices.astype(np.int32)), digest(b.src_nodes.astype(np.int32)),
                            digest(b.weights.astype(np.float32))))
        last = blocks[-1]
        x = oracle.gather(feat, last.src_nodes)
        out = oracle.aggregate(last.indptr, last.indices, last.weights, x)
        lines.append("%s gather=%s aggregate_fp32=%s" % (name, digest(x), digest(out.astype(np.float32))))
    return lines


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_config1_batch.txt")
    with open(path, "w") as f:
        f.write("# written by tests/golden/make_golden.py from the CPU oracle alone (not from the paper, which prints no worked example)\n")
        f.write("\n".join(compute()) + "\n")
    print(open(path).read())
