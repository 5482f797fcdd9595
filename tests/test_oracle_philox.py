"""Pins for the oracle's Philox4x32-10.

Three independent references, none of which shares code with the oracle:
 1. a word-size-generic big-integer Philox-4 written here from the algorithm's
    definition (Salmon et al., SC'11), whose round wiring, key schedule and
    round count are validated at W=64 against numpy's Philox bit generator
    (a library routine) and which is then instantiated at W=32;
 2. rocRAND's own philox4x32_10 engine (AMD's published header), compiled for
    the host at test time;
 3. structural facts: the map counter -> output is a bijection for a fixed key
    (checked by running the rounds backwards).
"""
import os
import shutil
import subprocess

import numpy as np
import pytest

import oracle

M32 = (0xD2511F53, 0xCD9E8D57)
W32 = (0x9E3779B9, 0xBB67AE85)
M64 = (0xD2E7470EE14C6C93, 0xCA5A826395121157)
W64 = (0x9E3779B97F4A7C15, 0xBB67AE8584CAA73B)


def philox4_generic(ctr, key, bits, mult, weyl, rounds=10):
    mask = (1 << bits) - 1
    c = [int(x) for x in ctr]
    k = [int(x) for x in key]
    for _ in range(rounds):
        p0 = mult[0] * c[0]
        p1 = mult[1] * c[2]
        c = [(p1 >> bits) ^ c[1] ^ k[0], p1 & mask, (p0 >> bits) ^ c[3] ^ k[1], p0 & mask]
        k = [(k[0] + weyl[0]) & mask, (k[1] + weyl[1]) & mask]
    return c


def test_generic_philox_structure_matches_numpy_philox4x64():
    # numpy's Philox is the 4x64-10 member of the same family: same wiring, key
    # schedule and round count, other word size and constants.  It advances the
    # counter by one before producing each block of four outputs.
    rng = np.random.default_rng(0)
    for _ in range(20):
        ctr = [int(x) for x in rng.integers(0, 2 ** 63, size=4, dtype=np.uint64)]
        key = [int(x) for x in rng.integers(0, 2 ** 63, size=2, dtype=np.uint64)]
        bg = np.random.Philox(counter=np.array(ctr, dtype=np.uint64), key=np.array(key, dtype=np.uint64))
        got = [int(x) for x in bg.random_raw(4)]
        bumped = list(ctr)
        bumped[0] += 1  # < 2^63 so no carry
        assert got == philox4_generic(bumped, key, 64, M64, W64)


def test_oracle_philox_matches_generic_at_32_bits():
    rng = np.random.default_rng(1)
    cases = [([0, 0, 0, 0], [0, 0]), ([0xFFFFFFFF] * 4, [0xFFFFFFFF] * 2), ([1, 0, 0, 0], [0, 0]), ([0, 0, 0, 0], [1, 0])]
    for _ in range(200):
        cases.append(([int(x) for x in rng.integers(0, 2 ** 32, size=4)], [int(x) for x in rng.integers(0, 2 ** 32, size=2)]))
    for ctr, key in cases:
        ref = philox4_generic(ctr, key, 32, M32, W32)
        assert [int(x) for x in oracle.philox4x32_10(ctr, key)] == ref


def _inverse_round(c, k):
    # out = [hi1^c1^k0, lo1, hi0^c3^k1, lo0], lo0 = M0*c0 mod 2^32, lo1 = M1*c2 mod 2^32
    inv0 = pow(M32[0], -1, 1 << 32)
    inv1 = pow(M32[1], -1, 1 << 32)
    c0 = (c[3] * inv0) & 0xFFFFFFFF
    c2 = (c[1] * inv1) & 0xFFFFFFFF
    hi0 = (M32[0] * c0) >> 32
    hi1 = (M32[1] * c2) >> 32
    return [c0, c[0] ^ hi1 ^ k[0], c2, c[2] ^ hi0 ^ k[1]]


def test_oracle_philox_is_invertible_for_fixed_key():
    rng = np.random.default_rng(2)
    for _ in range(50):
        ctr = [int(x) for x in rng.integers(0, 2 ** 32, size=4)]
        key = [int(x) for x in rng.integers(0, 2 ** 32, size=2)]
        out = [int(x) for x in oracle.philox4x32_10(ctr, key)]
        keys = [[(key[0] + r * W32[0]) & 0xFFFFFFFF, (key[1] + r * W32[1]) & 0xFFFFFFFF] for r in range(10)]
        c = out
        for r in reversed(range(10)):
            c = _inverse_round(c, keys[r])
        assert c == ctr


def test_oracle_philox_matches_rocrand_engine(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    header = "/opt/rocm/include/rocrand/rocrand_philox4x32_10.h"
    if not (os.path.exists(hipcc) and os.path.exists(header)):
        pytest.skip("hipcc / rocRAND header not present")
    src = os.path.join(os.path.dirname(__file__), "helpers", "rocrand_philox_ref.cpp")
    exe = str(tmp_path / "rocrand_philox_ref")
    subprocess.check_call([hipcc, "--cuda-host-only", "-O1", "-o", exe, src])
    rng = np.random.default_rng(3)
    rows = []
    for _ in range(64):
        seed = int(rng.integers(0, 2 ** 63))
        sub = int(rng.integers(0, 2 ** 63))
        blk = int(rng.integers(0, 2 ** 61))  # offset = 4*blk must fit 64 bits
        rows.append((seed, sub, blk))
    rows += [(0, 0, 0), (2 ** 64 - 1, 2 ** 64 - 1, 2 ** 62 - 1), (5002, 0x4341434800000000, 12345)]
    text = "".join("%d %d %d\n" % (s, sub, 4 * blk) for s, sub, blk in rows)
    out = subprocess.run([exe], input=text, capture_output=True, text=True, check=True).stdout.split("\n")
    for (seed, sub, blk), line in zip(rows, out):
        ref = [int(x, 16) for x in line.split()]
        ctr = [blk & 0xFFFFFFFF, blk >> 32, sub & 0xFFFFFFFF, sub >> 32]
        key = [seed & 0xFFFFFFFF, seed >> 32]
        assert [int(x) for x in oracle.philox4x32_10(ctr, key)] == ref
