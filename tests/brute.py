"""Definition-level brute force for tiny inputs, in pure Python integers.

Nothing here sorts: the top-r set is found by enumerating every r-subset and
testing the defining inequality of Definition 1, the random k-subset of
Definition 3 by counting, for every member, how many members have a smaller
key. The generator is typed out a second time on Python ints. It shares no
code with ``oracle/`` or with the HIP library and is only usable for d of a
dozen or so.
"""
from __future__ import annotations

import itertools
import struct
from typing import List, Sequence, Tuple

import numpy as np

M32 = 0xFFFFFFFF


def philox4x32_10(ctr: Sequence[int], key: Sequence[int]) -> Tuple[int, int, int, int]:
    """Philox4x32-10 (Salmon et al., SC'11) on Python integers."""
    x = [c & M32 for c in ctr]
    ks = [key[0] & M32, key[1] & M32]
    for rnd in range(10):
        prod_a = 0xD2511F53 * x[0]
        prod_b = 0xCD9E8D57 * x[2]
        x = [((prod_b >> 32) ^ x[1] ^ ks[0]) & M32, prod_b & M32,
             ((prod_a >> 32) ^ x[3] ^ ks[1]) & M32, prod_a & M32]
        ks = [(ks[0] + 0x9E3779B9) & M32, (ks[1] + 0xBB67AE85) & M32]
    return tuple(x)


def key64(seed: int, step: int, index: int) -> int:
    o = philox4x32_10((index, 0, step & M32, (step >> 32) & M32),
                      (seed & M32, (seed >> 32) & M32))
    return (o[0] << 32) | o[1]


def mag_bits(x: float) -> int:
    return struct.unpack("<I", struct.pack("<f", x))[0] & 0x7FFFFFFF


def top_r_set(a: Sequence[float], r: int) -> Tuple[int, ...]:
    """The r-subset R with min |a| over R >= max |a| outside R. When several
    subsets qualify (ties), the one that prefers lower indices, which is the
    lexicographically first sorted index tuple; ``combinations`` yields the
    subsets in exactly that order."""
    d = len(a)
    mags = [mag_bits(float(v)) for v in a]
    for cand in itertools.combinations(range(d), r):
        inside = set(cand)
        lo = min(mags[i] for i in cand)
        hi_out = max((mags[i] for i in range(d) if i not in inside), default=-1)
        if lo >= hi_out:
            return cand
    raise AssertionError("no valid top-r set")


def random_k_subset(members: Sequence[int], k: int, seed: int, step: int) -> List[int]:
    keyed = {i: (key64(seed, step, i), i) for i in members}
    chosen = [i for i in members
              if sum(1 for j in members if keyed[j] < keyed[i]) < k]
    assert len(chosen) == k
    return sorted(chosen)


def encode(grad, residual, r: int, k: int, seed: int, step: int):
    """One node step of Algorithm 1 by brute force. float32 arithmetic is
    delegated to numpy's elementwise float32 add/subtract."""
    g = np.asarray(grad, dtype=np.float32)
    m = np.asarray(residual, dtype=np.float32)
    a = g + m
    R = top_r_set([float(v) for v in a], r)
    U = random_k_subset(R, k, seed, step)
    ghat = np.zeros_like(a)
    ghat[U] = a[U]
    return (np.array(U, dtype=np.uint32), a[U].astype(np.float32), a - ghat)
