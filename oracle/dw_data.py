"""Plain CPU oracle for the data side of the method: the overlap partition and the minibatch draws.

TEST INFRASTRUCTURE ONLY, like the rest of this package: only the tests, the smoke check and the
benchmark's CPU-baseline leg may import it, and it shares no code with the HIP kernels.

  * shared subset O and private subsets S_j, D_j = O u S_j     -- Section V-A ("Data Overlap")
  * a worker's minibatch drawn from its own D_j                -- Section II eq.(3): the gradient of
                                                                  a sampled minibatch, per worker

Readings of what the paper leaves open:

  * "Randomly sample O ... the remaining points are randomly distributed among the k workers": one
    seeded random permutation pi of the n points decides both.  O is its first o entries, S_j the
    next blocks of floor((n - o)/k) entries each, in worker order.  When k does not divide n - o
    the last (n - o) mod k entries of pi belong to no worker (the paper fixes |S_j| by the floor and
    states the union equals D - O, which both hold only when k divides n - o).
  * The permutation is the order of the points by a 64-bit key, ties (which a 64-bit key makes
    vanishingly rare) broken by the point's index: key_i = mix(mix(seed) + GAMMA*(i+1)) with the
    SplitMix64 output function `mix` of the Rademacher stream.  mix(seed) is that stream's first-level
    key for "worker -1", which no worker uses.
  * The sampler: the paper does not say how a worker picks its minibatch.  Here draw b of worker j at
    its local step t is element floor(u * |D_j| / 2^64) of D_j (O first, then S_j, both in
    permutation order), u = mix(key(seed, j, t) + GAMMA*(b+1)): independent uniform draws with
    replacement, the plain reading of "a sampled minibatch".  The key is the Rademacher stream's
    key function, so a caller gives the sampler a seed of its own.
"""
from __future__ import annotations

from typing import List, Tuple

import numpy as np

from .dw_oracle import _GAMMA, _MASK, _mix64, rademacher_key


def partition_keys(n: int, seed: int) -> List[int]:
    k1 = _mix64(seed)
    return [_mix64(k1 + _GAMMA * (i + 1)) for i in range(n)]


def overlap_partition(n: int, o: int, k: int, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """Section V-A: returns (O [o], S [k][floor((n-o)/k)]) as point indices in permutation order."""
    assert n >= 1 and 0 <= o <= n and k >= 1
    keys = partition_keys(n, seed)
    pi = sorted(range(n), key=lambda i: (keys[i], i))
    s = (n - o) // k
    O = np.array(pi[:o], dtype=np.int64)
    S = np.array([pi[o + j * s: o + (j + 1) * s] for j in range(k)], dtype=np.int64).reshape(k, s)
    return O, S


def worker_datasets(n: int, o: int, k: int, seed: int) -> np.ndarray:
    """D_j = O u S_j as rows [k][o + s]: the shared points first, then the worker's own."""
    O, S = overlap_partition(n, o, k, seed)
    return np.concatenate([np.broadcast_to(O, (k, O.size)), S], axis=1)


def batch_positions(seed: int, worker: int, step: int, batch: int, m: int) -> np.ndarray:
    """Positions within D_j (|D_j| = m) of the `batch` draws of `worker` at its local step `step`."""
    assert m >= 1
    key = rademacher_key(seed, worker, step)
    out = np.empty(batch, dtype=np.int64)
    for b in range(batch):
        u = _mix64(key + _GAMMA * (b + 1))
        out[b] = (u * m) >> 64                      # exact integer arithmetic
    return out


def draw_batch(data: np.ndarray, labels: np.ndarray, D: np.ndarray, seed: int, steps, batch: int):
    """x [k][batch][...], y [k][batch]: every worker's minibatch at its own local step steps[j]."""
    k, m = D.shape
    xs, ys = [], []
    for j in range(k):
        idx = D[j][batch_positions(seed, j, int(steps[j]), batch, m)]
        xs.append(data[idx])
        ys.append(labels[idx])
    return np.stack(xs), np.stack(ys)
