"""TEST INFRASTRUCTURE - not part of the product.

Oracle for the metric-aware selection steps that sit next to the hot path
(TimelyFreeze Sec. 2.3 "AutoFreeze" score; App. "Hybrid Variants Algorithm",
Alg. 2).  Plain numpy in fp64 / exact integers, written from the definitions:

* AutoFreeze: Delta_K is the cumulative parameter update since the previous
  check, i.e. p_now - p_at_previous_check; the per-layer score is
  | ||Delta_{K-1}|| - ||Delta_K|| | / ||Delta_{K-1}||; a layer is frozen when
  every layer before it is frozen and its score lies in the lower P_Auto-th
  percentile of the layers that are still trained.
* Alg. 2: given a base mask over the N_s parameters of a stage and a budget
  N_freeze = floor(r N_s), leave the mask alone when it already holds
  N_freeze ones, otherwise add (remove) uniformly drawn indices among its
  zeros (ones) until it does.

"Uniformly drawn" needs random numbers that the GPU side can reproduce: both
sides rank the candidates by the image of their stage-wide index under the
same keyed 32-bit permutation (a 6-round Feistel network, spelled out in
``perm32``) and take the lowest ranks.  A permutation has no ties, so the
result is unique and its size exact.

Pins (tests/test_oracle_selection.py): norms of hand-made vectors, score
closed forms, numpy's nearest-rank percentile, the prefix property by brute
force over all score orderings of small L; for Alg. 2 exact budget,
superset/subset, identity when the budget is met, invertibility of the
permutation (hence no ties), determinism, chi-square uniformity over seeds.
"""
from __future__ import annotations

import math
from typing import Sequence

import numpy as np

# ---------------------------------------------------------------------------
# AutoFreeze (Sec. 2.3; P_Auto in Table exp_setup)
# ---------------------------------------------------------------------------


def autofreeze_sqnorm(p, snapshot) -> float:
    """||Delta_K||^2 with Delta_K = p - snapshot, the cumulative update since
    the check at which `snapshot` was taken."""
    d = np.asarray(p, dtype=np.float64).ravel() - np.asarray(snapshot, dtype=np.float64).ravel()
    return float(np.dot(d, d))


def autofreeze_score(sq_prev: float, sq_cur: float) -> float:
    """| ||D_{K-1}|| - ||D_K|| | / ||D_{K-1}||.  A layer that did not move in
    the previous interval has no defined change: 0 if it did not move in this
    one either (nothing changed), +inf otherwise (never in a lower percentile)."""
    a, b = math.sqrt(sq_prev), math.sqrt(sq_cur)
    if a == 0.0:
        return 0.0 if b == 0.0 else math.inf
    return abs(a - b) / a


def autofreeze_select(scores: Sequence[float], n_already_frozen: int, percentile: float) -> np.ndarray:
    """Mask (1 = frozen) after one stability check.  Layers [0, n_already_frozen)
    are frozen already.  The threshold is the nearest-rank P-th percentile of
    the scores of the layers still trained; going on from the first trained
    layer, layers are frozen for as long as their score does not exceed it."""
    L = len(scores)
    if not (0 <= n_already_frozen <= L) or not (0.0 <= percentile <= 100.0):
        raise ValueError("bad arguments")
    mask = np.zeros(L, dtype=np.uint8)
    mask[:n_already_frozen] = 1
    active = sorted(float(s) for s in scores[n_already_frozen:])
    if not active:
        return mask
    rank = math.ceil(percentile / 100.0 * len(active) - 1e-9)
    if rank == 0:
        return mask
    tau = active[rank - 1]
    l = n_already_frozen
    while l < L and scores[l] <= tau:
        mask[l] = 1
        l += 1
    return mask


# ---------------------------------------------------------------------------
# Alg. 2 (metric-aware parameter selection): budget reconciliation
# ---------------------------------------------------------------------------

_ROUNDS = 6
_MULT = 0x9E3779B1


def _round_keys(seed: int):
    """Six 16-bit round keys from a 64-bit seed: its four 16-bit pieces, then
    the two low pieces of seed * 0xD1342543DE82EF95 (mod 2^64)."""
    seed &= (1 << 64) - 1
    s2 = (seed * 0xD1342543DE82EF95) & ((1 << 64) - 1)
    return [(seed >> (16 * r)) & 0xFFFF for r in range(4)] + [(s2 >> 32) & 0xFFFF, (s2 >> 48) & 0xFFFF]


def _feistel_f(half: np.ndarray, key: int) -> np.ndarray:
    """Round function on 16-bit halves: the top 16 bits of ((half ^ key) + 1) * 0x9E3779B1 mod 2^32."""
    t = (((half ^ np.uint64(key)) + np.uint64(1)) * np.uint64(_MULT)) & np.uint64(0xFFFFFFFF)
    return (t >> np.uint64(16)) & np.uint64(0xFFFF)


def perm32(x, seed: int) -> np.ndarray:
    """Keyed permutation of [0, 2^32): 6-round Feistel network on (hi16, lo16)."""
    x = np.asarray(x, dtype=np.uint64)
    hi, lo = (x >> np.uint64(16)) & np.uint64(0xFFFF), x & np.uint64(0xFFFF)
    for k in _round_keys(seed):
        hi, lo = lo, hi ^ _feistel_f(lo, k)
    return ((hi << np.uint64(16)) | lo).astype(np.uint32)


def perm32_inverse(y, seed: int) -> np.ndarray:
    y = np.asarray(y, dtype=np.uint64)
    hi, lo = (y >> np.uint64(16)) & np.uint64(0xFFFF), y & np.uint64(0xFFFF)
    for k in reversed(_round_keys(seed)):
        hi, lo = lo ^ _feistel_f(hi, k), hi
    return ((hi << np.uint64(16)) | lo).astype(np.uint32)


def unpack_bits(words, numel: int) -> np.ndarray:
    """uint32 words, bit j & 31 of word j >> 5 (LSB first) -> numel 0/1 bytes."""
    w = np.ascontiguousarray(words, dtype="<u4")
    return np.unpackbits(w.view(np.uint8), bitorder="little")[:numel]


def pack_bits(bits) -> np.ndarray:
    b = np.asarray(bits, dtype=np.uint8)
    pad = (-len(b)) % 32
    by = np.packbits(np.concatenate([b, np.zeros(pad, np.uint8)]), bitorder="little")
    return by.view("<u4").copy()


def reconcile_mask(base_bits: Sequence[np.ndarray], numel: Sequence[int], n_freeze: int, seed: int):
    """Alg. 2 on the stage-wide index space (tensors concatenated in order).

    base_bits[i]: 0/1 array of numel[i] entries (1 = frozen by the base method).
    Returns (list of new 0/1 arrays, ||base||_1).  The new mask has exactly
    n_freeze ones: a superset of the base mask when that has fewer, a subset
    when it has more, the base mask itself when it has exactly n_freeze."""
    N = int(sum(numel))
    if N >= 1 << 32:
        raise ValueError("stage too large for 32-bit keys")
    if not (0 <= n_freeze <= N):
        raise ValueError("budget out of range")
    flat = np.concatenate([np.asarray(b, dtype=np.uint8).ravel() for b in base_bits]) if N else np.zeros(0, np.uint8)
    assert flat.size == N
    count = int(flat.sum())
    new = flat.copy()
    if count < n_freeze:
        cand = np.flatnonzero(flat == 0)
        keys = perm32(cand, seed)
        take = cand[np.argsort(keys, kind="stable")[: n_freeze - count]]
        new[take] = 1
    elif count > n_freeze:
        cand = np.flatnonzero(flat == 1)
        keys = perm32(cand, seed)
        drop = cand[np.argsort(keys, kind="stable")[: count - n_freeze]]
        new[drop] = 0
    out, o = [], 0
    for n in numel:
        out.append(new[o:o + n].copy())
        o += n
    return out, count


# ---------------------------------------------------------------------------
# Sub-tensor freezing: the unit is a block of `block_rows` consecutive rows of
# a weight tensor (rows = input features), so that the frozen fraction of the
# parameters can follow the freeze ratio closely (Sec. 3.2.1: the parameter-
# gradient time shrinks with the fraction of parameters frozen; Alg. 1: a
# random subset with |I| = AFR |P_s| in expectation).
# ---------------------------------------------------------------------------


def select_row_blocks(shapes: Sequence[tuple], block_rows: int, r: float, seed: int):
    """Seeded draw of row blocks whose parameters add up to at most floor(r P).

    Units are numbered layer by layer, block by block.  They are visited in the
    order of the keys perm32(unit, seed); a unit is frozen if it still fits into
    what is left of the budget.  Returns (list of uint8 masks, one per layer, 1 =
    frozen block; number of frozen parameters)."""
    sizes, owner = [], []
    for l, (K, N) in enumerate(shapes):
        if K % block_rows:
            raise ValueError("block_rows must divide K")
        for b in range(K // block_rows):
            sizes.append(block_rows * N)
            owner.append((l, b))
    P = int(sum(sizes))
    budget = int(math.floor(r * P + 1e-9))
    order = np.argsort(perm32(np.arange(len(sizes)), seed), kind="stable")
    masks = [np.zeros(K // block_rows, dtype=np.uint8) for K, _ in shapes]
    frozen = 0
    for u in order:
        if frozen + sizes[u] <= budget:
            frozen += sizes[u]
            l, b = owner[u]
            masks[l][b] = 1
    return masks, frozen


def row_blocks_to_elem_mask(shape, block_rows: int, row_mask) -> np.ndarray:
    """0/1 per element of a [K x N] tensor (row-major, flattened): 1 where the row's block is frozen."""
    K, N = shape
    rm = np.asarray(row_mask, dtype=np.uint8)
    assert rm.shape == (K // block_rows,)
    return np.repeat(rm, block_rows * N)
