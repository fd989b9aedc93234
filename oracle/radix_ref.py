"""Step-by-step numpy model of radix top-k -- TEST INFRASTRUCTURE ONLY.

Follows the paper's Algorithm 1 (Section 2.3.1) in its own order and notation:
``countBin`` -> ``selectBin`` -> ``selectCandidate`` per digit, most significant
digit first, then ``filter`` over the original input with the pivot as cutoff.
The adaptive scaling of Section 4.3 (subtract one randomly drawn input element
from every element before digits are taken) is modelled too.

Nothing here is shared with the GPU path; it exists so that per-pass internals
(histogram, chosen bin, remaining k, candidate count) and the robustness claims
of Section 4.2 can be checked on the CPU.  Its final answer is pinned against the
sort-based oracle in the CPU test-suite.

Readings of points the paper leaves open (all restated in the design notes):

* Elements are "bit strings" (Section 5.2) but raw IEEE bits do not sort like
  the numbers for negatives.  The key of an element is its bit pattern with the
  sign bit set when the number is non-negative and with all bits inverted when
  it is negative; every NaN gets the all-ones key.  "Smallest" complements the
  key.  -0 therefore sorts just below +0.
* ``selectBin`` scans the histogram from the highest bin down; the chosen bin
  ``b`` satisfies  sum(hist[b+1:]) < k <= sum(hist[b:])  and the new k is
  k - sum(hist[b+1:]).
* The loop runs while digits remain (Algorithm 1 stops when one candidate is
  left; running on is equivalent because further passes keep that candidate).
  The last digit is narrower when d does not divide the key width
  (low = max(low - d, 0)).
* ``filter`` keeps everything strictly better than the pivot and, among elements
  equal to the pivot, the lowest indices until exactly k are taken.
* Scaling: a_s is one element of the row; subtraction is a single fp32
  round-to-nearest operation; if a_s is not finite, 0 is used.  The rounded
  difference is a non-decreasing function of x, so after the scaled digits are
  exhausted the survivors may still differ in their original keys: selection
  continues on the original key's digits.  The result is then independent of
  a_s.  16-bit inputs are not scaled.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

F32, F16, BF16 = 0, 1, 2
_WIDTH = {F32: 32, F16: 16, BF16: 16}


# --------------------------------------------------------------------------
# keys
# --------------------------------------------------------------------------

def is_nan_bits(bits: np.ndarray, dtype: int) -> np.ndarray:
    """NaN test on raw storage words (exponent all ones, fraction non-zero)."""
    b = bits.astype(np.uint32)
    if dtype == F32:
        return (b & 0x7FFFFFFF) > 0x7F800000
    if dtype == F16:
        return (b & 0x7FFF) > 0x7C00
    return (b & 0x7FFF) > 0x7F80


def order_key(bits: np.ndarray, dtype: int, largest: bool = True) -> np.ndarray:
    """Order-preserving unsigned key (uint32, right-aligned in ``w`` bits)."""
    w = _WIDTH[dtype]
    full = np.uint32(0xFFFFFFFF if w == 32 else 0xFFFF)
    sign = np.uint32(1 << (w - 1))
    b = bits.astype(np.uint32) & full
    neg = (b & sign) != 0
    u = np.where(neg, ~b & full, b | sign).astype(np.uint32)
    u = np.where(is_nan_bits(b, dtype), full, u).astype(np.uint32)
    if not largest:
        u = (~u) & full
    return u.astype(np.uint32)


def get_digit(u: np.ndarray, low: int, high: int) -> np.ndarray:
    """Bits [low, high) of the key -- the paper's getDigit<LOW, HIGH>."""
    return ((u.astype(np.uint64) >> np.uint64(low)) & np.uint64((1 << (high - low)) - 1)).astype(np.int64)


# --------------------------------------------------------------------------
# the four subroutines of Section 2.3.1
# --------------------------------------------------------------------------

def count_bin(cand_keys: np.ndarray, low: int, high: int) -> np.ndarray:
    """histogram[j] = number of candidates whose digit is j."""
    return np.bincount(get_digit(cand_keys, low, high), minlength=1 << (high - low)).astype(np.int64)


def select_bin(histogram: np.ndarray, k: int) -> Tuple[int, int]:
    """Bin holding the k-th best candidate and the pivot's rank inside that bin."""
    above = 0                                   # candidates in bins better than the current one
    for b in range(len(histogram) - 1, -1, -1):
        if above + int(histogram[b]) >= k:
            return b, k - above
        above += int(histogram[b])
    raise ValueError("k exceeds the number of candidates")


def select_candidate(cand_keys: np.ndarray, cand_idx: np.ndarray, bin_: int, low: int, high: int):
    """Candidates whose digit equals ``bin_`` (input order kept)."""
    keep = get_digit(cand_keys, low, high) == bin_
    return cand_keys[keep], cand_idx[keep]


def filter_topk(all_keys: np.ndarray, pivot_key: int, k: int) -> np.ndarray:
    """Indices of exactly k elements: keys above the pivot, then pivot-equal keys by lowest index."""
    better = np.flatnonzero(all_keys > np.uint64(pivot_key))
    equal = np.flatnonzero(all_keys == np.uint64(pivot_key))
    need = k - better.size
    if need < 0 or need > equal.size:
        raise AssertionError("pivot is not the k-th key")
    return np.concatenate([better, equal[:need]]).astype(np.int64)


# --------------------------------------------------------------------------
# Algorithm 1
# --------------------------------------------------------------------------

@dataclass
class PassRecord:
    source: str          # "scaled" or "key"
    low: int
    high: int
    bin: int
    k_after: int         # rank of the pivot inside the chosen bin
    candidates_after: int


@dataclass
class RadixResult:
    values: np.ndarray   # raw storage words of the k selected elements
    indices: np.ndarray  # int64 positions
    passes: List[PassRecord] = field(default_factory=list)
    a_s: Optional[float] = None


def scaled_bits(bits: np.ndarray, a_s: np.float32) -> np.ndarray:
    """fp32 bits of fl(x - a_s), one rounding (Section 4.3)."""
    x = bits.astype(np.uint32).view(np.float32)
    with np.errstate(all="ignore"):
        y = (x - np.float32(a_s)).astype(np.float32)
    return y.view(np.uint32)


def draw_scale_index(seed: int, row: int, n: int) -> int:
    """Which element of the row serves as a_s.  Any index is valid; the answer never depends on it."""
    z = (int(seed) + 0x9E3779B97F4A7C15 * (int(row) + 1)) & 0xFFFFFFFFFFFFFFFF
    z ^= z >> 30
    z = (z * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
    z ^= z >> 27
    z = (z * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
    z ^= z >> 31
    return int(z % n)


def _digit_windows(width: int, d: int) -> List[Tuple[int, int]]:
    """[(low, high), ...] from the most significant digit down (Algorithm 1's high/low updates)."""
    out = []
    high, low = width, max(width - d, 0)
    while high > 0:
        out.append((low, high))
        high -= d
        low = max(low - d, 0)
    return out


def radix_topk(bits: np.ndarray, dtype: int, k: int, d: int = 12, largest: bool = True,
               scale_index: Optional[int] = None) -> RadixResult:
    """Radix top-k of ONE row of raw storage words.

    ``scale_index`` = position of a_s in the row (None: no scaling).  Output
    order: elements better than the pivot in input order, then the kept
    pivot-equal elements in input order (the paper's output is unsorted).
    """
    bits = np.ascontiguousarray(bits)
    n = bits.shape[0]
    if not (1 <= k <= n):
        raise ValueError("need 1 <= k <= n")
    w = _WIDTH[dtype]
    k_wanted = int(k)                                 # the loop below overwrites k with the pivot's rank
    res = RadixResult(values=None, indices=None)

    keys = order_key(bits, dtype, largest)            # original keys, used by filter
    cand_idx = np.arange(n, dtype=np.int64)

    phases = []
    if scale_index is not None and dtype == F32:
        a_s = bits.astype(np.uint32).view(np.float32)[int(scale_index)]
        if not np.isfinite(a_s):
            a_s = np.float32(0.0)
        res.a_s = float(a_s)
        phases.append(("scaled", order_key(scaled_bits(bits, a_s), F32, largest), 32))
    phases.append(("key", keys, w))

    for source, phase_keys, width in phases:
        cand_keys = phase_keys[cand_idx]
        for low, high in _digit_windows(width, d):
            histogram = count_bin(cand_keys, low, high)
            bin_, k = select_bin(histogram, k)
            cand_keys, cand_idx = select_candidate(cand_keys, cand_idx, bin_, low, high)
            res.passes.append(PassRecord(source, low, high, bin_, k, int(cand_idx.size)))
        # every survivor now has the same key in this phase

    pivot = int(keys[cand_idx[0]])
    assert np.all(keys[cand_idx] == np.uint32(pivot)), "one distinct candidate must remain"
    out_idx = filter_topk(keys.astype(np.uint64), pivot, k_wanted)
    res.indices = out_idx
    res.values = bits[out_idx]
    return res
