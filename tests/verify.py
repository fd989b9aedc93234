"""Checks of a top-k result that need no second implementation of the method.

``check_topk_properties`` decides, in O(n) numpy work and from the definition
alone, whether (values, indices) is THE top-k of a row under the stated rules
(NaN greatest, -0 < +0, lowest index first among equals).  It is used where a
full oracle sort would take too long (n = 2^26 .. 2^28) and, on small inputs, to
pin the oracle itself.  It is written with float comparisons on decoded values
and does not share code with the oracle or with the GPU path.
"""
from __future__ import annotations

import numpy as np

F32, F16, BF16 = 0, 1, 2


def decode_bits(bits: np.ndarray, dtype: int) -> np.ndarray:
    """Raw storage words -> float values (fp32 for fp32 input, else exact float32)."""
    if dtype == F32:
        return np.ascontiguousarray(bits, dtype=np.uint32).view(np.float32)
    if dtype == F16:
        return np.ascontiguousarray(bits, dtype=np.uint16).view(np.float16).astype(np.float32)
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def as_bits(x: np.ndarray, dtype: int) -> np.ndarray:
    if dtype == F32:
        return np.ascontiguousarray(x).view(np.uint32)
    return np.ascontiguousarray(x).view(np.uint16)


def _class_masks(x: np.ndarray, pivot: float, pivot_neg_zero: bool, largest: bool):
    """(strictly better than the pivot's class, inside the pivot's class) for every element of x."""
    isn = np.isnan(x)
    sb = np.signbit(x)
    if np.isnan(pivot):
        same = isn
        above = np.zeros_like(isn)                      # nothing ranks above NaN
        below = ~isn
    else:
        if pivot == 0.0:
            same = (~isn) & (x == 0.0) & (sb == pivot_neg_zero)
            zero_above = (x == 0.0) & (~sb) & pivot_neg_zero          # +0 above -0
            zero_below = (x == 0.0) & sb & (not pivot_neg_zero)       # -0 below +0
        else:
            same = (~isn) & (x == pivot)
            zero_above = zero_below = np.zeros_like(isn)
        with np.errstate(invalid="ignore"):
            above = isn | (x > pivot) | zero_above
            below = ((~isn) & (x < pivot)) | zero_below
    return (above if largest else below), same


def check_topk_properties(x_bits: np.ndarray, dtype: int, k: int, largest: bool,
                          out_val_bits: np.ndarray, out_idx: np.ndarray) -> None:
    """Raise AssertionError unless (out_val_bits, out_idx) is exactly the top-k of the row ``x_bits``."""
    n = x_bits.shape[0]
    out_idx = np.asarray(out_idx)
    assert out_idx.shape == (k,) and out_val_bits.shape == (k,), "exactly k outputs"
    assert out_idx.dtype == np.int64
    assert out_idx.min() >= 0 and out_idx.max() < n, "indices in range"
    sidx = np.sort(out_idx)
    assert np.all(sidx[1:] != sidx[:-1]), "indices distinct"
    assert np.array_equal(np.asarray(x_bits)[out_idx], out_val_bits), "value bits are the input's bits at the index"

    x = decode_bits(x_bits, dtype)
    ov = x[out_idx]
    # worst selected element under the preorder
    onan = np.isnan(ov)
    if largest:
        if onan.all():
            pivot, pneg = np.nan, False
        else:
            pivot = ov[~onan].min()
            pneg = bool(pivot == 0.0 and np.any(np.signbit(ov[(~onan) & (ov == 0.0)])))
    else:
        if onan.any():
            pivot, pneg = np.nan, False
        else:
            pivot = ov.max()
            pneg = bool(pivot == 0.0 and not np.any(~np.signbit(ov[ov == 0.0])))
    better, same = _class_masks(x, pivot, pneg, largest)
    nb = int(np.count_nonzero(better))
    ns = int(np.count_nonzero(same))
    assert nb < k <= nb + ns, "the worst output is the k-th key (better=%d, tied=%d, k=%d)" % (nb, ns, k)
    chosen = np.zeros(n, dtype=bool)
    chosen[out_idx] = True
    assert np.all(chosen[better]), "every element better than the k-th key is selected"
    tied_pos = np.flatnonzero(same)
    need = k - nb
    assert np.all(chosen[tied_pos[:need]]), "ties at the k-th key: lowest indices first"
    assert not np.any(chosen[tied_pos[need:]]), "ties at the k-th key: no higher index selected"


def assert_same_selection(x_bits: np.ndarray, got_vals: np.ndarray, got_idx: np.ndarray,
                          want_vals: np.ndarray, want_idx: np.ndarray) -> None:
    """Bit-exact parity of one row: same index set, values are the input's bits, same sorted value words,
    and the same k-th key."""
    got_idx = np.asarray(got_idx)
    assert got_idx.shape == want_idx.shape
    assert np.array_equal(np.sort(got_idx), np.sort(want_idx)), "index set differs from the oracle's"
    assert np.array_equal(np.asarray(x_bits)[got_idx], got_vals), "values are not the input's bits at the index"
    order_g = np.argsort(got_idx, kind="stable")
    order_w = np.argsort(want_idx, kind="stable")
    assert np.array_equal(got_vals[order_g], want_vals[order_w]), "value words differ from the oracle's"
