"""Pins for the CPU oracle (oracle/topk_oracle.c): it is checked against things other than itself --
library conversions, IEEE facts, closed forms, numpy's own sort/partition on inputs where the rules reduce
to plain numeric order, an independent property checker, and brute force on tiny inputs."""
import itertools

import numpy as np
import pytest

import oracle
from paper_2501_14336_amd import workloads as W
from tests import verify

F32, F16, BF16 = oracle.F32, oracle.F16, oracle.BF16


# ---------------------------------------------------------------- decoders

def test_decode_f16_exhaustive_against_numpy():
    allbits = np.arange(65536, dtype=np.uint16)
    want = allbits.view(np.float16).astype(np.float64)
    got = np.array([oracle.decode(F16, int(b)) for b in allbits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_decode_bf16_exhaustive_against_fp32_widening():
    allbits = np.arange(65536, dtype=np.uint16)
    want = (allbits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    got = np.array([oracle.decode(BF16, int(b)) for b in allbits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_decode_bf16_matches_torch():
    torch = pytest.importorskip("torch")
    bits = np.array([0x0000, 0x8000, 0x3F80, 0xC000, 0x7F80, 0xFF80, 0x0001, 0x807F, 0x7F7F, 0x4049], dtype=np.uint16)
    t = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([oracle.decode(BF16, int(b)) for b in bits])
    assert np.array_equal(got, t)


# ---------------------------------------------------------------- preorder

def _b32(x):
    return int(np.array([x], dtype=np.float32).view(np.uint32)[0])


def test_rank_cmp_ieee_facts():
    inf, ninf = _b32(np.inf), _b32(-np.inf)
    pz, nz = 0x00000000, 0x80000000
    nan_a, nan_b, nan_neg = 0x7FC00000, 0x7F800001, 0xFFC12345
    one, sub = _b32(1.0), 0x00000001
    # NaN is the greatest class, whatever its sign or payload, and all NaNs tie
    for nn in (nan_a, nan_b, nan_neg):
        for other in (inf, ninf, pz, nz, one, sub):
            assert oracle.rank_cmp(F32, nn, other) == 1
            assert oracle.rank_cmp(F32, other, nn) == -1
        for mm in (nan_a, nan_b, nan_neg):
            assert oracle.rank_cmp(F32, nn, mm) == 0
    # infinities are ordinary extreme keys
    assert oracle.rank_cmp(F32, inf, _b32(3.0e38)) == 1
    assert oracle.rank_cmp(F32, ninf, _b32(-3.0e38)) == -1
    # signed zeros: -0 just below +0, both between the subnormals
    assert oracle.rank_cmp(F32, nz, pz) == -1 and oracle.rank_cmp(F32, pz, nz) == 1
    assert oracle.rank_cmp(F32, pz, pz) == 0 and oracle.rank_cmp(F32, nz, nz) == 0
    assert oracle.rank_cmp(F32, sub, pz) == 1 and oracle.rank_cmp(F32, 0x80000001, nz) == -1


@pytest.mark.parametrize("dtype", [F32, F16, BF16])
def test_rank_cmp_is_numeric_order_on_ordinary_values(dtype):
    rng = np.random.default_rng(7)
    if dtype == F32:
        bits = rng.integers(0, 1 << 32, size=4000, dtype=np.uint64).astype(np.uint32)
    else:
        bits = rng.integers(0, 1 << 16, size=4000, dtype=np.uint64).astype(np.uint16)
    vals = verify.decode_bits(bits, dtype).astype(np.float64)
    ok = np.isfinite(vals) & (vals != 0)
    bits, vals = bits[ok], vals[ok]
    a, b = bits[:-1], bits[1:]
    want = np.sign(vals[:-1] - vals[1:]).astype(int)
    got = np.array([oracle.rank_cmp(dtype, int(x), int(y)) for x, y in zip(a, b)])
    assert np.array_equal(got, want)


# ---------------------------------------------------------------- closed forms

def test_k_equals_n_returns_every_index_once():
    x = W.normal(257, seed=1)
    v, i = oracle.topk(x, F32, 257, True)
    assert np.array_equal(np.sort(i[0]), np.arange(257))


def test_k1_is_first_argmax():
    x = np.array([1.0, 5.0, 3.0, 5.0, -2.0, 5.0], dtype=np.float32)
    v, i = oracle.topk(x, F32, 1, True)
    assert i[0, 0] == 1 and v.view(np.float32)[0, 0] == 5.0
    v, i = oracle.topk(x, F32, 1, False)
    assert i[0, 0] == 4


@pytest.mark.parametrize("largest", [True, False])
def test_all_equal_input_takes_lowest_indices(largest):
    x = np.full(100, 0.999, dtype=np.float32)
    v, i = oracle.topk(x, F32, 37, largest)
    assert np.array_equal(i[0], np.arange(37))


def test_sorted_inputs():
    n, k = 1000, 17
    desc = np.linspace(5.0, -5.0, n).astype(np.float32)
    assert np.array_equal(oracle.topk(desc, F32, k, True)[1][0], np.arange(k))
    assert np.array_equal(oracle.topk(desc, F32, k, False)[1][0], np.arange(n - 1, n - 1 - k, -1))
    asc = desc[::-1].copy()
    assert np.array_equal(oracle.topk(asc, F32, k, True)[1][0], np.arange(n - 1, n - 1 - k, -1))
    assert np.array_equal(oracle.topk(asc, F32, k, False)[1][0], np.arange(k))


def test_fp16_narrow_range_collapses_to_one_value():
    # fp16 spacing at 1.0 is 2^-10, wider than the whole range [1, 1 + 2^-12)
    x = W.narrow(4096, seed=3, dtype=np.float16)
    assert np.all(x == np.float16(1.0))
    v, i = oracle.topk(x, F16, 100, True)
    assert np.array_equal(i[0], np.arange(100))


def test_special_value_order_written_out():
    # position:        0     1      2     3     4      5        6          7
    x = np.array([0.0, -0.0, np.inf, -np.inf, 1.0, np.nan, -1e-45, 1e-45], dtype=np.float32)
    xb = x.view(np.uint32).copy()
    xb[5] = 0xFFC00001          # a negative, payload-carrying NaN is still the greatest key
    want_desc = [5, 2, 4, 7, 0, 1, 6, 3]
    v, i = oracle.topk(xb, F32, 8, True)
    assert list(i[0]) == want_desc
    assert np.array_equal(v[0], xb[want_desc])          # original bits, payload preserved
    v, i = oracle.topk(xb, F32, 8, False)
    assert list(i[0]) == want_desc[::-1]


# ---------------------------------------------------------------- library routines on reducible inputs

@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("largest", [True, False])
def test_matches_numpy_stable_argsort_when_rules_reduce_to_numeric_order(seed, largest):
    # heavy duplicates, no NaN and no zeros: the preorder is plain numeric order, ties by index
    rng = np.random.default_rng(seed)
    x = rng.integers(1, 40, size=5000).astype(np.float32) * np.float32(0.25) - np.float32(5.125)
    for k in (1, 7, 500, 5000):
        order = np.argsort(-x if largest else x, kind="stable")[:k]
        v, i = oracle.topk(x, F32, k, largest)
        assert np.array_equal(i[0], order)
        assert np.array_equal(v.view(np.float32)[0], x[order])


@pytest.mark.parametrize("k", [1, 100, 65536, 1 << 19])
def test_kth_key_equals_numpy_partition(k):
    x = W.normal(1 << 20, seed=11)
    v, _ = oracle.topk(x, F32, k, True)
    kth = np.partition(x, x.size - k)[x.size - k]
    assert v.view(np.float32)[0, -1] == kth
    v, _ = oracle.topk(x, F32, k, False)
    assert v.view(np.float32)[0, -1] == np.partition(x, k - 1)[k - 1]


# ---------------------------------------------------------------- brute force on tiny inputs

_SYMS32 = np.array([0x00000000, 0x80000000, 0x3F800000, 0x7FC00000, 0xFF800000], dtype=np.uint32)  # +0 -0 1 NaN -inf


@pytest.mark.parametrize("largest", [True, False])
def test_exhaustive_tiny_alphabet_sort_vs_bruteforce_vs_properties(largest):
    for n in range(1, 6):
        for combo in itertools.product(range(len(_SYMS32)), repeat=n):
            xb = _SYMS32[list(combo)]
            for k in range(1, n + 1):
                v1, i1 = oracle.topk(xb, F32, k, largest)
                v2, i2 = oracle.topk_bruteforce(xb, F32, k, largest)
                assert np.array_equal(i1, i2) and np.array_equal(v1, v2)
                verify.check_topk_properties(xb, F32, k, largest, v1[0], i1[0])


@pytest.mark.parametrize("dtype", [F32, F16, BF16])
@pytest.mark.parametrize("largest", [True, False])
def test_random_small_sort_vs_bruteforce_vs_properties(dtype, largest):
    rng = np.random.default_rng(100 + dtype)
    for trial in range(60):
        n = int(rng.integers(1, 65))
        if dtype == F32:
            xb = W.specials_ramp(n, seed=trial, with_nan=True).view(np.uint32).copy()
            dup = rng.integers(0, n, size=n // 2)
            xb[dup] = xb[rng.integers(0, n)]
        else:
            xb = rng.integers(0, 1 << 16, size=n, dtype=np.uint64).astype(np.uint16)
            xb[rng.integers(0, n, size=n // 2)] = xb[0]
        for k in sorted({1, max(1, n // 3), n}):
            v1, i1 = oracle.topk(xb, dtype, k, largest)
            v2, i2 = oracle.topk_bruteforce(xb, dtype, k, largest)
            assert np.array_equal(i1, i2) and np.array_equal(v1, v2)
            verify.check_topk_properties(xb, dtype, k, largest, v1[0], i1[0])


def test_batch_rows_are_independent():
    x = W.normal(3 * 500, seed=5).reshape(3, 500)
    v, i = oracle.topk(x, F32, 20, True)
    for r in range(3):
        vr, ir = oracle.topk(x[r], F32, 20, True)
        assert np.array_equal(v[r], vr[0]) and np.array_equal(i[r], ir[0])


def test_sort_row_prefixes_answer_every_k():
    x = W.duplicates(3000, seed=9)
    order = oracle.sort_row(x, F32, True)
    for k in (1, 10, 2999, 3000):
        _, i = oracle.topk(x, F32, k, True)
        assert np.array_equal(order[:k], i[0])


# ---------------------------------------------------------------- the property checker rejects planted mistakes

def test_property_checker_rejects_wrong_answers():
    x = W.duplicates(2000, seed=4)
    xb = x.view(np.uint32)
    v, i = oracle.topk(x, F32, 1500, True)          # k-th key lies inside the duplicate class
    verify.check_topk_properties(xb, F32, 1500, True, v[0], i[0])
    # swap a selected tied index for an unselected, higher one
    tied = np.flatnonzero(x == np.float32(0.999))
    unselected = np.setdiff1d(tied, i[0])
    bad_i = i[0].copy()
    pos = np.flatnonzero(np.isin(bad_i, tied))[0]
    bad_i[pos] = unselected[-1]
    with pytest.raises(AssertionError):
        verify.check_topk_properties(xb, F32, 1500, True, xb[bad_i], bad_i)
    # drop the best element for a worse one
    bad_i = i[0].copy()
    worse = np.setdiff1d(np.arange(2000), i[0])[0]
    bad_i[0] = worse
    with pytest.raises(AssertionError):
        verify.check_topk_properties(xb, F32, 1500, True, xb[bad_i], bad_i)
