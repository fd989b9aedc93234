"""Pins for oracle/radix_ref.py (Algorithm 1 step by step): the paper's worked numbers, the order-preserving
key against the oracle's float comparator, and equality of its answer with the sort oracle for every digit
width and with scaling on or off."""
import json
import os

import numpy as np
import pytest

import oracle
from oracle import radix_ref as R
from paper_2501_14336_amd import workloads as W
from tests import verify

F32, F16, BF16 = oracle.F32, oracle.F16, oracle.BF16
PINS = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_pins.json")))


# ---------------------------------------------------------------- numbers printed in the paper

def test_paper_fp32_example_top_digit_0x430():
    pin = PINS["fp32_top12_digit_of_range_128p6_128p7"]
    x = W.uniform_range(20000, seed=1, lo=pin["lo"], hi=pin["hi"])
    x = np.concatenate([x, np.array([pin["lo"], pin["hi"]], dtype=np.float32)])
    raw = x.view(np.uint32)
    assert set(R.get_digit(raw, 20, 32).tolist()) == {int(pin["raw_top12_hex"], 16)}
    # after the order-preserving transform the digit is still a single one (sign bit set for positives)
    assert set(R.get_digit(R.order_key(raw, F32), 20, 32).tolist()) == {int(pin["raw_top12_hex"], 16) | 0x800}


def test_paper_range_0p6_0p7_spans_adjacent_top_digits():
    pin = PINS["fp32_range_0p6_0p7_is_distinguishable_by_top12"]
    x = W.uniform_range(20000, seed=2, lo=pin["lo"], hi=pin["hi"])
    digs = sorted(set(R.get_digit(R.order_key(x.view(np.uint32), F32), 20, 32).tolist()))
    assert len(digs) >= 2 and digs == list(range(digs[0], digs[-1] + 1))


def test_paper_eq3_value():
    pin = PINS["expected_flushes_per_block_per_pass_one_slot_per_thread"]
    r = 2 ** pin["d"]
    assert abs((1 - ((r - 1) / r) ** pin["block"]) - pin["value"]) < pin["abs_tol"]


def test_paper_eq6_same_top12_bits_bound():
    x = W.normal(200000, seed=3, sigma=50.0)
    x = x[(x != 0) & np.isfinite(x)]
    top = R.get_digit(x.view(np.uint32), 20, 32)
    order = np.argsort(top, kind="stable")
    x, top = x[order].astype(np.float64), top[order]
    same = top[1:] == top[:-1]
    h = np.floor(np.log2(np.abs(x[1:])))
    assert np.all(np.abs(x[1:] - x[:-1])[same] < 2.0 ** (h[same] - 3))


def test_uniform_survivor_fraction_is_about_one_over_radix():
    # uniform BIT STRINGS (the paper's model); floats are not uniform over digits
    bits = (W._mix(np.arange(1 << 18, dtype=np.uint64), 5, 0) >> np.uint64(32)).astype(np.uint32)
    bits &= np.uint32(0x7F7FFFFF)                      # finite, positive
    res = R.radix_topk(bits, F32, k=1 << 17, d=8)
    frac = res.passes[0].candidates_after / bits.size
    assert 0.5 / 128 < frac < 2.0 / 128               # 128 reachable top digits for positive finite keys


# ---------------------------------------------------------------- key transform against the float comparator

@pytest.mark.parametrize("dtype", [F16, BF16])
def test_order_key_exhaustive_16bit(dtype):
    allbits = np.arange(65536, dtype=np.uint16)
    order = oracle.sort_row(allbits, dtype, largest=False)          # ascending by the oracle's comparator
    keys = R.order_key(allbits, dtype)[order].astype(np.int64)
    sorted_bits = allbits[order]
    assert np.all(np.diff(keys) >= 0)
    for j in range(65535):
        c = oracle.rank_cmp(dtype, int(sorted_bits[j]), int(sorted_bits[j + 1]))
        assert (keys[j] == keys[j + 1]) == (c == 0)
    nan = R.is_nan_bits(allbits, dtype)
    assert np.all(R.order_key(allbits[nan], dtype) == 0xFFFF)
    # "smallest" is the complement
    assert np.array_equal(R.order_key(allbits, dtype, largest=False), (~R.order_key(allbits, dtype)) & 0xFFFF)


def test_order_key_fp32_boundaries_neighbours_and_random():
    edge = np.array([0x00000000, 0x80000000, 0x00000001, 0x80000001, 0x007FFFFF, 0x00800000, 0x807FFFFF,
                     0x80800000, 0x3F800000, 0xBF800000, 0x7F7FFFFF, 0xFF7FFFFF, 0x7F800000, 0xFF800000,
                     0x7F800001, 0xFFFFFFFF, 0x7FC00000, 0xFFC00000], dtype=np.uint32)
    rng = np.random.default_rng(0)
    rnd = rng.integers(0, 1 << 32, size=3000, dtype=np.uint64).astype(np.uint32)
    nb = np.concatenate([rnd[:500] + np.uint32(1), rnd[:500] - np.uint32(1)])
    bits = np.concatenate([edge, rnd, nb])
    keys = R.order_key(bits, F32).astype(np.int64)
    a, b = bits[:-1], bits[1:]
    for x, y, kx, ky in zip(a, b, keys[:-1], keys[1:]):
        assert np.sign(kx - ky) == oracle.rank_cmp(F32, int(x), int(y))


# ---------------------------------------------------------------- Algorithm 1 reaches the oracle's answer

def _inputs(dtype, n, seed):
    if dtype == F32:
        kinds = [W.normal(n, seed), W.duplicates(n, seed), W.narrow(n, seed),
                 W.specials_ramp(n, seed, with_nan=True), W.uniform_range(n, seed, -1e6, 1e6)]
        return [x.view(np.uint32) for x in kinds]
    if dtype == F16:
        kinds = [W.normal(n, seed).astype(np.float16), W.duplicates(n, seed, dtype=np.float16),
                 W.specials_ramp(n, seed, dtype=np.float16, with_nan=True)]
        return [x.view(np.uint16) for x in kinds]
    return [W.llm_logits(1, n, seed)[0], W.to_bf16_bits(W.specials_ramp(n, seed, with_nan=True))]


@pytest.mark.parametrize("dtype", [F32, F16, BF16])
@pytest.mark.parametrize("d", [4, 8, 11, 12])
@pytest.mark.parametrize("largest", [True, False])
def test_radix_topk_equals_oracle_for_every_digit_width(dtype, d, largest):
    n = 3000
    for seed, bits in enumerate(_inputs(dtype, n, 21)):
        for k in (1, 50, 1500, n):
            want_v, want_i = oracle.topk(bits, dtype, k, largest)
            got = R.radix_topk(bits, dtype, k, d=d, largest=largest)
            verify.assert_same_selection(bits, got.values, got.indices, want_v[0], want_i[0])


@pytest.mark.parametrize("largest", [True, False])
def test_scaling_never_changes_the_answer(largest):
    n = 4000
    for bits in _inputs(F32, n, 33):
        for k in (1, 64, 2000):
            want_v, want_i = oracle.topk(bits, F32, k, largest)
            for s_idx in (0, 17, n - 1, R.draw_scale_index(123, 0, n)):
                got = R.radix_topk(bits, F32, k, d=12, largest=largest, scale_index=s_idx)
                verify.assert_same_selection(bits, got.values, got.indices, want_v[0], want_i[0])


def test_scaling_spreads_the_adversarial_range():
    # Section 5.5: without scaling every key of U[128.6, 128.7] lands in the pivot's bin in pass one;
    # with scaling the first pass already discards most of them.
    n = 1 << 16
    x = W.uniform_range(n, seed=8, lo=128.6, hi=128.7).view(np.uint32)
    plain = R.radix_topk(x, F32, 512, d=12)
    scaled = R.radix_topk(x, F32, 512, d=12, scale_index=R.draw_scale_index(0, 0, n))
    assert plain.passes[0].candidates_after == n
    assert scaled.passes[0].source == "scaled"
    assert scaled.passes[0].candidates_after < n // 4


def test_pass_records_are_consistent():
    x = W.normal(50000, seed=4).view(np.uint32)
    res = R.radix_topk(x, F32, 777, d=12)
    keys = R.order_key(x, F32)
    assert [(p.low, p.high) for p in res.passes] == [(20, 32), (8, 20), (0, 8)]
    cand = np.arange(x.size)
    k = 777
    for p in res.passes:
        dig = R.get_digit(keys[cand], p.low, p.high)
        above = int(np.count_nonzero(dig > p.bin))
        inside = int(np.count_nonzero(dig == p.bin))
        assert above < k <= above + inside           # the two inequalities that define the chosen bin
        k -= above
        assert k == p.k_after and inside == p.candidates_after
        cand = cand[dig == p.bin]


# ------------------------------------------------------------------------------------------------
# the bound the one-sweep kernels rest on: selectBin on a part of a row never overshoots the row's bin, and the
# elements of the bins from that bound upwards carry the whole top of the row's histogram (Section 2.3.1's
# selectBin only looks at the bins from the pivot's bin upwards)
# ------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("largest", [True, False])
@pytest.mark.parametrize("dtype,d", [(oracle.F32, 12), (oracle.BF16, 11), (oracle.F16, 11), (oracle.F32, 8)])
def test_select_bin_on_a_part_bounds_the_row_from_below(dtype, d, largest):
    width = 32 if dtype == oracle.F32 else 16
    low, high = width - d, width
    for seed, bits in enumerate(b for s in range(2) for b in _inputs(dtype, 20000, 200 + s)):
        keys = R.order_key(bits, dtype, largest)
        for k in (1, 7, 50, 999):
            b, _ = R.select_bin(R.count_bin(keys, low, high), k)
            for part in (k, 2500, 10000, 20000):
                if part < k:
                    continue
                b0, _ = R.select_bin(R.count_bin(keys[:part], low, high), k)
                assert b0 <= b
                # what lies in bins >= b0 decides everything: same bin, same pivot rank, and it contains the top k
                kept = R.get_digit(keys, low, high) >= b0
                assert R.select_bin(R.count_bin(keys[kept], low, high), k) == R.select_bin(R.count_bin(keys, low, high), k)
                want_v, want_i = oracle.topk(bits, dtype, k, largest)
                assert np.all(kept[want_i[0]])
            # any subset will do, not just a prefix
            sub = keys[seed::3]
            if sub.size >= k:
                assert R.select_bin(R.count_bin(sub, low, high), k)[0] <= b
