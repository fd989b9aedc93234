"""GPU parity tests: the HIP path, called through the C-ABI binding, against the CPU oracle.

Bar: bit-exact.  For every row the index SET equals the oracle's (lowest-index-first ties), every output
value is the input's bit pattern at its index, and the sorted value words equal the oracle's.  The order of
outputs inside a row is unspecified at the boundary, so comparisons are made on sets.

Small and medium cases are compared element by element with the sort oracle; they span several 8192-element
tiles, ragged tails, misaligned rows and every code path (one workgroup per row, many workgroups per row,
single-workgroup finish, every digit width, scaling on and off).  The full-size configurations are compared
with the oracle where a full sort finishes in seconds and otherwise checked with the O(n) property test in
tests/verify.py, which decides from the definition alone whether an answer is THE top-k.
"""
import sys

import numpy as np
import pytest

import oracle
from oracle import radix_ref as R
from paper_2501_14336_amd import workloads as W
from tests import verify
from tests.gpu_util import BF16, F16, F32, gpu_topk, to_device

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def _check_rows(bits2d, dtype, k, largest, gv, gi, traces, rows=None):
    rows = range(bits2d.shape[0]) if rows is None else rows
    for r in rows:
        assert traces[r].error == 0, "device error flag %d in row %d" % (traces[r].error, r)
        assert traces[r].done, "row %d did not finish" % r
        wv, wi = oracle.topk(bits2d[r], dtype, k, largest)
        verify.assert_same_selection(bits2d[r], gv[r], gi[r], wv[0], wi[0])


def _run_and_check(name, bits, dtype, k, largest=True, scaling=False, seed=0, tuning=None):
    _say("case:", name, "shape", bits.shape, "k", k, "largest", largest, "scaling", scaling, "tuning", tuning)
    x = to_device(bits, dtype)
    gv, gi, tr, _ = gpu_topk(x, dtype, k, largest, scaling, seed, tuning)
    b2 = bits.reshape(1, -1) if bits.ndim == 1 else bits
    _check_rows(b2, dtype, k, largest, gv, gi, tr)
    return tr


def _expected_a_s(bits_row, seed, row):
    """The element the library must draw as a_s: position from the model's draw, non-finite -> 0 (Section 4.3)."""
    a = np.asarray(bits_row, np.uint32).view(np.float32)[R.draw_scale_index(seed, row, bits_row.shape[0])]
    return np.float32(a) if np.isfinite(a) else np.float32(0.0)


# ------------------------------------------------------------------------------------------------ small / medium

SIZES = [1, 2, 63, 64, 65, 1000, 8191, 8192, 8193, 40000, 100003]


@pytest.mark.parametrize("path", [1, 2, 3])
@pytest.mark.parametrize("n", SIZES)
def test_fp32_normal_all_sizes_both_paths(path, n):
    bits = W.normal(n, seed=n).view(np.uint32)
    for k in sorted({1, min(n, 7), max(1, n // 2), n}):
        for largest in (True, False):
            _run_and_check("normal", bits, F32, k, largest, tuning=dict(path=path))


@pytest.mark.parametrize("path", [1, 2, 3])
def test_duplicates_ties_at_kth_key(path):
    bits = W.duplicates(50000, seed=1).view(np.uint32)
    for k in (10, 30000, 49000):
        _run_and_check("dup", bits, F32, k, True, tuning=dict(path=path))
        # force the many-workgroup kernels through every pass, including the index (tie-break) digits
        _run_and_check("dup multi", bits, F32, k, True, tuning=dict(path=path, small_threshold=1, wgs_per_row=7))
        _run_and_check("dup smallest", bits, F32, k, False, tuning=dict(path=path, small_threshold=1, wgs_per_row=3))


@pytest.mark.parametrize("path", [1, 2, 3])
@pytest.mark.parametrize("d", [8, 11, 12])
def test_special_values_every_digit_width(path, d):
    bits = W.specials_ramp(30001, seed=2, with_nan=True).view(np.uint32)
    for k in (5, 1000, 20000):            # k = 5 lies inside the NaN class
        for largest in (True, False):
            _run_and_check("specials", bits, F32, k, largest, tuning=dict(path=path, digit_bits=d))


@pytest.mark.parametrize("path", [1, 2, 3])
def test_zero_boundary_and_signed_zero_ties(path):
    # many +0 and -0: the k-th key falls on the boundary where a float comparison cannot replace the key
    n = 70001
    x = W.uniform_range(n, 11, -1e6, 1e6)
    x[::7] = 0.0
    x[3::7] = -0.0
    npos = int((x > 0).sum())
    for dtype, bits in ((F32, x.view(np.uint32)), (F16, x.astype(np.float16).view(np.uint16)),
                        (BF16, W.to_bf16_bits(x))):
        for k in (npos, npos + 5, npos + n // 7 + 3, n // 2):
            for largest in (True, False):
                _run_and_check("zero boundary", bits, dtype, k, largest, tuning=dict(path=path))


@pytest.mark.parametrize("path", [1, 2])
def test_scaling_is_result_neutral(path):
    for bits in (W.specials_ramp(30001, seed=3, with_nan=True).view(np.uint32),
                 W.narrow(60000, seed=4).view(np.uint32),
                 W.uniform_range(60000, 5, 128.6, 128.7).view(np.uint32),
                 W.duplicates(60000, seed=6).view(np.uint32)):
        for k in (1, 512, 30000):
            for largest in (True, False):
                for seed in (0, 12345):
                    _run_and_check("scaled", bits, F32, k, largest, scaling=True, seed=seed, tuning=dict(path=path))


@pytest.mark.parametrize("dtype", [F16, BF16])
@pytest.mark.parametrize("path", [1, 2, 3])
def test_16bit_types(dtype, path):
    n = 50001
    if dtype == F16:
        data = [W.normal(n, 7).astype(np.float16).view(np.uint16),
                W.specials_ramp(n, 8, dtype=np.float16, with_nan=True).view(np.uint16),
                W.narrow(n, 9, dtype=np.float16).view(np.uint16)]          # every key equal: ties only
    else:
        data = [W.llm_logits(1, n, 10)[0], W.to_bf16_bits(W.specials_ramp(n, 11, with_nan=True))]
    for bits in data:
        for k in (1, 50, 8192, n):
            for largest in (True, False):
                _run_and_check("16-bit", bits, dtype, k, largest, tuning=dict(path=path))
        _run_and_check("16-bit scaling flag ignored", bits, dtype, 100, True, scaling=True, tuning=dict(path=path))


@pytest.mark.parametrize("path", [1, 2, 3])
def test_batch_with_misaligned_rows(path):
    # odd row lengths: only row 0 starts on a 16-byte boundary
    for dtype, bits in ((BF16, W.llm_logits(9, 4099, 12)), (F32, W.normal(9 * 10007, 13).view(np.uint32).reshape(9, 10007)),
                        (F16, W.normal(5 * 8195, 14).astype(np.float16).view(np.uint16).reshape(5, 8195))):
        for k in (1, 50, 2000):
            _run_and_check("batch misaligned", bits, dtype, k, True, tuning=dict(path=path))
            _run_and_check("batch misaligned", bits, dtype, k, False, tuning=dict(path=path, wgs_per_row=3))


@pytest.mark.parametrize("dtype", [F32, BF16, F16])
def test_rows_at_and_around_the_register_capacity(dtype):
    # one workgroup keeps a row of up to 256 KiB in registers; one element more takes the streaming kernel.
    # Odd lengths also give rows 1 and 2 a lead-in; k = 700 leaves more candidates than the ranking step takes.
    cap = 65536 if dtype == F32 else 131072
    for n in (cap - 1, cap, cap + 1):
        x = W.normal(3 * n, 21 + n % 7, sigma=3.0)
        x[5] = np.inf                      # the raw-bit histogram must notice it and count again exactly
        if dtype == F32:
            bits = x.view(np.uint32)
        elif dtype == BF16:
            bits = W.to_bf16_bits(x)
        else:
            bits = x.astype(np.float16).view(np.uint16)
        bits = bits.reshape(3, n)
        for k in (1, 50, 700):
            for largest in (True, False):
                _run_and_check("register capacity", bits, dtype, k, largest, tuning=dict(path=1))


def test_ranking_step_breaks_ties_by_index_and_leaves_a_record():
    # every key equal: the first digit keeps all n candidates; up to 512 of them are ranked directly (by index,
    # keys being equal), more than that go through further digit passes first
    for n, k in ((300, 100), (512, 1), (512, 512), (513, 100), (5000, 4990)):
        bits = np.full(n, np.float32(2.5)).view(np.uint32)
        for path in (1, 2):
            tr = _run_and_check("all equal", bits, F32, k, True, tuning=dict(path=path))[0]
            last = tr.passes[-1]
            assert last.out_before + last.winners == k
            if n <= 512 and k < n:
                assert [r.source for r in tr.passes] == [1, 3] and last.cand_before == n and last.winners == k
    # ties inside the ranked set with distinct keys around them
    x = W.duplicates(400, seed=31)
    for k in (1, 37, 399):
        for largest in (True, False):
            _run_and_check("dup ranked", x.view(np.uint32), F32, k, largest, tuning=dict(path=1))
            _run_and_check("dup ranked bf16", W.to_bf16_bits(x), BF16, k, largest, tuning=dict(path=2, small_threshold=1))


def test_one_sweep_kernel_and_its_hand_over():
    # path 3: the one-sweep kernel for small k, with every reason it has to hand a row to the two-sweep kernel.
    # Rows that went the short way carry the one-sweep kernel's mark (4) in their records.
    T = dict(path=3)
    short = lambda tr: all(r.where == 4 for r in tr.passes)
    # long rows (several chunks of the hit masks), all three types, both directions, odd lengths in a batch
    x = W.normal(3 * 300001, 41, sigma=3.0)
    for dtype, bits in ((F32, x.view(np.uint32)), (BF16, W.to_bf16_bits(x)), (F16, x.astype(np.float16).view(np.uint16))):
        for k in (1, 50, 256):
            for largest in (True, False):
                trs = _run_and_check("one sweep long rows", bits.reshape(3, 300001), dtype, k, largest, tuning=T)
                if dtype == F32:
                    assert all(short(t) for t in trs)
    # the benchmark's batch shape, a few rows of it
    trs = _run_and_check("one sweep logits", W.llm_logits(24, 131072, 42), BF16, 50, True, tuning=T)
    assert sum(short(t) for t in trs) >= 20
    # +inf / NaN in the first part of the row: raw-bit bins cannot be trusted
    y = W.normal(100000, 43)
    y[7] = np.inf
    assert not short(_run_and_check("inf first", y.view(np.uint32), F32, 20, True, tuning=T)[0])
    y[7] = np.nan
    y[90000] = -np.nan
    _run_and_check("nan first and last", y.view(np.uint32), F32, 20, True, tuning=T)
    # NaN / inf only in the swept part: set aside like any large element, no hand-over needed
    z = W.normal(100000, 44)
    z[60000], z[70000], z[80000] = np.inf, np.nan, -np.inf
    for largest in (True, False):
        _run_and_check("specials late", z.view(np.uint32), F32, 20, largest, tuning=T)
        _run_and_check("specials late bf16", W.to_bf16_bits(z), BF16, 20, largest, tuning=T)
    # the k-th key at a zero / the bin edge is not a number
    q = W.uniform_range(50000, 45, 0.0, 1.0)
    q[::3] = 0.0
    q[1::3] = -0.0
    assert not short(_run_and_check("edge at zero", q.view(np.uint32), F32, 20, False, tuning=T)[0])
    # everything equal: the whole row would be set aside; many equal keys at the k-th: too many to rank
    assert not short(_run_and_check("all equal", np.full(60000, np.float32(3.0)).view(np.uint32), F32, 10, True, tuning=T)[0])
    e = W.normal(80000, 46)
    e[e > 1.5] = 1.5                        # about 5000 copies of the largest value
    assert not short(_run_and_check("flat top", e.view(np.uint32), F32, 100, True, tuning=T)[0])
    # a wide bin at the edge (uniform data just below 1): the early estimate gives the row up
    _run_and_check("uniform", W.uniform01(65536, 47).view(np.uint32), F32, 32, True, tuning=T)
    # descending and ascending sorted rows (hits all in one place / nothing learnt from the first part)
    srt = np.sort(W.normal(70000, 48))
    for arr in (srt, srt[::-1].copy()):
        for largest in (True, False):
            _run_and_check("sorted", arr.view(np.uint32), F32, 64, largest, tuning=T)
    # k beyond what the automatic choice would send here, and k = n
    _run_and_check("large k", W.normal(40000, 49).view(np.uint32), F32, 5000, True, tuning=T)
    _run_and_check("k = n", W.normal(9000, 50).view(np.uint32), F32, 9000, True, tuning=T)


def test_one_sweep_kernel_with_a_sampled_bound():
    # 256 < k <= 512 on rows of 64K keys up: the one-sweep kernel takes its bound from every 4th tile of the row and
    # checks afterwards that the list holds k elements (a guaranteed bound would need most of the row counted first)
    T = dict(path=3)
    short = lambda tr: all(r.where == 4 for r in tr.passes)
    x = W.normal(5 * 70001, 141, sigma=3.0)      # odd length: every row starts off the 16-byte grid
    for dtype, bits in ((F32, x.view(np.uint32)), (BF16, W.to_bf16_bits(x)), (F16, x.astype(np.float16).view(np.uint16))):
        for k in (257, 400, 512):
            for largest in (True, False):
                trs = _run_and_check("sampled bound", bits.reshape(5, 70001), dtype, k, largest, tuning=T)
                if dtype == F32:
                    assert all(short(t) and t.redo_why == 0 for t in trs)
    # the automatic choice takes this way for such batches (a few rows of the benchmark's shape)
    trs = _run_and_check("sampled bound logits", W.llm_logits(100, 131072, 142), BF16, 300, True)
    assert sum(short(t) for t in trs) >= 80
    # a sample that misleads: the 250 largest elements all sit in sampled tiles (tile 0, 4, 8, ... of 8192 elements),
    # so the bound taken from the sample lies above the k-th key and the list comes out short: reason 8, handed over
    n = 16 * 8192
    y = W.uniform01(n, 143)
    pos = np.flatnonzero((np.arange(n) // 8192) % 4 == 0)[:: len(np.flatnonzero((np.arange(n) // 8192) % 4 == 0)) // 250][:250]
    y[pos] = 100.0 + np.arange(len(pos), dtype=np.float32)
    tr = _run_and_check("sample misled", y.view(np.uint32), F32, 400, True, tuning=T)[0]
    assert not short(tr) and tr.redo_why == 8
    # a row whose last tile is one of the sampled ones and is short; a trend along the row; specials in the sample
    z = np.sort(W.normal(8 * 8192 + 100, 144))
    for arr in (z, z[::-1].copy()):
        for largest in (True, False):
            _run_and_check("sampled sorted", arr.view(np.uint32), F32, 300, largest, tuning=T)
    w = W.normal(90000, 145)
    w[3], w[40000] = np.nan, np.inf
    for largest in (True, False):
        _run_and_check("sampled specials", w.view(np.uint32), F32, 300, largest, tuning=T)
    # k above what the automatic choice sends this way (the kernel tries, or hands the row over)
    _run_and_check("k beyond", W.normal(70000, 146).view(np.uint32), F32, 600, True, tuning=T)


@pytest.mark.parametrize("G", [0, 3, 7])
def test_prefilter_sweep(G):
    # many workgroups per row with the prefilter forced on: histogram of a sample of the row, one sweep that counts
    # every digit and keeps the bins from the sample's bound upwards, pass 0 on what was kept
    T = dict(path=2, prefilter=1, wgs_per_row=G)
    for n in (1, 65, 8193, 100003, 300001):
        bits = W.normal(n, seed=60 + n % 13).view(np.uint32)
        for k in sorted({1, min(n, 50), max(1, n // 2), n}):
            for largest in (True, False):
                tr = _run_and_check("prefilter", bits, F32, k, largest, tuning=T)[0]
                assert tr.pre_elems <= n and tr.pre_kept <= n
                if not tr.pre_missed:
                    assert tr.passes[0].cand_before == tr.pre_kept and tr.passes[0].bin >= tr.pre_bound
                if n == 300001:     # 36 full tiles of 8192 elements: tiles 0 and 31 are the sample
                    assert tr.pre_elems == 2 * 8192
    sp = W.specials_ramp(30001, seed=61, with_nan=True).view(np.uint32)
    for k in (5, 1000, 20000):
        for largest in (True, False):
            _run_and_check("prefilter specials", sp, F32, k, largest, tuning=dict(T, small_threshold=1))
    _run_and_check("prefilter duplicates", W.duplicates(50000, seed=62).view(np.uint32), F32, 30000, True,
                   tuning=dict(T, small_threshold=1))
    _run_and_check("prefilter bf16 rows", W.llm_logits(5, 40001, 63), BF16, 50, True, tuning=T)
    _run_and_check("prefilter f16 rows", W.normal(3 * 8195, 64).astype(np.float16).view(np.uint16).reshape(3, 8195), F16, 17, False,
                   tuning=T)
    z = W.uniform_range(70001, 65, -1e6, 1e6)
    z[::7] = 0.0
    z[3::7] = -0.0
    npos = int((z > 0).sum())
    for k in (npos, npos + 5, npos + 70001 // 7 + 3):
        for largest in (True, False):
            _run_and_check("prefilter zero boundary", z.view(np.uint32), F32, k, largest, tuning=T)
    # with scaling the prefilter stays off (the flag wins)
    tr = _run_and_check("prefilter vs scaling", W.uniform_range(60000, 66, 128.6, 128.7).view(np.uint32), F32, 512, True,
                        scaling=True, tuning=T)[0]
    assert tr.pre_elems == 0


@pytest.mark.parametrize("tuning", [dict(), dict(wgs_per_row=7, small_threshold=100)])
def test_prefilter_with_a_misleading_sample(tuning):
    # The sample is every 31st full tile (8192 fp32 elements) of the row.  Here exactly those tiles hold values far
    # better than the rest (spread over many bins, so that the sample does not look crowded), and k exceeds their
    # number, so the bin taken from the sample lies above the k-th key's: the exact counts of the sweep show it, the
    # second sweep over X runs, and the selection is still the oracle's.
    n, k = 2000003, 70000
    planted = (10.0 ** (2.0 + 6.0 * W.uniform01(n, 77))).astype(np.float32)
    for largest in (True, False):
        y = W.normal(n, 6).copy()
        for t in range(0, n // 8192, 31):
            y[t * 8192:(t + 1) * 8192] = planted[t * 8192:(t + 1) * 8192] * (1.0 if largest else -1.0)
        tr = _run_and_check("misleading sample", y.view(np.uint32), F32, k, largest,
                            tuning=dict(path=2, prefilter=1, **tuning))[0]
        assert tr.pre_missed == 1 and tr.pre_elems == 8 * 8192 and 0 < tr.pre_kept < tr.pre_elems
        assert tr.passes[0].bin < tr.pre_bound and tr.passes[0].cand_before == n


def test_prefilter_declines_when_the_keys_crowd_into_the_bins_to_keep():
    # a narrow range, or mostly one value: the sample shows that nearly the whole row would be kept, so the sweep
    # keeps nothing (it only counts) and pass 0 is the ordinary sweep over X
    T = dict(path=2, prefilter=1)
    # (duplicates: nine in ten keys are 0.999, the rest uniform in [0, 1) -- crowded only from the top)
    for name, bits, directions in (("narrow", W.narrow(300001, 75).view(np.uint32), (True, False)),
                                   ("duplicates", W.duplicates(300001, 76).view(np.uint32), (True,))):
        for k in (100, 20000):
            for largest in directions:
                tr = _run_and_check("declined " + name, bits, F32, k, largest, tuning=T)[0]
                assert tr.pre_missed == 2 and tr.pre_kept == 0 and tr.pre_bound == 4096
                assert tr.passes[0].cand_before == 300001


def test_declined_prefilter_counts_two_digits_of_the_crowded_bin():
    # The sweep that declines also counts the second digit of the bin the sample crowds into.  When the exact counts
    # confirm that bin and it holds at least 7/8 of the row, pass 0 has no sweep of its own (an in-place pass whose
    # record says: source X) and pass 1 classifies X by both digits at once.
    T = dict(path=2, prefilter=1, small_threshold=64)
    n = 300001
    cases = [("narrow", W.narrow(n, 175)), ("negative narrow", -W.narrow(n, 176)),
             ("all equal", np.full(n, np.float32(-2.5))), ("duplicates", W.duplicates(n, 177)),
             ("two values", np.where(W.uniform01(n, 178) < 0.5, np.float32(3.0), np.float32(3.0000002)).astype(np.float32))]
    for name, x in cases:
        for k in (100, 20000, n - 5):
            for largest in (True, False):
                tr = _run_and_check("crowd " + name, x.view(np.uint32), F32, k, largest, tuning=T)[0]
                if tr.pre_missed == 2 and tr.pre_merged:
                    r0, r1 = tr.passes[0], tr.passes[1]
                    assert tr.pre_crowd == r0.bin and r0.cand_before == n and (r0.window >> 25) & 3 == 3
                    assert r0.cand_after * 8 > n * 7 and r1.cand_before == r0.cand_after
    # rows that start off the 16-byte grid (the index digits read from X are bounded by position: lead-in included),
    # several rows, 16-bit keys too
    m = 70001
    dup = W.duplicates(3 * m, 180)
    T2 = dict(path=2, small_threshold=64)
    for k in (50, 30000, m - 3):
        for largest in (True, False):
            _run_and_check("in place, odd rows", dup.view(np.uint32).reshape(3, m), F32, k, largest, tuning=T2)
            _run_and_check("in place, odd rows bf16", W.to_bf16_bits(dup).reshape(3, m), BF16, k, largest, tuning=T2)
            _run_and_check("in place, equal rows f16", np.full((3, m), np.float16(1.0)).view(np.uint16), F16, k, largest, tuning=T2)
    # the narrow range and the all-equal row do go that way
    for x in (W.narrow(n, 175), np.full(n, np.float32(-2.5))):
        tr = _run_and_check("crowd taken", x.view(np.uint32), F32, 1000, True, tuning=T)[0]
        assert tr.pre_missed == 2 and tr.pre_merged == 1
    # a crowd of infinities or NaNs: their bin can hold NaNs, which raw bits do not count right -- no second digit
    for v in (np.inf, np.nan):
        y = np.full(n, np.float32(v))
        y[::7] = W.normal(n, 179)[::7]
        for largest in (True, False):
            tr = _run_and_check("crowd of specials", y.view(np.uint32), F32, 5000, largest, tuning=T)[0]
            assert not (tr.pre_missed == 2 and tr.pre_merged)


def test_prefilter_sample_holds_on_independent_draws():
    # On rows of independent draws the bin taken from the sample (with its margin) never lies above the k-th key's
    # bin: the second sweep stays unused, whatever k, and what is kept stays a small part of the row.
    T = dict(path=2, prefilter=1)
    for n, seed in ((1 << 20, 71), (3000001, 72), (1 << 22, 73)):
        for gen in (lambda: W.normal(n, seed), lambda: W.uniform_range(n, seed, -1e6, 1e6), lambda: W.zipf(n, seed).astype(np.float32)):
            bits = gen().view(np.uint32)
            for k in (1, 37, 1000, n // 1000, n // 100, n // 64):
                tr = _run_and_check("independent draws", bits, F32, k, True, tuning=T)[0]
                assert tr.pre_missed == 0 and tr.pre_bound <= tr.passes[0].bin
    bits = W.llm_logits(4, 1 << 20, 74)
    x = to_device(bits, BF16)
    _, _, trs, _ = gpu_topk(x, BF16, 50, True, tuning=T)
    assert all(t.pre_missed == 0 for t in trs)


def test_batch_many_rows_grid_path():
    bits = W.normal(64 * 20000, 15).view(np.uint32).reshape(64, 20000)
    _run_and_check("batch 64 grid", bits, F32, 333, True, tuning=dict(path=2, small_threshold=16))


def test_closed_forms_on_gpu():
    n, k = 100000, 777
    desc = np.linspace(5.0, -5.0, n).astype(np.float32)
    for path in (1, 2):
        x = to_device(desc.view(np.uint32), F32)
        _, gi, _, _ = gpu_topk(x, F32, k, True, tuning=dict(path=path))
        assert np.array_equal(np.sort(gi[0]), np.arange(k))                      # descending input: first k
        _, gi, _, _ = gpu_topk(x, F32, k, False, tuning=dict(path=path))
        assert np.array_equal(np.sort(gi[0]), np.arange(n - k, n))
        eq = np.full(n, 0.999, dtype=np.float32)
        _, gi, _, _ = gpu_topk(to_device(eq.view(np.uint32), F32), F32, k, True, tuning=dict(path=path))
        assert np.array_equal(np.sort(gi[0]), np.arange(k))                      # all equal: lowest indices
        _, gi, _, _ = gpu_topk(to_device(eq.view(np.uint32), F32), F32, n, True, tuning=dict(path=path))
        assert np.array_equal(np.sort(gi[0]), np.arange(n))                      # k = n: everything


def test_same_set_for_every_tuning_and_repeated_runs():
    bits = W.uniform_range(300000, 16, -1e6, 1e6).view(np.uint32)
    k = 20000
    x = to_device(bits, F32)
    want = None
    for tuning in (None, dict(path=1), dict(path=2), dict(path=2, wgs_per_row=1), dict(path=2, wgs_per_row=37),
                   dict(path=2, digit_bits=8, small_threshold=1), dict(digit_bits=11), dict(path=2, small_threshold=100000)):
        for rep in range(3):
            _say("tuning", tuning, "rep", rep)
            gv, gi, tr, _ = gpu_topk(x, F32, k, True, tuning=tuning)
            got = np.sort(gi[0])
            if want is None:
                _check_rows(bits.reshape(1, -1), F32, k, True, gv, gi, tr)
                want = got
            assert np.array_equal(got, want)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_randomised_shapes_types_and_tunings(seed):
    # a seeded walk over (type, batch, n, k, direction, value distribution, every tuning knob): whichever kernels
    # the call ends up in, the selection is the oracle's
    rng = np.random.default_rng(seed)
    kinds = {
        "normal": lambda t, s: W.normal(t, s),
        "uniform": lambda t, s: W.uniform01(t, s),
        "duplicates": lambda t, s: W.duplicates(t, s),
        "narrow": lambda t, s: W.narrow(t, s),
        "specials": lambda t, s: W.specials_ramp(t, s, with_nan=True),
        "constant": lambda t, s: np.full(t, 1.5, np.float32),
        "ascending": lambda t, s: np.arange(t, dtype=np.float32) - t / 3,
        "descending": lambda t, s: t / 3 - np.arange(t, dtype=np.float32),
        "five values": lambda t, s: np.floor(W.uniform01(t, s) * 5).astype(np.float32) - 2,
    }
    names = sorted(kinds)
    for case in range(60):
        dtype = int(rng.integers(0, 3))
        if rng.integers(0, 3):
            n, batch = int(2 ** rng.uniform(0, 17)), int(rng.integers(1, 20))
        else:
            n, batch = int(2 ** rng.uniform(14, 21)), int(rng.integers(1, 4))
        k = [1, int(rng.integers(1, min(n, 64) + 1)), int(rng.integers(1, min(n, 1024) + 1)),
             int(rng.integers(1, n + 1)), max(1, n // 2), n][int(rng.integers(0, 6))]
        largest = bool(rng.integers(0, 2))
        tuning = {}
        if rng.integers(0, 3) == 0:
            tuning["digit_bits"] = int(rng.integers(8, 13))
        if rng.integers(0, 2):
            tuning["path"] = int(rng.integers(1, 4))
        if rng.integers(0, 3) == 0:
            tuning["wgs_per_row"] = int(rng.integers(1, 40))
        if rng.integers(0, 3) == 0:
            tuning["small_threshold"] = int(2 ** rng.uniform(5, 17))
        if rng.integers(0, 3) == 0:
            tuning["prefilter"] = int(rng.integers(-1, 2))
        scaling = dtype == F32 and rng.integers(0, 5) == 0
        name = names[int(rng.integers(0, len(names)))]
        x = np.asarray(kinds[name](batch * n, int(rng.integers(1, 1 << 30))), np.float32)
        with np.errstate(over="ignore"):   # ramps longer than 65504 become infinities in fp16: more ties
            bits = (x.view(np.uint32) if dtype == F32 else
                    x.astype(np.float16).view(np.uint16) if dtype == F16 else W.to_bf16_bits(x)).reshape(batch, n)
        if case % 4 == 3:   # every fourth case with the sorted-output flag: the oracle's order, position by position
            _check_sorted("walk %d/%d %s" % (seed, case, name), bits, dtype, k, largest, tuning=tuning or None,
                          scaling=bool(scaling))
        else:
            _run_and_check("walk %d/%d %s" % (seed, case, name), bits, dtype, k, largest, scaling=bool(scaling),
                           seed=case, tuning=tuning or None)


def test_pass_records_match_algorithm_1_model():
    # the chosen bin, the pivot's rank in it and the candidate count of every key-digit pass equal what the
    # step-by-step numpy model of Algorithm 1 computes (oracle/radix_ref.py)
    bits = W.normal(200000, 17).view(np.uint32)
    for d in (8, 12):
        for largest in (True, False):
            ref = R.radix_topk(bits, F32, 5000, d=d, largest=largest)
            for tuning in (dict(path=1, digit_bits=d), dict(path=2, digit_bits=d, small_threshold=1)):
                tr = _run_and_check("trace", bits, F32, 5000, largest, tuning=tuning)[0]
                out = 0
                for j, rec in enumerate(tr.passes):
                    if rec.source != 1:                 # index digits: tie break, not part of Algorithm 1
                        break
                    want = ref.passes[j]
                    assert (rec.shift, rec.shift + rec.bits) == (want.low, want.high)
                    assert rec.bin == want.bin
                    assert rec.out_before == out
                    if rec.cand_after:
                        assert rec.k_after == want.k_after and rec.cand_after == want.candidates_after
                    else:                                # whole bin taken: the model's pivot rank equals the bin size
                        assert want.k_after == want.candidates_after
                    out += rec.winners
                assert tr.passes[-1].out_before + tr.passes[-1].winners == 5000


def test_scaling_spreads_adversarial_range_on_gpu():
    # Section 5.5's case: every key of U[128.6, 128.7] shares its top 12 bits; with scaling the first pass
    # already discards most keys
    n = 1 << 20
    bits = W.uniform_range(n, 18, 128.6, 128.7).view(np.uint32)
    plain = _run_and_check("adversarial plain", bits, F32, 512, True, tuning=dict(path=2))[0]
    scaled = _run_and_check("adversarial scaled", bits, F32, 512, True, scaling=True, tuning=dict(path=2))[0]
    assert plain.passes[0].cand_after == n
    assert scaled.passes[0].source == 0 and scaled.passes[0].cand_after < n // 4
    assert scaled.a_s == _expected_a_s(bits, 0, 0) and scaled.a_s != 0.0


def test_scaling_draw_is_the_models_and_a_non_finite_draw_disables_it():
    # a_s is the row's element at the position the model draws (one draw per row); inf or NaN there means a_s = 0
    bits = W.uniform_range(5 * 40000, 19, 128.6, 128.7).view(np.uint32).reshape(5, 40000)
    for path in (1, 2):
        for seed in (0, 77, (1 << 40) + 3):
            trs = _run_and_check("a_s draw", bits, F32, 300, True, scaling=True, seed=seed, tuning=dict(path=path))
            for r in range(5):
                assert trs[r].a_s == _expected_a_s(bits[r], seed, r)
                assert trs[r].passes[0].source == 0
    n = 50000
    j = R.draw_scale_index(5, 0, n)
    for bad in (np.inf, -np.inf, np.nan):
        y = W.normal(n, 20)
        y[j] = bad
        for path in (1, 2):
            for largest in (True, False):
                tr = _run_and_check("a_s not finite", y.view(np.uint32), F32, 1000, largest, scaling=True, seed=5,
                                    tuning=dict(path=path))[0]
                assert tr.a_s == 0.0


def test_pass_records_match_algorithm_1_model_with_scaling():
    # with the flag the digits of fl(x - a_s) come first, then the digits of x: bins, pivot ranks and candidate
    # counts of every pass equal the model's for the same draw
    n, k, seed = 200000, 5000, 9
    bits = W.uniform_range(n, 22, 128.6, 128.7).view(np.uint32)
    j = R.draw_scale_index(seed, 0, n)
    names = {0: "scaled", 1: "key"}
    for d in (8, 12):
        for largest in (True, False):
            ref = R.radix_topk(bits, F32, k, d=d, largest=largest, scale_index=j)
            for tuning in (dict(path=1, digit_bits=d), dict(path=2, digit_bits=d, small_threshold=1)):
                tr = _run_and_check("scaled trace", bits, F32, k, largest, scaling=True, seed=seed, tuning=tuning)[0]
                assert tr.a_s == np.float32(ref.a_s)
                out = 0
                for q, rec in enumerate(tr.passes):
                    if rec.source not in names:       # index digits or the ranking step: not part of Algorithm 1
                        break
                    want = ref.passes[q]
                    assert names[rec.source] == want.source
                    assert (rec.shift, rec.shift + rec.bits) == (want.low, want.high)
                    assert rec.bin == want.bin and rec.out_before == out
                    if rec.cand_after:
                        assert rec.k_after == want.k_after and rec.cand_after == want.candidates_after
                    else:
                        assert want.k_after == want.candidates_after
                    out += rec.winners
                assert tr.passes[-1].out_before + tr.passes[-1].winners == k


def test_kernels_stay_inside_the_workspace_and_the_outputs():
    # The workspace (exactly the reported size) and both outputs are carved out of larger pattern-filled buffers;
    # the bytes on either side must be untouched afterwards, whichever kernels ran.
    import torch
    from paper_2501_14336_amd import binding as B
    guard = 1 << 16
    cases = [
        (W.normal(100003, 81).view(np.uint32), F32, 777, dict(path=2)),
        (W.normal(100003, 81).view(np.uint32), F32, 100003, dict(path=2, wgs_per_row=5, small_threshold=1)),
        (W.normal(300001, 82).view(np.uint32), F32, 5000, dict(path=2, prefilter=1)),
        (W.narrow(300001, 83).view(np.uint32), F32, 5000, dict(path=2, prefilter=1)),                # declines
        (W.duplicates(90001, 84).view(np.uint32), F32, 45000, dict(path=2, small_threshold=1, digit_bits=8)),
        (W.normal(7 * 10007, 85).view(np.uint32).reshape(7, 10007), F32, 333, dict(path=2, wgs_per_row=3)),
        (W.llm_logits(9, 40001, 86), BF16, 50, dict(path=2, prefilter=1)),
        (W.llm_logits(9, 4099, 87), BF16, 4099, dict(path=1)),
        (W.normal(5 * 8195, 88).astype(np.float16).view(np.uint16).reshape(5, 8195), F16, 17, dict(path=3)),
        (W.normal(3 * 300001, 89).view(np.uint32).reshape(3, 300001), F32, 256, dict(path=3)),
        (W.normal(70001, 90).view(np.uint32), F32, 35000, None),
        (np.full(300001, np.float32(1.25)).view(np.uint32), F32, 777, dict(path=2, prefilter=1, small_threshold=64)),  # crowded bin
        (W.llm_logits(5, 70001, 91), BF16, 400, dict(path=3)),                                       # sampled bound
        (W.normal(100003, 92).view(np.uint32), F32, 20000, dict(path=2, sorted=True)),                # radix sort on the grid
        (W.normal(3 * 20001, 93).view(np.uint32).reshape(3, 20001), F32, 8192, dict(path=1, sorted=True)),   # sort in LDS
    ]
    for bits, dtype, k, tuning in cases:
        tuning = dict(tuning) if tuning else None
        sorted_out = bool(tuning.pop("sorted", False)) if tuning else False
        for scaling in ((False, True) if dtype == F32 and not (tuning or {}).get("prefilter") else (False,)):
            _say("guards:", bits.shape, dtype, k, tuning, "scaling", scaling, "sorted", sorted_out)
            x = to_device(bits, dtype)
            batch, n = (1, bits.shape[0]) if bits.ndim == 1 else bits.shape
            es = 4 if dtype == F32 else 2
            need = B.rtopk_workspace_bytes(batch, n, k, dtype, (B.RTOPK_FLAG_SCALING if scaling else 0) |
                                           (B.RTOPK_FLAG_SORTED if sorted_out else 0), tuning)
            wbuf = torch.full((need + 2 * guard,), 0xA5, dtype=torch.uint8, device="cuda")
            vbuf = torch.full((batch * k * es + 2 * guard,), 0xA5, dtype=torch.uint8, device="cuda")
            ibuf = torch.full((batch * k * 8 + 2 * guard,), 0xA5, dtype=torch.uint8, device="cuda")
            assert wbuf.data_ptr() % 256 == 0 and vbuf.data_ptr() % 256 == 0 and ibuf.data_ptr() % 256 == 0
            ws = wbuf[guard:guard + need]
            vals = vbuf[guard:guard + batch * k * es].view(x.dtype).view(batch, k)
            idx = ibuf[guard:guard + batch * k * 8].view(torch.int64).view(batch, k)
            B.topk(x, k, True, scaling=scaling, seed=3, tuning=tuning, workspace=ws, out=(vals, idx), check=True,
                   sorted=sorted_out)
            torch.cuda.synchronize()
            for name, buf, size in (("workspace", wbuf, need), ("values", vbuf, batch * k * es), ("indices", ibuf, batch * k * 8)):
                assert bool((buf[:guard] == 0xA5).all()), "%s: bytes before the buffer were written" % name
                assert bool((buf[guard + size:] == 0xA5).all()), "%s: bytes after the buffer were written" % name
            gv = vals.view(torch.int32 if dtype == F32 else torch.int16).cpu().numpy().view(bits.dtype)
            b2 = bits.reshape(1, -1) if bits.ndim == 1 else bits
            _check_rows(b2, dtype, k, True, gv, idx.cpu().numpy(), B.read_trace(ws, batch))


def _check_sorted(name, bits, dtype, k, largest, tuning=None, scaling=False):
    """With the sorted-output flag the result equals the oracle's position by position (the oracle's order is best
    first, lowest index first among equal elements)."""
    _say("sorted:", name, bits.shape, "dtype", dtype, "k", k, "largest", largest, "tuning", tuning)
    x = to_device(bits, dtype)
    gv, gi, tr, _ = gpu_topk(x, dtype, k, largest, scaling=scaling, seed=5, tuning=tuning, sorted=True)
    b2 = bits.reshape(1, -1) if bits.ndim == 1 else bits
    wv, wi = oracle.topk(b2, dtype, k, largest)
    for r in range(b2.shape[0]):
        assert tr[r].error == 0 and tr[r].done
        assert np.array_equal(gi[r], wi[r]), "row %d: indices differ from the oracle's order" % r
        assert np.array_equal(gv[r], wv[r]), "row %d: value words differ from the oracle's order" % r


@pytest.mark.parametrize("path", [1, 2])
def test_sorted_output_small_k_in_lds(path):
    T = dict(path=path)
    x = W.normal(100003, 101)
    for k in (1, 2, 50, 63, 64, 65, 1000, 4097, 8191, 8192):
        for largest in (True, False):
            _check_sorted("normal", x.view(np.uint32), F32, k, largest, T)
    # ties: equal keys come out in index order; special values in their places (NaN first for largest)
    for k in (10, 5000, 8192):
        for largest in (True, False):
            _check_sorted("duplicates", W.duplicates(50000, 102).view(np.uint32), F32, k, largest, T)
            _check_sorted("specials", W.specials_ramp(30001, 103, with_nan=True).view(np.uint32), F32, k, largest, T)
            _check_sorted("specials fp16", W.specials_ramp(30001, 104, dtype=np.float16, with_nan=True).view(np.uint16), F16,
                          k, largest, T)
            _check_sorted("constant", np.full(20000, np.float32(1.5)).view(np.uint32), F32, k, largest, T)
    _check_sorted("logits batch", W.llm_logits(9, 40001, 105), BF16, 50, True, T)
    _check_sorted("logits batch", W.llm_logits(9, 40001, 105), BF16, 8192, True, T)
    _check_sorted("fp32 batch odd rows", W.normal(7 * 10007, 106).view(np.uint32).reshape(7, 10007), F32, 333, False, T)
    _check_sorted("k = n", W.normal(5000, 107).view(np.uint32), F32, 5000, True, T)
    _check_sorted("scaled", W.uniform_range(60000, 108, 128.6, 128.7).view(np.uint32), F32, 512, True, T, scaling=True)


def test_sorted_output_large_k_radix_sort():
    # beyond one workgroup's LDS: radix sort on the grid, chunks per workgroup, skipped passes
    x = W.normal(300001, 111)
    for k in (8193, 50000, 300001):
        for largest in (True, False):
            _check_sorted("normal", x.view(np.uint32), F32, k, largest)
    _check_sorted("duplicates", W.duplicates(200003, 112).view(np.uint32), F32, 150000, True)
    _check_sorted("duplicates", W.duplicates(200003, 112).view(np.uint32), F32, 150000, False, dict(path=2, wgs_per_row=7))
    _check_sorted("constant", np.full(100000, np.float32(-2.0)).view(np.uint32), F32, 60000, True)
    _check_sorted("specials", W.specials_ramp(100001, 113, with_nan=True).view(np.uint32), F32, 70000, True)
    _check_sorted("specials", W.specials_ramp(100001, 113, with_nan=True).view(np.uint32), F32, 70000, False)
    _check_sorted("bf16", W.llm_logits(3, 100001, 114), BF16, 20000, True)            # 16-bit keys: low key bytes skipped
    _check_sorted("fp16", W.normal(2 * 70001, 115).astype(np.float16).view(np.uint16).reshape(2, 70001), F16, 70001, False)
    _check_sorted("batch", W.normal(5 * 40000, 116).view(np.uint32).reshape(5, 40000), F32, 9000, True, dict(path=1))
    _check_sorted("2^22", W.uniform_range(1 << 22, 117, -1e6, 1e6).view(np.uint32), F32, 1 << 20, True)


# ------------------------------------------------------------------------------------------------ full sizes

def test_config1_full():
    bits = W.config1().view(np.uint32)
    _run_and_check("config 1", bits, F32, 32, True)
    _check_sorted("config 1", bits, F32, 32, True)


def test_config2_full_k_sweep_both_directions():
    x = W.config2()
    bits = x.view(np.uint32)
    xd = to_device(bits, F32)
    ws = None
    for largest in (True, False):
        _say("config 2: oracle sort, largest =", largest)
        order = oracle.sort_row(bits, F32, largest)
        for k in (16, 256, 4096, 65536, 1 << 20):
            _say("config 2 k", k)
            gv, gi, tr, ws = gpu_topk(xd, F32, k, largest, workspace=ws)
            assert tr[0].error == 0 and tr[0].done
            verify.assert_same_selection(bits, gv[0], gi[0], bits[order[:k]], order[:k])


def test_config3_full_batch_bf16():
    _say("config 3: generating 1024 x 131072 bf16")
    bits = W.config3()
    xd = to_device(bits, BF16)
    ws = None
    sample_rows = list(range(0, 1024, 97))
    for k in (50, 1024, 8192):
        _say("config 3 k", k)
        gv, gi, tr, ws = gpu_topk(xd, BF16, k, True, workspace=ws)
        _check_rows(bits, BF16, k, True, gv, gi, tr, rows=sample_rows)           # sort oracle on sampled rows
        for r in range(1024):                                                     # definition check on every row
            assert tr[r].error == 0 and tr[r].done
            verify.check_topk_properties(bits[r], BF16, k, True, gv[r], gi[r])


@pytest.mark.timeout(900)
def test_config4_full_large_k():
    # the headline configuration against the sort oracle: ONE full sort of the 2^28 (element, index) pairs, whose
    # first k entries are the answer for every k; the property check stays beside it as a second, independent test
    _say("config 4: generating 2^28 fp32")
    x = W.config4()
    bits = x.view(np.uint32)
    xd = to_device(bits, F32)
    _say("config 4: oracle sort of 2^28 pairs")
    order = oracle.sort_row(bits, F32, True)
    ws = None
    for k in (1 << 20, 1 << 24, 1 << 27):
        _say("config 4 k", k)
        gv, gi, tr, ws = gpu_topk(xd, F32, k, True, workspace=ws)
        assert tr[0].error == 0 and tr[0].done
        _say("config 4 k", k, ": comparing with the oracle's first k")
        verify.assert_same_selection(bits, gv[0], gi[0], bits[order[:k]], order[:k])
        _say("config 4 k", k, ": definition check")
        verify.check_topk_properties(bits, F32, k, True, gv[0], gi[0])


@pytest.mark.timeout(900)
@pytest.mark.parametrize("case", ["a", "b", "c"])
@pytest.mark.parametrize("dt", [np.float32, np.float16])
def test_config5_full_adversarial(case, dt):
    # one oracle sort per (dataset, direction); scaling on and off must both give its first k
    _say("config 5", case, dt.__name__, ": generating 2^26")
    x = W.config5(case, dtype=dt)
    dtype = F32 if dt == np.float32 else F16
    bits = verify.as_bits(x, dtype)
    xd = to_device(bits, dtype)
    k = 1 << 16
    ws = None
    for largest in (True, False):
        _say("config 5", case, "largest", largest, ": oracle sort of 2^26 pairs")
        order = oracle.sort_row(bits, dtype, largest)
        for scaling in ((False, True) if dtype == F32 else (False,)):
            _say("config 5", case, "largest", largest, "scaling", scaling)
            gv, gi, tr, ws = gpu_topk(xd, dtype, k, largest, scaling=scaling, seed=77, workspace=ws)
            assert tr[0].error == 0 and tr[0].done
            verify.assert_same_selection(bits, gv[0], gi[0], bits[order[:k]], order[:k])
            verify.check_topk_properties(bits, dtype, k, largest, gv[0], gi[0])
            if scaling:
                assert tr[0].a_s == _expected_a_s(bits, 77, 0)
    if case == "a" and dtype == F16:
        # every fp16 key equals 1.0: the answer is the first k indices
        assert np.array_equal(np.sort(gi[0]), np.arange(k))


def test_streamed_row_whose_prefilter_declines():
    # 2^27 fp32 keys (512 MB: read with non-temporal loads) in a narrow range: the sample shows the keys crowded
    # into one bin, the prefilter sweep only counts, and pass 0 is the second sweep over X in its streaming form.
    # (No full sort here: the definition check decides; the same shape at 2^26 is compared with the oracle above.)
    n, k = 1 << 27, 1 << 16
    _say("narrow 2^27: generating")
    bits = W.narrow(n, 5101).view(np.uint32)
    xd = to_device(bits, F32)
    for largest in (True, False):
        _say("narrow 2^27 largest", largest)
        gv, gi, tr, _ = gpu_topk(xd, F32, k, largest)
        assert tr[0].error == 0 and tr[0].done
        assert tr[0].pre_missed == 2 and tr[0].pre_kept == 0 and tr[0].passes[0].cand_before == n
        verify.check_topk_properties(bits, F32, k, largest, gv[0], gi[0])
