"""Ragged batches (paper Section 3.2.2; the ablation workload of Section 5.3.3): rows of different lengths in one
array, each with its own k, through rtopk_select_ragged; every row against the sort oracle."""
import numpy as np
import pytest

import oracle
from paper_2501_14336_amd import workloads as W
from tests import verify
from tests.gpu_util import BF16, F16, F32

pytestmark = pytest.mark.gpu


def _run_ragged(rows, dtype, ks, largest=True, tuning=None, sorted=False, scaling=False, n_max=None, k_max=None):
    """rows: list of 1-D arrays of storage words.  Returns (value words [B,k_max], indices [B,k_max], traces)."""
    import torch
    from paper_2501_14336_amd import binding as B
    lens = [int(r.shape[0]) for r in rows]
    word = np.uint32 if dtype == F32 else np.uint16
    flat = np.concatenate([np.asarray(r, word) for r in rows]) if sum(lens) else np.zeros(0, word)
    flat = np.concatenate([flat, np.zeros(8, word)])          # (so that an empty batch still has an address)
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    n_max = n_max or max(max(lens), 1)
    k_max = k_max or max(max(ks), 1)
    if dtype == F32:
        x = torch.from_numpy(flat.view(np.float32)).cuda()
    else:
        x = torch.from_numpy(flat.view(np.int16)).cuda().view(torch.float16 if dtype == F16 else torch.bfloat16)
    vals, idx, ws = B.topk_ragged(x, torch.from_numpy(offs).cuda(), torch.from_numpy(np.asarray(ks, np.int64)).cuda(),
                                  n_max, k_max, largest, scaling=scaling, seed=3, tuning=tuning, sorted=sorted)
    torch.cuda.synchronize()
    gv = vals.view(torch.int32 if dtype == F32 else torch.int16).cpu().numpy().view(word)
    return gv, idx.cpu().numpy(), B.read_trace(ws, len(rows))


def _check_ragged(name, rows, dtype, ks, largest=True, tuning=None, sorted=False, scaling=False):
    print("ragged:", name, "rows", len(rows), "dtype", dtype, "largest", largest, "tuning", tuning, "sorted", sorted, flush=True)
    gv, gi, tr = _run_ragged(rows, dtype, ks, largest, tuning, sorted, scaling)
    for r, (row, k) in enumerate(zip(rows, ks)):
        k = min(k, row.shape[0])
        assert np.all(gi[r, k:] == -1), "row %d: output beyond its k was written" % r
        if k == 0:
            assert not tr[r].passes and tr[r].error == 0
            continue
        assert tr[r].error == 0 and tr[r].done, "row %d: error %d" % (r, tr[r].error)
        wv, wi = oracle.topk(row, dtype, k, largest)
        if sorted:
            assert np.array_equal(gi[r, :k], wi[0]) and np.array_equal(gv[r, :k], wv[0]), "row %d: order" % r
        else:
            verify.assert_same_selection(row, gv[r, :k], gi[r, :k], wv[0], wi[0])


def test_ablation_shape_first_task_one_short():
    # Section 5.3.3: a batch of 16 tasks of 2^20 elements, the first one element shorter, k = 2048, uniform [0, 1)
    n = 1 << 20
    rows = [W.uniform01(n - 1 if r == 0 else n, 200 + r).view(np.uint32) for r in range(16)]
    _check_ragged("ablation", rows, F32, [2048] * 16)
    _check_ragged("ablation sorted", rows, F32, [2048] * 16, sorted=True)


@pytest.mark.parametrize("tuning", [None, dict(path=1), dict(path=2), dict(path=3), dict(path=2, prefilter=1, wgs_per_row=5)])
def test_mixed_lengths_and_ks(tuning):
    lens = [1, 2, 63, 64, 65, 0, 1000, 8191, 8192, 8193, 40000, 100003, 5, 1 << 17, 7]
    rng = np.random.default_rng(5)
    for dtype in (F32, BF16, F16):
        rows, ks = [], []
        for r, n in enumerate(lens):
            x = W.normal(n, 300 + r, sigma=3.0) if r % 3 else W.duplicates(n, 300 + r)
            bits = x.view(np.uint32) if dtype == F32 else W.to_bf16_bits(x) if dtype == BF16 else x.astype(np.float16).view(np.uint16)
            rows.append(bits)
            ks.append(0 if n == 0 else [1, n, max(1, n // 2), min(n, 50), 0][int(rng.integers(0, 5))])
        ks[10] = 256                                        # (something for the one-sweep kernel)
        for largest in (True, False):
            _check_ragged("mixed", rows, dtype, ks, largest, tuning)
        _check_ragged("mixed sorted", rows, dtype, ks, True, tuning, sorted=True)


def test_long_rows_of_different_lengths_large_k_and_scaling():
    lens = [1 << 20, 300001, (1 << 19) + 3, 12345]
    rows = [W.uniform_range(n, 400 + r, 128.6, 128.7).view(np.uint32) for r, n in enumerate(lens)]
    ks = [1 << 18, 300001, 20000, 12000]
    _check_ragged("long", rows, F32, ks)
    _check_ragged("long scaled", rows, F32, ks, scaling=True)
    _check_ragged("long sorted", rows, F32, ks, largest=False, sorted=True)


def test_bad_row_k_is_cut_down_and_reported():
    rows = [W.normal(1000, 500).view(np.uint32), W.normal(2000, 501).view(np.uint32), W.normal(50, 502).view(np.uint32)]
    gv, gi, tr = _run_ragged(rows, F32, [10, 3000, -5], n_max=2000, k_max=2000)
    assert tr[0].error == 0 and tr[1].error == 8 and tr[2].error == 8
    wv, wi = oracle.topk(rows[0], F32, 10, True)
    verify.assert_same_selection(rows[0], gv[0, :10], gi[0, :10], wv[0], wi[0])
    wv, wi = oracle.topk(rows[1], F32, 2000, True)        # cut down to the row's length
    verify.assert_same_selection(rows[1], gv[1, :2000], gi[1, :2000], wv[0], wi[0])
    assert np.all(gi[2] == -1) and not tr[2].passes


def test_ragged_arguments_are_validated_on_the_host():
    import torch
    from paper_2501_14336_amd import binding as B
    x = torch.zeros(64, device="cuda")
    o = torch.zeros(3, dtype=torch.int64, device="cuda")
    v = torch.zeros(8, device="cuda")
    i = torch.zeros(8, dtype=torch.int64, device="cuda")
    ws = torch.zeros(B.rtopk_workspace_bytes(2, 32, 4, F32), dtype=torch.uint8, device="cuda")
    for bad in (dict(offs=0), dict(ks=0), dict(k_max=0), dict(k_max=33), dict(batch=0)):
        a = dict(offs=o.data_ptr(), ks=o.data_ptr(), k_max=4, batch=2)
        a.update(bad)
        with pytest.raises(B.RtopkError) as e:
            B.rtopk_select_ragged(x.data_ptr(), a["offs"], a["ks"], a["batch"], 32, a["k_max"], F32, True, 0, 0, v.data_ptr(),
                                  i.data_ptr(), ws.data_ptr(), ws.numel(), 0)
        assert e.value.status == 1, bad
