"""The entry point that allocates nothing (rtopk_select_static: the scratch memory is a buffer inside the
library's device code) against rtopk_select with a caller-owned workspace, through the C-ABI: same selection,
bit for bit, on two calls in a row of which the second has the smaller input, for several launch shapes."""
import numpy as np
import pytest

from paper_2501_14336_amd import workloads as W
from tests.gpu_util import BF16, F16, F32, to_device

pytestmark = pytest.mark.gpu


def _both(bits, dtype, k, largest, flags=0, seed=0):
    import torch
    from paper_2501_14336_amd import binding as B
    x = to_device(bits, dtype)
    batch, n = (1, bits.shape[0]) if bits.ndim == 1 else bits.shape
    stream = torch.cuda.current_stream().cuda_stream
    out = []
    for static in (False, True):
        vals = torch.zeros((batch, k), dtype=x.dtype, device="cuda")
        idx = torch.full((batch, k), -1, dtype=torch.int64, device="cuda")
        if static:
            before = torch.cuda.memory_allocated()
            B.rtopk_select_static(x.data_ptr(), batch, n, k, dtype, largest, flags, seed, vals.data_ptr(),
                                  idx.data_ptr(), stream)
            assert torch.cuda.memory_allocated() <= before      # (torch may release, never acquire, meanwhile)
        else:
            need = B.rtopk_workspace_bytes(batch, n, k, dtype, flags)
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            B.rtopk_select(x.data_ptr(), batch, n, k, dtype, largest, flags, seed, vals.data_ptr(), idx.data_ptr(),
                           ws.data_ptr(), need, stream)
        torch.cuda.synchronize()
        gv = vals.view(torch.int32 if dtype == F32 else torch.int16).cpu().numpy().view(bits.dtype)
        out.append((gv, idx.cpu().numpy()))
    (v0, i0), (v1, i1) = out
    b2 = bits.reshape(1, -1) if bits.ndim == 1 else bits
    for r in range(batch):
        o0, o1 = np.argsort(i0[r], kind="stable"), np.argsort(i1[r], kind="stable")
        assert np.array_equal(i0[r][o0], i1[r][o1]), "row %d: index sets differ" % r
        assert np.array_equal(v0[r][o0], v1[r][o1]), "row %d: value words differ" % r
        assert np.array_equal(b2[r][i1[r]], v1[r]), "row %d: values are not the input's bits" % r
        assert i1[r].min() >= 0


def test_static_scratch_matches_the_workspace_entry_point_twice_in_a_row():
    # larger input first, then a smaller one of the same kind: what the first call left in the buffer must not
    # matter to the second.  Shapes: one workgroup per row (registers, streaming, one sweep), many workgroups per
    # row (two sweeps and, forced by size, the later grid passes), ties, scaling.
    pairs = [
        (lambda n: W.llm_logits(24, n, 91), BF16, (65536, 40001), 50, True, 0),
        (lambda n: W.normal(2 * n, 92).view(np.uint32).reshape(2, n), F32, (300001, 70001), 256, False, 0),
        (lambda n: W.normal(n, 93).view(np.uint32), F32, (2500001, 500001), 4096, True, 0),
        (lambda n: W.duplicates(n, 94).view(np.uint32), F32, (2000003, 300001), 150000, True, 0),
        (lambda n: W.uniform_range(n, 95, 128.6, 128.7).view(np.uint32), F32, (1 << 21, 1 << 19), 512, True, 1),
        (lambda n: W.normal(3 * n, 96).astype(np.float16).view(np.uint16).reshape(3, n), F16, (400001, 8195), 1000, False, 0),
    ]
    for gen, dtype, sizes, k, largest, flags in pairs:
        for n in sizes:
            print("static scratch:", dtype, n, k, largest, flags, flush=True)
            _both(gen(n), dtype, k, largest, flags, seed=11)


def test_static_scratch_rejects_what_does_not_fit_and_bad_arguments():
    import torch
    from paper_2501_14336_amd import binding as B
    x = torch.zeros(16, device="cuda")
    v = torch.zeros(4, device="cuda")
    i = torch.zeros(4, dtype=torch.int64, device="cuda")
    with pytest.raises(B.RtopkError) as e:      # 2^23 fp32 keys in one row need 128 MiB of candidate arrays
        B.rtopk_select_static(x.data_ptr(), 1, 1 << 23, 4, F32, True, 0, 0, v.data_ptr(), i.data_ptr(), 0)
    assert e.value.status == 5 and "RTOPK_STATIC_SCRATCH_BYTES" in str(e.value)
    assert B.rtopk_workspace_bytes(1, 1 << 23, 4, F32) > B.RTOPK_STATIC_SCRATCH_BYTES
    for bad in (dict(k=0), dict(k=17), dict(batch=0), dict(dtype=9), dict(flags=8), dict(keys=0), dict(out_v=0)):
        a = dict(keys=x.data_ptr(), batch=1, n=16, k=4, dtype=F32, flags=0, out_v=v.data_ptr())
        a.update(bad)
        with pytest.raises(B.RtopkError) as e:
            B.rtopk_select_static(a["keys"], a["batch"], a["n"], a["k"], a["dtype"], True, a["flags"], 0, a["out_v"],
                                  i.data_ptr(), 0)
        assert e.value.status == 1, bad
