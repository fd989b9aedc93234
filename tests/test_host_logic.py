"""CPU-only checks of the boundary: the C-ABI library loads, exports what include/rtopk.h declares, validates
its arguments on the host (no kernel is launched by any of these calls), and sizes its workspace sensibly.
Also pins the seeded workload generators."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2501_14336_amd import binding as B
from paper_2501_14336_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "rtopk.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rtopk_[a-z_]+)\s*\(", text)))


def test_library_loads_without_a_gpu_and_exports_every_declared_symbol():
    lib = B.load()
    declared = _declared_functions()
    assert set(declared) == set(B.EXPORTS), "binding.EXPORTS must list exactly the header's functions"
    for name in declared:
        assert hasattr(lib, name), "library does not export %s" % name
    assert B.rtopk_version() == "0.1"


def test_header_constants_match_binding():
    text = open(HEADER).read()
    assert int(re.search(r"#define RTOPK_TRACE_STRIDE (\d+)", text).group(1)) == B.RTOPK_TRACE_STRIDE
    assert int(re.search(r"#define RTOPK_TRACE_MAX_PASSES (\d+)", text).group(1)) == B.RTOPK_TRACE_MAX_PASSES
    assert ctypes.sizeof(B.RtopkRowTrace) <= B.RTOPK_TRACE_STRIDE
    assert ctypes.sizeof(B.RtopkTuning) == 20


def test_status_strings():
    assert B.rtopk_status_string(0) == "ok"
    for code in range(1, 5):
        assert B.rtopk_status_string(code) not in ("ok", "unknown status")
    assert B.rtopk_status_string(99) == "unknown status"


def test_workspace_bytes_scales_with_the_candidate_arrays():
    # two candidate arrays of n (raw bits, index) pairs per row dominate
    for batch, n in ((1, 1 << 20), (16, 1 << 18), (1024, 131072)):
        need = B.rtopk_workspace_bytes(batch, n, 10, B.RTOPK_F32)
        assert need >= 2 * 8 * batch * n
        assert need <= 2 * 8 * batch * n + (64 << 20)
    # independent of k and of the direction-independent flags
    assert B.rtopk_workspace_bytes(1, 1 << 20, 1, 0) == B.rtopk_workspace_bytes(1, 1 << 20, 1 << 20, 0)
    # a forced workgroup count changes only the small per-workgroup records
    a = B.rtopk_workspace_bytes(1, 1 << 24, 5, 0, tuning=dict(path=2, wgs_per_row=64))
    b = B.rtopk_workspace_bytes(1, 1 << 24, 5, 0, tuning=dict(path=2, wgs_per_row=512))
    assert 0 < b - a < (32 << 20)


@pytest.mark.parametrize("args", [
    dict(batch=0), dict(n=0), dict(k=0), dict(k=11), dict(dtype=3), dict(dtype=-1), dict(flags=8),
    dict(n=(1 << 31) + 1, k=1),
    dict(tuning=dict(digit_bits=7)), dict(tuning=dict(digit_bits=13)), dict(tuning=dict(path=4)), dict(tuning=dict(prefilter=2)),
    dict(tuning=dict(prefilter=-2)),
    dict(tuning=dict(wgs_per_row=-1)),
])
def test_workspace_bytes_rejects_bad_arguments(args):
    kw = dict(batch=1, n=10, k=5, dtype=0, flags=0, tuning=None)
    kw.update(args)
    with pytest.raises(B.RtopkError) as e:
        B.rtopk_workspace_bytes(kw["batch"], kw["n"], kw["k"], kw["dtype"], kw["flags"], kw["tuning"])
    assert e.value.status == 1


def _select(keys=0x10000, batch=1, n=1000, k=10, dtype=0, largest=True, flags=0, out_v=0x20000, out_i=0x30000,
            ws=0x40000, ws_bytes=1 << 30, tuning=None):
    # fake device addresses: every call below fails validation on the host before anything is launched
    B.rtopk_select(keys, batch, n, k, dtype, largest, flags, 0, out_v, out_i, ws, ws_bytes, 0, tuning)


def test_select_validates_on_the_host_before_launching():
    for bad in (dict(keys=0), dict(out_v=0), dict(out_i=0), dict(ws=0), dict(k=0), dict(k=1001), dict(batch=0),
                dict(dtype=7), dict(flags=8)):
        with pytest.raises(B.RtopkError) as e:
            _select(**bad)
        assert e.value.status == 1, bad
    for bad in (dict(keys=0x10002), dict(out_v=0x20001), dict(out_i=0x30004), dict(ws=0x40010),
                dict(dtype=1, keys=0x10001)):
        with pytest.raises(B.RtopkError) as e:
            _select(**bad)
        assert e.value.status == 3, bad
    with pytest.raises(B.RtopkError) as e:
        _select(ws_bytes=B.rtopk_workspace_bytes(1, 1000, 10, 0) - 1)
    assert e.value.status == 2
    with pytest.raises(B.RtopkError) as e:
        _select(batch=70000, n=100, k=1, tuning=dict(path=2), ws_bytes=1 << 40)
    assert e.value.status == 1          # rows are a grid dimension in the many-workgroup path


def test_sizing_calls_pair_with_the_selection_calls():
    # the plain sizing call is the _ex call with no tuning; the debug-counters flag is accepted and changes nothing
    for batch, n, dt in ((1, 1 << 20, 0), (1024, 131072, 2), (3, 5000, 1)):
        plain = B.rtopk_workspace_bytes(batch, n, 7, dt)
        assert plain == B.rtopk_workspace_bytes(batch, n, 7, dt, tuning=dict())
        assert plain == B.rtopk_workspace_bytes(batch, n, 7, dt, flags=B.RTOPK_FLAG_DEBUG_COUNTERS)
    # a tuning that forces many workgroups per row on a short-row shape needs the candidate arrays: a buffer sized
    # without the tuning is refused (status 2) before anything is launched, and the message says how to size it
    small = B.rtopk_workspace_bytes(1024, 131072, 50, 2)
    forced = B.rtopk_workspace_bytes(1024, 131072, 50, 2, tuning=dict(path=2))
    assert forced > small
    with pytest.raises(B.RtopkError) as e:
        _select(batch=1024, n=131072, k=50, dtype=2, ws_bytes=small, tuning=dict(path=2))
    assert e.value.status == 2 and "rtopk_workspace_bytes_ex" in str(e.value)


def test_topk_wrapper_refuses_cpu_tensors():
    torch = pytest.importorskip("torch")
    with pytest.raises(B.RtopkError):
        B.topk(torch.zeros(10), 3)


# ------------------------------------------------------------------------------------------------ workloads

def test_generators_depend_only_on_seed_and_position():
    a = W.normal(3 * W._CHUNK // 2 + 17, seed=5)
    b = W.normal(100, seed=5)
    assert np.array_equal(a[:100], b)
    assert not np.array_equal(W.normal(100, seed=6), b)
    assert np.array_equal(W.uniform01(1000, 0), W.uniform01(2000, 0)[:1000])
    u = W.uniform01(1 << 16, 0)
    assert u.min() >= 0 and u.max() < 1 and np.all(u * (1 << 24) == np.round(u * (1 << 24)))


def test_bf16_rounding_matches_torch():
    torch = pytest.importorskip("torch")
    x = np.concatenate([W.normal(100000, 1, sigma=30.0), np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1e-40, 3.4e38],
                                                                    dtype=np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = W.to_bf16_bits(x)
    nan = np.isnan(x)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.all((got[nan] & 0x7FFF) > 0x7F80)
    assert np.array_equal(W.bf16_bits_to_f32(got[~nan]), torch.from_numpy(x[~nan]).to(torch.bfloat16).float().numpy())


def test_workload_shapes_and_structure():
    x = W.config5("a", n=1 << 16)
    assert x.min() >= 1.0 and x.max() < 1.0 + 2.0 ** -12 and np.unique(x).size <= 2048
    assert np.all(W.config5("a", n=4096, dtype=np.float16) == np.float16(1.0))
    d = W.config5("b", n=1 << 16)
    assert 0.88 < np.mean(d == np.float32(0.999)) < 0.92
    c = W.config5("c", n=1 << 16)
    assert np.isinf(c).sum() > 0 and np.sum(c == 0) > 0 and not np.isnan(c).any()
    ramp = c[np.isfinite(c) & (np.abs(c) > 1e-30)]
    assert np.all(np.diff(ramp) <= 0)                      # non-increasing ramp
    logits = W.bf16_bits_to_f32(W.llm_logits(4, 8192, 3000))
    assert np.all((logits > 12).sum(axis=1) >= 4)          # the +15 spikes stand out of N(0, 9)
    assert 2.5 < logits.std() < 3.6
    c4 = W.config4(n=1 << 16)
    assert c4.min() >= -1e6 and c4.max() <= 1e6 and abs(c4.mean()) < 2e4
