"""ctypes binding of the C-ABI library (include/rtopk.h).

Argument marshalling only: every step of the selection runs in the HIP kernels.
PyTorch supplies device memory (``data_ptr()``) and the current stream.  There is
no fallback: if the library is not built or no GPU is present, calls raise.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
_SRC_DIR = os.path.join(_HERE, "csrc")
_LIB_PATH = os.path.join(_HERE, "librtopk.so")

RTOPK_F32, RTOPK_F16, RTOPK_BF16 = 0, 1, 2
RTOPK_OK = 0
RTOPK_FLAG_SCALING = 1
RTOPK_FLAG_DEBUG_COUNTERS = 2
RTOPK_FLAG_SORTED = 4
RTOPK_TRACE_STRIDE = 512
RTOPK_TRACE_MAX_PASSES = 12

EXPORTS = (
    "rtopk_workspace_bytes",
    "rtopk_workspace_bytes_ex",
    "rtopk_select",
    "rtopk_select_ex",
    "rtopk_select_events",
    "rtopk_select_static",
    "rtopk_select_ragged",
    "rtopk_status_string",
    "rtopk_version",
)


class RtopkTuning(ctypes.Structure):
    _fields_ = [
        ("digit_bits", ctypes.c_int32),
        ("path", ctypes.c_int32),
        ("wgs_per_row", ctypes.c_int32),
        ("small_threshold", ctypes.c_int32),
        ("prefilter", ctypes.c_int32),
    ]


class _PassRec(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in
                ("where", "bin", "k_after", "cand_after", "winners", "out_before", "cand_before", "window")]

    @property
    def source(self):
        return self.window & 0xFF

    @property
    def shift(self):
        return (self.window >> 8) & 0xFF

    @property
    def bits(self):
        return (self.window >> 16) & 0xFF

    @property
    def array(self):
        return (self.window >> 24) & 1


class RtopkRowTrace(ctypes.Structure):
    _fields_ = [("a_s", ctypes.c_float), ("error", ctypes.c_uint32), ("redo", ctypes.c_uint32), ("redo_why", ctypes.c_uint32), ("pre_elems", ctypes.c_uint32), ("pre_bound", ctypes.c_uint32), ("pre_kept", ctypes.c_uint32), ("pre_missed", ctypes.c_uint32), ("pre_merged", ctypes.c_uint32), ("pre_crowd", ctypes.c_uint32), ("reserved", ctypes.c_uint32 * 6),
                ("pass_rec", _PassRec * RTOPK_TRACE_MAX_PASSES)]

    @property
    def passes(self):
        """Records of the passes that ran, in order."""
        out = []
        for r in self.pass_rec:
            if r.where == 0:
                break
            out.append(r)
        return out

    @property
    def done(self):
        ps = self.passes
        return bool(ps) and ps[-1].cand_after == 0


class RtopkError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("rtopk: %s (status %d)" % (message, status))
        self.status = status


_SOURCES = ("rtopk_api.hip", "rtopk_f32.hip", "rtopk_f16.hip", "rtopk_bf16.hip")
_HEADERS = ("rtopk_device.h", "rtopk_host.h", "rtopk_kernels.inl")


def build(force: bool = True) -> str:
    """Compile csrc/ for gfx950 into librtopk.so next to this file (hipcc cross-compiles without a GPU).
    The kernels are instantiated once per key type in separate translation units, compiled in parallel."""
    srcs = [os.path.join(_SRC_DIR, f) for f in _SOURCES]
    deps = srcs + [os.path.join(_SRC_DIR, f) for f in _HEADERS] + [os.path.join(_ROOT, "include", "rtopk.h")]
    if not force and os.path.exists(_LIB_PATH) and all(os.path.getmtime(_LIB_PATH) >= os.path.getmtime(d) for d in deps):
        return _LIB_PATH
    objdir = os.path.join(_HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    common = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
              "-I", os.path.join(_ROOT, "include"), "-I", _SRC_DIR]
    procs, objs = [], []
    for src in srcs:
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        objs.append(obj)
        procs.append((src, subprocess.Popen(common + ["-c", src, "-o", obj], stderr=subprocess.PIPE)))
    # (the device-only feature switch is unknown to hipcc's host pass, which says so once per file: that line is
    # dropped from what is shown; everything else the compiler prints is passed on)
    noise = "'-packed-fp32-ops' is not a recognized feature for this target"
    for src, pr in procs:
        err = pr.communicate()[1].decode(errors="replace")
        shown = "\n".join(l for l in err.splitlines() if noise not in l)
        if shown.strip():
            print(shown, file=sys.stderr)
        if pr.returncode != 0:
            raise RuntimeError("hipcc failed on %s" % src)
    tmp = _LIB_PATH + ".tmp%d" % os.getpid()
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
    os.replace(tmp, _LIB_PATH)
    return _LIB_PATH


_lib = None


def load():
    """Load librtopk.so (built beforehand; built now only if it is missing)."""
    global _lib
    if _lib is None:
        try:  # PyTorch ships its own HIP runtime: let it be the one this process uses
            import torch  # noqa: F401
        except ImportError:
            pass
        if not os.path.exists(_LIB_PATH):
            build(force=True)
        lib = ctypes.CDLL(_LIB_PATH)
        i64, u32, u64, vp, sz = ctypes.c_int64, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_size_t
        lib.rtopk_workspace_bytes.restype = ctypes.c_int
        lib.rtopk_workspace_bytes.argtypes = [i64, i64, i64, ctypes.c_int, u32, ctypes.POINTER(sz)]
        lib.rtopk_workspace_bytes_ex.restype = ctypes.c_int
        lib.rtopk_workspace_bytes_ex.argtypes = [i64, i64, i64, ctypes.c_int, u32, ctypes.POINTER(RtopkTuning),
                                                 ctypes.POINTER(sz)]
        lib.rtopk_select.restype = ctypes.c_int
        lib.rtopk_select.argtypes = [vp, i64, i64, i64, ctypes.c_int, ctypes.c_int, u32, u64, vp, vp, vp, sz, vp]
        lib.rtopk_select_ex.restype = ctypes.c_int
        lib.rtopk_select_ex.argtypes = lib.rtopk_select.argtypes + [ctypes.POINTER(RtopkTuning)]
        lib.rtopk_select_events.restype = ctypes.c_int
        lib.rtopk_select_events.argtypes = lib.rtopk_select_ex.argtypes + [ctypes.POINTER(ctypes.c_void_p)]
        lib.rtopk_select_static.restype = ctypes.c_int
        lib.rtopk_select_static.argtypes = [vp, i64, i64, i64, ctypes.c_int, ctypes.c_int, u32, u64, vp, vp, vp]
        lib.rtopk_select_ragged.restype = ctypes.c_int
        lib.rtopk_select_ragged.argtypes = [vp, vp, vp, i64, i64, i64, ctypes.c_int, ctypes.c_int, u32, u64, vp, vp, vp, sz, vp,
                                            ctypes.POINTER(RtopkTuning)]
        lib.rtopk_status_string.restype = ctypes.c_char_p
        lib.rtopk_status_string.argtypes = [ctypes.c_int]
        lib.rtopk_version.restype = ctypes.c_char_p
        lib.rtopk_version.argtypes = []
        _lib = lib
    return _lib


def rtopk_status_string(status: int) -> str:
    return load().rtopk_status_string(int(status)).decode()


def rtopk_version() -> str:
    return load().rtopk_version().decode()


def _tuning_ptr(tuning):
    if tuning is None:
        return None
    if isinstance(tuning, dict):
        tuning = RtopkTuning(**tuning)
    return ctypes.byref(tuning)


def rtopk_workspace_bytes(batch: int, n: int, k: int, dtype: int, flags: int = 0, tuning=None) -> int:
    """Workspace size: rtopk_workspace_bytes, or rtopk_workspace_bytes_ex when a tuning is given."""
    out = ctypes.c_size_t(0)
    if tuning is None:
        st = load().rtopk_workspace_bytes(batch, n, k, dtype, flags, ctypes.byref(out))
    else:
        st = load().rtopk_workspace_bytes_ex(batch, n, k, dtype, flags, _tuning_ptr(tuning), ctypes.byref(out))
    if st != RTOPK_OK:
        raise RtopkError(st, rtopk_status_string(st))
    return int(out.value)


RTOPK_NUM_EVENTS = 5


def rtopk_select(keys_ptr: int, batch: int, n: int, k: int, dtype: int, largest: bool, flags: int, seed: int,
                 out_values_ptr: int, out_indices_ptr: int, workspace_ptr: int, workspace_bytes: int,
                 stream: int = 0, tuning=None, events=None) -> None:
    """Raw call: device addresses in, nothing allocated, nothing synchronised.
    ``events``: optional sequence of RTOPK_NUM_EVENTS raw hipEvent_t handles (0 = skip), see rtopk_select_events."""
    if events is None:
        st = load().rtopk_select_ex(keys_ptr, batch, n, k, dtype, 1 if largest else 0, flags, seed, out_values_ptr,
                                    out_indices_ptr, workspace_ptr, workspace_bytes, stream, _tuning_ptr(tuning))
    else:
        arr = (ctypes.c_void_p * RTOPK_NUM_EVENTS)(*[int(e) if e else None for e in events])
        st = load().rtopk_select_events(keys_ptr, batch, n, k, dtype, 1 if largest else 0, flags, seed,
                                        out_values_ptr, out_indices_ptr, workspace_ptr, workspace_bytes, stream,
                                        _tuning_ptr(tuning), arr)
    if st != RTOPK_OK:
        raise RtopkError(st, rtopk_status_string(st))


RTOPK_STATIC_SCRATCH_BYTES = 64 << 20


def rtopk_select_static(keys_ptr: int, batch: int, n: int, k: int, dtype: int, largest: bool, flags: int, seed: int,
                        out_values_ptr: int, out_indices_ptr: int, stream: int = 0) -> None:
    """Raw call of the entry point that brings its own scratch memory (no workspace argument, nothing allocated)."""
    st = load().rtopk_select_static(keys_ptr, batch, n, k, dtype, 1 if largest else 0, flags, seed, out_values_ptr,
                                    out_indices_ptr, stream)
    if st != RTOPK_OK:
        raise RtopkError(st, rtopk_status_string(st))


def rtopk_select_ragged(keys_ptr: int, row_offsets_ptr: int, row_k_ptr: int, batch: int, n_max: int, k_max: int, dtype: int,
                        largest: bool, flags: int, seed: int, out_values_ptr: int, out_indices_ptr: int,
                        workspace_ptr: int, workspace_bytes: int, stream: int = 0, tuning=None) -> None:
    """Raw call for a ragged batch: rows of different lengths in one array, each with its own k (device arrays)."""
    st = load().rtopk_select_ragged(keys_ptr, row_offsets_ptr, row_k_ptr, batch, n_max, k_max, dtype, 1 if largest else 0,
                                    flags, seed, out_values_ptr, out_indices_ptr, workspace_ptr, workspace_bytes, stream,
                                    _tuning_ptr(tuning))
    if st != RTOPK_OK:
        raise RtopkError(st, rtopk_status_string(st))


def topk_ragged(x, row_offsets, row_k, n_max: int, k_max: int, largest: bool = True, scaling: bool = False, seed: int = 0,
                tuning=None, sorted: bool = False):
    """Top-k of every row of a ragged batch: ``x`` is the 1-D concatenation of the rows (a CUDA/HIP tensor),
    ``row_offsets`` (batch + 1) and ``row_k`` (batch) are int64 CUDA/HIP tensors.  Returns (values [batch, k_max],
    indices [batch, k_max] filled with -1 beyond each row's k, workspace)."""
    import torch
    batch = row_k.numel()
    code = _torch_dtype_code(x)
    flags = (RTOPK_FLAG_SCALING if scaling else 0) | (RTOPK_FLAG_SORTED if sorted else 0)
    need = rtopk_workspace_bytes(batch, n_max, k_max, code, flags, tuning)
    ws = torch.empty(need, dtype=torch.uint8, device=x.device)
    vals = torch.zeros((batch, k_max), dtype=x.dtype, device=x.device)
    idx = torch.full((batch, k_max), -1, dtype=torch.int64, device=x.device)
    stream = torch.cuda.current_stream(x.device).cuda_stream
    rtopk_select_ragged(x.data_ptr(), row_offsets.data_ptr(), row_k.data_ptr(), batch, n_max, k_max, code, largest, flags,
                        seed, vals.data_ptr(), idx.data_ptr(), ws.data_ptr(), ws.numel(), stream, tuning)
    return vals, idx, ws


# ---------------------------------------------------------------------------
# torch conveniences (memory and stream plumbing only)
# ---------------------------------------------------------------------------

def _torch_dtype_code(t):
    import torch
    return {torch.float32: RTOPK_F32, torch.float16: RTOPK_F16, torch.bfloat16: RTOPK_BF16}[t.dtype]


def topk(x, k: int, largest: bool = True, scaling: bool = False, seed: int = 0, tuning=None, workspace=None,
         out=None, events=None, check: bool = False, sorted: bool = False):
    """Top-k of every row of a CUDA/HIP tensor ``x`` ([n] or [batch, n]; fp32, fp16 or bf16).

    Returns (values [batch, k] of x.dtype, indices [batch, k] int64, workspace).  The order inside a row is
    unspecified unless ``sorted`` (then: best first, lowest index first among equals).  ``workspace`` (a uint8 tensor) and ``out`` (a (values, indices) pair) are reused if given.
    ``check``: synchronise and raise if a kernel flagged an inconsistent state in any row's record (the status
    of the call itself only covers arguments and launches).
    """
    import torch
    if not x.is_cuda:
        raise RtopkError(1, "input tensor must live on the GPU; there is no CPU path")
    if x.dim() == 1:
        x = x[None, :]
    if x.dim() != 2 or not x.is_contiguous():
        raise RtopkError(1, "input must be a contiguous [batch, n] tensor")
    batch, n = x.shape
    code = _torch_dtype_code(x)
    flags = (RTOPK_FLAG_SCALING if scaling else 0) | (RTOPK_FLAG_SORTED if sorted else 0)
    need = rtopk_workspace_bytes(batch, n, k, code, flags, tuning)
    if workspace is None or workspace.numel() < need:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    if out is None:
        vals = torch.empty((batch, k), dtype=x.dtype, device=x.device)
        idx = torch.empty((batch, k), dtype=torch.int64, device=x.device)
    else:
        vals, idx = out
    stream = torch.cuda.current_stream(x.device).cuda_stream
    rtopk_select(x.data_ptr(), batch, n, k, code, largest, flags, seed, vals.data_ptr(), idx.data_ptr(),
                 workspace.data_ptr(), workspace.numel(), stream, tuning, events)
    if check:
        for r, tr in enumerate(read_trace(workspace, batch)):
            if tr.error or not tr.done:
                raise RtopkError(4, "row %d: device error bits %#x, finished=%s" % (r, tr.error, tr.done))
    return vals, idx, workspace


def read_trace(workspace, batch: int):
    """Per-row pass records of the last call that used ``workspace`` (synchronises)."""
    import numpy as np
    raw = workspace[: batch * RTOPK_TRACE_STRIDE].cpu().numpy().tobytes()
    out = []
    for r in range(batch):
        t = RtopkRowTrace.from_buffer_copy(raw[r * RTOPK_TRACE_STRIDE: r * RTOPK_TRACE_STRIDE + ctypes.sizeof(RtopkRowTrace)])
        out.append(t)
    return out
