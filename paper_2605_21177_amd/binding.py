"""ctypes binding of libchunkft: argument marshalling only.

Function names match the C ABI in include/chunkft.h.  Tensors are torch
tensors on the GPU (torch is used for device memory and streams only); every
step of the path runs in the library's kernels.  There is no fallback: if the
shared library is missing, loading raises.
"""

from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libchunkft.so")

OK = 0
ERR_INVALID_ARG = -1
ERR_RANGE = -2
ERR_DTYPE = -3
ERR_WORKSPACE = -4
ERR_BUFFER_TOO_SMALL = -5
ERR_HIP = -6
ERR_OVERFLOW = -7
ERR_STATIC_WORKSPACE = -8
STATIC_WORKSPACE_BYTES = 64 << 20

F32 = 0
BF16 = 1
LINEAR = 0
VECTOR = 1
EMBEDDING = 2
RMSNORM = 3
LAYERNORM = 4

PLAN_GREEDY = 0
PLAN_TRAINING_COST = 1
PLAN_BALANCED = 2
PLAN_ROWS8 = 4


class TensorDesc(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64), ("dtype", C.c_int32), ("kind", C.c_int32)]


class Segment(C.Structure):
    _fields_ = [("tensor", C.c_int32), ("reserved", C.c_int32), ("begin", C.c_int64),
                ("end", C.c_int64), ("chunk_off", C.c_int64)]


class Chunk(C.Structure):
    _fields_ = [("seg_begin", C.c_int64), ("seg_end", C.c_int64), ("numel", C.c_int64),
                ("cost_bytes", C.c_int64)]


class PlanSummary(C.Structure):
    _fields_ = [("n_chunks", C.c_int64), ("min_cost_bytes", C.c_int64), ("max_cost_bytes", C.c_int64),
                ("mean_cost_bytes", C.c_double), ("imbalance_bytes", C.c_double), ("jitter", C.c_double),
                ("jitter_bound", C.c_double)]


class AdamWHparams(C.Structure):
    _fields_ = [("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double),
                ("weight_decay", C.c_double), ("step", C.c_int64)]


class Layer(C.Structure):
    _fields_ = [("kind", C.c_int32), ("dtype", C.c_int32), ("out", C.c_int64), ("n_in", C.c_int64),
                ("T", C.c_int64), ("X", C.c_void_p), ("ldx", C.c_int64), ("dY", C.c_void_p),
                ("lddy", C.c_int64), ("split_k", C.c_int32), ("reserved", C.c_int32),
                ("norm_eps", C.c_double)]


class GroupSegment(C.Structure):
    _fields_ = [("layer", Layer), ("begin", C.c_int64), ("end", C.c_int64), ("W", C.c_void_p),
                ("master", C.c_void_p), ("m", C.c_void_p), ("v", C.c_void_p)]


class ScheduleEntry(C.Structure):
    _fields_ = [("active", C.c_int32), ("load_before", C.c_int32), ("offload_after", C.c_int32),
                ("reserved", C.c_int32), ("local_step", C.c_int64)]


class ChunkFTError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None
TIMELINE_LIB_PATH = os.path.join(_HERE, "libchunkft_timeline.so")


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        _lib = _load(LIB_PATH)
    return _lib


class use_library:
    """with use_library(handle): the calls of this module go to another build of the library (the
    diagnostic twin that bench.py --timeline loads)."""

    def __init__(self, handle):
        self.handle = handle

    def __enter__(self):
        global _lib
        self.prev, _lib = _lib, self.handle
        return self.handle

    def __exit__(self, *exc):
        global _lib
        _lib = self.prev


def load_timeline_library() -> C.CDLL:
    """libchunkft_timeline.so: the same sources with the MFMA kernel's phase time stamps compiled in."""
    L = _load(TIMELINE_LIB_PATH)
    L.chunkft_timeline_buffer.restype = C.c_int
    L.chunkft_timeline_buffer.argtypes = [C.c_void_p, C.c_size_t]
    return L


def _load(path) -> C.CDLL:
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} is missing: build it with `python -m paper_2605_21177_amd.build` "
            "(there is no fallback path)")
    L = C.CDLL(path)
    L.chunkft_plan_cycle.restype = C.c_int
    L.chunkft_plan_cycle.argtypes = [C.POINTER(TensorDesc), C.c_int32, C.c_int64, C.c_uint32,
                                     C.POINTER(Chunk), C.c_int64, C.POINTER(C.c_int64),
                                     C.POINTER(Segment), C.c_int64, C.POINTER(C.c_int64)]
    L.chunkft_plan_stats.restype = C.c_int
    L.chunkft_plan_stats.argtypes = [C.POINTER(Chunk), C.c_int64, C.c_int64, C.POINTER(PlanSummary)]
    L.chunkft_split_k.restype = C.c_int
    L.chunkft_split_k.argtypes = [C.POINTER(Layer), C.c_int64, C.c_int64]
    L.chunkft_workspace_bytes.restype = C.c_size_t
    L.chunkft_workspace_bytes.argtypes = [C.POINTER(Layer), C.c_int64, C.c_int64]
    L.chunkft_chunk_wgrad.restype = C.c_int
    L.chunkft_chunk_wgrad.argtypes = [C.POINTER(Layer), C.c_int64, C.c_int64, C.c_void_p, C.c_int,
                                      C.c_void_p, C.c_size_t, C.c_void_p]
    L.chunkft_adamw_chunk.restype = C.c_int
    L.chunkft_adamw_chunk.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_int32, C.c_int64, C.POINTER(AdamWHparams), C.c_void_p]
    L.chunkft_wgrad_adamw_fused.restype = C.c_int
    L.chunkft_wgrad_adamw_fused.argtypes = [C.POINTER(Layer), C.c_int64, C.c_int64, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.POINTER(AdamWHparams), C.c_void_p, C.c_size_t,
                                            C.c_void_p]
    L.chunkft_group_workspace_bytes.restype = C.c_size_t
    L.chunkft_group_workspace_bytes.argtypes = [C.POINTER(GroupSegment), C.c_int32]
    L.chunkft_wgrad_adamw_fused_group.restype = C.c_int
    L.chunkft_wgrad_adamw_fused_group.argtypes = [C.POINTER(GroupSegment), C.c_int32, C.POINTER(AdamWHparams),
                                                  C.c_void_p, C.c_size_t, C.c_void_p]
    L.chunkft_wgrad_adamw_fused_static.restype = C.c_int
    L.chunkft_wgrad_adamw_fused_static.argtypes = [C.POINTER(Layer), C.c_int64, C.c_int64, C.c_void_p,
                                                   C.c_void_p, C.c_void_p, C.c_void_p,
                                                   C.POINTER(AdamWHparams), C.c_void_p]
    L.chunkft_status_string.restype = C.c_char_p
    L.chunkft_status_string.argtypes = [C.c_int]
    L.chunkft_version.restype = C.c_int
    L.chunkft_version.argtypes = []
    L.chunkft_mover_create.restype = C.c_int
    L.chunkft_mover_create.argtypes = [C.POINTER(C.c_void_p)]
    L.chunkft_mover_destroy.restype = None
    L.chunkft_mover_destroy.argtypes = [C.c_void_p]
    L.chunkft_mover_load.restype = C.c_int
    L.chunkft_mover_load.argtypes = [C.c_void_p] + [C.c_void_p] * 6 + [C.c_int64, C.c_void_p]
    L.chunkft_mover_await_load.restype = C.c_int
    L.chunkft_mover_await_load.argtypes = [C.c_void_p, C.c_void_p]
    L.chunkft_mover_offload.restype = C.c_int
    L.chunkft_mover_offload.argtypes = [C.c_void_p] + [C.c_void_p] * 6 + [C.c_int64, C.c_void_p]
    L.chunkft_mover_sync.restype = C.c_int
    L.chunkft_mover_sync.argtypes = [C.c_void_p]
    L.chunkft_schedule_at.restype = C.c_int
    L.chunkft_schedule_at.argtypes = [C.c_int64, C.c_int32, C.c_int64, C.POINTER(ScheduleEntry)]
    L.chunkft_calib_mfma_bf16_shape.restype = C.c_int
    L.chunkft_calib_mfma_bf16_shape.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t,
                                                C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_void_p]
    L.chunkft_calib_mfma_bf16.restype = C.c_int
    L.chunkft_calib_mfma_bf16.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.POINTER(C.c_double),
                                          C.POINTER(C.c_double), C.c_void_p]
    return L


EXPORTS = ("chunkft_plan_cycle", "chunkft_plan_stats", "chunkft_split_k", "chunkft_workspace_bytes", "chunkft_chunk_wgrad",
           "chunkft_adamw_chunk", "chunkft_wgrad_adamw_fused", "chunkft_wgrad_adamw_fused_static",
           "chunkft_wgrad_adamw_fused_group", "chunkft_group_workspace_bytes", "chunkft_status_string",
           "chunkft_version", "chunkft_calib_mfma_bf16", "chunkft_calib_mfma_bf16_shape", "chunkft_schedule_at",
           "chunkft_mover_create", "chunkft_mover_destroy", "chunkft_mover_load", "chunkft_mover_await_load",
           "chunkft_mover_offload", "chunkft_mover_sync")


def status_string(status: int) -> str:
    return lib().chunkft_status_string(int(status)).decode()


def version() -> int:
    return lib().chunkft_version()


# ---------------------------------------------------------------- planner
def chunkft_plan_cycle(tensors: Sequence[Tuple[int, int, int, int]], budget_bytes: int, flags: int = 0,
                       check: bool = True):
    """tensors: (rows, cols, dtype, kind).  Returns (status, chunks, segments) with
    chunks = [(seg_begin, seg_end, numel, cost_bytes)] and
    segments = [(tensor, begin, end, chunk_off)]."""
    n = len(tensors)
    arr = (TensorDesc * max(n, 1))()
    for i, (r, c, d, k) in enumerate(tensors):
        arr[i] = TensorDesc(r, c, d, k)
    nc, ns = C.c_int64(0), C.c_int64(0)
    st = lib().chunkft_plan_cycle(arr, n, budget_bytes, flags, None, 0, C.byref(nc), None, 0, C.byref(ns))
    if st not in (OK, ERR_BUFFER_TOO_SMALL):
        if check:
            raise ChunkFTError(st, "chunkft_plan_cycle")
        return st, [], []
    chunks = (Chunk * max(nc.value, 1))()
    segs = (Segment * max(ns.value, 1))()
    st = lib().chunkft_plan_cycle(arr, n, budget_bytes, flags, chunks, nc.value, C.byref(nc), segs,
                                  ns.value, C.byref(ns))
    if st != OK:
        if check:
            raise ChunkFTError(st, "chunkft_plan_cycle")
        return st, [], []
    out_c = [(chunks[i].seg_begin, chunks[i].seg_end, chunks[i].numel, chunks[i].cost_bytes)
             for i in range(nc.value)]
    out_s = [(segs[i].tensor, segs[i].begin, segs[i].end, segs[i].chunk_off) for i in range(ns.value)]
    return OK, out_c, out_s


def chunkft_plan_stats(chunks: Sequence[Tuple[int, int, int, int]], resident_bytes: int, check: bool = True):
    """chunks as chunkft_plan_cycle returns them.  Returns a dict with the fields of
    chunkft_plan_summary, or the status."""
    n = len(chunks)
    arr = (Chunk * max(n, 1))()
    for i, (s0, s1, numel, cost) in enumerate(chunks):
        arr[i] = Chunk(s0, s1, numel, cost)
    out = PlanSummary()
    st = lib().chunkft_plan_stats(arr, n, resident_bytes, C.byref(out))
    if st != OK:
        if check:
            raise ChunkFTError(st, "chunkft_plan_stats")
        return st
    return {name: getattr(out, name) for name, _ in PlanSummary._fields_}


# ---------------------------------------------------------- device calls
def _torch_dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def make_layer(kind: int, X, dY, out: int, n_in: int, split_k: int = 0, norm_eps: float = 0.0) -> Layer:
    """Describe a backward step from two row-major device tensors: X [T, in] and dY
    (for EMBEDDING X is the 1-D int64 tensor of token ids)."""
    if dY.dim() != 2 or dY.stride(1) != 1:
        raise ValueError("dY must be 2-D with unit inner stride")
    if not (X.is_cuda and dY.is_cuda):
        raise ValueError("X and dY must live on the GPU")
    d = _torch_dtype_code(dY)
    if kind == EMBEDDING:
        import torch
        if X.dim() != 1 or X.dtype != torch.int64 or X.stride(0) != 1 or X.shape[0] != dY.shape[0]:
            raise ValueError("token ids must be a contiguous 1-D int64 tensor with one id per row of dY")
        return Layer(kind, d, out, n_in, X.shape[0], X.data_ptr(), 1, dY.data_ptr(), dY.stride(0), split_k, 0, 0.0)
    if X.dim() != 2 or X.stride(1) != 1:
        raise ValueError("X must be 2-D with unit inner stride")
    if _torch_dtype_code(X) != d:
        raise TypeError("X and dY must share a dtype")
    return Layer(kind, d, out, n_in, X.shape[0], X.data_ptr(), X.stride(0), dY.data_ptr(), dY.stride(0),
                 split_k, 0, float(norm_eps))


def chunk_array(n: int, begin: int, device="cuda", fill=None):
    """An fp32 device array of n elements for a chunk segment that starts at tensor element
    `begin` (g, master, m or v), placed so that element i has the 128-byte phase of tensor
    element begin + i: the 16-byte groups and the memory lines of the array then coincide with
    those of the tensor's rows, which is the layout the fused call streams fastest (any 4-byte
    aligned pointer is accepted).  Allocation only."""
    import torch
    full = torch.empty(n + 32, dtype=torch.float32, device=device)
    lead = (begin - full.data_ptr() // 4) % 32
    view = full[lead:lead + n]
    if fill is not None:
        view.copy_(fill)
    return view


def chunk_state(n: int, begin: int, device="cuda", count: int = 3):
    """`count` fp32 device arrays of n elements each for one chunk segment (master, m, v; with
    count = 4 also g), cut from one allocation.  Each sits at the 128-byte phase of tensor element
    `begin`, like chunk_array's, and consecutive arrays lie a whole number of MiB plus 256 KiB
    apart: streams that advance together through arrays a whole MiB multiple apart can fall on the
    same memory channels (the fused call on 128 MiB arrays: 188 us at this spacing, 203 - 229 us
    at 129 MiB).  Contents are uninitialised."""
    import torch
    mib = 1 << 18                                           # floats
    pitch = -(-n // mib) * mib + mib // 4
    buf = torch.empty(pitch * (count - 1) + n + 32, dtype=torch.float32, device=device)
    lead = (begin - buf.data_ptr() // 4) % 32
    return tuple(buf[lead + i * pitch: lead + i * pitch + n] for i in range(count))


def _stream_ptr(stream) -> int:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def chunkft_split_k(layer: Layer, begin: int, end: int) -> int:
    return lib().chunkft_split_k(C.byref(layer), begin, end)


def chunkft_workspace_bytes(layer: Layer, begin: int, end: int) -> int:
    return lib().chunkft_workspace_bytes(C.byref(layer), begin, end)


def chunkft_chunk_wgrad(layer: Layer, begin: int, end: int, g, accumulate: bool = False, ws=None,
                        stream=None, check: bool = True) -> int:
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    st = lib().chunkft_chunk_wgrad(C.byref(layer), begin, end, _ptr(g), int(accumulate), _ptr(ws),
                                   ws_bytes, _stream_ptr(stream))
    if check and st != OK:
        raise ChunkFTError(st, "chunkft_chunk_wgrad")
    return st


def hparams(lr, beta1, beta2, eps, weight_decay, step) -> AdamWHparams:
    return AdamWHparams(lr, beta1, beta2, eps, weight_decay, step)


def chunkft_adamw_chunk(g, master, m, v, W_at_begin, n: int, hp: AdamWHparams, w_dtype: int = BF16,
                        stream=None, check: bool = True) -> int:
    st = lib().chunkft_adamw_chunk(_ptr(g), _ptr(master), _ptr(m), _ptr(v), _ptr(W_at_begin), w_dtype,
                                   n, C.byref(hp), _stream_ptr(stream))
    if check and st != OK:
        raise ChunkFTError(st, "chunkft_adamw_chunk")
    return st


def chunkft_wgrad_adamw_fused(layer: Layer, begin: int, end: int, W, master, m, v, hp: AdamWHparams,
                              ws=None, stream=None, check: bool = True) -> int:
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    st = lib().chunkft_wgrad_adamw_fused(C.byref(layer), begin, end, _ptr(W), _ptr(master), _ptr(m),
                                         _ptr(v), C.byref(hp), _ptr(ws), ws_bytes, _stream_ptr(stream))
    if check and st != OK:
        raise ChunkFTError(st, "chunkft_wgrad_adamw_fused")
    return st


CALIB_SCRATCH_BYTES = 4096


def _calib_scratch():
    import torch
    return torch.empty(CALIB_SCRATCH_BYTES, dtype=torch.uint8, device="cuda")


class GroupCall:
    """The segments of one chunk marshalled once for chunkft_wgrad_adamw_fused_group.
    segments: (layer, begin, end, W, master, m, v) with the state arrays already offset to the segment.
    Keeps the tensors alive and allocates the workspace the call asks for (usually none)."""

    def __init__(self, segments, device="cuda", workspace=None):
        import torch
        self._keep = list(segments)
        n = len(self._keep)
        self.n = n
        self.arr = (GroupSegment * max(n, 1))()
        for i, (layer, begin, end, W, master, m, v) in enumerate(self._keep):
            self.arr[i] = GroupSegment(layer, begin, end, _ptr(W), _ptr(master), _ptr(m), _ptr(v))
        self.ws_bytes = lib().chunkft_group_workspace_bytes(self.arr, n) if n else 0
        self.ws = workspace
        if self.ws is None and self.ws_bytes:
            self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=device)

    def __call__(self, hp: AdamWHparams, stream=None, check: bool = True) -> int:
        ws_bytes = 0 if self.ws is None else self.ws.numel() * self.ws.element_size()
        st = lib().chunkft_wgrad_adamw_fused_group(self.arr, self.n, C.byref(hp), _ptr(self.ws), ws_bytes,
                                                   _stream_ptr(stream))
        if check and st != OK:
            raise ChunkFTError(st, "chunkft_wgrad_adamw_fused_group")
        return st


def chunkft_wgrad_adamw_fused_static(layer: Layer, begin: int, end: int, W, master, m, v, hp: AdamWHparams,
                                     stream=None, check: bool = True) -> int:
    """The fused call with its workspace in the library's own static device array (no allocation)."""
    st = lib().chunkft_wgrad_adamw_fused_static(C.byref(layer), begin, end, _ptr(W), _ptr(master), _ptr(m),
                                                _ptr(v), C.byref(hp), _stream_ptr(stream))
    if check and st != OK:
        raise ChunkFTError(st, "chunkft_wgrad_adamw_fused_static")
    return st


def chunkft_calib_mfma_bf16(random_operands: bool, steps: int = 4000, stream=None) -> Tuple[float, float]:
    """(TFLOP/s, shader MHz) that 32x32x16 MFMAs issued from registers sustain on the current device."""
    tf, mhz = C.c_double(0.0), C.c_double(0.0)
    scratch = _calib_scratch()
    st = lib().chunkft_calib_mfma_bf16(1 if random_operands else 0, steps, scratch.data_ptr(), CALIB_SCRATCH_BYTES,
                                       C.byref(tf), C.byref(mhz), _stream_ptr(stream))
    if st != OK:
        raise ChunkFTError(st, "chunkft_calib_mfma_bf16")
    return tf.value, mhz.value


def chunkft_calib_mfma_bf16_shape(shape: int, random_operands: bool, steps: int = 4000,
                                  stream=None) -> Tuple[float, float]:
    """The same for MFMA shape 32 (32x32x16) or 16 (16x16x32)."""
    tf, mhz = C.c_double(0.0), C.c_double(0.0)
    scratch = _calib_scratch()
    st = lib().chunkft_calib_mfma_bf16_shape(shape, 1 if random_operands else 0, steps, scratch.data_ptr(),
                                             CALIB_SCRATCH_BYTES, C.byref(tf), C.byref(mhz), _stream_ptr(stream))
    if st != OK:
        raise ChunkFTError(st, "chunkft_calib_mfma_bf16_shape")
    return tf.value, mhz.value


def chunkft_schedule_at(step: int, n_chunks: int, interval: int, check: bool = True):
    """(active chunk, load_before, offload_after, local_step) of a training step, or the status."""
    e = ScheduleEntry()
    st = lib().chunkft_schedule_at(step, n_chunks, interval, C.byref(e))
    if st != OK:
        if check:
            raise ChunkFTError(st, "chunkft_schedule_at")
        return st
    return e.active, bool(e.load_before), bool(e.offload_after), e.local_step


class Mover:
    """chunkft_mover_*: asynchronous host <-> device copies of a chunk's (master, m, v)."""

    def __init__(self):
        h = C.c_void_p()
        st = lib().chunkft_mover_create(C.byref(h))
        if st != OK:
            raise ChunkFTError(st, "chunkft_mover_create")
        self._h = h

    def close(self):
        if self._h:
            lib().chunkft_mover_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st, where):
        if st != OK:
            raise ChunkFTError(st, where)

    def load(self, dev3, host3, n, after_stream=None):
        self._check(lib().chunkft_mover_load(self._h, *[_ptr(t) for t in dev3], *[_ptr(t) for t in host3], n,
                                             _stream_ptr(after_stream)), "chunkft_mover_load")

    def await_load(self, compute_stream=None):
        self._check(lib().chunkft_mover_await_load(self._h, _stream_ptr(compute_stream)), "chunkft_mover_await_load")

    def offload(self, host3, dev3, n, compute_stream=None):
        self._check(lib().chunkft_mover_offload(self._h, *[_ptr(t) for t in host3], *[_ptr(t) for t in dev3], n,
                                                _stream_ptr(compute_stream)), "chunkft_mover_offload")

    def sync(self):
        self._check(lib().chunkft_mover_sync(self._h), "chunkft_mover_sync")
