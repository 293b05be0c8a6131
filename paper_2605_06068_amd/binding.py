"""Thin ctypes binding over libpa_decode.so — same names as the C ABI in include/pa_decode.h.

Argument marshalling only: device tensors are torch CUDA tensors (torch supplies device
memory and the current HIP stream), shapes go in a ``pa_shape`` struct, and every step of the
computation runs inside the library's kernels.  There is no CPU fallback: if the library is
missing or cannot be loaded, ``lib()`` raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libpa_decode.so")

PA_OK = 0
PA_ERR_INVALID_ARG = 1
PA_ERR_UNSUPPORTED = 2
PA_ERR_WORKSPACE_TOO_SMALL = 3
PA_ERR_HIP = 4

PA_KV_BF16 = 0
PA_KV_FP8_E4M3 = 1

PA_OUT_F32 = 0
PA_OUT_BF16 = 1

EXPORTS = ("pa_num_partitions", "pa_split_plan", "pa_decode_workspace_size", "pa_decode",
           "pa_decode_static", "pa_kv_append", "pa_decode_trace", "pa_check_tables", "pa_decode_profile", "pa_kernel_variant", "pa_source_digest", "pa_status_string")


class pa_shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "batch", "num_q_heads", "num_kv_heads", "head_dim", "block_size", "max_blocks_per_seq", "num_blocks",
        "max_context_len", "num_partitions", "q_len", "shared_prefix_blocks", "out_dtype", "window", "precise_weights")]


class PaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}")


_lib = None


def lib() -> ctypes.CDLL:
    """Open the in-tree library.  It is built by ``paper_2605_06068_amd.build.build()`` (hipcc).  A
    library that is missing, or that was not built from the sources beside it (its
    pa_source_digest() differs from theirs), is compiled here first; raises if that is impossible."""
    global _lib
    if _lib is not None:
        return _lib
    from . import build as _build

    if _build.built_digest() != _build.source_digest():
        _build.build()
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i32p = ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)
    shp = ctypes.POINTER(pa_shape)
    fp = ctypes.POINTER(ctypes.c_float)
    L.pa_num_partitions.restype = i32
    L.pa_num_partitions.argtypes = [shp, ctypes.c_int]
    L.pa_split_plan.restype = i32
    L.pa_split_plan.argtypes = [shp, ctypes.c_int, i32p, i32p]
    L.pa_decode_workspace_size.restype = ctypes.c_size_t
    L.pa_decode_workspace_size.argtypes = [shp, ctypes.c_int]
    common = [vp, vp, vp, vp, vp, ctypes.c_float, ctypes.c_int, vp, vp, vp, shp, vp, ctypes.c_size_t, vp]
    L.pa_decode.restype = ctypes.c_int
    L.pa_decode.argtypes = common
    L.pa_decode_static.restype = ctypes.c_int
    L.pa_decode_static.argtypes = common[:11] + [vp]
    L.pa_decode_trace.restype = ctypes.c_int
    L.pa_decode_trace.argtypes = common + [vp]
    L.pa_decode_profile.restype = ctypes.c_int
    L.pa_decode_profile.argtypes = common + [i32, fp, fp]
    L.pa_kv_append.restype = ctypes.c_int
    L.pa_kv_append.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.c_int, vp, vp, shp, vp]
    L.pa_check_tables.restype = ctypes.c_int
    L.pa_check_tables.argtypes = [vp, vp, shp, vp, vp]
    L.pa_kernel_variant.restype = ctypes.c_char_p
    L.pa_kernel_variant.argtypes = [shp, ctypes.c_int]
    L.pa_source_digest.restype = ctypes.c_char_p
    L.pa_source_digest.argtypes = []
    L.pa_status_string.restype = ctypes.c_char_p
    L.pa_status_string.argtypes = [ctypes.c_int]
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().pa_status_string(int(status)).decode()


def make_shape(batch, num_q_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq, num_blocks,
               max_context_len=0, num_partitions=0, q_len=0, shared_prefix_blocks=0, window=0,
               out_dtype=PA_OUT_F32, precise_weights=0) -> pa_shape:
    return pa_shape(batch=int(batch), num_q_heads=int(num_q_heads), num_kv_heads=int(num_kv_heads),
                    head_dim=int(head_dim), block_size=int(block_size), max_blocks_per_seq=int(max_blocks_per_seq),
                    num_blocks=int(num_blocks), max_context_len=int(max_context_len),
                    num_partitions=int(num_partitions), q_len=int(q_len),
                    shared_prefix_blocks=int(shared_prefix_blocks), out_dtype=int(out_dtype), window=int(window),
                    precise_weights=int(precise_weights))


def _neg_is_error(v: int, where: str) -> int:
    if v < 0:
        raise PaError(-v, where)
    return v


def pa_num_partitions(shape: pa_shape, kv_dtype: int) -> int:
    return _neg_is_error(lib().pa_num_partitions(ctypes.byref(shape), kv_dtype), "pa_num_partitions")


def pa_split_plan(shape: pa_shape, kv_dtype: int, context_lens):
    """Host plan for a host copy of the context lengths: returns (T, block_partition [B, MB] numpy int32)."""
    import numpy as np

    lens = np.ascontiguousarray(context_lens, dtype=np.int32)
    assert lens.shape == (shape.batch,)
    out = np.zeros((shape.batch, shape.max_blocks_per_seq), dtype=np.int32)
    T = _neg_is_error(lib().pa_split_plan(ctypes.byref(shape), kv_dtype,
                                          lens.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                          out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))), "pa_split_plan")
    return T, out


def pa_decode_workspace_size(shape: pa_shape, kv_dtype: int) -> int:
    return int(lib().pa_decode_workspace_size(ctypes.byref(shape), kv_dtype))


def pa_kernel_variant(shape: pa_shape, kv_dtype: int) -> Optional[str]:
    r = lib().pa_kernel_variant(ctypes.byref(shape), kv_dtype)
    return None if r is None else r.decode()


def _dev_ptr(t, name):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")
    return ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    import torch

    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _common_args(q, k_cache, v_cache, block_tables, context_lens, scale, kv_dtype, out, k_scale, v_scale, shape,
                 workspace, stream):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    return [_dev_ptr(q, "q"), _dev_ptr(k_cache, "k_cache"), _dev_ptr(v_cache, "v_cache"),
            _dev_ptr(block_tables, "block_tables"), _dev_ptr(context_lens, "context_lens"),
            ctypes.c_float(float(scale)), int(kv_dtype), _dev_ptr(out, "out"), _dev_ptr(k_scale, "k_scale"),
            _dev_ptr(v_scale, "v_scale"), ctypes.byref(shape), _dev_ptr(workspace, "workspace"),
            ctypes.c_size_t(ws_bytes), _stream_ptr(stream)]


def pa_decode(q, k_cache, v_cache, block_tables, context_lens, scale, kv_dtype, out, k_scale=None, v_scale=None, *,
              shape: pa_shape, workspace=None, stream=None) -> None:
    """Enqueue one decode attention step on ``stream`` (default: torch's current stream)."""
    st = lib().pa_decode(*_common_args(q, k_cache, v_cache, block_tables, context_lens, scale, kv_dtype, out, k_scale,
                                       v_scale, shape, workspace, stream))
    if st != PA_OK:
        raise PaError(st, "pa_decode")


PA_STATIC_SCRATCH_BYTES = 16 << 20


def pa_decode_static(q, k_cache, v_cache, block_tables, context_lens, scale, kv_dtype, out, k_scale=None, v_scale=None,
                     *, shape: pa_shape, stream=None) -> None:
    """The same step with the library's static scratch array as the workspace (nothing to allocate)."""
    a = _common_args(q, k_cache, v_cache, block_tables, context_lens, scale, kv_dtype, out, k_scale, v_scale, shape,
                     None, stream)
    st = lib().pa_decode_static(*a[:11], a[13])
    if st != PA_OK:
        raise PaError(st, "pa_decode_static")


def pa_kv_append(k_new, v_new, k_cache, v_cache, block_tables, context_lens, kv_dtype, k_scale=None, v_scale=None, *,
                 shape: pa_shape, stream=None) -> None:
    """Enqueue the append of this step's key/value rows into the paged cache."""
    st = lib().pa_kv_append(_dev_ptr(k_new, "k_new"), _dev_ptr(v_new, "v_new"), _dev_ptr(k_cache, "k_cache"),
                            _dev_ptr(v_cache, "v_cache"), _dev_ptr(block_tables, "block_tables"),
                            _dev_ptr(context_lens, "context_lens"), int(kv_dtype), _dev_ptr(k_scale, "k_scale"),
                            _dev_ptr(v_scale, "v_scale"), ctypes.byref(shape), _stream_ptr(stream))
    if st != PA_OK:
        raise PaError(st, "pa_kv_append")


def pa_decode_trace(q, k_cache, v_cache, block_tables, context_lens, scale, kv_dtype, out, k_scale=None, v_scale=None,
                    *, shape: pa_shape, workspace=None, stream=None, visited_blocks) -> None:
    st = lib().pa_decode_trace(*_common_args(q, k_cache, v_cache, block_tables, context_lens, scale, kv_dtype, out,
                                             k_scale, v_scale, shape, workspace, stream),
                               _dev_ptr(visited_blocks, "visited_blocks"))
    if st != PA_OK:
        raise PaError(st, "pa_decode_trace")


PA_TABLES_OK = 0
PA_TABLES_BAD_LENGTH = 1
PA_TABLES_BAD_BLOCK_ID = 2
PA_TABLES_PREFIX_MISMATCH = 3


def pa_check_tables(block_tables, context_lens, *, shape: pa_shape, report, stream=None) -> None:
    """Enqueue the device-side check of the tables and lengths; ``report`` is a device int32[8]."""
    st = lib().pa_check_tables(_dev_ptr(block_tables, "block_tables"), _dev_ptr(context_lens, "context_lens"),
                               ctypes.byref(shape), _dev_ptr(report, "report"), _stream_ptr(stream))
    if st != PA_OK:
        raise PaError(st, "pa_check_tables")


def pa_decode_profile(q, k_cache, v_cache, block_tables, context_lens, scale, kv_dtype, out, k_scale=None,
                      v_scale=None, *, shape: pa_shape, workspace=None, stream=None, steps: int = 10):
    """Returns (partition_ms, merge_ms): mean kernel durations over ``steps`` runs (synchronises)."""
    a, b = ctypes.c_float(0), ctypes.c_float(0)
    st = lib().pa_decode_profile(*_common_args(q, k_cache, v_cache, block_tables, context_lens, scale, kv_dtype, out,
                                               k_scale, v_scale, shape, workspace, stream),
                                 int(steps), ctypes.byref(a), ctypes.byref(b))
    if st != PA_OK:
        raise PaError(st, "pa_decode_profile")
    return float(a.value), float(b.value)


# --------------------------------------------------------------------------------------
# Convenience for tests and the benchmark: put a host-side batch (numpy arrays with the
# fields of workloads.DecodeBatch) into device memory.  torch is used for memory only.
# --------------------------------------------------------------------------------------
class DeviceBatch:
    def __init__(self, batch, device="cuda:0", max_context_len: Optional[int] = None, num_partitions: int = 0,
                 shared_prefix_blocks: Optional[int] = None, window: Optional[int] = None,
                 out_dtype: int = PA_OUT_F32, precise_weights: int = 0):
        import numpy as np
        import torch

        dev = torch.device(device)
        self.host = batch
        self.kv_dtype = int(batch.kv_dtype)
        self.scale = float(batch.scale)

        def up(a):
            return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev)

        # bf16 bit patterns travel as int16 storage; the library only sees the pointer
        self.q = up(batch.q.view(np.int16))
        kv_view = np.int16 if self.kv_dtype == PA_KV_BF16 else np.uint8
        self.k_cache = up(batch.k_cache.view(kv_view))
        self.v_cache = up(batch.v_cache.view(kv_view))
        self.block_tables = up(batch.block_tables)
        self.context_lens = up(batch.context_lens)
        self.k_scale = up(batch.k_scale)
        self.v_scale = up(batch.v_scale)
        q_len = int(getattr(batch, "q_len", 1))
        # bf16 output travels as int16 storage (NaN pattern 0x7FC0 until the library writes it)
        self.out = (torch.full(tuple(batch.q.shape), float("nan"), dtype=torch.float32, device=dev)
                    if out_dtype == PA_OUT_F32 else
                    torch.full(tuple(batch.q.shape), 0x7FC0, dtype=torch.int16, device=dev))
        if max_context_len is None:
            max_context_len = int(batch.context_lens.max(initial=0))
        self.shape = make_shape(batch.batch, batch.num_q_heads, batch.num_kv_heads, batch.head_dim, batch.block_size,
                                batch.max_blocks_per_seq, batch.num_blocks, max_context_len, num_partitions, q_len,
                                int(getattr(batch, "shared_prefix_blocks", 0)) if shared_prefix_blocks is None
                                else shared_prefix_blocks,
                                int(getattr(batch, "window", 0)) if window is None else window, out_dtype,
                                precise_weights)
        nbytes = pa_decode_workspace_size(self.shape, self.kv_dtype)
        # NaN-filled so that a read of an entry this call did not write shows up in the output
        self.workspace = None if nbytes == 0 else torch.full((nbytes // 4,), float("nan"), dtype=torch.float32,
                                                             device=dev)

    def args(self):
        return (self.q, self.k_cache, self.v_cache, self.block_tables, self.context_lens, self.scale, self.kv_dtype,
                self.out, self.k_scale, self.v_scale)

    def decode(self, stream=None):
        pa_decode(*self.args(), shape=self.shape, workspace=self.workspace, stream=stream)
        return self.out
