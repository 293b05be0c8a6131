"""ctypes front end of the float64 CPU oracle in pa_oracle.c.

TEST INFRASTRUCTURE: imported only by the tests, the smoke check and the benchmark's
CPU-baseline leg.  It never imports the HIP binding and the HIP binding never imports it.
Arrays go in as numpy (bf16 bit patterns as uint16, fp8 bytes as uint8) and come out as
numpy; all arithmetic happens in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pa_oracle.c")
_LIB = os.path.join(_HERE, "libpa_oracle.so")
_lib = None

KV_BF16 = 0
KV_FP8_E4M3 = 1


def build(force: bool = False) -> str:
    """Compile pa_oracle.c with gcc (-O2, OpenMP over output rows) into libpa_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        p = ctypes.c_void_p
        i32, i64 = ctypes.c_int32, ctypes.c_int64
        L.pa_oracle_decode.restype = ctypes.c_int
        L.pa_oracle_decode.argtypes = [p, p, p, p, p, ctypes.c_float, ctypes.c_int, p, p,
                                       i32, i32, i32, i32, i32, i32, i32, i64, p, p, p, p, p, p, i64]
        L.pa_oracle_verify.restype = ctypes.c_int
        L.pa_oracle_verify.argtypes = [p, p, p, p, p, ctypes.c_float, ctypes.c_int, p, p,
                                       i32, i32, i32, i32, i32, i32, i32, i32, i64, p, p, p, p, p, p, p, i64]
        L.pa_oracle_window.restype = ctypes.c_int
        L.pa_oracle_window.argtypes = [p, p, p, p, p, ctypes.c_float, ctypes.c_int, p, p,
                                       i32, i32, i32, i32, i32, i32, i32, i32, i32, i64, p, p, p, p, p, p, p, i64]
        L.pa_oracle_window_blocks.restype = i32
        L.pa_oracle_window_blocks.argtypes = [p, p, i32, i32, i32, i32, p, p, i32]
        L.pa_oracle_block_partition_window.restype = i64
        L.pa_oracle_block_partition_window.argtypes = [p, i32, i32, i32, i32, i32, p]
        L.pa_oracle_e4m3_table.restype = None
        L.pa_oracle_e4m3_table.argtypes = [p]
        L.pa_oracle_visited_blocks.restype = i32
        L.pa_oracle_visited_blocks.argtypes = [p, p, i32, i32, i32, p, i32]
        L.pa_oracle_block_partition.restype = i64
        L.pa_oracle_block_partition.argtypes = [p, i32, i32, i32, i32, p]
        L.pa_oracle_e4m3_encode.restype = ctypes.c_uint
        L.pa_oracle_e4m3_encode.argtypes = [ctypes.c_float]
        L.pa_oracle_kv_append.restype = ctypes.c_int
        L.pa_oracle_kv_append.argtypes = [p, p, p, p, p, p, ctypes.c_int, p, p, i32, i32, i32, i32, i32, i32, i32]
        L.pa_oracle_check_tables.restype = i64
        L.pa_oracle_check_tables.argtypes = [p, p, i32, i32, i32, i32, i32, i32, i32, i32, p]
        L.pa_oracle_set_num_threads.restype = None
        L.pa_oracle_set_num_threads.argtypes = [ctypes.c_int]
        L.pa_oracle_num_threads.restype = ctypes.c_int
        L.pa_oracle_num_threads.argtypes = []
        _lib = L
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a)
    assert a.dtype == dtype, (a.dtype, dtype)
    return a


def decode(q_bits: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray, block_tables: np.ndarray,
           context_lens: np.ndarray, scale, kv_dtype: int = KV_BF16, k_scale: Optional[np.ndarray] = None,
           v_scale: Optional[np.ndarray] = None, rows: Optional[Sequence[Tuple[int, int]]] = None,
           want_f64: bool = False, want_lse: bool = False, want_probs: bool = False):
    """Run the oracle.  Returns a dict with 'out' float32 [B,Hq,D] (or [n_rows,D] when ``rows``
    selects (b,h) pairs) and, on request, 'out_f64', 'lse' and 'probs' ([.., MB*BS], zero past L_b)."""
    q_bits = _c(q_bits, np.uint16)
    kv_np = np.uint16 if kv_dtype == KV_BF16 else np.uint8
    k_cache = _c(k_cache, kv_np)
    v_cache = _c(v_cache, kv_np)
    block_tables = _c(block_tables, np.int32)
    context_lens = _c(context_lens, np.int32)
    B, Hq, D = q_bits.shape
    NB, Hkv, BS, D2 = k_cache.shape
    assert D2 == D and v_cache.shape == k_cache.shape and block_tables.shape[0] == B == context_lens.shape[0]
    MB = block_tables.shape[1]
    if kv_dtype == KV_FP8_E4M3:
        k_scale = _c(k_scale, np.float32)
        v_scale = _c(v_scale, np.float32)
        assert k_scale.shape == (Hkv,) and v_scale.shape == (Hkv,)
    if rows is None:
        n_rows, rb, rh, shape = B * Hq, None, None, (B, Hq, D)
    else:
        rb = np.ascontiguousarray([r[0] for r in rows], dtype=np.int32)
        rh = np.ascontiguousarray([r[1] for r in rows], dtype=np.int32)
        n_rows, shape = len(rows), (len(rows), D)
    out = np.zeros((n_rows, D), dtype=np.float32)
    out64 = np.zeros((n_rows, D), dtype=np.float64) if want_f64 else None
    lse = np.zeros(n_rows, dtype=np.float64) if want_lse else None
    stride = MB * BS
    probs = np.zeros((n_rows, stride), dtype=np.float64) if want_probs else None
    rc = lib().pa_oracle_decode(_ptr(q_bits), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables), _ptr(context_lens),
                                ctypes.c_float(float(np.float32(scale))), int(kv_dtype), _ptr(k_scale), _ptr(v_scale),
                                B, Hq, Hkv, D, BS, MB, NB, n_rows, _ptr(rb), _ptr(rh), _ptr(out), _ptr(out64),
                                _ptr(lse), _ptr(probs), stride)
    if rc != 0:
        raise RuntimeError(f"pa_oracle_decode failed with code {rc}")
    res = {"out": out.reshape(shape)}
    if want_f64:
        res["out_f64"] = out64.reshape(shape)
    if want_lse:
        res["lse"] = lse.reshape(shape[:-1])
    if want_probs:
        res["probs"] = probs.reshape(shape[:-1] + (stride,))
    return res


def verify(q_bits: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray, block_tables: np.ndarray,
           context_lens: np.ndarray, scale, kv_dtype: int = KV_BF16, k_scale: Optional[np.ndarray] = None,
           v_scale: Optional[np.ndarray] = None, rows: Optional[Sequence[Tuple[int, int, int]]] = None,
           want_f64: bool = False, want_lse: bool = False, want_probs: bool = False, window: int = 0):
    """Multi-token causal verification: q_bits is [B, Q, Hq, D]; query token i of sequence b sees the
    logical tokens 0 .. L_b - Q + i, or with ``window`` > 0 only the last ``window`` of them (sliding
    window).  Returns 'out' float32 [B,Q,Hq,D] (or [n_rows,D] when ``rows`` selects (b,i,h) triples)
    and, on request, 'out_f64', 'lse', 'probs' as ``decode`` does."""
    q_bits = _c(q_bits, np.uint16)
    kv_np = np.uint16 if kv_dtype == KV_BF16 else np.uint8
    k_cache = _c(k_cache, kv_np)
    v_cache = _c(v_cache, kv_np)
    block_tables = _c(block_tables, np.int32)
    context_lens = _c(context_lens, np.int32)
    B, Q, Hq, D = q_bits.shape
    NB, Hkv, BS, D2 = k_cache.shape
    assert D2 == D and v_cache.shape == k_cache.shape and block_tables.shape[0] == B == context_lens.shape[0]
    MB = block_tables.shape[1]
    if kv_dtype == KV_FP8_E4M3:
        k_scale = _c(k_scale, np.float32)
        v_scale = _c(v_scale, np.float32)
        assert k_scale.shape == (Hkv,) and v_scale.shape == (Hkv,)
    if rows is None:
        n_rows, rb, ri, rh, shape = B * Q * Hq, None, None, None, (B, Q, Hq, D)
    else:
        rb = np.ascontiguousarray([r[0] for r in rows], dtype=np.int32)
        ri = np.ascontiguousarray([r[1] for r in rows], dtype=np.int32)
        rh = np.ascontiguousarray([r[2] for r in rows], dtype=np.int32)
        n_rows, shape = len(rows), (len(rows), D)
    out = np.zeros((n_rows, D), dtype=np.float32)
    out64 = np.zeros((n_rows, D), dtype=np.float64) if want_f64 else None
    lse = np.zeros(n_rows, dtype=np.float64) if want_lse else None
    stride = MB * BS
    probs = np.zeros((n_rows, stride), dtype=np.float64) if want_probs else None
    common = (_ptr(q_bits), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables), _ptr(context_lens),
              ctypes.c_float(float(np.float32(scale))), int(kv_dtype), _ptr(k_scale), _ptr(v_scale))
    tail = (Hq, Hkv, D, BS, MB, NB, n_rows, _ptr(rb), _ptr(ri), _ptr(rh), _ptr(out), _ptr(out64), _ptr(lse),
            _ptr(probs), stride)
    if window > 0:
        rc = lib().pa_oracle_window(*common, B, Q, int(window), *tail)
    else:
        rc = lib().pa_oracle_verify(*common, B, Q, *tail)
    if rc != 0:
        raise RuntimeError(f"pa_oracle_verify / pa_oracle_window failed with code {rc}")
    res = {"out": out.reshape(shape)}
    if want_f64:
        res["out_f64"] = out64.reshape(shape)
    if want_lse:
        res["lse"] = lse.reshape(shape[:-1])
    if want_probs:
        res["probs"] = probs.reshape(shape[:-1] + (stride,))
    return res


def decode_batch(batch, **kw):
    """Convenience: run on an object with the fields of workloads.DecodeBatch (duck-typed); a batch
    whose q has a query-token axis ([B, Q, Hq, D]) goes through ``verify``, and so does one with a
    sliding window (plain decode is then a window of one query token; rows are (b, h) pairs and
    the result has the shape of q in both cases)."""
    args = (batch.k_cache, batch.v_cache, batch.block_tables, batch.context_lens, batch.scale, batch.kv_dtype,
            batch.k_scale, batch.v_scale)
    window = int(getattr(batch, "window", 0))
    if np.ndim(batch.q) == 4:
        return verify(batch.q, *args, window=window, **kw)
    if window == 0:
        return decode(batch.q, *args, **kw)
    rows = kw.pop("rows", None)
    res = verify(batch.q[:, None], *args, window=window,
                 rows=None if rows is None else [(b, 0, h) for b, h in rows], **kw)
    return res if rows is not None else {k: v[:, 0] for k, v in res.items()}


def e4m3_table() -> np.ndarray:
    t = np.zeros(256, dtype=np.float64)
    lib().pa_oracle_e4m3_table(_ptr(t))
    return t


def visited_blocks(block_tables: np.ndarray, context_lens: np.ndarray, block_size: int, b: int) -> np.ndarray:
    block_tables = _c(block_tables, np.int32)
    context_lens = _c(context_lens, np.int32)
    MB = block_tables.shape[1]
    ids = np.zeros(MB, dtype=np.int32)
    n = lib().pa_oracle_visited_blocks(_ptr(block_tables), _ptr(context_lens), MB, block_size, b, _ptr(ids), MB)
    return ids[:n].copy()


def block_partition(context_lens: np.ndarray, max_blocks_per_seq: int, block_size: int, num_partitions: int,
                    reach: int = 0):
    """Owner partition of every KV block under the balanced split plan; returns (T, [B, MB] int32).
    ``reach`` = window + q_len - 1 > 0 restricts the plan to what a sliding window can see."""
    context_lens = _c(context_lens, np.int32)
    out = np.zeros((len(context_lens), max_blocks_per_seq), dtype=np.int32)
    T = lib().pa_oracle_block_partition_window(_ptr(context_lens), len(context_lens), max_blocks_per_seq, block_size,
                                               int(num_partitions), int(reach), _ptr(out))
    return int(T), out


def window_blocks(block_tables: np.ndarray, context_lens: np.ndarray, block_size: int, b: int, reach: int):
    """Blocks of sequence b that hold a token some query of a sliding-window call can see: returns
    (logical index of the first one, their physical ids in logical order)."""
    block_tables = _c(block_tables, np.int32)
    context_lens = _c(context_lens, np.int32)
    MB = block_tables.shape[1]
    ids = np.zeros(MB, dtype=np.int32)
    first = ctypes.c_int32(0)
    n = lib().pa_oracle_window_blocks(_ptr(block_tables), _ptr(context_lens), MB, block_size, b, int(reach),
                                      ctypes.byref(first), _ptr(ids), MB)
    return int(first.value), ids[:n].copy()


def check_tables(block_tables: np.ndarray, context_lens: np.ndarray, block_size: int, num_blocks: int,
                 max_context_len: int, reach: int = 0, shared_prefix_blocks: int = 0, q_len: int = 1):
    """Check a block table and its lengths against the pool: returns (number of offending entries,
    (kind, b, j, value) of the first in batch order then block order); kind 0 = none, 1 = length,
    2 = block id outside the pool, 3 = shared-prefix entry that differs from row 0."""
    block_tables = _c(block_tables, np.int32)
    context_lens = _c(context_lens, np.int32)
    first = np.zeros(4, dtype=np.int32)
    n = lib().pa_oracle_check_tables(_ptr(block_tables), _ptr(context_lens), len(context_lens), block_tables.shape[1],
                                     int(block_size), int(num_blocks), int(max_context_len), int(reach),
                                     int(shared_prefix_blocks), int(q_len), _ptr(first))
    return int(n), tuple(int(x) for x in first)


def e4m3_encode(x: float) -> int:
    return int(lib().pa_oracle_e4m3_encode(ctypes.c_float(float(x))))


def kv_append(k_new: np.ndarray, v_new: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray,
              block_tables: np.ndarray, context_lens: np.ndarray, kv_dtype: int = KV_BF16,
              k_scale: Optional[np.ndarray] = None, v_scale: Optional[np.ndarray] = None) -> None:
    """Append in place: k_new/v_new are bf16 bit patterns [B, Hkv, D], or [B, Q, Hkv, D] for the Q
    last tokens of every context; caches are modified."""
    k_new = _c(k_new, np.uint16)
    v_new = _c(v_new, np.uint16)
    kv_np = np.uint16 if kv_dtype == KV_BF16 else np.uint8
    assert k_cache.dtype == kv_np and v_cache.dtype == kv_np
    assert k_cache.flags.c_contiguous and v_cache.flags.c_contiguous
    block_tables = _c(block_tables, np.int32)
    context_lens = _c(context_lens, np.int32)
    Q = 1 if k_new.ndim == 3 else k_new.shape[1]
    B, Hkv, D = k_new.shape[0], k_new.shape[-2], k_new.shape[-1]
    assert v_new.shape == k_new.shape
    NB, Hkv2, BS, D2 = k_cache.shape
    assert (Hkv2, D2) == (Hkv, D) and block_tables.shape[0] == B
    if kv_dtype == KV_FP8_E4M3:
        k_scale = _c(k_scale, np.float32)
        v_scale = _c(v_scale, np.float32)
    rc = lib().pa_oracle_kv_append(_ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables),
                                   _ptr(context_lens), int(kv_dtype), _ptr(k_scale), _ptr(v_scale), B, Q, Hkv, D, BS,
                                   block_tables.shape[1], NB)
    if rc != 0:
        raise RuntimeError(f"pa_oracle_kv_append failed with code {rc}")


def set_num_threads(n: int) -> None:
    """Threads the oracle's row loops use from now on."""
    lib().pa_oracle_set_num_threads(int(n))


def num_threads() -> int:
    return int(lib().pa_oracle_num_threads())
