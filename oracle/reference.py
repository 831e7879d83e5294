"""ctypes front end of the fp64 CPU oracle (``pod_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, the smoke check and the
``cpu_baseline`` leg of the benchmark, never by the product path.  It imports
nothing from the GPU package.

The oracle evaluates the attention equation of the paper's Section 2.1 for a
hybrid batch (causal chunked-prefill rows plus single-token decode rows) in
double precision, straight from the definition.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pod_oracle.c")
_LIB = os.path.join(_HERE, "libpod_oracle.so")

F16, BF16 = 0, 1
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc; returns the path of the shared object."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               _SRC, "-o", tmp, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def bind(path: str):
    """Load a compiled oracle (this one, or a deliberately broken copy a test has built) and
    declare its entry points."""
    lib = ctypes.CDLL(path)
    _declare(lib)
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = bind(build())
    return _lib


def _declare(lib):
    u16p = ctypes.POINTER(ctypes.c_uint16)
    i32p = ctypes.POINTER(ctypes.c_int32)
    lib.pod_oracle_attention.restype = ctypes.c_int
    lib.pod_oracle_attention.argtypes = [
        u16p, u16p, u16p, u16p, i32p, i32p,
        ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
        ctypes.c_double, ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int,
        i32p, ctypes.c_int64, ctypes.POINTER(ctypes.c_double)]
    lib.pod_oracle_widen.restype = ctypes.c_double
    lib.pod_oracle_widen.argtypes = [ctypes.c_int, ctypes.c_uint16]
    lib.pod_oracle_num_threads.restype = ctypes.c_int


def num_threads() -> int:
    """Threads the oracle's parallel loop will use."""
    return int(_load().pod_oracle_num_threads())


def widen(dtype: int, bits: int) -> float:
    """Exact double value of one 16-bit pattern (binary16 or bfloat16)."""
    return float(_load().pod_oracle_widen(dtype, bits))


def _u16(a: Optional[np.ndarray]):
    if a is None:
        return None, ctypes.POINTER(ctypes.c_uint16)()
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("16-bit inputs are passed as their uint16 bit patterns")
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def _i32(a: Optional[np.ndarray]):
    if a is None:
        return None, ctypes.POINTER(ctypes.c_int32)()
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def attention(prefill_q_bits, decode_q_bits, k_bits, v_bits, seq_meta, block_table, *,
              n_prefill: int, n_decode: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
              dtype: int, softmax_scale: float, block_size: int = 0,
              max_blocks_per_seq: int = 0, kv_seq_stride: int = 0, head_major: bool = False,
              rows=None) -> np.ndarray:
    """Oracle output as float64 ``[rows, Hq, d]``.

    All 16-bit tensors are numpy ``uint16`` bit patterns.  ``seq_meta`` is int32
    ``[n_prefill + n_decode, 4]`` = ``(q_start, q_len, kv_len, cache_row)``, prefill
    requests first.  Output rows are the prefill rows followed by one row per decode
    request.  With ``rows`` (global output row indices) only those rows are computed.
    ``head_major``: the cache is [.., Hkv, tokens, d] instead of [.., tokens, Hkv, d].
    """
    lib = _load()
    seq_meta = np.ascontiguousarray(seq_meta, dtype=np.int32).reshape(-1, 4)
    if seq_meta.shape[0] != n_prefill + n_decode:
        raise ValueError("seq_meta must have n_prefill + n_decode rows")
    n_pref_rows = 0
    for r in range(n_prefill):
        n_pref_rows = max(n_pref_rows, int(seq_meta[r, 0] + seq_meta[r, 1]))
    n_total = n_pref_rows + n_decode
    if rows is None:
        rows_arr, rows_ptr, n_rows = None, ctypes.POINTER(ctypes.c_int32)(), n_total
    else:
        rows_arr, rows_ptr = _i32(np.asarray(rows))
        n_rows = int(rows_arr.size)
    out = np.empty((n_rows, n_q_heads, head_dim), dtype=np.float64)
    keep = []
    ptrs = []
    for a in (prefill_q_bits, decode_q_bits, k_bits, v_bits):
        arr, p = _u16(a)
        keep.append(arr)
        ptrs.append(p)
    meta_arr, meta_ptr = _i32(seq_meta)
    bt_arr, bt_ptr = _i32(block_table)
    rc = lib.pod_oracle_attention(
        ptrs[0], ptrs[1], ptrs[2], ptrs[3], meta_ptr, bt_ptr,
        n_prefill, n_decode, n_q_heads, n_kv_heads, head_dim, dtype,
        float(softmax_scale), block_size, max_blocks_per_seq, kv_seq_stride, int(bool(head_major)),
        rows_ptr, n_rows, out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    if rc != 0:
        raise ValueError(f"pod_oracle_attention rejected its arguments (code {rc})")
    del keep, meta_arr, bt_arr, rows_arr
    return out
