"""ctypes front end of the CPU oracle (oracle/jo_attention.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
module; the GPU library never does.  It compiles the C file with gcc on first use
(`build()`), and passes numpy arrays straight through: no attention arithmetic is
done in Python.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "jo_attention.c")
_LIB = os.path.join(_HERE, "libjo_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over output rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def load_library(path: str):
    """Load an oracle shared library and declare its signatures."""
    lib = C.CDLL(path)
    p = C.c_void_p
    common = [p, p, p, p, p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_double]
    lib.jo_decode_attention.argtypes = common + [p, C.c_int, p, p, C.c_int]
    lib.jo_decode_attention.restype = C.c_int
    lib.jo_softmax_weights.argtypes = common + [C.c_int, C.c_int, p]
    lib.jo_softmax_weights.restype = C.c_int
    lib.jo_partial_state.argtypes = common + [C.c_int, C.c_int, p, C.c_int, p, p, p]
    lib.jo_partial_state.restype = C.c_int
    lib.jo_merge_states.argtypes = [C.c_int, p, p, p, C.c_int, p]
    lib.jo_merge_states.restype = C.c_int
    lib.jo_prefill_attention.argtypes = [p, p, p, p, p, p, p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                         C.c_int, C.c_double, p, p, C.c_int]
    lib.jo_prefill_attention.restype = C.c_int
    lib.jo_max_threads.restype = C.c_int
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = load_library(build())
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _common(q, k_pages, v_pages, block_table, seq_lens, scale):
    q = np.ascontiguousarray(q, dtype=np.uint16)
    k_pages = np.ascontiguousarray(k_pages, dtype=np.uint16)
    v_pages = np.ascontiguousarray(v_pages, dtype=np.uint16)
    block_table = np.ascontiguousarray(block_table, dtype=np.int32)
    seq_lens = np.ascontiguousarray(seq_lens, dtype=np.int32)
    B, Hq, D = q.shape
    NP, Hkv, page, D2 = k_pages.shape
    assert D2 == D and v_pages.shape == k_pages.shape
    assert block_table.ndim == 2 and block_table.shape[0] == B and seq_lens.shape == (B,)
    keep = (q, k_pages, v_pages, block_table, seq_lens)
    args = [_ptr(a) for a in keep] + [B, Hq, Hkv, D, page, block_table.shape[1], float(scale)]
    return keep, args, (B, Hq, Hkv, D)


def decode_attention(q, k_pages, v_pages, block_table, seq_lens, *, scale=0.0, rows=None,
                     threads=0, want64=False):
    """Attention output of one decode step.

    Inputs are bf16 bit patterns (uint16) in the documented layouts.  Returns
    float32 [B, Hq, D] (or [n_rows, D] when `rows`, a list of (b, h), is given);
    with want64 also the unrounded float64 array.
    """
    keep, args, (B, Hq, Hkv, D) = _common(q, k_pages, v_pages, block_table, seq_lens, scale)
    if rows is None:
        n, rows_arr, shape = B * Hq, None, (B, Hq, D)
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 2)
        n, shape = rows_arr.shape[0], (rows_arr.shape[0], D)
    o64 = np.empty(shape, dtype=np.float64) if want64 else None
    o32 = np.empty(shape, dtype=np.float32)
    rc = _load().jo_decode_attention(*args, _ptr(rows_arr), n, _ptr(o64), _ptr(o32), int(threads))
    if rc:
        raise ValueError("jo_decode_attention: malformed arguments")
    return (o32, o64) if want64 else o32


def softmax_weights(q, k_pages, v_pages, block_table, seq_lens, b, h, *, scale=0.0):
    keep, args, _ = _common(q, k_pages, v_pages, block_table, seq_lens, scale)
    L = max(int(keep[4][b]), 0)
    w = np.empty(L + 1, dtype=np.float64)
    n = _load().jo_softmax_weights(*args, int(b), int(h), _ptr(w))
    if n < 0:
        raise ValueError("jo_softmax_weights: malformed arguments")
    return w[:n]


def partial_state(q, k_pages, v_pages, block_table, seq_lens, b, h, tokens, *, scale=0.0):
    """(m, l, acc[D]) of row (b, h) over the token subset `tokens`."""
    keep, args, (_, _, _, D) = _common(q, k_pages, v_pages, block_table, seq_lens, scale)
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    m, l = C.c_double(), C.c_double()
    acc = np.empty(D, dtype=np.float64)
    rc = _load().jo_partial_state(*args, int(b), int(h), _ptr(tokens), tokens.size,
                                  C.byref(m), C.byref(l), _ptr(acc))
    if rc:
        raise ValueError("jo_partial_state: malformed arguments")
    return m.value, l.value, acc


def merge_states(ms, ls, accs):
    ms = np.ascontiguousarray(ms, dtype=np.float64)
    ls = np.ascontiguousarray(ls, dtype=np.float64)
    accs = np.ascontiguousarray(accs, dtype=np.float64).reshape(ms.size, -1)
    out = np.empty(accs.shape[1], dtype=np.float64)
    if _load().jo_merge_states(ms.size, _ptr(ms), _ptr(ls), _ptr(accs), accs.shape[1], _ptr(out)):
        raise ValueError("jo_merge_states: malformed arguments")
    return out


def prefill_attention(q, k_pages, v_pages, block_table, seq_lens, q_lens, q_offsets, *, scale=0.0, threads=0,
                      want64=False):
    """Causal attention of each request's last q_lens[b] tokens over its paged cache.

    q is [TQ, Hq, D] (bf16 bits); request b's new tokens are rows q_offsets[b] .. q_offsets[b]+q_lens[b]-1.
    Returns float32 [TQ, Hq, D] (rows no request owns are zero); with want64 also the float64 array."""
    q = np.ascontiguousarray(q, dtype=np.uint16)
    k_pages = np.ascontiguousarray(k_pages, dtype=np.uint16)
    v_pages = np.ascontiguousarray(v_pages, dtype=np.uint16)
    block_table = np.ascontiguousarray(block_table, dtype=np.int32)
    seq_lens = np.ascontiguousarray(seq_lens, dtype=np.int32)
    q_lens = np.ascontiguousarray(q_lens, dtype=np.int32)
    q_offsets = np.ascontiguousarray(q_offsets, dtype=np.int32)
    TQ, Hq, D = q.shape
    NP, Hkv, page, _ = k_pages.shape
    B = seq_lens.shape[0]
    assert q_lens.shape == (B,) and q_offsets.shape[0] >= B and block_table.shape[0] == B
    if B and int(q_offsets[B - 1]) + int(q_lens[B - 1]) > TQ:
        raise ValueError("jo_prefill_attention: q has fewer rows than the offsets and lengths address")
    o32 = np.zeros((TQ, Hq, D), dtype=np.float32)
    o64 = np.zeros((TQ, Hq, D), dtype=np.float64) if want64 else None
    rc = _load().jo_prefill_attention(_ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table), _ptr(seq_lens),
                                      _ptr(q_lens), _ptr(q_offsets), B, Hq, Hkv, D, page, block_table.shape[1],
                                      float(scale), _ptr(o64), _ptr(o32), int(threads))
    if rc:
        raise ValueError("jo_prefill_attention: malformed arguments")
    return (o32, o64) if want64 else o32


def max_threads() -> int:
    return int(_load().jo_max_threads())
