"""CPU oracle for the mask-only logits path (Mosaic, arXiv 2601.06562, sections 2.1, 3 obs. #2, 4.2).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this; only the
tests, the smoke check and the benchmark's ``cpu_baseline`` leg do.  The arithmetic
lives in ``mosaic_oracle.c`` (plain C, fp64 accumulation); this file only builds that
C file with gcc and marshals numpy arrays to it.

bf16 arrays are passed as ``numpy.uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mosaic_oracle.c")
_LIB = os.path.join(_HERE, "libmosaic_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile mosaic_oracle.c into libmosaic_oracle.so beside it (gcc, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-mavx2", "-mfma", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        p = ctypes.c_void_p
        i64, i32 = ctypes.c_int64, ctypes.c_int32
        lib.oracle_mask_select.restype = i64
        lib.oracle_mask_select.argtypes = [p, i64, p]
        lib.oracle_row_logits.restype = None
        lib.oracle_row_logits.argtypes = [p, p, i32, i32, p]
        lib.oracle_row_logits_f32seq.restype = None
        lib.oracle_row_logits_f32seq.argtypes = [p, p, i32, i32, p]
        lib.oracle_row_reduce.restype = None
        lib.oracle_row_reduce.argtypes = [p, i32, p, p, p, p, p]
        lib.oracle_positions.restype = ctypes.c_int
        lib.oracle_positions.argtypes = [p, i64, i32, i64, p, i32, p, i64, p, p, p, p, p, p]
        lib.oracle_full_then_select.restype = i64
        lib.oracle_full_then_select.argtypes = [p, i64, i32, i64, p, i32, p, p, p, p, p, p, p]
        lib.oracle_unmask_topn.restype = i64
        lib.oracle_unmask_topn.argtypes = [p, p, p, i64, p, i32, p, p, p]
        lib.oracle_shift_indices.restype = None
        lib.oracle_shift_indices.argtypes = [p, i64, p, i32, p]
        lib.oracle_philox4x32_10.restype = None
        lib.oracle_philox4x32_10.argtypes = [p, p, p]
        lib.oracle_uniform.restype = ctypes.c_double
        lib.oracle_uniform.argtypes = [ctypes.c_uint64, i32, i32]
        lib.oracle_gumbel.restype = ctypes.c_double
        lib.oracle_gumbel.argtypes = [ctypes.c_uint64, i32, i32]
        lib.oracle_row_sample.restype = None
        lib.oracle_row_sample.argtypes = [p, i32, ctypes.c_double, ctypes.c_uint64, i32, p, p, p, p]
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_num_threads.argtypes = []
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _u16(a, name):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError(f"{name}: bf16 data must be passed as uint16 bit patterns, got {a.dtype}")
    return a


@dataclass
class RowResults:
    """Per-row oracle results, in the order of the rows asked for."""
    tok: np.ndarray      # int32  arg-max vocabulary id (lowest id on ties)
    conf: np.ndarray     # float32 soft-max probability of tok
    lse: np.ndarray      # float32 log-sum-exp of the row
    gap: np.ndarray      # float32 top-1 minus top-2 logit (0 on a repeated maximum)
    rowmax: np.ndarray   # float32 the maximum logit


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def mask_select(mask: np.ndarray) -> np.ndarray:
    """Ascending positions whose mask byte is nonzero (int32)."""
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    idx = np.empty(max(mask.size, 1), dtype=np.int32)
    m = _load().oracle_mask_select(_ptr(mask), mask.size, _ptr(idx))
    return idx[:m].copy()


def row_logits(h_row: np.ndarray, W: np.ndarray) -> np.ndarray:
    """All V fp32 logits of one hidden row (bf16 bits) against W[V,d] (bf16 bits)."""
    h_row, W = _u16(h_row, "h_row"), _u16(W, "W")
    V, d = W.shape
    assert h_row.shape == (d,)
    x = np.empty(V, dtype=np.float32)
    _load().oracle_row_logits(_ptr(h_row), _ptr(W), d, V, _ptr(x))
    return x


def row_logits_f32seq(h_row: np.ndarray, W: np.ndarray) -> np.ndarray:
    """The same logits by sequential fp32 accumulation (to measure the effect of accumulation order)."""
    h_row, W = _u16(h_row, "h_row"), _u16(W, "W")
    V, d = W.shape
    assert h_row.shape == (d,)
    x = np.empty(V, dtype=np.float32)
    _load().oracle_row_logits_f32seq(_ptr(h_row), _ptr(W), d, V, _ptr(x))
    return x


def row_reduce(x: np.ndarray):
    """(tok, conf, lse, gap, rowmax) of one row of fp32 logits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    tok = ctypes.c_int32()
    conf, lse, gap, mx = ctypes.c_float(), ctypes.c_float(), ctypes.c_float(), ctypes.c_float()
    _load().oracle_row_reduce(_ptr(x), x.size, ctypes.byref(tok), ctypes.byref(conf), ctypes.byref(lse),
                              ctypes.byref(gap), ctypes.byref(mx))
    return int(tok.value), float(conf.value), float(lse.value), float(gap.value), float(mx.value)


def positions(H: np.ndarray, W: np.ndarray, pos, return_logits: bool = False):
    """Oracle results at the listed positions of H[T,d] (restriction of the full computation)."""
    H, W = _u16(H, "H"), _u16(W, "W")
    T, d = H.shape
    V, d2 = W.shape
    assert d == d2
    pos = np.ascontiguousarray(pos, dtype=np.int64)
    n = pos.size
    res = RowResults(np.empty(n, np.int32), np.empty(n, np.float32), np.empty(n, np.float32),
                     np.empty(n, np.float32), np.empty(n, np.float32))
    logits = np.empty((n, V), np.float32) if return_logits else None
    rc = _load().oracle_positions(_ptr(H), T, d, d, _ptr(W), V, _ptr(pos), n, _ptr(res.tok), _ptr(res.conf),
                                  _ptr(res.lse), _ptr(res.gap), _ptr(res.rowmax),
                                  _ptr(logits) if return_logits else None)
    if rc != 0:
        raise ValueError("position out of range")
    return (res, logits) if return_logits else res


def full_then_select(H: np.ndarray, W: np.ndarray, mask: np.ndarray):
    """Results for every position, then the masked ones kept.  Returns (idx, RowResults)."""
    H, W = _u16(H, "H"), _u16(W, "W")
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    T, d = H.shape
    V, _ = W.shape
    assert mask.shape == (T,)
    cap = max(T, 1)
    idx = np.empty(cap, np.int32)
    res = RowResults(np.empty(cap, np.int32), np.empty(cap, np.float32), np.empty(cap, np.float32),
                     np.empty(cap, np.float32), np.empty(cap, np.float32))
    m = _load().oracle_full_then_select(_ptr(H), T, d, d, _ptr(W), V, _ptr(mask), _ptr(idx), _ptr(res.tok),
                                        _ptr(res.conf), _ptr(res.lse), _ptr(res.gap), _ptr(res.rowmax))
    out = RowResults(res.tok[:m].copy(), res.conf[:m].copy(), res.lse[:m].copy(), res.gap[:m].copy(),
                     res.rowmax[:m].copy())
    return idx[:m].copy(), out


def unmask_topn(conf, tok, idx, seq_starts, n_per_seq, tokens, mask):
    """Per sequence, the n highest-confidence masked rows (ties: lower position) get their token written
    into `tokens` and their mask byte cleared.  Returns (tokens, mask, number unmasked); inputs are copied."""
    conf = np.ascontiguousarray(conf, dtype=np.float32)
    tok = np.ascontiguousarray(tok, dtype=np.int32)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    seq_starts = np.ascontiguousarray(seq_starts, dtype=np.int32)
    n_per_seq = np.ascontiguousarray(n_per_seq, dtype=np.int32)
    tokens = np.array(tokens, dtype=np.int32, copy=True)
    mask = np.array(mask, dtype=np.uint8, copy=True)
    assert conf.size == tok.size == idx.size and seq_starts.size == n_per_seq.size + 1
    n = _load().oracle_unmask_topn(_ptr(conf), _ptr(tok), _ptr(idx), conf.size, _ptr(seq_starts), n_per_seq.size,
                                   _ptr(n_per_seq), _ptr(tokens), _ptr(mask))
    return tokens, mask, int(n)


def shift_indices(idx, seq_starts):
    """Hidden rows to read for Dream-style shifted prediction: idx - 1, except at sequence starts."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    seq_starts = np.ascontiguousarray(seq_starts, dtype=np.int32)
    out = np.empty(max(idx.size, 1), np.int32)
    _load().oracle_shift_indices(_ptr(idx), idx.size, _ptr(seq_starts), seq_starts.size - 1, _ptr(out))
    return out[:idx.size].copy()


def philox4x32_10(ctr, key):
    ctr = np.ascontiguousarray(ctr, dtype=np.uint32)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.empty(4, np.uint32)
    _load().oracle_philox4x32_10(_ptr(ctr), _ptr(key), _ptr(out))
    return out


def uniform(seed, position, v) -> float:
    return float(_load().oracle_uniform(seed, position, v))


def gumbel(seed, position, v) -> float:
    return float(_load().oracle_gumbel(seed, position, v))


def row_sample(x, tau, seed, position):
    """(tok, conf, lse, ygap) of one row of fp32 logits under Gumbel-max sampling with temperature tau."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    tok = ctypes.c_int32()
    conf, lse, gap = ctypes.c_float(), ctypes.c_float(), ctypes.c_float()
    _load().oracle_row_sample(_ptr(x), x.size, float(tau), int(seed), int(position), ctypes.byref(tok),
                              ctypes.byref(conf), ctypes.byref(lse), ctypes.byref(gap))
    return int(tok.value), float(conf.value), float(lse.value), float(gap.value)
