"""CPU oracle for pack -> ragged attention -> unpack (test infrastructure, NOT the product).

Thin ctypes wrapper over ``ragged_oracle.c`` (plain C, fp64 arithmetic).  Only ``tests/``,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import this package.
It imports nothing from the HIP package and the HIP package imports nothing from here.

All arrays are NumPy.  16-bit floating inputs travel as raw ``uint16`` words plus a dtype tag
("f16" or "bf16"), because NumPy has no bfloat16; the C code decodes them to double itself.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "ragged_oracle.c"
_LIB = _HERE / "libragged_oracle.so"
_DTYPES = {"f16": 0, "bf16": 1}

_lib = None


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math).  Rebuilds when the source is newer."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".tmp{os.getpid()}.so")
        subprocess.run(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
             "-o", str(tmp), str(_SRC), "-lm"],
            check=True,
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_LIB))
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        lib.oracle_decode.argtypes = [vp, i64, i32, vp]
        lib.oracle_decode.restype = None
        lib.oracle_pack.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp]
        lib.oracle_pack.restype = i64
        lib.oracle_unpack.argtypes = [vp, vp, vp, i32, i32, i32, vp, i32]
        lib.oracle_unpack.restype = None
        lib.oracle_attn.argtypes = [vp, vp, vp, i32, vp, i32, i32, i32, ctypes.c_float, vp, i32]
        lib.oracle_attn.restype = i32
        lib.oracle_attn_row.argtypes = [vp, vp, vp, i32, vp, i32, i32, i32, i32, i32,
                                        ctypes.c_float, vp, vp]
        lib.oracle_attn_row.restype = i32
        lib.oracle_attn_padded.argtypes = [vp, vp, vp, i32, vp, i32, i32, i32, i32, ctypes.c_float, vp]
        lib.oracle_attn_padded.restype = i32
        lib.oracle_repack.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp]
        lib.oracle_repack.restype = i64
        lib.oracle_cls_extract.argtypes = [vp, vp, i32, i32, vp]
        lib.oracle_cls_extract.restype = None
        lib.oracle_linear.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, i32]
        lib.oracle_linear.restype = i32
        lib.oracle_layernorm.argtypes = [vp, vp, vp, i32, i32, i32, ctypes.c_double, vp]
        lib.oracle_layernorm.restype = None
        lib.oracle_scores_l2.argtypes = [vp, i32, i64, i32, vp]
        lib.oracle_scores_l2.restype = None
        lib.oracle_keep_topk.argtypes = [vp, i32, i32, i32, vp]
        lib.oracle_keep_topk.restype = None
        lib.oracle_max_threads.argtypes = []
        lib.oracle_max_threads.restype = i32
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _words(a, shape_len=None) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype == np.int16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError(f"expected raw 16-bit words (uint16/int16/float16), got {a.dtype}")
    if shape_len is not None and a.ndim != shape_len:
        raise ValueError(f"expected {shape_len} dimensions, got shape {a.shape}")
    return a


def _mask(keep, B=None, N=None) -> np.ndarray:
    keep = np.ascontiguousarray(keep)
    if keep.dtype == np.bool_:
        keep = keep.view(np.uint8)
    if keep.dtype != np.uint8 or keep.ndim != 2:
        raise TypeError("keep must be a [B, N] uint8/bool array")
    if B is not None and keep.shape != (B, N):
        raise ValueError(f"keep shape {keep.shape} != {(B, N)}")
    return keep


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def decode(words, dtype: str) -> np.ndarray:
    """Raw 16-bit words -> float64, exactly."""
    w = _words(words)
    out = np.empty(w.shape, dtype=np.float64)
    _load().oracle_decode(_ptr(w), w.size, _DTYPES[dtype], _ptr(out))
    return out


def pack(x_words, keep):
    """x_words [B,N,C] words, keep [B,N] -> (packed [T,C] words, cu_seqlens [B+1] i32, gather_idx [T] i32)."""
    x = _words(x_words, 3)
    B, N, C = x.shape
    keep = _mask(keep, B, N)
    packed = np.zeros((B * N, C), dtype=np.uint16)
    cu = np.zeros(B + 1, dtype=np.int32)
    gidx = np.zeros(B * N, dtype=np.int32)
    T = int(_load().oracle_pack(_ptr(x), _ptr(keep), B, N, C, _ptr(packed), _ptr(cu), _ptr(gidx)))
    return packed[:T].copy(), cu, gidx[:T].copy()


def unpack(src_words, keep, cu_seqlens, C: int, fill_mode: int, out_init=None) -> np.ndarray:
    """src [T,C] words -> out [B,N,C] words.  fill_mode 0 keeps ``out_init`` on dropped rows."""
    src = _words(src_words, 2)
    keep = _mask(keep)
    B, N = keep.shape
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    if cu.shape != (B + 1,):
        raise ValueError("cu_seqlens must have B+1 entries")
    if src.shape != (int(cu[B]), C):
        raise ValueError(f"src shape {src.shape} != {(int(cu[B]), C)}")
    if fill_mode not in (0, 1):
        raise ValueError("fill_mode must be 0 or 1")
    if out_init is None:
        out = np.zeros((B, N, C), dtype=np.uint16)
    else:
        out = _words(out_init, 3).copy()
        if out.shape != (B, N, C):
            raise ValueError("out_init shape mismatch")
    _load().oracle_unpack(_ptr(src), _ptr(keep), _ptr(cu), B, N, C, _ptr(out), fill_mode)
    return out


def _check_qkv(q, k, v, cu):
    q, k, v = _words(q, 3), _words(k, 3), _words(v, 3)
    if not (q.shape == k.shape == v.shape):
        raise ValueError("q, k, v shapes differ")
    cu = np.ascontiguousarray(cu, dtype=np.int32)
    if cu.ndim != 1 or cu.size < 1 or cu[0] != 0 or np.any(np.diff(cu) < 0):
        raise ValueError("cu_seqlens must start at 0 and be non-decreasing")
    if int(cu[-1]) != q.shape[0]:
        raise ValueError(f"cu_seqlens[-1]={int(cu[-1])} but q has {q.shape[0]} rows")
    return q, k, v, cu


def attn(q, k, v, cu_seqlens, scale: float, dtype: str = "f16", threads: int = 1) -> np.ndarray:
    """softmax(scale * q k^T) v per image and head, fp64.  q,k,v [T,H,D] words -> [T,H,D] float64."""
    q, k, v, cu = _check_qkv(q, k, v, cu_seqlens)
    T, H, D = q.shape
    out = np.zeros((T, H, D), dtype=np.float64)
    rc = _load().oracle_attn(_ptr(q), _ptr(k), _ptr(v), _DTYPES[dtype], _ptr(cu), cu.size - 1,
                             H, D, float(scale), _ptr(out), int(threads))
    if rc != 0:
        raise MemoryError("oracle_attn failed to allocate scratch")
    return out


def attn_row(q, k, v, cu_seqlens, i: int, h: int, r: int, scale: float, dtype: str = "f16"):
    """(probabilities p_j/L over image i's keys, output row) for query r of image i, head h."""
    q, k, v, cu = _check_qkv(q, k, v, cu_seqlens)
    T, H, D = q.shape
    n = int(cu[i + 1] - cu[i])
    probs = np.zeros(n, dtype=np.float64)
    o = np.zeros(D, dtype=np.float64)
    rc = _load().oracle_attn_row(_ptr(q), _ptr(k), _ptr(v), _DTYPES[dtype], _ptr(cu), i, h, r,
                                 H, D, float(scale), _ptr(probs), _ptr(o))
    if rc != 0:
        raise IndexError("row out of range")
    return probs, o


def attn_padded(q, k, v, keep, scale: float, dtype: str = "f16") -> np.ndarray:
    """Attention on the padded layout: q,k,v [B,N,H,D] words, keep [B,N] -> [B,N,H,D] float64 with
    the kept tokens of each image attending among themselves and +0.0 rows for dropped tokens."""
    q, k, v = _words(q, 4), _words(k, 4), _words(v, 4)
    if not (q.shape == k.shape == v.shape):
        raise ValueError("q, k, v shapes differ")
    B, N, H, D = q.shape
    keep = _mask(keep, B, N)
    out = np.full((B, N, H, D), np.nan, dtype=np.float64)
    rc = _load().oracle_attn_padded(_ptr(q), _ptr(k), _ptr(v), _DTYPES[dtype], _ptr(keep), B, N, H, D,
                                    float(scale), _ptr(out))
    if rc != 0:
        raise MemoryError("oracle_attn_padded failed to allocate scratch")
    return out


def repack(packed_words, keep_rows, cu_seqlens):
    """packed [T,C] words, keep_rows [>=T] bytes, cu [B+1] -> (packed_out [T',C], cu_out [B+1], gather_out [T'])."""
    src = _words(packed_words, 2)
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    T, C = src.shape
    if int(cu[-1]) != T:
        raise ValueError("cu_seqlens[-1] must equal the number of packed rows")
    kr = np.ascontiguousarray(keep_rows)
    if kr.dtype == np.bool_:
        kr = kr.view(np.uint8)
    if kr.dtype != np.uint8 or kr.ndim != 1 or kr.size < T:
        raise TypeError("keep_rows must be a uint8/bool vector with at least T entries")
    out = np.zeros((max(T, 1), C), dtype=np.uint16)
    cu_out = np.zeros(cu.size, dtype=np.int32)
    gidx = np.zeros(max(T, 1), dtype=np.int32)
    T2 = int(_load().oracle_repack(_ptr(src), _ptr(kr), _ptr(cu), cu.size - 1, C, _ptr(out), _ptr(cu_out), _ptr(gidx)))
    return out[:T2].copy(), cu_out, gidx[:T2].copy()


def cls_extract(packed_words, cu_seqlens) -> np.ndarray:
    """First packed row of every image ([B,C] words; +0 for an image with no rows)."""
    src = _words(packed_words, 2)
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    out = np.full((cu.size - 1, src.shape[1]), 0xFFFF, dtype=np.uint16)
    _load().oracle_cls_extract(_ptr(src), _ptr(cu), cu.size - 1, src.shape[1], _ptr(out))
    return out


def linear(x, w, bias=None, residual=None, act: str = "none", dtype: str = "f16", threads: int = 1) -> np.ndarray:
    """act(x @ w.T + bias) + residual in fp64.  x [M,K], w [N,K], bias [N], residual [M,N] as raw words."""
    x, w = _words(x, 2), _words(w, 2)
    M, K = x.shape
    N = w.shape[0]
    if w.shape[1] != K:
        raise ValueError("w must be [N, K] with K = x.shape[1]")
    b = None if bias is None else _words(bias, 1)
    r = None if residual is None else _words(residual, 2)
    if b is not None and b.shape != (N,):
        raise ValueError("bias must have N entries")
    if r is not None and r.shape != (M, N):
        raise ValueError("residual must be [M, N]")
    y = np.zeros((M, N), dtype=np.float64)
    rc = _load().oracle_linear(_ptr(x), _ptr(w), None if b is None else _ptr(b), None if r is None else _ptr(r),
                               _DTYPES[dtype], M, N, K, {"none": 0, "gelu": 1}[act], _ptr(y), int(threads))
    if rc != 0:
        raise MemoryError("oracle_linear failed to allocate scratch")
    return y


def layernorm(x, gamma, beta, eps: float, dtype: str = "f16") -> np.ndarray:
    """Row-wise LayerNorm in fp64 (biased variance).  x [M,C], gamma/beta [C] as raw words."""
    x = _words(x, 2)
    M, C = x.shape
    g, b = _words(gamma, 1), _words(beta, 1)
    if g.shape != (C,) or b.shape != (C,):
        raise ValueError("gamma and beta must have C entries")
    y = np.zeros((M, C), dtype=np.float64)
    _load().oracle_layernorm(_ptr(x), _ptr(g), _ptr(b), _DTYPES[dtype], M, C, float(eps), _ptr(y))
    return y


def scores_l2(x_words, dtype: str = "f16") -> np.ndarray:
    """Squared l2 norm of every token row: x [B,N,C] words -> [B,N] float64."""
    x = _words(x_words, 3)
    B, N, C = x.shape
    out = np.zeros((B, N), dtype=np.float64)
    _load().oracle_scores_l2(_ptr(x), _DTYPES[dtype], B * N, C, _ptr(out))
    return out


def keep_topk(scores, k: int) -> np.ndarray:
    """Per image: token 0 plus the k-1 highest-scoring other tokens (ties: lower position first) -> [B,N] uint8."""
    s = np.ascontiguousarray(scores, dtype=np.float64)
    if s.ndim != 2 or k < 1:
        raise ValueError("scores must be [B, N] and k >= 1")
    B, N = s.shape
    keep = np.zeros((B, N), dtype=np.uint8)
    _load().oracle_keep_topk(_ptr(s), B, N, int(k), _ptr(keep))
    return keep
