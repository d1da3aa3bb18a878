"""ctypes binding of the C ABI in ``include/ragged.h`` (argument marshalling only).

Every function takes torch tensors that already live on the GPU, checks shapes/dtypes/contiguity,
passes raw device pointers and the current HIP stream to the library and returns at once; all
computation happens in the HIP kernels.  There is no CPU fallback: if the shared library has not
been built, loading raises.
"""
from __future__ import annotations

import ctypes
from pathlib import Path

import torch

_PKG = Path(__file__).resolve().parent
LIB_PATH = _PKG / "libragged_hip.so"

RAGGED_OK = 0
RAGGED_F16, RAGGED_BF16, RAGGED_F32 = 0, 1, 2
_DTYPE_CODE = {torch.float16: RAGGED_F16, torch.bfloat16: RAGGED_BF16, torch.float32: RAGGED_F32}

EXPORTS = ("ragged_pack", "ragged_attn", "ragged_attn_strided", "ragged_attn_checked", "ragged_attn_padded", "ragged_unpack",
           "ragged_repack", "ragged_cls_extract", "ragged_pack_attn_unpack", "ragged_linear", "ragged_layernorm",
           "ragged_token_scores_l2", "ragged_keep_topk", "ragged_noop", "ragged_status_string", "ragged_version")

_lib = None


class RaggedError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__(f"{fn} failed with status {status}: {status_string(status)}")


def load() -> ctypes.CDLL:
    """Open the in-tree shared library (built by ``paper_2604_15408_amd.build``)."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2604_15408_amd.build` "
                "(there is no fallback implementation)")
        lib = ctypes.CDLL(str(LIB_PATH))
        vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_float
        lib.ragged_pack.argtypes = [vp, vp, i32, i32, i32, i32, vp, i64, vp, vp, vp]
        lib.ragged_pack.restype = i32
        lib.ragged_attn.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, f32, i32, i32, vp]
        lib.ragged_attn.restype = i32
        lib.ragged_attn_strided.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i64, i64, f32, i32, i32, vp]
        lib.ragged_attn_strided.restype = i32
        lib.ragged_attn_checked.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i64, i64, f32, i32, i32, vp, vp]
        lib.ragged_attn_checked.restype = i32
        lib.ragged_repack.argtypes = [vp, vp, vp, i32, i64, i32, i32, vp, i64, vp, vp, vp]
        lib.ragged_repack.restype = i32
        lib.ragged_cls_extract.argtypes = [vp, vp, i32, i32, i32, vp, vp]
        lib.ragged_cls_extract.restype = i32
        lib.ragged_pack_attn_unpack.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, f32, i32, vp, i64, vp, vp,
                                                vp, vp, i32, vp]
        lib.ragged_pack_attn_unpack.restype = i32
        lib.ragged_linear.argtypes = [vp, vp, vp, vp, vp, i64, vp, i64, i32, i32, i32, i32, vp]
        lib.ragged_linear.restype = i32
        lib.ragged_layernorm.argtypes = [vp, vp, vp, vp, i64, vp, i32, f32, i32, vp]
        lib.ragged_layernorm.restype = i32
        lib.ragged_token_scores_l2.argtypes = [vp, i64, i32, i32, vp, vp]
        lib.ragged_token_scores_l2.restype = i32
        lib.ragged_keep_topk.argtypes = [vp, i32, i32, i32, vp, vp]
        lib.ragged_keep_topk.restype = i32
        lib.ragged_attn_padded.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, f32, i32, i32, i32, vp]
        lib.ragged_attn_padded.restype = i32
        lib.ragged_unpack.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, vp, i32, vp]
        lib.ragged_unpack.restype = i32
        lib.ragged_noop.argtypes = [i32, vp]
        lib.ragged_noop.restype = i32
        lib.ragged_status_string.argtypes = [i32]
        lib.ragged_status_string.restype = ctypes.c_char_p
        lib.ragged_version.argtypes = []
        lib.ragged_version.restype = i32
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().ragged_status_string(int(status)).decode()


def version() -> int:
    return int(load().ragged_version())


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _dev(t: torch.Tensor, name: str, dtype=None, shape=None) -> int:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a GPU tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype not in (dtype if isinstance(dtype, tuple) else (dtype,)):
        raise TypeError(f"{name} has dtype {t.dtype}, expected {dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    return t.data_ptr()


def _check(fn: str, status: int) -> None:
    if status != RAGGED_OK:
        raise RaggedError(fn, status)


def _pack_args(x, keep, packed, cu_seqlens, gather_idx, stream):
    B, N, C = x.shape
    cap = packed.shape[0]
    return (_dev(x, "x", (torch.float16, torch.bfloat16)),
            _dev(keep, "keep", (torch.uint8, torch.bool), (B, N)), B, N, C, _DTYPE_CODE[x.dtype],
            _dev(packed, "packed", x.dtype, (cap, C)), cap,
            _dev(cu_seqlens, "cu_seqlens", torch.int32, (B + 1,)),
            _dev(gather_idx, "gather_idx", torch.int32, (cap,)), _stream(stream))


def ragged_pack(x, keep, packed, cu_seqlens, gather_idx, stream=None) -> None:
    """x [B,N,C] f16/bf16, keep [B,N] uint8/bool -> packed [cap,C], cu_seqlens [B+1] i32,
    gather_idx [cap] i32 (all caller-allocated; cap = packed.shape[0])."""
    _check("ragged_pack", load().ragged_pack(*_pack_args(x, keep, packed, cu_seqlens, gather_idx, stream)))


def _attn_args(q, k, v, o, cu_seqlens, max_seqlen, scale, stream):
    rows, H, D = q.shape
    B = cu_seqlens.shape[0] - 1
    return (_dev(q, "q", (torch.float16, torch.bfloat16)), _dev(k, "k", q.dtype, q.shape),
            _dev(v, "v", q.dtype, q.shape), _dev(o, "o", (q.dtype, torch.float32), q.shape),
            _dev(cu_seqlens, "cu_seqlens", torch.int32), B, int(max_seqlen), H, D, float(scale),
            _DTYPE_CODE[q.dtype], _DTYPE_CODE[o.dtype], _stream(stream))


def ragged_attn(q, k, v, o, cu_seqlens, max_seqlen: int, scale: float, stream=None) -> None:
    """q,k,v [rows,H,D] f16/bf16 and o [rows,H,D] (same dtype or f32); only rows < cu_seqlens[-1]
    are read / written."""
    _check("ragged_attn", load().ragged_attn(*_attn_args(q, k, v, o, cu_seqlens, max_seqlen, scale, stream)))


def _token_rows(t: torch.Tensor, name: str, dtype, shape):
    """(pointer, token stride) of a [rows, H, D] view whose tokens are a constant number of elements
    apart and whose [H, D] block is contiguous inside a token (e.g. ``qkv[:, 0]`` of [rows, 3, H, D])."""
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a GPU tensor")
    if t.dtype not in (dtype if isinstance(dtype, tuple) else (dtype,)):
        raise TypeError(f"{name} has dtype {t.dtype}, expected {dtype}")
    if t.dim() != 3 or (shape is not None and tuple(t.shape) != tuple(shape)):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected [rows, H, D]")
    rows, H, D = t.shape
    if t.stride(2) != 1 or t.stride(1) != D:
        raise ValueError(f"{name}: the [H, D] block of a token must be contiguous")
    return t.data_ptr(), (t.stride(0) if rows > 1 else max(t.stride(0), H * D))


def _attn_strided_args(q, k, v, o, cu_seqlens, max_seqlen, scale, stream):
    rows, H, D = q.shape
    B = cu_seqlens.shape[0] - 1
    (qp, qs), (kp, ks), (vp, vs) = (_token_rows(t, n, (torch.float16, torch.bfloat16), q.shape)
                                    for t, n in ((q, "q"), (k, "k"), (v, "v")))
    if not (k.dtype == v.dtype == q.dtype) or not (qs == ks == vs):
        raise ValueError("q, k, v must share dtype and token stride")
    op, os_ = _token_rows(o, "o", (q.dtype, torch.float32), q.shape)
    return (qp, kp, vp, op, _dev(cu_seqlens, "cu_seqlens", torch.int32), B, int(max_seqlen), H, D,
            int(qs), int(os_), float(scale), _DTYPE_CODE[q.dtype], _DTYPE_CODE[o.dtype], _stream(stream))


def ragged_attn_strided(q, k, v, o, cu_seqlens, max_seqlen: int, scale: float, stream=None) -> None:
    """ragged_attn on [rows,H,D] views with a token stride, e.g. the three slices of a fused
    [rows,3,H,D] QKV buffer; o may be a strided view too."""
    _check("ragged_attn_strided",
           load().ragged_attn_strided(*_attn_strided_args(q, k, v, o, cu_seqlens, max_seqlen, scale, stream)))


FLAG_SEQLEN_EXCEEDED = 1


def ragged_attn_checked(q, k, v, o, cu_seqlens, max_seqlen: int, scale: float, flags, stream=None) -> None:
    """ragged_attn_strided that ORs FLAG_SEQLEN_EXCEEDED into flags[0] (int32 GPU tensor, zeroed by the caller)
    when some image holds more than max_seqlen tokens."""
    args = _attn_strided_args(q, k, v, o, cu_seqlens, max_seqlen, scale, stream)
    _check("ragged_attn_checked", load().ragged_attn_checked(*args[:-1], _dev(flags, "flags", torch.int32), args[-1]))


def _repack_args(packed_in, keep_rows, cu_in, packed_out, cu_out, gather_out, stream):
    cap_in, C = packed_in.shape
    cap_out = packed_out.shape[0]
    B = cu_in.shape[0] - 1
    return (_dev(packed_in, "packed_in", (torch.float16, torch.bfloat16)),
            _dev(keep_rows, "keep_rows", (torch.uint8, torch.bool), (cap_in,)),
            _dev(cu_in, "cu_in", torch.int32), B, cap_in, C, _DTYPE_CODE[packed_in.dtype],
            _dev(packed_out, "packed_out", packed_in.dtype, (cap_out, C)), cap_out,
            _dev(cu_out, "cu_out", torch.int32, (B + 1,)),
            _dev(gather_out, "gather_out", torch.int32, (cap_out,)), _stream(stream))


def ragged_repack(packed_in, keep_rows, cu_in, packed_out, cu_out, gather_out, stream=None) -> None:
    """packed_in [cap_in,C], keep_rows [cap_in], cu_in [B+1] -> packed_out [cap_out,C], cu_out [B+1],
    gather_out [cap_out]: a second keep decision on packed rows."""
    _check("ragged_repack",
           load().ragged_repack(*_repack_args(packed_in, keep_rows, cu_in, packed_out, cu_out, gather_out, stream)))


def _cls_args(packed, cu_seqlens, out, stream):
    B = cu_seqlens.shape[0] - 1
    C = packed.shape[1]
    return (_dev(packed, "packed", (torch.float16, torch.bfloat16)),
            _dev(cu_seqlens, "cu_seqlens", torch.int32), B, C, _DTYPE_CODE[packed.dtype],
            _dev(out, "out", packed.dtype, (B, C)), _stream(stream))


def ragged_cls_extract(packed, cu_seqlens, out, stream=None) -> None:
    """out[i] = packed[cu_seqlens[i]] (first kept row of image i; zeros if the image has none)."""
    _check("ragged_cls_extract", load().ragged_cls_extract(*_cls_args(packed, cu_seqlens, out, stream)))


def _attn_padded_args(q, k, v, o, keep, scale, fill_mode, stream):
    B, N, H, D = q.shape
    return (_dev(q, "q", (torch.float16, torch.bfloat16)), _dev(k, "k", q.dtype, q.shape),
            _dev(v, "v", q.dtype, q.shape), _dev(o, "o", (q.dtype, torch.float32), q.shape),
            _dev(keep, "keep", (torch.uint8, torch.bool), (B, N)), B, N, H, D, float(scale),
            _DTYPE_CODE[q.dtype], _DTYPE_CODE[o.dtype], int(fill_mode), _stream(stream))


def ragged_attn_padded(q, k, v, o, keep, scale: float, fill_mode: int = 0, stream=None) -> None:
    """q,k,v,o [B,N,H,D], keep [B,N]: pack + attention + unpack of one layer in a single launch."""
    _check("ragged_attn_padded",
           load().ragged_attn_padded(*_attn_padded_args(q, k, v, o, keep, scale, fill_mode, stream)))


def _step_args(x, keep, q, k, v, packed, cu_seqlens, gather_idx, o, out, scale, fill_mode, stream):
    B, N, C = x.shape
    cap, H, D = q.shape
    return (_dev(x, "x", (torch.float16, torch.bfloat16)), _dev(keep, "keep", (torch.uint8, torch.bool), (B, N)),
            _dev(q, "q", x.dtype), _dev(k, "k", x.dtype, q.shape), _dev(v, "v", x.dtype, q.shape),
            B, N, H, D, float(scale), _DTYPE_CODE[x.dtype], _dev(packed, "packed", x.dtype, (cap, C)), cap,
            _dev(cu_seqlens, "cu_seqlens", torch.int32, (B + 1,)),
            _dev(gather_idx, "gather_idx", torch.int32, (cap,)), _dev(o, "o", x.dtype, q.shape),
            _dev(out, "out", x.dtype, (B, N, C)), int(fill_mode), _stream(stream))


def ragged_pack_attn_unpack(x, keep, q, k, v, packed, cu_seqlens, gather_idx, o, out, scale: float,
                            fill_mode: int = 0, stream=None) -> None:
    """ragged_pack(x, keep) + ragged_attn(q, k, v) + ragged_unpack(o -> out) in one launch; q, k, v,
    o, packed, gather_idx hold cap >= B*N rows."""
    _check("ragged_pack_attn_unpack", load().ragged_pack_attn_unpack(
        *_step_args(x, keep, q, k, v, packed, cu_seqlens, gather_idx, o, out, scale, fill_mode, stream)))


def prepare_pack_attn_unpack(x, keep, q, k, v, packed, cu_seqlens, gather_idx, o, out, scale: float,
                             fill_mode: int = 0, stream=None) -> "Prepared":
    return Prepared("ragged_pack_attn_unpack", load().ragged_pack_attn_unpack,
                    _step_args(x, keep, q, k, v, packed, cu_seqlens, gather_idx, o, out, scale, fill_mode, stream),
                    (x, keep, q, k, v, packed, cu_seqlens, gather_idx, o, out))


def _rows_dev(rows_dev):
    """Device pointer to an int32 row count: a 1-element int32 GPU tensor (e.g. cu_seqlens[B:]) or None."""
    if rows_dev is None:
        return None
    if not (isinstance(rows_dev, torch.Tensor) and rows_dev.is_cuda and rows_dev.dtype == torch.int32
            and rows_dev.numel() >= 1):
        raise TypeError("rows_dev must be an int32 GPU tensor with at least one element")
    return rows_dev.data_ptr()


def _linear_args(x, w, bias, residual, y, rows_dev, act, stream, rows_hint=0):
    rows, K = x.shape
    N = w.shape[0]
    return (_dev(x, "x", (torch.float16, torch.bfloat16)), _dev(w, "w", x.dtype, (N, K)),
            None if bias is None else _dev(bias, "bias", x.dtype, (N,)),
            None if residual is None else _dev(residual, "residual", x.dtype, (rows, N)),
            _dev(y, "y", x.dtype, (rows, N)), rows, _rows_dev(rows_dev), int(rows_hint), N, K, {"none": 0, "gelu": 1}[act],
            _DTYPE_CODE[x.dtype], _stream(stream))


def ragged_linear(x, w, bias, residual, y, rows_dev=None, act: str = "none", stream=None, rows_hint: int = 0) -> None:
    """y = act(x @ w.T + bias) + residual over the first min(rows, *rows_dev) rows.  x [rows,K], w [N,K].
    rows_hint: an estimate of *rows_dev known on the host (0 = rows); it only picks the launch shape."""
    _check("ragged_linear",
           load().ragged_linear(*_linear_args(x, w, bias, residual, y, rows_dev, act, stream, rows_hint)))


def prepare_linear(x, w, bias, residual, y, rows_dev=None, act: str = "none", stream=None,
                   rows_hint: int = 0) -> "Prepared":
    return Prepared("ragged_linear", load().ragged_linear,
                    _linear_args(x, w, bias, residual, y, rows_dev, act, stream, rows_hint),
                    (x, w, bias, residual, y, rows_dev))


def _layernorm_args(x, gamma, beta, y, rows_dev, eps, stream):
    rows, C = x.shape
    return (_dev(x, "x", (torch.float16, torch.bfloat16)), _dev(gamma, "gamma", x.dtype, (C,)),
            _dev(beta, "beta", x.dtype, (C,)), _dev(y, "y", x.dtype, (rows, C)), rows, _rows_dev(rows_dev), C,
            float(eps), _DTYPE_CODE[x.dtype], _stream(stream))


def ragged_layernorm(x, gamma, beta, y, rows_dev=None, eps: float = 1e-6, stream=None) -> None:
    """Row-wise LayerNorm of x [rows,C] into y over the first min(rows, *rows_dev) rows."""
    _check("ragged_layernorm", load().ragged_layernorm(*_layernorm_args(x, gamma, beta, y, rows_dev, eps, stream)))


def prepare_layernorm(x, gamma, beta, y, rows_dev=None, eps: float = 1e-6, stream=None) -> "Prepared":
    return Prepared("ragged_layernorm", load().ragged_layernorm, _layernorm_args(x, gamma, beta, y, rows_dev, eps, stream),
                    (x, gamma, beta, y, rows_dev))


def ragged_token_scores_l2(x, scores, stream=None) -> None:
    """scores[b, t] = squared l2 norm of x[b, t, :] (fp64).  x [B,N,C] f16/bf16, scores [B,N] float64."""
    B, N, C = x.shape
    _check("ragged_token_scores_l2", load().ragged_token_scores_l2(
        _dev(x, "x", (torch.float16, torch.bfloat16)), B * N, C, _DTYPE_CODE[x.dtype],
        _dev(scores, "scores", torch.float64, (B, N)), _stream(stream)))


def ragged_keep_topk(scores, k: int, keep, stream=None) -> None:
    """keep[b] = token 0 plus the k-1 highest-scoring other tokens of image b (ties: lower position)."""
    B, N = scores.shape
    _check("ragged_keep_topk", load().ragged_keep_topk(
        _dev(scores, "scores", torch.float64), B, N, int(k), _dev(keep, "keep", (torch.uint8, torch.bool), (B, N)),
        _stream(stream)))


def _unpack_args(src, keep, cu_seqlens, gather_idx, out, fill_mode, stream):
    B, N, C = out.shape
    return (_dev(src, "src", (torch.float16, torch.bfloat16)),
            None if keep is None else _dev(keep, "keep", (torch.uint8, torch.bool), (B, N)),
            _dev(cu_seqlens, "cu_seqlens", torch.int32, (B + 1,)),
            None if gather_idx is None else _dev(gather_idx, "gather_idx", torch.int32),
            B, N, C, _DTYPE_CODE[src.dtype], _dev(out, "out", src.dtype), int(fill_mode), _stream(stream))


def ragged_unpack(src, keep, cu_seqlens, gather_idx, out, fill_mode: int, stream=None) -> None:
    """src [rows,C] -> out [B,N,C].  fill_mode 0 needs gather_idx (keep may be None); fill_mode 1
    needs keep (gather_idx may be None)."""
    _check("ragged_unpack",
           load().ragged_unpack(*_unpack_args(src, keep, cu_seqlens, gather_idx, out, fill_mode, stream)))


_UNTYPED = None


def _untyped() -> ctypes.CDLL:
    """A second handle of the library whose functions carry no argument types (see Prepared)."""
    global _UNTYPED
    if _UNTYPED is None:
        load()
        _UNTYPED = ctypes.CDLL(str(LIB_PATH))
    return _UNTYPED


class Prepared:
    """A call with its arguments marshalled once: ``prepared()`` re-issues the same launch on the
    stream it was prepared for, skipping the per-call tensor checks (serving loops re-launch the same
    buffers every step, and at ViT sizes the host-side dispatch cost is what the caller sees).
    The tensors must stay alive and in place for as long as the object is used."""

    __slots__ = ("_fn", "_args", "_name", "_keepalive")

    def __init__(self, name, fn, args, keepalive):
        # The arguments are converted to C values once, with the checked function's own argument types,
        # and the call goes through an untyped handle of the same symbol: ctypes then has nothing left
        # to convert per call (1.0 instead of 1.7 us of host time for the 19 arguments of a step).
        self._name, self._keepalive = name, keepalive
        self._args = tuple(t(a) for t, a in zip(fn.argtypes, args))
        self._fn = getattr(_untyped(), name)
        self._fn.restype = ctypes.c_int

    def __call__(self) -> None:
        st = self._fn(*self._args)
        if st != RAGGED_OK:
            raise RaggedError(self._name, st)


def prepare_pack(x, keep, packed, cu_seqlens, gather_idx, stream=None) -> Prepared:
    return Prepared("ragged_pack", load().ragged_pack, _pack_args(x, keep, packed, cu_seqlens, gather_idx, stream),
                    (x, keep, packed, cu_seqlens, gather_idx))


def prepare_attn(q, k, v, o, cu_seqlens, max_seqlen: int, scale: float, stream=None) -> Prepared:
    return Prepared("ragged_attn", load().ragged_attn, _attn_args(q, k, v, o, cu_seqlens, max_seqlen, scale, stream),
                    (q, k, v, o, cu_seqlens))


def prepare_attn_strided(q, k, v, o, cu_seqlens, max_seqlen: int, scale: float, stream=None) -> Prepared:
    return Prepared("ragged_attn_strided", load().ragged_attn_strided,
                    _attn_strided_args(q, k, v, o, cu_seqlens, max_seqlen, scale, stream), (q, k, v, o, cu_seqlens))


def prepare_repack(packed_in, keep_rows, cu_in, packed_out, cu_out, gather_out, stream=None) -> Prepared:
    return Prepared("ragged_repack", load().ragged_repack,
                    _repack_args(packed_in, keep_rows, cu_in, packed_out, cu_out, gather_out, stream),
                    (packed_in, keep_rows, cu_in, packed_out, cu_out, gather_out))


def prepare_cls_extract(packed, cu_seqlens, out, stream=None) -> Prepared:
    return Prepared("ragged_cls_extract", load().ragged_cls_extract, _cls_args(packed, cu_seqlens, out, stream),
                    (packed, cu_seqlens, out))


def prepare_attn_padded(q, k, v, o, keep, scale: float, fill_mode: int = 0, stream=None) -> Prepared:
    return Prepared("ragged_attn_padded", load().ragged_attn_padded,
                    _attn_padded_args(q, k, v, o, keep, scale, fill_mode, stream), (q, k, v, o, keep))


def prepare_unpack(src, keep, cu_seqlens, gather_idx, out, fill_mode: int, stream=None) -> Prepared:
    return Prepared("ragged_unpack", load().ragged_unpack,
                    _unpack_args(src, keep, cu_seqlens, gather_idx, out, fill_mode, stream),
                    (src, keep, cu_seqlens, gather_idx, out))


def ragged_noop(grid: int, stream=None) -> None:
    _check("ragged_noop", load().ragged_noop(int(grid), _stream(stream)))
