"""Thin ctypes binding of libcastling_attn.so (include/castling_attn.h).

Argument marshalling only: every step of the layer runs in the HIP kernels.
Tensors are torch tensors on the GPU, used here for device memory and streams.
If the shared library has not been built this module raises: there is no
fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libcastling_attn.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_HIP, ERR_ALIAS, ERR_TOO_LARGE = 0, 1, 2, 3, 4, 5
STATIC_SCRATCH_BYTES = 32 << 20
F32, BF16, F16 = 0, 1, 2
NORM_ROWSUM, NORM_NONE = 0, 1
BRANCH_LINEAR, BRANCH_DWCONV, BRANCH_ALL = 1, 2, 3
FLAG_KEEP_STATE = 1
FLAG_RESIDUAL_Q = 2
FLAG_TRAINING = 4
FLAG_SEPARATE_PASSES = 8
FLAG_VECTOR_ALU = 16

EXPORTS = (
    "castling_attn_validate", "castling_attn_create", "castling_attn_forward",
    "castling_attn_reduce", "castling_attn_apply", "castling_attn_prepare_weights",
    "castling_attn_destroy",
    "castling_attn_workspace_bytes", "castling_attn_get_state", "castling_attn_num_splits",
    "castling_attn_num_launches", "castling_attn_pairwise", "castling_attn_backward",
    "castling_attn_strerror", "castling_attn_forward_static",
)


class Desc(C.Structure):
    _fields_ = [("B", C.c_int32), ("heads", C.c_int32), ("N", C.c_int32), ("d", C.c_int32),
                ("grid_h", C.c_int32), ("grid_w", C.c_int32), ("dw_kernel", C.c_int32),
                ("io_dtype", C.c_int32), ("norm", C.c_int32), ("branches", C.c_uint32),
                ("eps", C.c_float),
                ("in_stride_b", C.c_int64), ("in_stride_h", C.c_int64), ("in_stride_n", C.c_int64),
                ("out_stride_b", C.c_int64), ("out_stride_h", C.c_int64),
                ("out_stride_n", C.c_int64), ("flags", C.c_uint32), ("extra_tokens", C.c_int32),
                ("q_pool", C.c_int32), ("reserved0", C.c_int32),
                ("q_stride_b", C.c_int64), ("q_stride_h", C.c_int64), ("q_stride_n", C.c_int64)]


PAIR_SPARSE_SOFTMAX, PAIR_ANGULAR = 0, 1


class PairParams(C.Structure):
    _fields_ = [("mode", C.c_int32), ("normalize", C.c_int32), ("scale", C.c_float),
                ("threshold", C.c_float), ("accumulate", C.c_int32)]


class CastlingError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"castling_attn status {status}: {msg}")
        self.status = status


_lib = None


def lib():
    """Loads the built library; raises if it is missing (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is not built; run `python -m paper_2211_10526_amd.build` "
                "(needs hipcc). The layer has no other implementation.")
        # torch ships its own HIP runtime; load it first so that this library binds to
        # the same runtime instance that owns torch's device memory and streams
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp = C.c_void_p
        L.castling_attn_validate.argtypes = [C.POINTER(Desc)]
        L.castling_attn_create.argtypes = [C.POINTER(Desc), C.POINTER(vp)]
        L.castling_attn_forward.argtypes = [vp] * 8
        L.castling_attn_forward_static.argtypes = [C.POINTER(Desc)] + [vp] * 7
        L.castling_attn_reduce.argtypes = [vp] * 4
        L.castling_attn_apply.argtypes = [vp] * 7
        L.castling_attn_prepare_weights.argtypes = [vp] * 3
        L.castling_attn_destroy.argtypes = [vp]
        L.castling_attn_workspace_bytes.argtypes = [vp]
        L.castling_attn_workspace_bytes.restype = C.c_size_t
        L.castling_attn_get_state.argtypes = [vp, vp, C.c_size_t, vp]
        L.castling_attn_num_splits.argtypes = [vp]
        L.castling_attn_num_launches.argtypes = [vp]
        L.castling_attn_pairwise.argtypes = [vp, C.POINTER(PairParams)] + [vp] * 6
        L.castling_attn_backward.argtypes = [vp] * 12
        L.castling_attn_strerror.argtypes = [C.c_int]
        L.castling_attn_strerror.restype = C.c_char_p
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().castling_attn_strerror(int(status)).decode()


def _check(status: int):
    if status != OK:
        raise CastlingError(status, strerror(status))


def fused_qkv_strides(heads, N, d):
    """(batch, head, token) element strides of q, k, v taken as the slices [:, :, i] of a
    fused projection output [B][N][3][heads][d]."""
    return (N * 3 * heads * d, d, 3 * heads * d)


def token_major_strides(heads, N, d):
    """(batch, head, token) element strides of a [B][N][heads * d] tensor."""
    return (N * heads * d, d, heads * d)


def make_desc(B, heads, N, d, grid_h, grid_w, dw_kernel, io_dtype, norm=NORM_ROWSUM,
              branches=BRANCH_ALL, eps=0.0, in_strides=None, out_strides=None, flags=0,
              extra_tokens=0, q_pool=0, q_strides=None) -> Desc:
    """in_strides / out_strides: (batch, head, token) element strides of q, k, v and of out;
    None = contiguous [B][heads][N][d].  q_pool = 2: q and out hold the pooled queries of a
    downsampling layer (q_strides: their strides, None = contiguous)."""
    if isinstance(io_dtype, str):
        io_dtype = {"f32": F32, "bf16": BF16, "f16": F16}[io_dtype]
    ins = tuple(in_strides) if in_strides is not None else (0, 0, 0)
    outs = tuple(out_strides) if out_strides is not None else (0, 0, 0)
    qs = tuple(q_strides) if q_strides is not None else (0, 0, 0)
    return Desc(B, heads, N, d, grid_h, grid_w, dw_kernel, io_dtype, norm, branches, eps,
                *ins, *outs, flags, extra_tokens, q_pool, 0, *qs)


def validate(desc: Desc) -> int:
    """castling_attn_validate: returns the status code (host only)."""
    return lib().castling_attn_validate(C.byref(desc))


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def forward_static(desc: Desc, q, k, v, w, bias, out, stream=None):
    """castling_attn_forward_static: the forward without a handle or device allocation."""
    _check(lib().castling_attn_forward_static(C.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(w),
                                              _ptr(bias), _ptr(out), _stream_ptr(stream)))
    return out


class CastlingAttn:
    """castling_attn_create / forward / reduce / apply / destroy on one handle."""

    def __init__(self, desc: Desc):
        self.desc = desc
        self._h = C.c_void_p()
        _check(lib().castling_attn_create(C.byref(desc), C.byref(self._h)))

    @classmethod
    def for_workload(cls, wl, norm=NORM_ROWSUM, branches=BRANCH_ALL, eps=0.0, in_strides=None,
                     out_strides=None, flags=0, extra_tokens=0):
        return cls(make_desc(wl.B, wl.heads, wl.N + extra_tokens, wl.d, wl.grid_h, wl.grid_w,
                             wl.dw_kernel, wl.dtype, norm, branches, eps, in_strides, out_strides,
                             flags, extra_tokens))

    def forward(self, q, k, v, w, bias, out, stream=None):
        _check(lib().castling_attn_forward(self._h, _ptr(q), _ptr(k), _ptr(v), _ptr(w),
                                           _ptr(bias), _ptr(out), _stream_ptr(stream)))
        return out

    def reduce(self, k, v, stream=None):
        _check(lib().castling_attn_reduce(self._h, _ptr(k), _ptr(v), _stream_ptr(stream)))

    def apply(self, q, v, w, bias, out, stream=None):
        _check(lib().castling_attn_apply(self._h, _ptr(q), _ptr(v), _ptr(w), _ptr(bias),
                                         _ptr(out), _stream_ptr(stream)))
        return out

    def backward(self, q, k, v, w, grad_out, grad_q, grad_k, grad_v, grad_w, grad_bias=None,
                 stream=None):
        """castling_attn_backward; grad_w / grad_bias: fp32 device tensors."""
        _check(lib().castling_attn_backward(self._h, _ptr(q), _ptr(k), _ptr(v), _ptr(w),
                                            _ptr(grad_out), _ptr(grad_q), _ptr(grad_k), _ptr(grad_v),
                                            _ptr(grad_w), _ptr(grad_bias), _stream_ptr(stream)))

    def pairwise(self, mode, q, k, v, out, kept=None, normalize=True, scale=1.0, threshold=0.0,
                 accumulate=False, stream=None):
        """castling_attn_pairwise; kept: int64 / uint64 device tensor [B * heads] or None."""
        params = PairParams(mode, int(bool(normalize)), scale, threshold, int(bool(accumulate)))
        _check(lib().castling_attn_pairwise(self._h, C.byref(params), _ptr(q), _ptr(k), _ptr(v),
                                            _ptr(out), _ptr(kept), _stream_ptr(stream)))
        return out

    def prepare_weights(self, w, stream=None):
        _check(lib().castling_attn_prepare_weights(self._h, _ptr(w), _stream_ptr(stream)))

    def workspace_bytes(self) -> int:
        return lib().castling_attn_workspace_bytes(self._h)

    def num_splits(self) -> int:
        return lib().castling_attn_num_splits(self._h)

    def num_launches(self) -> int:
        return lib().castling_attn_num_launches(self._h)

    def get_state(self, stream=None) -> np.ndarray:
        d = self.desc
        st = np.empty((d.B, d.heads, d.d + 1, d.d + 1), dtype=np.float32)
        _check(lib().castling_attn_get_state(self._h, C.c_void_p(st.ctypes.data), st.nbytes,
                                             _stream_ptr(stream)))
        return st

    def destroy(self):
        if self._h:
            _check(lib().castling_attn_destroy(self._h))
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
