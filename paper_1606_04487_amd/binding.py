"""ctypes binding over libomniconv.so -- argument marshalling only.

Every function here has the name of the C entry point it calls (minus the `omni_` prefix),
takes torch tensors that live on the GPU, passes their `data_ptr()` and the current torch
stream to the library, and raises `OmniError` on a non-zero status.  torch is used for device
memory and streams; no arithmetic of the method happens in Python.

The library must have been built (`python -m paper_1606_04487_amd.build` or
`__graft_entry__.build()`); importing this module without it raises ImportError -- there is no
fallback path.
"""
from __future__ import annotations

import ctypes
from pathlib import Path
from typing import Optional, Sequence

import torch

_LIB_PATH = Path(__file__).resolve().parent / "libomniconv.so"
if not _LIB_PATH.exists():
    raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_1606_04487_amd.build`")
_lib = ctypes.CDLL(str(_LIB_PATH))

F32, BF16 = 0, 1
PASS_FORWARD, PASS_BACKWARD_DATA, PASS_BACKWARD_WEIGHTS = 0, 1, 2
FLAG_RELU, FLAG_DHAT_CACHED, FLAG_FUSED, FLAG_SPLIT_K = 1, 2, 4, 8

SYMBOLS = [
    "omni_conv_output_dims", "omni_conv_dhat_ld", "omni_conv_workspace_bytes", "omni_conv_fused_supported",
    "omni_conv_forward", "omni_conv_forward_partial", "omni_conv_forward_static", "omni_conv_static_scratch_need",
    "omni_conv_backward_data", "omni_conv_backward_weights", "omni_sgd_momentum_step", "omni_lower",
    "omni_conv_packed_weights_bytes", "omni_conv_pack_weights", "omni_conv_forward_packed", "omni_conv_backward_data_packed",
    "omni_col2im", "omni_relu_forward", "omni_relu_backward", "omni_pool_output_dim",
    "omni_maxpool_forward", "omni_maxpool_backward", "omni_maxpool_relu_backward",
    "omni_conv_dy_rows_layout", "omni_relu_backward_rows", "omni_maxpool_backward_rows", "omni_conv_backward_weights_rows",
    "omni_conv_backward_data_rows", "omni_conv_backward_data_relu_rows_sums", "omni_conv_backward_data_relu_rows",
    "omni_lrn_forward", "omni_lrn_backward", "omni_dropout_forward", "omni_dropout_backward", "omni_status_string", "omni_version", "omni_tuning_set",
    "omni_profile_enable", "omni_profile_select", "omni_profile_select_mask", "omni_profile_kernel_count", "omni_profile_kernel_name", "omni_profile_summary",
]


class ConvDesc(ctypes.Structure):
    """Mirror of `omni_conv_desc`."""
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "C", "H", "W", "F", "kh", "kw", "stride_h", "stride_w", "pad_h", "pad_w", "dtype")
                ] + [("flags", ctypes.c_uint32)]

    def with_flags(self, flags: int) -> "ConvDesc":
        d = ConvDesc.from_buffer_copy(self)
        d.flags = flags
        return d


class OmniError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"omniconv status {status}: {status_string(status)}")


_vp, _i32, _i64, _sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
_dp = ctypes.POINTER(ConvDesc)
_lib.omni_status_string.restype = ctypes.c_char_p
_lib.omni_status_string.argtypes = [ctypes.c_int]
_lib.omni_version.restype = ctypes.c_char_p
_lib.omni_conv_output_dims.argtypes = [_dp, ctypes.POINTER(_i32), ctypes.POINTER(_i32)]
_lib.omni_conv_dhat_ld.argtypes = [_dp, ctypes.POINTER(_i64)]
_lib.omni_conv_fused_supported.argtypes = [_dp, ctypes.c_int]
_lib.omni_conv_forward_partial.argtypes = [_dp, _i32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.omni_conv_forward_static.argtypes = [_dp, _vp, _vp, _vp, _vp, _vp]
_lib.omni_conv_static_scratch_need.argtypes = [_dp, ctypes.POINTER(_sz)]
_lib.omni_conv_workspace_bytes.argtypes = [_dp, ctypes.c_int, ctypes.POINTER(_sz)]
_lib.omni_conv_forward.argtypes = [_dp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.omni_conv_backward_data.argtypes = [_dp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.omni_conv_backward_weights.argtypes = [_dp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.omni_conv_packed_weights_bytes.argtypes = [_dp, ctypes.c_int, ctypes.POINTER(_sz)]
_lib.omni_conv_pack_weights.argtypes = [_i32, _vp, _vp, _vp, _vp, _vp]
_lib.omni_conv_forward_packed.argtypes = [_dp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.omni_conv_backward_data_packed.argtypes = [_dp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.omni_conv_dy_rows_layout.argtypes = [_dp, ctypes.POINTER(_i64), ctypes.POINTER(_i64)]
_lib.omni_relu_backward_rows.argtypes = [_i32, _i32, _i32, _i64, _vp, _vp, _vp, _i64, _vp, _vp]
_lib.omni_maxpool_backward_rows.argtypes = [_i32, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _i64, _vp, _vp]
_lib.omni_conv_backward_weights_rows.argtypes = [_dp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _sz, _vp]
_lib.omni_conv_backward_data_relu_rows_sums.argtypes = [_dp, ctypes.POINTER(_i32)]
_lib.omni_conv_backward_data_relu_rows.argtypes = [_dp, _vp, _vp, _vp, _vp, _i64, _vp, _vp, _sz, _vp]
_lib.omni_conv_backward_data_rows.argtypes = [_dp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.omni_sgd_momentum_step.argtypes = [_i32, _vp, _vp, _vp, _vp, _vp, ctypes.c_float, ctypes.c_float,
                                        ctypes.c_float, _vp]
_lib.omni_lower.argtypes = [_dp, _vp, _vp, _i64, _vp]
_lib.omni_col2im.argtypes = [_dp, _vp, _i64, _vp, _vp]
_lib.omni_relu_forward.argtypes = [_i32, _i64, _vp, _vp, _vp]
_lib.omni_relu_backward.argtypes = [_i32, _i64, _vp, _vp, _vp, _vp]
_lib.omni_pool_output_dim.argtypes = [_i32, _i32, _i32, _i32]
_lib.omni_maxpool_forward.argtypes = [_i32, _i64, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp]
_lib.omni_maxpool_backward.argtypes = [_i32, _i64, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp]
_lib.omni_maxpool_relu_backward.argtypes = [_i32, _i64, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp]
_f, _u64 = ctypes.c_float, ctypes.c_uint64
_lib.omni_lrn_forward.argtypes = [_i32, _i64, _i32, _i64, _i32, _f, _f, _f, _vp, _vp, _vp, _vp]
_lib.omni_lrn_backward.argtypes = [_i32, _i64, _i32, _i64, _i32, _f, _f, _f, _vp, _vp, _vp, _vp, _vp]
_lib.omni_dropout_forward.argtypes = [_i32, _i64, _f, _u64, _u64, _vp, _vp, _vp]
_lib.omni_dropout_backward.argtypes = [_i32, _i64, _f, _u64, _u64, _vp, _vp, _vp]


_lib.omni_profile_enable.argtypes = [ctypes.c_int]
_lib.omni_profile_select_mask.argtypes = [ctypes.c_uint64]
_lib.omni_profile_kernel_name.restype = ctypes.c_char_p
_lib.omni_profile_kernel_name.argtypes = [ctypes.c_int]
_lib.omni_profile_summary.argtypes = [ctypes.c_int, ctypes.POINTER(_i64), ctypes.POINTER(ctypes.c_double),
                                      ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]


def raw():
    """The ctypes library handle (for tests of the error paths)."""
    return _lib


TUNE_GEMM_TILE, TUNE_FUSED_BN, TUNE_FUSED_BM, TUNE_WGRAD_SPLITS, TUNE_WGRAD_PATCH, TUNE_FUSED_PITCH, TUNE_POOL_LDS = 0, 1, 2, 3, 4, 5, 6


def tuning_set(knob: int, value: int) -> None:
    """omni_tuning_set: tile overrides for sweeps and tests."""
    _check(_lib.omni_tuning_set(int(knob), int(value)))


def status_string(status: int) -> str:
    return _lib.omni_status_string(int(status)).decode()


def version() -> str:
    return _lib.omni_version().decode()


def _check(status: int) -> None:
    if status != 0:
        raise OmniError(status)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _p(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous and live on the GPU")
    return t.data_ptr()


def torch_dtype(dtype: int):
    return torch.bfloat16 if dtype == BF16 else torch.float32


def dtype_code(t: torch.dtype) -> int:
    if t == torch.float32:
        return F32
    if t == torch.bfloat16:
        return BF16
    raise ValueError(f"unsupported dtype {t}")


def conv_desc(N, C, H, W, F, kh, kw=None, stride=1, pad=0, dtype=F32, flags=0) -> ConvDesc:
    kw = kh if kw is None else kw
    sh, sw = (stride, stride) if isinstance(stride, int) else stride
    ph, pw = (pad, pad) if isinstance(pad, int) else pad
    return ConvDesc(N, C, H, W, F, kh, kw, sh, sw, ph, pw, dtype, flags)


def conv_output_dims(desc: ConvDesc):
    ho, wo = _i32(), _i32()
    _check(_lib.omni_conv_output_dims(ctypes.byref(desc), ctypes.byref(ho), ctypes.byref(wo)))
    return ho.value, wo.value


def conv_dhat_ld(desc: ConvDesc) -> int:
    ld = _i64()
    _check(_lib.omni_conv_dhat_ld(ctypes.byref(desc), ctypes.byref(ld)))
    return ld.value


def conv_fused_supported(desc: ConvDesc, which_pass: int) -> bool:
    r = _lib.omni_conv_fused_supported(ctypes.byref(desc), which_pass)
    if r < 0:
        raise OmniError(r)
    return bool(r)


def conv_workspace_bytes(desc: ConvDesc, which_pass: int) -> int:
    b = _sz()
    _check(_lib.omni_conv_workspace_bytes(ctypes.byref(desc), which_pass, ctypes.byref(b)))
    return b.value


def alloc_workspace(desc: ConvDesc, which_pass: int, device="cuda") -> torch.Tensor:
    return torch.empty(conv_workspace_bytes(desc, which_pass), dtype=torch.uint8, device=device)


def conv_forward(desc: ConvDesc, X, W, bias=None, Y=None, workspace=None):
    """omni_conv_forward: lowering of the whole batch, one GEMM, epilogue into Y [N][F][Ho][Wo]."""
    ho, wo = conv_output_dims(desc)
    if Y is None:
        Y = torch.empty((desc.N, desc.F, ho, wo), dtype=torch_dtype(desc.dtype), device=X.device)
    if workspace is None:
        workspace = alloc_workspace(desc, PASS_FORWARD, X.device)
    _check(_lib.omni_conv_forward(ctypes.byref(desc), _p(X), _p(W), _p(bias), _p(Y), _p(workspace),
                                  workspace.numel(), _stream()))
    return Y


STATIC_SCRATCH_BYTES = 32 << 20


def conv_static_scratch_need(desc: ConvDesc) -> int:
    b = _sz()
    _check(_lib.omni_conv_static_scratch_need(ctypes.byref(desc), ctypes.byref(b)))
    return b.value


def conv_forward_static(desc: ConvDesc, X, W, bias, Y):
    """omni_conv_forward_static: the forward pass on the library's own static scratch; allocates nothing
    (the caller passes the output tensor)."""
    _check(_lib.omni_conv_forward_static(ctypes.byref(desc), _p(X), _p(W), _p(bias), _p(Y), _stream()))
    return Y


def conv_forward_partial(desc: ConvDesc, b_p: int, X, W, bias=None, Y=None, workspace=None):
    """omni_conv_forward_partial: the forward pass b_p images at a time through a workspace sized for b_p."""
    ho, wo = conv_output_dims(desc)
    if Y is None:
        Y = torch.empty((desc.N, desc.F, ho, wo), dtype=torch_dtype(desc.dtype), device=X.device)
    if workspace is None:
        sub = ConvDesc.from_buffer_copy(desc)
        sub.N = b_p
        workspace = alloc_workspace(sub, PASS_FORWARD, X.device)
    _check(_lib.omni_conv_forward_partial(ctypes.byref(desc), b_p, _p(X), _p(W), _p(bias), _p(Y), _p(workspace),
                                          workspace.numel(), _stream()))
    return Y


def conv_backward_data(desc: ConvDesc, dY, W, dX=None, workspace=None):
    """omni_conv_backward_data: dY-hat packing, one GEMM, col2im into dX [N][C][H][W]."""
    if dX is None:
        dX = torch.empty((desc.N, desc.C, desc.H, desc.W), dtype=torch_dtype(desc.dtype), device=dY.device)
    if workspace is None:
        workspace = alloc_workspace(desc, PASS_BACKWARD_DATA, dY.device)
    _check(_lib.omni_conv_backward_data(ctypes.byref(desc), _p(dY), _p(W), _p(dX), _p(workspace),
                                        workspace.numel(), _stream()))
    return dX


def conv_packed_weights_bytes(desc: ConvDesc, which: int) -> int:
    """omni_conv_packed_weights_bytes: bytes of the repacked weights that pass `which` reads (0: none)."""
    b = _sz()
    _check(_lib.omni_conv_packed_weights_bytes(ctypes.byref(desc), which, ctypes.byref(b)))
    return b.value


def conv_pack_weights(descs: Sequence[ConvDesc], passes: Sequence[int], W: Sequence[torch.Tensor],
                      packed: Sequence[torch.Tensor]) -> None:
    """omni_conv_pack_weights: the repacked weights of several layer-and-pass pairs in one launch."""
    n = len(descs)
    if not (len(passes) == n and len(W) == n and len(packed) == n):
        raise ValueError("descs, passes, W and packed must have equal length")
    darr = (ConvDesc * max(n, 1))(*descs)
    parr = (_i32 * max(n, 1))(*passes)
    arr = _vp * max(n, 1)
    _check(_lib.omni_conv_pack_weights(n, darr, parr, arr(*[_p(t) for t in W]), arr(*[_p(t) for t in packed]), _stream()))


def conv_forward_packed(desc: ConvDesc, X, packed, bias=None, Y=None, workspace=None):
    """omni_conv_forward_packed: omni_conv_forward reading weights repacked by conv_pack_weights."""
    ho, wo = conv_output_dims(desc)
    if Y is None:
        Y = torch.empty((desc.N, desc.F, ho, wo), dtype=torch_dtype(desc.dtype), device=X.device)
    if workspace is None:
        workspace = alloc_workspace(desc, PASS_FORWARD, X.device)
    _check(_lib.omni_conv_forward_packed(ctypes.byref(desc), _p(X), _p(packed), _p(bias), _p(Y), _p(workspace),
                                         workspace.numel(), _stream()))
    return Y


def conv_backward_data_packed(desc: ConvDesc, dY, packed, dX=None, workspace=None):
    """omni_conv_backward_data_packed: omni_conv_backward_data reading weights repacked by conv_pack_weights."""
    if dX is None:
        dX = torch.empty((desc.N, desc.C, desc.H, desc.W), dtype=torch_dtype(desc.dtype), device=dY.device)
    if workspace is None:
        workspace = alloc_workspace(desc, PASS_BACKWARD_DATA, dY.device)
    _check(_lib.omni_conv_backward_data_packed(ctypes.byref(desc), _p(dY), _p(packed), _p(dX), _p(workspace),
                                               workspace.numel(), _stream()))
    return dX


def conv_backward_weights(desc: ConvDesc, X, dY, dW=None, dbias=None, workspace=None, want_dbias=True):
    """omni_conv_backward_weights: fp32 dW [F][C][kh][kw] (and dbias [F]) summed over the batch."""
    if dW is None:
        dW = torch.empty((desc.F, desc.C, desc.kh, desc.kw), dtype=torch.float32, device=dY.device)
    if dbias is None and want_dbias:
        dbias = torch.empty((desc.F,), dtype=torch.float32, device=dY.device)
    if workspace is None:
        workspace = alloc_workspace(desc, PASS_BACKWARD_WEIGHTS, dY.device)
    _check(_lib.omni_conv_backward_weights(ctypes.byref(desc), _p(X), _p(dY), _p(dW), _p(dbias),
                                           _p(workspace), workspace.numel(), _stream()))
    return dW, dbias


def sgd_momentum_step(W: Sequence[torch.Tensor], V: Sequence[torch.Tensor], G: Sequence[torch.Tensor],
                      lr: float, momentum: float, weight_decay: float = 0.0,
                      W_shadow: Optional[Sequence[Optional[torch.Tensor]]] = None) -> None:
    """omni_sgd_momentum_step: V <- mu V - lr (G + lambda W); W <- W + V, in place, all tensors at once."""
    n = len(W)
    if not (len(V) == n and len(G) == n and (W_shadow is None or len(W_shadow) == n)):
        raise ValueError("W, V, G (and W_shadow) must have equal length")
    for t in list(W) + list(V) + list(G):
        if t.dtype != torch.float32:
            raise ValueError("W, V and G must be float32")
    arr = _vp * max(n, 1)
    cnt = (_i64 * max(n, 1))(*[w.numel() for w in W])
    pw, pv, pg = arr(*[_p(t) for t in W]), arr(*[_p(t) for t in V]), arr(*[_p(t) for t in G])
    ps = None
    if W_shadow is not None:
        for t in W_shadow:
            if t is not None and t.dtype != torch.bfloat16:
                raise ValueError("W_shadow tensors must be bfloat16")
        ps = arr(*[_p(t) for t in W_shadow])
    _check(_lib.omni_sgd_momentum_step(n, pw, pv, pg, cnt, ps, lr, momentum, weight_decay, _stream()))


def lower(desc: ConvDesc, X, Dhat=None, ld: Optional[int] = None):
    """omni_lower: D-hat [C*kh*kw][ld] in the canonical layout (ld defaults to N*Ho*Wo)."""
    ho, wo = conv_output_dims(desc)
    M = desc.N * ho * wo
    ld = M if ld is None else ld
    if Dhat is None:
        Dhat = torch.empty((desc.C * desc.kh * desc.kw, ld), dtype=torch_dtype(desc.dtype), device=X.device)
    _check(_lib.omni_lower(ctypes.byref(desc), _p(X), _p(Dhat), ld, _stream()))
    return Dhat


def col2im(desc: ConvDesc, dDhat, dX=None, ld: Optional[int] = None):
    """omni_col2im: sums a D-hat-shaped matrix back into dX [N][C][H][W]."""
    ld = dDhat.shape[1] if ld is None else ld
    if dX is None:
        dX = torch.empty((desc.N, desc.C, desc.H, desc.W), dtype=torch_dtype(desc.dtype), device=dDhat.device)
    _check(_lib.omni_col2im(ctypes.byref(desc), _p(dDhat), ld, _p(dX), _stream()))
    return dX


def relu_forward(x, y=None):
    y = torch.empty_like(x) if y is None else y
    _check(_lib.omni_relu_forward(dtype_code(x.dtype), x.numel(), _p(x), _p(y), _stream()))
    return y


def relu_backward(y, dy, dx=None):
    dx = torch.empty_like(dy) if dx is None else dx
    _check(_lib.omni_relu_backward(dtype_code(y.dtype), y.numel(), _p(y), _p(dy), _p(dx), _stream()))
    return dx


def pool_output_dim(n: int, k: int = 3, stride: int = 2, ceil_mode: bool = True) -> int:
    o = _lib.omni_pool_output_dim(n, k, stride, int(ceil_mode))
    if o < 0:
        raise OmniError(o)
    return o


def maxpool_forward(x, k: int = 3, stride: int = 2, ceil_mode: bool = True, y=None, argmax=None):
    """omni_maxpool_forward over the last two axes; returns (y, argmax uint8 = ky*k+kx of the winner)."""
    H, W = x.shape[-2:]
    planes = x.numel() // (H * W)
    ho, wo = pool_output_dim(H, k, stride, ceil_mode), pool_output_dim(W, k, stride, ceil_mode)
    if y is None:
        y = torch.empty(tuple(x.shape[:-2]) + (ho, wo), dtype=x.dtype, device=x.device)
    if argmax is None:
        argmax = torch.empty(tuple(x.shape[:-2]) + (ho, wo), dtype=torch.uint8, device=x.device)
    _check(_lib.omni_maxpool_forward(dtype_code(x.dtype), planes, H, W, k, stride, int(ceil_mode), _p(x), _p(y),
                                     _p(argmax), _stream()))
    return y, argmax


def maxpool_backward(dy, argmax, H: int, W: int, k: int = 3, stride: int = 2, ceil_mode: bool = True, dx=None):
    planes = dy.numel() // (dy.shape[-1] * dy.shape[-2])
    if dx is None:
        dx = torch.empty(tuple(dy.shape[:-2]) + (H, W), dtype=dy.dtype, device=dy.device)
    _check(_lib.omni_maxpool_backward(dtype_code(dy.dtype), planes, H, W, k, stride, int(ceil_mode), _p(dy),
                                      _p(argmax), _p(dx), _stream()))
    return dx


def maxpool_relu_backward(dy, argmax, y_pooled, H: int, W: int, k: int = 3, stride: int = 2, ceil_mode: bool = True,
                          dx=None):
    """omni_maxpool_relu_backward: pool backward times the gradient of the ReLU in front of the pool, in one
    pass; y_pooled is the forward pool's output (same shape as dy)."""
    planes = dy.numel() // (dy.shape[-1] * dy.shape[-2])
    if dx is None:
        dx = torch.empty(tuple(dy.shape[:-2]) + (H, W), dtype=dy.dtype, device=dy.device)
    _check(_lib.omni_maxpool_relu_backward(dtype_code(dy.dtype), planes, H, W, k, stride, int(ceil_mode), _p(dy),
                                           _p(argmax), _p(y_pooled), _p(dx), _stream()))
    return dx


def conv_dy_rows_layout(desc: ConvDesc):
    """omni_conv_dy_rows_layout: (ld, plane_pitch) of the rows form of dY this layer's model gradient reads, or None
    when it reads no such form."""
    ld, pitch = _i64(0), _i64(0)
    st = _lib.omni_conv_dy_rows_layout(ctypes.byref(desc), ctypes.byref(ld), ctypes.byref(pitch))
    if st == -2:
        return None
    _check(st)
    return ld.value, pitch.value


def _rows_out(dx_rows, plane_sums, N, C, plane, ld, want_sums, device):
    if ld is None:
        ld = N * ((plane + 7) // 8 * 8)
    if dx_rows is None:
        dx_rows = torch.zeros((C, ld), dtype=torch.bfloat16, device=device)
    if plane_sums is None and want_sums:
        plane_sums = torch.empty((C, N), dtype=torch.float32, device=device)
    return dx_rows, plane_sums, ld


def relu_backward_rows(y, dy, dx_rows=None, plane_sums=None, ld=None, want_sums=True):
    """omni_relu_backward_rows: ReLU backward of [N][C][...] tensors written as the rows matrix [C][ld]; returns
    (dx_rows, plane_sums [C][N])."""
    N, C = y.shape[:2]
    plane = y.numel() // (N * C) if N * C else 0
    dx_rows, plane_sums, ld = _rows_out(dx_rows, plane_sums, N, C, plane, ld, want_sums, y.device)
    _check(_lib.omni_relu_backward_rows(dtype_code(y.dtype), N, C, plane, _p(y), _p(dy), _p(dx_rows), ld, _p(plane_sums),
                                        _stream()))
    return dx_rows, plane_sums


def maxpool_backward_rows(dy, argmax, y_pooled, H: int, W: int, k: int = 3, stride: int = 2, ceil_mode: bool = True,
                          dx_rows=None, plane_sums=None, ld=None, want_sums=True):
    """omni_maxpool_backward_rows: max-pool backward (times the ReLU's gradient when y_pooled is given) of dy
    [N][C][Ho][Wo], written as the rows matrix [C][ld] of the [N][C][H][W] gradient; returns (dx_rows, plane_sums)."""
    N, C = dy.shape[:2]
    dx_rows, plane_sums, ld = _rows_out(dx_rows, plane_sums, N, C, H * W, ld, want_sums, dy.device)
    _check(_lib.omni_maxpool_backward_rows(dtype_code(dy.dtype), N, C, H, W, k, stride, int(ceil_mode), _p(dy), _p(argmax),
                                           _p(y_pooled), _p(dx_rows), ld, _p(plane_sums), _stream()))
    return dx_rows, plane_sums


def conv_backward_weights_rows(desc: ConvDesc, X, dY_rows, plane_sums, dW=None, dbias=None, workspace=None, want_dbias=True):
    """omni_conv_backward_weights_rows: omni_conv_backward_weights reading dY in its rows form; plane_sums [F][any] are
    partial sums of every filter's row (for the bias gradient)."""
    if dW is None:
        dW = torch.empty((desc.F, desc.C, desc.kh, desc.kw), dtype=torch.float32, device=X.device)
    if dbias is None and want_dbias:
        dbias = torch.empty((desc.F,), dtype=torch.float32, device=X.device)
    if workspace is None:
        workspace = alloc_workspace(desc, PASS_BACKWARD_WEIGHTS, X.device)
    per = plane_sums.shape[1] if plane_sums is not None else 0
    _check(_lib.omni_conv_backward_weights_rows(ctypes.byref(desc), _p(X), _p(dY_rows), _p(plane_sums), per, _p(dW), _p(dbias),
                                                _p(workspace), workspace.numel(), _stream()))
    return dW, dbias


def conv_backward_data_rows(desc: ConvDesc, dY_rows, packed, dX=None, workspace=None):
    """omni_conv_backward_data_rows: omni_conv_backward_data_packed reading dY in its rows form."""
    if dX is None:
        dX = torch.empty((desc.N, desc.C, desc.H, desc.W), dtype=torch_dtype(desc.dtype), device=dY_rows.device)
    if workspace is None:
        workspace = alloc_workspace(desc, PASS_BACKWARD_DATA, dY_rows.device)
    _check(_lib.omni_conv_backward_data_rows(ctypes.byref(desc), _p(dY_rows), _p(packed), _p(dX), _p(workspace),
                                             workspace.numel(), _stream()))
    return dX


def conv_backward_data_relu_rows_sums(desc: ConvDesc):
    """omni_conv_backward_data_relu_rows_sums: partial sums per channel that conv_backward_data_relu_rows writes, or
    None when this layer's data gradient cannot store the masked rows form."""
    n = _i32(0)
    st = _lib.omni_conv_backward_data_relu_rows_sums(ctypes.byref(desc), ctypes.byref(n))
    if st == -2:
        return None
    _check(st)
    return n.value


def conv_backward_data_relu_rows(desc: ConvDesc, dY_rows, packed, y_front, dX_rows=None, col_sums=None, ld_out=None,
                                 workspace=None, want_sums=True):
    """omni_conv_backward_data_relu_rows: the data gradient stored as the rows form of (y_front > 0 ? dX : 0), the
    output gradient of the convolution + ReLU layer in front; returns (dX_rows [C][ld_out], col_sums)."""
    pitch = (desc.H * desc.W + 7) // 8 * 8
    if ld_out is None:
        ld_out = desc.N * pitch
    if dX_rows is None:
        dX_rows = torch.zeros((desc.C, ld_out), dtype=torch.bfloat16, device=dY_rows.device)
    if col_sums is None and want_sums:
        col_sums = torch.empty((desc.C, conv_backward_data_relu_rows_sums(desc)), dtype=torch.float32, device=dY_rows.device)
    if workspace is None:
        workspace = alloc_workspace(desc, PASS_BACKWARD_DATA, dY_rows.device)
    _check(_lib.omni_conv_backward_data_relu_rows(ctypes.byref(desc), _p(dY_rows), _p(packed), _p(y_front), _p(dX_rows), ld_out,
                                                  _p(col_sums), _p(workspace), workspace.numel(), _stream()))
    return dX_rows, col_sums


def lrn_forward(x, size: int = 5, alpha: float = 1e-4, beta: float = 0.75, k: float = 1.0, y=None, scale=None,
                want_scale: bool = True):
    """omni_lrn_forward over x [N][C][...]; returns (y, scale) -- scale (fp32) is what lrn_backward needs."""
    N, C = x.shape[:2]
    plane = x.numel() // (N * C) if N * C else 0
    y = torch.empty_like(x) if y is None else y
    if scale is None and want_scale:
        scale = torch.empty(x.shape, dtype=torch.float32, device=x.device)
    _check(_lib.omni_lrn_forward(dtype_code(x.dtype), N, C, plane, size, alpha, beta, k, _p(x), _p(y), _p(scale), _stream()))
    return y, scale


def lrn_backward(x, dy, scale, size: int = 5, alpha: float = 1e-4, beta: float = 0.75, k: float = 1.0, dx=None):
    """omni_lrn_backward: gradient w.r.t. the normalisation's input."""
    N, C = x.shape[:2]
    plane = x.numel() // (N * C) if N * C else 0
    dx = torch.empty_like(x) if dx is None else dx
    _check(_lib.omni_lrn_backward(dtype_code(x.dtype), N, C, plane, size, alpha, beta, k, _p(x), _p(dy), _p(scale), _p(dx),
                                  _stream()))
    return dx


def dropout_forward(x, p: float, seed: int, stream_id: int = 0, y=None):
    """omni_dropout_forward: keep with probability 1 - p, scale by 1 / (1 - p); the mask is a function of
    (p, seed, stream_id, element index)."""
    y = torch.empty_like(x) if y is None else y
    _check(_lib.omni_dropout_forward(dtype_code(x.dtype), x.numel(), p, seed, stream_id, _p(x), _p(y), _stream()))
    return y


def dropout_backward(dy, p: float, seed: int, stream_id: int = 0, dx=None):
    """omni_dropout_backward: the same mask and scale applied to the gradient."""
    dx = torch.empty_like(dy) if dx is None else dx
    _check(_lib.omni_dropout_backward(dtype_code(dy.dtype), dy.numel(), p, seed, stream_id, _p(dy), _p(dx), _stream()))
    return dx


def profile_enable(on: bool) -> None:
    """omni_profile_enable: start (and clear) or stop per-kernel event timing."""
    _check(_lib.omni_profile_enable(int(bool(on))))


def profile_select(kernel_name: Optional[str]) -> None:
    """omni_profile_select: record events for one kernel class only (None: all classes)."""
    if kernel_name is None:
        _check(_lib.omni_profile_select(-1))
        return
    names = [_lib.omni_profile_kernel_name(i).decode() for i in range(_lib.omni_profile_kernel_count())]
    _check(_lib.omni_profile_select(names.index(kernel_name)))


def profile_select_many(kernel_names) -> None:
    """omni_profile_select_mask: record events for the named kernel classes only."""
    names = [_lib.omni_profile_kernel_name(i).decode() for i in range(_lib.omni_profile_kernel_count())]
    mask = 0
    for n in kernel_names:
        mask |= 1 << names.index(n)
    _check(_lib.omni_profile_select_mask(ctypes.c_uint64(mask)))


def profile_summary() -> dict:
    """omni_profile_summary for every kernel class: name -> launches, total_ms, flops, bytes."""
    out = {}
    for kid in range(_lib.omni_profile_kernel_count()):
        n, ms, fl, by = _i64(), ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
        _check(_lib.omni_profile_summary(kid, ctypes.byref(n), ctypes.byref(ms), ctypes.byref(fl), ctypes.byref(by)))
        if n.value:
            out[_lib.omni_profile_kernel_name(kid).decode()] = {
                "launches": n.value, "total_ms": ms.value, "flops": fl.value, "bytes": by.value}
    return out
