"""Thin ctypes binding of libcirc.so: argument marshalling only.

Every step of the layers runs inside the HIP library; PyTorch is used here for
device buffers and the current stream.  There is no CPU fallback: if the shared
library is missing the first call raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libcirc.so")

CIRC_OK, CIRC_EINVAL, CIRC_ENOTSUP, CIRC_EWORKSPACE, CIRC_EHIP = 0, -1, -2, -3, -4
EPI_NONE, EPI_BIAS, EPI_RELU = 0, 1, 2

_lib = None

_c_int, _c_size, _c_ptr = ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p

SIGNATURES = {
    "circ_status_string": (ctypes.c_char_p, [_c_int]),
    "circ_spectra_bytes": (_c_size, [_c_int] * 4),
    "circ_precompute_spectra": (_c_int, [_c_ptr, _c_int, _c_int, _c_int, _c_int, _c_ptr, _c_ptr]),
    "circ_fc_workspace_bytes": (_c_size, [_c_int] * 5),
    "circ_fc_forward": (_c_int, [_c_ptr, _c_ptr, _c_ptr, _c_ptr, _c_int, _c_int, _c_int, _c_int, _c_int,
                                 _c_ptr, _c_size, _c_ptr]),
    "circ_fc_forward_static": (_c_int, [_c_ptr, _c_ptr, _c_ptr, _c_ptr, _c_int, _c_int, _c_int, _c_int, _c_int, _c_ptr]),
    "circ_fc_backward": (_c_int, [_c_ptr, _c_ptr, _c_ptr, _c_ptr, _c_ptr, _c_int, _c_int, _c_int, _c_int,
                                  _c_ptr, _c_size, _c_ptr]),
    "circ_conv_workspace_bytes": (_c_size, [_c_int] * 9),
    "circ_conv_forward": (_c_int, [_c_ptr, _c_ptr, _c_ptr, _c_ptr] + [_c_int] * 10 + [_c_ptr, _c_size, _c_ptr]),
    "circ_conv_forward_f16": (_c_int, [_c_ptr, _c_ptr, _c_ptr, _c_ptr] + [_c_int] * 10 + [_c_ptr, _c_size, _c_ptr]),
    "circ_conv_forward_bf16": (_c_int, [_c_ptr, _c_ptr, _c_ptr, _c_ptr] + [_c_int] * 10 + [_c_ptr, _c_size, _c_ptr]),
    "circ_conv_backward_f16": (_c_int, [_c_ptr] * 5 + [_c_int] * 9 + [_c_ptr, _c_size, _c_ptr]),
    "circ_conv_backward_bf16": (_c_int, [_c_ptr] * 5 + [_c_int] * 9 + [_c_ptr, _c_size, _c_ptr]),
    "circ_conv_backward_workspace_bytes": (_c_size, [_c_int] * 9),
    "circ_conv_backward": (_c_int, [_c_ptr] * 5 + [_c_int] * 9 + [_c_ptr, _c_size, _c_ptr]),
    "circ_bias_grad": (_c_int, [_c_ptr, _c_ptr, ctypes.c_longlong, _c_int, ctypes.c_longlong, _c_ptr]),
    "circ_fc_sgd_step": (_c_int, [_c_ptr] * 4 + [ctypes.c_float] + [_c_int] * 4 + [_c_ptr, _c_size, _c_ptr]),
    "circ_conv_sgd_step": (_c_int, [_c_ptr] * 4 + [ctypes.c_float] + [_c_int] * 9 + [_c_ptr, _c_size, _c_ptr]),
    "circ_export_weights": (_c_int, [_c_ptr] + [_c_int] * 4 + [_c_ptr, _c_ptr]),
    "circ_spectra_bytes_f16": (_c_size, [_c_int] * 3),
    "circ_precompute_spectra_f16": (_c_int, [_c_ptr, _c_int, _c_int, _c_int, _c_ptr, _c_ptr]),
    "circ_fc_workspace_bytes_f16": (_c_size, [_c_int] * 4),
    "circ_fc_forward_f16": (_c_int, [_c_ptr, _c_ptr, _c_ptr, _c_ptr, _c_int, _c_int, _c_int, _c_int, _c_int,
                                     _c_ptr, _c_size, _c_ptr]),
    "circ_fc_backward_workspace_bytes_f16": (_c_size, [_c_int] * 4),
    "circ_fc_backward_f16": (_c_int, [_c_ptr] * 5 + [_c_int] * 4 + [_c_ptr, _c_size, _c_ptr]),
    "circ_fc_backward_workspace_bytes_bf16": (_c_size, [_c_int] * 4),
    "circ_fc_backward_bf16": (_c_int, [_c_ptr] * 5 + [_c_int] * 4 + [_c_ptr, _c_size, _c_ptr]),
    "circ_spectra_bytes_bf16": (_c_size, [_c_int] * 3),
    "circ_precompute_spectra_bf16": (_c_int, [_c_ptr, _c_int, _c_int, _c_int, _c_ptr, _c_ptr]),
    "circ_fc_workspace_bytes_bf16": (_c_size, [_c_int] * 4),
    "circ_fc_forward_bf16": (_c_int, [_c_ptr, _c_ptr, _c_ptr, _c_ptr, _c_int, _c_int, _c_int, _c_int, _c_int,
                                      _c_ptr, _c_size, _c_ptr]),
}


LAYER_FC, LAYER_CONV, LAYER_MAXPOOL = 0, 1, 2


class CircLayer(ctypes.Structure):
    """circ_layer of include/circ.h (one layer of a chain; a host-side descriptor)."""
    _fields_ = [("kind", _c_int), ("epilogue", _c_int), ("w_hat", _c_ptr), ("bias", _c_ptr), ("k", _c_int),
                ("p", _c_int), ("q", _c_int), ("C_in", _c_int), ("C_out", _c_int), ("H", _c_int), ("W", _c_int),
                ("r", _c_int), ("stride", _c_int), ("pad", _c_int)]


SIGNATURES.update({
    "circ_maxpool_forward": (_c_int, [_c_ptr, _c_ptr] + [_c_int] * 6 + [_c_ptr]),
    "circ_chain_workspace_bytes": (_c_size, [ctypes.POINTER(CircLayer), _c_int, _c_int]),
    "circ_chain_forward": (_c_int, [ctypes.POINTER(CircLayer), _c_int, _c_ptr, _c_ptr, _c_int, _c_ptr, _c_size, _c_ptr]),
})


class CircError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}")


def lib() -> ctypes.CDLL:
    """Load libcirc.so (built by paper_1708_08917_amd.build); fail loudly if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not found: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().circ_status_string(status).decode()


def _ptr(t, dtype=None):
    """Device pointer of a dense device tensor (None passes through as NULL).  The library reads raw
    memory, so a host tensor, a strided view or a tensor of another element type is refused here."""
    if t is None:
        return None
    if not (t.is_cuda and t.is_contiguous()):
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected a {dtype} tensor, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _f32(t):
    return _ptr(t, torch.float32)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status: int, where: str):
    if status != CIRC_OK:
        raise CircError(status, where)


def circ_spectra_bytes(n_grids: int, p: int, q: int, k: int) -> int:
    return lib().circ_spectra_bytes(n_grids, p, q, k)


def circ_fc_workspace_bytes(p: int, q: int, k: int, batch: int, backward: bool = False) -> int:
    return lib().circ_fc_workspace_bytes(p, q, k, batch, int(backward))


def circ_conv_workspace_bytes(N, C_in, C_out, H, W, r, stride, pad, k) -> int:
    return lib().circ_conv_workspace_bytes(N, C_in, C_out, H, W, r, stride, pad, k)


def circ_precompute_spectra(w: torch.Tensor, w_hat: torch.Tensor | None = None) -> torch.Tensor:
    """w: device fp32 [p][q][k] or [r][r][p][q][k] -> opaque spectra blob (uint8 tensor)."""
    assert w.is_cuda and w.dtype == torch.float32 and w.is_contiguous()
    p, q, k = w.shape[-3:]
    n_grids = int(w.numel() // (p * q * k))
    nbytes = circ_spectra_bytes(n_grids, p, q, k)
    if nbytes == 0:
        raise CircError(CIRC_EINVAL, "circ_spectra_bytes")
    if w_hat is None:
        w_hat = torch.empty(nbytes, dtype=torch.uint8, device=w.device)
    _check(lib().circ_precompute_spectra(_f32(w), n_grids, p, q, k, _ptr(w_hat), _stream()), "circ_precompute_spectra")
    return w_hat


def circ_fc_forward(w_hat, x, bias, y, p, q, k, epilogue=EPI_NONE, workspace=None):
    """x: [batch][q*k] -> y: [batch][p*k] (y allocated if None).  Returns y."""
    batch = x.shape[0]
    if y is None:
        y = torch.empty(batch, p * k, dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = torch.empty(max(1, circ_fc_workspace_bytes(p, q, k, batch)), dtype=torch.uint8, device=x.device)
    _check(lib().circ_fc_forward(_ptr(w_hat), _f32(x), _f32(bias), _f32(y), p, q, k, batch, epilogue,
                                 _ptr(workspace), workspace.numel(), _stream()), "circ_fc_forward")
    return y


STATIC_SCRATCH_BYTES = 32 << 20


def circ_fc_forward_static(w_hat, x, bias, y, p, q, k, epilogue=EPI_NONE):
    """circ_fc_forward on the library's own fixed scratch array: y must be given (nothing is allocated)."""
    _check(lib().circ_fc_forward_static(_ptr(w_hat), _f32(x), _f32(bias), _f32(y), p, q, k, x.shape[0], epilogue,
                                        _stream()), "circ_fc_forward_static")
    return y


def circ_fc_backward(w_hat, x, dy, p, q, k, need_dx=True, need_dw=True, dx=None, dw=None, workspace=None):
    """Returns (dx [batch][q*k] or None, dw [p][q][k] or None)."""
    batch = dy.shape[0]
    if need_dx and dx is None:
        dx = torch.empty(batch, q * k, dtype=torch.float32, device=dy.device)
    if need_dw and dw is None:
        dw = torch.empty(p, q, k, dtype=torch.float32, device=dy.device)
    if workspace is None:
        workspace = torch.empty(max(1, circ_fc_workspace_bytes(p, q, k, batch, True)), dtype=torch.uint8,
                                device=dy.device)
    _check(lib().circ_fc_backward(_ptr(w_hat), _f32(x), _f32(dy), _f32(dx if need_dx else None),
                                  _f32(dw if need_dw else None), p, q, k, batch, _ptr(workspace),
                                  workspace.numel(), _stream()), "circ_fc_backward")
    return (dx if need_dx else None), (dw if need_dw else None)


def circ_conv_forward(w_hat, x, bias, y, C_out, r, stride, pad, k, epilogue=EPI_NONE, workspace=None):
    """x: NCHW -> y: NCHW (allocated if None).  Returns y."""
    N, C_in, H, W = x.shape
    Ho, Wo = (H + 2 * pad - r) // stride + 1, (W + 2 * pad - r) // stride + 1
    if y is None:
        y = torch.empty(N, C_out, Ho, Wo, dtype=torch.float32, device=x.device)
    if workspace is None:
        nb = circ_conv_workspace_bytes(N, C_in, C_out, H, W, r, stride, pad, k)
        workspace = torch.empty(max(1, nb), dtype=torch.uint8, device=x.device)
    _check(lib().circ_conv_forward(_ptr(w_hat), _f32(x), _f32(bias), _f32(y), N, C_in, C_out, H, W, r, stride, pad,
                                   k, epilogue, _ptr(workspace), workspace.numel(), _stream()), "circ_conv_forward")
    return y


def circ_conv_backward_workspace_bytes(N, C_in, C_out, H, W, r, stride, pad, k) -> int:
    return lib().circ_conv_backward_workspace_bytes(N, C_in, C_out, H, W, r, stride, pad, k)


def circ_conv_backward(w_hat, x, dy, C_in, H, W, r, stride, pad, k, need_dx=True, need_dw=True, dx=None, dw=None,
                       workspace=None):
    """dy: NCHW [N][C_out][Ho][Wo] -> (dx NCHW [N][C_in][H][W] or None, dw [r][r][p][q][k] or None)."""
    N, C_out = dy.shape[0], dy.shape[1]
    p, q = C_out // k, C_in // k
    if need_dx and dx is None:
        dx = torch.empty(N, C_in, H, W, dtype=torch.float32, device=dy.device)
    if need_dw and dw is None:
        dw = torch.empty(r, r, p, q, k, dtype=torch.float32, device=dy.device)
    if workspace is None:
        nb = circ_conv_backward_workspace_bytes(N, C_in, C_out, H, W, r, stride, pad, k)
        workspace = torch.empty(max(1, nb), dtype=torch.uint8, device=dy.device)
    _check(lib().circ_conv_backward(_ptr(w_hat), _f32(x), _f32(dy), _f32(dx if need_dx else None),
                                    _f32(dw if need_dw else None), N, C_in, C_out, H, W, r, stride, pad, k,
                                    _ptr(workspace), workspace.numel(), _stream()), "circ_conv_backward")
    return (dx if need_dx else None), (dw if need_dw else None)


def circ_fc_sgd_step(w_hat, x, dy, lr, p, q, k, need_dx=False, dx=None, workspace=None):
    """Updates the blob in place by -lr * dL/dw; returns dx [batch][q*k] (from the old weights) or None."""
    batch = dy.shape[0]
    if need_dx and dx is None:
        dx = torch.empty(batch, q * k, dtype=torch.float32, device=dy.device)
    if workspace is None:
        workspace = torch.empty(max(1, circ_fc_workspace_bytes(p, q, k, batch, True)), dtype=torch.uint8,
                                device=dy.device)
    _check(lib().circ_fc_sgd_step(_ptr(w_hat), _f32(x), _f32(dy), _f32(dx if need_dx else None), float(lr), p, q, k,
                                  batch, _ptr(workspace), workspace.numel(), _stream()), "circ_fc_sgd_step")
    return dx if need_dx else None


def circ_conv_sgd_step(w_hat, x, dy, lr, C_in, H, W, r, stride, pad, k, need_dx=False, dx=None, workspace=None):
    """CONV counterpart of circ_fc_sgd_step; dy: NCHW [N][C_out][Ho][Wo]."""
    N, C_out = dy.shape[0], dy.shape[1]
    if need_dx and dx is None:
        dx = torch.empty(N, C_in, H, W, dtype=torch.float32, device=dy.device)
    if workspace is None:
        nb = circ_conv_backward_workspace_bytes(N, C_in, C_out, H, W, r, stride, pad, k)
        workspace = torch.empty(max(1, nb), dtype=torch.uint8, device=dy.device)
    _check(lib().circ_conv_sgd_step(_ptr(w_hat), _f32(x), _f32(dy), _f32(dx if need_dx else None), float(lr), N, C_in,
                                    C_out, H, W, r, stride, pad, k, _ptr(workspace), workspace.numel(), _stream()),
           "circ_conv_sgd_step")
    return dx if need_dx else None


def circ_export_weights(w_hat, n_grids, p, q, k, w=None):
    """Block vectors [n_grids][p][q][k] recovered from a spectra blob."""
    if w is None:
        w = torch.empty(n_grids, p, q, k, dtype=torch.float32, device=w_hat.device)
    _check(lib().circ_export_weights(_ptr(w_hat), n_grids, p, q, k, _f32(w), _stream()), "circ_export_weights")
    return w


def _half_suffix(dtype) -> str:
    assert dtype in (torch.float16, torch.bfloat16)
    return "f16" if dtype == torch.float16 else "bf16"


def circ_precompute_spectra_f16(w: torch.Tensor, w_hat: torch.Tensor | None = None, dtype=torch.float16) -> torch.Tensor:
    """w: device fp32 [p][q][k] -> opaque 16-bit spectra blob (uint8 tensor) in `dtype` (fp16 or bf16)."""
    assert w.is_cuda and w.dtype == torch.float32 and w.is_contiguous() and w.dim() == 3
    p, q, k = w.shape
    sfx = _half_suffix(dtype)
    nbytes = getattr(lib(), f"circ_spectra_bytes_{sfx}")(p, q, k)
    if nbytes == 0:
        raise CircError(CIRC_EINVAL, f"circ_spectra_bytes_{sfx}")
    if w_hat is None:
        w_hat = torch.empty(nbytes, dtype=torch.uint8, device=w.device)
    _check(getattr(lib(), f"circ_precompute_spectra_{sfx}")(_f32(w), p, q, k, _ptr(w_hat), _stream()),
           f"circ_precompute_spectra_{sfx}")
    return w_hat


def circ_fc_workspace_bytes_f16(p, q, k, batch) -> int:
    return lib().circ_fc_workspace_bytes_f16(p, q, k, batch)      # the same for both 16-bit formats


def circ_fc_forward_f16(w_hat, x, bias, y, p, q, k, epilogue=EPI_NONE, workspace=None):
    """x: fp16 or bf16 [batch][q*k] -> y of the same type [batch][p*k] (allocated if None); bias fp32.
    The blob must come from circ_precompute_spectra_f16 with the same dtype.  Returns y."""
    sfx = _half_suffix(x.dtype)
    assert x.is_contiguous()
    batch = x.shape[0]
    if y is None:
        y = torch.empty(batch, p * k, dtype=x.dtype, device=x.device)
    if workspace is None:
        workspace = torch.empty(max(1, circ_fc_workspace_bytes_f16(p, q, k, batch)), dtype=torch.uint8, device=x.device)
    _check(getattr(lib(), f"circ_fc_forward_{sfx}")(_ptr(w_hat), _ptr(x), _f32(bias), _ptr(y, x.dtype), p, q, k, batch, epilogue,
                                                    _ptr(workspace), workspace.numel(), _stream()), f"circ_fc_forward_{sfx}")
    return y


def circ_fc_backward_workspace_bytes_f16(p, q, k, batch) -> int:
    return lib().circ_fc_backward_workspace_bytes_f16(p, q, k, batch)      # the same for both 16-bit formats


def circ_fc_backward_f16(w_hat, x, dy, p, q, k, need_dx=True, need_dw=True, dx=None, dw=None, workspace=None):
    """dy (and x when need_dw): fp16 or bf16.  Returns (dx of the same type or None, dw fp32 [p][q][k] or None)."""
    sfx = _half_suffix(dy.dtype)
    assert dy.is_contiguous() and (x is None or (x.is_contiguous() and x.dtype == dy.dtype))
    batch = dy.shape[0]
    if need_dx and dx is None:
        dx = torch.empty(batch, q * k, dtype=dy.dtype, device=dy.device)
    if need_dw and dw is None:
        dw = torch.empty(p, q, k, dtype=torch.float32, device=dy.device)
    if workspace is None:
        workspace = torch.empty(max(1, circ_fc_backward_workspace_bytes_f16(p, q, k, batch)), dtype=torch.uint8, device=dy.device)
    _check(getattr(lib(), f"circ_fc_backward_{sfx}")(_ptr(w_hat), _ptr(x), _ptr(dy), _ptr(dx, dy.dtype) if need_dx else None,
                                                     _f32(dw) if need_dw else None, p, q, k, batch, _ptr(workspace),
                                                     workspace.numel(), _stream()), f"circ_fc_backward_{sfx}")
    return (dx if need_dx else None), (dw if need_dw else None)


def circ_conv_forward_f16(w_hat, x, bias, y, C_out, r, stride, pad, k, epilogue=EPI_NONE, workspace=None):
    """x: fp16 or bf16 NCHW -> y of the same type (allocated if None); w_hat from circ_precompute_spectra, bias fp32."""
    sfx = _half_suffix(x.dtype)
    assert x.is_contiguous()
    N, C_in, H, W = x.shape
    Ho, Wo = (H + 2 * pad - r) // stride + 1, (W + 2 * pad - r) // stride + 1
    if y is None:
        y = torch.empty(N, C_out, Ho, Wo, dtype=x.dtype, device=x.device)
    if workspace is None:
        nb = circ_conv_workspace_bytes(N, C_in, C_out, H, W, r, stride, pad, k)
        workspace = torch.empty(max(1, nb), dtype=torch.uint8, device=x.device)
    _check(getattr(lib(), f"circ_conv_forward_{sfx}")(_ptr(w_hat), _ptr(x), _f32(bias), _ptr(y, x.dtype), N, C_in, C_out, H, W, r, stride,
                                                      pad, k, epilogue, _ptr(workspace), workspace.numel(), _stream()),
           f"circ_conv_forward_{sfx}")
    return y


def circ_conv_backward_f16(w_hat, x, dy, C_in, H, W, r, stride, pad, k, need_dx=True, need_dw=True, dx=None, dw=None,
                           workspace=None):
    """dy (and x when need_dw): fp16 or bf16 NCHW.  Returns (dx of the same type or None, dw fp32 [r][r][p][q][k] or None)."""
    sfx = _half_suffix(dy.dtype)
    assert dy.is_contiguous() and (x is None or (x.is_contiguous() and x.dtype == dy.dtype))
    N, C_out = dy.shape[0], dy.shape[1]
    if need_dx and dx is None:
        dx = torch.empty(N, C_in, H, W, dtype=dy.dtype, device=dy.device)
    if need_dw and dw is None:
        dw = torch.empty(r, r, C_out // k, C_in // k, k, dtype=torch.float32, device=dy.device)
    if workspace is None:
        nb = circ_conv_backward_workspace_bytes(N, C_in, C_out, H, W, r, stride, pad, k)
        workspace = torch.empty(max(1, nb), dtype=torch.uint8, device=dy.device)
    _check(getattr(lib(), f"circ_conv_backward_{sfx}")(_ptr(w_hat), _ptr(x), _ptr(dy), _ptr(dx, dy.dtype) if need_dx else None,
                                                       _f32(dw) if need_dw else None, N, C_in, C_out, H, W, r, stride, pad, k,
                                                       _ptr(workspace), workspace.numel(), _stream()), f"circ_conv_backward_{sfx}")
    return (dx if need_dx else None), (dw if need_dw else None)


def circ_bias_grad(dy, db=None):
    """dy: [batch][m] (FC) or NCHW (CONV) -> db: [m] or [C]."""
    channels = dy.shape[1]
    outer = dy.shape[0]
    inner = int(dy.numel() // (outer * channels))
    if db is None:
        db = torch.empty(channels, dtype=torch.float32, device=dy.device)
    _check(lib().circ_bias_grad(_f32(dy), _f32(db), outer, channels, inner, _stream()), "circ_bias_grad")
    return db



def circ_maxpool_forward(x, window, stride, y=None):
    """x: NCHW fp32 -> y: NCHW [(H - window) // stride + 1][(W - window) // stride + 1] (allocated if None)."""
    N, C, H, W = x.shape
    if y is None:
        y = torch.empty(N, C, (H - window) // stride + 1, (W - window) // stride + 1, dtype=torch.float32, device=x.device)
    _check(lib().circ_maxpool_forward(_f32(x), _f32(y), N, C, H, W, window, stride, _stream()), "circ_maxpool_forward")
    return y


def fc_layer(w_hat, bias, p, q, k, epilogue=EPI_NONE) -> CircLayer:
    return CircLayer(kind=LAYER_FC, epilogue=epilogue, w_hat=_ptr(w_hat), bias=_f32(bias), k=k, p=p, q=q)


def conv_layer(w_hat, bias, C_in, C_out, H, W, r, stride, pad, k, epilogue=EPI_NONE) -> CircLayer:
    return CircLayer(kind=LAYER_CONV, epilogue=epilogue, w_hat=_ptr(w_hat), bias=_f32(bias), k=k, C_in=C_in, C_out=C_out,
                     H=H, W=W, r=r, stride=stride, pad=pad)


def maxpool_layer(C, H, W, window, stride) -> CircLayer:
    return CircLayer(kind=LAYER_MAXPOOL, C_in=C, H=H, W=W, r=window, stride=stride)


def circ_chain_workspace_bytes(layers, batch) -> int:
    arr = (CircLayer * len(layers))(*layers)
    return lib().circ_chain_workspace_bytes(arr, len(layers), batch)


def circ_chain_forward(layers, x, y, workspace=None):
    """layers: list of CircLayer (the tensors they point to must stay alive); x: [batch][...] device fp32;
    y: output of the last layer, preallocated.  Returns y."""
    batch = x.shape[0]
    arr = (CircLayer * len(layers))(*layers)
    if workspace is None:
        nb = lib().circ_chain_workspace_bytes(arr, len(layers), batch)
        if nb == 0:
            raise CircError(CIRC_EINVAL, "circ_chain_workspace_bytes")
        workspace = torch.empty(nb, dtype=torch.uint8, device=x.device)
    _check(lib().circ_chain_forward(arr, len(layers), _f32(x), _f32(y), batch, _ptr(workspace), workspace.numel(), _stream()),
           "circ_chain_forward")
    return y
