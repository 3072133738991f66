"""ctypes binding of libkst.so: same names as include/kst.h, marshalling only.

PyTorch supplies device memory (``tensor.data_ptr()``) and the stream
(``torch.cuda.current_stream()``); every step of the path runs in the HIP
library.  There is no fallback: if the library has not been built, or a call
returns a non-zero status, this raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

KST_F32, KST_BF16, KST_F16 = 0, 1, 2
KST_PATH_AUTO, KST_PATH_DIRECT, KST_PATH_IGEMM, KST_PATH_IGEMM_EVEN, KST_PATH_IGEMM_PASSES = 0, 1, 2, 3, 4
KST_ACT_NONE, KST_ACT_RELU, KST_ACT_TANH = 0, 1, 2
KST_OK = 0
KST_STATIC_SCRATCH_BYTES = 64 << 20

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libkst.so")
_lib = None

_c_int, _c_size_t, _c_void_p = ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p

# name -> (restype, argtypes): the whole exported surface of include/kst.h
SIGNATURES = {
    "kst_version": (_c_int, []),
    "kst_status_string": (ctypes.c_char_p, [_c_int]),
    "kst_out_size": (_c_int, [_c_int, _c_int]),
    "kst_subkernel_shape": (_c_int, [_c_int, _c_int, ctypes.POINTER(_c_int), ctypes.POINTER(_c_int)]),
    "kst_segregated_elems": (_c_size_t, [_c_int, _c_int, _c_int, _c_int]),
    "kst_segregated_offset": (_c_size_t, [_c_int, _c_int, _c_int, _c_int, _c_int]),
    "kst_segregate_weights": (_c_int, [_c_void_p, _c_void_p, _c_int, _c_int, _c_int, _c_int, _c_void_p]),
    "kst_workspace_bytes": (_c_size_t, [_c_int] * 7),
    "kst_forward_seg": (_c_int, [_c_void_p, _c_void_p, _c_void_p, _c_void_p, _c_size_t] + [_c_int] * 7 + [_c_void_p]),
    "kst_forward": (_c_int, [_c_void_p, _c_void_p, _c_void_p] + [_c_int] * 6 + [_c_void_p]),
    "kst_forward_seg_static": (_c_int, [_c_void_p, _c_void_p, _c_void_p] + [_c_int] * 7 + [_c_void_p]),
    "kst_forward_zero_insert": (_c_int, [_c_void_p] * 4 + [_c_int] * 6 + [_c_void_p]),
    "kst_out_size_padded": (_c_int, [_c_int] * 3),
    "kst_workspace_bytes_padded": (_c_size_t, [_c_int] * 8),
    "kst_forward_seg_padded": (_c_int, [_c_void_p, _c_void_p, _c_void_p, _c_void_p, _c_size_t] + [_c_int] * 8 + [_c_void_p]),
    "kst_forward_seg_epilogue": (_c_int, [_c_void_p, _c_void_p, _c_void_p, _c_void_p, _c_void_p, _c_size_t] + [_c_int] * 9
                                 + [_c_void_p]),
    "kst_forward_padded": (_c_int, [_c_void_p, _c_void_p, _c_void_p] + [_c_int] * 7 + [_c_void_p]),
    "kst_backward_input_workspace_bytes": (_c_size_t, [_c_int] * 7),
    "kst_backward_weight_workspace_bytes": (_c_size_t, [_c_int] * 7),
    "kst_backward_input": (_c_int, [_c_void_p, _c_void_p, _c_void_p, _c_void_p, _c_size_t] + [_c_int] * 7 + [_c_void_p]),
    "kst_backward_weight": (_c_int, [_c_void_p, _c_void_p, _c_void_p, _c_void_p, _c_size_t] + [_c_int] * 7 + [_c_void_p]),
    "kst_yardstick_mfma_sink_elems": (_c_size_t, []),
    "kst_yardstick_mfma_flops": (ctypes.c_double, [_c_int, _c_int]),
    "kst_yardstick_mfma": (_c_int, [_c_int, _c_int, _c_void_p, _c_size_t, _c_void_p]),
    "kst_yardstick_copy": (_c_int, [_c_void_p, _c_void_p, _c_size_t, _c_void_p]),
}


class KstError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().kst_status_string(status).decode()
        super().__init__("%s: kst status %d (%s)" % (where, status, msg))


def lib():
    """The loaded libkst.so.  Raises if it has not been built (python -m paper_2209_03704_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libkst.so is not built: run `python -m paper_2209_03704_amd.build` "
                               "(there is no fallback path)")
        l = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype = res
            fn.argtypes = args
        _lib = l
    return _lib


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return KST_F32
    if t.dtype == torch.bfloat16:
        return KST_BF16
    if t.dtype == torch.float16:
        return KST_F16
    raise TypeError("kst supports float32, bfloat16 and float16 operands, got %s" % t.dtype)


def _dev(t: torch.Tensor, what: str) -> int:
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU" % what)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % what)
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dims(x: torch.Tensor, n: int, Cout: int):
    B, Cin, N, N2 = x.shape
    if N != N2:
        raise ValueError("square maps only")
    return B, Cin, Cout, N, n


def kst_version() -> int:
    return lib().kst_version()


def kst_status_string(status: int) -> str:
    return lib().kst_status_string(status).decode()


def kst_out_size(N: int, n: int) -> int:
    return lib().kst_out_size(N, n)


def kst_subkernel_shape(n: int, p: int):
    ta, tb = _c_int(), _c_int()
    st = lib().kst_subkernel_shape(n, p, ctypes.byref(ta), ctypes.byref(tb))
    if st != KST_OK:
        raise KstError(st, "kst_subkernel_shape")
    return ta.value, tb.value


def kst_segregated_elems(Cin: int, Cout: int, n: int, dtype: int) -> int:
    return lib().kst_segregated_elems(Cin, Cout, n, dtype)


def kst_segregated_offset(Cin: int, Cout: int, n: int, p: int, dtype: int) -> int:
    return lib().kst_segregated_offset(Cin, Cout, n, p, dtype)


def kst_workspace_bytes(B, Cin, Cout, N, n, dtype: int, path: int = KST_PATH_AUTO) -> int:
    return lib().kst_workspace_bytes(B, Cin, Cout, N, n, dtype, path)


def kst_segregate_weights(w: torch.Tensor, w_seg: torch.Tensor | None = None) -> torch.Tensor:
    """w[Cout][Cin][n][n] (device) -> segregated buffer (device, same dtype)."""
    Cout, Cin, n, n2 = w.shape
    if n != n2:
        raise ValueError("square kernels only")
    dt = _dtype_code(w)
    elems = kst_segregated_elems(Cin, Cout, n, dt)
    if elems == 0:
        raise KstError(2, "kst_segregated_elems")
    if w_seg is None:
        w_seg = torch.empty(elems, dtype=w.dtype, device=w.device)
    elif w_seg.numel() < elems or w_seg.dtype != w.dtype:
        raise ValueError("w_seg too small or of the wrong dtype")
    st = lib().kst_segregate_weights(_dev(w, "w"), _dev(w_seg, "w_seg"), Cin, Cout, n, dt, _stream())
    if st != KST_OK:
        raise KstError(st, "kst_segregate_weights")
    return w_seg


def kst_forward_seg(x: torch.Tensor, w_seg: torch.Tensor, Cout: int, n: int, out: torch.Tensor | None = None,
                    ws: torch.Tensor | None = None, path: int = KST_PATH_AUTO) -> torch.Tensor:
    B, Cin, Cout, N, n = _dims(x, n, Cout)
    dt = _dtype_code(x)
    if w_seg.dtype != x.dtype:
        raise TypeError("x and w_seg must share a dtype")
    M = 2 * N - n
    if out is None:
        out = torch.empty((B, Cout, max(M, 0), max(M, 0)), dtype=torch.float32, device=x.device)
    elif out.dtype != torch.float32:
        raise TypeError("out must be float32")
    need = kst_workspace_bytes(B, Cin, Cout, N, n, dt, path)
    if ws is None and need:
        ws = torch.empty(need, dtype=torch.uint8, device=x.device)
    ws_ptr = _dev(ws, "ws") if ws is not None else None
    ws_bytes = ws.numel() * ws.element_size() if ws is not None else 0
    st = lib().kst_forward_seg(_dev(x, "x"), _dev(w_seg, "w_seg"), _dev(out, "out"), ws_ptr, ws_bytes,
                               B, Cin, Cout, N, n, dt, path, _stream())
    if st != KST_OK:
        raise KstError(st, "kst_forward_seg")
    return out


def kst_forward_seg_static(x: torch.Tensor, w_seg: torch.Tensor, Cout: int, n: int, out: torch.Tensor,
                           path: int = KST_PATH_AUTO) -> torch.Tensor:
    """kst_forward_seg with the library's own fixed workspace; `out` is the caller's (nothing is allocated)."""
    B, Cin, Cout, N, n = _dims(x, n, Cout)
    if w_seg.dtype != x.dtype:
        raise TypeError("x and w_seg must share a dtype")
    if out.dtype != torch.float32:
        raise TypeError("out must be float32")
    st = lib().kst_forward_seg_static(_dev(x, "x"), _dev(w_seg, "w_seg"), _dev(out, "out"), B, Cin, Cout, N, n,
                                      _dtype_code(x), path, _stream())
    if st != KST_OK:
        raise KstError(st, "kst_forward_seg_static")
    return out


def kst_forward(x: torch.Tensor, w: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    Cout, Cin_w, n, _ = w.shape
    B, Cin, Cout, N, n = _dims(x, n, Cout)
    if Cin_w != Cin or w.dtype != x.dtype:
        raise ValueError("x and w disagree on Cin or dtype")
    M = 2 * N - n
    if out is None:
        out = torch.empty((B, Cout, max(M, 0), max(M, 0)), dtype=torch.float32, device=x.device)
    st = lib().kst_forward(_dev(x, "x"), _dev(w, "w"), _dev(out, "out"), B, Cin, Cout, N, n,
                           _dtype_code(x), _stream())
    if st != KST_OK:
        raise KstError(st, "kst_forward")
    return out


def kst_forward_zero_insert(x: torch.Tensor, w: torch.Tensor, U: torch.Tensor | None = None,
                            out: torch.Tensor | None = None) -> torch.Tensor:
    Cout, Cin_w, n, _ = w.shape
    B, Cin, Cout, N, n = _dims(x, n, Cout)
    if Cin_w != Cin or w.dtype != x.dtype:
        raise ValueError("x and w disagree on Cin or dtype")
    M, S = 2 * N - n, 2 * N - 1
    if U is None:
        U = torch.empty((B, Cin, S, S), dtype=x.dtype, device=x.device)
    if out is None:
        out = torch.empty((B, Cout, max(M, 0), max(M, 0)), dtype=torch.float32, device=x.device)
    st = lib().kst_forward_zero_insert(_dev(x, "x"), _dev(w, "w"), _dev(U, "U"), _dev(out, "out"),
                                       B, Cin, Cout, N, n, _dtype_code(x), _stream())
    if st != KST_OK:
        raise KstError(st, "kst_forward_zero_insert")
    return out


def kst_out_size_padded(N: int, n: int, P: int) -> int:
    return lib().kst_out_size_padded(N, n, P)


def kst_workspace_bytes_padded(B, Cin, Cout, N, n, P, dtype: int, path: int = KST_PATH_AUTO) -> int:
    return lib().kst_workspace_bytes_padded(B, Cin, Cout, N, n, P, dtype, path)


def kst_forward_seg_padded(x: torch.Tensor, w_seg: torch.Tensor, Cout: int, n: int, P: int,
                           out: torch.Tensor | None = None, ws: torch.Tensor | None = None,
                           path: int = KST_PATH_AUTO) -> torch.Tensor:
    B, Cin, Cout, N, n = _dims(x, n, Cout)
    dt = _dtype_code(x)
    if w_seg.dtype != x.dtype:
        raise TypeError("x and w_seg must share a dtype")
    M = 2 * N + 2 * P - n
    if out is None:
        out = torch.empty((B, Cout, max(M, 0), max(M, 0)), dtype=torch.float32, device=x.device)
    elif out.dtype != torch.float32:
        raise TypeError("out must be float32")
    need = kst_workspace_bytes_padded(B, Cin, Cout, N, n, P, dt, path)
    if ws is None and need:
        ws = torch.empty(need, dtype=torch.uint8, device=x.device)
    ws_ptr = _dev(ws, "ws") if ws is not None else None
    ws_bytes = ws.numel() * ws.element_size() if ws is not None else 0
    st = lib().kst_forward_seg_padded(_dev(x, "x"), _dev(w_seg, "w_seg"), _dev(out, "out"), ws_ptr, ws_bytes,
                                      B, Cin, Cout, N, n, P, dt, path, _stream())
    if st != KST_OK:
        raise KstError(st, "kst_forward_seg_padded")
    return out


def kst_forward_seg_epilogue(x: torch.Tensor, w_seg: torch.Tensor, Cout: int, n: int, bias: torch.Tensor | None = None,
                             act: int = KST_ACT_NONE, P: int = 0, out: torch.Tensor | None = None,
                             ws: torch.Tensor | None = None, path: int = KST_PATH_AUTO) -> torch.Tensor:
    """act(transpose convolution + bias[co]); bias: Cout float32 values on the device, or None."""
    B, Cin, Cout, N, n = _dims(x, n, Cout)
    dt = _dtype_code(x)
    if w_seg.dtype != x.dtype:
        raise TypeError("x and w_seg must share a dtype")
    if bias is not None and (bias.dtype != torch.float32 or bias.numel() != Cout or not bias.is_contiguous()):
        raise TypeError("bias must hold Cout contiguous float32 values")
    M = 2 * N + 2 * P - n
    if out is None:
        out = torch.empty((B, Cout, max(M, 0), max(M, 0)), dtype=torch.float32, device=x.device)
    elif out.dtype != torch.float32:
        raise TypeError("out must be float32")
    need = kst_workspace_bytes_padded(B, Cin, Cout, N, n, P, dt, path)
    if ws is None and need:
        ws = torch.empty(need, dtype=torch.uint8, device=x.device)
    ws_ptr = _dev(ws, "ws") if ws is not None else None
    ws_bytes = ws.numel() * ws.element_size() if ws is not None else 0
    st = lib().kst_forward_seg_epilogue(_dev(x, "x"), _dev(w_seg, "w_seg"), _dev(bias, "bias") if bias is not None else None,
                                        _dev(out, "out"), ws_ptr, ws_bytes, B, Cin, Cout, N, n, P, dt, act, path,
                                        _stream())
    if st != KST_OK:
        raise KstError(st, "kst_forward_seg_epilogue")
    return out


def kst_forward_padded(x: torch.Tensor, w: torch.Tensor, P: int, out: torch.Tensor | None = None) -> torch.Tensor:
    Cout, Cin_w, n, _ = w.shape
    B, Cin, Cout, N, n = _dims(x, n, Cout)
    if Cin_w != Cin or w.dtype != x.dtype:
        raise ValueError("x and w disagree on Cin or dtype")
    M = 2 * N + 2 * P - n
    if out is None:
        out = torch.empty((B, Cout, max(M, 0), max(M, 0)), dtype=torch.float32, device=x.device)
    st = lib().kst_forward_padded(_dev(x, "x"), _dev(w, "w"), _dev(out, "out"), B, Cin, Cout, N, n, P,
                                  _dtype_code(x), _stream())
    if st != KST_OK:
        raise KstError(st, "kst_forward_padded")
    return out


def _ws(need: int, ws, device):
    if ws is None and need:
        ws = torch.empty(need, dtype=torch.uint8, device=device)
    ptr = _dev(ws, "ws") if ws is not None else None
    size = ws.numel() * ws.element_size() if ws is not None else 0
    return ws, ptr, size


def kst_backward_input(g: torch.Tensor, w: torch.Tensor, N: int, P: int = 0, din: torch.Tensor | None = None,
                       ws: torch.Tensor | None = None) -> torch.Tensor:
    """d(loss)/d(in) [B][Cin][N][N] (fp32) from g = d(loss)/d(out) (fp32) and the un-segregated w."""
    Cout, Cin, n, n2 = w.shape
    B, Cout_g, M, M2 = g.shape
    if n != n2 or M != M2 or Cout_g != Cout or g.dtype != torch.float32:
        raise ValueError("g must be float32 [B][Cout][M][M] matching w")
    if M != 2 * N + 2 * P - n:
        raise ValueError("g's edge %d is not 2N + 2P - n" % M)
    dt = _dtype_code(w)
    if din is None:
        din = torch.empty((B, Cin, N, N), dtype=torch.float32, device=g.device)
    need = lib().kst_backward_input_workspace_bytes(B, Cin, Cout, N, n, P, dt)
    ws, ws_ptr, ws_bytes = _ws(need, ws, g.device)
    st = lib().kst_backward_input(_dev(g, "g"), _dev(w, "w"), _dev(din, "din"), ws_ptr, ws_bytes,
                                  B, Cin, Cout, N, n, P, dt, _stream())
    if st != KST_OK:
        raise KstError(st, "kst_backward_input")
    return din


def kst_backward_weight(x: torch.Tensor, g: torch.Tensor, n: int, P: int = 0, dw: torch.Tensor | None = None,
                        ws: torch.Tensor | None = None) -> torch.Tensor:
    """d(loss)/d(w) [Cout][Cin][n][n] (fp32) from x and g = d(loss)/d(out) (fp32)."""
    B, Cin, N, N2 = x.shape
    B2, Cout, M, M2 = g.shape
    if N != N2 or M != M2 or B != B2 or g.dtype != torch.float32:
        raise ValueError("g must be float32 [B][Cout][M][M] matching x")
    if M != 2 * N + 2 * P - n:
        raise ValueError("g's edge %d is not 2N + 2P - n" % M)
    dt = _dtype_code(x)
    if dw is None:
        dw = torch.empty((Cout, Cin, n, n), dtype=torch.float32, device=x.device)
    need = lib().kst_backward_weight_workspace_bytes(B, Cin, Cout, N, n, P, dt)
    ws, ws_ptr, ws_bytes = _ws(need, ws, x.device)
    st = lib().kst_backward_weight(_dev(x, "x"), _dev(g, "g"), _dev(dw, "dw"), ws_ptr, ws_bytes,
                                   B, Cin, Cout, N, n, P, dt, _stream())
    if st != KST_OK:
        raise KstError(st, "kst_backward_weight")
    return dw


def kst_backward_input_workspace_bytes(B, Cin, Cout, N, n, P, dtype: int) -> int:
    return lib().kst_backward_input_workspace_bytes(B, Cin, Cout, N, n, P, dtype)


def kst_backward_weight_workspace_bytes(B, Cin, Cout, N, n, P, dtype: int) -> int:
    return lib().kst_backward_weight_workspace_bytes(B, Cin, Cout, N, n, P, dtype)


def kst_yardstick_mfma_sink_elems() -> int:
    return lib().kst_yardstick_mfma_sink_elems()


def kst_yardstick_mfma_flops(dtype: int, iters: int) -> float:
    return lib().kst_yardstick_mfma_flops(dtype, iters)


def kst_yardstick_mfma(dtype: int, iters: int, sink: torch.Tensor | None = None) -> torch.Tensor:
    """One launch of the matrix-core-only loop; returns the sink tensor (values carry no meaning)."""
    need = lib().kst_yardstick_mfma_sink_elems()
    if sink is None:
        sink = torch.empty(need, dtype=torch.float32, device="cuda")
    if sink.dtype != torch.float32:
        raise ValueError("sink must be float32")
    st = lib().kst_yardstick_mfma(dtype, iters, _dev(sink, "sink"), sink.numel(), _stream())
    if st != KST_OK:
        raise KstError(st, "kst_yardstick_mfma")
    return sink


def kst_yardstick_copy(src: torch.Tensor, dst: torch.Tensor) -> torch.Tensor:
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("src and dst differ in size")
    st = lib().kst_yardstick_copy(_dev(src, "src"), _dev(dst, "dst"), nbytes, _stream())
    if st != KST_OK:
        raise KstError(st, "kst_yardstick_copy")
    return dst
