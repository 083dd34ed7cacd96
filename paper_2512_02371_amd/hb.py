"""ctypes binding of the C-ABI library declared in ``include/hb.h``.

Argument marshalling only: every function takes torch CUDA tensors (used purely
as device memory), pulls out pointers, shapes and pitches, and calls the entry
point of the same name on torch's current stream.  There is no fallback: if the
library is missing, ``load()`` raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhb.so")

HB_OK = 0
HB_ERR_INVALID_ARG = 1
HB_ERR_UNSUPPORTED = 2
HB_ERR_WORKSPACE = 3
HB_ERR_HIP = 4
HB_MAX_TAPS = 64            # per axis, hb_sepblur
HB_MAX_TAPS_FIR1D = 256     # hb_fir1d
HB_MAX_TAPS_CONV2D = 32     # per axis, hb_conv2d

# every symbol include/hb.h declares
SYMBOLS = [
    "hb_status_string",
    "hb_fir1d", "hb_fir1d_valu",
    "hb_conv2d", "hb_conv2d_valu",
    "hb_down2", "hb_down2_valu", "hb_up2", "hb_up2_valu",
    "hb_resize_workspace_size", "hb_resize", "hb_resize_valu", "hb_lanczos3_band", "hb_lanczos3_matrix",
    "hb_iir2_workspace_size", "hb_iir2_abs_gain", "hb_iir2", "hb_iir2_valu",
    "hb_dct_denoise_workspace_size", "hb_dct_denoise", "hb_dct_denoise_valu",
    "hb_sepblur", "hb_sepblur_valu",
    "hb_sat2d_workspace_size", "hb_sat2d", "hb_sat2d_valu", "hb_sat2d_noalloc", "hb_sat2d_set_wait_limit",
    "hb_conv3x3", "hb_conv3x3_valu",
    "hb_pyr_level", "hb_pyr_level_valu",
    "hb_copy_f16_f32", "hb_mfma_probe",
]

_lib = None


class HbError(RuntimeError):
    def __init__(self, fn: str, code: int):
        self.code = code
        super().__init__(f"{fn} failed: {status_string(code)} ({code})")


def load() -> ctypes.CDLL:
    """Load libhb.so (built by ``__graft_entry__.build()``); raise if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`. "
            "There is no CPU fallback.")
    # torch first: it ships its own copy of the HIP runtime, and libhb.so must bind to that copy (the
    # one that owns torch's streams and allocations), not load a second runtime from the system path
    import torch  # noqa: F401
    L = ctypes.CDLL(LIB_PATH)
    vp, I, I64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    L.hb_status_string.argtypes = [I]
    L.hb_status_string.restype = ctypes.c_char_p
    fir = [vp, vp, I, I, I64, I64, vp, I, I, vp]
    sep = [vp, vp, I, I, I64, I64, vp, I, I, vp, I, I, vp]
    c2d = [vp, vp, I, I, I64, I64, vp, I, I, I, I, vp]
    sat = [vp, vp, I, I, I64, I64, vp, ctypes.c_size_t, vp]
    conv = [vp, vp, vp, I, I, I, I, I, vp]
    pyr = [vp, vp, vp, I, I, I64, I64, I64, vp]
    for name, sig in (("hb_fir1d", fir), ("hb_fir1d_valu", fir), ("hb_conv2d", c2d), ("hb_conv2d_valu", c2d),
                      ("hb_down2", c2d), ("hb_down2_valu", c2d), ("hb_up2", c2d), ("hb_up2_valu", c2d), ("hb_sepblur", sep), ("hb_sepblur_valu", sep),
                      ("hb_sat2d", sat), ("hb_sat2d_valu", sat), ("hb_conv3x3", conv), ("hb_conv3x3_valu", conv),
                      ("hb_pyr_level", pyr), ("hb_pyr_level_valu", pyr),
                      ("hb_copy_f16_f32", [vp, vp, I64, vp]), ("hb_mfma_probe", [I, vp, vp, vp, vp])):
        f = getattr(L, name)
        f.argtypes = sig
        f.restype = I
    rsz = [vp, vp, vp, ctypes.c_size_t, I, I, I, I, I, I64, I64, I64, I64, vp, vp, I, vp, vp, I, vp]
    for name in ("hb_resize", "hb_resize_valu"):
        getattr(L, name).argtypes = rsz
        getattr(L, name).restype = I
    L.hb_resize_workspace_size.argtypes = [I, I, I]
    L.hb_resize_workspace_size.restype = ctypes.c_size_t
    L.hb_lanczos3_band.argtypes = [I, I]
    L.hb_lanczos3_band.restype = I
    L.hb_lanczos3_matrix.argtypes = [I, I, vp, vp]
    L.hb_lanczos3_matrix.restype = I
    iir = [vp, vp, I, I64, I64, I64, ctypes.c_float, ctypes.c_float, vp, ctypes.c_size_t, vp]
    for name in ("hb_iir2", "hb_iir2_valu"):
        getattr(L, name).argtypes = iir
        getattr(L, name).restype = I
    L.hb_iir2_workspace_size.argtypes = [I, I64]
    L.hb_iir2_workspace_size.restype = ctypes.c_size_t
    L.hb_iir2_abs_gain.argtypes = [ctypes.c_float, ctypes.c_float, I64]
    L.hb_iir2_abs_gain.restype = ctypes.c_double
    dct = [vp, vp, I, I, I, I64, I64, I64, I64, ctypes.c_float, vp, ctypes.c_size_t, vp]
    for name in ("hb_dct_denoise", "hb_dct_denoise_valu"):
        getattr(L, name).argtypes = dct
        getattr(L, name).restype = I
    L.hb_dct_denoise_workspace_size.argtypes = [I, I, I]
    L.hb_dct_denoise_workspace_size.restype = ctypes.c_size_t
    L.hb_sat2d_noalloc.argtypes = [vp, vp, I, I, I64, I64, vp]
    L.hb_sat2d_noalloc.restype = I
    L.hb_sat2d_set_wait_limit.argtypes = [I]
    L.hb_sat2d_set_wait_limit.restype = I
    L.hb_sat2d_workspace_size.argtypes = [I, I]
    L.hb_sat2d_workspace_size.restype = ctypes.c_size_t
    _lib = L
    return L


def status_string(code: int) -> str:
    return load().hb_status_string(int(code)).decode()


hb_status_string = status_string          # the entry point's own name


def _check(fn: str, code: int) -> None:
    if code != HB_OK:
        raise HbError(fn, code)


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _taps(t):
    """Host fp16 bit patterns -> (keep-alive array, pointer, count)."""
    a = np.ascontiguousarray(t)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    a = np.ascontiguousarray(a, dtype=np.uint16)
    return a, a.ctypes.data_as(ctypes.c_void_p), int(a.size)


def _img2d(t, dtype):
    import torch
    assert t.is_cuda and t.dim() == 2 and t.dtype == dtype and t.stride(1) == 1, "row-major 2-D CUDA tensor expected"
    return ctypes.c_void_p(t.data_ptr()), int(t.shape[0]), int(t.shape[1]), int(t.stride(0))


def _fir(name, inp, out, taps, anchor):
    import torch
    pi, H, W, ip = _img2d(inp, torch.float16)
    po, Ho, Wo, op = _img2d(out, torch.float32)
    assert (H, W) == (Ho, Wo)
    keep, pt, n = _taps(taps)
    _check(name, getattr(load(), name)(pi, po, H, W, ip, op, pt, n, int(anchor), _stream()))
    return out


def hb_fir1d(inp, out, taps, anchor):
    return _fir("hb_fir1d", inp, out, taps, anchor)


def hb_fir1d_valu(inp, out, taps, anchor):
    return _fir("hb_fir1d_valu", inp, out, taps, anchor)


def _conv2d(name, inp, out, taps2d, anchor_y, anchor_x, shape=lambda H, W: (H, W)):
    import torch
    pi, H, W, ip = _img2d(inp, torch.float16)
    po, Ho, Wo, op = _img2d(out, torch.float32)
    assert shape(H, W) == (Ho, Wo), "output shape"
    k = np.asarray(taps2d)
    assert k.ndim == 2, "kh x kw tap array expected"
    keep, pt, n = _taps(k)
    _check(name, getattr(load(), name)(pi, po, H, W, ip, op, pt, int(k.shape[0]), int(k.shape[1]),
                                        int(anchor_y), int(anchor_x), _stream()))
    return out


def hb_conv2d(inp, out, taps2d, anchor_y, anchor_x):
    return _conv2d("hb_conv2d", inp, out, taps2d, anchor_y, anchor_x)


def hb_conv2d_valu(inp, out, taps2d, anchor_y, anchor_x):
    return _conv2d("hb_conv2d_valu", inp, out, taps2d, anchor_y, anchor_x)


def _half_shape(H, W):
    return (H + 1) // 2, (W + 1) // 2


def _double_shape(H, W):
    return 2 * H, 2 * W


def hb_down2(inp, out, taps2d, anchor_y, anchor_x):
    return _conv2d("hb_down2", inp, out, taps2d, anchor_y, anchor_x, _half_shape)


def hb_down2_valu(inp, out, taps2d, anchor_y, anchor_x):
    return _conv2d("hb_down2_valu", inp, out, taps2d, anchor_y, anchor_x, _half_shape)


def hb_up2(inp, out, taps2d, anchor_y, anchor_x):
    return _conv2d("hb_up2", inp, out, taps2d, anchor_y, anchor_x, _double_shape)


def hb_up2_valu(inp, out, taps2d, anchor_y, anchor_x):
    return _conv2d("hb_up2_valu", inp, out, taps2d, anchor_y, anchor_x, _double_shape)


def hb_dct_denoise_workspace_size(C, H, W):
    return int(load().hb_dct_denoise_workspace_size(int(C), int(H), int(W)))


def _dct(name, inp, out, threshold, workspace):
    import torch
    assert inp.is_cuda and inp.dim() == 3 and inp.dtype == torch.float16 and inp.stride(2) == 1
    assert out.is_cuda and out.dim() == 3 and out.dtype == torch.float32 and out.stride(2) == 1
    assert tuple(inp.shape) == tuple(out.shape)
    assert workspace.is_cuda and workspace.dtype == torch.uint8 and workspace.is_contiguous()
    C, H, W = (int(v) for v in inp.shape)
    _check(name, getattr(load(), name)(
        ctypes.c_void_p(inp.data_ptr()), ctypes.c_void_p(out.data_ptr()), C, H, W,
        int(inp.stride(1)), int(inp.stride(0)), int(out.stride(1)), int(out.stride(0)), float(threshold),
        ctypes.c_void_p(workspace.data_ptr()), int(workspace.numel()), _stream()))
    return out


def hb_dct_denoise(inp, out, threshold, workspace):
    return _dct("hb_dct_denoise", inp, out, threshold, workspace)


def hb_dct_denoise_valu(inp, out, threshold, workspace):
    return _dct("hb_dct_denoise_valu", inp, out, threshold, workspace)


def hb_iir2_workspace_size(C, T):
    return int(load().hb_iir2_workspace_size(int(C), int(T)))


def hb_iir2_abs_gain(alpha, beta, T):
    return float(load().hb_iir2_abs_gain(float(alpha), float(beta), int(T)))


def _iir2(name, inp, out, alpha, beta, workspace):
    import torch
    pi, C, T, ip = _img2d(inp, torch.float16)
    po, Co, To, op = _img2d(out, torch.float32)
    assert (C, T) == (Co, To)
    assert workspace.is_cuda and workspace.dtype == torch.uint8 and workspace.is_contiguous()
    _check(name, getattr(load(), name)(pi, po, C, T, ip, op, float(alpha), float(beta),
                                        ctypes.c_void_p(workspace.data_ptr()), int(workspace.numel()), _stream()))
    return out


def hb_iir2(inp, out, alpha, beta, workspace):
    return _iir2("hb_iir2", inp, out, alpha, beta, workspace)


def hb_iir2_valu(inp, out, alpha, beta, workspace):
    return _iir2("hb_iir2_valu", inp, out, alpha, beta, workspace)


def hb_resize_workspace_size(C, H, Wo):
    return int(load().hb_resize_workspace_size(int(C), int(H), int(Wo)))


def hb_lanczos3_band(n_in, n_out):
    return int(load().hb_lanczos3_band(int(n_in), int(n_out)))


def hb_lanczos3_matrix(n_in, n_out):
    """Host arrays (start int32 [n_out], coef fp16 bit patterns [n_out, band]) built by the library."""
    band = hb_lanczos3_band(n_in, n_out)
    if band <= 0:
        raise HbError("hb_lanczos3_band", HB_ERR_INVALID_ARG)
    start = np.empty(n_out, dtype=np.int32)
    coef = np.empty((n_out, band), dtype=np.uint16)
    _check("hb_lanczos3_matrix", load().hb_lanczos3_matrix(int(n_in), int(n_out), start.ctypes.data_as(ctypes.c_void_p),
                                                          coef.ctypes.data_as(ctypes.c_void_p)))
    return start, coef


def _resize(name, inp, out, workspace, start_y, coef_y, start_x, coef_x):
    import torch
    assert inp.is_cuda and inp.dim() == 3 and inp.dtype == torch.float16 and inp.stride(2) == 1
    assert out.is_cuda and out.dim() == 3 and out.dtype == torch.float32 and out.stride(2) == 1
    C, H, W = (int(v) for v in inp.shape)
    Co, Ho, Wo = (int(v) for v in out.shape)
    assert C == Co
    for st, cf, n in ((start_y, coef_y, Ho), (start_x, coef_x, Wo)):
        assert st.is_cuda and st.dtype == torch.int32 and st.is_contiguous() and tuple(st.shape) == (n,)
        assert cf.is_cuda and cf.dtype == torch.float16 and cf.is_contiguous() and cf.dim() == 2 and cf.shape[0] == n
    assert workspace.is_cuda and workspace.dtype == torch.uint8 and workspace.is_contiguous()
    _check(name, getattr(load(), name)(
        ctypes.c_void_p(inp.data_ptr()), ctypes.c_void_p(out.data_ptr()),
        ctypes.c_void_p(workspace.data_ptr()), int(workspace.numel()), C, H, W, Ho, Wo,
        int(inp.stride(1)), int(inp.stride(0)), int(out.stride(1)), int(out.stride(0)),
        ctypes.c_void_p(start_y.data_ptr()), ctypes.c_void_p(coef_y.data_ptr()), int(coef_y.shape[1]),
        ctypes.c_void_p(start_x.data_ptr()), ctypes.c_void_p(coef_x.data_ptr()), int(coef_x.shape[1]), _stream()))
    return out


def hb_resize(inp, out, workspace, start_y, coef_y, start_x, coef_x):
    return _resize("hb_resize", inp, out, workspace, start_y, coef_y, start_x, coef_x)


def hb_resize_valu(inp, out, workspace, start_y, coef_y, start_x, coef_x):
    return _resize("hb_resize_valu", inp, out, workspace, start_y, coef_y, start_x, coef_x)


def _sep(name, inp, out, tx, ax, ty, ay):
    import torch
    pi, H, W, ip = _img2d(inp, torch.float16)
    po, Ho, Wo, op = _img2d(out, torch.float32)
    assert (H, W) == (Ho, Wo)
    kx, px, nx = _taps(tx)
    ky, py, ny = _taps(ty)
    _check(name, getattr(load(), name)(pi, po, H, W, ip, op, px, nx, int(ax), py, ny, int(ay), _stream()))
    return out


def hb_sepblur(inp, out, taps_x, anchor_x, taps_y, anchor_y):
    return _sep("hb_sepblur", inp, out, taps_x, anchor_x, taps_y, anchor_y)


def hb_sepblur_valu(inp, out, taps_x, anchor_x, taps_y, anchor_y):
    return _sep("hb_sepblur_valu", inp, out, taps_x, anchor_x, taps_y, anchor_y)


def hb_sat2d_workspace_size(H, W) -> int:
    return int(load().hb_sat2d_workspace_size(int(H), int(W)))


def _sat(name, inp, out, workspace):
    import torch
    pi, H, W, ip = _img2d(inp, torch.float16)
    po, Ho, Wo, op = _img2d(out, torch.float32)
    assert (H, W) == (Ho, Wo)
    assert workspace.is_cuda and workspace.is_contiguous()
    nbytes = workspace.numel() * workspace.element_size()
    _check(name, getattr(load(), name)(pi, po, H, W, ip, op, ctypes.c_void_p(workspace.data_ptr()),
                                       nbytes, _stream()))
    return out


def hb_sat2d(inp, out, workspace):
    return _sat("hb_sat2d", inp, out, workspace)


def hb_sat2d_valu(inp, out, workspace):
    return _sat("hb_sat2d_valu", inp, out, workspace)


HB_SAT2D_NOALLOC_SCRATCH_BYTES = 5 << 20


def hb_sat2d_set_wait_limit(polls: int) -> int:
    return int(load().hb_sat2d_set_wait_limit(int(polls)))


def hb_sat2d_noalloc(inp, out):
    import torch
    pi, H, W, ip = _img2d(inp, torch.float16)
    po, Ho, Wo, op = _img2d(out, torch.float32)
    assert (H, W) == (Ho, Wo)
    _check("hb_sat2d_noalloc", load().hb_sat2d_noalloc(pi, po, H, W, ip, op, _stream()))
    return out


def _conv(name, x, w, out):
    import torch
    assert x.is_cuda and x.dtype == torch.float16 and x.is_contiguous() and x.dim() == 4
    assert w.is_cuda and w.dtype == torch.float16 and w.is_contiguous() and w.dim() == 4
    assert out.is_cuda and out.dtype == torch.float16 and out.is_contiguous() and out.dim() == 4
    N, H, W, Ci = x.shape
    Co = w.shape[3]
    assert tuple(w.shape) == (3, 3, Ci, Co) and tuple(out.shape) == (N, H, W, Co)
    _check(name, getattr(load(), name)(ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(w.data_ptr()),
                                       ctypes.c_void_p(out.data_ptr()), N, H, W, Ci, Co, _stream()))
    return out


def hb_conv3x3(x_nhwc, w_hwio, out_nhwc):
    return _conv("hb_conv3x3", x_nhwc, w_hwio, out_nhwc)


def hb_conv3x3_valu(x_nhwc, w_hwio, out_nhwc):
    return _conv("hb_conv3x3_valu", x_nhwc, w_hwio, out_nhwc)


def _pyr(name, inp, res, down):
    import torch
    pi, H, W, ip = _img2d(inp, torch.float16)
    pr, Hr, Wr, rp = _img2d(res, torch.float32)
    assert (H, W) == (Hr, Wr)
    if down is not None:
        pd, Hd, Wd, dp = _img2d(down, torch.float16)
        assert (Hd, Wd) == (H // 2, W // 2)
    else:
        pd, dp = ctypes.c_void_p(0), 0
    _check(name, getattr(load(), name)(pi, pr, pd, H, W, ip, rp, dp, _stream()))
    return res


def hb_pyr_level(inp, residual, down=None):
    return _pyr("hb_pyr_level", inp, residual, down)


def hb_pyr_level_valu(inp, residual, down=None):
    return _pyr("hb_pyr_level_valu", inp, residual, down)


def hb_copy_f16_f32(inp, out):
    n = inp.numel()
    assert out.numel() == n
    _check("hb_copy_f16_f32", load().hb_copy_f16_f32(ctypes.c_void_p(inp.data_ptr()),
                                                     ctypes.c_void_p(out.data_ptr()), n, _stream()))
    return out


def hb_mfma_probe(which, A, B, D):
    _check("hb_mfma_probe", load().hb_mfma_probe(int(which), ctypes.c_void_p(A.data_ptr()),
                                                 ctypes.c_void_p(B.data_ptr()),
                                                 ctypes.c_void_p(D.data_ptr()), _stream()))
    return D
