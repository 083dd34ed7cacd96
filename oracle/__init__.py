"""fp64 CPU oracle for the five image stages.  TEST INFRASTRUCTURE ONLY.

Thin ctypes loader around ``hb_oracle.c`` (plain C loops, double precision).
Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package; the HIP library and its Python binding
never do, and this package imports nothing from them.

fp16 arrays are ``numpy.uint16`` bit patterns; results are ``numpy.float64``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hb_oracle.c")
_LIB = os.path.join(_HERE, "libhb_oracle.so")


def build(force: bool = False) -> str:
    """Compile hb_oracle.c with gcc (a second or two)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f64p = ctypes.POINTER(ctypes.c_double)
        i32p = ctypes.POINTER(ctypes.c_int)
        I, Lg = ctypes.c_int, ctypes.c_long
        L.hbo_half_to_double.argtypes = [ctypes.c_uint16]
        L.hbo_half_to_double.restype = ctypes.c_double
        L.hbo_num_threads.restype = I
        L.hbo_set_num_threads.argtypes = [I]
        L.hbo_fir1d.argtypes = [u16p, f64p, I, I, Lg, Lg, u16p, I, I]
        L.hbo_sepblur.argtypes = [u16p, f64p, I, I, Lg, Lg, u16p, I, I, u16p, I, I]
        L.hbo_conv2d.argtypes = [u16p, f64p, I, I, Lg, Lg, u16p, I, I, I, I]
        L.hbo_conv2d.restype = None
        L.hbo_band_resize.argtypes = [u16p, f64p, I, I, I, I, Lg, Lg, i32p, u16p, I, i32p, u16p, I]
        L.hbo_band_resize.restype = None
        L.hbo_iir2.argtypes = [u16p, f64p, I, Lg, Lg, Lg, ctypes.c_double, ctypes.c_double]
        L.hbo_iir2.restype = None
        for f in (L.hbo_down2, L.hbo_up2):
            f.argtypes = [u16p, f64p, I, I, Lg, Lg, u16p, I, I, I, I]
            f.restype = None
        L.hbo_sat2d.argtypes = [u16p, f64p, I, I, Lg, Lg]
        L.hbo_conv3x3.argtypes = [u16p, u16p, f64p, I, I, I, I, I]
        L.hbo_conv3x3_rows.argtypes = [u16p, u16p, f64p, I, I, I, I, I, I, I]
        L.hbo_conv3x3_points.argtypes = [u16p, u16p, f64p, I, I, I, I, I, Lg, i32p, i32p, i32p]
        L.hbo_pyr_level.argtypes = [u16p, f64p, f64p, I, I, Lg, Lg, Lg]
        for f in (L.hbo_set_num_threads, L.hbo_fir1d, L.hbo_sepblur, L.hbo_sat2d, L.hbo_conv3x3,
                  L.hbo_conv3x3_rows, L.hbo_conv3x3_points, L.hbo_pyr_level):
            f.restype = None
        _lib = L
    return _lib


def _u16(a):
    a = np.ascontiguousarray(a, dtype=np.uint16)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def _f64(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def num_threads() -> int:
    return int(_load().hbo_num_threads())


def set_num_threads(n: int) -> None:
    _load().hbo_set_num_threads(int(n))


def half_to_double(bits: int) -> float:
    return float(_load().hbo_half_to_double(int(bits)))


_half_table = None


def halves_to_doubles(bits):
    """fp16 bit patterns -> float64 array, through the oracle's own binary16 decoder (a table of
    all 65536 patterns, decoded once by hbo_half_to_double)."""
    global _half_table
    if _half_table is None:
        f = _load().hbo_half_to_double
        _half_table = np.array([f(b) for b in range(65536)], dtype=np.float64)
    return _half_table[np.ascontiguousarray(bits, dtype=np.uint16)]


def fir1d(img, taps, anchor):
    """out[y][x] = sum_r k[r] in[y][clampW(x + r - anchor)]  (Sec. V-A 1-D form)."""
    img, pi = _u16(img)
    taps, pt = _u16(taps)
    H, W = img.shape
    out = np.empty((H, W), dtype=np.float64)
    _load().hbo_fir1d(pi, _f64(out), H, W, W, W, pt, len(taps), int(anchor))
    return out


def conv2d(img, taps2d, anchor_y, anchor_x):
    """out[y][x] = sum_{ry, rx} k[ry][rx] in[clampH(y + ry - ay)][clampW(x + rx - ax)]  (Sec. V-A 2-D form)."""
    img, pi = _u16(img)
    k = np.ascontiguousarray(taps2d)
    assert k.ndim == 2
    k, pk = _u16(k)
    H, W = img.shape
    out = np.empty((H, W), dtype=np.float64)
    _load().hbo_conv2d(pi, _f64(out), H, W, W, W, pk, k.shape[0], k.shape[1], int(anchor_y), int(anchor_x))
    return out


def down2(img, taps2d, anchor_y, anchor_x):
    """out[y][x] = sum_{ry, rx} k[ry][rx] in[clampH(2y + ry - ay)][clampW(2x + rx - ax)]  (Sec. V-B, strided form)."""
    img, pi = _u16(img)
    k = np.ascontiguousarray(taps2d)
    assert k.ndim == 2
    k, pk = _u16(k)
    H, W = img.shape
    Ho, Wo = (H + 1) // 2, (W + 1) // 2
    out = np.empty((Ho, Wo), dtype=np.float64)
    _load().hbo_down2(pi, _f64(out), H, W, W, Wo, pk, k.shape[0], k.shape[1], int(anchor_y), int(anchor_x))
    return out


def up2(img, taps2d, anchor_y, anchor_x):
    """out[y][x] = sum_{ry < kh/2, rx < kw/2} k[2ry + y%2][2rx + x%2] in[clampH(y//2 + ry - ay)][clampW(x//2 + rx - ax)]
    (Sec. V-B, multiphase form)."""
    img, pi = _u16(img)
    k = np.ascontiguousarray(taps2d)
    assert k.ndim == 2 and k.shape[0] % 2 == 0 and k.shape[1] % 2 == 0
    k, pk = _u16(k)
    H, W = img.shape
    out = np.empty((2 * H, 2 * W), dtype=np.float64)
    _load().hbo_up2(pi, _f64(out), H, W, W, 2 * W, pk, k.shape[0], k.shape[1], int(anchor_y), int(anchor_x))
    return out


def iir2(sig, alpha, beta):
    """y[c][t] = x[c][t] + alpha y[c][t-1] + beta y[c][t-2], zero initial state (Sec. V-D); sig is [C, T] fp16."""
    sig, ps = _u16(sig)
    C, T = sig.shape
    out = np.empty((C, T), dtype=np.float64)
    _load().hbo_iir2(ps, _f64(out), C, T, T, T, float(alpha), float(beta))
    return out


def dct16_matrix():
    """Orthonormal 16-point DCT-II: D[u][i] = s_u cos(pi (2i + 1) u / 32), s_0 = 1/4, s_u = sqrt(2)/4."""
    u = np.arange(16, dtype=np.float64)[:, None]
    i = np.arange(16, dtype=np.float64)[None, :]
    D = np.cos(np.pi * (2.0 * i + 1.0) * u / 32.0) * np.sqrt(2.0 / 16.0)
    D[0] = 0.25
    return D


def sine_window16():
    """w(i) = sin(pi (i + 1/2) / 16): w(i)^2 + w(i + 8)^2 = 1, so half-overlapping tiles sum to one."""
    return np.sin(np.pi * (np.arange(16, dtype=np.float64) + 0.5) / 16.0)


def dct_denoise(img, threshold, margin=0.0):
    """Transform-domain coring of one plane (Sec. V-E): 16 x 16 tiles at stride 8, each multiplied by
    the separable sine window, transformed by the 2-D DCT (D T D^T), every bin except DC whose magnitude
    is below `threshold` set to zero, transformed back (D^T Y D), windowed again and blended,
    out = sum_tiles(w rec) / sum_tiles(w^2).  Tile origins are (8 ty, 8 tx), 0 <= ty < H/8 - 1.
    Also returns a mask of the pixels touched by a tile with a bin within `margin` of the threshold
    (a hard threshold makes those bins, and only those, sensitive to rounding)."""
    X = halves_to_doubles(img)
    H, W = X.shape
    assert H % 8 == 0 and W % 8 == 0 and H >= 16 and W >= 16
    D, w = dct16_matrix(), sine_window16()
    w2 = np.outer(w, w)
    num = np.zeros((H, W))
    den = np.zeros((H, W))
    risky = np.zeros((H, W), dtype=bool)
    for ty in range(H // 8 - 1):
        for tx in range(W // 8 - 1):
            y0, x0 = 8 * ty, 8 * tx
            Y = D @ (X[y0:y0 + 16, x0:x0 + 16] * w2) @ D.T
            keep = np.abs(Y) >= threshold
            keep[0, 0] = True
            if margin > 0.0:
                near = np.abs(np.abs(Y) - threshold) < margin
                near[0, 0] = False
                if near.any():
                    risky[y0:y0 + 16, x0:x0 + 16] = True
            rec = D.T @ (Y * keep) @ D
            num[y0:y0 + 16, x0:x0 + 16] += rec * w2
            den[y0:y0 + 16, x0:x0 + 16] += w2 * w2
    return num / den, risky


def band_resize(img, start_y, coef_y, start_x, coef_x):
    """One plane resized with two banded matrices (Sec. V-C): row o of a matrix holds `band` fp16
    coefficients for the input indices start[o] .. start[o] + band - 1 (clamped into the image)."""
    img, pi = _u16(img)
    H, W = img.shape
    cy, pcy = _u16(np.ascontiguousarray(coef_y))
    cx, pcx = _u16(np.ascontiguousarray(coef_x))
    sy = np.ascontiguousarray(start_y, dtype=np.int32)
    sx = np.ascontiguousarray(start_x, dtype=np.int32)
    Ho, by = cy.shape
    Wo, bx = cx.shape
    assert sy.shape == (Ho,) and sx.shape == (Wo,)
    i32p = ctypes.POINTER(ctypes.c_int)
    out = np.empty((Ho, Wo), dtype=np.float64)
    _load().hbo_band_resize(pi, _f64(out), H, W, Ho, Wo, W, Wo, sy.ctypes.data_as(i32p), pcy, by,
                            sx.ctypes.data_as(i32p), pcx, bx)
    return out


def lanczos3(x):
    """The three-lobed Lanczos window sinc(x) sinc(x/3) on [-3, 3], 0 outside (Sec. V-C)."""
    x = np.asarray(x, dtype=np.float64)
    return np.where(np.abs(x) < 3.0, np.sinc(x) * np.sinc(x / 3.0), 0.0)


def lanczos3_matrix(n_in: int, n_out: int):
    """Banded matrix (start, coef) that resamples n_in samples to n_out <= n_in (Sec. V-C): output o
    sits at input position (o + 1/2) n_in/n_out - 1/2; the pre-filter is the Lanczos window stretched
    by the factor n_in/n_out; every row is normalised to sum 1 in fp64.  Returned in fp64, unrounded."""
    assert 1 <= n_out <= n_in
    scale = n_in / n_out
    band = lanczos3_band(n_in, n_out)
    start = np.empty(n_out, dtype=np.int32)
    coef = np.zeros((n_out, band), dtype=np.float64)
    for o in range(n_out):
        centre = (o + 0.5) * scale - 0.5
        first = int(np.ceil(centre - 3.0 * scale))
        idx = first + np.arange(band)
        w = lanczos3((idx - centre) / scale)
        start[o] = first
        coef[o] = w / w.sum()
    return start, coef


def lanczos3_band(n_in: int, n_out: int) -> int:
    """Entries per row: the stretched window covers at most floor(6 n_in/n_out) + 1 input samples."""
    return int(np.floor(6.0 * n_in / n_out)) + 1


def sepblur(img, taps_x, anchor_x, taps_y, anchor_y):
    """Row FIR then column FIR, clamp-to-edge, fp64 intermediate."""
    img, pi = _u16(img)
    tx, ptx = _u16(taps_x)
    ty, pty = _u16(taps_y)
    H, W = img.shape
    out = np.empty((H, W), dtype=np.float64)
    _load().hbo_sepblur(pi, _f64(out), H, W, W, W, ptx, len(tx), int(anchor_x),
                        pty, len(ty), int(anchor_y))
    return out


def sat2d(img):
    """Inclusive 2-D prefix sum."""
    img, pi = _u16(img)
    H, W = img.shape
    out = np.empty((H, W), dtype=np.float64)
    _load().hbo_sat2d(pi, _f64(out), H, W, W, W)
    return out


def conv3x3(x_nhwc, w_hwio):
    """3x3, zero pad 1, stride 1, NHWC x HWIO -> NHWC (fp64, unrounded)."""
    x, px = _u16(x_nhwc)
    w, pw = _u16(w_hwio)
    N, H, W, Ci = x.shape
    assert w.shape[:3] == (3, 3, Ci)
    Co = w.shape[3]
    out = np.empty((N, H, W, Co), dtype=np.float64)
    _load().hbo_conv3x3(px, pw, _f64(out), N, H, W, Ci, Co)
    return out


def conv3x3_rows(x_nhwc, w_hwio, y0, y1):
    """Output rows y0..y1-1 only, returned as an (N, y1-y0, W, Cout) array."""
    x, px = _u16(x_nhwc)
    w, pw = _u16(w_hwio)
    N, H, W, Ci = x.shape
    Co = w.shape[3]
    assert N == 1, "row-band variant is used on single images"
    full = np.empty((N, H, W, Co), dtype=np.float64)   # virtual memory; only the band is touched
    _load().hbo_conv3x3_rows(px, pw, _f64(full), N, H, W, Ci, Co, int(y0), int(y1))
    return full[:, y0:y1].copy()


def conv3x3_points(x_nhwc, w_hwio, ns, ys, xs):
    """All Cout channels at the listed (n, y, x) positions -> (npts, Cout)."""
    x, px = _u16(x_nhwc)
    w, pw = _u16(w_hwio)
    N, H, W, Ci = x.shape
    Co = w.shape[3]
    ns = np.ascontiguousarray(ns, dtype=np.int32)
    ys = np.ascontiguousarray(ys, dtype=np.int32)
    xs = np.ascontiguousarray(xs, dtype=np.int32)
    out = np.empty((len(ys), Co), dtype=np.float64)
    i32p = ctypes.POINTER(ctypes.c_int)
    _load().hbo_conv3x3_points(px, pw, _f64(out), N, H, W, Ci, Co, len(ys),
                               ns.ctypes.data_as(i32p), ys.ctypes.data_as(i32p),
                               xs.ctypes.data_as(i32p))
    return out


def pyr_level(img, want_down: bool = False):
    """Residual of one Laplacian level with the [1,4,6,4,1]/16 kernel (and D if asked)."""
    img, pi = _u16(img)
    H, W = img.shape
    assert H % 2 == 0 and W % 2 == 0
    res = np.empty((H, W), dtype=np.float64)
    down = np.empty((H // 2, W // 2), dtype=np.float64) if want_down else None
    _load().hbo_pyr_level(pi, _f64(res), _f64(down) if want_down else None,
                          H, W, W, W, W // 2)
    return (res, down) if want_down else res
