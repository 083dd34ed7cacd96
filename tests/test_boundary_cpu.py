"""Boundary checks that need no GPU: the library loads, exports every declared
symbol, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2512_02371_amd import hb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(hb.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return hb.load()


def test_every_declared_symbol_is_exported(lib):
    text = open(os.path.join(ROOT, "include", "hb.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(hb_[a-z0-9_]+)\s*\(", text))
    assert declared == set(hb.SYMBOLS)
    for s in declared:
        assert hasattr(lib, s), s
        assert callable(getattr(hb, s, None)), f"the binding has no function named {s}"


def test_status_strings(lib):
    assert hb.status_string(0) == "HB_OK"
    assert hb.status_string(1) == "HB_ERR_INVALID_ARG"
    assert hb.status_string(3) == "HB_ERR_WORKSPACE"


FAKE = ctypes.c_void_p(0x1000)          # never dereferenced: validation fails first
TAPS = np.zeros(8, dtype=np.uint16).ctypes.data_as(ctypes.c_void_p)
_keep = np.zeros(8, dtype=np.uint16)
TAPS = _keep.ctypes.data_as(ctypes.c_void_p)


@pytest.mark.parametrize("fn", ["hb_fir1d", "hb_fir1d_valu"])
def test_fir_argument_validation(lib, fn):
    f = getattr(lib, fn)
    ok = dict(i=FAKE, o=FAKE, H=16, W=16, ip=16, op=16, t=TAPS, n=8, a=3)

    def call(**kw):
        p = dict(ok, **kw)
        return f(p["i"], p["o"], p["H"], p["W"], p["ip"], p["op"], p["t"], p["n"], p["a"], None)
    assert call(i=None) == hb.HB_ERR_INVALID_ARG
    assert call(o=None) == hb.HB_ERR_INVALID_ARG
    assert call(t=None) == hb.HB_ERR_INVALID_ARG
    assert call(H=0) == hb.HB_ERR_INVALID_ARG
    assert call(W=-1) == hb.HB_ERR_INVALID_ARG
    assert call(ip=15) == hb.HB_ERR_INVALID_ARG
    assert call(op=8) == hb.HB_ERR_INVALID_ARG
    assert call(n=0) == hb.HB_ERR_INVALID_ARG
    assert call(n=257) == hb.HB_ERR_INVALID_ARG
    assert call(a=-1) == hb.HB_ERR_INVALID_ARG
    assert call(a=8) == hb.HB_ERR_INVALID_ARG
    assert call(i=ctypes.c_void_p(0x1001)) == hb.HB_ERR_INVALID_ARG


@pytest.mark.parametrize("fn", ["hb_sepblur", "hb_sepblur_valu"])
def test_sepblur_argument_validation(lib, fn):
    f = getattr(lib, fn)
    ok = dict(i=FAKE, o=FAKE, H=16, W=16, ip=16, op=16, tx=TAPS, nx=8, ax=3, ty=TAPS, ny=8, ay=3)

    def call(**kw):
        p = dict(ok, **kw)
        return f(p["i"], p["o"], p["H"], p["W"], p["ip"], p["op"], p["tx"], p["nx"], p["ax"], p["ty"], p["ny"], p["ay"], None)
    assert call(i=None) == hb.HB_ERR_INVALID_ARG
    assert call(o=None) == hb.HB_ERR_INVALID_ARG
    assert call(tx=None) == hb.HB_ERR_INVALID_ARG
    assert call(ty=None) == hb.HB_ERR_INVALID_ARG
    assert call(H=0) == hb.HB_ERR_INVALID_ARG
    assert call(W=0) == hb.HB_ERR_INVALID_ARG
    assert call(ip=15) == hb.HB_ERR_INVALID_ARG
    assert call(op=15) == hb.HB_ERR_INVALID_ARG
    assert call(nx=0) == hb.HB_ERR_INVALID_ARG
    assert call(ny=hb.HB_MAX_TAPS + 1) == hb.HB_ERR_INVALID_ARG
    assert call(ax=8) == hb.HB_ERR_INVALID_ARG
    assert call(ay=-1) == hb.HB_ERR_INVALID_ARG
    assert call(o=ctypes.c_void_p(0x1002)) == hb.HB_ERR_INVALID_ARG      # fp32 output on a 2-byte boundary


@pytest.mark.parametrize("fn", ["hb_sat2d", "hb_sat2d_valu"])
def test_sat2d_argument_validation(lib, fn):
    f = getattr(lib, fn)
    need = lib.hb_sat2d_workspace_size(100, 200)
    assert need > 0 and lib.hb_sat2d_workspace_size(0, 5) == 0 and lib.hb_sat2d_workspace_size(5, -1) == 0
    # the workspace holds row and column sums per tile: it grows with the image
    assert lib.hb_sat2d_workspace_size(1000, 2000) > need
    WS = ctypes.c_void_p(0x10000)
    ok = dict(i=FAKE, o=FAKE, H=100, W=200, ip=200, op=200, ws=WS, wsb=need)

    def call(**kw):
        p = dict(ok, **kw)
        return f(p["i"], p["o"], p["H"], p["W"], p["ip"], p["op"], p["ws"], p["wsb"], None)
    assert call(i=None) == hb.HB_ERR_INVALID_ARG
    assert call(o=None) == hb.HB_ERR_INVALID_ARG
    assert call(H=0) == hb.HB_ERR_INVALID_ARG
    assert call(W=-3) == hb.HB_ERR_INVALID_ARG
    assert call(ip=199) == hb.HB_ERR_INVALID_ARG
    assert call(op=100) == hb.HB_ERR_INVALID_ARG
    assert call(ws=None) == hb.HB_ERR_WORKSPACE
    assert call(wsb=need - 1) == hb.HB_ERR_WORKSPACE
    assert call(ws=ctypes.c_void_p(0x100010)) == hb.HB_ERR_WORKSPACE       # not 256-byte aligned


@pytest.mark.parametrize("fn", ["hb_conv3x3", "hb_conv3x3_valu"])
def test_conv3x3_argument_validation(lib, fn):
    f = getattr(lib, fn)
    ok = dict(i=FAKE, w=FAKE, o=FAKE, N=1, H=8, W=8, ci=64, co=64)

    def call(**kw):
        p = dict(ok, **kw)
        return f(p["i"], p["w"], p["o"], p["N"], p["H"], p["W"], p["ci"], p["co"], None)
    assert call(i=None) == hb.HB_ERR_INVALID_ARG
    assert call(w=None) == hb.HB_ERR_INVALID_ARG
    assert call(o=None) == hb.HB_ERR_INVALID_ARG
    assert call(N=0) == hb.HB_ERR_INVALID_ARG
    assert call(H=0) == hb.HB_ERR_INVALID_ARG
    assert call(W=-1) == hb.HB_ERR_INVALID_ARG
    assert call(ci=0) == hb.HB_ERR_INVALID_ARG
    assert call(i=ctypes.c_void_p(0x1008)) == hb.HB_ERR_INVALID_ARG      # pixels are read 16 bytes at a time
    assert call(ci=32) == hb.HB_ERR_UNSUPPORTED
    assert call(co=128) == hb.HB_ERR_UNSUPPORTED


@pytest.mark.parametrize("fn", ["hb_pyr_level", "hb_pyr_level_valu"])
def test_pyr_level_argument_validation(lib, fn):
    f = getattr(lib, fn)
    ok = dict(i=FAKE, r=FAKE, d=FAKE, H=16, W=32, ip=32, rp=32, dp=16)

    def call(**kw):
        p = dict(ok, **kw)
        return f(p["i"], p["r"], p["d"], p["H"], p["W"], p["ip"], p["rp"], p["dp"], None)
    assert call(i=None) == hb.HB_ERR_INVALID_ARG
    assert call(r=None) == hb.HB_ERR_INVALID_ARG
    assert call(H=15) == hb.HB_ERR_INVALID_ARG                             # odd sizes have no half-size level
    assert call(W=31, ip=32) == hb.HB_ERR_INVALID_ARG
    assert call(H=0) == hb.HB_ERR_INVALID_ARG
    assert call(ip=31) == hb.HB_ERR_INVALID_ARG
    assert call(rp=16) == hb.HB_ERR_INVALID_ARG
    assert call(dp=15) == hb.HB_ERR_INVALID_ARG                            # down is W / 2 wide
    assert call(d=ctypes.c_void_p(0x1001)) == hb.HB_ERR_INVALID_ARG
    assert call(dp=(1 << 26) + 2) == hb.HB_ERR_UNSUPPORTED


@pytest.mark.parametrize("fn", ["hb_conv2d", "hb_conv2d_valu"])
def test_conv2d_argument_validation(lib, fn):
    f = getattr(lib, fn)
    k = np.zeros(32 * 32, dtype=np.uint16)
    kp = k.ctypes.data_as(ctypes.c_void_p)
    ok = dict(i=FAKE, o=FAKE, H=16, W=16, ip=16, op=16, t=kp, kh=5, kw=7, ay=2, ax=3)

    def call(**kw):
        p = dict(ok, **kw)
        return f(p["i"], p["o"], p["H"], p["W"], p["ip"], p["op"], p["t"], p["kh"], p["kw"], p["ay"], p["ax"], None)
    assert call(i=None) == hb.HB_ERR_INVALID_ARG
    assert call(o=None) == hb.HB_ERR_INVALID_ARG
    assert call(t=None) == hb.HB_ERR_INVALID_ARG
    assert call(H=0) == hb.HB_ERR_INVALID_ARG
    assert call(ip=15) == hb.HB_ERR_INVALID_ARG
    assert call(kh=0) == hb.HB_ERR_INVALID_ARG
    assert call(kw=33) == hb.HB_ERR_INVALID_ARG
    assert call(kh=33) == hb.HB_ERR_INVALID_ARG
    assert call(ay=5) == hb.HB_ERR_INVALID_ARG
    assert call(ax=-1) == hb.HB_ERR_INVALID_ARG
    assert call(ax=7) == hb.HB_ERR_INVALID_ARG
    # rows are addressed with 32-bit byte offsets: larger images are reported, not wrapped
    assert call(H=1 << 16, W=1 << 15, ip=1 << 15, op=1 << 15) == hb.HB_ERR_UNSUPPORTED


@pytest.mark.parametrize("fn", ["hb_down2", "hb_down2_valu", "hb_up2", "hb_up2_valu"])
def test_resample2_argument_validation(lib, fn):
    f = getattr(lib, fn)
    k = np.zeros(32 * 32, dtype=np.uint16)
    kp = k.ctypes.data_as(ctypes.c_void_p)
    upsample = "up2" in fn
    # 16 x 16 input; the output pitch must cover 8 (down) or 32 (up) samples
    ok = dict(i=FAKE, o=FAKE, H=16, W=16, ip=16, op=32, t=kp, kh=6, kw=8, ay=2, ax=3)

    def call(**kw):
        p = dict(ok, **kw)
        return f(p["i"], p["o"], p["H"], p["W"], p["ip"], p["op"], p["t"], p["kh"], p["kw"], p["ay"], p["ax"], None)
    assert call(i=None) == hb.HB_ERR_INVALID_ARG
    assert call(o=None) == hb.HB_ERR_INVALID_ARG
    assert call(t=None) == hb.HB_ERR_INVALID_ARG
    assert call(W=0) == hb.HB_ERR_INVALID_ARG
    assert call(ip=15) == hb.HB_ERR_INVALID_ARG
    assert call(op=31 if upsample else 7) == hb.HB_ERR_INVALID_ARG
    assert call(kh=0) == hb.HB_ERR_INVALID_ARG
    assert call(kw=34) == hb.HB_ERR_INVALID_ARG
    assert call(ay=-1) == hb.HB_ERR_INVALID_ARG
    if upsample:
        assert call(kh=5) == hb.HB_ERR_INVALID_ARG          # odd kernel sizes have no two phases
        assert call(kw=7) == hb.HB_ERR_INVALID_ARG
        assert call(ay=3) == hb.HB_ERR_INVALID_ARG          # anchors count input pixels: < kh / 2
        assert call(ax=4) == hb.HB_ERR_INVALID_ARG
    else:
        assert call(ay=6) == hb.HB_ERR_INVALID_ARG
        assert call(ax=8) == hb.HB_ERR_INVALID_ARG
    assert call(H=1 << 16, W=1 << 15, ip=1 << 15, op=1 << 16) == hb.HB_ERR_UNSUPPORTED


def test_lanczos3_matrix_matches_the_oracle_definition(lib):
    """The library's host-side matrix against the oracle's own fp64 construction rounded to fp16:
    same starts, same band, coefficients equal up to one fp16 step (the two evaluate sin() and round
    through different paths)."""
    import oracle
    for n_in, n_out in ((2048, 143), (2048, 921), (300, 31), (64, 64), (7, 1)):
        start, coef = hb.hb_lanczos3_matrix(n_in, n_out)
        o_start, o_coef = oracle.lanczos3_matrix(n_in, n_out)
        assert coef.shape[1] == oracle.lanczos3_band(n_in, n_out) == hb.hb_lanczos3_band(n_in, n_out)
        assert np.array_equal(start, o_start)
        want = o_coef.astype(np.float16)
        got = coef.view(np.float16)
        step = np.maximum(np.spacing(np.abs(want)), np.float16(6e-8)).astype(np.float64)
        assert np.all(np.abs(got.astype(np.float64) - want.astype(np.float64)) <= step)
        assert np.mean(got == want) > 0.99
    assert hb.hb_lanczos3_band(10, 11) == 0            # upsampling is not this function's job
    assert lib.hb_lanczos3_matrix(4096, 40, FAKE, FAKE) == hb.HB_ERR_UNSUPPORTED    # band 615 > 512
    assert lib.hb_lanczos3_matrix(10, 5, None, FAKE) == hb.HB_ERR_INVALID_ARG


@pytest.mark.parametrize("fn", ["hb_resize", "hb_resize_valu"])
def test_resize_argument_validation(lib, fn):
    f = getattr(lib, fn)
    WS = ctypes.c_void_p(0x10000)
    ok = dict(i=FAKE, o=FAKE, ws=WS, wsb=1 << 20, C=3, H=64, W=64, Ho=20, Wo=20, ip=64, ipl=64 * 64, op=20, opl=400,
              sy=FAKE, cy=FAKE, by=20, sx=FAKE, cx=FAKE, bx=20)

    def call(**kw):
        p = dict(ok, **kw)
        return f(p["i"], p["o"], p["ws"], p["wsb"], p["C"], p["H"], p["W"], p["Ho"], p["Wo"], p["ip"], p["ipl"],
                 p["op"], p["opl"], p["sy"], p["cy"], p["by"], p["sx"], p["cx"], p["bx"], None)
    for k in ("i", "o", "sy", "cy", "sx", "cx"):
        assert call(**{k: None}) == hb.HB_ERR_INVALID_ARG
    assert call(C=0) == hb.HB_ERR_INVALID_ARG
    assert call(Ho=0) == hb.HB_ERR_INVALID_ARG
    assert call(ip=63) == hb.HB_ERR_INVALID_ARG
    assert call(op=19) == hb.HB_ERR_INVALID_ARG
    assert call(ipl=64 * 63) == hb.HB_ERR_INVALID_ARG
    assert call(opl=399) == hb.HB_ERR_INVALID_ARG
    assert call(by=0) == hb.HB_ERR_INVALID_ARG
    assert call(bx=513) == hb.HB_ERR_INVALID_ARG
    assert call(ws=None) == hb.HB_ERR_WORKSPACE
    assert call(wsb=lib.hb_resize_workspace_size(3, 64, 20) - 1) == hb.HB_ERR_WORKSPACE
    assert call(ws=ctypes.c_void_p(0x10010)) == hb.HB_ERR_WORKSPACE
    assert lib.hb_resize_workspace_size(3, 64, 20) == 3 * 20 * 64 * 2
    assert lib.hb_resize_workspace_size(1, 61, 20) == 20 * 64 * 2      # rows padded to 8 samples


@pytest.mark.parametrize("fn", ["hb_iir2", "hb_iir2_valu"])
def test_iir2_argument_validation(lib, fn):
    f = getattr(lib, fn)
    WS = ctypes.c_void_p(0x10000)
    ok = dict(i=FAKE, o=FAKE, C=2, T=5000, ip=5000, op=5000, a=1.6, b=-0.8, ws=WS, wsb=1 << 20)

    def call(**kw):
        p = dict(ok, **kw)
        return f(p["i"], p["o"], p["C"], p["T"], p["ip"], p["op"], p["a"], p["b"], p["ws"], p["wsb"], None)
    assert call(i=None) == hb.HB_ERR_INVALID_ARG
    assert call(o=None) == hb.HB_ERR_INVALID_ARG
    assert call(C=0) == hb.HB_ERR_INVALID_ARG
    assert call(T=0) == hb.HB_ERR_INVALID_ARG
    assert call(ip=4999) == hb.HB_ERR_INVALID_ARG
    assert call(op=10) == hb.HB_ERR_INVALID_ARG
    assert call(a=float("nan")) == hb.HB_ERR_INVALID_ARG
    assert call(b=5.0) == hb.HB_ERR_INVALID_ARG
    assert call(a=3.0, b=2.0) == hb.HB_ERR_UNSUPPORTED          # impulse response leaves the fp16 range within 32 samples
    # filters whose error magnification sum|h| exceeds 2^14 are refused: the running sum beyond 16384 samples,
    # a pole pair almost on the unit circle; the same filters on short signals pass this check
    big = dict(T=40000, ip=40000, op=40000, wsb=1 << 24)
    assert call(a=1.0, b=0.0, **big) == hb.HB_ERR_UNSUPPORTED
    assert call(a=1.99999, b=-0.99999, **big) == hb.HB_ERR_UNSUPPORTED
    assert call(ws=None) == hb.HB_ERR_WORKSPACE
    assert call(wsb=lib.hb_iir2_workspace_size(2, 5000) - 1) == hb.HB_ERR_WORKSPACE
    assert lib.hb_iir2_workspace_size(2, 5000) == 2 * 10 * 16     # 10 tiles of 512 samples, two states of two floats


@pytest.mark.parametrize("fn", ["hb_dct_denoise", "hb_dct_denoise_valu"])
def test_dct_denoise_argument_validation(lib, fn):
    f = getattr(lib, fn)
    WS = ctypes.c_void_p(0x10000)
    ok = dict(i=FAKE, o=FAKE, C=3, H=64, W=96, ip=96, ipl=64 * 96, op=96, opl=64 * 96, thr=0.05, ws=WS, wsb=1 << 24)

    def call(**kw):
        p = dict(ok, **kw)
        return f(p["i"], p["o"], p["C"], p["H"], p["W"], p["ip"], p["ipl"], p["op"], p["opl"], p["thr"], p["ws"], p["wsb"], None)
    assert call(i=None) == hb.HB_ERR_INVALID_ARG
    assert call(o=None) == hb.HB_ERR_INVALID_ARG
    assert call(C=0) == hb.HB_ERR_INVALID_ARG
    assert call(H=8) == hb.HB_ERR_INVALID_ARG                   # at least one 16 x 16 tile
    assert call(W=100) == hb.HB_ERR_INVALID_ARG                 # multiples of the tile stride
    assert call(ip=95) == hb.HB_ERR_INVALID_ARG
    assert call(opl=64 * 96 - 1) == hb.HB_ERR_INVALID_ARG
    assert call(thr=-1.0) == hb.HB_ERR_INVALID_ARG
    assert call(thr=float("nan")) == hb.HB_ERR_INVALID_ARG
    assert call(ws=None) == hb.HB_ERR_WORKSPACE
    assert call(wsb=lib.hb_dct_denoise_workspace_size(3, 64, 96) - 1) == hb.HB_ERR_WORKSPACE
    assert lib.hb_dct_denoise_workspace_size(3, 64, 96) == 3 * 7 * 11 * 1024
    assert lib.hb_dct_denoise_workspace_size(1, 60, 96) == 0


def test_copy_and_probe_validation(lib):
    assert lib.hb_copy_f16_f32(None, FAKE, 8, None) == hb.HB_ERR_INVALID_ARG
    assert lib.hb_copy_f16_f32(FAKE, FAKE, 0, None) == hb.HB_ERR_INVALID_ARG
    assert lib.hb_copy_f16_f32(ctypes.c_void_p(0x1004), FAKE, 8, None) == hb.HB_ERR_INVALID_ARG
    assert lib.hb_mfma_probe(5, FAKE, FAKE, FAKE, None) == hb.HB_ERR_INVALID_ARG
    assert lib.hb_mfma_probe(0, None, FAKE, FAKE, None) == hb.HB_ERR_INVALID_ARG


def test_size_limits_are_reported_not_wrapped(lib):
    """Sizes beyond the 32-bit offsets the kernels use come back as HB_ERR_UNSUPPORTED."""
    big = dict(H=1 << 20, W=16, ip=1 << 12, op=1 << 12)          # H * pitch = 2^32 elements
    assert lib.hb_fir1d(FAKE, FAKE, big["H"], big["W"], big["ip"], big["op"], TAPS, 8, 3, None) == hb.HB_ERR_UNSUPPORTED
    assert lib.hb_sepblur(FAKE, FAKE, big["H"], big["W"], big["ip"], big["op"], TAPS, 8, 3, TAPS, 8, 3,
                          None) == hb.HB_ERR_UNSUPPORTED
    assert lib.hb_fir1d(FAKE, FAKE, 16, 16, (1 << 26) + 8, 16, TAPS, 8, 3, None) == hb.HB_ERR_UNSUPPORTED
    # one conv image of 2^24 pixels or more (2 GiB of fp16 x 64 channels)
    assert lib.hb_conv3x3(FAKE, FAKE, FAKE, 1, 4096, 4096, 64, 64, None) == hb.HB_ERR_UNSUPPORTED
    assert lib.hb_conv3x3(FAKE, FAKE, FAKE, 1, 4096, 4095, 64, 32, None) == hb.HB_ERR_UNSUPPORTED


def test_iir2_abs_gain_is_the_sum_of_the_impulse_response(lib):
    """Against the definition: h from the recurrence in fp64, summed over T samples."""
    for alpha, beta, T in [(1.6, -0.8, 5000), (1.2, -0.52, 100), (0.5, 0.3, 7), (-0.9, 0.0, 1000), (0.0, 0.0, 50),
                           (1.0, 0.0, 12345), (1.9, -0.95, 100000)]:
        al, be = float(np.float32(alpha)), float(np.float32(beta))
        h = np.zeros(min(T, 200000))
        for i in range(len(h)):
            h[i] = 1.0 if i == 0 else al * h[i - 1] + (be * h[i - 2] if i >= 2 else 0.0)
        want = np.abs(h).sum()
        got = hb.hb_iir2_abs_gain(alpha, beta, T)
        assert abs(got - want) <= 1e-9 * want, (alpha, beta, T, got, want)
    assert hb.hb_iir2_abs_gain(1.0, 0.0, 1 << 30) == float(1 << 30)     # extrapolated past the summed samples
    assert hb.hb_iir2_abs_gain(5.0, 0.0, 10) == -1.0
    assert hb.hb_iir2_abs_gain(3.0, 2.0, 100000) == float("inf") or hb.hb_iir2_abs_gain(3.0, 2.0, 100000) > 1e100


def test_matrix_builtins_appear_only_in_the_wrappers():
    """The stage kernels issue matrix products through the wrappers of hb_device.hpp alone, and the
    K = 16 fp16 shape exists only in the self-check kernel: a kernel cannot mix shapes on an accumulator."""
    csrc = os.path.join(ROOT, "paper_2512_02371_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        text = open(os.path.join(csrc, name)).read()
        text = re.sub(r"//[^\n]*", "", text)
        uses = re.findall(r"__builtin_amdgcn_mfma_\w+", text)
        if name == "hb_device.hpp":
            assert sorted(set(uses)) == ["__builtin_amdgcn_mfma_f32_16x16x32_f16", "__builtin_amdgcn_mfma_f32_16x16x4f32",
                                         "__builtin_amdgcn_mfma_f32_32x32x16_f16"], uses
        elif name == "util.hip":
            assert uses == ["__builtin_amdgcn_mfma_f32_16x16x16f16"], uses
        else:
            assert not uses, f"{name} issues {uses} directly"
        assert "v_mfma" not in re.sub(r"/\*.*?\*/", "", text, flags=re.S), f"{name}: matrix instruction in inline assembly"


def test_sat2d_noalloc_and_wait_limit_validation(lib):
    """The allocation-free entry point checks its arguments and its size limit before it looks the
    array's address up (no GPU needed for these paths); the wait limit is a plain process-wide value."""
    f = lib.hb_sat2d_noalloc
    assert f(None, FAKE, 64, 64, 64, 64, None) == hb.HB_ERR_INVALID_ARG
    assert f(FAKE, None, 64, 64, 64, 64, None) == hb.HB_ERR_INVALID_ARG
    assert f(FAKE, FAKE, 0, 64, 64, 64, None) == hb.HB_ERR_INVALID_ARG
    assert f(FAKE, FAKE, 64, 64, 63, 64, None) == hb.HB_ERR_INVALID_ARG
    assert f(FAKE, FAKE, 64, 64, 64, 10, None) == hb.HB_ERR_INVALID_ARG
    # 4096 x 4096 fits the array, 8192 x 8192 does not
    assert lib.hb_sat2d_workspace_size(4096, 4096) <= hb.HB_SAT2D_NOALLOC_SCRATCH_BYTES
    assert lib.hb_sat2d_workspace_size(8192, 8192) > hb.HB_SAT2D_NOALLOC_SCRATCH_BYTES
    assert f(FAKE, FAKE, 8192, 8192, 8192, 8192, None) == hb.HB_ERR_UNSUPPORTED
    prev = lib.hb_sat2d_set_wait_limit(123)
    try:
        assert lib.hb_sat2d_set_wait_limit(-5) == 123          # returns the previous limit
        assert lib.hb_sat2d_set_wait_limit(0) == 0             # negative: "give up at once" is stored as 0
        assert lib.hb_sat2d_set_wait_limit(7) == 16384         # 0 restored the default
    finally:
        lib.hb_sat2d_set_wait_limit(prev if prev > 0 else 0)
