"""Seeded random shapes, taps, anchors, offsets and pitches for every entry point (matrix-unit path and
vector-ALU twin) against the fp64 oracle.  Inputs sit inside NaN-filled buffers at odd element offsets,
outputs inside canary-filled ones: a read outside the image shows up as a non-finite output, a write
outside as a damaged canary."""
import numpy as np
import pytest

from paper_2512_02371_amd import synth
from hbtest import TOL

pytestmark = pytest.mark.gpu

GUARD = 3           # guard rows above and below
CASES = 64          # per entry point and variant


class Draw:
    def __init__(self, seed):
        self.rng = np.random.default_rng(seed)

    def i(self, a, b):
        return int(self.rng.integers(a, b + 1))

    def seed(self):
        return self.i(0, 1 << 20)


def in_view(d, bits):
    import torch
    H, W = bits.shape
    off, extra = d.i(0, 9), d.i(0, 9)
    base = torch.full((H + 2 * GUARD, off + W + extra), float("nan"), dtype=torch.float16, device="cuda:0")
    base[GUARD:GUARD + H, off:off + W] = torch.from_numpy(np.ascontiguousarray(bits).view(np.float16)).to("cuda:0")
    return base[GUARD:GUARD + H, off:off + W]


def out_view(d, H, W, dtype=None):
    import torch
    off, extra = 4 * d.i(0, 2), d.i(0, 9)
    base = torch.full((H + 2 * GUARD, off + W + extra), 7.0, dtype=dtype or torch.float32, device="cuda:0")
    return base, base[GUARD:GUARD + H, off:off + W]


def verify(what, base, view, ref, scale=None):
    import torch
    torch.cuda.synchronize()
    got = view.cpu().numpy().astype(np.float64)
    H, W = view.shape
    whole = base.cpu().numpy().astype(np.float64)
    off = view.storage_offset() % base.shape[1]
    outside = np.ones(whole.shape, bool)
    outside[GUARD:GUARD + H, off:off + W] = False
    assert np.all(whole[outside] == 7.0), f"{what}: wrote outside the output"
    assert np.all(np.isfinite(got)), f"{what}: non-finite output (a read outside the image?)"
    err = np.abs(got - ref) / (scale if scale is not None else np.maximum(1.0, np.abs(ref)))
    i = np.unravel_index(np.argmax(err), err.shape)
    assert err[i] <= TOL, f"{what}: max scaled error {err[i]:.3e} at {i}"


@pytest.mark.parametrize("v", ["", "_valu"])
def test_random_fir1d(orc, v):
    from paper_2512_02371_amd import hb
    d = Draw(101 + len(v))
    for _ in range(CASES):
        H, W = d.i(1, 90), d.i(1, 700)
        T = d.i(1, 256) if d.i(0, 2) == 0 else d.i(1, 64)
        a = d.i(0, T - 1)
        img, taps = synth.uniform01_f16(d.seed(), (H, W)), synth.random_taps_f16(d.seed(), T)
        what = f"hb_fir1d{v} H={H} W={W} T={T} a={a}"
        print(what, flush=True)
        base, out = out_view(d, H, W)
        getattr(hb, "hb_fir1d" + v)(in_view(d, img), out, taps, a)
        verify(what, base, out, orc.fir1d(img, taps, a))


@pytest.mark.parametrize("v", ["", "_valu"])
def test_random_sepblur(orc, v):
    from paper_2512_02371_amd import hb
    d = Draw(201 + len(v))
    for _ in range(CASES):
        H, W, tx, ty = d.i(1, 150), d.i(1, 500), d.i(1, 64), d.i(1, 64)
        ax, ay = d.i(0, tx - 1), d.i(0, ty - 1)
        img = synth.uniform01_f16(d.seed(), (H, W))
        kx, ky = synth.random_taps_f16(d.seed(), tx), synth.random_taps_f16(d.seed(), ty)
        what = f"hb_sepblur{v} H={H} W={W} tx={tx} ax={ax} ty={ty} ay={ay}"
        print(what, flush=True)
        base, out = out_view(d, H, W)
        getattr(hb, "hb_sepblur" + v)(in_view(d, img), out, kx, ax, ky, ay)
        verify(what, base, out, orc.sepblur(img, kx, ax, ky, ay))


@pytest.mark.parametrize("v", ["", "_valu"])
def test_random_sat2d(orc, v):
    import torch
    from paper_2512_02371_amd import hb
    d = Draw(301 + len(v))
    for _ in range(CASES):
        H, W = d.i(1, 300), d.i(1, 500)
        img = synth.uniform01_f16(d.seed(), (H, W))
        what = f"hb_sat2d{v} H={H} W={W}"
        print(what, flush=True)
        base, out = out_view(d, H, W)
        ws = torch.full((hb.hb_sat2d_workspace_size(H, W),), 0xff, dtype=torch.uint8, device="cuda:0")
        getattr(hb, "hb_sat2d" + v)(in_view(d, img), out, ws)
        ref = orc.sat2d(img)
        verify(what, base, out, ref, scale=max(ref[-1, -1], 1e-30))


@pytest.mark.parametrize("v", ["", "_valu"])
def test_random_pyr_level(orc, v):
    import torch
    from paper_2512_02371_amd import hb
    d = Draw(401 + len(v))
    for _ in range(CASES):
        H, W, want = 2 * d.i(1, 120), 2 * d.i(1, 300), d.i(0, 1) == 1
        img = synth.uniform01_f16(d.seed(), (H, W))
        what = f"hb_pyr_level{v} H={H} W={W} down={want}"
        print(what, flush=True)
        base, out = out_view(d, H, W)
        dbase, down = out_view(d, H // 2, W // 2, torch.float16) if want else (None, None)
        getattr(hb, "hb_pyr_level" + v)(in_view(d, img), out, down)
        ref = orc.pyr_level(img, want)
        verify(what, base, out, ref[0] if want else ref)
        if want:
            verify(what + " (down)", dbase, down, ref[1])


@pytest.mark.parametrize("v", ["", "_valu"])
def test_random_conv3x3(orc, v):
    import torch
    from paper_2512_02371_amd import hb
    d = Draw(501 + len(v))
    for _ in range(CASES // 2):
        N, H, W = d.i(1, 2), d.i(1, 40), d.i(1, 70)
        x = synth.uniform_pm1_f16(d.seed(), (N, H, W, 64))
        w = synth.normal_f16(d.seed(), (3, 3, 64, 64), 1.0 / 24.0)
        what = f"hb_conv3x3{v} N={N} H={H} W={W}"
        print(what, flush=True)
        o = torch.full((N + 1, H, W, 64), 7.0, dtype=torch.float16, device="cuda:0")
        up = lambda a: torch.from_numpy(a.view(np.float16)).to("cuda:0")
        getattr(hb, "hb_conv3x3" + v)(up(x), up(w), o[:N])
        torch.cuda.synchronize()
        got, ref = o.cpu().numpy().astype(np.float64), orc.conv3x3(x, w)
        assert np.all(got[N] == 7.0), f"{what}: wrote past the output"
        assert np.all(np.isfinite(got[:N])), f"{what}: non-finite output"
        err = np.abs(got[:N] - ref) / np.maximum(1.0, np.abs(ref))
        assert err.max() <= TOL, f"{what}: max scaled error {err.max():.3e}"


@pytest.mark.parametrize("v", ["", "_valu"])
@pytest.mark.parametrize("kind", ["conv2d", "down2", "up2"])
def test_random_kernel2d_stages(orc, kind, v):
    from paper_2512_02371_amd import hb
    d = Draw(601 + len(v) + 10 * len(kind))
    for _ in range(CASES):
        if kind == "up2":
            kh, kw = 2 * d.i(1, 16), 2 * d.i(1, 16)
            ay, ax = d.i(0, kh // 2 - 1), d.i(0, kw // 2 - 1)
        else:
            kh, kw = d.i(1, 32), d.i(1, 32)
            ay, ax = d.i(0, kh - 1), d.i(0, kw - 1)
        H, W = d.i(1, 100), d.i(1, 500)
        img, k = synth.uniform01_f16(d.seed(), (H, W)), synth.random_kernel2d_f16(d.seed(), kh, kw)
        Ho, Wo = {"conv2d": (H, W), "down2": ((H + 1) // 2, (W + 1) // 2), "up2": (2 * H, 2 * W)}[kind]
        what = f"hb_{kind}{v} H={H} W={W} k={kh}x{kw} a=({ay},{ax})"
        print(what, flush=True)
        base, out = out_view(d, Ho, Wo)
        getattr(hb, "hb_" + kind + v)(in_view(d, img), out, k, ay, ax)
        verify(what, base, out, getattr(orc, kind)(img, k, ay, ax))


@pytest.mark.parametrize("v", ["", "_valu"])
def test_random_resize(orc, v):
    import torch
    from paper_2512_02371_amd import hb
    d = Draw(701 + len(v))
    done = 0
    while done < CASES:
        C, H, W = d.i(1, 3), d.i(1, 260), d.i(1, 400)
        Ho, Wo = d.i(1, H), d.i(1, W)
        if max(hb.hb_lanczos3_band(H, Ho), hb.hb_lanczos3_band(W, Wo)) > 512:
            continue                                   # beyond the largest band the library builds
        done += 1
        sy, cy = hb.hb_lanczos3_matrix(H, Ho)
        sx, cx = hb.hb_lanczos3_matrix(W, Wo)
        imgs = [synth.uniform01_f16(d.seed(), (H, W)) for _ in range(C)]
        what = f"hb_resize{v} C={C} {H}x{W} -> {Ho}x{Wo}"
        print(what, flush=True)
        inp = torch.from_numpy(np.stack(imgs).view(np.float16)).to("cuda:0")
        out = torch.full((C + 1, Ho, Wo), 7.0, dtype=torch.float32, device="cuda:0")
        ws = torch.full((hb.hb_resize_workspace_size(C, H, Wo),), 0xff, dtype=torch.uint8, device="cuda:0")
        di = lambda a: torch.from_numpy(a).to("cuda:0")
        dh = lambda a: torch.from_numpy(a.view(np.int16)).to("cuda:0").view(torch.float16)
        getattr(hb, "hb_resize" + v)(inp, out[:C], ws, di(sy), dh(cy), di(sx), dh(cx))
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        assert np.all(got[C] == 7.0), f"{what}: wrote past the output"
        for c in range(C):
            ref = orc.band_resize(imgs[c], sy, cy, sx, cx)
            assert np.all(np.isfinite(got[c])), f"{what}: non-finite output"
            err = np.abs(got[c] - ref) / np.maximum(1.0, np.abs(ref))
            assert err.max() <= TOL, f"{what} plane {c}: max scaled error {err.max():.3e}"


@pytest.mark.parametrize("v", ["", "_valu"])
def test_random_iir2(orc, v):
    """Filters inside the accuracy domain the header states: complex pairs of radius <= 0.93 away from
    the real axis, or two real poles of magnitude <= 0.9."""
    import torch
    from paper_2512_02371_amd import hb
    d = Draw(801 + len(v))
    for _ in range(CASES):
        C, T = d.i(1, 4), d.i(1, 9000)
        if d.i(0, 1):
            r, th = d.rng.uniform(0.3, 0.93), d.rng.uniform(0.3, np.pi - 0.3)
            alpha, beta = 2 * r * np.cos(th), -r * r
        else:
            p, q = d.rng.uniform(-0.9, 0.9), d.rng.uniform(-0.9, 0.9)
            alpha, beta = p + q, -p * q
        alpha, beta = float(np.float32(alpha)), float(np.float32(beta))
        sig = synth.uniform_pm1_f16(d.seed(), (C, T))
        what = f"hb_iir2{v} C={C} T={T} alpha={alpha} beta={beta}"
        print(what, flush=True)
        y = torch.full((C + 1, T), 7.0, dtype=torch.float32, device="cuda:0")
        ws = torch.full((hb.hb_iir2_workspace_size(C, T),), 0xff, dtype=torch.uint8, device="cuda:0")
        getattr(hb, "hb_iir2" + v)(torch.from_numpy(sig.view(np.float16)).to("cuda:0"), y[:C], alpha, beta, ws)
        torch.cuda.synchronize()
        got, ref = y.cpu().numpy().astype(np.float64), orc.iir2(sig, alpha, beta)
        assert np.all(got[C] == 7.0), f"{what}: wrote past the output"
        assert np.all(np.isfinite(got[:C])), f"{what}: non-finite output"
        err = np.abs(got[:C] - ref) / np.maximum(1.0, np.abs(ref))
        assert err.max() <= TOL, f"{what}: max scaled error {err.max():.3e}"


@pytest.mark.parametrize("v", ["", "_valu"])
def test_random_dct_denoise(orc, v):
    import torch
    from paper_2512_02371_amd import hb
    d = Draw(901 + len(v))
    for _ in range(CASES // 2):
        C, H, W = d.i(1, 2), 8 * d.i(2, 20), 8 * d.i(2, 30)
        thr = [0.0, 0.02, 0.05, 0.2][d.i(0, 3)]
        imgs = [synth.uniform01_f16(d.seed(), (H, W)) for _ in range(C)]
        what = f"hb_dct_denoise{v} C={C} {H}x{W} threshold={thr}"
        print(what, flush=True)
        inp = torch.from_numpy(np.stack(imgs).view(np.float16)).to("cuda:0")
        out = torch.full((C + 1, H, W), 7.0, dtype=torch.float32, device="cuda:0")
        ws = torch.full((hb.hb_dct_denoise_workspace_size(C, H, W),), 0xff, dtype=torch.uint8, device="cuda:0")
        getattr(hb, "hb_dct_denoise" + v)(inp, out[:C], thr, ws)
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        assert np.all(got[C] == 7.0), f"{what}: wrote past the output"
        for c in range(C):
            # bins within the margin of the threshold may fall either way: their pixels are not compared
            ref, risky = orc.dct_denoise(imgs[c], thr, 2e-5 if thr > 0 else 0.0)
            assert np.all(np.isfinite(got[c])), f"{what}: non-finite output"
            err = np.abs(got[c] - ref) / np.maximum(1.0, np.abs(ref))
            err[risky] = 0.0
            assert err.max() <= TOL, f"{what} plane {c}: max scaled error {err.max():.3e}"
