"""hb_dct_denoise / hb_dct_denoise_valu (DCT-domain coring, Sec. V-E) against the fp64 oracle.

The hard threshold makes a bin whose magnitude is within rounding distance of the threshold
flip between kept and cut; the oracle marks the pixels of every tile that has such a bin (margin
2e-5, more than ten times the fp32 error of a bin) and those pixels may differ from the oracle by what the
near-threshold bins of their tiles can move them (a bound computed per pixel from the number of
such bins, the transform's largest entry and the blend weights); all other pixels meet the usual
tolerance."""
import numpy as np
import pytest

from paper_2512_02371_amd import synth
from hbtest import assert_close, scaled_err, up, TOL

pytestmark = pytest.mark.gpu

MARGIN = 2e-5


def noisy_image(seed, C, H, W):
    """A smooth ramp plus small uniform noise, on the fp16 grid, in [0, 1)."""
    yy, xx = np.meshgrid(np.arange(H), np.arange(W), indexing="ij")
    base = 0.25 + 0.5 * (yy / H) * (xx / W)
    noise = synth.f16_bits_to_f64(synth.uniform_pm1_f16(seed, (C, H, W))) * 0.04
    return synth.f64_to_f16_bits(np.clip(base[None] + noise, 0.0, 0.999))


def run(fn, img, threshold, pitch_extra=0):
    import torch
    from paper_2512_02371_amd import hb
    C, H, W = img.shape
    d_in = up(img)
    if pitch_extra:
        base = torch.full((C, H + 1, W + pitch_extra), 3.0, dtype=torch.float16, device="cuda:0")
        base[:, :H, :W] = d_in
        d_in = base[:, :H, :W]
    obuf = torch.full((C, H + 1, W + pitch_extra), 7.0, dtype=torch.float32, device="cuda:0")
    out = obuf[:, :H, :W]
    ws = torch.empty(hb.hb_dct_denoise_workspace_size(C, H, W), dtype=torch.uint8, device="cuda:0")
    print(f"{fn} C={C} {H}x{W} threshold={threshold} pitch+{pitch_extra}", flush=True)
    getattr(hb, fn)(d_in, out, threshold, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy(), obuf.cpu().numpy()


def flip_bound(orc, plane_bits, thr):
    """Per pixel, the most that bins flipping between kept and cut can move the output.  A bin of
    magnitude |Y| <= thr + MARGIN reaches a pixel of its tile through D[u][i] D[v][j], at most
    (sqrt(2)/4)^2 = 1/8 in magnitude, so a tile with n bins near the threshold moves its
    reconstruction by at most n (thr + MARGIN) / 8 anywhere; the blend weighs tile t by
    w2_t / sum_t w2_t^2.  (The forward transform is redone here only to COUNT the near bins.)"""
    X = synth.f16_bits_to_f64(plane_bits)
    H, W = X.shape
    D, w = orc.dct16_matrix(), orc.sine_window16()
    w2 = np.outer(w, w)
    tiles = np.lib.stride_tricks.sliding_window_view(X, (16, 16))[::8, ::8]           # [ty, tx, 16, 16]
    Y = np.einsum("ui,abij,vj->abuv", D, tiles * w2, D, optimize=True)
    near = np.abs(np.abs(Y) - thr) < MARGIN
    near[:, :, 0, 0] = False
    n = near.sum(axis=(2, 3)).astype(np.float64)
    num = np.zeros((H, W))
    den = np.zeros((H, W))
    for ty in range(n.shape[0]):
        for tx in range(n.shape[1]):
            ys, xs = slice(8 * ty, 8 * ty + 16), slice(8 * tx, 8 * tx + 16)
            den[ys, xs] += w2 * w2
            if n[ty, tx]:
                num[ys, xs] += n[ty, tx] * w2
    return (thr + MARGIN) / 8.0 * num / den


def check(orc, got, img, threshold, what, max_masked=0.5):
    thr = float(np.float32(threshold))                 # the library receives fp32
    for c in range(img.shape[0]):
        ref, risky = orc.dct_denoise(img[c], thr, margin=MARGIN if thr > 0 else 0.0)   # nothing can flip at threshold 0
        g = got[c]
        assert np.all(np.isfinite(g)), what
        e = scaled_err(g, ref)
        assert e[~risky].max(initial=0.0) <= TOL, f"{what} plane {c}: {e[~risky].max():.3e}"
        print(f"{what} plane {c}: {risky.mean():.4f} of the pixels lie in a tile with a bin within {MARGIN} of the "
              f"threshold", flush=True)
        assert risky.mean() < max_masked, "the margin should not swallow the test"
        if risky.any():
            # those pixels: within the usual tolerance plus what the flipped bins can move them
            bound = flip_bound(orc, img[c], thr)
            assert np.all((bound > 0) == risky), "the near-threshold tiles counted here are not the oracle's"
            slack = np.abs(g - ref) - TOL * np.maximum(1.0, np.abs(ref)) - bound
            assert slack[risky].max() <= 0.0, f"{what} plane {c}: {slack[risky].max():.3e} beyond the flip bound"


@pytest.mark.parametrize("fn", ["hb_dct_denoise", "hb_dct_denoise_valu"])
@pytest.mark.parametrize("C,H,W,thr", [
    (1, 16, 16, 0.05),        # a single tile
    (1, 64, 64, 0.0),         # no coring: the identity
    (3, 64, 96, 0.05),
    (2, 128, 72, 0.2),        # strong coring: most of the noise bins go
    (1, 24, 40, 1000.0),      # only DC survives
    (1, 200, 136, 0.03),
])
def test_dct_denoise_matches_oracle(orc, fn, C, H, W, thr):
    img = noisy_image(9800 + H + W, C, H, W)
    got, _ = run(fn, img, thr)
    check(orc, got, img, thr, f"{fn} {C}x{H}x{W} thr {thr}")


@pytest.mark.parametrize("fn", ["hb_dct_denoise", "hb_dct_denoise_valu"])
def test_dct_denoise_identity_at_threshold_zero(fn):
    """Needs no oracle: with nothing cut the windows' overlap identity gives the image back."""
    img = noisy_image(9850, 2, 80, 112)
    got, _ = run(fn, img, 0.0)
    assert np.max(np.abs(got - synth.f16_bits_to_f64(img))) < 2e-5


@pytest.mark.parametrize("fn", ["hb_dct_denoise", "hb_dct_denoise_valu"])
def test_dct_denoise_pitched_planes(orc, fn):
    img = noisy_image(9860, 2, 48, 56)
    got, obuf = run(fn, img, 0.05, pitch_extra=5)
    check(orc, got, img, 0.05, fn)
    assert np.all(obuf[:, :, 56:] == 7.0) and np.all(obuf[:, 48:, :] == 7.0), "wrote outside the output planes"


def test_dct_denoise_reduces_noise():
    """What the stage is for: on a smooth image with added noise the result is closer to the smooth image."""
    C, H, W = 1, 256, 256
    yy, xx = np.meshgrid(np.arange(H), np.arange(W), indexing="ij")
    clean = 0.25 + 0.5 * (yy / H) * (xx / W)
    img = noisy_image(9870, C, H, W)
    got, _ = run("hb_dct_denoise", img, 0.08)
    before = np.sqrt(np.mean((synth.f16_bits_to_f64(img)[0] - clean) ** 2))
    after = np.sqrt(np.mean((got[0, 16:-16, 16:-16] - clean[16:-16, 16:-16]) ** 2))
    assert after < 0.5 * before


def test_dct_denoise_full_size(orc):
    """The paper's workload: a one-megapixel three-channel image; one plane is compared in full."""
    C, H, W = 3, 1024, 1024
    img = noisy_image(9880, C, H, W)
    got, _ = run("hb_dct_denoise", img, 0.05)
    check(orc, got[1:2], img[1:2], 0.05, "3 x 1024 x 1024, plane 1", max_masked=0.15)
