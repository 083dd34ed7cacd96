"""hb_resize / hb_resize_valu (resampling with banded matrices, Sec. V-C) against the fp64 oracle.
Both sides apply the SAME fp16 matrices (built by hb_lanczos3_matrix or drawn at random)."""
import numpy as np
import pytest

from paper_2512_02371_amd import synth
from hbtest import assert_close, up

pytestmark = pytest.mark.gpu


def run(fn, img, sy, cy, sx, cx, pitch_extra=0):
    """img: [C, H, W] fp16 bits; matrices as host arrays.  Returns the [C, Ho, Wo] result and its canary columns."""
    import torch
    from paper_2512_02371_amd import hb
    C, H, W = img.shape
    Ho, Wo = cy.shape[0], cx.shape[0]
    d_in = up(img)
    if pitch_extra:
        base = torch.full((C, H + 1, W + pitch_extra), 3.0, dtype=torch.float16, device="cuda:0")
        base[:, :H, :W] = d_in
        d_in = base[:, :H, :W]
    obuf = torch.full((C, Ho + 1, Wo + pitch_extra), 7.0, dtype=torch.float32, device="cuda:0")
    out = obuf[:, :Ho, :Wo]
    ws = torch.empty(hb.hb_resize_workspace_size(C, H, Wo), dtype=torch.uint8, device="cuda:0")
    dev = lambda a, t: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0").view(t) if t else torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    d_sy, d_sx = dev(sy.astype(np.int32), None), dev(sx.astype(np.int32), None)
    d_cy, d_cx = dev(cy.view(np.int16), torch.float16), dev(cx.view(np.int16), torch.float16)
    print(f"{fn} C={C} {H}x{W} -> {Ho}x{Wo} bands {cy.shape[1]},{cx.shape[1]} pitch+{pitch_extra}", flush=True)
    getattr(hb, fn)(d_in, out, ws, d_sy, d_cy, d_sx, d_cx)
    torch.cuda.synchronize()
    return out.cpu().numpy(), obuf.cpu().numpy()


def lanczos(hb, n_in, n_out):
    return hb.hb_lanczos3_matrix(n_in, n_out)


@pytest.mark.parametrize("fn", ["hb_resize", "hb_resize_valu"])
@pytest.mark.parametrize("C,H,W,Ho,Wo", [
    (3, 256, 256, 115, 115),      # the paper's factors 2.22 .. 14.3 on a smaller image
    (3, 256, 320, 56, 70),
    (1, 300, 200, 31, 18),        # factor ~10: bands of 59 and 67 samples, groups span > 200 samples
    (2, 130, 190, 130, 190),      # same size: the identity matrix with its 7-sample band
    (1, 97, 131, 45, 100),        # ragged everything
    (3, 64, 64, 1, 1),            # one output sample
    (2, 254, 175, 3, 154),        # factor 85: band 509, the three rows together span 679 samples (two rounds)
    (1, 40, 1300, 30, 16),        # factor 81 along x: one group of 16 outputs spans the whole row (three rounds)
    (1, 1, 1, 1, 1),
])
def test_resize_lanczos_matches_oracle(orc, fn, C, H, W, Ho, Wo):
    from paper_2512_02371_amd import hb
    img = synth.uniform01_f16(9000 + H + 3 * W, (C, H, W))
    sy, cy = lanczos(hb, H, Ho)
    sx, cx = lanczos(hb, W, Wo)
    got, _ = run(fn, img, sy, cy, sx, cx)
    for c in range(C):
        assert_close(got[c], orc.band_resize(img[c], sy, cy, sx, cx), f"{fn} plane {c} {H}x{W}->{Ho}x{Wo}")


@pytest.mark.parametrize("fn", ["hb_resize", "hb_resize_valu"])
def test_resize_random_bands_and_irregular_starts(orc, fn):
    """Not a Lanczos matrix: random coefficients, starts that jump, repeat and leave the image on both sides."""
    C, H, W, Ho, Wo, by, bx = 2, 150, 210, 70, 90, 9, 14
    img = synth.uniform01_f16(9100, (C, H, W))
    cy = synth.random_kernel2d_f16(9101, Ho, by) .view(np.uint16)
    cx = synth.random_kernel2d_f16(9102, Wo, bx).view(np.uint16)
    # scale the rows back up (the generator normalises the whole array to sum |k| = 1)
    cy = (cy.view(np.float16).astype(np.float64) * Ho).astype(np.float16).view(np.uint16)
    cx = (cx.view(np.float16).astype(np.float64) * Wo).astype(np.float16).view(np.uint16)
    h = synth.hash_u64(9103, 0, Ho + Wo)
    sy = (np.arange(Ho) * 2 + (h[:Ho] % np.uint64(13)).astype(np.int64) - 8).astype(np.int32)
    sx = (np.arange(Wo) * 2 + (h[Ho:] % np.uint64(40)).astype(np.int64) - 15).astype(np.int32)
    sy[-1], sx[-1] = H + 5, W - 3                      # entirely / partly past the far edge
    got, _ = run(fn, img, sy, cy, sx, cx)
    for c in range(C):
        assert_close(got[c], orc.band_resize(img[c], sy, cy, sx, cx), f"{fn} plane {c}")


@pytest.mark.parametrize("fn", ["hb_resize", "hb_resize_valu"])
def test_resize_starts_far_apart_and_far_outside(orc, fn):
    """Starts of one group scattered over a long row (several rounds of the coefficient block) and
    starts far outside the image on both sides (every sample clamps to the first / last pixel)."""
    C, H, W, Ho, Wo, by, bx = 1, 70, 3000, 20, 40, 5, 33
    img = synth.uniform01_f16(9400, (C, H, W))
    cy = (synth.random_kernel2d_f16(9401, Ho, by).view(np.float16).astype(np.float64) * Ho).astype(np.float16).view(np.uint16)
    cx = (synth.random_kernel2d_f16(9402, Wo, bx).view(np.float16).astype(np.float64) * Wo).astype(np.float16).view(np.uint16)
    h = synth.hash_u64(9403, 0, Ho + Wo)
    sy = ((h[:Ho] % np.uint64(H + 20)).astype(np.int64) - 10).astype(np.int32)
    sx = ((h[Ho:] % np.uint64(W + 100)).astype(np.int64) - 50).astype(np.int32)
    sx[0], sx[1], sx[17], sx[18] = -(1 << 30), 1 << 30, -5000, 7000
    sy[0], sy[1] = -(2 ** 31), 2 ** 31 - 1
    got, _ = run(fn, img, sy, cy, sx, cx)
    assert_close(got[0], orc.band_resize(img[0], sy, cy, sx, cx), fn)


@pytest.mark.parametrize("fn", ["hb_resize", "hb_resize_valu"])
def test_resize_pitched_planes(orc, fn):
    from paper_2512_02371_amd import hb
    C, H, W, Ho, Wo = 2, 140, 203, 50, 77
    img = synth.uniform01_f16(9200, (C, H, W))
    sy, cy = lanczos(hb, H, Ho)
    sx, cx = lanczos(hb, W, Wo)
    got, obuf = run(fn, img, sy, cy, sx, cx, pitch_extra=5)
    for c in range(C):
        assert_close(got[c], orc.band_resize(img[c], sy, cy, sx, cx), f"{fn} plane {c}")
    assert np.all(obuf[:, :, Wo:] == 7.0) and np.all(obuf[:, Ho:, :] == 7.0), "wrote outside the output planes"


def test_resize_full_size(orc):
    """The paper's workload: a 2048 x 2048 RGB image to 143, 245, 450 and 921 squared; one plane each is
    compared in full (the oracle needs ~1 s per plane at the largest size)."""
    from paper_2512_02371_amd import hb
    C, H, W = 3, 2048, 2048
    img = synth.uniform01_f16(9300, (C, H, W))
    for n, c in ((143, 0), (245, 1), (450, 2), (921, 0)):
        s, k = lanczos(hb, H, n)
        got, _ = run("hb_resize", img, s, k, s, k)
        assert_close(got[c], orc.band_resize(img[c], s, k, s, k), f"2048 -> {n}, plane {c}")
