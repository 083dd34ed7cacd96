"""hb_conv2d / hb_conv2d_valu (arbitrary 2-D kernel, Sec. V-A 2-D form) against the fp64 oracle."""
import numpy as np
import pytest

from paper_2512_02371_amd import synth
from hbtest import assert_close, padded, up

pytestmark = pytest.mark.gpu

CASES = [
    # H, W, kh, kw, ay, ax
    (64, 256, 16, 16, 7, 7),      # one window chunk per tile
    (70, 300, 16, 16, 8, 8),      # ragged rows and columns
    (33, 200, 32, 32, 15, 15),    # maximum kernel, two window chunks
    (40, 333, 32, 32, 31, 31),    # anchors at the far corner
    (40, 333, 32, 32, 0, 0),      # the paper's left/top-anchored form
    (50, 260, 5, 7, 1, 4),        # odd anchor: the window is moved to an even pixel
    (50, 260, 7, 17, 3, 8),       # 17 taps per row: needs the second chunk
    (21, 500, 1, 9, 0, 4),        # a single kernel row (a row-wise FIR)
    (90, 190, 9, 1, 4, 0),        # a single kernel column
    (17, 130, 3, 3, 1, 1),
    (1, 1, 1, 1, 0, 0),           # degenerate
    (3, 5, 32, 32, 16, 16),       # image smaller than the kernel: all clamps
    (16, 64, 16, 16, 7, 7),       # exactly one strip wide: border kernel only
    (48, 128, 16, 16, 7, 7),      # two strips wide
    (31, 1100, 31, 29, 11, 20),
]


def run(fn, H, W, kh, kw, ay, ax, pitch_extra=0, offset=0, seed=0):
    import torch
    from paper_2512_02371_amd import hb
    img = synth.uniform01_f16(7000 + seed + H * 7 + W, (H, W))
    k = synth.random_kernel2d_f16(7100 + seed + kh * 33 + kw, kh, kw)
    d_in = up(img)
    if pitch_extra or offset:
        base = torch.full((H, W + pitch_extra + offset), 3.0, dtype=torch.float16, device="cuda:0")
        base[:, offset:offset + W] = d_in
        d_in = base[:, offset:offset + W]
    obuf, out = padded(torch.zeros((H, W), dtype=torch.float32, device="cuda:0"), W + pitch_extra)
    print(f"{fn} H={H} W={W} k={kh}x{kw} a=({ay},{ax}) pitch+{pitch_extra} off={offset}", flush=True)
    getattr(hb, fn)(d_in, out, k, ay, ax)
    torch.cuda.synchronize()
    return img, k, out.cpu().numpy(), obuf.cpu().numpy()


@pytest.mark.parametrize("fn", ["hb_conv2d", "hb_conv2d_valu"])
@pytest.mark.parametrize("H,W,kh,kw,ay,ax", CASES)
def test_conv2d_matches_oracle(orc, fn, H, W, kh, kw, ay, ax):
    img, k, got, _ = run(fn, H, W, kh, kw, ay, ax)
    assert_close(got, orc.conv2d(img, k, ay, ax), f"{fn} {H}x{W} k={kh}x{kw} a=({ay},{ax})")


@pytest.mark.parametrize("fn", ["hb_conv2d", "hb_conv2d_valu"])
@pytest.mark.parametrize("extra,offset", [(8, 0), (3, 0), (5, 1), (12, 8)])
def test_conv2d_pitched_and_misaligned_layouts(orc, fn, extra, offset):
    H, W, kh, kw, ay, ax = 40, 330, 11, 13, 5, 6
    img, k, got, obuf = run(fn, H, W, kh, kw, ay, ax, pitch_extra=extra, offset=offset)
    assert_close(got, orc.conv2d(img, k, ay, ax), f"{fn} pitch+{extra} off {offset}")
    assert np.all(obuf[:, W:] == 7.0), "wrote past the row end"


@pytest.mark.parametrize("fn", ["hb_conv2d", "hb_conv2d_valu"])
def test_conv2d_impulse_and_constant(fn):
    """Invariants that need no oracle: an impulse gives the mirrored kernel, a constant image the tap sum."""
    import torch
    from paper_2512_02371_amd import hb
    kh, kw, ay, ax, H, W = 6, 9, 2, 5, 40, 200
    k = synth.random_kernel2d_f16(11, kh, kw)
    K = synth.f16_bits_to_f64(k)
    img = torch.zeros((H, W), dtype=torch.float16, device="cuda:0")
    y0, x0 = 20, 101
    img[y0, x0] = 1.0
    out = torch.empty((H, W), dtype=torch.float32, device="cuda:0")
    getattr(hb, fn)(img, out, k, ay, ax)
    got = out.cpu().numpy().astype(np.float64)
    expect = np.zeros((H, W))
    for ry in range(kh):
        for rx in range(kw):
            expect[y0 - ry + ay, x0 - rx + ax] = K[ry, rx]
    assert np.array_equal(got, expect)
    img.fill_(0.5)
    getattr(hb, fn)(img, out, k, ay, ax)
    assert np.allclose(out.cpu().numpy(), 0.5 * K.sum(), atol=1e-5)


def test_conv2d_full_size_sampled_bands(orc):
    """32 x 32 taps on 4096 x 4096 (the launch the benchmark's supplementary line times): bands of
    rows at the top, the bottom and a strip seam are compared with the oracle run on the rows they need."""
    import torch
    from paper_2512_02371_amd import hb
    H = W = 4096
    kh = kw = 32
    ay = ax = 15
    img = synth.uniform01_f16(7777, (H, W))
    k = synth.random_kernel2d_f16(7778, kh, kw)
    out = torch.empty((H, W), dtype=torch.float32, device="cuda:0")
    print("hb_conv2d 4096x4096 k=32x32", flush=True)
    hb.hb_conv2d(up(img), out, k, ay, ax)
    torch.cuda.synchronize()
    for lo, hi in ((0, 24), (2040, 2064), (H - 24, H)):
        a, b = max(0, lo - ay), min(H, hi + kh - 1 - ay)
        ref = orc.conv2d(img[a:b], k, ay, ax)
        # rows whose window stays inside [a, b) or clamps at the true image border
        ys = [y for y in range(lo, hi) if (y - ay >= a or a == 0) and (y + kh - 1 - ay < b or b == H)]
        got = out[ys[0]:ys[-1] + 1].cpu().numpy()
        assert_close(got, ref[ys[0] - a:ys[-1] + 1 - a], f"rows {ys[0]}..{ys[-1]}")
