"""hb_down2 / hb_up2 (resampling by two with an arbitrary 2-D kernel, Sec. V-B) and their vector-ALU
twins against the fp64 oracle."""
import numpy as np
import pytest

from paper_2512_02371_amd import synth
from hbtest import assert_close, padded, up

pytestmark = pytest.mark.gpu

DOWN_CASES = [
    # H, W, kh, kw, ay, ax
    (128, 512, 16, 16, 7, 7),
    (140, 600, 16, 16, 8, 8),     # ragged
    (66, 400, 32, 32, 15, 15),    # maximum kernel
    (80, 666, 32, 32, 31, 31),    # anchors at the far corner
    (80, 666, 32, 32, 0, 0),      # the paper's left/top-anchored form
    (90, 520, 5, 5, 2, 2),        # the pyramid's shape of kernel
    (61, 333, 7, 9, 3, 4),        # odd sizes: the last output row/column reads clamped pixels
    (50, 500, 6, 8, 1, 3),        # odd anchors: the kernel rows split unevenly over the row parities
    (42, 260, 1, 11, 0, 5),       # one kernel row: one parity has no rows at all
    (42, 260, 11, 1, 5, 0),
    (1, 1, 1, 1, 0, 0),
    (5, 9, 32, 32, 16, 16),       # image smaller than the kernel
    (33, 128, 16, 16, 7, 7),      # exactly one strip of outputs
    (47, 2300, 31, 29, 11, 20),
]

UP_CASES = [
    (64, 256, 16, 16, 3, 3),
    (70, 300, 16, 16, 4, 4),      # ragged
    (33, 200, 32, 32, 7, 7),      # maximum kernel
    (40, 170, 32, 32, 15, 15),    # anchors at the far end
    (40, 170, 32, 32, 0, 0),
    (50, 130, 6, 6, 1, 1),        # the pyramid's phases
    (50, 131, 4, 10, 1, 2),       # odd anchor along x
    (21, 250, 2, 2, 0, 0),        # pixel replication weights
    (1, 1, 2, 2, 0, 0),
    (3, 5, 32, 32, 8, 8),         # image smaller than the kernel
    (16, 32, 16, 16, 3, 3),       # exactly one strip
    (31, 550, 30, 28, 5, 10),
]


def run(fn, H, W, kh, kw, ay, ax, pitch_extra=0, offset=0, seed=0):
    import torch
    from paper_2512_02371_amd import hb
    img = synth.uniform01_f16(8000 + seed + H * 7 + W, (H, W))
    k = synth.random_kernel2d_f16(8100 + seed + kh * 33 + kw, kh, kw)
    d_in = up(img)
    if pitch_extra or offset:
        base = torch.full((H, W + pitch_extra + offset), 3.0, dtype=torch.float16, device="cuda:0")
        base[:, offset:offset + W] = d_in
        d_in = base[:, offset:offset + W]
    Ho, Wo = ((H + 1) // 2, (W + 1) // 2) if "down" in fn else (2 * H, 2 * W)
    obuf, out = padded(torch.zeros((Ho, Wo), dtype=torch.float32, device="cuda:0"), Wo + pitch_extra)
    print(f"{fn} H={H} W={W} k={kh}x{kw} a=({ay},{ax}) pitch+{pitch_extra} off={offset}", flush=True)
    getattr(hb, fn)(d_in, out, k, ay, ax)
    torch.cuda.synchronize()
    return img, k, out.cpu().numpy(), obuf.cpu().numpy(), Wo


@pytest.mark.parametrize("fn", ["hb_down2", "hb_down2_valu"])
@pytest.mark.parametrize("H,W,kh,kw,ay,ax", DOWN_CASES)
def test_down2_matches_oracle(orc, fn, H, W, kh, kw, ay, ax):
    img, k, got, _, _ = run(fn, H, W, kh, kw, ay, ax)
    assert_close(got, orc.down2(img, k, ay, ax), f"{fn} {H}x{W} k={kh}x{kw} a=({ay},{ax})")


@pytest.mark.parametrize("fn", ["hb_up2", "hb_up2_valu"])
@pytest.mark.parametrize("H,W,kh,kw,ay,ax", UP_CASES)
def test_up2_matches_oracle(orc, fn, H, W, kh, kw, ay, ax):
    img, k, got, _, _ = run(fn, H, W, kh, kw, ay, ax)
    assert_close(got, orc.up2(img, k, ay, ax), f"{fn} {H}x{W} k={kh}x{kw} a=({ay},{ax})")


@pytest.mark.parametrize("fn", ["hb_down2", "hb_down2_valu", "hb_up2", "hb_up2_valu"])
@pytest.mark.parametrize("extra,offset", [(8, 0), (3, 0), (5, 1), (12, 8)])
def test_resample2_pitched_and_misaligned_layouts(orc, fn, extra, offset):
    H, W, kh, kw, ay, ax = 40, 330, 10, 12, 3, 4
    img, k, got, obuf, Wo = run(fn, H, W, kh, kw, ay, ax, pitch_extra=extra, offset=offset)
    ref = orc.down2(img, k, ay, ax) if "down" in fn else orc.up2(img, k, ay, ax)
    assert_close(got, ref, f"{fn} pitch+{extra} off {offset}")
    assert np.all(obuf[:, Wo:] == 7.0), "wrote past the row end"


@pytest.mark.parametrize("fn", ["hb_down2", "hb_down2_valu"])
def test_down2_impulse(fn):
    """Needs no oracle: an impulse gives every second tap of the mirrored kernel, exactly."""
    import torch
    from paper_2512_02371_amd import hb
    kh, kw, ay, ax, H, W = 6, 9, 2, 5, 60, 400
    k = synth.random_kernel2d_f16(12, kh, kw)
    K = synth.f16_bits_to_f64(k)
    img = torch.zeros((H, W), dtype=torch.float16, device="cuda:0")
    r0, c0 = 31, 203
    img[r0, c0] = 1.0
    out = torch.empty((H // 2, W // 2), dtype=torch.float32, device="cuda:0")
    getattr(hb, fn)(img, out, k, ay, ax)
    expect = np.zeros((H // 2, W // 2))
    for y in range(H // 2):
        for x in range(W // 2):
            ry, rx = r0 - 2 * y + ay, c0 - 2 * x + ax
            if 0 <= ry < kh and 0 <= rx < kw:
                expect[y, x] = K[ry, rx]
    assert np.array_equal(out.cpu().numpy().astype(np.float64), expect)


@pytest.mark.parametrize("fn", ["hb_up2", "hb_up2_valu"])
def test_up2_constant_image_gives_phase_sums(fn):
    import torch
    from paper_2512_02371_amd import hb
    kh, kw = 8, 6
    k = synth.random_kernel2d_f16(13, kh, kw)
    K = synth.f16_bits_to_f64(k)
    img = torch.full((40, 100), 0.25, dtype=torch.float16, device="cuda:0")
    out = torch.empty((80, 200), dtype=torch.float32, device="cuda:0")
    getattr(hb, fn)(img, out, k, 1, 2)
    got = out.cpu().numpy()
    for dy in range(2):
        for dx in range(2):
            assert np.allclose(got[dy::2, dx::2], 0.25 * K[dy::2, dx::2].sum(), atol=1e-6)


def test_down2_full_size_sampled_bands(orc):
    """32 x 32 taps, 4096 x 4096 -> 2048 x 2048 (the launch the benchmark's supplementary line times)."""
    import torch
    from paper_2512_02371_amd import hb
    H = W = 4096
    kh = kw = 32
    ay = ax = 15
    img = synth.uniform01_f16(8777, (H, W))
    k = synth.random_kernel2d_f16(8778, kh, kw)
    out = torch.empty((H // 2, W // 2), dtype=torch.float32, device="cuda:0")
    print("hb_down2 4096x4096 k=32x32", flush=True)
    hb.hb_down2(up(img), out, k, ay, ax)
    torch.cuda.synchronize()
    # output rows [lo, hi) need input rows 2 lo - ay .. 2 (hi - 1) + kh - 1 - ay; bands start on even input rows
    for lo, hi in ((0, 16), (1016, 1040), (H // 2 - 16, H // 2)):
        a = max(0, 2 * lo - ay - 1) & ~1
        b = min(H, 2 * (hi - 1) + kh - ay)
        ref = orc.down2(img[a:b], k, ay, ax)               # its row j is output row a / 2 + j
        ys = [y for y in range(lo, hi) if (2 * y - ay >= a or a == 0) and (2 * y + kh - 1 - ay < b or b == H)]
        got = out[ys[0]:ys[-1] + 1].cpu().numpy()
        assert_close(got, ref[ys[0] - a // 2:ys[-1] + 1 - a // 2], f"rows {ys[0]}..{ys[-1]}")


def test_up2_full_size_sampled_bands(orc):
    """32 x 32 taps, 2048 x 2048 -> 4096 x 4096."""
    import torch
    from paper_2512_02371_amd import hb
    H = W = 2048
    kh = kw = 32
    ay = ax = 7
    img = synth.uniform01_f16(8877, (H, W))
    k = synth.random_kernel2d_f16(8878, kh, kw)
    out = torch.empty((2 * H, 2 * W), dtype=torch.float32, device="cuda:0")
    print("hb_up2 2048x2048 k=32x32", flush=True)
    hb.hb_up2(up(img), out, k, ay, ax)
    torch.cuda.synchronize()
    # input-row bands [lo, hi): output rows 2 lo .. 2 hi - 1 need input rows lo - ay .. hi - 1 + kh/2 - 1 - ay
    for lo, hi in ((0, 12), (1018, 1034), (H - 12, H)):
        a, b = max(0, lo - ay), min(H, hi + kh // 2 - 1 - ay)
        ref = orc.up2(img[a:b], k, ay, ax)
        ys = [y for y in range(lo, hi) if (y - ay >= a or a == 0) and (y + kh // 2 - 1 - ay < b or b == H)]
        got = out[2 * ys[0]:2 * ys[-1] + 2].cpu().numpy()
        assert_close(got, ref[2 * (ys[0] - a):2 * (ys[-1] + 1 - a)], f"input rows {ys[0]}..{ys[-1]}")
