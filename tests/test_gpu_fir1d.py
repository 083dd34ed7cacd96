"""hb_fir1d / hb_fir1d_valu against the fp64 oracle, element by element."""
import numpy as np
import pytest

from paper_2512_02371_amd import synth
from hbtest import assert_close, padded, up

pytestmark = pytest.mark.gpu

CASES = [
    # H, W, T, anchor
    (256, 256, 8, 3),        # the benchmark configuration
    (37, 53, 8, 3),          # ragged in both directions, narrower than one tile
    (1, 1, 1, 0),            # degenerate
    (5, 7, 5, 4),
    (130, 300, 16, 7),       # several tiles plus a ragged tail
    (64, 200, 16, 0),        # the paper's left-anchored form
    (33, 129, 64, 63),
    (33, 129, 64, 0),
    (48, 96, 33, 16),
    (16, 70, 17, 1),
    # the large-tap regime: 4 to 9 windows of 32 pixels per tile, fewer tiles per strip
    (40, 700, 100, 50),
    (40, 700, 128, 0),
    (33, 640, 129, 128),
    (20, 1000, 200, 99),
    (48, 1200, 256, 127),    # maximum taps
    (17, 600, 256, 255),     # rightmost anchor
    (17, 600, 256, 0),
    (9, 250, 256, 100),      # narrower than one window: falls to the vector-ALU kernel
]


def run(fn, H, W, T, a, pitch_extra=0, offset=0, seed=0):
    import torch
    from paper_2512_02371_amd import hb
    img = synth.uniform01_f16(1000 + seed + H * 7 + W, (H, W))
    taps = synth.random_taps_f16(2000 + seed + T, T)
    d_in = up(img)
    if pitch_extra or offset:
        base = torch.full((H, W + pitch_extra + offset), 3.0, dtype=torch.float16, device="cuda:0")
        base[:, offset:offset + W] = d_in
        d_in = base[:, offset:offset + W]
    obuf, out = padded(torch.zeros((H, W), dtype=torch.float32, device="cuda:0"), W + pitch_extra)
    print(f"{fn} H={H} W={W} T={T} a={a} pitch+{pitch_extra} off={offset}", flush=True)
    getattr(hb, fn)(d_in, out, taps, a)
    torch.cuda.synchronize()
    return img, taps, out.cpu().numpy(), obuf.cpu().numpy()


@pytest.mark.parametrize("fn", ["hb_fir1d", "hb_fir1d_valu"])
@pytest.mark.parametrize("H,W,T,a", CASES)
def test_fir1d_matches_oracle(orc, fn, H, W, T, a):
    img, taps, got, _ = run(fn, H, W, T, a)
    assert_close(got, orc.fir1d(img, taps, a), f"{fn} {H}x{W} T={T} a={a}")


@pytest.mark.parametrize("fn", ["hb_fir1d", "hb_fir1d_valu"])
@pytest.mark.parametrize("extra,offset", [(8, 0), (3, 0), (5, 1), (12, 8)])
def test_fir1d_pitched_and_misaligned_layouts(orc, fn, extra, offset):
    H, W, T, a = 40, 150, 8, 3
    img, taps, got, obuf = run(fn, H, W, T, a, pitch_extra=extra, offset=offset)
    assert_close(got, orc.fir1d(img, taps, a), f"{fn} pitch+{extra} off {offset}")
    assert np.all(obuf[:, W:] == 7.0), "wrote past the row end"


def test_fir1d_long_filter_at_blur_size(orc):
    """256 taps on a 512-row slab of a 4096-wide image (the width of the blur benchmark)."""
    img, taps, got, _ = run("hb_fir1d", 512, 4096, 256, 127, seed=9)
    assert_close(got, orc.fir1d(img, taps, 127), "256 taps, 512 x 4096")


@pytest.mark.parametrize("fn", ["hb_fir1d", "hb_fir1d_valu"])
def test_fir1d_impulse_and_constant(fn):
    """Invariants that need no oracle: mirrored taps, tap sum."""
    import torch
    from paper_2512_02371_amd import hb
    T, a, H, W = 8, 3, 20, 100
    taps = synth.random_taps_f16(5, T)
    k = synth.f16_bits_to_f64(taps)
    img = np.zeros((H, W))
    img[7, 50] = 1.0
    out = torch.zeros((H, W), dtype=torch.float32, device="cuda:0")
    getattr(hb, fn)(up(synth.f64_to_f16_bits(img)), out, taps, a)
    got = out.cpu().numpy()
    for x in range(W):
        r = 50 - x + a
        assert got[7, x] == (np.float32(k[r]) if 0 <= r < T else 0.0)
    getattr(hb, fn)(up(synth.f64_to_f16_bits(np.full((H, W), 0.5))), out, taps, a)
    assert np.allclose(out.cpu().numpy(), 0.5 * k.sum(), atol=1e-6)
