"""hb_sepblur / hb_sepblur_valu against the fp64 oracle, element by element."""
import numpy as np
import pytest

from paper_2512_02371_amd import synth
from hbtest import assert_close, padded, up

pytestmark = pytest.mark.gpu

CASES = [
    # H, W, Tx, ax, Ty, ay
    (64, 64, 16, 7, 16, 7),
    (37, 53, 16, 7, 16, 7),
    (1, 1, 1, 0, 1, 0),
    (3, 200, 5, 2, 1, 0),
    (130, 300, 16, 7, 16, 7),      # several strips and row segments, ragged tail
    (100, 70, 8, 0, 2, 1),
    (70, 100, 17, 16, 17, 0),
    (90, 80, 18, 3, 18, 9),        # three row tiles in the column window
    (90, 80, 33, 32, 33, 16),
    (120, 150, 34, 10, 34, 20),    # four
    (120, 150, 50, 25, 50, 49),    # five
    (160, 96, 64, 31, 64, 32),     # maximum taps
    (160, 96, 64, 0, 64, 63),
]


def run(fn, H, W, Tx, ax, Ty, ay, pitch_extra=0):
    import torch
    from paper_2512_02371_amd import hb
    img = synth.uniform01_f16(3000 + H * 7 + W, (H, W))
    tx = synth.gaussian_taps_f16(Tx, max(Tx / 5.0, 0.5))
    ty = synth.random_taps_f16(4000 + Ty, Ty)
    d_in = up(img)
    if pitch_extra:
        _, d_in = padded(d_in, W + pitch_extra)
    obuf, out = padded(torch.zeros((H, W), dtype=torch.float32, device="cuda:0"), W + pitch_extra)
    print(f"{fn} H={H} W={W} Tx={Tx} ax={ax} Ty={Ty} ay={ay} pitch+{pitch_extra}", flush=True)
    getattr(hb, fn)(d_in, out, tx, ax, ty, ay)
    torch.cuda.synchronize()
    return img, tx, ty, out.cpu().numpy(), obuf.cpu().numpy()


@pytest.mark.parametrize("fn", ["hb_sepblur", "hb_sepblur_valu"])
@pytest.mark.parametrize("H,W,Tx,ax,Ty,ay", CASES)
def test_sepblur_matches_oracle(orc, fn, H, W, Tx, ax, Ty, ay):
    img, tx, ty, got, _ = run(fn, H, W, Tx, ax, Ty, ay)
    assert_close(got, orc.sepblur(img, tx, ax, ty, ay), f"{fn} {H}x{W}")


@pytest.mark.parametrize("fn", ["hb_sepblur", "hb_sepblur_valu"])
@pytest.mark.parametrize("extra", [8, 3])
def test_sepblur_pitched_layouts(orc, fn, extra):
    H, W = 50, 150
    img, tx, ty, got, obuf = run(fn, H, W, 16, 7, 16, 7, pitch_extra=extra)
    assert_close(got, orc.sepblur(img, tx, 7, ty, 7), f"{fn} pitch+{extra}")
    assert np.all(obuf[:, W:] == 7.0), "wrote past the row end"


@pytest.mark.parametrize("fn", ["hb_sepblur", "hb_sepblur_valu"])
def test_sepblur_benchmark_shape_rows_sampled_densely(orc, fn):
    """A 512-row slab of the 4096-wide benchmark image: same strip count as the full
    configuration, several row segments, compared in full."""
    import torch
    from paper_2512_02371_amd import hb
    H, W = 512, 4096
    img = synth.uniform01_f16(1002, (H, W))
    t = synth.gaussian_taps_f16(16, 3.0)
    out = torch.zeros((H, W), dtype=torch.float32, device="cuda:0")
    getattr(hb, fn)(up(img), out, t, 7, t, 7)
    torch.cuda.synchronize()
    assert_close(out.cpu().numpy(), orc.sepblur(img, t, 7, t, 7), fn)


def test_sepblur_full_benchmark_size_sampled_bands(orc):
    """The benchmark's 4096 x 4096 launch, checked on row bands: the oracle runs on a crop with 16
    rows of margin (more than the 15-row reach of the column pass), whose inner rows do not see the crop."""
    import torch
    from paper_2512_02371_amd import hb
    H = W = 4096
    img = synth.uniform01_f16(1002, (H, W))
    t = synth.gaussian_taps_f16(16, 3.0)
    out = torch.zeros((H, W), dtype=torch.float32, device="cuda:0")
    print(f"hb_sepblur {H}x{W}", flush=True)
    hb.hb_sepblur(up(img), out, t, 7, t, 7)
    torch.cuda.synchronize()
    for y0 in (0, 48, 1000, 2047, 3333, H - 80):
        lo, hi = max(y0 - 16, 0), min(y0 + 80 + 16, H)
        ref = orc.sepblur(img[lo:hi], t, 7, t, 7)
        a, b = (0 if lo == 0 else 16), (hi - lo if hi == H else hi - lo - 16)
        assert_close(out[lo + a:lo + b].cpu().numpy(), ref[a:b], f"rows {lo + a}..{lo + b}")
