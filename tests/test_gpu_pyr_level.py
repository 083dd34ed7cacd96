"""hb_pyr_level / hb_pyr_level_valu against the fp64 oracle, element by element."""
import numpy as np
import pytest

from paper_2512_02371_amd import synth
from hbtest import assert_close, padded, up

pytestmark = pytest.mark.gpu

CASES = [(64, 64), (2, 2), (4, 6), (34, 70), (130, 300), (256, 256), (96, 62), (66, 192), (30, 1026)]


def run(fn, H, W, want_down, pitch_extra=0, seed=0):
    import torch
    from paper_2512_02371_amd import hb
    img = synth.uniform01_f16(5000 + seed + H * 3 + W, (H, W))
    d_in = up(img)
    if pitch_extra:
        _, d_in = padded(d_in, W + pitch_extra)
    rbuf, res = padded(torch.zeros((H, W), dtype=torch.float32, device="cuda:0"), W + pitch_extra)
    dbuf, down = padded(torch.zeros((H // 2, W // 2), dtype=torch.float16, device="cuda:0"), W // 2 + pitch_extra)
    print(f"{fn} H={H} W={W} down={want_down} pitch+{pitch_extra}", flush=True)
    getattr(hb, fn)(d_in, res, down if want_down else None)
    torch.cuda.synchronize()
    return img, res.cpu().numpy(), down.cpu().numpy(), rbuf.cpu().numpy(), dbuf.cpu().numpy()


@pytest.mark.parametrize("fn", ["hb_pyr_level", "hb_pyr_level_valu"])
@pytest.mark.parametrize("H,W", CASES)
def test_pyr_matches_oracle(orc, fn, H, W):
    img, res, down, _, _ = run(fn, H, W, True)
    ref, dref = orc.pyr_level(img, want_down=True)
    assert_close(res, ref, f"{fn} residual {H}x{W}")
    assert_close(down.astype(np.float64), dref, f"{fn} down {H}x{W}")


@pytest.mark.parametrize("fn", ["hb_pyr_level", "hb_pyr_level_valu"])
def test_pyr_without_down_and_with_pitch(orc, fn):
    H, W = 70, 150
    img, res, down, rbuf, dbuf = run(fn, H, W, False, pitch_extra=6)
    assert_close(res, orc.pyr_level(img), f"{fn} pitched")
    assert np.all(rbuf[:, W:] == 7.0) and np.all(dbuf == np.float16(7.0)) or np.all(down == 0), "stray writes"
    assert np.all(down == 0), "down written although not requested"


@pytest.mark.parametrize("pitch_extra", [5, 8])
def test_pyr_pitched_image_with_interior_tasks(orc, pitch_extra):
    """Large enough for interior tasks; an odd pitch puts every second row on a 2-byte boundary."""
    H, W = 130, 300
    img, res, down, rbuf, dbuf = run("hb_pyr_level", H, W, True, pitch_extra=pitch_extra, seed=3)
    ref, dref = orc.pyr_level(img, want_down=True)
    assert_close(res, ref, f"pitched +{pitch_extra} residual")
    assert_close(down.astype(np.float64), dref, f"pitched +{pitch_extra} down")
    assert np.all(rbuf[:, W:] == 7.0), "stray writes beyond the row"


@pytest.mark.parametrize("fn", ["hb_pyr_level", "hb_pyr_level_valu"])
def test_pyr_constant_image_has_zero_residual(fn):
    import torch
    from paper_2512_02371_amd import hb
    H, W = 96, 160
    res = torch.ones((H, W), dtype=torch.float32, device="cuda:0")
    getattr(hb, fn)(up(synth.f64_to_f16_bits(np.full((H, W), 0.75))), res, None)
    assert float(res.abs().max()) == 0.0


@pytest.mark.parametrize("fn", ["hb_pyr_level", "hb_pyr_level_valu"])
def test_pyr_benchmark_width_slab(orc, fn):
    """A 320-row slab at the benchmark's 8192-pixel width: same strips as the full image."""
    import torch
    from paper_2512_02371_amd import hb
    H, W = 320, 8192
    img = synth.uniform01_f16(1005, (H, W))
    res = torch.zeros((H, W), dtype=torch.float32, device="cuda:0")
    getattr(hb, fn)(up(img), res, None)
    torch.cuda.synchronize()
    assert_close(res.cpu().numpy(), orc.pyr_level(img), fn)


@pytest.mark.parametrize("want_down", [False, True])
def test_pyr_full_benchmark_size_sampled_bands(orc, want_down):
    """The benchmark's 8192 x 8192 launch (long interior tasks, many rounds of the tile ring), checked on
    row bands: the oracle runs on a crop with 16 rows of margin, whose inner rows do not see the crop."""
    import torch
    from paper_2512_02371_amd import hb
    H = W = 8192
    img = synth.uniform01_f16(1005, (H, W))
    res = torch.zeros((H, W), dtype=torch.float32, device="cuda:0")
    down = torch.zeros((H // 2, W // 2), dtype=torch.float16, device="cuda:0") if want_down else None
    print(f"hb_pyr_level {H}x{W} down={want_down}", flush=True)
    hb.hb_pyr_level(up(img), res, down)
    torch.cuda.synchronize()
    for y0 in (0, 16, 480, 1008, 2040, 4096 - 32, 6000, H - 96, H - 64):
        lo, hi = max(y0 - 16, 0), min(y0 + 64 + 16, H)
        ref, dref = orc.pyr_level(img[lo:hi], want_down=True)
        a, b = (0 if lo == 0 else 16), (hi - lo if hi == H else hi - lo - 16)
        assert_close(res[lo + a:lo + b].cpu().numpy(), ref[a:b], f"residual rows {lo + a}..{lo + b}")
        if want_down:
            got = down[(lo + a) // 2:(lo + b) // 2].cpu().numpy().astype(np.float64)
            assert_close(got, dref[a // 2:b // 2], f"down rows {(lo + a) // 2}..{(lo + b) // 2}")
