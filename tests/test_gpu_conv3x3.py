"""hb_conv3x3 / hb_conv3x3_valu against the fp64 oracle (unrounded), element by element."""
import numpy as np
import pytest

from paper_2512_02371_amd import synth
from hbtest import assert_close, up

pytestmark = pytest.mark.gpu

CASES = [(1, 8, 32), (1, 1, 1), (1, 5, 7), (2, 19, 45), (1, 64, 96), (1, 33, 130), (3, 9, 33)]


def run(fn, x, w):
    import torch
    from paper_2512_02371_amd import hb
    N, H, W, C = x.shape
    out = torch.full((N, H, W, w.shape[3]), 9.0, dtype=torch.float16, device="cuda:0")
    print(f"{fn} N={N} H={H} W={W}", flush=True)
    getattr(hb, fn)(up(x), up(w), out)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("fn", ["hb_conv3x3", "hb_conv3x3_valu"])
@pytest.mark.parametrize("N,H,W", CASES)
def test_conv_matches_oracle(orc, fn, N, H, W):
    x = synth.uniform_pm1_f16(9000 + H + 5 * W, (N, H, W, 64))
    w = synth.normal_f16(9500 + H, (3, 3, 64, 64), 1 / 24)
    assert_close(run(fn, x, w), orc.conv3x3(x, w), f"{fn} {N}x{H}x{W}")


@pytest.mark.parametrize("fn", ["hb_conv3x3", "hb_conv3x3_valu"])
def test_conv_centre_identity_is_exact_and_one_hot_mirrors_weights(fn):
    x = synth.uniform_pm1_f16(9100, (1, 20, 40, 64))
    w = np.zeros((3, 3, 64, 64))
    w[1, 1] = np.eye(64)
    got = run(fn, x, synth.f64_to_f16_bits(w))
    assert np.array_equal(got, synth.f16_bits_to_f64(x))
    wb = synth.normal_f16(9101, (3, 3, 64, 64), 1 / 24)
    xo = np.zeros((1, 12, 35, 64))
    xo[0, 5, 31, 17] = 1.0                      # next to a tile seam
    got = run(fn, synth.f64_to_f16_bits(xo), wb)
    wd = synth.f16_bits_to_f64(wb)
    for y in range(12):
        for xx in range(35):
            ky, kx = 5 - y + 1, 31 - xx + 1
            exp = wd[ky, kx, 17] if 0 <= ky < 3 and 0 <= kx < 3 else np.zeros(64)
            assert np.array_equal(got[0, y, xx], exp)


@pytest.mark.parametrize("fn", ["hb_conv3x3", "hb_conv3x3_valu"])
def test_conv_benchmark_shape_sampled(orc, fn):
    """The full 1 x 1024 x 1024 x 64 configuration; the oracle is evaluated on two complete row
    bands (top border, a tile seam) and on 1500 scattered pixels."""
    x = synth.uniform_pm1_f16(1004, (1, 1024, 1024, 64))
    w = synth.normal_f16(2004, (3, 3, 64, 64), 1 / 24)
    got = run(fn, x, w)
    for y0, y1 in ((0, 3), (510, 515), (1021, 1024)):
        assert_close(got[:, y0:y1], orc.conv3x3_rows(x, w, y0, y1), f"{fn} rows {y0}:{y1}")
    h = synth.hash_u64(4242, 0, 3000)
    ys = (h[:1500] % np.uint64(1024)).astype(np.int32)
    xs = (h[1500:] % np.uint64(1024)).astype(np.int32)
    ref = orc.conv3x3_points(x, w, np.zeros(1500, np.int32), ys, xs)
    assert_close(got[0, ys, xs], ref, f"{fn} scattered")


def test_conv_rejects_other_channel_counts():
    import torch
    from paper_2512_02371_amd import hb
    x = torch.zeros((1, 4, 4, 32), dtype=torch.float16, device="cuda:0")
    w = torch.zeros((3, 3, 32, 32), dtype=torch.float16, device="cuda:0")
    o = torch.zeros((1, 4, 4, 32), dtype=torch.float16, device="cuda:0")
    with pytest.raises(hb.HbError) as e:
        hb.hb_conv3x3(x, w, o)
    assert e.value.code == hb.HB_ERR_UNSUPPORTED
