"""The benchmark's own launches, compared with the fp64 oracle on EVERY output element (the oracle
runs a few seconds per stage on the host cores), for the matrix-unit path and for the vector-ALU twin
of each stage."""
import numpy as np
import pytest

from paper_2512_02371_amd import synth
from hbtest import TOL, assert_close, scaled_err, up

pytestmark = pytest.mark.gpu


def test_conv3x3_benchmark_size_every_output(orc):
    """1 x 1024 x 1024 x 64: all 67 M outputs, in slabs of 128 rows."""
    import torch
    from paper_2512_02371_amd import hb
    x = synth.uniform_pm1_f16(1004, (1, 1024, 1024, 64))
    w = synth.normal_f16(2004, (3, 3, 64, 64), 1 / 24)
    dx, dw = up(x), up(w)
    outs = {}
    for fn in ("hb_conv3x3", "hb_conv3x3_valu"):
        out = torch.full((1, 1024, 1024, 64), 9.0, dtype=torch.float16, device="cuda:0")
        print(f"{fn} 1x1024x1024x64", flush=True)
        getattr(hb, fn)(dx, dw, out)
        torch.cuda.synchronize()
        outs[fn] = out.cpu().numpy()
    worst = 0.0
    for y0 in range(0, 1024, 128):
        ref = orc.conv3x3_rows(x, w, y0, y0 + 128)
        for fn, got in outs.items():
            worst = max(worst, assert_close(got[:, y0:y0 + 128].astype(np.float64), ref, f"{fn} rows {y0}..{y0 + 128}"))
    print(f"conv3x3 full image: max scaled error {worst:.3e}", flush=True)


def test_sepblur_benchmark_size_every_output(orc):
    """4096 x 4096, 16 x 16 taps: all 16.8 M outputs of both paths."""
    import torch
    from paper_2512_02371_amd import hb
    H = W = 4096
    img = synth.uniform01_f16(1002, (H, W))
    t = synth.gaussian_taps_f16(16, 3.0)
    ref = orc.sepblur(img, t, 7, t, 7)
    d_in = up(img)
    for fn in ("hb_sepblur", "hb_sepblur_valu"):
        out = torch.zeros((H, W), dtype=torch.float32, device="cuda:0")
        print(f"{fn} {H}x{W}", flush=True)
        getattr(hb, fn)(d_in, out, t, 7, t, 7)
        torch.cuda.synchronize()
        e = assert_close(out.cpu().numpy(), ref, fn)
        print(f"{fn} full image: max scaled error {e:.3e}", flush=True)


@pytest.mark.parametrize("fn", ["hb_pyr_level", "hb_pyr_level_valu"])
@pytest.mark.parametrize("want_down", [False, True])
def test_pyr_level_benchmark_size_every_output(orc, fn, want_down):
    """8192 x 8192: every residual pixel and, when asked for, every pixel of the coarser level."""
    import torch
    from paper_2512_02371_amd import hb
    H = W = 8192
    img = synth.uniform01_f16(1005, (H, W))
    res = torch.zeros((H, W), dtype=torch.float32, device="cuda:0")
    down = torch.full((H // 2, W // 2), 9.0, dtype=torch.float16, device="cuda:0")
    print(f"{fn} {H}x{W} down={want_down}", flush=True)
    getattr(hb, fn)(up(img), res, down if want_down else None)
    torch.cuda.synchronize()
    ref, dref = orc.pyr_level(img, want_down=True)
    e = assert_close(res.cpu().numpy(), ref, f"{fn} residual")
    print(f"{fn} residual, full image: max scaled error {e:.3e}", flush=True)
    got = down.cpu().numpy().astype(np.float64)
    if want_down:
        assert_close(got, dref, f"{fn} coarser level")
    else:
        assert np.all(got == 9.0), "the coarser level was written although it was not asked for"


def test_sat2d_valu_benchmark_size(orc):
    """The vector-ALU twin at 4096 x 4096: error over the total and per element, and a 0/1 image bit-exactly."""
    import torch
    from paper_2512_02371_amd import hb
    H = W = 4096
    ws = torch.empty(hb.hb_sat2d_workspace_size(H, W) + 256, dtype=torch.uint8, device="cuda:0")
    ws = ws[(-ws.data_ptr()) % 256:]
    img = synth.uniform01_f16(1003, (H, W))
    out = torch.zeros((H, W), dtype=torch.float32, device="cuda:0")
    print(f"hb_sat2d_valu {H}x{W}", flush=True)
    hb.hb_sat2d_valu(up(img), out, ws)
    torch.cuda.synchronize()
    got, ref = out.cpu().numpy(), orc.sat2d(img)
    assert np.abs(got - ref).max() / ref[-1, -1] <= TOL
    assert scaled_err(got, ref).max() <= TOL
    bits = synth.binary01_f16(78, (H, W))
    hb.hb_sat2d_valu(up(bits), out, ws)
    torch.cuda.synchronize()
    ref = np.cumsum(np.cumsum(synth.f16_bits_to_f64(bits), axis=0), axis=1)
    assert np.array_equal(out.cpu().numpy().astype(np.float64), ref)
