"""Images just below the documented size limits (rows are addressed with 32-bit byte offsets:
H * in_pitch < 2^31 and H * out_pitch < 2^30 elements; one conv image below 2 GiB).  The image is a
seeded block repeated down the rows (built on the GPU, several GB), and row bands at the top, in the
middle and at the very end are compared with the oracle run on a crop with a margin wider than the
stage's vertical reach."""
import numpy as np
import pytest

from paper_2512_02371_amd import synth
from hbtest import assert_close

pytestmark = pytest.mark.gpu

H_MAX, W_MAX = 65534, 16384            # H * W = 2^30 - 32768: the largest fp32 output the row stages take


def tiled_image(seed, H, W, pitch, block_rows=2048):
    """fp16 image of H x W inside rows of `pitch` elements: a seeded block repeated vertically."""
    import torch
    block = torch.from_numpy(synth.uniform01_f16(seed, (block_rows, W)).view(np.float16)).to("cuda:0")
    buf = torch.full((H, pitch), 3.0, dtype=torch.float16, device="cuda:0")
    for y in range(0, H, block_rows):
        n = min(block_rows, H - y)
        buf[y:y + n, :W] = block[:n]
    return buf[:, :W]


def bits(t):
    return t.contiguous().cpu().numpy().view(np.uint16)


def bands(H, rows, margin):
    """(lo, hi, a, b): crop rows lo..hi, of which a..b (relative) are far enough from the crop's cut edges."""
    for y0 in (0, H // 2 - 7, H - rows):
        lo, hi = max(y0 - margin, 0), min(y0 + rows + margin, H)
        yield lo, hi, (0 if lo == 0 else margin), (hi - lo if hi == H else hi - lo - margin)


@pytest.mark.parametrize("fn", ["hb_fir1d", "hb_fir1d_valu"])
def test_fir1d_at_the_size_limits(orc, fn):
    import torch
    from paper_2512_02371_amd import hb
    H, W = H_MAX + 1, W_MAX                                   # 65535 rows
    img = tiled_image(3001, H, W, 2 * W)                      # H * in_pitch = 2^31 - 32768
    taps = synth.random_taps_f16(3002, 24)
    out = torch.empty((H, W), dtype=torch.float32, device="cuda:0")
    print(f"{fn} {H}x{W} in_pitch {2 * W}", flush=True)
    getattr(hb, fn)(img, out, taps, 11)
    torch.cuda.synchronize()
    for lo, hi, a, b in bands(H, 40, 0):
        assert_close(out[lo:hi].cpu().numpy(), orc.fir1d(bits(img[lo:hi]), taps, 11), f"{fn} rows {lo}..{hi}")
    assert hb.load().hb_fir1d(img.data_ptr(), out.data_ptr(), H + 1, W, 2 * W, W, taps.ctypes.data, 24, 11, None) \
        == hb.HB_ERR_UNSUPPORTED, "one more row is beyond the limit and must be refused"


@pytest.mark.parametrize("fn", ["hb_sepblur", "hb_sepblur_valu"])
def test_sepblur_at_the_size_limits(orc, fn):
    import torch
    from paper_2512_02371_amd import hb
    H, W = H_MAX + 1, W_MAX
    img = tiled_image(3003, H, W, 2 * W)
    t = synth.gaussian_taps_f16(16, 3.0)
    out = torch.empty((H, W), dtype=torch.float32, device="cuda:0")
    print(f"{fn} {H}x{W} in_pitch {2 * W}", flush=True)
    getattr(hb, fn)(img, out, t, 7, t, 7)
    torch.cuda.synchronize()
    for lo, hi, a, b in bands(H, 48, 16):
        ref = orc.sepblur(bits(img[lo:hi]), t, 7, t, 7)
        assert_close(out[lo + a:lo + b].cpu().numpy(), ref[a:b], f"{fn} rows {lo + a}..{lo + b}")


@pytest.mark.parametrize("fn", ["hb_sat2d", "hb_sat2d_valu"])
def test_sat2d_at_a_gigapixel(orc, fn):
    """2^30 pixels: the table's last value is ~5e8, far beyond what fp32 counts exactly; the error over
    the total stays within the bar.  The oracle sums a top band directly and the rest through the
    block structure of the image (every block of rows is the same)."""
    import torch
    from paper_2512_02371_amd import hb
    H, W, B = 65536, 16384, 2048
    img = tiled_image(3004, H, W, W, block_rows=B)
    out = torch.empty((H, W), dtype=torch.float32, device="cuda:0")
    ws = torch.empty(hb.hb_sat2d_workspace_size(H, W), dtype=torch.uint8, device="cuda:0")
    print(f"{fn} {H}x{W}", flush=True)
    getattr(hb, fn)(img, out, ws)
    torch.cuda.synchronize()
    block = orc.sat2d(bits(img[:B]))                          # table of one block of rows
    total = block[-1, -1] * (H // B)
    # row y = q B + r of the full table = q * (last row of the block table) + row r of the block table
    for y in (0, 1, B - 1, B, 5 * B + 77, H // 2 + 3, H - B - 1, H - 2, H - 1):
        q, r = divmod(y, B)
        ref = q * block[-1] + block[r]
        err = np.abs(out[y].cpu().numpy().astype(np.float64) - ref) / total
        assert err.max() <= 1e-3, f"{fn} row {y}: error over total {err.max():.3e}"


@pytest.mark.parametrize("fn", ["hb_pyr_level", "hb_pyr_level_valu"])
def test_pyr_level_at_the_size_limits(orc, fn):
    import torch
    from paper_2512_02371_amd import hb
    H, W = H_MAX, W_MAX
    img = tiled_image(3005, H, W, W + 8)
    res = torch.empty((H, W), dtype=torch.float32, device="cuda:0")
    down = torch.empty((H // 2, W // 2), dtype=torch.float16, device="cuda:0")
    print(f"{fn} {H}x{W}", flush=True)
    getattr(hb, fn)(img, res, down)
    torch.cuda.synchronize()
    for lo, hi, a, b in bands(H, 64, 16):
        lo, hi = lo & ~1, hi + (hi & 1 if hi < H else 0)      # even crops
        ref, dref = orc.pyr_level(bits(img[lo:hi]), want_down=True)
        assert_close(res[lo + a:lo + b].cpu().numpy(), ref[a:b], f"{fn} residual rows {lo + a}..{lo + b}")
        got = down[(lo + a) // 2:(lo + b) // 2].cpu().numpy().astype(np.float64)
        assert_close(got, dref[a // 2:b // 2], f"{fn} down rows {(lo + a) // 2}..{(lo + b) // 2}")


@pytest.mark.parametrize("fn", ["hb_conv3x3", "hb_conv3x3_valu"])
def test_conv3x3_at_the_size_limits(orc, fn):
    """One image of 4095 x 4096 x 64 fp16 = 2 GiB - 512 KiB; the batch of two puts the second image
    beyond 2 GiB from the base pointer."""
    import torch
    from paper_2512_02371_amd import hb
    N, H, W, B = 2, 4095, 4096, 65
    block = torch.from_numpy(synth.uniform_pm1_f16(3006, (B, W, 64)).view(np.float16)).to("cuda:0")
    x = torch.empty((N, H, W, 64), dtype=torch.float16, device="cuda:0")
    for n in range(N):
        for y in range(0, H, B):
            x[n, y:y + B] = block[:min(B, H - y)]
    w = synth.normal_f16(3007, (3, 3, 64, 64), 1.0 / 24.0)
    o = torch.empty((N, H, W, 64), dtype=torch.float16, device="cuda:0")
    print(f"{fn} {N}x{H}x{W}x64", flush=True)
    getattr(hb, fn)(x, torch.from_numpy(w.view(np.float16)).to("cuda:0"), o)
    torch.cuda.synchronize()
    for n, y0 in ((0, 0), (0, H // 2), (1, 0), (1, H - 6)):
        lo, hi = max(y0 - 1, 0), min(y0 + 6 + 1, H)
        a, b = (0 if lo == 0 else 1), (hi - lo if hi == H else hi - lo - 1)
        ref = orc.conv3x3(bits(x[n:n + 1, lo:hi]), w)[0]
        assert_close(o[n, lo + a:lo + b].cpu().numpy().astype(np.float64), ref[a:b], f"{fn} image {n} rows {lo + a}..{lo + b}")
    assert hb.load().hb_conv3x3(x.data_ptr(), x.data_ptr(), o.data_ptr(), 1, 4096, 4096, 64, 64, None) \
        == hb.HB_ERR_UNSUPPORTED, "a 2 GiB image is beyond the limit and must be refused"


@pytest.mark.parametrize("kind", ["conv2d", "down2", "up2"])
@pytest.mark.parametrize("v", ["", "_valu"])
def test_kernel2d_stages_at_the_size_limits(orc, kind, v):
    import torch
    from paper_2512_02371_amd import hb
    fn = f"hb_{kind}{v}"
    if kind == "up2":
        H, W, pitch = 32767, 8192, 8192                       # output 65534 x 16384
        Ho, Wo, ay, ax = 2 * H, 2 * W, 2, 1
    elif kind == "down2":
        H, W, pitch = 65535, 16384, 32768                     # H * in_pitch = 2^31 - 32768, odd height
        Ho, Wo, ay, ax = (H + 1) // 2, W // 2, 5, 4
    else:
        H, W, pitch = 65535, 16384, 32768
        Ho, Wo, ay, ax = H, W, 5, 4
    img = tiled_image(3008, H, W, pitch)
    k = synth.random_kernel2d_f16(3009, 10, 8)
    out = torch.empty((Ho, Wo), dtype=torch.float32, device="cuda:0")
    print(f"{fn} {H}x{W} in_pitch {pitch}", flush=True)
    getattr(hb, fn)(img, out, k, ay, ax)
    torch.cuda.synchronize()
    for lo, hi, a, b in bands(H, 32, 12):
        if kind == "down2":
            lo, a, b = lo & ~1, a + (a & 1), b                # crops start on even rows
        ref = getattr(orc, kind)(bits(img[lo:hi]), k, ay, ax)
        if kind == "conv2d":
            got, r = out[lo + a:lo + b], ref[a:b]
        elif kind == "down2":
            got, r = out[(lo + a) // 2:(lo + b + 1) // 2], ref[a // 2:(b + 1) // 2]
        else:
            got, r = out[2 * (lo + a):2 * (lo + b)], ref[2 * a:2 * b]
        assert_close(got.cpu().numpy(), r, f"{fn} input rows {lo + a}..{lo + b}")


@pytest.mark.parametrize("fn", ["hb_resize", "hb_resize_valu"])
def test_resize_at_the_size_limits(orc, fn):
    """A plane of 65535 x 32768 (H * in_pitch = 2^31 - 32768) to 29999 x 30001: the transposed fp16
    intermediate is 30001 rows of 65536 (just below 2^31 elements), the output 0.9 * 2^30 floats."""
    import torch
    from paper_2512_02371_amd import hb
    H, W, Ho, Wo = 65535, 32768, 29999, 30001
    img = tiled_image(3010, H, W, W, block_rows=1024)
    sy, cy = hb.hb_lanczos3_matrix(H, Ho)
    sx, cx = hb.hb_lanczos3_matrix(W, Wo)
    out = torch.empty((1, Ho, Wo), dtype=torch.float32, device="cuda:0")
    ws = torch.empty(hb.hb_resize_workspace_size(1, H, Wo), dtype=torch.uint8, device="cuda:0")
    di = lambda a: torch.from_numpy(a).to("cuda:0")
    dh = lambda a: torch.from_numpy(a.view(np.int16)).to("cuda:0").view(torch.float16)
    print(f"{fn} {H}x{W} -> {Ho}x{Wo}", flush=True)
    getattr(hb, fn)(img[None], out, ws, di(sy), dh(cy), di(sx), dh(cx))
    torch.cuda.synchronize()
    band = cy.shape[1]
    for o0 in (0, Ho // 2 - 5, Ho - 16):
        rows = slice(o0, o0 + 16)
        lo, hi = max(int(sy[rows].min()), 0), min(int(sy[rows].max()) + band, H)
        # the crop ends where the image ends or beyond the rows these outputs read: clamping agrees
        ref = orc.band_resize(bits(img[lo:hi]), sy[rows] - lo, cy[rows], sx, cx)
        assert_close(out[0, rows].cpu().numpy(), ref, f"{fn} output rows {o0}..{o0 + 16}")
