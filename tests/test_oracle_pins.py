"""Pins for the fp64 oracle: every check compares it with something that is not
the oracle itself -- hand-computed fixtures, closed forms, the paper's matrix
formulations written out densely in numpy, library routines, brute force.

CPU only.  Nothing here touches the HIP library.
"""
import os

import numpy as np
import pytest

from paper_2512_02371_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def h(x):
    """float array -> fp16 bit patterns (values used here are exactly representable)."""
    return synth.f64_to_f16_bits(np.asarray(x, dtype=np.float64))


def d(bits):
    return synth.f16_bits_to_f64(bits)


def read_fixture(name):
    out = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = np.array([float(v) for v in vals])
    return out


def rand_img(seed, H, W):
    return synth.uniform01_f16(seed, (H, W))


# --------------------------------------------------------------------------
# half decoder
# --------------------------------------------------------------------------

def test_half_decoder_matches_numpy_on_all_bit_patterns(orc):
    bits = np.arange(65536, dtype=np.uint16)
    ref = d(bits)
    mine = np.array([orc.half_to_double(int(b)) for b in bits])
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(mine), nan)
    assert np.array_equal(mine[~nan], ref[~nan])
    assert np.array_equal(np.signbit(mine[~nan]), np.signbit(ref[~nan]))
    # the array form (used where the oracle's arithmetic is numpy) is the same decoder
    arr = orc.halves_to_doubles(bits.reshape(256, 256))
    assert arr.shape == (256, 256) and np.array_equal(arr.ravel()[~nan], ref[~nan]) and np.isnan(arr.ravel()[nan]).all()


# --------------------------------------------------------------------------
# FIR  (Sec. V-A: O(x) = sum_r I(x+r) K(r); matrix A_K(x,y) = K(y-x))
# --------------------------------------------------------------------------

def test_fir_hand_fixture(orc):
    fx = read_fixture("fir1d_hand.txt")
    out = orc.fir1d(h(fx["input"])[None, :], h(fx["taps"]), int(fx["anchor"][0]))
    assert np.array_equal(out[0], fx["expect"])


@pytest.mark.parametrize("T,a", [(8, 3), (8, 0), (5, 4), (1, 0), (16, 7)])
def test_fir_impulse_gives_mirrored_taps(orc, T, a):
    W, x0 = 64, 30
    taps = synth.random_taps_f16(7 + T, T)
    img = np.zeros((3, W))
    img[1, x0] = 1.0
    out = orc.fir1d(h(img), taps, a)
    k = d(taps)
    expect = np.zeros(W)
    for x in range(W):
        r = x0 - x + a           # tap r reads x + r - a == x0
        if 0 <= r < T:
            expect[x] = k[r]
    assert np.array_equal(out[1], expect)
    assert not out[0].any() and not out[2].any()


def test_fir_constant_image_scaled_by_tap_sum_including_edges(orc):
    taps = synth.random_taps_f16(3, 8)
    c = 0.625
    out = orc.fir1d(h(np.full((4, 19), c)), taps, 3)
    s = float(np.sum(d(taps) * c))
    assert np.allclose(out, s, rtol=0, atol=1e-15)


@pytest.mark.parametrize("T,a,W", [(8, 3, 50), (16, 7, 33), (3, 0, 8), (9, 8, 21)])
def test_fir_equals_dense_toeplitz_product(orc, T, a, W):
    """Second formulation: edge-replicated row (length W+T-1) times the
    (W+T-1) x W matrix A[y][x] = K(y - x) for 0 <= y - x < T."""
    img = rand_img(11, 5, W)
    taps = synth.random_taps_f16(12, T)
    k = d(taps)
    A = np.zeros((W + T - 1, W))
    for x in range(W):
        for y in range(W + T - 1):
            if 0 <= y - x < T:
                A[y, x] = k[y - x]
    rows = d(img)
    padded = np.concatenate([np.repeat(rows[:, :1], a, axis=1), rows,
                             np.repeat(rows[:, -1:], T - 1 - a, axis=1)], axis=1)
    expect = padded @ A
    out = orc.fir1d(img, taps, a)
    assert np.allclose(out, expect, rtol=0, atol=1e-14)


def test_fir_brute_force_tiny_and_three_tap_signal_of_eight(orc):
    # the paper's Fig. 2 size: a 3-tap kernel over 8 samples (valid part: anchor 0)
    sig = rand_img(21, 1, 8)
    taps = synth.random_taps_f16(22, 3)
    out = orc.fir1d(sig, taps, 0)
    s, k = d(sig)[0], d(taps)
    for x in range(8 - 2):
        assert out[0, x] == pytest.approx(sum(s[x + r] * k[r] for r in range(3)), abs=1e-15)
    # 8x8 with clamp, python loops
    img = rand_img(23, 8, 8)
    taps = synth.random_taps_f16(24, 5)
    out = orc.fir1d(img, taps, 2)
    I, k = d(img), d(taps)
    for y in range(8):
        for x in range(8):
            acc = 0.0
            for r in range(5):
                acc += k[r] * I[y, min(max(x + r - 2, 0), 7)]
            assert out[y, x] == pytest.approx(acc, abs=1e-15)


def test_fir_box_filter_is_difference_of_prefix_sums(orc):
    T, a, W = 8, 3, 40
    img = rand_img(31, 3, W)
    taps = h(np.full(T, 1.0 / T))
    out = orc.fir1d(img, taps, a)
    I = d(img)
    P = np.concatenate([np.zeros((3, 1)), np.cumsum(I, axis=1)], axis=1)
    for x in range(a, W - (T - 1 - a)):          # interior
        assert np.allclose(out[:, x], (P[:, x - a + T] - P[:, x - a]) / T, atol=1e-14)


def test_fir_linearity_and_shift_equivariance(orc):
    taps = synth.random_taps_f16(41, 8)
    # multiples of 2^-11 below 1/2, so a + b is again exactly representable in fp16
    a_img = np.floor(d(rand_img(42, 2, 64)) * 1024) / 2048
    b_img = np.floor(d(rand_img(43, 2, 64)) * 1024) / 2048
    s = orc.fir1d(h(a_img + b_img), taps, 3)
    assert np.allclose(s, orc.fir1d(h(a_img), taps, 3) + orc.fir1d(h(b_img), taps, 3), atol=1e-15)
    sh = np.roll(a_img, 5, axis=1)
    o1 = orc.fir1d(h(a_img), taps, 3)
    o2 = orc.fir1d(h(sh), taps, 3)
    assert np.allclose(o2[:, 16:48], o1[:, 11:43], atol=1e-15)


# --------------------------------------------------------------------------
# separable blur
# --------------------------------------------------------------------------

def test_sepblur_constant_and_impulse(orc):
    tx = synth.gaussian_taps_f16(16, 3.0)
    ty = synth.random_taps_f16(51, 7)
    c = 0.375
    out = orc.sepblur(h(np.full((20, 24), c)), tx, 7, ty, 2)
    assert np.allclose(out, c * d(tx).sum() * d(ty).sum(), atol=1e-15)
    img = np.zeros((40, 48))
    y0, x0 = 20, 25
    img[y0, x0] = 1.0
    out = orc.sepblur(h(img), tx, 7, ty, 2)
    kx, ky = d(tx), d(ty)
    expect = np.zeros_like(img)
    for y in range(40):
        for x in range(48):
            ry, rx = y0 - y + 2, x0 - x + 7
            if 0 <= ry < 7 and 0 <= rx < 16:
                expect[y, x] = ky[ry] * kx[rx]
    assert np.allclose(out, expect, atol=1e-17)


def test_sepblur_equals_direct_2d_correlation_brute_force(orc):
    H, W, Tx, ax, Ty, ay = 12, 10, 5, 1, 4, 2
    img = rand_img(61, H, W)
    tx, ty = synth.random_taps_f16(62, Tx), synth.random_taps_f16(63, Ty)
    out = orc.sepblur(img, tx, ax, ty, ay)
    I, kx, ky = d(img), d(tx), d(ty)
    for y in range(H):
        for x in range(W):
            acc = 0.0
            for ry in range(Ty):
                for rx in range(Tx):
                    yy = min(max(y + ry - ay, 0), H - 1)
                    xx = min(max(x + rx - ax, 0), W - 1)
                    acc += ky[ry] * kx[rx] * I[yy, xx]
            assert out[y, x] == pytest.approx(acc, abs=1e-14)


def test_sepblur_symmetric_input_gives_symmetric_output(orc):
    t = synth.gaussian_taps_f16(9, 2.0)          # odd length, centred anchor -> symmetric operator
    I = d(rand_img(71, 24, 24))
    I = (I + I[::-1, ::-1]) / 2
    out = orc.sepblur(h(I), t, 4, t, 4)
    assert np.allclose(out, out[::-1, ::-1], atol=1e-15)


def test_sepblur_separates_into_two_dense_matrix_products(orc):
    """out = Cy @ I @ Cx^T with clamp folded into the (square) operator matrices."""
    H, W, T, a = 21, 18, 16, 7
    img = rand_img(81, H, W)
    t = synth.gaussian_taps_f16(T, 3.0)
    k = d(t)

    def op(n):
        M = np.zeros((n, n))
        for o in range(n):
            for r in range(T):
                M[o, min(max(o + r - a, 0), n - 1)] += k[r]
        return M
    expect = op(H) @ d(img) @ op(W).T
    assert np.allclose(orc.sepblur(img, t, a, t, a), expect, atol=1e-14)


# --------------------------------------------------------------------------
# 2-D convolution with an arbitrary (non-separable) kernel
# --------------------------------------------------------------------------

def rand_kernel(seed, kh, kw):
    """kh x kw taps on the fp16 grid (multiples of 1/64 in [-1, 1))."""
    return h(np.round(d(synth.uniform_pm1_f16(seed, (kh, kw))) * 64) / 64)


def test_conv2d_impulse_gives_mirrored_kernel_and_constant_gives_tap_sum(orc):
    kh, kw, ay, ax = 5, 7, 1, 4
    k = rand_kernel(81, kh, kw)
    K = d(k)
    img = np.zeros((30, 34))
    y0, x0 = 14, 17
    img[y0, x0] = 1.0
    out = orc.conv2d(h(img), k, ay, ax)
    expect = np.zeros_like(img)
    for y in range(30):
        for x in range(34):
            ry, rx = y0 - y + ay, x0 - x + ax
            if 0 <= ry < kh and 0 <= rx < kw:
                expect[y, x] = K[ry, rx]
    assert np.array_equal(out, expect)
    out = orc.conv2d(h(np.full((9, 11), 0.25)), k, ay, ax)          # also on the clamped edges
    assert np.allclose(out, 0.25 * K.sum(), atol=1e-15)


def test_conv2d_equals_correlation_on_an_edge_replicated_array(orc):
    """Second formulation: replicate-pad the image (numpy), then plain windows times the kernel."""
    H, W, kh, kw, ay, ax = 13, 17, 6, 4, 5, 0
    img, k = rand_img(82, H, W), rand_kernel(83, kh, kw)
    out = orc.conv2d(img, k, ay, ax)
    P = np.pad(d(img), ((ay, kh - 1 - ay), (ax, kw - 1 - ax)), mode="edge")
    win = np.lib.stride_tricks.sliding_window_view(P, (kh, kw))      # [y][x][ry][rx]
    assert np.allclose(out, np.einsum("yxab,ab->yx", win, d(k)), atol=1e-14)


def test_conv2d_with_outer_product_kernel_equals_the_separable_blur(orc):
    """K = ky (x) kx with power-of-two taps (products exact in fp16): the blur oracle, pinned above."""
    ky = h([0.5, 0.25, 0.125, 0.0625, 0.0625])
    kx = h([0.25, 0.5, 0.125, 0.125])
    K = h(np.outer(d(ky), d(kx)))
    img = rand_img(84, 21, 19)
    assert np.allclose(orc.conv2d(img, K, 2, 1), orc.sepblur(img, kx, 1, ky, 2), atol=1e-15)


def test_conv2d_single_row_kernel_is_the_fir_and_single_column_its_transpose(orc):
    t = synth.random_taps_f16(85, 9)
    img = rand_img(86, 10, 40)
    assert np.allclose(orc.conv2d(img, t.reshape(1, 9), 0, 3), orc.fir1d(img, t, 3), atol=1e-15)
    imgT = np.ascontiguousarray(img.T)
    assert np.allclose(orc.conv2d(imgT, t.reshape(9, 1), 3, 0), orc.fir1d(img, t, 3).T, atol=1e-15)


def test_conv2d_is_a_sum_of_row_shifted_toeplitz_products(orc):
    """The paper's serial loop over r_y: out = sum_ry  shift_ry(I) * A_{K(., ry)}, written densely."""
    H, W, kh, kw, ay, ax = 8, 12, 3, 5, 1, 2
    img, k = rand_img(87, H, W), rand_kernel(88, kh, kw)
    I, K = d(img), d(k)
    Ipad = np.pad(I, ((0, 0), (ax, kw - 1 - ax)), mode="edge")      # W + kw - 1 samples per row
    total = np.zeros((H, W))
    for ry in range(kh):
        A = np.zeros((W + kw - 1, W))                                # A_K(x, y) = K(y - x)
        for x in range(W):
            A[x:x + kw, x] = K[ry]
        rows = np.clip(np.arange(H) + ry - ay, 0, H - 1)
        total += Ipad[rows] @ A
    assert np.allclose(orc.conv2d(img, k, ay, ax), total, atol=1e-14)


# --------------------------------------------------------------------------
# summed-area table
# --------------------------------------------------------------------------

def test_sat_hand_fixture(orc):
    fx = read_fixture("sat_hand.txt")
    H, W = int(fx["rows"][0]), int(fx["cols"][0])
    out = orc.sat2d(h(fx["input"].reshape(H, W)))
    assert np.array_equal(out, fx["expect"].reshape(H, W))


def test_sat_all_ones_closed_form(orc):
    H, W = 67, 45
    out = orc.sat2d(h(np.ones((H, W))))
    i, j = np.meshgrid(np.arange(H), np.arange(W), indexing="ij")
    assert np.array_equal(out, (i + 1.0) * (j + 1.0))


def test_sat_ramp_closed_form(orc):
    H, W = 33, 64
    img = np.tile(np.arange(W) / 2048.0, (H, 1))
    out = orc.sat2d(h(img))
    i, j = np.meshgrid(np.arange(H), np.arange(W), indexing="ij")
    assert np.array_equal(out, (i + 1.0) * j * (j + 1) / 2 / 2048.0)


def test_sat_inverse_identity_total_and_cumsum(orc):
    img = rand_img(91, 50, 70)
    out = orc.sat2d(img)
    I = d(img)
    P = np.pad(out, ((1, 0), (1, 0)))
    assert np.array_equal(P[1:, 1:] - P[:-1, 1:] - P[1:, :-1] + P[:-1, :-1], I)   # exact: multiples of 2^-11
    assert out[-1, -1] == float(np.sum(I.astype(np.longdouble)))
    assert np.array_equal(out, np.cumsum(np.cumsum(I, axis=0), axis=1))


def test_sat_brute_force_8x8_and_triangular_matrix_form(orc):
    img = rand_img(92, 8, 8)
    out = orc.sat2d(img)
    I = d(img)
    for i in range(8):
        for j in range(8):
            assert out[i, j] == sum(I[y, x] for y in range(i + 1) for x in range(j + 1))
    img = rand_img(93, 32, 32)
    L = np.tril(np.ones((32, 32)))
    assert np.array_equal(orc.sat2d(img), L @ d(img) @ L.T)


# --------------------------------------------------------------------------
# 3x3 multi-channel convolution
# --------------------------------------------------------------------------

def test_conv_one_hot_input_gives_mirrored_weight_slice(orc):
    H, W, Ci, Co = 7, 9, 16, 16
    w = synth.normal_f16(101, (3, 3, Ci, Co), 1 / 12)
    x = np.zeros((1, H, W, Ci))
    y0, x0, c0 = 3, 4, 5
    x[0, y0, x0, c0] = 1.0
    out = orc.conv3x3(h(x), w)
    wd = d(w)
    expect = np.zeros((1, H, W, Co))
    for y in range(H):
        for xx in range(W):
            ky, kx = y0 - y + 1, x0 - xx + 1
            if 0 <= ky < 3 and 0 <= kx < 3:
                expect[0, y, xx] = wd[ky, kx, c0]
    assert np.array_equal(out, expect)


def test_conv_centre_identity_reproduces_input(orc):
    H, W, C = 6, 5, 32
    x = synth.uniform_pm1_f16(102, (2, H, W, C))
    w = np.zeros((3, 3, C, C))
    w[1, 1] = np.eye(C)
    assert np.array_equal(orc.conv3x3(x, h(w)), d(x))


def test_conv_centre_tap_only_is_a_gemm(orc):
    H, W, Ci, Co = 5, 6, 32, 16
    x = synth.uniform_pm1_f16(103, (1, H, W, Ci))
    w = np.zeros((3, 3, Ci, Co))
    w[1, 1] = d(synth.normal_f16(104, (Ci, Co), 0.1))
    out = orc.conv3x3(x, h(w))
    assert np.allclose(out.reshape(-1, Co), d(x).reshape(-1, Ci) @ w[1, 1], atol=1e-13)


def test_conv_border_counts_with_all_ones(orc):
    H, W, C = 6, 7, 64
    out = orc.conv3x3(h(np.ones((1, H, W, C))), h(np.ones((3, 3, C, C))))
    assert np.all(out[0, 0, 0] == 4 * C) and np.all(out[0, -1, -1] == 4 * C)
    assert np.all(out[0, 0, 3] == 6 * C) and np.all(out[0, 2, 0] == 6 * C)
    assert np.all(out[0, 2, 3] == 9 * C)


def test_conv_equals_padded_einsum_and_variants_agree(orc):
    N, H, W, Ci, Co = 2, 6, 7, 16, 32
    x = synth.uniform_pm1_f16(105, (N, H, W, Ci))
    w = synth.normal_f16(106, (3, 3, Ci, Co), 1 / 12)
    xp = np.pad(d(x), ((0, 0), (1, 1), (1, 1), (0, 0)))
    wd = d(w)
    expect = np.zeros((N, H, W, Co))
    for kx in range(3):                 # different loop order from the oracle: taps outermost, kx first
        for ky in range(3):
            expect += np.einsum("nhwc,co->nhwo", xp[:, ky:ky + H, kx:kx + W], wd[ky, kx])
    out = orc.conv3x3(x, w)
    assert np.allclose(out, expect, atol=1e-13)
    ys = np.array([0, 5, 2, 3], dtype=np.int32)
    xs = np.array([0, 6, 3, 0], dtype=np.int32)
    ns = np.array([0, 1, 1, 0], dtype=np.int32)
    pts = orc.conv3x3_points(x, w, ns, ys, xs)
    assert np.allclose(pts, out[ns, ys, xs], atol=1e-14)
    band = orc.conv3x3_rows(x[:1], w, 2, 5)
    assert np.array_equal(band[0], out[0, 2:5])


def test_conv_rank1_kernel_with_diagonal_mixing_matches_blur_interior(orc):
    """w[ky][kx] = ky_taps[ky]*kx_taps[kx]*I  =>  per-channel separable blur (interior)."""
    H, W, C = 9, 10, 16
    t = h([0.25, 0.5, 0.25])
    k = d(t)
    w = np.einsum("a,b,cd->abcd", k, k, np.eye(C))
    x = synth.uniform01_f16(107, (1, H, W, C))
    out = orc.conv3x3(x, h(w))
    for c in (0, 7, 15):
        chan = np.ascontiguousarray(x[0, :, :, c])
        blur = orc.sepblur(chan, t, 1, t, 1)
        assert np.allclose(out[0, 1:-1, 1:-1, c], blur[1:-1, 1:-1], atol=1e-15)


# --------------------------------------------------------------------------
# Laplacian pyramid level  (Sec. V-B: A_down(x,y) = K(y-2x); K_phase(x,dx) = K(2x+dx))
# --------------------------------------------------------------------------

WT = np.array([1, 4, 6, 4, 1]) / 16.0


def test_pyr_hand_fixture(orc):
    fx = read_fixture("pyr_hand.txt")
    H, W = int(fx["rows"][0]), int(fx["cols"][0])
    res, down = orc.pyr_level(h(fx["input"].reshape(H, W)), want_down=True)
    assert np.array_equal(down, fx["down"].reshape(H // 2, W // 2))
    assert np.array_equal(res, fx["expect"].reshape(H, W))


def test_pyr_constant_and_affine_images_have_zero_residual(orc):
    res = orc.pyr_level(h(np.full((12, 16), 0.75)))
    assert np.array_equal(res, np.zeros((12, 16)))
    y, x = np.meshgrid(np.arange(24), np.arange(32), indexing="ij")
    img = (3 * x + 5 * y + 7) / 512.0                 # exact in fp16
    res = orc.pyr_level(h(img))
    assert np.allclose(res[4:-4, 4:-4], 0.0, atol=1e-15)
    assert np.abs(res).max() > 1e-4                   # the clamped border does respond


def test_pyr_impulse_down_is_sampled_outer_product(orc):
    H, W, m0, n0 = 16, 20, 3, 5
    img = np.zeros((H, W))
    img[2 * m0, 2 * n0] = 1.0
    _, down = orc.pyr_level(h(img), want_down=True)
    expect = np.zeros((H // 2, W // 2))
    for m in range(H // 2):
        for n in range(W // 2):
            i, j = 2 * m0 - 2 * m, 2 * n0 - 2 * n     # D[m][n] reads in[2m+i][2n+j]
            if abs(i) <= 2 and abs(j) <= 2:
                expect[m, n] = WT[i + 2] * WT[j + 2]
    assert np.array_equal(down, expect)


def test_pyr_down_is_blur_sampled_at_even_coordinates(orc):
    img = rand_img(111, 18, 22)
    _, down = orc.pyr_level(img, want_down=True)
    t = h(WT)
    blur = orc.sepblur(img, t, 2, t, 2)
    assert np.allclose(down, blur[::2, ::2], atol=1e-15)


def test_pyr_down_equals_strided_toeplitz_matrix(orc):
    """A_down(x, y) = K(y - 2x) on the edge-replicated signal, both axes."""
    H, W = 10, 14
    img = rand_img(112, H, W)
    _, down = orc.pyr_level(img, want_down=True)

    def adown(n):                                   # (n+4) x (n/2): padded index y = 2x + r
        A = np.zeros((n + 4, n // 2))
        for x in range(n // 2):
            for y in range(n + 4):
                if 0 <= y - 2 * x < 5:
                    A[y, x] = WT[y - 2 * x]
        return A
    P = np.pad(d(img), 2, mode="edge")
    assert np.allclose(down, adown(H).T @ P @ adown(W), atol=1e-15)


def test_pyr_upsample_equals_zero_stuffing_formulation(orc):
    """The paper's O -> O_phase equivalence: replicate-pad D by one, put it on the even
    positions of a zero image, correlate with 4 * w (x) w, crop."""
    H, W = 12, 16
    img = rand_img(113, H, W)
    res, down = orc.pyr_level(img, want_down=True)
    Hd, Wd = H // 2, W // 2
    Dp = np.pad(down, 1, mode="edge")
    Z = np.zeros((2 * (Hd + 2), 2 * (Wd + 2)))
    Z[::2, ::2] = Dp
    K2 = 4 * np.outer(WT, WT)
    Zp = np.pad(Z, 2)
    U = np.zeros_like(Z)
    for i in range(5):
        for j in range(5):
            U += K2[i, j] * Zp[i:i + Z.shape[0], j:j + Z.shape[1]]
    U = U[2:2 + H, 2:2 + W]
    assert np.allclose(res, d(img) - U, atol=1e-15)


def test_pyr_brute_force_8x8(orc):
    H = W = 8
    img = rand_img(114, H, W)
    res = orc.pyr_level(img)
    I = d(img)
    cl = lambda v, n: min(max(v, 0), n - 1)
    D = [[sum(WT[i + 2] * WT[j + 2] * I[cl(2 * m + i, H), cl(2 * n + j, W)]
              for i in range(-2, 3) for j in range(-2, 3)) for n in range(W // 2)] for m in range(H // 2)]
    # polyphase taps of 2*w: even phase (1,6,1)/8 on n-1,n,n+1; odd phase (1,1)/2 on n,n+1
    def up1(v, n):
        out = []
        for k in range(n):
            q = k // 2
            if k % 2 == 0:
                out.append((v(cl(q - 1, n // 2)) + 6 * v(q) + v(cl(q + 1, n // 2))) / 8)
            else:
                out.append((v(q) + v(cl(q + 1, n // 2))) / 2)
        return out
    Ux = [up1(lambda q, m=m: D[m][q], W) for m in range(H // 2)]
    for x in range(W):
        col = up1(lambda q, x=x: Ux[q][x], H)
        for y in range(H):
            assert res[y, x] == pytest.approx(I[y, x] - col[y], abs=1e-15)


# --------------------------------------------------------------------------
# down2 / up2: resampling by two with an arbitrary kernel (Sec. V-B)
# --------------------------------------------------------------------------

@pytest.mark.parametrize("H,W,kh,kw,ay,ax", [(14, 18, 6, 8, 2, 3), (9, 7, 5, 3, 4, 0), (8, 8, 1, 1, 0, 0)])
def test_down2_is_the_full_resolution_convolution_sampled_at_even_positions(orc, H, W, kh, kw, ay, ax):
    """Strided convolution = plain convolution (pinned above), every second row and column."""
    img, k = rand_img(121, H, W), rand_kernel(122, kh, kw)
    assert np.allclose(orc.down2(img, k, ay, ax), orc.conv2d(img, k, ay, ax)[::2, ::2], atol=1e-14)


def test_down2_impulse_and_constant(orc):
    kh, kw, ay, ax = 6, 7, 2, 3
    k = rand_kernel(123, kh, kw)
    K = d(k)
    img = np.zeros((20, 24))
    r0, c0 = 9, 13
    img[r0, c0] = 1.0
    out = orc.down2(h(img), k, ay, ax)
    expect = np.zeros((10, 12))
    for y in range(10):
        for x in range(12):
            ry, rx = r0 - 2 * y + ay, c0 - 2 * x + ax
            if 0 <= ry < kh and 0 <= rx < kw:
                expect[y, x] = K[ry, rx]
    assert np.array_equal(out, expect)
    assert np.allclose(orc.down2(h(np.full((11, 13), 0.5)), k, ay, ax), 0.5 * K.sum(), atol=1e-15)


def test_down2_with_the_binomial_kernel_is_the_pyramid_down_step(orc):
    """K = w (x) w, w = [1,4,6,4,1]/16 (products exact in fp16), anchor 2: the pyramid oracle's D, pinned above."""
    w = np.array([1, 4, 6, 4, 1]) / 16.0
    img = rand_img(124, 16, 20)
    _, D = orc.pyr_level(img, want_down=True)
    assert np.allclose(orc.down2(img, h(np.outer(w, w)), 2, 2), D, atol=1e-15)


@pytest.mark.parametrize("H,W,kh,kw,ay,ax", [(7, 9, 6, 8, 1, 2), (5, 6, 2, 2, 0, 0), (6, 5, 4, 10, 1, 4)])
def test_up2_phases_are_four_plain_convolutions(orc, H, W, kh, kw, ay, ax):
    """O(2x+dx, 2y+dy) = convolution of I with K^phase(., ., dx, dy) = K[dy::2, dx::2] (Sec. V-B)."""
    img, k = rand_img(125, H, W), rand_kernel(126, kh, kw)
    out = orc.up2(img, k, ay, ax)
    assert out.shape == (2 * H, 2 * W)
    for dy in range(2):
        for dx in range(2):
            ph = orc.conv2d(img, np.ascontiguousarray(k[dy::2, dx::2]), ay, ax)
            assert np.allclose(out[dy::2, dx::2], ph, atol=1e-14)


def test_up2_as_a_scatter_of_input_pixels(orc):
    """Second formulation: every (edge-padded) input pixel times every tap lands on exactly one output."""
    H, W, kh, kw, ay, ax = 6, 7, 6, 4, 2, 1
    img, k = rand_img(127, H, W), rand_kernel(128, kh, kw)
    I, K = d(img), d(k)
    P = np.pad(I, ((ay, kh // 2 - 1 - ay), (ax, kw // 2 - 1 - ax)), mode="edge")
    expect = np.zeros((2 * H, 2 * W))
    for i in range(P.shape[0]):
        for j in range(P.shape[1]):
            for u in range(kh):
                for v in range(kw):
                    # padded pixel (i, j) is input row i - ay; tap u = 2 ry + dy reads row y//2 + ry - ay
                    y, x = 2 * (i - u // 2) + u % 2, 2 * (j - v // 2) + v % 2
                    if 0 <= y < 2 * H and 0 <= x < 2 * W:
                        expect[y, x] += K[u, v] * P[i, j]
    assert np.allclose(orc.up2(img, k, ay, ax), expect, atol=1e-14)


def test_up2_constant_image_gives_the_phase_sums(orc):
    kh, kw = 8, 6
    k = rand_kernel(129, kh, kw)
    K = d(k)
    out = orc.up2(h(np.full((5, 6), 0.25)), k, 1, 2)
    for dy in range(2):
        for dx in range(2):
            assert np.allclose(out[dy::2, dx::2], 0.25 * K[dy::2, dx::2].sum(), atol=1e-15)


def test_up2_with_the_pyramid_phases_interpolates_a_ramp(orc):
    """The pyramid's 1-D phases (1,6,1)/8 and (1,1)/2 as K = [1,0,6,4,1,4]/8 per axis, anchor 1:
    a linear ramp is reproduced at x/2 (even outputs) and (x+1)/2 - 1/2 + 1/2 (odd outputs: the mean
    of two neighbours), away from the borders."""
    w = np.array([1, 0, 6, 4, 1, 4]) / 8.0
    H, W = 8, 12
    ramp = np.add.outer(np.arange(H) * 4.0, np.arange(W) * 2.0)            # exact in fp16
    out = orc.up2(h(ramp), h(np.outer(w, w)), 1, 1)
    yy, xx = np.meshgrid(np.arange(2 * H), np.arange(2 * W), indexing="ij")
    expect = 4.0 * (yy / 2.0) + 2.0 * (xx / 2.0)
    assert np.allclose(out[2:-2, 2:-2], expect[2:-2, 2:-2], atol=1e-12)


# --------------------------------------------------------------------------
# band_resize / lanczos3: resampling by a non-integer factor (Sec. V-C)
# --------------------------------------------------------------------------

def test_lanczos3_closed_form_values(orc):
    L = orc.lanczos3
    assert L(0.0) == 1.0
    assert np.allclose(L([1.0, -1.0, 2.0, -2.0, 3.0, -3.0, 3.5, -7.0]), 0.0, atol=1e-16)
    assert L(0.5) == pytest.approx(6.0 / np.pi ** 2, abs=1e-15)            # sinc(1/2) sinc(1/6) = (2/pi)(3/pi)
    assert L(1.5) == pytest.approx(-4.0 / (3.0 * np.pi ** 2), abs=1e-15)   # sinc(3/2) sinc(1/2)
    assert L(-2.5) == pytest.approx(L(2.5), abs=0)


def test_lanczos3_matrix_same_size_is_the_identity(orc):
    start, coef = orc.lanczos3_matrix(37, 37)
    assert coef.shape == (37, 7) and np.array_equal(start, np.arange(37) - 3)
    assert np.allclose(coef, np.eye(7)[3], atol=1e-15)


def test_lanczos3_matrix_rows_are_normalised_mirrored_and_centred(orc):
    n_in, n_out = 2048, 143
    start, coef = orc.lanczos3_matrix(n_in, n_out)
    assert coef.shape[1] == orc.lanczos3_band(n_in, n_out) == 86
    assert np.allclose(coef.sum(axis=1), 1.0, atol=1e-14)
    # the sampling grid is symmetric about the middle of the signal: row n_out-1-o is row o mirrored
    dense = np.zeros((n_out, n_in + 400))
    for o in range(n_out):
        dense[o, 200 + start[o]:200 + start[o] + coef.shape[1]] = coef[o]
    assert np.allclose(dense, dense[::-1, ::-1], atol=1e-14)
    # nothing of the window is cut off: the neighbours just outside the band lie outside [-3, 3] scales
    scale = n_in / n_out
    for o in (0, 71, 142):
        centre = (o + 0.5) * scale - 0.5
        assert start[o] - 1 < centre - 3 * scale <= start[o]
        assert start[o] + coef.shape[1] > centre + 3 * scale - 1


def test_lanczos3_matrix_factor_two_reproduces_a_ramp(orc):
    """n_in = 2 n_out: the taps sit symmetrically about the output position 2o + 1/2, so a linear
    signal is reproduced exactly (interior rows)."""
    start, coef = orc.lanczos3_matrix(64, 32)
    ramp = 3.0 * np.arange(64) + 1.0
    for o in range(4, 28):
        assert (coef[o] * ramp[start[o]:start[o] + coef.shape[1]]).sum() == pytest.approx(3.0 * (2 * o + 0.5) + 1.0, abs=1e-12)


def test_band_resize_with_identity_matrices_returns_the_image(orc):
    img = rand_img(131, 9, 11)
    sy, sx = np.arange(9), np.arange(11)
    one = lambda n: h(np.ones((n, 1)))
    assert np.array_equal(orc.band_resize(img, sy, one(9), sx, one(11)), d(img))


def test_band_resize_with_box_rows_is_the_strided_convolution(orc):
    """start[o] = 2o, coefficients (1/2, 1/2) on both axes = down2 (pinned above) with the 2 x 2 box."""
    img = rand_img(132, 12, 16)
    half = h(np.full((1, 2), 0.5))
    out = orc.band_resize(img, 2 * np.arange(6), np.repeat(half, 6, 0), 2 * np.arange(8), np.repeat(half, 8, 0))
    assert np.allclose(out, orc.down2(img, h(np.full((2, 2), 0.25)), 0, 0), atol=1e-15)


def test_band_resize_with_shifted_fixed_rows_is_the_separable_blur(orc):
    """start[o] = o - anchor and the same taps in every row: the blur oracle (pinned above), incl. its clamp."""
    H, W = 10, 13
    img = rand_img(133, H, W)
    ty, tx = rand_kernel(134, 1, 5)[0], rand_kernel(135, 1, 4)[0]
    out = orc.band_resize(img, np.arange(H) - 3, np.tile(ty, (H, 1)), np.arange(W) - 1, np.tile(tx, (W, 1)))
    assert np.allclose(out, orc.sepblur(img, tx, 1, ty, 3), atol=1e-14)


def test_band_resize_brute_force_with_irregular_starts(orc):
    H, W, Ho, Wo, by, bx = 9, 8, 4, 5, 3, 4
    img = rand_img(136, H, W)
    cy, cx = rand_kernel(137, Ho, by), rand_kernel(138, Wo, bx)
    sy, sx = np.array([-2, 1, 5, 8]), np.array([-1, 0, 3, 3, 6])
    I, Cy, Cx = d(img), d(cy), d(cx)
    cl = lambda v, n: min(max(v, 0), n - 1)
    for yo in range(Ho):
        for xo in range(Wo):
            e = sum(Cy[yo, i] * Cx[xo, j] * I[cl(sy[yo] + i, H), cl(sx[xo] + j, W)] for i in range(by) for j in range(bx))
            assert orc.band_resize(img, sy, cy, sx, cx)[yo, xo] == pytest.approx(e, abs=1e-14)


# --------------------------------------------------------------------------
# iir2: second-order recursive filter (Sec. V-D)
# --------------------------------------------------------------------------

def test_iir2_impulse_response_is_the_closed_form_in_the_poles(orc):
    """h_k = (p1^(k+1) - p2^(k+1)) / (p1 - p2) with p1, p2 the roots of z^2 - alpha z - beta (complex here)."""
    alpha, beta = 1.6, -0.8
    p1, p2 = np.roots([1.0, -alpha, -beta])
    x = np.zeros((1, 40))
    x[0, 3] = 1.0
    y = orc.iir2(h(x), alpha, beta)[0]
    k = np.arange(37)
    assert np.allclose(y[3:], ((p1 ** (k + 1) - p2 ** (k + 1)) / (p1 - p2)).real, atol=1e-12)
    assert np.all(y[:3] == 0.0)


def test_iir2_special_cases_are_the_running_sum_and_the_geometric_filter(orc):
    x = rand_img(141, 2, 50)
    assert np.allclose(orc.iir2(x, 1.0, 0.0), np.cumsum(d(x), axis=1), atol=1e-13)
    a = 0.75
    y = orc.iir2(x, a, 0.0)
    for t in (0, 1, 17, 49):
        assert y[1, t] == pytest.approx(sum(a ** k * d(x)[1, t - k] for k in range(t + 1)), abs=1e-13)


def test_iir2_matches_the_library_filter_and_the_step_response_limit(orc):
    from scipy.signal import lfilter
    alpha, beta = 1.2, -0.52
    x = rand_img(142, 2, 300)
    assert np.allclose(orc.iir2(x, alpha, beta), lfilter([1.0], [1.0, -alpha, -beta], d(x), axis=1), atol=1e-11)
    step = orc.iir2(h(np.ones((1, 400))), alpha, beta)[0]
    assert step[-1] == pytest.approx(1.0 / (1.0 - alpha - beta), abs=1e-9)


def test_iir2_channels_are_independent_and_the_recursion_holds_pointwise(orc):
    alpha, beta = 0.9, -0.3
    x = rand_img(143, 3, 64)
    y = orc.iir2(x, alpha, beta)
    X = d(x)
    assert np.allclose(y[:, 2:], X[:, 2:] + alpha * y[:, 1:-1] + beta * y[:, :-2], atol=1e-14)
    assert np.array_equal(orc.iir2(x[1:2], alpha, beta)[0], y[1])


# --------------------------------------------------------------------------
# dct_denoise: transform-domain coring on 16 x 16 windowed tiles (Sec. V-E)
# --------------------------------------------------------------------------

def test_dct16_matrix_is_orthonormal_and_is_the_library_dct(orc):
    from scipy.fft import dct
    D = orc.dct16_matrix()
    assert np.allclose(D @ D.T, np.eye(16), atol=1e-14)
    x = d(rand_img(151, 16, 16))
    assert np.allclose(D @ x, dct(x, type=2, norm="ortho", axis=0), atol=1e-13)
    assert D[0, 0] == 0.25 and D[1, 0] == pytest.approx(np.sqrt(2) / 4 * np.cos(np.pi / 32), abs=1e-16)


def test_sine_window_overlap_sums_to_one(orc):
    w = orc.sine_window16()
    assert np.allclose(w[:8] ** 2 + w[8:] ** 2, 1.0, atol=1e-15)
    assert np.allclose(w, w[::-1], atol=1e-15)


def test_dct_denoise_without_threshold_is_the_identity(orc):
    img = rand_img(152, 32, 40)
    out, _ = orc.dct_denoise(img, 0.0)
    assert np.allclose(out, d(img), atol=1e-13)


def test_dct_denoise_keeps_a_constant_image_at_any_threshold(orc):
    """A constant tile times the window is not constant, so this only holds because the threshold
    test is on the magnitude: with threshold 0 nothing is cut; with a huge one only DC survives and a
    tile reconstructs to the projection of its windowed content on the constant."""
    img = h(np.full((24, 24), 0.5))
    w = orc.sine_window16()
    out, _ = orc.dct_denoise(img, 1e9)
    # interior pixel (8..15, 8..15) is covered by four tiles; each tile's reconstruction is the constant
    # mean(0.5 w2) = 0.5 mean(w)^2; blended with weights w2: 0.5 mean(w)^2 sum(w2) / sum(w2^2)
    w2 = np.outer(w, w)
    y, x = 11, 13
    num = den = 0.0
    for ty in (0, 1):
        for tx in (0, 1):
            ww = w2[y - 8 * ty, x - 8 * tx]
            num += 0.5 * w2.mean() * ww
            den += ww * ww
    assert out[y, x] == pytest.approx(num / den, abs=1e-14)


def test_dct_denoise_removes_a_small_oscillation_and_keeps_a_large_one(orc):
    """One tile's worth of a pure DCT basis function: below the threshold it is cut, above it survives."""
    D, w = orc.dct16_matrix(), orc.sine_window16()
    base = np.outer(D[3], D[5])                       # a unit-energy basis image, |values| <= 1/8
    img16 = np.round((0.5 + 0.25 * base) * 1024) / 1024          # on the fp16 grid
    Y = D @ (img16 * np.outer(w, w)) @ D.T
    big = np.sort(np.abs(Y).ravel())[-2]                        # largest non-DC bin
    img = h(img16)
    cut, _ = orc.dct_denoise(img, big * 1.01)
    kept, _ = orc.dct_denoise(img, 0.0)
    rec_dc = D.T @ (Y * (np.arange(256).reshape(16, 16) == 0)) @ D
    assert np.allclose(kept, img16, atol=1e-13)
    assert np.allclose(cut, rec_dc * np.outer(w, w) / np.outer(w, w) ** 2, atol=1e-12)
