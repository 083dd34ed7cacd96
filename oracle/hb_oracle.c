/*
 * fp64 CPU oracle for the five image stages.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain nested loops over the definition of each stage, in double precision,
 * on the exact fp16 input values (decoded by this file's own half decoder).
 * No tiling, no matrix formulation, no blocking, no fusion: each function is
 * meant to be checked against the paper by eye.  Nothing here is shared with,
 * included by, or linked into the HIP library; only tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it.
 *
 * Conventions common to all functions
 *   - fp16 data arrives as uint16_t IEEE binary16 bit patterns;
 *   - images are row-major, pitches are in elements;
 *   - outputs are double and are NOT rounded to any narrower type;
 *   - "correlation" orientation as printed in the paper (Sec. V-A):
 *     O(x) = sum_r I(x + r) K(r), no kernel flip;
 *   - same-size output; the boundary rule named per function is applied to
 *     the INPUT index (the paper's own examples are valid-domain only; the
 *     benchmark configurations fix same-size output with clamp-to-edge, or
 *     zero padding for the multi-channel convolution);
 *   - an explicit anchor a shifts the window: tap r reads x + r - a, so a = 0
 *     is literally the paper's formula.
 *
 * Parity pins: every function below is pinned by tests/test_oracle_*.py
 * (impulse responses, constants, closed forms, dense Toeplitz products built
 * from the paper's matrix definitions, brute force on tiny inputs).  No
 * function is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- own binary16 decoder ------------------------------------------- */

double hbo_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = (double)frac / 16777216.0;                 /* frac * 2^-24 (zero, subnormal) */
    } else if (expo == 31) {
        if (frac == 0) {
            v = 1.0 / 0.0;
        } else {
            v = 0.0 / 0.0;
        }
    } else {
        v = ldexp(1.0 + (double)frac / 1024.0, expo - 15);   /* (1 + f/2^10) * 2^(e-15) */
    }
    return sign ? -v : v;
}

int hbo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void hbo_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

static inline long clampl(long i, long lo, long hi)
{
    return i < lo ? lo : (i > hi ? hi : i);
}

/* Decode an H x W fp16 image (pitch in elements) into a dense H x W double
 * array.  Every stage starts with this, so the loops below read doubles.  */
static double *decode_image(const uint16_t *in, long H, long W, long pitch)
{
    double *d = (double *)malloc((size_t)H * (size_t)W * sizeof(double));
    if (!d) return NULL;
#pragma omp parallel for schedule(static)
    for (long y = 0; y < H; ++y)
        for (long x = 0; x < W; ++x)
            d[y * W + x] = hbo_half_to_double(in[y * pitch + x]);
    return d;
}

/* ---- 1-D FIR along rows (Sec. V-A, 1-D convolution formula) ---------- */
/* out[y][x] = sum_{r<T} k[r] * in[y][clampW(x + r - a)]                  */

void hbo_fir1d(const uint16_t *in, double *out, int H, int W,
               long in_pitch, long out_pitch,
               const uint16_t *taps, int T, int a)
{
    double k[256];
    double *img = decode_image(in, H, W, in_pitch);
    if (!img) return;
    for (int r = 0; r < T && r < 256; ++r) k[r] = hbo_half_to_double(taps[r]);
#pragma omp parallel for schedule(static)
    for (int y = 0; y < H; ++y) {
        for (int x = 0; x < W; ++x) {
            double acc = 0.0;
            for (int r = 0; r < T; ++r) {
                long xi = clampl((long)x + r - a, 0, W - 1);
                acc += k[r] * img[(size_t)y * W + xi];
            }
            out[(long)y * out_pitch + x] = acc;
        }
    }
    free(img);
}

/* ---- single-channel 2-D convolution, any kernel (Sec. V-A, 2-D form:
 *      O(x, y) = sum_{rx, ry} I(x + rx, y + ry) K(rx, ry); correlation, explicit
 *      anchors, same-size output, clamp-to-edge on both INPUT indices) -------- */
/* taps is kh x kw, row-major: taps[ry * kw + rx] = K(rx, ry). */

void hbo_conv2d(const uint16_t *in, double *out, int H, int W,
                long in_pitch, long out_pitch,
                const uint16_t *taps, int kh, int kw, int ay, int ax)
{
    double *img = decode_image(in, H, W, in_pitch);
    double *k = (double *)malloc((size_t)kh * (size_t)kw * sizeof(double));
    if (!img || !k) { free(img); free(k); return; }
    for (int i = 0; i < kh * kw; ++i) k[i] = hbo_half_to_double(taps[i]);
#pragma omp parallel for schedule(static)
    for (int y = 0; y < H; ++y) {
        for (int x = 0; x < W; ++x) {
            double acc = 0.0;
            for (int ry = 0; ry < kh; ++ry) {
                long yi = clampl((long)y + ry - ay, 0, H - 1);
                for (int rx = 0; rx < kw; ++rx) {
                    long xi = clampl((long)x + rx - ax, 0, W - 1);
                    acc += k[ry * kw + rx] * img[(size_t)yi * W + xi];
                }
            }
            out[(long)y * out_pitch + x] = acc;
        }
    }
    free(img);
    free(k);
}

/* ---- resampling by a factor of two with an arbitrary kernel (Sec. V-B) ----
 * Downsampling (strided convolution): O(x, y) = sum_{rx, ry} I(2x + rx, 2y + ry) K(rx, ry),
 * here with explicit anchors and clamp-to-edge on both INPUT indices; the
 * output has ceil(H/2) x ceil(W/2) samples.  taps[ry * kw + rx] = K(rx, ry). */

void hbo_down2(const uint16_t *in, double *out, int H, int W,
               long in_pitch, long out_pitch,
               const uint16_t *taps, int kh, int kw, int ay, int ax)
{
    double *img = decode_image(in, H, W, in_pitch);
    double *k = (double *)malloc((size_t)kh * (size_t)kw * sizeof(double));
    if (!img || !k) { free(img); free(k); return; }
    for (int i = 0; i < kh * kw; ++i) k[i] = hbo_half_to_double(taps[i]);
    int Ho = (H + 1) / 2, Wo = (W + 1) / 2;
#pragma omp parallel for schedule(static)
    for (int y = 0; y < Ho; ++y) {
        for (int x = 0; x < Wo; ++x) {
            double acc = 0.0;
            for (int ry = 0; ry < kh; ++ry) {
                long yi = clampl(2L * y + ry - ay, 0, H - 1);
                for (int rx = 0; rx < kw; ++rx) {
                    long xi = clampl(2L * x + rx - ax, 0, W - 1);
                    acc += k[ry * kw + rx] * img[(size_t)yi * W + xi];
                }
            }
            out[(long)y * out_pitch + x] = acc;
        }
    }
    free(img);
    free(k);
}

/* Upsampling: O(x, y) = sum_{rx, ry} I(floor(x/2) + rx, floor(y/2) + ry) K(2 rx + x%2, 2 ry + y%2),
 * rx < kw/2, ry < kh/2 (kh, kw even), anchors in input pixels, clamp-to-edge on
 * both INPUT indices; the output has 2H x 2W samples. */

void hbo_up2(const uint16_t *in, double *out, int H, int W,
             long in_pitch, long out_pitch,
             const uint16_t *taps, int kh, int kw, int ay, int ax)
{
    double *img = decode_image(in, H, W, in_pitch);
    double *k = (double *)malloc((size_t)kh * (size_t)kw * sizeof(double));
    if (!img || !k) { free(img); free(k); return; }
    for (int i = 0; i < kh * kw; ++i) k[i] = hbo_half_to_double(taps[i]);
#pragma omp parallel for schedule(static)
    for (int y = 0; y < 2 * H; ++y) {
        for (int x = 0; x < 2 * W; ++x) {
            double acc = 0.0;
            for (int ry = 0; ry < kh / 2; ++ry) {
                long yi = clampl((long)(y / 2) + ry - ay, 0, H - 1);
                for (int rx = 0; rx < kw / 2; ++rx) {
                    long xi = clampl((long)(x / 2) + rx - ax, 0, W - 1);
                    acc += k[(2 * ry + y % 2) * kw + 2 * rx + x % 2] * img[(size_t)yi * W + xi];
                }
            }
            out[(long)y * out_pitch + x] = acc;
        }
    }
    free(img);
    free(k);
}

/* ---- resampling by a non-integer factor with precomputed banded matrices
 *      (Sec. V-C): each axis is one sparse matrix whose row o has `band`
 *      entries starting at input index start[o]; vertical and horizontal
 *      resizing are separable.  One plane:
 *        out[yo][xo] = sum_i sum_j cy[yo][i] cx[xo][j]
 *                      * in[clampH(sy[yo] + i)][clampW(sx[xo] + j)]        */

void hbo_band_resize(const uint16_t *in, double *out, int H, int W, int Ho, int Wo,
                     long in_pitch, long out_pitch,
                     const int *sy, const uint16_t *cy, int by,
                     const int *sx, const uint16_t *cx, int bx)
{
    double *img = decode_image(in, H, W, in_pitch);
    double *ky = (double *)malloc((size_t)Ho * (size_t)by * sizeof(double));
    double *kx = (double *)malloc((size_t)Wo * (size_t)bx * sizeof(double));
    if (!img || !ky || !kx) { free(img); free(ky); free(kx); return; }
    for (long i = 0; i < (long)Ho * by; ++i) ky[i] = hbo_half_to_double(cy[i]);
    for (long i = 0; i < (long)Wo * bx; ++i) kx[i] = hbo_half_to_double(cx[i]);
#pragma omp parallel for schedule(static)
    for (int yo = 0; yo < Ho; ++yo) {
        for (int xo = 0; xo < Wo; ++xo) {
            double acc = 0.0;
            for (int i = 0; i < by; ++i) {
                long yi = clampl((long)sy[yo] + i, 0, H - 1);
                double row = 0.0;
                for (int j = 0; j < bx; ++j) {
                    long xi = clampl((long)sx[xo] + j, 0, W - 1);
                    row += kx[(size_t)xo * bx + j] * img[(size_t)yi * W + xi];
                }
                acc += ky[(size_t)yo * by + i] * row;
            }
            out[(long)yo * out_pitch + xo] = acc;
        }
    }
    free(img);
    free(ky);
    free(kx);
}

/* ---- second-order recursive filter (Sec. V-D):
 *        Y_t = X_t + alpha Y_{t-1} + beta Y_{t-2},  Y_{-1} = Y_{-2} = 0,
 *      one independent recursion per channel, written as the serial loop it is. */

void hbo_iir2(const uint16_t *in, double *out, int C, long T, long in_pitch, long out_pitch,
              double alpha, double beta)
{
    for (int c = 0; c < C; ++c) {
        double y1 = 0.0, y2 = 0.0;
        for (long t = 0; t < T; ++t) {
            double y = hbo_half_to_double(in[(long)c * in_pitch + t]) + alpha * y1 + beta * y2;
            out[(long)c * out_pitch + t] = y;
            y2 = y1;
            y1 = y;
        }
    }
}

/* ---- separable blur: rows, then columns (Sec. V-A; the 2-D form with
 *      K(rx, ry) = kx[rx] * ky[ry]) ------------------------------------ */
/* tmp[y][x] = sum_r kx[r] in[y][clampW(x + r - ax)]
 * out[y][x] = sum_r ky[r] tmp[clampH(y + r - ay)][x];  tmp stays fp64.   */

void hbo_sepblur(const uint16_t *in, double *out, int H, int W,
                 long in_pitch, long out_pitch,
                 const uint16_t *taps_x, int Tx, int ax,
                 const uint16_t *taps_y, int Ty, int ay)
{
    double kx[256], ky[256];
    double *img = decode_image(in, H, W, in_pitch);
    double *tmp = (double *)malloc((size_t)H * (size_t)W * sizeof(double));
    if (!img || !tmp) { free(img); free(tmp); return; }
    for (int r = 0; r < Tx && r < 256; ++r) kx[r] = hbo_half_to_double(taps_x[r]);
    for (int r = 0; r < Ty && r < 256; ++r) ky[r] = hbo_half_to_double(taps_y[r]);
#pragma omp parallel for schedule(static)
    for (int y = 0; y < H; ++y) {
        for (int x = 0; x < W; ++x) {
            double acc = 0.0;
            for (int r = 0; r < Tx; ++r) {
                long xi = clampl((long)x + r - ax, 0, W - 1);
                acc += kx[r] * img[(size_t)y * W + xi];
            }
            tmp[(size_t)y * W + x] = acc;
        }
    }
#pragma omp parallel for schedule(static)
    for (int y = 0; y < H; ++y) {
        for (int x = 0; x < W; ++x) {
            double acc = 0.0;
            for (int r = 0; r < Ty; ++r) {
                long yi = clampl((long)y + r - ay, 0, H - 1);
                acc += ky[r] * tmp[(size_t)yi * W + x];
            }
            out[(long)y * out_pitch + x] = acc;
        }
    }
    free(img);
    free(tmp);
}

/* ---- summed-area table (inclusive 2-D prefix sum; the benchmark's own
 *      stage, not in the paper) --------------------------------------- */
/* S[i][j] = sum_{y<=i} sum_{x<=j} in[y][x], by a running row sum plus the
 * previous table row.                                                    */

void hbo_sat2d(const uint16_t *in, double *out, int H, int W,
               long in_pitch, long out_pitch)
{
    for (int i = 0; i < H; ++i) {
        double run = 0.0;
        for (int j = 0; j < W; ++j) {
            run += hbo_half_to_double(in[(long)i * in_pitch + j]);
            out[(long)i * out_pitch + j] = run + (i > 0 ? out[(long)(i - 1) * out_pitch + j] : 0.0);
        }
    }
}

/* ---- multi-channel 3x3 convolution, NHWC, zero padding 1, stride 1 ----
 *      (Sec. V-A 2-D formula summed over input channels; Sec. IV conv
 *      layer without bias/activation) ---------------------------------- */
/* out[n][y][x][co] = sum_{ky,kx<3} sum_ci in[n][y+ky-1][x+kx-1][ci] *
 *                    w[ky][kx][ci][co], terms outside the image omitted. */

/* Rows y0 <= y < y1 of every image in the batch; out is the full
 * N*H*W*Cout array, only the requested rows are written.                 */
void hbo_conv3x3_rows(const uint16_t *in, const uint16_t *w, double *out,
                      int N, int H, int W, int Cin, int Cout, int y0, int y1)
{
    double *wd = decode_image(w, 9L * Cin, Cout, Cout);
    if (!wd) return;
    for (int n = 0; n < N; ++n) {
        /* decode only the input rows the requested output rows touch */
        int r0 = y0 - 1 < 0 ? 0 : y0 - 1, r1 = y1 + 1 > H ? H : y1 + 1;
        double *img = decode_image(in + ((size_t)n * H + r0) * W * Cin,
                                   r1 - r0, (long)W * Cin, (long)W * Cin);
        if (!img) break;
#pragma omp parallel for schedule(static)
        for (int y = y0; y < y1; ++y) {
            for (int x = 0; x < W; ++x) {
                for (int co = 0; co < Cout; ++co) {
                    double acc = 0.0;
                    for (int ky = 0; ky < 3; ++ky) {
                        int yy = y + ky - 1;
                        if (yy < 0 || yy >= H) continue;
                        for (int kx = 0; kx < 3; ++kx) {
                            int xx = x + kx - 1;
                            if (xx < 0 || xx >= W) continue;
                            const double *px = img + ((size_t)(yy - r0) * W + xx) * Cin;
                            const double *wk = wd + ((size_t)(ky * 3 + kx) * Cin) * Cout + co;
                            for (int ci = 0; ci < Cin; ++ci)
                                acc += px[ci] * wk[(size_t)ci * Cout];
                        }
                    }
                    out[(((size_t)n * H + y) * W + x) * Cout + co] = acc;
                }
            }
        }
        free(img);
    }
    free(wd);
}

void hbo_conv3x3(const uint16_t *in, const uint16_t *w, double *out,
                 int N, int H, int W, int Cin, int Cout)
{
    hbo_conv3x3_rows(in, w, out, N, H, W, Cin, Cout, 0, H);
}

/* Selected output pixels (all Cout channels each): out[p*Cout + co].
 * Same sum as above, decoding operands where they are used.              */
void hbo_conv3x3_points(const uint16_t *in, const uint16_t *w, double *out,
                        int N, int H, int W, int Cin, int Cout,
                        long npts, const int *pn, const int *py, const int *px)
{
    (void)N;
#pragma omp parallel for schedule(static)
    for (long p = 0; p < npts; ++p) {
        for (int co = 0; co < Cout; ++co) {
            double acc = 0.0;
            for (int ky = 0; ky < 3; ++ky) {
                int yy = py[p] + ky - 1;
                if (yy < 0 || yy >= H) continue;
                for (int kx = 0; kx < 3; ++kx) {
                    int xx = px[p] + kx - 1;
                    if (xx < 0 || xx >= W) continue;
                    const uint16_t *pi = in + (((size_t)pn[p] * H + yy) * W + xx) * Cin;
                    const uint16_t *wk = w + ((size_t)(ky * 3 + kx) * Cin) * Cout + co;
                    for (int ci = 0; ci < Cin; ++ci)
                        acc += hbo_half_to_double(pi[ci]) * hbo_half_to_double(wk[(size_t)ci * Cout]);
                }
            }
            out[p * Cout + co] = acc;
        }
    }
}

/* ---- one Laplacian-pyramid level (Sec. V-B: strided convolution for the
 *      2x downsample, two-phase filter for the 2x upsample) ------------- */
/* wt = [1,4,6,4,1]/16 on offsets -2..2.
 * D[m][n] = sum_{i,j} wt[i] wt[j] in[clampH(2m+i)][clampW(2n+j)]   (H/2 x W/2)
 * per axis, gain 2, D index clamped to the D extent:
 *   U[2n]   = (D[c(n-1)] + 6 D[n] + D[c(n+1)]) / 8
 *   U[2n+1] = (D[n] + D[c(n+1)]) / 2
 * applied along x, then along y;  res = in - U.   D is not rounded.      */

void hbo_pyr_level(const uint16_t *in, double *res, double *down_or_null,
                   int H, int W, long in_pitch, long res_pitch, long down_pitch)
{
    static const double wt[5] = { 1.0 / 16, 4.0 / 16, 6.0 / 16, 4.0 / 16, 1.0 / 16 };
    int Hd = H / 2, Wd = W / 2;
    double *img = decode_image(in, H, W, in_pitch);
    double *D = (double *)malloc((size_t)Hd * Wd * sizeof(double));
    double *Ux = (double *)malloc((size_t)Hd * W * sizeof(double));
    if (!img || !D || !Ux) { free(img); free(D); free(Ux); return; }

#pragma omp parallel for schedule(static)
    for (int m = 0; m < Hd; ++m) {
        for (int n = 0; n < Wd; ++n) {
            double acc = 0.0;
            for (int i = -2; i <= 2; ++i) {
                long yy = clampl(2L * m + i, 0, H - 1);
                for (int j = -2; j <= 2; ++j) {
                    long xx = clampl(2L * n + j, 0, W - 1);
                    acc += wt[i + 2] * wt[j + 2] * img[(size_t)yy * W + xx];
                }
            }
            D[(size_t)m * Wd + n] = acc;
        }
    }
    if (down_or_null) {
        for (int m = 0; m < Hd; ++m)
            for (int n = 0; n < Wd; ++n)
                down_or_null[(long)m * down_pitch + n] = D[(size_t)m * Wd + n];
    }
    /* upsample along x */
#pragma omp parallel for schedule(static)
    for (int m = 0; m < Hd; ++m) {
        const double *d = D + (size_t)m * Wd;
        double *u = Ux + (size_t)m * W;
        for (int n = 0; n < Wd; ++n) {
            long nm = clampl(n - 1, 0, Wd - 1), np = clampl(n + 1, 0, Wd - 1);
            u[2 * n]     = (d[nm] + 6.0 * d[n] + d[np]) / 8.0;
            u[2 * n + 1] = (d[n] + d[np]) / 2.0;
        }
    }
    /* upsample along y and subtract */
#pragma omp parallel for schedule(static)
    for (int m = 0; m < Hd; ++m) {
        long mm = clampl(m - 1, 0, Hd - 1), mp = clampl(m + 1, 0, Hd - 1);
        const double *a = Ux + (size_t)mm * W, *b = Ux + (size_t)m * W, *c = Ux + (size_t)mp * W;
        for (int x = 0; x < W; ++x) {
            double ue = (a[x] + 6.0 * b[x] + c[x]) / 8.0;
            double uo = (b[x] + c[x]) / 2.0;
            res[(long)(2 * m) * res_pitch + x] = img[(size_t)(2 * m) * W + x] - ue;
            res[(long)(2 * m + 1) * res_pitch + x] = img[(size_t)(2 * m + 1) * W + x] - uo;
        }
    }
    free(img);
    free(D);
    free(Ux);
}
