// hb_pyr_level: one Laplacian-pyramid level (2x down, 2x up, residual) as four chained
// products with strided-Toeplitz and two-phase coefficient matrices (Sec. V-B), and its
// vector-ALU twin.
//
// MFMA formulation.  w = [1,4,6,4,1]/16.  Every pass contracts over the index that the
// previous accumulator holds per lane, so the whole chain stays in registers:
//   1 down, x   T1[y][n]  = sum_k P[y][k]  * Adx[k][n]    Adx[k][n] = w[k - 2n]        (A_down)
//   2 down, y   D'[n][m]  = sum_k T1[k][n] * Ady[k][m]    Ady[k][m] = w[k - 2m]
//   3 up,   x   U1[m][x]  = sum_k D[m][k]  * Aux[k][x]    Aux[k][x] = K_phase(k - x/2, x%2)
//   4 up,   y   U'[x][y]  = sum_k U1[k][x] * Auy[k][y]    Auy[k][y] = K_phase(k - y/2, y%2)
// with K_phase the two phases of 2w: even outputs (1,6,1)/8 on D[q-1..q+1], odd outputs
// (1,1)/2 on D[q..q+1].  The phases are interleaved by the coefficient matrix itself
// (column x of Aux belongs to phase x%2), so pass 4 ends with four consecutive output
// columns of one row per lane and the residual in - U leaves with 16-byte stores.
//
// Geometry.  A wave owns a strip of NS blocks of 32 output columns and walks down in steps
// of 32 output rows.  D tiles (16 x 16) lie on a grid shifted by 8 so that the K = 32
// window of an up pass (two adjacent D tiles) covers the 18 values that 32 outputs need:
// NS + 1 column tiles per strip, one extra row tile per task.  A D tile needs 35 image
// rows/columns: a K = 32 plus a K = 16 product over three image row tiles / a 48-pixel
// window.  At the image border the up passes clamp the D index; there the coefficient
// fragments are rebuilt from absolute indices (taps that clamp onto the same D sample
// add up), which also makes out-of-range D tiles (computed from clamped pixels) inert.
#include "hb_device.hpp"
#include "hb_host.hpp"

#ifndef HB_PYR_NS
#define HB_PYR_NS 2           // 32-column output blocks per wave strip
#endif
#ifndef HB_PYR_WAVES
#define HB_PYR_WAVES 8192     // aim for about this many wave tasks per launch
#endif

namespace hb {

struct PyrArgs {
    const half_t* in;
    float* res;
    half_t* down;      // may be null
    int H, W, Hd, Wd;
    int64_t in_pitch, res_pitch, down_pitch;
    int steps;         // 32-row output steps per task
    TaskGrid grid;     // strips x row segments
};

__device__ __forceinline__ half_t w5(int t) {
    // [1,4,6,4,1]/16, zero outside
    const float v = (t == 0 || t == 4) ? 0.0625f : (t == 1 || t == 3) ? 0.25f : (t == 2) ? 0.375f : 0.f;
    return (half_t)v;
}
// Weight of D[q + delta] in output 2q + phase (gain 2 per axis).
__device__ __forceinline__ float upw(int phase, int delta) {
    if (phase) return (delta == 0 || delta == 1) ? 0.5f : 0.f;
    return (delta == 0) ? 0.75f : (delta == -1 || delta == 1) ? 0.125f : 0.f;
}
// Weight of D[dabs] in output xabs when the D index is clamped to [0, n-1].
__device__ __forceinline__ float upw_clamped(int dabs, int xabs, int n) {
    const int q = xabs >> 1, ph = xabs & 1;
    float s = 0.f;
#pragma unroll
    for (int delta = -1; delta <= 1; ++delta)
        if (clampi(q + delta, 0, n - 1) == dabs) s += upw(ph, delta);
    return s;
}

// Weight of pixel u in D sample n when the pixel index 2n + i (i = -2..2) is clamped to [0, len-1].
__device__ __forceinline__ half_t down_tap_clamped(int n, int u, int len) {
    float s = 0.f;
#pragma unroll
    for (int i = -2; i <= 2; ++i)
        if (clampi(2 * n + i, 0, len - 1) == u) s += (float)w5(i + 2);
    return (half_t)s;                                     // multiples of 1/16 up to 1: exact
}

// B fragment of an up pass for the K = 32 window starting at D index d0 and the 16 outputs
// starting at x0abs (lane c = output, chained slot order), D extent n.
__device__ __forceinline__ half8 up_fragment_clamped(int d0, int x0abs, int n, int c, int g) {
    half8 r;
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = (half_t)upw_clamped(d0 + krow32(g, i), x0abs + c, n);
    return r;
}

// Interior coefficient fragments (B operands; lane c = output index of the pass).
struct PyrCoef {
    half8 dx32;        // A_down, slots = pixels 0..31 of the window (natural order)
    half8 dy32;        // A_down, slots = rows 0..31 of the window (chained order)
    half8 d16;         // A_down for pixels / rows 32..35, in slots 8g + (0..3); zero in 8g + (4..7)
    half8 up[2];       // phase matrix for the first / second 16 outputs of a 32-output block
};

// One task: a strip of NS blocks, nsteps output steps.  FAST = the task touches no image
// border: plain loads, interior fragments, unmasked stores.
template <int NS, bool FAST, bool STREAM>
__device__ __forceinline__ void pyr_task(const PyrArgs& p, const PyrCoef& k, float* patch, int X0, int R0,
                                         int nsteps, int c, int g) {
    constexpr int NT = NS + 1;                            // D column tiles per strip
    const int Dx0 = X0 / 2 - 8;                           // first D column of tile 0
    const int M0 = R0 / 2 - 8;                            // first D row of row tile 0
    const int px0 = 2 * Dx0 - 2;                          // first pixel of tile 0's window
    const int y00 = 2 * M0 - 2;                           // first image row of image tile 0
    const half4 z4 = half4{0, 0, 0, 0};

    half4 T1[3][NT];                                      // row-filtered image tiles r-2, r-1, r
    half4 U1[2][NS][2];                                   // up-x results of D row tiles q-1, q
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
        for (int t = 0; t < NT; ++t) T1[a][t] = z4;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int t = 0; t < NS; ++t)
#pragma unroll
            for (int h = 0; h < 2; ++h) U1[a][t][h] = z4;

    // border tasks: per D column tile, a pixel window moved inside the row and A_down
    // fragments with the column clamp folded in
    int wsx[NT];
    half8 fdx32[FAST ? 1 : NT], fdx16[FAST ? 1 : NT];
    if (!FAST) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            wsx[t] = clampi(px0 + 32 * t, 0, p.W - 48);
            const int n = Dx0 + 16 * t + c;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                fdx32[t][i] = down_tap_clamped(n, wsx[t] + 8 * g + i, p.W);
                fdx16[t][i] = (i < 4) ? down_tap_clamped(n, wsx[t] + 32 + 4 * g + i, p.W) : (half_t)0;
            }
        }
    }

    half8 win32[NT], nxt32[NT];
    half4 win16[NT], nxt16[NT];
    auto load_rows = [&](int r, half8 (&a32)[NT], half4 (&a16)[NT]) {
        if (FAST) {
            const half_t* src = p.in + px0;
            const uint32_t off = ((uint32_t)(y00 + 16 * r + c) * (uint32_t)p.in_pitch) * 2u;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                a32[t] = ldg8(src, off + 2u * (32u * t + 8u * g));
                a16[t] = ldg4(src, off + 2u * (32u * t + 32u + 4u * g));
            }
        } else {
            const half_t* row = p.in + (int64_t)clampi(y00 + 16 * r + c, 0, p.H - 1) * p.in_pitch;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                a32[t] = *reinterpret_cast<const half8_u*>(row + wsx[t] + 8 * g);
                a16[t] = *reinterpret_cast<const half4_u*>(row + wsx[t] + 32 + 4 * g);
            }
        }
    };

    const int ntiles = 2 * nsteps + 3;                    // image row tiles of this task
    load_rows(0, win32, win16);
    for (int r = 0; r < ntiles; ++r) {
        if (r + 1 < ntiles) load_rows(r + 1, nxt32, nxt16);   // next row tile in flight during the products
        // pass 1: this image row tile, all D column tiles
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            T1[0][t] = T1[1][t];
            T1[1][t] = T1[2][t];
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
            acc = mfma16x16x32(win32[t], FAST ? k.dx32 : fdx32[t], acc);
            acc = mfma16x16x32(join(win16[t], z4), FAST ? k.d16 : fdx16[t], acc);
            T1[2][t] = to_half4(acc);
        }
        if ((r & 1) == 0 && r >= 2) {
            const int q = r / 2 - 1;                      // D row tile completed by image tiles 2q .. 2q+2
            // pass 2: D tile (lane c = D row, four D columns)
            half4 D[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                floatx4 acc = {0.f, 0.f, 0.f, 0.f};
                acc = mfma16x16x32(join(T1[0][t], T1[1][t]), k.dy32, acc);
                acc = mfma16x16x32(join(T1[2][t], z4), k.d16, acc);
                D[t] = to_half4(acc);
            }
            if (p.down) {
                // each task writes the D samples under its own outputs
                const int m = M0 + 16 * q + c;
                if (m >= R0 / 2 && m < min(R0 / 2 + 16 * nsteps, p.Hd)) {
                    half_t* drow = p.down + (int64_t)m * p.down_pitch;
#pragma unroll
                    for (int t = 0; t < NT; ++t)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int n = Dx0 + 16 * t + 4 * g + v;
                            if (n >= X0 / 2 && n < min(X0 / 2 + 16 * NS, p.Wd)) drow[n] = D[t][v];
                        }
                }
            }
            // pass 3: up along x (lane c = output column, four D rows)
#pragma unroll
            for (int t = 0; t < NS; ++t)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    U1[0][t][h] = U1[1][t][h];
                    const half8 b = FAST ? k.up[h]
                                         : up_fragment_clamped(Dx0 + 16 * t, X0 + 32 * t + 16 * h, p.Wd, c, g);
                    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
                    acc = mfma16x16x32(join(D[t], D[t + 1]), b, acc);
                    U1[1][t][h] = to_half4(acc);
                }
            if (q >= 1) {
                // pass 4: up along y for output rows R0 + 32 (q-1) + (0..31), then the residual
                const int Rq = R0 + 32 * (q - 1);
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2) {
                    const half8 b = FAST ? k.up[h2]
                                         : up_fragment_clamped(M0 + 16 * (q - 1), Rq + 16 * h2, p.Hd, c, g);
                    const int yo = Rq + 16 * h2 + c;
                    if (FAST) {
                        const half_t* isrc = p.in + X0;
                        float* odst = p.res + X0;
                        const uint32_t ioff = ((uint32_t)yo * (uint32_t)p.in_pitch + 4u * g) * 2u;
                        const uint32_t ooff = ((uint32_t)yo * (uint32_t)p.res_pitch + 4u * g) * 4u;
                        half4 px[NS][2];
#pragma unroll
                        for (int t = 0; t < NS; ++t)
#pragma unroll
                            for (int h = 0; h < 2; ++h) px[t][h] = ldg4(isrc, ioff + 2u * (32u * t + 16u * h));
                        floatx4 rv[2 * NS];
#pragma unroll
                        for (int t = 0; t < NS; ++t)
#pragma unroll
                            for (int h = 0; h < 2; ++h) {
                                floatx4 acc = {0.f, 0.f, 0.f, 0.f};
                                acc = mfma16x16x32(join(U1[0][t][h], U1[1][t][h]), b, acc);
                                rv[2 * t + h] = floatx4{(float)px[t][h][0] - acc[0], (float)px[t][h][1] - acc[1],
                                                        (float)px[t][h][2] - acc[2], (float)px[t][h][3] - acc[3]};
                            }
#ifdef HB_DIRECT_STORES
#pragma unroll
                        for (int w = 0; w < 2 * NS; ++w) stg4<STREAM>(odst, ooff + 64u * w, rv[w]);
#else
                        store_rows_via_lds<2 * NS, STREAM>(patch, odst + (int64_t)(Rq + 16 * h2) * p.res_pitch,
                                                           (uint32_t)p.res_pitch, rv, (g << 4) | c);
#endif
                    } else {
                        const half_t* irow = p.in + (int64_t)min(yo, p.H - 1) * p.in_pitch;
                        float* orow = p.res + (int64_t)yo * p.res_pitch;
#pragma unroll
                        for (int t = 0; t < NS; ++t)
#pragma unroll
                            for (int h = 0; h < 2; ++h) {
                                floatx4 acc = {0.f, 0.f, 0.f, 0.f};
                                acc = mfma16x16x32(join(U1[0][t][h], U1[1][t][h]), b, acc);
                                const int xo = X0 + 32 * t + 16 * h + 4 * g;
                                if (yo < p.H && xo < p.W) {
                                    const half4 px = load4_clamp(irow, xo, p.W);
                                    floatx4 rv = {(float)px[0] - acc[0], (float)px[1] - acc[1],
                                                  (float)px[2] - acc[2], (float)px[3] - acc[3]};
                                    store4_mask(orow, xo, p.W, rv);
                                }
                            }
                    }
                }
            }
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            win32[t] = nxt32[t];
            win16[t] = nxt16[t];
        }
    }
}

template <bool STREAM>
__global__ void __launch_bounds__(256) pyr_mfma_kernel(PyrArgs p) {
    constexpr int NS = HB_PYR_NS;
    const int lane = threadIdx.x & 63;
    const int c = lane & 15, g = lane >> 4;

    __shared__ __attribute__((aligned(16))) float s_patch[4][RowPatch<2 * NS>::kFloats];
    PyrCoef k;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        k.dx32[i] = w5(8 * g + i - 2 * c);
        k.dy32[i] = w5(krow32(g, i) - 2 * c);
        k.d16[i] = (i < 4) ? w5(32 + 4 * g + i - 2 * c) : (half_t)0;
#pragma unroll
        for (int h = 0; h < 2; ++h)
            k.up[h][i] = (half_t)upw(c & 1, krow32(g, i) - 8 - 8 * h - (c >> 1));
    }

#ifdef HB_NO_XCD_MAP
    const int wgpos = blockIdx.x;
#else
    const int wgpos = xcd_contiguous(blockIdx.x, gridDim.x);
#endif
    const int wave = __builtin_amdgcn_readfirstlane(wgpos * 4 + (threadIdx.x >> 6));
    const int nwaves = (gridDim.x * blockDim.x) >> 6;
    const int ntasks = p.grid.count();
    for (int task = wave; task < ntasks; task += nwaves) {
        const int seg = task / p.grid.nct, ct = task - seg * p.grid.nct;
        const int X0 = 32 * NS * ct;                      // first output column
        const int R0 = seg * p.steps * 32;                // first output row
        const int nsteps = min(p.steps, (p.H - R0 + 31) / 32);
        if (p.grid.interior(seg, ct)) {
            pyr_task<NS, true, STREAM>(p, k, s_patch[threadIdx.x >> 6], X0, R0, nsteps, c, g);
        } else {
#ifndef HB_PYR_NOBORDER
            // border task: one 32-column block at a time keeps this path's register use low
#pragma unroll 1
            for (int b = 0; b < NS; ++b)
                if (X0 + 32 * b < p.W) pyr_task<1, false, STREAM>(p, k, s_patch[threadIdx.x >> 6], X0 + 32 * b, R0, nsteps, c, g);
#endif
        }
    }
}

// ---------------------------------------------------------------------------
// Vector-ALU twin: a 32 x 64 output tile per workgroup, every stage through LDS with
// plain fp32 FMAs.  D is rounded to fp16 as in the MFMA path; the D tile is gathered at
// clamped D indices, which is the definition's border rule verbatim.
constexpr int kPTH = 32, kPTW = 64;
constexpr int kPRows = kPTH + 7;             // image rows 2(M-1)-2 .. 2(M+16)+2
constexpr int kPPitch = 88;                  // image columns X0-8 .. X0+79
constexpr int kPDR = kPTH / 2 + 2, kPDC = kPTW / 2 + 2;

__global__ void __launch_bounds__(256) pyr_valu_kernel(PyrArgs p) {
    __shared__ half_t s_px[kPRows * kPPitch];
    __shared__ float s_hx[kPRows * (kPDC + 1)];
    __shared__ half_t s_d[kPDR * (kPDC + 2)];
    __shared__ float s_u1[kPDR * (kPTW + 4)];
    const float wt[5] = {0.0625f, 0.25f, 0.375f, 0.25f, 0.0625f};
    const int nctv = (p.W + kPTW - 1) / kPTW;
    const int rt = blockIdx.x / nctv, ct = blockIdx.x - rt * nctv;
    const int X0 = ct * kPTW, R0 = rt * kPTH;
    const int xs = X0 - 8, ys = R0 - 4;
    for (int idx = threadIdx.x; idx < kPRows * (kPPitch / 8); idx += 256) {
        const int r = idx / (kPPitch / 8), ch = idx - r * (kPPitch / 8);
        const half_t* row = p.in + (int64_t)clampi(ys + r, 0, p.H - 1) * p.in_pitch;
        *reinterpret_cast<half8*>(&s_px[r * kPPitch + 8 * ch]) = load8_clamp(row, xs + 8 * ch, p.W);
    }
    __syncthreads();
    // down along x at the (clamped) D columns this tile's up pass reads
    for (int idx = threadIdx.x; idx < kPRows * kPDC; idx += 256) {
        const int r = idx / kPDC, j = idx - r * kPDC;
        const int dc = clampi(X0 / 2 - 1 + j, 0, p.Wd - 1);
        float acc = 0.f;
#pragma unroll
        for (int k = 0; k < 5; ++k)
            acc = fmaf(wt[k], (float)s_px[r * kPPitch + clampi(2 * dc + k - 2, 0, p.W - 1) - xs], acc);
        s_hx[r * (kPDC + 1) + j] = acc;
    }
    __syncthreads();
    // down along y -> D (fp16), optional store of the D samples under this tile
    for (int idx = threadIdx.x; idx < kPDR * kPDC; idx += 256) {
        const int i = idx / kPDC, j = idx - i * kPDC;
        const int dr = clampi(R0 / 2 - 1 + i, 0, p.Hd - 1);
        float acc = 0.f;
#pragma unroll
        for (int k = 0; k < 5; ++k)
            acc = fmaf(wt[k], s_hx[(clampi(2 * dr + k - 2, 0, p.H - 1) - ys) * (kPDC + 1) + j], acc);
        const half_t dv = (half_t)acc;
        s_d[i * (kPDC + 2) + j] = dv;
        if (p.down && i >= 1 && i <= kPTH / 2 && j >= 1 && j <= kPTW / 2) {
            const int m = R0 / 2 - 1 + i, n = X0 / 2 - 1 + j;
            if (m < p.Hd && n < p.Wd) p.down[(int64_t)m * p.down_pitch + n] = dv;
        }
    }
    __syncthreads();
    // up along x
    for (int idx = threadIdx.x; idx < kPDR * kPTW; idx += 256) {
        const int i = idx / kPTW, x = idx - i * kPTW;
        const half_t* d = &s_d[i * (kPDC + 2) + (x >> 1)];       // d[0] = D[q-1], d[1] = D[q], d[2] = D[q+1]
        s_u1[i * (kPTW + 4) + x] = (x & 1) ? 0.5f * ((float)d[1] + (float)d[2])
                                           : 0.125f * ((float)d[0] + (float)d[2]) + 0.75f * (float)d[1];
    }
    __syncthreads();
    // up along y, residual; four consecutive columns per thread
    for (int idx = threadIdx.x; idx < kPTH * (kPTW / 4); idx += 256) {
        const int y = idx / (kPTW / 4), cg = idx - y * (kPTW / 4);
        const int yo = R0 + y, xo = X0 + 4 * cg;
        if (yo >= p.H || xo >= p.W) continue;
        const float* u = &s_u1[(y >> 1) * (kPTW + 4) + 4 * cg];  // rows q-1, q, q+1
        const half_t* px = &s_px[(y + 4) * kPPitch + 4 * cg + 8];
        floatx4 rv;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const float a = u[v], b = u[(kPTW + 4) + v], cc = u[2 * (kPTW + 4) + v];
            const float up = (y & 1) ? 0.5f * (b + cc) : 0.125f * (a + cc) + 0.75f * b;
            rv[v] = (float)px[v] - up;
        }
        store4_mask(p.res + (int64_t)yo * p.res_pitch, xo, p.W, rv);
    }
}

static hb_status pyr_prepare(PyrArgs& a, const hb_half* in, float* res, hb_half* down,
                             int H, int W, int64_t in_pitch, int64_t res_pitch, int64_t down_pitch) {
    hb_status s = check_image(in, res, H, W, in_pitch, res_pitch);
    if (s != HB_OK) return s;
    if ((H & 1) || (W & 1)) return HB_ERR_INVALID_ARG;
    if (down && (down_pitch < W / 2 || !aligned_to(down, 2))) return HB_ERR_INVALID_ARG;
    if (down && down_pitch > ((int64_t)1 << 26)) return HB_ERR_UNSUPPORTED;
    a.in = reinterpret_cast<const half_t*>(in);
    a.res = res;
    a.down = reinterpret_cast<half_t*>(down);
    a.H = H;
    a.W = W;
    a.Hd = H / 2;
    a.Wd = W / 2;
    a.in_pitch = in_pitch;
    a.res_pitch = res_pitch;
    a.down_pitch = down_pitch;
    const int nct = ceil_div(W, 32 * HB_PYR_NS);
    const int rowsteps = ceil_div(H, 32);
    int steps = (int)(((int64_t)rowsteps * nct + HB_PYR_WAVES - 1) / HB_PYR_WAVES);
    steps = steps < 1 ? 1 : steps;
    a.steps = steps;
    a.grid.nct = nct;
    a.grid.nseg = ceil_div(rowsteps, steps);
    // interior task: its pixel windows start 18 before its first output and end 30 past its
    // last one, in both directions; then no up pass reads a clamped D index either
    interior_range(nct, 32 * HB_PYR_NS, 18, 32 * HB_PYR_NS + 30, W, a.grid.c0, a.grid.c1);
    interior_range(a.grid.nseg, 32 * steps, 18, 32 * steps + 30, H, a.grid.s0, a.grid.s1);
    if (a.grid.c1 <= a.grid.c0 || a.grid.s1 <= a.grid.s0) a.grid.c0 = a.grid.c1 = a.grid.s0 = a.grid.s1 = 0;
    return HB_OK;
}

}  // namespace hb

extern "C" hb_status hb_pyr_level_valu(const hb_half* in, float* residual, hb_half* down_or_null,
                                       int H, int W, int64_t in_pitch, int64_t res_pitch, int64_t down_pitch,
                                       hb_stream stream);

extern "C" hb_status hb_pyr_level(const hb_half* in, float* residual, hb_half* down_or_null,
                                  int H, int W, int64_t in_pitch, int64_t res_pitch, int64_t down_pitch,
                                  hb_stream stream) {
    using namespace hb;
    PyrArgs a;
    hb_status s = pyr_prepare(a, in, residual, down_or_null, H, W, in_pitch, res_pitch, down_pitch);
    if (s != HB_OK) return s;
    if (W < 48)   // narrower than one pixel window of the matrix formulation: vector-ALU kernel
        return hb_pyr_level_valu(in, residual, down_or_null, H, W, in_pitch, res_pitch, down_pitch, stream);
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const dim3 grid(min(ceil_div(a.grid.count(), 4), kMaxStreamBlocks));
    if ((int64_t)H * W * 4 <= kStreamStoreMaxBytes)
        hipLaunchKernelGGL((pyr_mfma_kernel<true>), grid, dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL((pyr_mfma_kernel<false>), grid, dim3(256), 0, st, a);
    return launch_status();
}

extern "C" hb_status hb_pyr_level_valu(const hb_half* in, float* residual, hb_half* down_or_null,
                                       int H, int W, int64_t in_pitch, int64_t res_pitch, int64_t down_pitch,
                                       hb_stream stream) {
    using namespace hb;
    PyrArgs a;
    hb_status s = pyr_prepare(a, in, residual, down_or_null, H, W, in_pitch, res_pitch, down_pitch);
    if (s != HB_OK) return s;
    const int64_t blocks = (int64_t)ceil_div(H, kPTH) * ceil_div(W, kPTW);
    if (blocks > 0x7fffffff) return HB_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(pyr_valu_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       reinterpret_cast<hipStream_t>(stream), a);
    return launch_status();
}
