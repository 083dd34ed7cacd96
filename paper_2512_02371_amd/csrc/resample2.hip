// hb_down2 / hb_up2: resampling by a factor of two with an arbitrary 2-D kernel, and their
// vector-ALU twins (Sec. V-B).
//
// Downsampling is a strided convolution, O(x, y) = sum I(2x + rx, 2y + ry) K(rx, ry).  Along x it
// is a product with the strided Toeplitz matrix A^down_K(x, y) = K(y - 2x): a tile of 16 outputs
// reads a window of 30 + kw pixels (two K = 32 products).  Along y the kernel rows split by the
// parity of the input row they read: rows ry with ry - anchor_y = 2t + par read input row
// 2(y + t) + par.  Each parity is a walk over "half rows" exactly like hb_conv2d's (16 input rows
// of one parity fixed in registers, product tile of shift b = t - t_min added into two open output
// groups with lane-shifted additions), and the two parities with the same shift share one
// addition because the matrix unit accumulates their products first.
//
// Upsampling is the multiphase filter O(2x + dx, 2y + dy) = sum I(x + rx, y + ry) K(2rx + dx, 2ry + dy).
// Along x the two column phases interleave inside one coefficient matrix (row 2i + dx of the
// matrix holds K(2(k - i) + dx, .)), so a tile of 16 outputs comes from a window of 8 + kw/2 - 1
// input pixels and is stored as it is.  Along y each row phase dy is one walk with kh/2 kernel rows
// into its own pair of open groups; its 16 rows are every second output row.
#include "hb_device.hpp"
#include "hb_host.hpp"
#include "walk2d.hpp"

namespace hb {

struct Rs2Args {
    const half_t* in;
    float* out;
    int H, W;                                 // input
    int Ho, Wo;                               // output
    int64_t in_pitch, out_pitch;
    int kh, kw, ay, ax;
    // matrix kernels: nstrips strips of 64 output columns; a task = one strip x seg_len groups of
    // 16 output rows (down) / 16 input rows = 32 output rows (up); ngroups = groups of the image
    int nstrips, ngroups, seg_len, nseg, ntasks;
    // down: first half-row offset t_min and number of kernel rows of each input-row parity
    int tmin[2], nrows[2];
    uint16_t taps[HB_MAX_TAPS_CONV2D * HB_MAX_TAPS_CONV2D];   // kh x kw, row-major
};

__device__ __forceinline__ half_t rs2_tap(const Rs2Args& p, int ry, int rx) {
    return (ry >= 0 && ry < p.kh && rx >= 0 && rx < p.kw) ? __builtin_bit_cast(half_t, p.taps[ry * p.kw + rx]) : (half_t)0;
}

// Eight pixels of one image row from column xs on, column clamped; 32-bit byte offsets from the image base.
__device__ __forceinline__ half8 rs2_load8_clamped(const half_t* base, uint32_t rowoff, int xs, int W) {
    half8 r;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int x = clampi(xs + i, 0, W - 1);
        r[i] = *reinterpret_cast<const half_t*>(reinterpret_cast<const char*>(base) + (rowoff + 2u * (uint32_t)x));
    }
    return r;
}

// ---------------------------------------------------------------------------
// Downsampling on the matrix units.
template <bool STREAM>
__global__ void __launch_bounds__(kC2Threads) down2_mfma_kernel(Rs2Args p) {
    constexpr int NW = kC2Tiles, NK = 2;
    extern __shared__ __attribute__((aligned(16))) char s_dyn[];
    // [32 rows: parity 0 shifts 0..15, parity 1 shifts 0..15][NK][64 lanes] fragments, then one row patch per wave
    half8* s_frag = reinterpret_cast<half8*>(s_dyn);
    float* s_patch = reinterpret_cast<float*>(s_dyn + (size_t)32 * NK * 1024);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int e = p.ax & 1;
    const int aw = p.ax + e;                  // window start, left of the tile's first input pixel (even pixel)

    // Strided Toeplitz fragments, A-operand layout: lane (m, g) holds A[m][32 kk + 8g + i] = K(32 kk + 8g + i - 2m - e, ry)
    for (int idx = tid; idx < 32 * NK * 64; idx += kC2Threads) {
        const int l = idx & 63, kk = (idx >> 6) % NK, row = idx / (64 * NK);
        const int par = row >> 4, b = row & 15;
        const int ry = b < p.nrows[par] ? 2 * (b + p.tmin[par]) + par + p.ay : -1;
        const int t0 = 32 * kk + 8 * (l >> 4) - 2 * (l & 15) - e;
        half8 f;
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = rs2_tap(p, ry, t0 + i);
        s_frag[idx] = f;
    }
    __syncthreads();

    // every XCD takes one contiguous run of the tasks: neighbouring strips and row segments share their
    // halo pixels in one L2 (measured reads 1.36x / 1.2x the input instead of 2.2x / 1.6x, same time)
    const int task = xcd_contiguous(blockIdx.x, gridDim.x) * (kC2Threads / 64) + wv;
    if (task >= p.ntasks) return;
    const int sg = task / p.nstrips, ct = task - sg * p.nstrips;
    const int x0 = 16 * NW * ct;              // first output column of the strip
    const int q0 = sg * p.seg_len, q1 = min(q0 + p.seg_len, p.ngroups);
    float* patch = s_patch + wv * RowPatch<NW>::kFloats;
    const uint32_t rowbytes = (uint32_t)p.in_pitch * 2u;
    // windows of the strip: input pixels 2 x0 - aw .. 2 x0 - aw + 159
    const int xs0 = 2 * x0 - aw;
    const bool inside = xs0 >= 0 && xs0 + 32 * (NW - 1) + 32 * NK <= p.W;
    const bool whole = x0 + 16 * NW <= p.Wo;
    const half_t* src = p.in + xs0;           // uniform; only used by strips inside the row
    float* dst = p.out + x0;

    auto load_group = [&](int G, half8 (&d)[2][NW][NK]) {
#pragma unroll
        for (int par = 0; par < 2; ++par) {
            // input rows 2 (16 G + c + t_min) + par, clamped into the image
            const int yr = clampi(2 * (16 * G + c + p.tmin[par]) + par, 0, p.H - 1);
            const uint32_t rowoff = (uint32_t)yr * rowbytes;
            // window kk of tile w starts at pixel 32 (w + kk): NW + NK - 1 different windows, each loaded once
            half8 win[NW + NK - 1];
            if (inside) {
#pragma unroll
                for (int u = 0; u < NW + NK - 1; ++u) win[u] = ldg8(src, rowoff + 16u * g + 2u * (32u * u));
            } else {
#pragma unroll
                for (int u = 0; u < NW + NK - 1; ++u) win[u] = rs2_load8_clamped(p.in, rowoff, xs0 + 8 * g + 32 * u, p.W);
            }
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) d[par][w][kk] = win[w + kk];
        }
    };
    auto store_group = [&](int Q, const floatx4 (&acc)[NW]) {
        const int y0 = 16 * Q;
        if (whole && y0 + 16 <= p.Ho) {
            store_rows_via_lds<NW, STREAM>(patch, dst + (int64_t)y0 * p.out_pitch, (uint32_t)p.out_pitch, acc, lane);
        } else if (y0 + c < p.Ho) {
            float* row = p.out + (int64_t)(y0 + c) * p.out_pitch;
#pragma unroll
            for (int w = 0; w < NW; ++w) store4_mask(row, x0 + 16 * w + 4 * g, p.Wo, acc[w]);
        }
    };

    floatx4 ring[2][NW], done[NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        ring[0][w] = floatx4{0.f, 0.f, 0.f, 0.f};
        ring[1][w] = floatx4{0.f, 0.f, 0.f, 0.f};
        done[w] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
    half8 cur[2][NW][NK], nxt[2][NW][NK];
    load_group(q0, cur);
    const int nmax = max(p.nrows[0], p.nrows[1]);
    // output group Q takes its rows n >= b parts in step Q and its rows n < b parts in step Q + 1
#pragma unroll 1
    for (int G = q0; G <= q1; ++G) {
        // stores ahead of the loads: one counter serves both, see hb_conv2d
        if (G - 2 >= q0) store_group(G - 2, done);
        load_group(G + 1, nxt);               // clamped rows: always inside the image
        int fl = lane;                        // keeps the fragment reads inside the loop
        asm volatile("" : "+v"(fl));
        c2_step<NK, true>(s_frag, fl, nmax, p.nrows[1], cur[0], cur[1], ring);
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            done[w] = ring[0][w];
            ring[0][w] = ring[1][w];
            ring[1][w] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) {
                cur[0][w][kk] = nxt[0][w][kk];
                cur[1][w][kk] = nxt[1][w][kk];
            }
        }
    }
    if (q1 > q0) store_group(q1 - 1, done);
}

// ---------------------------------------------------------------------------
// Upsampling on the matrix units.
template <bool STREAM>
__global__ void __launch_bounds__(kC2Threads) up2_mfma_kernel(Rs2Args p) {
    constexpr int NW = kC2Tiles, NK = 1;
    extern __shared__ __attribute__((aligned(16))) char s_dyn[];
    // [dy][16 kernel rows][64 lanes] fragments, then one row patch per wave
    half8* s_frag = reinterpret_cast<half8*>(s_dyn);
    float* s_patch = reinterpret_cast<float*>(s_dyn + (size_t)2 * 16 * 1024);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int e = p.ax & 1;
    const int aw = p.ax + e;

    // Two-phase fragments, A-operand layout: lane (m = 2i + dx, g) holds
    // A[m][8g + ii] = K(2 (8g + ii - i - e) + dx, 2 ry + dy)
    for (int idx = tid; idx < 2 * 16 * 64; idx += kC2Threads) {
        const int l = idx & 63, ry = (idx >> 6) & 15, dy = idx >> 10;
        const int m = l & 15, i = m >> 1, dx = m & 1;
        const int r0 = 8 * (l >> 4) - i - e;
        half8 f;
#pragma unroll
        for (int ii = 0; ii < 8; ++ii) {
            const int rx = r0 + ii;
            f[ii] = (2 * ry + dy < p.kh && rx >= 0) ? rs2_tap(p, 2 * ry + dy, 2 * rx + dx) : (half_t)0;
        }
        s_frag[idx] = f;
    }
    __syncthreads();

    // every XCD takes one contiguous run of the tasks: neighbouring strips and row segments share their
    // halo pixels in one L2 (measured reads 1.36x / 1.2x the input instead of 2.2x / 1.6x, same time)
    const int task = xcd_contiguous(blockIdx.x, gridDim.x) * (kC2Threads / 64) + wv;
    if (task >= p.ntasks) return;
    const int sg = task / p.nstrips, ct = task - sg * p.nstrips;
    const int x0 = 16 * NW * ct;              // first output column of the strip
    const int xi0 = x0 / 2 - aw;              // first input pixel of its windows
    const int q0 = sg * p.seg_len, q1 = min(q0 + p.seg_len, p.ngroups);
    float* patch = s_patch + wv * RowPatch<NW>::kFloats;
    const uint32_t rowbytes = (uint32_t)p.in_pitch * 2u;
    const bool inside = xi0 >= 0 && xi0 + 8 * (NW - 1) + 32 <= p.W;
    const bool whole = x0 + 16 * NW <= p.Wo;
    const half_t* src = p.in + xi0;
    float* dst = p.out + x0;

    auto load_group = [&](int G, half8 (&d)[NW][NK]) {
        const int yr = clampi(16 * G - p.ay + c, 0, p.H - 1);
        const uint32_t rowoff = (uint32_t)yr * rowbytes;
        if (inside) {
#pragma unroll
            for (int w = 0; w < NW; ++w) d[w][0] = ldg8(src, rowoff + 16u * g + 2u * (8u * w));
        } else {
#pragma unroll
            for (int w = 0; w < NW; ++w) d[w][0] = rs2_load8_clamped(p.in, rowoff, xi0 + 8 * g + 8 * w, p.W);
        }
    };
    // group Q of row phase dy: output rows 2 (16 Q + n) + dy
    auto store_group = [&](int Q, int dy, const floatx4 (&acc)[NW]) {
        const int y0 = 16 * Q;
        if (whole && y0 + 16 <= p.H) {
            store_rows_via_lds<NW, STREAM>(patch, dst + (int64_t)(2 * y0 + dy) * p.out_pitch, 2u * (uint32_t)p.out_pitch, acc, lane);
        } else if (y0 + c < p.H) {
            float* row = p.out + (int64_t)(2 * (y0 + c) + dy) * p.out_pitch;
#pragma unroll
            for (int w = 0; w < NW; ++w) store4_mask(row, x0 + 16 * w + 4 * g, p.Wo, acc[w]);
        }
    };

    floatx4 ring[2][2][NW], done[2][NW];
#pragma unroll
    for (int dy = 0; dy < 2; ++dy)
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            ring[dy][0][w] = floatx4{0.f, 0.f, 0.f, 0.f};
            ring[dy][1][w] = floatx4{0.f, 0.f, 0.f, 0.f};
            done[dy][w] = floatx4{0.f, 0.f, 0.f, 0.f};
        }
    half8 cur[NW][NK], nxt[NW][NK], far[NW][NK];
    load_group(q0, cur);
    load_group(q0 + 1, nxt);
    const int nr = p.kh / 2;
#pragma unroll 1
    for (int G = q0; G <= q1; ++G) {
        if (G - 2 >= q0) {
            store_group(G - 2, 0, done[0]);
            store_group(G - 2, 1, done[1]);
        }
        load_group(G + 2, far);               // clamped rows: always inside the image
        int fl = lane;
        asm volatile("" : "+v"(fl));
        c2_step<NK, false>(s_frag, fl, nr, 0, cur, cur, ring[0]);
        c2_step<NK, false>(s_frag + 16 * 64, fl, nr, 0, cur, cur, ring[1]);
#pragma unroll
        for (int dy = 0; dy < 2; ++dy)
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                done[dy][w] = ring[dy][0][w];
                ring[dy][0][w] = ring[dy][1][w];
                ring[dy][1][w] = floatx4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            cur[w][0] = nxt[w][0];
            nxt[w][0] = far[w][0];
        }
    }
    if (q1 > q0) {
        store_group(q1 - 1, 0, done[0]);
        store_group(q1 - 1, 1, done[1]);
    }
}

// ---------------------------------------------------------------------------
// Vector-ALU kernels.  The input pixels an output tile needs are staged in LDS as fp32 with both
// indices clamped (the definition's border rule verbatim).  A thread owns 8 consecutive outputs of
// one row: for every kernel row it reads the pixels under them once (16-byte LDS reads) and slides
// the taps over them in registers, 8 FMAs per tap read.  KWP = kernel width rounded up to 8, 16 or
// 32; the taps beyond kw are zeros, and so are the staged columns only they can reach.
constexpr int kRsTaps = HB_MAX_TAPS_CONV2D;
constexpr int kRsDownRows = 2 * 15 + kRsTaps;                          // 62
constexpr int kRsDownPitch = 2 * 64 + kRsTaps;                         // 160 floats
constexpr int kRsUpRows = 8 + kRsTaps / 2 - 1;                         // 23
constexpr int kRsUpPitch = 64 + kRsTaps / 2;                           // 80 floats

template <int KWP>
__device__ __forceinline__ void rs2_stage_taps(const Rs2Args& p, float* s_k, int nthreads) {
    for (int i = threadIdx.x; i < p.kh * KWP; i += nthreads) {
        const int ry = i / KWP, t = i - ry * KWP;
        s_k[i] = t < p.kw ? (float)__builtin_bit_cast(half_t, p.taps[ry * p.kw + t]) : 0.f;
    }
}

// 16 x 64 outputs per workgroup of 128 threads
template <int KWP>
__global__ void __launch_bounds__(128) down2_valu_kernel(Rs2Args p) {
    __shared__ __attribute__((aligned(16))) float s_px[kRsDownRows * kRsDownPitch];
    __shared__ float s_k[kRsTaps * KWP];
    rs2_stage_taps<KWP>(p, s_k, 128);
    const int nt = (p.Wo + 63) / 64;
    const int rg = blockIdx.x / nt, tc = blockIdx.x - rg * nt;
    const int x0 = 64 * tc, y0 = 16 * rg;
    const int nrows = 30 + p.kh;
    for (int idx = threadIdx.x; idx < nrows * kRsDownPitch; idx += 128) {
        const int r = idx / kRsDownPitch, cc = idx - r * kRsDownPitch;
        float v = 0.f;
        if (cc < 126 + p.kw) {
            const int y = clampi(2 * y0 + r - p.ay, 0, p.H - 1), x = clampi(2 * x0 + cc - p.ax, 0, p.W - 1);
            v = (float)p.in[(int64_t)y * p.in_pitch + x];
        }
        s_px[idx] = v;
    }
    __syncthreads();
    const int r = threadIdx.x >> 3, xl = 8 * (threadIdx.x & 7);
    const int y = y0 + r;
    if (y >= p.Ho || x0 + xl >= p.Wo) return;
    float acc[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] = 0.f;
    for (int ry = 0; ry < p.kh; ++ry) {
        float w[KWP + 16];                                 // inputs 2 xl .. 2 xl + KWP + 15 of row 2 r + ry
        const floatx4* src = reinterpret_cast<const floatx4*>(&s_px[(2 * r + ry) * kRsDownPitch + 2 * xl]);
#pragma unroll
        for (int i = 0; i < (KWP + 16) / 4; ++i) {
            const floatx4 v = src[i];
            w[4 * i] = v[0];
            w[4 * i + 1] = v[1];
            w[4 * i + 2] = v[2];
            w[4 * i + 3] = v[3];
        }
        const float* k = &s_k[ry * KWP];
#pragma unroll
        for (int t = 0; t < KWP; ++t) {
            const float kv = k[t];
#pragma unroll
            for (int q = 0; q < 8; ++q) acc[q] = fmaf(kv, w[2 * q + t], acc[q]);
        }
    }
    float* row = p.out + (int64_t)y * p.out_pitch;
    store4_mask(row, x0 + xl, p.Wo, floatx4{acc[0], acc[1], acc[2], acc[3]});
    store4_mask(row, x0 + xl + 4, p.Wo, floatx4{acc[4], acc[5], acc[6], acc[7]});
}

// 16 x 128 outputs per workgroup of 256 threads = 8 x 64 input positions plus halo
template <int KWP>
__global__ void __launch_bounds__(256) up2_valu_kernel(Rs2Args p) {
    constexpr int RXP = KWP / 2;
    __shared__ __attribute__((aligned(16))) float s_px[kRsUpRows * kRsUpPitch];
    __shared__ float s_k[kRsTaps * KWP];
    rs2_stage_taps<KWP>(p, s_k, 256);
    const int nt = (p.Wo + 127) / 128;
    const int rg = blockIdx.x / nt, tc = blockIdx.x - rg * nt;
    const int x0 = 128 * tc, y0 = 16 * rg;    // output tile; input tile starts at (y0 / 2, x0 / 2)
    const int nrows = 8 + p.kh / 2 - 1;
    for (int idx = threadIdx.x; idx < nrows * kRsUpPitch; idx += 256) {
        const int r = idx / kRsUpPitch, cc = idx - r * kRsUpPitch;
        float v = 0.f;
        if (cc < 64 + p.kw / 2 - 1) {
            const int y = clampi(y0 / 2 + r - p.ay, 0, p.H - 1), x = clampi(x0 / 2 + cc - p.ax, 0, p.W - 1);
            v = (float)p.in[(int64_t)y * p.in_pitch + x];
        }
        s_px[idx] = v;
    }
    __syncthreads();
    const int r = threadIdx.x >> 4, xl = 8 * (threadIdx.x & 15);
    const int y = y0 + r;
    if (y >= p.Ho || x0 + xl >= p.Wo) return;
    const int dy = y & 1;
    float acc[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] = 0.f;
    for (int ry = 0; ry < p.kh / 2; ++ry) {
        float w[RXP + 4];                                  // inputs xl / 2 .. xl / 2 + RXP + 3 of row r / 2 + ry
        const floatx4* src = reinterpret_cast<const floatx4*>(&s_px[(r / 2 + ry) * kRsUpPitch + xl / 2]);
#pragma unroll
        for (int i = 0; i < (RXP + 4) / 4; ++i) {
            const floatx4 v = src[i];
            w[4 * i] = v[0];
            w[4 * i + 1] = v[1];
            w[4 * i + 2] = v[2];
            w[4 * i + 3] = v[3];
        }
        const float* k = &s_k[(2 * ry + dy) * KWP];
#pragma unroll
        for (int rx = 0; rx < RXP; ++rx) {
            const float k0 = k[2 * rx], k1 = k[2 * rx + 1];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc[2 * i] = fmaf(k0, w[i + rx], acc[2 * i]);
                acc[2 * i + 1] = fmaf(k1, w[i + rx], acc[2 * i + 1]);
            }
        }
    }
    float* row = p.out + (int64_t)y * p.out_pitch;
    store4_mask(row, x0 + xl, p.Wo, floatx4{acc[0], acc[1], acc[2], acc[3]});
    store4_mask(row, x0 + xl + 4, p.Wo, floatx4{acc[4], acc[5], acc[6], acc[7]});
}

// ---------------------------------------------------------------------------
static int floor_half(int s) { return s >= 0 ? s / 2 : -((-s + 1) / 2); }

static hb_status rs2_prepare(Rs2Args& a, bool up, const hb_half* in, float* out, int H, int W,
                             int64_t in_pitch, int64_t out_pitch,
                             const hb_half* taps_host, int kh, int kw, int ay, int ax) {
    if (H <= 0 || W <= 0 || H > (1 << 29) || W > (1 << 29)) return HB_ERR_INVALID_ARG;
    const int Ho = up ? 2 * H : (H + 1) / 2, Wo = up ? 2 * W : (W + 1) / 2;
    // check_image wants one shape for both sides: validate each side against its own width
    hb_status s = check_image(in, out, H, W, in_pitch, in_pitch);
    if (s != HB_OK) return s;
    s = check_image(in, out, Ho, Wo, Wo, out_pitch);
    if (s != HB_OK) return s;
    // lanes address rows with 32-bit byte offsets from the image base
    if ((int64_t)H * in_pitch >= ((int64_t)1 << 31) || (int64_t)Ho * out_pitch >= ((int64_t)1 << 30)) return HB_ERR_UNSUPPORTED;
    if (!taps_host) return HB_ERR_INVALID_ARG;
    if (kh < 1 || kh > HB_MAX_TAPS_CONV2D || kw < 1 || kw > HB_MAX_TAPS_CONV2D) return HB_ERR_INVALID_ARG;
    if (up) {
        if ((kh & 1) || (kw & 1)) return HB_ERR_INVALID_ARG;
        if (ay < 0 || ay >= kh / 2 || ax < 0 || ax >= kw / 2) return HB_ERR_INVALID_ARG;
    } else {
        if (ay < 0 || ay >= kh || ax < 0 || ax >= kw) return HB_ERR_INVALID_ARG;
    }
    a.in = reinterpret_cast<const half_t*>(in);
    a.out = out;
    a.H = H;
    a.W = W;
    a.Ho = Ho;
    a.Wo = Wo;
    a.in_pitch = in_pitch;
    a.out_pitch = out_pitch;
    a.kh = kh;
    a.kw = kw;
    a.ay = ay;
    a.ax = ax;
    memset(a.taps, 0, sizeof(a.taps));
    memcpy(a.taps, taps_host, sizeof(uint16_t) * (size_t)kh * (size_t)kw);
    for (int par = 0; par < 2; ++par) {
        // kernel rows ry with ry - ay = 2 t + par: the first one and how many
        int s0 = -ay;
        if (((s0 % 2) + 2) % 2 != par) ++s0;
        a.tmin[par] = floor_half(s0);
        const int last = kh - 1 - ay;         // largest ry - ay
        a.nrows[par] = s0 <= last ? (last - s0) / 2 + 1 : 0;
    }
    a.nstrips = ceil_div(Wo, 16 * kC2Tiles);
    a.ngroups = up ? ceil_div(H, 16) : ceil_div(Ho, 16);
    // one task per wave: a strip times a run of groups, as long as filling the chip allows
    const int waves = num_cu() * (kC2Threads / 64);
    int len = (int)(((int64_t)a.nstrips * a.ngroups + waves - 1) / waves);
    if (len < 2) len = a.ngroups < 2 ? a.ngroups : 2;
    a.seg_len = len;
    a.nseg = ceil_div(a.ngroups, len);
    const int64_t ntasks = (int64_t)a.nstrips * a.nseg;
    if (ntasks > 0x7fffffff / 2) return HB_ERR_UNSUPPORTED;
    a.ntasks = (int)ntasks;
    return HB_OK;
}

template <class K>
static hb_status rs2_launch_mfma(K kernel, const Rs2Args& a, size_t table_bytes, hipStream_t st) {
    const size_t lds = table_bytes + (kC2Threads / 64) * RowPatch<kC2Tiles>::kFloats * sizeof(float);
    if (allow_dynamic_lds(reinterpret_cast<const void*>(kernel), lds) != HB_OK) return HB_ERR_HIP;
    hipLaunchKernelGGL(kernel, dim3(ceil_div(a.ntasks, kC2Threads / 64)), dim3(kC2Threads), lds, st, a);
    return launch_status();
}

template <class K>
static hb_status rs2_launch_valu(K kernel, const Rs2Args& a, int tile_w, int threads, hipStream_t st) {
    const int64_t blocks = (int64_t)ceil_div(a.Ho, 16) * ceil_div(a.Wo, tile_w);
    if (blocks > 0x7fffffff) return HB_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(threads), 0, st, a);
    return launch_status();
}

}  // namespace hb

extern "C" hb_status hb_down2(const hb_half* in, float* out, int H, int W, int64_t in_pitch, int64_t out_pitch,
                              const hb_half* taps_host, int kh, int kw, int anchor_y, int anchor_x, hb_stream stream) {
    using namespace hb;
    Rs2Args a;
    hb_status s = rs2_prepare(a, false, in, out, H, W, in_pitch, out_pitch, taps_host, kh, kw, anchor_y, anchor_x);
    if (s != HB_OK) return s;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if ((int64_t)a.Ho * a.Wo * 4 <= kStreamStoreMaxBytes) return rs2_launch_mfma(down2_mfma_kernel<true>, a, 32 * 2 * 1024, st);
    return rs2_launch_mfma(down2_mfma_kernel<false>, a, 32 * 2 * 1024, st);
}

extern "C" hb_status hb_down2_valu(const hb_half* in, float* out, int H, int W, int64_t in_pitch, int64_t out_pitch,
                                   const hb_half* taps_host, int kh, int kw, int anchor_y, int anchor_x, hb_stream stream) {
    using namespace hb;
    Rs2Args a;
    hb_status s = rs2_prepare(a, false, in, out, H, W, in_pitch, out_pitch, taps_host, kh, kw, anchor_y, anchor_x);
    if (s != HB_OK) return s;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (kw <= 8) return rs2_launch_valu(down2_valu_kernel<8>, a, 64, 128, st);
    if (kw <= 16) return rs2_launch_valu(down2_valu_kernel<16>, a, 64, 128, st);
    return rs2_launch_valu(down2_valu_kernel<32>, a, 64, 128, st);
}

extern "C" hb_status hb_up2(const hb_half* in, float* out, int H, int W, int64_t in_pitch, int64_t out_pitch,
                            const hb_half* taps_host, int kh, int kw, int anchor_y, int anchor_x, hb_stream stream) {
    using namespace hb;
    Rs2Args a;
    hb_status s = rs2_prepare(a, true, in, out, H, W, in_pitch, out_pitch, taps_host, kh, kw, anchor_y, anchor_x);
    if (s != HB_OK) return s;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if ((int64_t)a.Ho * a.Wo * 4 <= kStreamStoreMaxBytes) return rs2_launch_mfma(up2_mfma_kernel<true>, a, 2 * 16 * 1024, st);
    return rs2_launch_mfma(up2_mfma_kernel<false>, a, 2 * 16 * 1024, st);
}

extern "C" hb_status hb_up2_valu(const hb_half* in, float* out, int H, int W, int64_t in_pitch, int64_t out_pitch,
                                 const hb_half* taps_host, int kh, int kw, int anchor_y, int anchor_x, hb_stream stream) {
    using namespace hb;
    Rs2Args a;
    hb_status s = rs2_prepare(a, true, in, out, H, W, in_pitch, out_pitch, taps_host, kh, kw, anchor_y, anchor_x);
    if (s != HB_OK) return s;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (kw <= 8) return rs2_launch_valu(up2_valu_kernel<8>, a, 128, 256, st);
    if (kw <= 16) return rs2_launch_valu(up2_valu_kernel<16>, a, 128, 256, st);
    return rs2_launch_valu(up2_valu_kernel<32>, a, 128, 256, st);
}
