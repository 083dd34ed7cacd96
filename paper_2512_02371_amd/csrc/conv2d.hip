// hb_conv2d: single-channel 2-D convolution with an arbitrary (non-separable) kernel, and its
// vector-ALU twin (Sec. V-A, 2-D form: O(x, y) = sum_{rx, ry} I(x + rx, y + ry) K(rx, ry)).
//
// MFMA formulation: the serial loop over the kernel rows r_y of Sec. V-A.  For every r_y the
// contribution is a row-wise FIR with taps K(., r_y) applied to the image shifted up by r_y rows,
// i.e. one Toeplitz product per tile exactly as in hb_fir1d (transposed: D'[m][n] += A[m][k] P[k][n],
// m = output column, n = image row in a 16-row group, k = pixel in the window), accumulated over
// r_y in the same accumulator.  The kh Toeplitz fragments per 32-pixel window chunk are built once
// per workgroup into LDS (one conflict-free 16-byte read per product); the image operand is read
// straight from memory, 16 image rows (clamped) shifted by r_y.
//
// The clamp along x is not folded into the fragments here (there would be kh folded pairs per
// border tile): strips that touch the left or right image border are computed by the vector-ALU
// kernel in a second launch on the same stream; the matrix kernel covers the interior strips.
#include "hb_device.hpp"
#include "hb_host.hpp"

namespace hb {

constexpr int kC2Tiles = 4;                   // 16-column tiles per wave strip
constexpr int kC2Threads = 512;               // 8 waves share one fragment table

struct Conv2dArgs {
    const half_t* in;
    float* out;
    int H, W;
    int64_t in_pitch, out_pitch;
    int kh, kw, ay, ax;
    // matrix kernel: interior strips [c0, c1) of 64 columns, 16-row groups, tasks = (c1 - c0) * rowgroups
    int c0, c1, rowgroups, ntasks;
    // vector-ALU kernel: computes the columns [0, xa) and [xb, W)
    int xa, xb;
    uint16_t taps[HB_MAX_TAPS_CONV2D * HB_MAX_TAPS_CONV2D];   // kh x kw, row-major
};

// ---------------------------------------------------------------------------
// Matrix-unit kernel.  NK = 32-pixel chunks of a tile's window (16 + kw - 1 pixels from x0 - ax on,
// one more when the window is moved to an even pixel).
template <int NK, bool STREAM>
__global__ void __launch_bounds__(kC2Threads) conv2d_mfma_kernel(Conv2dArgs p) {
    constexpr int NW = kC2Tiles;
    extern __shared__ __attribute__((aligned(16))) char s_dyn[];
    // [kh][NK][64 lanes] fragments, then one row patch per wave
    half8* s_frag = reinterpret_cast<half8*>(s_dyn);
    float* s_patch = reinterpret_cast<float*>(s_dyn + (size_t)p.kh * NK * 1024);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int e = p.ax & 1;
    const int aw = p.ax + e;                  // window start, left of the tile (even pixel)

    // Toeplitz fragments, A-operand layout: lane (c, g) holds A[c][32 kk + 8g + i] = K(32 kk + 8g + i - c - e, ry)
    for (int idx = tid; idx < p.kh * NK * 64; idx += kC2Threads) {
        const int l = idx & 63, kk = (idx >> 6) % NK, ry = idx / (64 * NK);
        const int t0 = 32 * kk + 8 * (l >> 4) - (l & 15) - e;
        half8 f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int t = t0 + i;
            f[i] = (t >= 0 && t < p.kw) ? __builtin_bit_cast(half_t, p.taps[ry * p.kw + t]) : (half_t)0;
        }
        s_frag[idx] = f;
    }
    __syncthreads();

    const int nstrips = p.c1 - p.c0;
    const int wave0 = blockIdx.x * (kC2Threads / 64) + wv;
    const int nwaves = gridDim.x * (kC2Threads / 64);
    float* patch = s_patch + wv * RowPatch<NW>::kFloats;
    const uint32_t rowbytes = (uint32_t)p.in_pitch * 2u;
    for (int task = wave0; task < p.ntasks; task += nwaves) {
        const int rg = task / nstrips, ct = p.c0 + (task - rg * nstrips);
        const int x0 = 16 * NW * ct, y0 = 16 * rg;
        const half_t* src = p.in + (x0 - aw);             // uniform; lanes add row * pitch + 8g
        floatx4 acc[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) acc[w] = floatx4{0.f, 0.f, 0.f, 0.f};

        auto load_rows = [&](int ry, half8 (&d)[NW][NK]) {
            // image rows y0 + c + ry - ay, clamped; past the last kernel row: the last one again
            const int yr = clampi(y0 + c + min(ry, p.kh - 1) - p.ay, 0, p.H - 1);
            const uint32_t off = (uint32_t)yr * rowbytes + 16u * g;
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) d[w][kk] = ldg8(src, off + 2u * (16u * w + 32u * kk));
        };
        auto products = [&](int ry, const half8 (&d)[NW][NK]) {
            half8 coef[NK];
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) coef[kk] = s_frag[(ry * NK + kk) * 64 + lane];
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) acc[w] = mfma16x16x32(coef[kk], d[w][kk], acc[w]);
        };
        // two window buffers used alternately; the next kernel row's windows are always requested
        half8 bufa[NW][NK], bufb[NW][NK];
        load_rows(0, bufa);
        for (int ry = 0; ry < p.kh; ry += 2) {
            load_rows(ry + 1, bufb);
            products(ry, bufa);
            if (ry + 1 >= p.kh) break;
            load_rows(ry + 2, bufa);
            products(ry + 1, bufb);
        }
        float* dst = p.out + x0;
        if (y0 + 16 <= p.H) {
            store_rows_via_lds<NW, STREAM>(patch, dst + (int64_t)y0 * p.out_pitch, (uint32_t)p.out_pitch, acc, lane);
        } else if (y0 + c < p.H) {
            const uint32_t off = ((uint32_t)(y0 + c) * (uint32_t)p.out_pitch + 4u * g) * 4u;
#pragma unroll
            for (int w = 0; w < NW; ++w) stg4<STREAM>(dst, off + 64u * w, acc[w]);
        }
    }
}

// ---------------------------------------------------------------------------
// Vector-ALU kernel: a 16 x 64 output tile per workgroup; the tile and its halo are staged in LDS
// with both indices clamped (the definition's border rule verbatim), every thread slides the kernel
// over 4 consecutive outputs with fp32 FMAs.  Tiles cover the column ranges [0, xa) and [xb, W).
constexpr int kC2vW = 64;
constexpr int kC2vRows = 16 + HB_MAX_TAPS_CONV2D - 1;                 // 47
constexpr int kC2vPitch = kC2vW + HB_MAX_TAPS_CONV2D - 1 + 1;          // 96 halves

__global__ void __launch_bounds__(256) conv2d_valu_kernel(Conv2dArgs p) {
    __shared__ half_t s_px[kC2vRows * kC2vPitch];
    __shared__ float s_k[HB_MAX_TAPS_CONV2D * HB_MAX_TAPS_CONV2D];
    for (int i = threadIdx.x; i < p.kh * p.kw; i += 256) s_k[i] = (float)__builtin_bit_cast(half_t, p.taps[i]);

    const int nl = (p.xa + kC2vW - 1) / kC2vW, nr = (p.W - p.xb + kC2vW - 1) / kC2vW;
    const int rg = blockIdx.x / (nl + nr), tc = blockIdx.x - rg * (nl + nr);
    const int x0 = tc < nl ? kC2vW * tc : p.xb + kC2vW * (tc - nl);
    const int xend = tc < nl ? min(x0 + kC2vW, p.xa) : min(x0 + kC2vW, p.W);
    const int y0 = 16 * rg;
    const int nrows = 16 + p.kh - 1, ncols = kC2vW + p.kw - 1;   // ncols <= 95
    {
        const int cc = threadIdx.x & 127;
        const int x = clampi(x0 + cc - p.ax, 0, p.W - 1);
        if (cc < ncols)
            for (int r = threadIdx.x >> 7; r < nrows; r += 2) {
                const int y = clampi(y0 + r - p.ay, 0, p.H - 1);
                s_px[r * kC2vPitch + cc] = p.in[(int64_t)y * p.in_pitch + x];
            }
    }
    __syncthreads();

    const int r = threadIdx.x >> 4, xl = 4 * (threadIdx.x & 15);
    const int y = y0 + r;
    if (y >= p.H || x0 + xl >= xend) return;
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int ry = 0; ry < p.kh; ++ry) {
        const half_t* src = &s_px[(r + ry) * kC2vPitch + xl];
        const float* k = &s_k[ry * p.kw];
        float v0 = (float)src[0], v1 = (float)src[1], v2 = (float)src[2];
        for (int t = 0; t < p.kw; ++t) {
            const float v3 = (float)src[t + 3], kv = k[t];
            acc[0] = fmaf(kv, v0, acc[0]);
            acc[1] = fmaf(kv, v1, acc[1]);
            acc[2] = fmaf(kv, v2, acc[2]);
            acc[3] = fmaf(kv, v3, acc[3]);
            v0 = v1;
            v1 = v2;
            v2 = v3;
        }
    }
    store4_mask(p.out + (int64_t)y * p.out_pitch, x0 + xl, xend, acc);
}

static hb_status conv2d_prepare(Conv2dArgs& a, const hb_half* in, float* out, int H, int W,
                                int64_t in_pitch, int64_t out_pitch,
                                const hb_half* taps_host, int kh, int kw, int ay, int ax) {
    hb_status s = check_image(in, out, H, W, in_pitch, out_pitch);
    if (s != HB_OK) return s;
    // lanes address rows with 32-bit byte offsets from the image base
    if ((int64_t)H * in_pitch >= ((int64_t)1 << 31) || (int64_t)H * out_pitch >= ((int64_t)1 << 30)) return HB_ERR_UNSUPPORTED;
    if (!taps_host) return HB_ERR_INVALID_ARG;
    if (kh < 1 || kh > HB_MAX_TAPS_CONV2D || kw < 1 || kw > HB_MAX_TAPS_CONV2D) return HB_ERR_INVALID_ARG;
    if (ay < 0 || ay >= kh || ax < 0 || ax >= kw) return HB_ERR_INVALID_ARG;
    a.in = reinterpret_cast<const half_t*>(in);
    a.out = out;
    a.H = H;
    a.W = W;
    a.in_pitch = in_pitch;
    a.out_pitch = out_pitch;
    a.kh = kh;
    a.kw = kw;
    a.ay = ay;
    a.ax = ax;
    memset(a.taps, 0, sizeof(a.taps));
    memcpy(a.taps, taps_host, sizeof(uint16_t) * (size_t)kh * (size_t)kw);
    a.rowgroups = ceil_div(H, 16);
    a.c0 = a.c1 = 0;
    a.ntasks = 0;
    a.xa = a.xb = W;                          // vector-ALU kernel: everything
    return HB_OK;
}

static hb_status conv2d_launch_valu(const Conv2dArgs& a, hipStream_t st) {
    const int64_t blocks = (int64_t)a.rowgroups * (ceil_div(a.xa, kC2vW) + ceil_div(a.W - a.xb, kC2vW));
    if (blocks > 0x7fffffff) return HB_ERR_UNSUPPORTED;
    if (blocks > 0) hipLaunchKernelGGL(conv2d_valu_kernel, dim3((unsigned)blocks), dim3(256), 0, st, a);
    return launch_status();
}

}  // namespace hb

extern "C" hb_status hb_conv2d(const hb_half* in, float* out, int H, int W,
                               int64_t in_pitch, int64_t out_pitch,
                               const hb_half* taps_host, int kh, int kw, int anchor_y, int anchor_x,
                               hb_stream stream) {
    using namespace hb;
    Conv2dArgs a;
    hb_status s = conv2d_prepare(a, in, out, H, W, in_pitch, out_pitch, taps_host, kh, kw, anchor_y, anchor_x);
    if (s != HB_OK) return s;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    // interior strips: the windows of all their tiles lie inside the row
    const int e = anchor_x & 1, aw = anchor_x + e;
    const int nk = ceil_div(15 + kw + e, 32);                // 1 or 2
    const int sw = 16 * kC2Tiles;
    const int c0 = ceil_div(aw, sw);
    const int last = W - (sw - 16) + aw - 32 * nk;           // x0 <= last keeps the last window inside
    int c1 = last >= 0 ? last / sw + 1 : 0;
    if (c1 > W / sw) c1 = W / sw;
    if (c1 > c0) {
        a.c0 = c0;
        a.c1 = c1;
        a.ntasks = (c1 - c0) * a.rowgroups;
        a.xa = sw * c0;
        a.xb = sw * c1;
        const size_t lds = (size_t)kh * nk * 1024 + (kC2Threads / 64) * RowPatch<kC2Tiles>::kFloats * sizeof(float);
        // fewer workgroups than tasks: every workgroup builds the fragment table once
        const int per_cu = lds <= 48 * 1024 ? 3 : lds <= 80 * 1024 ? 2 : 1;
        const int blocks = min(ceil_div(a.ntasks, kC2Threads / 64), kNumCU * per_cu);
        const bool ss = (int64_t)H * W * 4 <= kStreamStoreMaxBytes;
#define HB_C2_LAUNCH(N, S)                                                                            \
    {                                                                                                 \
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&conv2d_mfma_kernel<N, S>),             \
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)  \
            return HB_ERR_HIP;                                                                        \
        hipLaunchKernelGGL((conv2d_mfma_kernel<N, S>), dim3(blocks), dim3(kC2Threads), lds, st, a);   \
    }
        if (nk == 1) { if (ss) HB_C2_LAUNCH(1, true) else HB_C2_LAUNCH(1, false) }
        else { if (ss) HB_C2_LAUNCH(2, true) else HB_C2_LAUNCH(2, false) }
#undef HB_C2_LAUNCH
        s = launch_status();
        if (s != HB_OK) return s;
    }
    return conv2d_launch_valu(a, st);                         // border strips (everything if there is no interior)
}

extern "C" hb_status hb_conv2d_valu(const hb_half* in, float* out, int H, int W,
                                    int64_t in_pitch, int64_t out_pitch,
                                    const hb_half* taps_host, int kh, int kw, int anchor_y, int anchor_x,
                                    hb_stream stream) {
    using namespace hb;
    Conv2dArgs a;
    hb_status s = conv2d_prepare(a, in, out, H, W, in_pitch, out_pitch, taps_host, kh, kw, anchor_y, anchor_x);
    if (s != HB_OK) return s;
    a.xa = W;                                 // one range covers all columns
    a.xb = W;
    return conv2d_launch_valu(a, reinterpret_cast<hipStream_t>(stream));
}
