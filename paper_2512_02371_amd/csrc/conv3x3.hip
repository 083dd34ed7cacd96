// hb_conv3x3: 64 -> 64 channel 3x3 convolution (stride 1, zero padding 1, NHWC) as an implicit
// GEMM on the matrix units (Sec. V-A 2-D form summed over channels; the conv layer of Sec. IV
// without bias and activation), and its vector-ALU twin.
//
// MFMA formulation, transposed so that a lane ends with consecutive output channels of one pixel:
//   O'[m][n] = sum_k Wt[m][k] * X[k][n]     m = output channel, n = pixel, k = (tap, input channel)
// with v_mfma_f32_32x32x16_f16: 32 channels x 32 pixels per product, K = 16 input channels.
//   A (coefficients): the 9 x 64 x 32 weights of one 32-channel tile live in the registers of a
//     wave for the whole kernel (36 K-steps x 8 halves per lane = 144 registers), gathered once.
//   B (pixels): a workgroup stages an (8+2) x (32+2) pixel tile of all 64 input channels in LDS,
//     laid out [row][16-channel chunk][8-channel half][pixel][8 channels], so that the pixels of
//     one K-step are two runs of 512 contiguous bytes for every tap shift (the overlapped view of
//     Eq. 1: the three horizontal taps read the same LDS row at pixel offsets 0, 1, 2) and every
//     16-byte lane read is bank-conflict free.  Pixels outside the image are written as zeros,
//     which is the zero padding.
//   A workgroup has 8 waves, two per SIMD, so that one wave's LDS reads hide behind the other's
//   products: wave (q, j) owns output rows 2q, 2q+1 of the tile and channel tile j, i.e. 2 x 36
//   products per tile.  fp32 accumulators are rounded to fp16 (RNE) and leave as 8-byte stores of 4
//   consecutive channels.  The tile buffer is double: the next tile's pixels are fetched into
//   registers before a wave starts multiplying and written to the other buffer afterwards.
// Workgroups are persistent (one per compute unit) and walk over the tiles.
#include "hb_device.hpp"
#include "hb_host.hpp"

namespace hb {

constexpr int kCvC = 64;                 // channels in and out
constexpr int kCvTY = 8, kCvTX = 32;     // output tile (rows x pixels) per workgroup step
constexpr int kCvRows = kCvTY + 2, kCvPx = kCvTX + 2;
constexpr int kCvLdsHalves = kCvRows * 4 * kCvPx * 16;

struct ConvArgs {
    const half_t* in;
    const half_t* w;
    half_t* out;
    int N, H, W;
    int tiles_x, tiles_y;      // per image
    int ntiles;                // N * tiles_y * tiles_x
};

// LDS layout [row][16-channel chunk][8-channel half][pixel][8 channels]: the lanes of one half-wave
// (same half, consecutive pixels) read 512 contiguous bytes for any tap shift.
__device__ __forceinline__ int cv_lds_index(int r, int kc, int half, int px) {
    return (((r * 4 + kc) * 2 + half) * kCvPx + px) * 8;
}

// 16-byte pieces of one staged tile, spread over the 512 threads in two batches so that a wave
// has the next tile's pixels in flight while it multiplies the current one.
constexpr int kCvThreads = 512;
constexpr int kCvPieces = kCvRows * kCvPx * 8;                               // 2720
constexpr int kCvIters = (kCvPieces + kCvThreads - 1) / kCvThreads;          // 6
constexpr int kCvBatchA = 3, kCvBatchB = kCvIters - kCvBatchA;               // 3 + 3

struct CvTile {
    int n, y0, x0;
};
__device__ __forceinline__ CvTile cv_tile(const ConvArgs& p, int tile) {
    CvTile t;
    t.n = tile / (p.tiles_x * p.tiles_y);
    const int rem = tile - t.n * (p.tiles_x * p.tiles_y);
    const int ty = rem / p.tiles_x;
    t.y0 = ty * kCvTY;
    t.x0 = (rem - ty * p.tiles_x) * kCvTX;
    return t;
}
// piece idx of a tile = (staged row r, staged pixel px, 8-channel piece)
__device__ __forceinline__ void cv_piece(int idx, int& r, int& px, int& piece) {
    idx = min(idx, kCvPieces - 1);                        // the tail repeats the last piece (same data)
    piece = idx & 7;
    const int pr = idx >> 3;
    r = pr / kCvPx;
    px = pr - r * kCvPx;
}
// border tiles: pixels (y0-1+r, x0-1+px), zeros outside the image
__device__ __forceinline__ half8 cv_fetch(const ConvArgs& p, const CvTile& t, int idx) {
    int r, px, piece;
    cv_piece(idx, r, px, piece);
    half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
    const int y = t.y0 - 1 + r, x = t.x0 - 1 + px;
    if (y >= 0 && y < p.H && x >= 0 && x < p.W)
        v = *reinterpret_cast<const half8*>(p.in + (((int64_t)t.n * p.H + y) * p.W + x) * kCvC + 8 * piece);
    return v;
}
// interior tiles: byte offset of the piece from the tile's first staged pixel (the same for every tile)
__device__ __forceinline__ uint32_t cv_goff(const ConvArgs& p, int idx) {
    int r, px, piece;
    cv_piece(idx, r, px, piece);
    return (uint32_t)(((r * p.W + px) * kCvC + 8 * piece) * 2);
}
__device__ __forceinline__ void cv_put(half_t* buf, int idx, half8 v) {
    int r, px, piece;
    cv_piece(idx, r, px, piece);
    *reinterpret_cast<half8*>(&buf[cv_lds_index(r, piece >> 1, piece & 1, px)]) = v;
}
// whole staged tile inside the image?
__device__ __forceinline__ bool cv_interior(const ConvArgs& p, const CvTile& t) {
    return t.y0 >= 1 && t.y0 + kCvTY + 1 <= p.H && t.x0 >= 1 && t.x0 + kCvTX + 1 <= p.W;
}
__device__ __forceinline__ const half_t* cv_origin(const ConvArgs& p, const CvTile& t) {
    return p.in + (((int64_t)t.n * p.H + (t.y0 - 1)) * p.W + (t.x0 - 1)) * kCvC;
}

// Two output rows (2 x 32 pixels) x 32 channels from the staged tile: K-steps S0 .. S1-1 of 36, two
// products each.
template <int S0, int S1>
__device__ __forceinline__ void cv_rows(const half_t* buf, const half8 (&wf)[36], int ro, int c32, int h,
                                        floatx16 (&acc)[2]) {
    const half_t* base = buf + cv_lds_index(ro, 0, h, c32);
#pragma unroll
    for (int s = S0; s < S1; ++s) {
        const int tap = s >> 2, kc = s & 3, ky = tap / 3, kx = tap - 3 * ky;
        const half_t* q = base + cv_lds_index(ky, kc, 0, kx);
        const half8 b0 = *reinterpret_cast<const half8*>(q);
        const half8 b1 = *reinterpret_cast<const half8*>(q + cv_lds_index(1, 0, 0, 0));   // next tile row
        acc[0] = mfma32x32x16(wf[s], b0, acc[0]);
        acc[1] = mfma32x32x16(wf[s], b1, acc[1]);
    }
}

__device__ __forceinline__ void cv_store_row(const ConvArgs& p, const CvTile& t, int ro, int j, int c32, int h,
                                             const floatx16& acc) {
    const int y = t.y0 + ro, x = t.x0 + c32;
    if (y < p.H && x < p.W) {
        half_t* o = p.out + (((int64_t)t.n * p.H + y) * p.W + x) * kCvC + 32 * j;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            half4 v4;
#pragma unroll
            for (int r = 0; r < 4; ++r) v4[r] = (half_t)acc[4 * q + r];
            *reinterpret_cast<half4*>(o + 8 * q + 4 * h) = v4;
        }
    }
}

__global__ void __launch_bounds__(kCvThreads) conv3x3_mfma_kernel(ConvArgs p) {
    extern __shared__ __attribute__((aligned(16))) half_t s_dyn[];   // two tile buffers
    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    const int c32 = lane & 31, h = lane >> 5;
    const int j = wv >> 2;                                // channel tile of this wave
    const int ro = 2 * (wv & 3);                          // its two output rows inside the tile

    int tile = blockIdx.x;
    if (tile >= p.ntiles) return;

    // coefficient fragments: wf[s] lane (c32, h) = w[tap][16 kc + 8h + i][32 j + c32], s = 4 tap + kc.
    // The 72 KB of weights pass through LDS once (coalesced 16-byte copies in, 2-byte gathers out:
    // lanes of a half-wave read 32 consecutive halves, no bank conflict).
    half8 wf[36];
    for (int i = tid; i < 9 * kCvC * kCvC / 8; i += kCvThreads)
        reinterpret_cast<half8*>(s_dyn)[i] = reinterpret_cast<const half8*>(p.w)[i];
    __syncthreads();
#pragma unroll
    for (int s = 0; s < 36; ++s)
#pragma unroll
        for (int i = 0; i < 8; ++i)
            wf[s][i] = s_dyn[((s >> 2) * kCvC + 16 * (s & 3) + 8 * h + i) * kCvC + 32 * j + c32];
    __syncthreads();

    {
        const CvTile t = cv_tile(p, tile);
        for (int it = 0; it < kCvIters; ++it)
            cv_put(s_dyn, tid + kCvThreads * it, cv_fetch(p, t, tid + kCvThreads * it));
    }
    __syncthreads();

    int cur = 0;
    for (; tile < p.ntiles; tile += gridDim.x) {
        const CvTile t = cv_tile(p, tile);
        const int next = tile + gridDim.x;
        const bool more = next < p.ntiles;                // uniform
        CvTile tn = t;
        if (more) tn = cv_tile(p, next);
        const half_t* buf = s_dyn + cur * kCvLdsHalves;
        half_t* nbuf = s_dyn + (cur ^ 1) * kCvLdsHalves;

        half8 g[kCvBatchA];
        floatx16 acc[2];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[u][v] = 0.f;
        const bool fast = more && cv_interior(p, tn);     // uniform
        const half_t* org = cv_origin(p, tn);
        if (fast) {
#pragma unroll
            for (int it = 0; it < kCvBatchA; ++it) g[it] = ldg8(org, cv_goff(p, tid + kCvThreads * it));
        } else if (more) {
#pragma unroll
            for (int it = 0; it < kCvBatchA; ++it) g[it] = cv_fetch(p, tn, tid + kCvThreads * it);
        }
        cv_rows<0, 18>(buf, wf, ro, c32, h, acc);
        if (more) {
#pragma unroll
            for (int it = 0; it < kCvBatchA; ++it) cv_put(nbuf, tid + kCvThreads * it, g[it]);
        }
        if (fast) {
#pragma unroll
            for (int it = 0; it < kCvBatchB; ++it)
                g[it] = ldg8(org, cv_goff(p, tid + kCvThreads * (kCvBatchA + it)));
        } else if (more) {
#pragma unroll
            for (int it = 0; it < kCvBatchB; ++it) g[it] = cv_fetch(p, tn, tid + kCvThreads * (kCvBatchA + it));
        }
        cv_rows<18, 36>(buf, wf, ro, c32, h, acc);
        if (more) {                                       // before the output stores: waits on the fetches only
#pragma unroll
            for (int it = 0; it < kCvBatchB; ++it) cv_put(nbuf, tid + kCvThreads * (kCvBatchA + it), g[it]);
        }
        cv_store_row(p, t, ro, j, c32, h, acc[0]);
        cv_store_row(p, t, ro + 1, j, c32, h, acc[1]);
        __syncthreads();                                  // next buffer complete, current one released
        cur ^= 1;
    }
}

// ---------------------------------------------------------------------------
// Vector-ALU twin: one thread per output pixel and 32 output channels, fp32 FMAs; pixels from the
// same LDS tile, weights through uniform (scalar) loads.
__global__ void __launch_bounds__(512) conv3x3_valu_kernel(ConvArgs p) {
    __shared__ __attribute__((aligned(16))) half_t s_in[kCvLdsHalves];
    const int tid = threadIdx.x;
    const int tile = blockIdx.x;
    const int n = tile / (p.tiles_x * p.tiles_y);
    const int rem = tile - n * (p.tiles_x * p.tiles_y);
    const int ty = rem / p.tiles_x, tx = rem - ty * p.tiles_x;
    const int y0 = ty * kCvTY, x0 = tx * kCvTX;
    const half_t* img = p.in + (int64_t)n * p.H * p.W * kCvC;
    for (int idx = tid; idx < kCvRows * kCvPx * 8; idx += 512) {
        const int piece = idx & 7;
        const int pr = idx >> 3;
        const int r = pr / kCvPx, px = pr - r * kCvPx;
        const int y = y0 - 1 + r, x = x0 - 1 + px;
        half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
        if (y >= 0 && y < p.H && x >= 0 && x < p.W)
            v = *reinterpret_cast<const half8*>(img + ((int64_t)y * p.W + x) * kCvC + 8 * piece);
        *reinterpret_cast<half8*>(&s_in[cv_lds_index(r, piece >> 1, piece & 1, px)]) = v;
    }
    __syncthreads();
    const int cohalf = __builtin_amdgcn_readfirstlane(tid >> 8);   // waves 0-3: channels 0..31, waves 4-7: 32..63
    const int pid = tid & 255;
    const int ro = pid >> 5, xi = pid & 31;
    float acc[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = 0.f;
    for (int tap = 0; tap < 9; ++tap) {
        const int ky = tap / 3, kx = tap - 3 * ky;
        for (int kc = 0; kc < 4; ++kc) {
            const half8 a = *reinterpret_cast<const half8*>(&s_in[cv_lds_index(ro + ky, kc, 0, xi + kx)]);
            const half8 b = *reinterpret_cast<const half8*>(&s_in[cv_lds_index(ro + ky, kc, 1, xi + kx)]);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float xv = (float)(i < 8 ? a[i] : b[i - 8]);
                const half_t* wrow = p.w + ((tap * kCvC) + 16 * kc + i) * kCvC + 32 * cohalf;   // uniform
#pragma unroll
                for (int co = 0; co < 32; ++co) acc[co] = fmaf(xv, (float)wrow[co], acc[co]);
            }
        }
    }
    const int y = y0 + ro, x = x0 + xi;
    if (y < p.H && x < p.W) {
        half_t* o = p.out + (((int64_t)n * p.H + y) * p.W + x) * kCvC + 32 * cohalf;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            half8 v8;
#pragma unroll
            for (int r = 0; r < 8; ++r) v8[r] = (half_t)acc[8 * q + r];
            *reinterpret_cast<half8*>(o + 8 * q) = v8;
        }
    }
}

static hb_status conv_prepare(ConvArgs& a, const hb_half* in, const hb_half* w, hb_half* out,
                              int N, int H, int W, int Cin, int Cout) {
    if (!in || !w || !out) return HB_ERR_INVALID_ARG;
    if (N < 1 || H < 1 || W < 1 || Cin < 1 || Cout < 1) return HB_ERR_INVALID_ARG;
    if (!aligned_to(in, 16) || !aligned_to(w, 16) || !aligned_to(out, 16)) return HB_ERR_INVALID_ARG;
    if (Cin != kCvC || Cout != kCvC) return HB_ERR_UNSUPPORTED;
    const int64_t tiles = (int64_t)N * ceil_div(H, kCvTY) * ceil_div(W, kCvTX);
    if (tiles > 0x7fffffff || (int64_t)N * H * W > ((int64_t)1 << 40)) return HB_ERR_UNSUPPORTED;
    a.in = reinterpret_cast<const half_t*>(in);
    a.w = reinterpret_cast<const half_t*>(w);
    a.out = reinterpret_cast<half_t*>(out);
    a.N = N;
    a.H = H;
    a.W = W;
    a.tiles_x = ceil_div(W, kCvTX);
    a.tiles_y = ceil_div(H, kCvTY);
    a.ntiles = (int)tiles;
    return HB_OK;
}

}  // namespace hb

extern "C" hb_status hb_conv3x3(const hb_half* in_nhwc, const hb_half* w_hwio, hb_half* out_nhwc,
                                int N, int H, int W, int Cin, int Cout, hb_stream stream) {
    using namespace hb;
    ConvArgs a;
    hb_status s = conv_prepare(a, in_nhwc, w_hwio, out_nhwc, N, H, W, Cin, Cout);
    if (s != HB_OK) return s;
    const int blocks = min(a.ntiles, kNumCU);
    const size_t lds = 2 * kCvLdsHalves * sizeof(half_t);      // 85 KB of the 160 KB per compute unit
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&conv3x3_mfma_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return HB_ERR_HIP;
    hipLaunchKernelGGL(conv3x3_mfma_kernel, dim3(blocks), dim3(kCvThreads), lds,
                       reinterpret_cast<hipStream_t>(stream), a);
    return launch_status();
}

extern "C" hb_status hb_conv3x3_valu(const hb_half* in_nhwc, const hb_half* w_hwio, hb_half* out_nhwc,
                                     int N, int H, int W, int Cin, int Cout, hb_stream stream) {
    using namespace hb;
    ConvArgs a;
    hb_status s = conv_prepare(a, in_nhwc, w_hwio, out_nhwc, N, H, W, Cin, Cout);
    if (s != HB_OK) return s;
    hipLaunchKernelGGL(conv3x3_valu_kernel, dim3(a.ntiles), dim3(512), 0, reinterpret_cast<hipStream_t>(stream), a);
    return launch_status();
}
