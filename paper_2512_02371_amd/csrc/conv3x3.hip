// hb_conv3x3: 64 -> 64 channel 3x3 convolution (stride 1, zero padding 1, NHWC) as an implicit
// GEMM on the matrix units (Sec. V-A 2-D form summed over channels; the conv layer of Sec. IV
// without bias and activation), and its vector-ALU twin.
//
// MFMA formulation, transposed so that a lane ends with consecutive output channels of one pixel:
//   O'[m][n] = sum_k Wt[m][k] * X[k][n]     m = output channel, n = pixel, k = (tap, input channel)
// with v_mfma_f32_32x32x16_f16: 32 channels x 32 pixels per product, K = 16 input channels.
//   A (coefficients): all 9 x 64 x 64 weights live in the registers of every wave for the whole
//     kernel: 2 channel tiles x 36 K-steps x 8 halves per lane.  They are gathered once per wave.
//   B (pixels): a workgroup stages an (8+2) x (32+2) pixel tile of all 64 input channels in LDS,
//     laid out [row][16-channel chunk][pixel][16 channels], so that the 32 pixels x 16 channels of
//     one K-step are 1 KB of contiguous LDS for every tap shift (the overlapped view of Eq. 1: the
//     three horizontal taps read the same LDS row at pixel offsets 0, 1, 2) and every 16-byte lane
//     read is bank-conflict free.  Pixels outside the image are written as zeros, which is the
//     zero padding.
//   Each of the 4 waves owns 2 of the 8 output rows: 2 x 2 x 36 products per tile.  fp32
//   accumulators are rounded to fp16 (RNE) and leave as 8-byte stores of 4 consecutive channels.
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

__device__ __forceinline__ int cv_lds_index(int r, int kc, int px) { return ((r * 4 + kc) * kCvPx + px) * 16; }

__global__ void __launch_bounds__(256) conv3x3_mfma_kernel(ConvArgs p) {
    __shared__ __attribute__((aligned(16))) half_t s_in[kCvLdsHalves];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    const int c32 = lane & 31, h = lane >> 5;

    // coefficient fragments: wf[j][s] lane (c32, h) = w[tap][16 kc + 8h + i][32 j + c32], s = 4 tap + kc
    half8 wf[2][36];
#pragma unroll
    for (int s = 0; s < 36; ++s)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int i = 0; i < 8; ++i)
                wf[j][s][i] = p.w[((s >> 2) * kCvC + 16 * (s & 3) + 8 * h + i) * kCvC + 32 * j + c32];

    for (int tile = blockIdx.x; tile < p.ntiles; tile += gridDim.x) {
        const int n = tile / (p.tiles_x * p.tiles_y);
        const int rem = tile - n * (p.tiles_x * p.tiles_y);
        const int ty = rem / p.tiles_x, tx = rem - ty * p.tiles_x;
        const int y0 = ty * kCvTY, x0 = tx * kCvTX;
        const half_t* img = p.in + (int64_t)n * p.H * p.W * kCvC;

        __syncthreads();                                  // previous tile fully consumed
        // stage rows y0-1 .. y0+8, pixels x0-1 .. x0+32, all channels; 16-byte pieces
        for (int idx = tid; idx < kCvRows * kCvPx * 8; idx += 256) {
            const int piece = idx & 7;                    // 8 channels each
            const int pr = idx >> 3;
            const int r = pr / kCvPx, px = pr - r * kCvPx;
            const int y = y0 - 1 + r, x = x0 - 1 + px;
            half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (y >= 0 && y < p.H && x >= 0 && x < p.W)
                v = *reinterpret_cast<const half8*>(img + ((int64_t)y * p.W + x) * kCvC + 8 * piece);
            *reinterpret_cast<half8*>(&s_in[cv_lds_index(r, piece >> 1, px) + 8 * (piece & 1)]) = v;
        }
        __syncthreads();

#pragma unroll 1
        for (int rr = 0; rr < 2; ++rr) {
            const int ro = 2 * wv + rr;                   // output row inside the tile
            floatx16 acc[2];
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
#pragma unroll
            for (int s = 0; s < 36; ++s) {
                const int tap = s >> 2, kc = s & 3;
                const int ky = tap / 3, kx = tap - 3 * ky;
                const half8 b = *reinterpret_cast<const half8*>(&s_in[cv_lds_index(ro + ky, kc, c32 + kx) + 8 * h]);
                acc[0] = mfma32x32x16(wf[0][s], b, acc[0]);
                acc[1] = mfma32x32x16(wf[1][s], b, acc[1]);
            }
            const int y = y0 + ro, x = x0 + c32;
            if (y < p.H && x < p.W) {
                half_t* o = p.out + (((int64_t)n * p.H + y) * p.W + x) * kCvC;
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        half4 v4;
#pragma unroll
                        for (int r = 0; r < 4; ++r) v4[r] = (half_t)acc[j][4 * q + r];
                        *reinterpret_cast<half4*>(o + 32 * j + 8 * q + 4 * h) = v4;
                    }
            }
        }
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
        *reinterpret_cast<half8*>(&s_in[cv_lds_index(r, piece >> 1, px) + 8 * (piece & 1)]) = v;
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
            const half_t* px = &s_in[cv_lds_index(ro + ky, kc, xi + kx)];
            const half8 a = *reinterpret_cast<const half8*>(px), b = *reinterpret_cast<const half8*>(px + 8);
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
    hipLaunchKernelGGL(conv3x3_mfma_kernel, dim3(blocks), dim3(256), 0, reinterpret_cast<hipStream_t>(stream), a);
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
