// hb_fir1d: row-wise FIR as a product with a Toeplitz matrix held in registers
// (Sec. V-A: O(x..x+k-1) = I(x..x+k+l-1) * A_K, A_K(x, y) = K(y - x)), and its
// vector-ALU twin.
//
// MFMA formulation.  The paper lifts the vector-matrix product to a matrix-matrix
// product by stacking overlapped segments of ONE row (Eq. 1).  An image already
// has the second dimension: 16 image rows are the 16 independent vectors, so the
// image operand is read straight from memory in its natural layout (each lane: 8
// consecutive pixels of one row, one 16-byte load) and no overlapped view has to
// be staged.  We compute the transposed tile
//     D'[m][n] = sum_k A[m][k] * P[k][n],   m = output column in a 16-wide tile,
//                                            n = image row in a 16-row group,
//                                            k = pixel inside an aligned 32-pixel block,
// with A[m][k] = taps[32*delta + k - (16*par + m) + anchor] (zero outside the taps),
// one A fragment per (half-block par, neighbouring block delta), built once per
// wave.  In D' a lane owns four consecutive output columns of one row, so the
// result leaves with one 16-byte store per lane.
#include "hb_device.hpp"
#include "hb_host.hpp"

namespace hb {

struct FirArgs {
    const half_t* in;
    float* out;
    int H, W;
    int64_t in_pitch, out_pitch;
    int T, anchor;
    int dmin;            // first neighbouring block (relative) that a 32-column output block reads
    int nct;             // 64-column tiles per row
    int ntasks;          // (16-row groups) x nct
    int vec_in, vec_out; // layouts allow 16-byte accesses
    Taps taps;
};

__device__ __forceinline__ half_t tap_from_bits(uint16_t b) {
    return __builtin_bit_cast(half_t, b);
}

template <int ND>
__global__ void __launch_bounds__(256) fir1d_mfma_kernel(FirArgs p) {
    __shared__ half_t s_taps[HB_MAX_TAPS];
    if (threadIdx.x < HB_MAX_TAPS) s_taps[threadIdx.x] = tap_from_bits(p.taps.v[threadIdx.x]);
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int c = lane & 15, g = lane >> 4;

    // Toeplitz fragments, A-operand layout: lane (c, g) holds A[c][8g .. 8g+7].
    half8 coef[2][ND];
#pragma unroll
    for (int par = 0; par < 2; ++par)
#pragma unroll
        for (int d = 0; d < ND; ++d)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                int t = 32 * (p.dmin + d) + 8 * g + i - (16 * par + c) + p.anchor;
                coef[par][d][i] = (t >= 0 && t < p.T) ? s_taps[t] : (half_t)0;
            }

    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int nwaves = (gridDim.x * blockDim.x) >> 6;
    for (int task = wave; task < p.ntasks; task += nwaves) {
        const int rg = task / p.nct, ct = task - rg * p.nct;
        const int y = 16 * rg + c;
        const half_t* row = p.in + (int64_t)min(y, p.H - 1) * p.in_pitch;
        const int x0 = 64 * ct;

        half8 blk[ND + 1];
#pragma unroll
        for (int j = 0; j <= ND; ++j)
            blk[j] = load8_clamp(row, x0 + 32 * (p.dmin + j) + 8 * g, p.W, p.vec_in);

        float* orow = p.out + (int64_t)y * p.out_pitch;
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int par = 0; par < 2; ++par) {
                floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int d = 0; d < ND; ++d) acc = mfma16x16x32(coef[par][d], blk[tb + d], acc);
                const int xo = x0 + 32 * tb + 16 * par + 4 * g;
                if (y < p.H && xo < p.W) store4_mask(orow, xo, p.W, acc, p.vec_out);
            }
    }
}

// Vector-ALU twin: a 16 x 256 tile is staged in LDS with its halo, every thread
// slides the taps over 4 x 4 outputs with fp32 FMAs.
constexpr int kValuTileW = 256;
constexpr int kValuMaxChunks = (kValuTileW + 64 + 64) / 8;   // tile + left slack + right halo
constexpr int kValuPitch = kValuMaxChunks * 8 + 8;

__global__ void __launch_bounds__(256) fir1d_valu_kernel(FirArgs p) {
    __shared__ half_t s_px[16 * kValuPitch];
    __shared__ float s_k[HB_MAX_TAPS];
    if (threadIdx.x < HB_MAX_TAPS) s_k[threadIdx.x] = (float)tap_from_bits(p.taps.v[threadIdx.x]);

    const int nctv = (p.W + kValuTileW - 1) / kValuTileW;
    const int rg = blockIdx.x / nctv, ct = blockIdx.x - rg * nctv;
    const int x0 = ct * kValuTileW;
    const int lead = 8 * ((p.anchor + 7) / 8);                 // aligned slack left of the tile
    const int nch = (kValuTileW + lead + (p.T - 1 - p.anchor) + 7) / 8;
    for (int idx = threadIdx.x; idx < 16 * nch; idx += 256) {
        const int r = idx / nch, ch = idx - r * nch;
        const half_t* row = p.in + (int64_t)min(16 * rg + r, p.H - 1) * p.in_pitch;
        half8 v = load8_clamp(row, x0 - lead + 8 * ch, p.W, p.vec_in);
        *reinterpret_cast<half8*>(&s_px[r * kValuPitch + 8 * ch]) = v;
    }
    __syncthreads();

    const int r = threadIdx.x >> 4, cg = threadIdx.x & 15;
    const int y = 16 * rg + r;
    if (y >= p.H) return;
    float* orow = p.out + (int64_t)y * p.out_pitch;
    const int off = lead - p.anchor;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int xl = 4 * cg + 64 * j;
        if (x0 + xl >= p.W) continue;
        const half_t* src = &s_px[r * kValuPitch + xl + off];
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int u = 0; u < p.T + 3; ++u) {
            const float v = (float)src[u];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int t = u - q;
                if (t >= 0 && t < p.T) acc[q] = fmaf(s_k[t], v, acc[q]);
            }
        }
        store4_mask(orow, x0 + xl, p.W, acc, p.vec_out);
    }
}

static hb_status fir1d_prepare(FirArgs& a, const hb_half* in, float* out, int H, int W,
                               int64_t in_pitch, int64_t out_pitch,
                               const hb_half* taps_host, int ntaps, int anchor) {
    hb_status s = check_image(in, out, H, W, in_pitch, out_pitch);
    if (s != HB_OK) return s;
    s = check_taps(taps_host, ntaps, anchor);
    if (s != HB_OK) return s;
    a.in = reinterpret_cast<const half_t*>(in);
    a.out = out;
    a.H = H;
    a.W = W;
    a.in_pitch = in_pitch;
    a.out_pitch = out_pitch;
    a.T = ntaps;
    a.anchor = anchor;
    a.dmin = floor_div(-anchor, 32);
    a.nct = ceil_div(W, 64);
    a.ntasks = ceil_div(H, 16) * a.nct;
    a.vec_in = aligned_to(in, 16) && (in_pitch % 8 == 0);
    a.vec_out = aligned_to(out, 16) && (out_pitch % 4 == 0);
    a.taps = pack_taps(taps_host, ntaps);
    return HB_OK;
}

}  // namespace hb

extern "C" hb_status hb_fir1d(const hb_half* in, float* out, int H, int W,
                              int64_t in_pitch, int64_t out_pitch,
                              const hb_half* taps_host, int ntaps, int anchor, hb_stream stream) {
    using namespace hb;
    FirArgs a;
    hb_status s = fir1d_prepare(a, in, out, H, W, in_pitch, out_pitch, taps_host, ntaps, anchor);
    if (s != HB_OK) return s;
    // blocks dmin .. dmax (relative) hold the pixels a 32-column output block reads
    const int dmax = floor_div(31 - anchor + ntaps - 1, 32);
    const int nd = dmax - a.dmin + 1;
    const int blocks = min(ceil_div(a.ntasks, 4), kMaxStreamBlocks);
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    switch (nd) {
        case 1: hipLaunchKernelGGL(fir1d_mfma_kernel<1>, dim3(blocks), dim3(256), 0, st, a); break;
        case 2: hipLaunchKernelGGL(fir1d_mfma_kernel<2>, dim3(blocks), dim3(256), 0, st, a); break;
        case 3: hipLaunchKernelGGL(fir1d_mfma_kernel<3>, dim3(blocks), dim3(256), 0, st, a); break;
        case 4: hipLaunchKernelGGL(fir1d_mfma_kernel<4>, dim3(blocks), dim3(256), 0, st, a); break;
        default: return HB_ERR_UNSUPPORTED;
    }
    return launch_status();
}

extern "C" hb_status hb_fir1d_valu(const hb_half* in, float* out, int H, int W,
                                   int64_t in_pitch, int64_t out_pitch,
                                   const hb_half* taps_host, int ntaps, int anchor, hb_stream stream) {
    using namespace hb;
    FirArgs a;
    hb_status s = fir1d_prepare(a, in, out, H, W, in_pitch, out_pitch, taps_host, ntaps, anchor);
    if (s != HB_OK) return s;
    const int64_t blocks = (int64_t)ceil_div(H, 16) * ceil_div(W, kValuTileW);
    if (blocks > 0x7fffffff) return HB_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(fir1d_valu_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       reinterpret_cast<hipStream_t>(stream), a);
    return launch_status();
}
