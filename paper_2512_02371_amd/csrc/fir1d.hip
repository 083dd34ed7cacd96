// hb_fir1d: row-wise FIR as a product with a Toeplitz matrix held in registers
// (Sec. V-A: O(x..x+k-1) = I(x..x+k+l-1) * A_K, A_K(x, y) = K(y - x)), and its
// vector-ALU twin.
//
// MFMA formulation.  The paper lifts the vector-matrix product to a matrix-matrix
// product by stacking overlapped segments of ONE row (Eq. 1).  An image already
// has the second dimension: 16 image rows are the 16 independent vectors, so the
// image operand is read straight from memory in its natural layout (each lane: 8
// consecutive pixels of one row, one 16-byte load at any pixel offset) and no
// overlapped view has to be staged.  For a 16-column output tile starting at x0 the
// window is the 32*NK pixels from x0 - anchor - e on (e = anchor & 1 keeps the window
// on an even pixel, i.e. dword aligned: 16-byte loads at odd pixel offsets run at a
// fraction of the rate), and we compute the transposed tile
//     D'[m][n] = sum_k A[m][k] * P[k][n],   m = output column in the tile,
//                                            n = image row in a 16-row group,
//                                            k = pixel in the window,
// with A[m][k] = taps[k - m - e] (zero outside the taps): A_K itself, built once per
// wave from a zero-padded tap table.  In D' a lane owns four consecutive output
// columns of one row, so the result leaves with one 16-byte store per lane.
#include "hb_device.hpp"
#include "hb_host.hpp"

#ifndef HB_FIR_TILES
#define HB_FIR_TILES 4        // 16-column tiles per wave strip (fewer for long filters, see fir_tiles)
#endif
#ifndef HB_FIR_WAVES
#define HB_FIR_WAVES (1 << 20) // wave tasks per launch before a task takes more than one 16-row step;
                              // rows are independent here, so short-lived waves stream best
#endif

#ifndef HB_FIR_LONG_WAVES
#define HB_FIR_LONG_WAVES 4096 // the same for filters of more than 80 taps (four or more windows per tile)
#endif

namespace hb {

struct FirArgs {
    const half_t* in;
    float* out;
    int H, W;
    int64_t in_pitch, out_pitch;
    int T, anchor;
    int nct;             // strips per row group
    int steps;           // 16-row steps per task
    int ntasks;          // strips x row segments
    TapsT<HB_MAX_TAPS_FIR1D> taps;
    FoldTablesT<HB_MAX_TAPS_FIR1D> fold;
};

// Tiles per wave strip: a strip keeps 2 x tiles x NK window fragments in registers.
constexpr int fir_tiles(int nk) { return nk <= 3 ? HB_FIR_TILES : nk <= 6 ? 2 : 1; }

__device__ __forceinline__ half_t tap_from_bits(uint16_t b) {
    return __builtin_bit_cast(half_t, b);
}

// A wave owns a strip of HB_FIR_TILES tiles and walks down it in steps of 16 rows; the pixels of
// the next step are requested before the current step is multiplied.
template <int NK, bool STREAM>
__global__ void __launch_bounds__(256) fir1d_mfma_kernel(FirArgs p) {
    constexpr int NW = fir_tiles(NK);
    __shared__ __attribute__((aligned(16))) float s_patch[4][RowPatch<NW>::kFloats];

    const int lane = threadIdx.x & 63;
    const int c = lane & 15, g = lane >> 4;

    // Toeplitz fragments, A-operand layout: lane (c, g) holds A[c][32kk + 8g + i] = taps[32kk + 8g + i - c - e].
    const int e = p.anchor & 1;
    const int aw = p.anchor + e;              // window start, left of the tile
    half8 coef[NK];
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) coef[kk] = tap_run(p.taps.tab, 32 * kk + 8 * g - c - e);
    const int wmax = p.W - 32 * NK;           // last window start that stays inside the row

    const int wgpos = xcd_contiguous(blockIdx.x, gridDim.x);
    const int wave = __builtin_amdgcn_readfirstlane(wgpos * 4 + (threadIdx.x >> 6));
    const int nwaves = (gridDim.x * blockDim.x) >> 6;
    for (int task = wave; task < p.ntasks; task += nwaves) {
        const int seg = task / p.nct, ct = task - seg * p.nct;
        const int x0 = 16 * NW * ct;
        const int Y0 = seg * p.steps * 16;
        const int nsteps = min(p.steps, (p.H - Y0 + 15) / 16);
        const bool xin = (x0 - aw >= 0) && (x0 + 16 * (NW - 1) - aw + 32 * NK <= p.W) && (x0 + 16 * NW <= p.W);
        if (xin) {
            // strip inside the row: uniform bases, 32-bit lane offsets, coalesced row stores
            const half_t* src = p.in + (x0 - aw);
            float* dst = p.out + x0;
            half8 cur[NW][NK], nxt[NW][NK];
            auto load_step = [&](int q, half8 (&d)[NW][NK]) {
                const int yr = min(Y0 + 16 * q + c, p.H - 1);
                const uint32_t off = ((uint32_t)yr * (uint32_t)p.in_pitch + 8u * g) * 2u;
#pragma unroll
                for (int w = 0; w < NW; ++w)
#pragma unroll
                    for (int kk = 0; kk < NK; ++kk) d[w][kk] = ldg8(src, off + 2u * (16u * w + 32u * kk));
            };
            load_step(0, cur);
            for (int q = 0; q < nsteps; ++q) {
                if (q + 1 < nsteps) load_step(q + 1, nxt);
                floatx4 acc[NW];
#pragma unroll
                for (int w = 0; w < NW; ++w) {
                    acc[w] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kk = 0; kk < NK; ++kk) acc[w] = mfma16x16x32(coef[kk], cur[w][kk], acc[w]);
                }
                const int y0 = Y0 + 16 * q;
                if (y0 + 16 <= p.H) {
                    store_rows_via_lds<NW, STREAM>(s_patch[threadIdx.x >> 6], dst + (int64_t)y0 * p.out_pitch,
                                                   (uint32_t)p.out_pitch, acc, lane);
                } else if (y0 + c < p.H) {
                    const uint32_t off = ((uint32_t)(y0 + c) * (uint32_t)p.out_pitch + 4u * g) * 4u;
#pragma unroll
                    for (int w = 0; w < NW; ++w) stg4<STREAM>(dst, off + 64u * w, acc[w]);
                }
#pragma unroll
                for (int w = 0; w < NW; ++w)
#pragma unroll
                    for (int kk = 0; kk < NK; ++kk) cur[w][kk] = nxt[w][kk];
            }
        } else {
            // border strip, tile by tile: the window is moved inside the row and the clamp is
            // folded into the fragment; rows past the image repeat the last one
#pragma unroll 1
            for (int w = 0; w < NW; ++w) {
                const int xt = x0 + 16 * w;
                if (xt >= p.W) break;
                const int ws = clampi(xt - aw, 0, wmax);
                const bool plain = (ws == xt - aw) && (xt + 16 <= p.W);
                half8 hi[NK], lo[NK];
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) {
                    if (plain) {
                        hi[kk] = coef[kk];
                        lo[kk] = half8{0, 0, 0, 0, 0, 0, 0, 0};
                    } else {
                        folded_fragment(p.fold, p.T, p.anchor, p.W, xt, ws, kk, c, g, hi[kk], lo[kk]);
                    }
                }
                for (int q = 0; q < nsteps; ++q) {
                    const int y = Y0 + 16 * q + c;
                    const half_t* row = p.in + (int64_t)min(y, p.H - 1) * p.in_pitch;
                    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kk = 0; kk < NK; ++kk) {
                        const half8 px = *reinterpret_cast<const half8_u*>(row + ws + 32 * kk + 8 * g);
                        acc = mfma16x16x32(hi[kk], px, acc);
                        acc = mfma16x16x32(lo[kk], px, acc);
                    }
                    if (y < p.H) store4_mask(p.out + (int64_t)y * p.out_pitch, xt + 4 * g, p.W, acc);
                }
            }
        }
    }
}

// Vector-ALU twin: a 16 x 256 tile is staged in LDS with its halo, every thread
// slides the taps over 4 x 4 outputs with fp32 FMAs.
constexpr int kValuTileW = 256;
constexpr int kValuMaxChunks = (kValuTileW + HB_MAX_TAPS_FIR1D + HB_MAX_TAPS_FIR1D) / 8;   // tile + left slack + right halo
constexpr int kValuPitch = kValuMaxChunks * 8 + 8;

__global__ void __launch_bounds__(256) fir1d_valu_kernel(FirArgs p) {
    __shared__ half_t s_px[16 * kValuPitch];
    __shared__ float s_k[HB_MAX_TAPS_FIR1D];
    static_assert(HB_MAX_TAPS_FIR1D <= 256, "one tap per thread");
    if (threadIdx.x < HB_MAX_TAPS_FIR1D) s_k[threadIdx.x] = (float)tap_at(p.taps.tab, threadIdx.x);

    const int nctv = (p.W + kValuTileW - 1) / kValuTileW;
    const int rg = blockIdx.x / nctv, ct = blockIdx.x - rg * nctv;
    const int x0 = ct * kValuTileW;
    const int lead = 8 * ((p.anchor + 7) / 8);                 // aligned slack left of the tile
    const int nch = (kValuTileW + lead + (p.T - 1 - p.anchor) + 7) / 8;
    for (int idx = threadIdx.x; idx < 16 * nch; idx += 256) {
        const int r = idx / nch, ch = idx - r * nch;
        const half_t* row = p.in + (int64_t)min(16 * rg + r, p.H - 1) * p.in_pitch;
        half8 v = load8_clamp(row, x0 - lead + 8 * ch, p.W);
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
        store4_mask(orow, x0 + xl, p.W, acc);
    }
}

static hb_status fir1d_prepare(FirArgs& a, const hb_half* in, float* out, int H, int W,
                               int64_t in_pitch, int64_t out_pitch,
                               const hb_half* taps_host, int ntaps, int anchor) {
    hb_status s = check_image(in, out, H, W, in_pitch, out_pitch);
    if (s != HB_OK) return s;
    // lanes address rows with 32-bit byte offsets from the image base
    if ((int64_t)H * in_pitch >= ((int64_t)1 << 31) || (int64_t)H * out_pitch >= ((int64_t)1 << 30)) return HB_ERR_UNSUPPORTED;
    s = check_taps(taps_host, ntaps, anchor, HB_MAX_TAPS_FIR1D);
    if (s != HB_OK) return s;
    a.in = reinterpret_cast<const half_t*>(in);
    a.out = out;
    a.H = H;
    a.W = W;
    a.in_pitch = in_pitch;
    a.out_pitch = out_pitch;
    a.T = ntaps;
    a.anchor = anchor;
    const int nk = ceil_div(15 + ntaps + (anchor & 1), 32);
    a.nct = ceil_div(W, 16 * fir_tiles(nk));
    const int rowsteps = ceil_div(H, 16);
    // long filters are bound by the latency of one step, not by bandwidth: their waves take several
    // steps each, with the next step's windows in flight during the products
    const int64_t waves = nk <= 3 ? (int64_t)HB_FIR_WAVES : HB_FIR_LONG_WAVES;
    int steps = (int)(((int64_t)rowsteps * a.nct + waves - 1) / waves);
    a.steps = steps < 1 ? 1 : steps;
    a.ntasks = ceil_div(rowsteps, a.steps) * a.nct;
    a.taps = pack_taps<HB_MAX_TAPS_FIR1D>(taps_host, ntaps);
    a.fold = pack_fold_tables<HB_MAX_TAPS_FIR1D>(taps_host, ntaps);
    return HB_OK;
}

}  // namespace hb

extern "C" hb_status hb_fir1d_valu(const hb_half* in, float* out, int H, int W,
                                   int64_t in_pitch, int64_t out_pitch,
                                   const hb_half* taps_host, int ntaps, int anchor, hb_stream stream);

extern "C" hb_status hb_fir1d(const hb_half* in, float* out, int H, int W,
                              int64_t in_pitch, int64_t out_pitch,
                              const hb_half* taps_host, int ntaps, int anchor, hb_stream stream) {
    using namespace hb;
    FirArgs a;
    hb_status s = fir1d_prepare(a, in, out, H, W, in_pitch, out_pitch, taps_host, ntaps, anchor);
    if (s != HB_OK) return s;
    // a 16-column tile reads the 16 + ntaps - 1 pixels from x0 - anchor on (one more when the
    // window is moved to an even pixel): NK windows of 32
    const int nk = ceil_div(15 + ntaps + (anchor & 1), 32);
    if (W < 32 * nk)   // narrower than one window of the matrix formulation: vector-ALU kernel
        return hb_fir1d_valu(in, out, H, W, in_pitch, out_pitch, taps_host, ntaps, anchor, stream);
    const int blocks = min(ceil_div(a.ntasks, 4), kMaxStreamBlocks);
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const bool ss = (int64_t)H * W * 4 <= kStreamStoreMaxBytes;
    const dim3 grid(blocks), block(256);
#define HB_FIR_LAUNCH(N)                                                                          \
    case N:                                                                                       \
        if (ss) hipLaunchKernelGGL((fir1d_mfma_kernel<N, true>), grid, block, 0, st, a);          \
        else hipLaunchKernelGGL((fir1d_mfma_kernel<N, false>), grid, block, 0, st, a);            \
        break;
    switch (nk) {
        HB_FIR_LAUNCH(1) HB_FIR_LAUNCH(2) HB_FIR_LAUNCH(3) HB_FIR_LAUNCH(4) HB_FIR_LAUNCH(5)
        HB_FIR_LAUNCH(6) HB_FIR_LAUNCH(7) HB_FIR_LAUNCH(8) HB_FIR_LAUNCH(9)
        default: return HB_ERR_UNSUPPORTED;
    }
#undef HB_FIR_LAUNCH
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
