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
#include <utility>

#include "hb_device.hpp"
#include "hb_host.hpp"

#ifndef HB_FIR_TILES
#define HB_FIR_TILES 4        // 16-column tiles per wave strip
#endif
#ifndef HB_FIR_WAVES
#define HB_FIR_WAVES (1 << 20) // wave tasks per launch before a task takes more than one 16-row step;
                              // rows are independent here, so short-lived waves stream best
#endif

#ifndef HB_FIR_WALK_WAVES
#define HB_FIR_WALK_WAVES 4096 // the walk of long filters: aim for about this many wave tasks per launch ...
#endif
#ifndef HB_FIR_WALK_MIN_NK
#define HB_FIR_WALK_MIN_NK 2    // windows per tile from which the walk is used
#endif
#ifndef HB_FIR_WALK_MIN_TURNS
#define HB_FIR_WALK_MIN_TURNS 2 // ... but no run shorter than this many turns of the accumulator ring (2 NK tiles each)
#endif

namespace hb {

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): a loop that is unrolled by construction,
// so that register arrays indexed by the step stay in registers.
template <class F, int... I>
__device__ __forceinline__ void unrolled_steps_impl(F& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void unrolled_steps(F& f) {
    unrolled_steps_impl(f, std::make_integer_sequence<int, N>{});
}

struct FirArgs {
    const half_t* in;
    float* out;
    int H, W;
    int64_t in_pitch, out_pitch;
    int T, anchor;
    int nct;             // strips per row group
    int steps;           // 16-row steps per task
    int ntasks;          // strips x row segments
    int ntiles, run_tiles, nruns, wtasks;   // the walk of long filters: tiles per row, per run, runs per row group, tasks
    TapsT<HB_MAX_TAPS_FIR1D> taps;
    FoldTablesT<HB_MAX_TAPS_FIR1D> fold;
};

// Tiles per wave strip of the one-window kernel (it is written for any NK, but filters with two or
// more windows per tile take the walk further down).
constexpr int fir_tiles(int) { return HB_FIR_TILES; }

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
    // (read from the tap table in the kernel arguments AFTER the first pixel loads are on their way: a
    // wave that waited for the table first would put a memory round trip in front of its pixel requests)
    auto fragments = [&](half8 (&coef)[NK]) {
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) coef[kk] = tap_run(p.taps.tab, 32 * kk + 8 * g - c - e);
    };
    const int wmax = p.W - 32 * NK;           // last window start that stays inside the row

    // (tasks in plain launch order: with one contiguous eighth of the tasks per XCD this kernel measured
    // 10 % slower on tall images, 100 against 89 us on 262144 x 256; groups of 2 to 8 neighbours per XCD
    // measured within 2 % of the plain order there)
    const int wave = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + (threadIdx.x >> 6));
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
            __builtin_amdgcn_sched_barrier(0);
            half8 coef[NK];
            fragments(coef);
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
            half8 coef[NK];
            fragments(coef);
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

// ---------------------------------------------------------------------------
// Long filters (three or more windows per tile): the walk along the row.
//
// In the kernel above every product loads its own window, NK loads of 16 rows x 64 bytes per
// 16 x 16 outputs, and with long filters those loads are all the kernel does (256 taps: 9 KB requested
// per 1 KB of outputs; the matrix units idle).  But window u (the 32 pixels from 16 u - aw on) is the
// kk-th window of tile u - 2 kk for every kk < NK: here a wave walks along a run of tiles of one
// 16-row group, loads each window ONCE and multiplies it with all NK fragments, each product going
// to the accumulator of its own tile.  2 NK - 1 tiles are open at any time (a ring of 2 NK
// accumulators, indexed at compile time: the walk is unrolled over one turn of the ring); a tile is
// complete 2 NK - 2 steps after its first window, and completed tiles leave in pairs through the LDS
// patch as 128-byte runs.  A pixel is requested twice (windows of 32 at a stride of 16) instead of
// 2 NK times.  Windows that reach over the row ends are loaded pixel by pixel with the column
// clamped: the Toeplitz matrix is indexed by window position, so the border rule needs nothing else.
// Runs start 2 NK - 2 windows early (products into accumulators of tiles left of the run are
// computed and dropped), the price of cutting a row into several tasks.
// Waves per workgroup of the walk: the longest filters (few, long-lived waves of 100+ registers) run
// best as single-wave workgroups, the shorter ones four to a workgroup (measured).
constexpr int fir_walk_waves(int nk) { return nk >= 7 ? 1 : 4; }

template <int NK, bool STREAM>
__global__ void __launch_bounds__(64 * fir_walk_waves(NK)) fir1d_walk_kernel(FirArgs p) {
    constexpr int R = 2 * NK;
    constexpr int WV = fir_walk_waves(NK);
    __shared__ __attribute__((aligned(16))) float s_patch[WV][RowPatch<2>::kFloats];
    const int lane = threadIdx.x & 63;
    const int c = lane & 15, g = lane >> 4;
    const int e = p.anchor & 1;
    const int aw = p.anchor + e;
    half8 coef[NK];
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) coef[kk] = tap_run(p.taps.tab, 32 * kk + 8 * g - c - e);

    const int wgpos = xcd_contiguous(blockIdx.x, gridDim.x);
    const int task = __builtin_amdgcn_readfirstlane(wgpos * WV + (threadIdx.x >> 6));
    if (task >= p.wtasks) return;
    const int rg = task / p.nruns, run = task - rg * p.nruns;
    const int t0 = run * p.run_tiles;                     // first tile of the run
    const int L = min(p.run_tiles, p.ntiles - t0);        // its tiles
    const int nsteps = L + 2 * (NK - 1);                  // windows t0 .. t0 + nsteps - 1
    const int y0 = 16 * rg;
    const uint32_t rowoff = (uint32_t)min(y0 + c, p.H - 1) * (uint32_t)p.in_pitch * 2u;
    float* patch = s_patch[threadIdx.x >> 6];
    const bool rows16 = y0 + 16 <= p.H;

    auto load_window = [&](int u) {
        const int xs = 16 * (t0 + u) - aw;                // uniform
        half8 v;
        if (xs >= 0 && xs + 32 <= p.W) {
            v = ldg8(p.in, rowoff + 2u * (uint32_t)(xs + 8 * g));
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int x = clampi(xs + 8 * g + i, 0, p.W - 1);
                v[i] = *reinterpret_cast<const half_t*>(reinterpret_cast<const char*>(p.in) + (rowoff + 2u * (uint32_t)x));
            }
        }
        return v;
    };
    floatx4 done[2] = {floatx4{0.f, 0.f, 0.f, 0.f}, floatx4{0.f, 0.f, 0.f, 0.f}};
    // the pair of tiles tb, tb + 1 (tb even, relative to the run), completed in the two steps before
    auto store_pair = [&](int tb) {
        if (tb < 0 || tb >= L) return;
        const int x = 16 * (t0 + tb);
        if (rows16 && x + 32 <= p.W) {
            store_rows_via_lds<2, STREAM>(patch, p.out + (int64_t)y0 * p.out_pitch + x, (uint32_t)p.out_pitch, done, lane);
        } else if (y0 + c < p.H) {
            float* row = p.out + (int64_t)(y0 + c) * p.out_pitch;
            store4_mask(row, x + 4 * g, p.W, done[0]);
            if (tb + 1 < L) store4_mask(row, x + 16 + 4 * g, p.W, done[1]);
        }
    };

    floatx4 acc[R];
#pragma unroll
    for (int i = 0; i < R; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    // NK windows in flight: the longer the filter, the more products a window feeds and the further
    // ahead the loads have to run to cover their latency
    half8 win[NK];
#pragma unroll
    for (int i = 0; i < NK; ++i) win[i] = load_window(i < nsteps ? i : 0);
    int ub = 0;
    // one step: window ub + S against every fragment; the tile whose last window this was leaves its slot
    auto step = [&](auto sc) {
        constexpr int S = decltype(sc)::value;
        const int u = ub + S;
        if (S % 2 == 0) store_pair(u - R);                // before the loads: loads and stores share one counter
        if (u < nsteps) {
            auto product = [&](auto kc) {
                constexpr int KK = decltype(kc)::value, slot = ((S - 2 * KK) % R + R) % R;
                acc[slot] = mfma16x16x32(coef[KK], win[S % NK], acc[slot]);
            };
            unrolled_steps<NK>(product);
            constexpr int last = (S + 2) % R;             // slot of tile u - 2 (NK - 1)
            done[S & 1] = acc[last];
            acc[last] = floatx4{0.f, 0.f, 0.f, 0.f};
            if (u + NK < nsteps) win[S % NK] = load_window(u + NK);
        }
    };
#pragma unroll 1
    for (ub = 0; ub < nsteps; ub += R) unrolled_steps<R>(step);
    store_pair(ub - R);
}

// Vector-ALU twin: a 16 x 128 tile is staged in LDS as fp32 with its halo, the column index clamped
// (the definition's border rule verbatim).  A thread owns 8 consecutive outputs of one row and slides
// the taps over them eight at a time: 8 taps and 8 new pixels are read (16-byte LDS reads), 64 FMAs use
// them.  Taps are padded with zeros to a multiple of 8.
constexpr int kValuTileW = 128;
constexpr int kValuPitch = kValuTileW + HB_MAX_TAPS_FIR1D + 8;   // floats per staged row

__global__ void __launch_bounds__(256) fir1d_valu_kernel(FirArgs p) {
    __shared__ __attribute__((aligned(16))) float s_px[16 * kValuPitch];
    __shared__ __attribute__((aligned(16))) float s_k[HB_MAX_TAPS_FIR1D];
    static_assert(HB_MAX_TAPS_FIR1D <= 256, "one tap per thread");
    const int tp = (p.T + 7) & ~7;
    if ((int)threadIdx.x < tp) s_k[threadIdx.x] = (int)threadIdx.x < p.T ? (float)tap_at(p.taps.tab, threadIdx.x) : 0.f;

    const int nctv = (p.W + kValuTileW - 1) / kValuTileW;
    const int rg = blockIdx.x / nctv, ct = blockIdx.x - rg * nctv;
    const int x0 = ct * kValuTileW;
    // staged column j holds pixel clampW(x0 - anchor + j); j < 128 + tp covers every window
    const int nch = (kValuTileW + tp) / 8;
    for (int idx = threadIdx.x; idx < 16 * nch; idx += 256) {
        const int r = idx / nch, ch = idx - r * nch;
        const half_t* row = p.in + (int64_t)min(16 * rg + r, p.H - 1) * p.in_pitch;
        const half8 v = load8_clamp(row, x0 - p.anchor + 8 * ch, p.W);
        floatx4* dst = reinterpret_cast<floatx4*>(&s_px[r * kValuPitch + 8 * ch]);
        dst[0] = floatx4{(float)v[0], (float)v[1], (float)v[2], (float)v[3]};
        dst[1] = floatx4{(float)v[4], (float)v[5], (float)v[6], (float)v[7]};
    }
    __syncthreads();

    const int r = threadIdx.x >> 4, xl = 8 * (threadIdx.x & 15);
    const int y = 16 * rg + r;
    if (y >= p.H || x0 + xl >= p.W) return;
    const floatx4* src = reinterpret_cast<const floatx4*>(&s_px[r * kValuPitch + xl]);
    float acc[8], w[16];
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] = 0.f;
    {
        const floatx4 a = src[0], b = src[1];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = a[i], w[4 + i] = b[i];
    }
    for (int tb = 0; tb < tp; tb += 8) {
        const floatx4 a = src[tb / 4 + 2], b = src[tb / 4 + 3];      // pixels xl + tb + 8 .. + 15
        const floatx4 ka = *reinterpret_cast<const floatx4*>(&s_k[tb]), kb = *reinterpret_cast<const floatx4*>(&s_k[tb + 4]);
#pragma unroll
        for (int i = 0; i < 4; ++i) w[8 + i] = a[i], w[12 + i] = b[i];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float kv = i < 4 ? ka[i] : kb[i - 4];
#pragma unroll
            for (int q = 0; q < 8; ++q) acc[q] = fmaf(kv, w[q + i], acc[q]);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) w[i] = w[8 + i];
    }
    float* orow = p.out + (int64_t)y * p.out_pitch;
    store4_mask(orow, x0 + xl, p.W, floatx4{acc[0], acc[1], acc[2], acc[3]});
    store4_mask(orow, x0 + xl + 4, p.W, floatx4{acc[4], acc[5], acc[6], acc[7]});
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
    const int64_t waves = HB_FIR_WAVES;
    int steps = (int)(((int64_t)rowsteps * a.nct + waves - 1) / waves);
    a.steps = steps < 1 ? 1 : steps;
    a.ntasks = ceil_div(rowsteps, a.steps) * a.nct;
    // the walk of long filters: runs of an even number of tiles, at least a few turns of the ring long
    a.ntiles = ceil_div(W, 16);
    const int want_runs = ceil_div(HB_FIR_WALK_WAVES, rowsteps);
    int max_runs = a.ntiles / (HB_FIR_WALK_MIN_TURNS * 2 * nk);
    if (max_runs < 1) max_runs = 1;
    const int runs = want_runs < max_runs ? want_runs : max_runs;
    a.run_tiles = (ceil_div(a.ntiles, runs) + 1) & ~1;
    a.nruns = ceil_div(a.ntiles, a.run_tiles);
    const int64_t wtasks = (int64_t)rowsteps * a.nruns;
    if (wtasks > 0x7fffffff / 4) return HB_ERR_UNSUPPORTED;
    a.wtasks = (int)wtasks;
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
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const bool ss = (int64_t)H * W * 4 <= kStreamStoreMaxBytes;
    if (nk >= HB_FIR_WALK_MIN_NK) {   // long filters: the walk along the row, every window loaded once
#define HB_FIR_WALK(N)                                                                            \
    case N: {                                                                                     \
        const dim3 wgrid(ceil_div(a.wtasks, fir_walk_waves(N))), wblock(64 * fir_walk_waves(N));  \
        if (ss) hipLaunchKernelGGL((fir1d_walk_kernel<N, true>), wgrid, wblock, 0, st, a);        \
        else hipLaunchKernelGGL((fir1d_walk_kernel<N, false>), wgrid, wblock, 0, st, a);          \
        break;                                                                                    \
    }
        switch (nk) {
            HB_FIR_WALK(2) HB_FIR_WALK(3) HB_FIR_WALK(4) HB_FIR_WALK(5) HB_FIR_WALK(6) HB_FIR_WALK(7) HB_FIR_WALK(8) HB_FIR_WALK(9)
            default: return HB_ERR_UNSUPPORTED;
        }
#undef HB_FIR_WALK
        return launch_status();
    }
    // one window per tile: nothing to share between tiles, every wave takes one strip of tiles
    const int blocks = min(ceil_div(a.ntasks, 4), kMaxStreamBlocks);
    const dim3 grid(blocks), block(256);
    if (ss) hipLaunchKernelGGL((fir1d_mfma_kernel<1, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((fir1d_mfma_kernel<1, false>), grid, block, 0, st, a);
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
