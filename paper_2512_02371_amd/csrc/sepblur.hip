// hb_sepblur: separable 2-D blur as two chained Toeplitz products per tile
// (Sec. V-A), and its vector-ALU twin.
//
// MFMA formulation.  A wave owns a strip of HB_SEP_TILES 16-column tiles and walks
// down it in steps of 16 rows.
//   row pass     T1[m][n] = sum_k P[m][k] * Bx[k][n]     m = image row, n = column, k = pixel
//                P = the 32*NKX pixels from x0 - ax - e on (e = ax & 1: even, dword-aligned
//                window start),   Bx[k][n] = taps_x[k - n - e]
//   column pass  O'[m][n] = sum_k T1h[m][k] * By[k][n]   m = column, n = output row, k = window row
//                By[k][n] = taps_y[window_row(k) - n]
// The row-pass accumulator holds, per lane, four consecutive ROWS of one column,
// which is exactly the operand layout of a product that contracts over rows: two
// stacked accumulators, rounded to fp16 (the stage's fp16 intermediate), are the
// K = 32 A-operand of the column pass without leaving the registers.  The paper
// handles the second axis with a serial loop over r_y; separability turns it into
// this second Toeplitz product with the roles of image and coefficients swapped.
// The column-pass accumulator holds four consecutive COLUMNS of one row per lane,
// so results leave with one 16-byte store per lane.
//
// The window rows of output rows [R, R+16) are [R - ay, R - ay + 15 + Ty - 1]; row
// tiles are laid on the grid R - ay + 16 q, so a step consumes NT = (Ty + 30) / 16
// consecutive tiles and produces one new tile.  Rows outside the image repeat the
// edge row: clamping the image row index at the load is the same as clamping the
// index of the row-filtered intermediate, because the row pass treats rows
// independently.  The pixels of the next row tile are requested before the current
// one is multiplied, so a wave always has one tile of loads in flight.
#include "hb_device.hpp"
#include "hb_host.hpp"

#ifndef HB_SEP_TILES
#define HB_SEP_TILES 2        // 16-column tiles per wave strip
#endif
#ifndef HB_SEP_WAVES
#define HB_SEP_WAVES 4096     // at most this many wave tasks per launch: one resident round, no straggler round
#endif


namespace hb {

struct SepArgs {
    const half_t* in;
    float* out;
    int H, W;
    int64_t in_pitch, out_pitch;
    int Tx, ax, Ty, ay;
    int steps;         // 16-row steps per task
    TaskGrid grid;     // strips x row segments
    Taps tx, ty;
    FoldTables foldx;
};

__device__ __forceinline__ half_t sep_tap(uint16_t b) { return __builtin_bit_cast(half_t, b); }

// One task: a strip of NW tiles, nsteps output steps.  XIN = every window of the strip
// lies inside the row and every tile is full: plain Toeplitz fragment, no store mask.
// Otherwise each tile's window is moved inside the row and the column clamp is folded
// into a per-tile hi + lo fragment.
template <int NKX, int NT, int NW, bool XIN, bool STREAM>
__device__ __forceinline__ void sep_task(const SepArgs& p, const FoldTables& fold, float* patch,
                                         const half8 (&coefx)[NKX],
                                         const half8 (&coefy)[(NT + 1) / 2],
                                         int x0, int Y0, int nsteps, int xw, int c, int g) {
    constexpr int NK = (NT + 1) / 2;
    const int ntiles = nsteps + NT - 1;

    // border strips: per-tile window start (absolute pixel, inside the row) and folded fragments
    int wsh[NW];
    half8 fh[XIN ? 1 : NW][NKX], fl[XIN ? 1 : NW][NKX];
    if (!XIN) {
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const int xt = x0 + 16 * w;
            const int ws = clampi(xt - xw, 0, p.W - 32 * NKX);
            wsh[w] = ws;
#pragma unroll
            for (int kk = 0; kk < NKX; ++kk) {
                if (ws == xt - xw && xt + 16 <= p.W) {
                    fh[w][kk] = coefx[kk];
                    fl[w][kk] = half8{0, 0, 0, 0, 0, 0, 0, 0};
                } else if (xt < p.W) {
                    folded_fragment(fold, p.Tx, p.ax, p.W, xt, ws, kk, c, g, fh[w][kk], fl[w][kk]);
                } else {
                    fh[w][kk] = fl[w][kk] = half8{0, 0, 0, 0, 0, 0, 0, 0};
                }
            }
        }
    }
    const half_t* src = p.in + (x0 - xw);                 // uniform; lanes add row * pitch + 8g
    float* dst = p.out + x0;

    half4 hist[NT][NW];                                   // row-filtered tiles q .. q+NT-1
#pragma unroll
    for (int q = 0; q < NT; ++q)
#pragma unroll
        for (int w = 0; w < NW; ++w) hist[q][w] = half4{0, 0, 0, 0};

    auto load_tile = [&](int q, half8 (&dstw)[NW][NKX]) {
        // tile q covers image rows Y0 - ay + 16 q + (0..15), clamped to the image
        const int yr = clampi(Y0 - p.ay + 16 * q + c, 0, p.H - 1);
        if (XIN) {
            const uint32_t off = ((uint32_t)yr * (uint32_t)p.in_pitch + 8u * g) * 2u;
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int kk = 0; kk < NKX; ++kk) dstw[w][kk] = ldg8(src, off + 2u * (16u * w + 32u * kk));
        } else {
            const half_t* row = p.in + (int64_t)yr * p.in_pitch + 8 * g;
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int kk = 0; kk < NKX; ++kk)
                    dstw[w][kk] = *reinterpret_cast<const half8_u*>(row + wsh[w] + 32 * kk);
        }
    };

    half8 cur[NW][NKX], nxt[NW][NKX];
    load_tile(0, cur);
    for (int q = 0; q < ntiles; ++q) {
        if (q + 1 < ntiles) load_tile(q + 1, nxt);        // next row tile in flight while this one is multiplied
#pragma unroll
        for (int u = 0; u < NT - 1; ++u)
#pragma unroll
            for (int w = 0; w < NW; ++w) hist[u][w] = hist[u + 1][w];
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < NKX; ++kk) {
                if (XIN) {
                    acc = mfma16x16x32(cur[w][kk], coefx[kk], acc);
                } else {
                    acc = mfma16x16x32(cur[w][kk], fh[w][kk], acc);
                    acc = mfma16x16x32(cur[w][kk], fl[w][kk], acc);
                }
            }
            hist[NT - 1][w] = to_half4(acc);
        }
        const int s = q - (NT - 1);                       // output step completed by this tile
        if (s >= 0) {
            const int yo = Y0 + 16 * s + c;
            floatx4 acc[NW];
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                acc[w] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < NK; ++j) {
                    const half4 lo = hist[2 * j][w];
                    const half4 hi = (2 * j + 1 < NT) ? hist[2 * j + 1][w] : half4{0, 0, 0, 0};
                    acc[w] = mfma16x16x32(join(lo, hi), coefy[j], acc[w]);
                }
            }
            if (XIN) {
                if (Y0 + 16 * s + 16 <= p.H) {
                    store_rows_via_lds<NW, STREAM>(patch, dst + (int64_t)(Y0 + 16 * s) * p.out_pitch,
                                                   (uint32_t)p.out_pitch, acc, (g << 4) | c);
                } else if (yo < p.H) {
                    const uint32_t off = ((uint32_t)yo * (uint32_t)p.out_pitch + 4u * g) * 4u;
#pragma unroll
                    for (int w = 0; w < NW; ++w) stg4<STREAM>(dst, off + 64u * w, acc[w]);
                }
            } else if (yo < p.H) {
                float* orow = p.out + (int64_t)yo * p.out_pitch;
#pragma unroll
                for (int w = 0; w < NW; ++w) {
                    const int xo = x0 + 16 * w + 4 * g;
                    if (xo < p.W) store4_mask(orow, xo, p.W, acc[w]);
                }
            }
        }
#pragma unroll
        for (int w = 0; w < NW; ++w)
#pragma unroll
            for (int kk = 0; kk < NKX; ++kk) cur[w][kk] = nxt[w][kk];
    }
}

// Coefficient fragments, read from the tap tables in the kernel arguments: coefx[kk] = B operand of the
// row pass, Bx[32 kk + 8g + i][c]; coefy[j] = B operand of the column pass in the chained slot order.
template <int NKX, int NK>
__device__ __forceinline__ void sep_fragments(const SepArgs& p, int c, int g, half8 (&coefx)[NKX], half8 (&coefy)[NK]) {
    const int e = p.ax & 1;
#pragma unroll
    for (int kk = 0; kk < NKX; ++kk) coefx[kk] = tap_run(p.tx.tab, 32 * kk + 8 * g - c - e);
#pragma unroll
    for (int j = 0; j < NK; ++j)
#pragma unroll
        for (int i = 0; i < 8; ++i) coefy[j][i] = tap_at(p.ty.tab, 32 * j + krow32(g, i) - c);
}

// Short task for the common case (one window per tile, up to three row tiles under an output tile):
// a strip of NW tiles x NS output steps whose NS + NT - 1 row tiles are ALL requested before the
// first product.  A wave then lives for one memory round trip plus its arithmetic, and what keeps
// the memory system busy is the number of such waves in flight (the dispatcher refills as they
// leave) rather than a chain of dependent steps inside one long-lived wave, each waiting for the
// one tile it has in flight.  Interior strips only (plain fragment, full tiles); rows are clamped
// per lane and rows beyond the image are not stored.
template <int NT, int NS, bool STREAM>
__device__ __forceinline__ void sep_task_short(const SepArgs& p, float* patch,
                                               int x0, int Y0, int xw, int c, int g) {
    constexpr int NW = HB_SEP_TILES, NL = NS + NT - 1, NK = (NT + 1) / 2;
    const half_t* src = p.in + (x0 - xw);                 // uniform; lanes add row * pitch + 8g
    float* dst = p.out + x0;
    half8 px[NL][NW];
#pragma unroll
    for (int q = 0; q < NL; ++q) {
        const int yr = clampi(Y0 - p.ay + 16 * q + c, 0, p.H - 1);
        const uint32_t off = ((uint32_t)yr * (uint32_t)p.in_pitch + 8u * g) * 2u;
#pragma unroll
        for (int w = 0; w < NW; ++w) px[q][w] = ldg8(src, off + 32u * w);
    }
    // The tap tables are read only now: a wave that waited for them first would put a memory round
    // trip in front of its pixel requests.
    __builtin_amdgcn_sched_barrier(0);
    half8 coefx1[1], coefy[NK];
    sep_fragments<1, NK>(p, c, g, coefx1, coefy);
    const half8 coefx = coefx1[0];
    half4 h[NL][NW];                                      // row-filtered tiles, rounded to fp16
#pragma unroll
    for (int q = 0; q < NL; ++q) {
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const floatx4 zero = {0.f, 0.f, 0.f, 0.f};
            h[q][w] = to_half4(mfma16x16x32(px[q][w], coefx, zero));
        }
        if (q < NT - 1) continue;
        const int s = q - (NT - 1);                       // output step completed by this tile
        floatx4 acc[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            acc[w] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < NK; ++j) {
                const half4 lo = h[s + 2 * j][w];
                const half4 hi = (2 * j + 1 < NT) ? h[s + 2 * j + 1][w] : half4{0, 0, 0, 0};
                acc[w] = mfma16x16x32(join(lo, hi), coefy[j], acc[w]);
            }
        }
        if (Y0 + 16 * s + 16 <= p.H) {
            store_rows_via_lds<NW, STREAM>(patch, dst + (int64_t)(Y0 + 16 * s) * p.out_pitch,
                                           (uint32_t)p.out_pitch, acc, (g << 4) | c);
        } else {
            const int yo = Y0 + 16 * s + c;
            if (yo < p.H) {
                const uint32_t off = ((uint32_t)yo * (uint32_t)p.out_pitch + 4u * g) * 4u;
#pragma unroll
                for (int w = 0; w < NW; ++w) stg4<STREAM>(dst, off + 64u * w, acc[w]);
            }
        }
    }
}

// Short tasks come in two lengths: 8 output steps while that still leaves the image in one resident
// round of waves (4096 x 4096: 4096 waves; measured 24 us against 27 us with 4 steps), else 4 steps
// (8192 x 8192: 98 us against 107 us).  NS = 0 selects the walking task.
constexpr bool sep_short_ok(int nkx, int nt) { return nkx == 1 && nt <= 3; }
constexpr int kSepOneRoundWaves = 4608;

template <int NKX, int NT, bool STREAM, int NS = 0>
__global__ void __launch_bounds__(256) sepblur_mfma_kernel(SepArgs p) {
    constexpr int NK = (NT + 1) / 2;          // K = 32 chunks of the column pass
    constexpr int NW = HB_SEP_TILES;
    __shared__ __attribute__((aligned(16))) float s_patch[4][RowPatch<HB_SEP_TILES>::kFloats];

    const int lane = threadIdx.x & 63;
    const int c = lane & 15, g = lane >> 4;

    const int e = p.ax & 1;
    const int xw = p.ax + e;                  // window start, left of the tile
    // of every 32 workgroups an XCD takes four neighbours (measured on 4096 x 4096 / 8192 x 8192: this
    // order 24.1 / 84.7 us, one contiguous eighth of the tasks per XCD 24.2 / 97.7, plain order 26.4 / 87.3)
    const int wgpos = xcd_blocked(blockIdx.x, gridDim.x, 4);
    const int wave = __builtin_amdgcn_readfirstlane(wgpos * 4 + (threadIdx.x >> 6));
    const int nwaves = (gridDim.x * blockDim.x) >> 6;
    const int ntasks = p.grid.count();
    for (int task = wave; task < ntasks; task += nwaves) {
        const int seg = task / p.grid.nct, ct = task - seg * p.grid.nct;
        const int x0 = 16 * NW * ct;
        const int Y0 = seg * p.steps * 16;
        const int nsteps = min(p.steps, (p.H - Y0 + 15) / 16);
        if constexpr (NS > 0) {
            if (p.grid.interior(seg, ct)) {   // builds its fragments itself, AFTER its pixel loads are on their way
                sep_task_short<NT, NS, STREAM>(p, s_patch[threadIdx.x >> 6], x0, Y0, xw, c, g);
                continue;
            }
        }
        half8 coefx[NKX], coefy[NK];
        sep_fragments<NKX, NK>(p, c, g, coefx, coefy);
        if (p.grid.interior(seg, ct)) sep_task<NKX, NT, NW, true, STREAM>(p, p.foldx, s_patch[threadIdx.x >> 6], coefx, coefy, x0, Y0, nsteps, xw, c, g);
        else sep_task<NKX, NT, NW, false, STREAM>(p, p.foldx, s_patch[threadIdx.x >> 6], coefx, coefy, x0, Y0, nsteps, xw, c, g);
    }
}

// ---------------------------------------------------------------------------
// Vector-ALU twin: 32 x 64 output tile per workgroup; pixels with halo in LDS (column and row indices
// clamped, the definition's border rule verbatim), row pass to an LDS intermediate (rounded to fp16 like
// the matrix kernel's, kept as fp32), column pass from it.  Both passes are register-blocked: a thread
// owns 8 consecutive outputs of a row (of a column) and reads 8 taps and 8 new samples per 64 FMAs.
// Taps are padded with zeros to a multiple of 8.
constexpr int kVTH = 32, kVTW = 64;
constexpr int kVRows = kVTH + HB_MAX_TAPS;              // 96: rows the column pass may touch
constexpr int kVPxPitch = kVTW + HB_MAX_TAPS + 8;       // 136 halves

__global__ void __launch_bounds__(256) sepblur_valu_kernel(SepArgs p) {
    __shared__ __attribute__((aligned(16))) half_t s_px[kVRows * kVPxPitch];
    __shared__ __attribute__((aligned(16))) float s_tmp[kVRows * kVTW];
    __shared__ __attribute__((aligned(16))) float s_kx[HB_MAX_TAPS], s_ky[HB_MAX_TAPS];
    static_assert(HB_MAX_TAPS % 8 == 0, "taps are processed eight at a time");
    if (threadIdx.x < HB_MAX_TAPS) {
        s_kx[threadIdx.x] = (int)threadIdx.x < p.Tx ? (float)tap_at(p.tx.tab, threadIdx.x) : 0.f;
        s_ky[threadIdx.x] = (int)threadIdx.x < p.Ty ? (float)tap_at(p.ty.tab, threadIdx.x) : 0.f;
    }
    const int nctv = (p.W + kVTW - 1) / kVTW;
    const int rt = blockIdx.x / nctv, ct = blockIdx.x - rt * nctv;
    const int x0 = ct * kVTW, y0 = rt * kVTH;
    const int txp = (p.Tx + 7) & ~7, typ = (p.Ty + 7) & ~7;
    const int nrows = kVTH + p.Ty - 1;                     // image rows under the tile
    // staged pixel (r, j) = in[clampH(y0 - ay + r)][clampW(x0 - ax + j)], j < 64 + txp covers every window
    const int nch = (kVTW + txp) / 8;
    for (int idx = threadIdx.x; idx < nrows * nch; idx += 256) {
        const int r = idx / nch, ch = idx - r * nch;
        const half_t* row = p.in + (int64_t)clampi(y0 - p.ay + r, 0, p.H - 1) * p.in_pitch;
        *reinterpret_cast<half8*>(&s_px[r * kVPxPitch + 8 * ch]) = load8_clamp(row, x0 - p.ax + 8 * ch, p.W);
    }
    __syncthreads();
    // row pass: thread = 8 consecutive columns of one staged row
    for (int idx = threadIdx.x; idx < nrows * (kVTW / 8); idx += 256) {
        const int r = idx >> 3, xl = 8 * (idx & 7);
        const half8* src = reinterpret_cast<const half8*>(&s_px[r * kVPxPitch + xl]);
        float acc[8], w[16];
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[q] = 0.f;
        {
            const half8 v = src[0];
#pragma unroll
            for (int i = 0; i < 8; ++i) w[i] = (float)v[i];
        }
        for (int tb = 0; tb < txp; tb += 8) {
            const half8 v = src[tb / 8 + 1];
            const floatx4 ka = *reinterpret_cast<const floatx4*>(&s_kx[tb]), kb = *reinterpret_cast<const floatx4*>(&s_kx[tb + 4]);
#pragma unroll
            for (int i = 0; i < 8; ++i) w[8 + i] = (float)v[i];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float kv = i < 4 ? ka[i] : kb[i - 4];
#pragma unroll
                for (int q = 0; q < 8; ++q) acc[q] = fmaf(kv, w[q + i], acc[q]);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) w[i] = w[8 + i];
        }
        floatx4* dst = reinterpret_cast<floatx4*>(&s_tmp[r * kVTW + xl]);
        dst[0] = floatx4{(float)(half_t)acc[0], (float)(half_t)acc[1], (float)(half_t)acc[2], (float)(half_t)acc[3]};
        dst[1] = floatx4{(float)(half_t)acc[4], (float)(half_t)acc[5], (float)(half_t)acc[6], (float)(half_t)acc[7]};
    }
    // rows only the zero taps reach
    for (int idx = nrows * kVTW + threadIdx.x; idx < (kVTH + typ) * kVTW; idx += 256) s_tmp[idx] = 0.f;
    __syncthreads();
    // column pass: thread = 8 consecutive rows of one column
    const int x = threadIdx.x & 63, r0 = 8 * (threadIdx.x >> 6);
    if (x0 + x >= p.W || y0 + r0 >= p.H) return;
    float acc[8], w[16];
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) w[i] = s_tmp[(r0 + i) * kVTW + x];
    for (int tb = 0; tb < typ; tb += 8) {
        const floatx4 ka = *reinterpret_cast<const floatx4*>(&s_ky[tb]), kb = *reinterpret_cast<const floatx4*>(&s_ky[tb + 4]);
#pragma unroll
        for (int i = 0; i < 8; ++i) w[8 + i] = s_tmp[(r0 + tb + 8 + i) * kVTW + x];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float kv = i < 4 ? ka[i] : kb[i - 4];
#pragma unroll
            for (int q = 0; q < 8; ++q) acc[q] = fmaf(kv, w[q + i], acc[q]);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) w[i] = w[8 + i];
    }
#pragma unroll
    for (int q = 0; q < 8; ++q)
        if (y0 + r0 + q < p.H) p.out[(int64_t)(y0 + r0 + q) * p.out_pitch + x0 + x] = acc[q];
}

static hb_status sep_prepare(SepArgs& a, const hb_half* in, float* out, int H, int W,
                             int64_t in_pitch, int64_t out_pitch,
                             const hb_half* tx, int ntx, int ax, const hb_half* ty, int nty, int ay) {
    hb_status s = check_image(in, out, H, W, in_pitch, out_pitch);
    if (s != HB_OK) return s;
    // lanes address rows with 32-bit byte offsets from the image base
    if ((int64_t)H * in_pitch >= ((int64_t)1 << 31) || (int64_t)H * out_pitch >= ((int64_t)1 << 30)) return HB_ERR_UNSUPPORTED;
    if ((s = check_taps(tx, ntx, ax)) != HB_OK) return s;
    if ((s = check_taps(ty, nty, ay)) != HB_OK) return s;
    a.in = reinterpret_cast<const half_t*>(in);
    a.out = out;
    a.H = H;
    a.W = W;
    a.in_pitch = in_pitch;
    a.out_pitch = out_pitch;
    a.Tx = ntx;
    a.ax = ax;
    a.Ty = nty;
    a.ay = ay;
    const int nct = ceil_div(W, 16 * HB_SEP_TILES);
    const int rowsteps = ceil_div(H, 16);
    // enough tasks to fill the chip, few enough that the (NT-1)-tile warm-up stays small; the short
    // tasks of the common case have a fixed length
    const int nkx0 = ceil_div(15 + ntx + (ax & 1), 32);
    int steps = (int)(((int64_t)rowsteps * nct + HB_SEP_WAVES - 1) / HB_SEP_WAVES);
    steps = steps < 1 ? 1 : steps;
    if (sep_short_ok(nkx0, (nty + 30) / 16))
        steps = (int64_t)ceil_div(rowsteps, 8) * nct <= kSepOneRoundWaves ? 8 : 4;
    a.steps = steps;
    a.grid.nct = nct;
    a.grid.nseg = ceil_div(rowsteps, steps);
    // a strip is interior when all its windows lie inside the row and its tiles are full;
    // rows are clamped per lane in both kernels
    const int xw = ax + (ax & 1);
    const int nkx = ceil_div(15 + ntx + (ax & 1), 32);
    const int after = 16 * (HB_SEP_TILES - 1) - xw + 32 * nkx;
    interior_range(nct, 16 * HB_SEP_TILES, xw, after > 16 * HB_SEP_TILES ? after : 16 * HB_SEP_TILES, W,
                   a.grid.c0, a.grid.c1);
    a.grid.s0 = 0;
    a.grid.s1 = a.grid.c1 > a.grid.c0 ? a.grid.nseg : 0;
    a.tx = pack_taps(tx, ntx);
    a.ty = pack_taps(ty, nty);
    a.foldx = pack_fold_tables(tx, ntx);
    return HB_OK;
}

template <int NKX, int NT, bool STREAM>
static void sep_launch2(hipStream_t st, const SepArgs& a) {
    const dim3 grid(min(ceil_div(a.grid.count(), 4), kMaxStreamBlocks));
    if constexpr (sep_short_ok(NKX, NT)) {
        if (a.steps == 8) hipLaunchKernelGGL((sepblur_mfma_kernel<NKX, NT, STREAM, 8>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((sepblur_mfma_kernel<NKX, NT, STREAM, 4>), grid, dim3(256), 0, st, a);
    } else {
        hipLaunchKernelGGL((sepblur_mfma_kernel<NKX, NT, STREAM, 0>), grid, dim3(256), 0, st, a);
    }
}
template <int NKX, bool STREAM>
static void sep_launch_nt(int nt, hipStream_t st, const SepArgs& a) {
    switch (nt) {
        case 1: sep_launch2<NKX, 1, STREAM>(st, a); break;
        case 2: sep_launch2<NKX, 2, STREAM>(st, a); break;
        case 3: sep_launch2<NKX, 3, STREAM>(st, a); break;
        case 4: sep_launch2<NKX, 4, STREAM>(st, a); break;
        default: sep_launch2<NKX, 5, STREAM>(st, a); break;
    }
}
template <int NKX>
static void sep_launch(bool stream_stores, int nt, hipStream_t st, const SepArgs& a) {
    if (stream_stores) sep_launch_nt<NKX, true>(nt, st, a);
    else sep_launch_nt<NKX, false>(nt, st, a);
}

}  // namespace hb

extern "C" hb_status hb_sepblur_valu(const hb_half* in, float* out, int H, int W,
                                     int64_t in_pitch, int64_t out_pitch,
                                     const hb_half* taps_x_host, int ntaps_x, int anchor_x,
                                     const hb_half* taps_y_host, int ntaps_y, int anchor_y, hb_stream stream);

extern "C" hb_status hb_sepblur(const hb_half* in, float* out, int H, int W,
                                int64_t in_pitch, int64_t out_pitch,
                                const hb_half* taps_x_host, int ntaps_x, int anchor_x,
                                const hb_half* taps_y_host, int ntaps_y, int anchor_y, hb_stream stream) {
    using namespace hb;
    SepArgs a;
    hb_status s = sep_prepare(a, in, out, H, W, in_pitch, out_pitch, taps_x_host, ntaps_x, anchor_x,
                              taps_y_host, ntaps_y, anchor_y);
    if (s != HB_OK) return s;
    const int nkx = ceil_div(15 + ntaps_x + (anchor_x & 1), 32);
    if (W < 32 * nkx)   // narrower than one window of the matrix formulation: vector-ALU kernel
        return hb_sepblur_valu(in, out, H, W, in_pitch, out_pitch, taps_x_host, ntaps_x, anchor_x,
                               taps_y_host, ntaps_y, anchor_y, stream);
    const int nt = (ntaps_y + 30) / 16;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const bool ss = (int64_t)H * W * 4 <= kStreamStoreMaxBytes;
    switch (nkx) {
        case 1: sep_launch<1>(ss, nt, st, a); break;
        case 2: sep_launch<2>(ss, nt, st, a); break;
        case 3: sep_launch<3>(ss, nt, st, a); break;
        default: return HB_ERR_UNSUPPORTED;
    }
    return launch_status();
}

extern "C" hb_status hb_sepblur_valu(const hb_half* in, float* out, int H, int W,
                                     int64_t in_pitch, int64_t out_pitch,
                                     const hb_half* taps_x_host, int ntaps_x, int anchor_x,
                                     const hb_half* taps_y_host, int ntaps_y, int anchor_y, hb_stream stream) {
    using namespace hb;
    SepArgs a;
    hb_status s = sep_prepare(a, in, out, H, W, in_pitch, out_pitch, taps_x_host, ntaps_x, anchor_x,
                              taps_y_host, ntaps_y, anchor_y);
    if (s != HB_OK) return s;
    const int64_t blocks = (int64_t)ceil_div(H, kVTH) * ceil_div(W, kVTW);
    if (blocks > 0x7fffffff) return HB_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(sepblur_valu_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       reinterpret_cast<hipStream_t>(stream), a);
    return launch_status();
}
