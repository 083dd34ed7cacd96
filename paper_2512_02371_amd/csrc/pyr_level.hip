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
// of 32 output rows.  D tiles (16 x 16) lie on a grid shifted against the outputs so that the
// K = 32 window of an up pass (two adjacent D tiles) covers the 18 values that 32 outputs need:
// NS + 1 column tiles per strip, one extra row tile per task.  A D tile needs 35 image
// rows/columns: a K = 32 plus a K = 16 product over three image row tiles / a 48-pixel window.
//
// Interior tasks (pyr_fast_task) shift the D grid by 7: image tiles then start 16 rows / columns
// before the outputs, so an image row tile holds exactly the rows of one 16-row output tile.  The
// loaded operand fragments are parked in a wave-private LDS ring and come back, three tiles
// later, as the B operand of a 0/1 selection product that seeds the accumulator of the last
// pass with the original pixels: the residual in - U then needs no second read of the image
// and no separate subtraction (the up-x pass stores -U1).  Image tiles are requested three
// tiles ahead into a register ring (the loop is unrolled over the ring, so no copy waits on a
// load in flight).
//
// At the image border (pyr_task) the up passes clamp the D index; there the coefficient
// fragments are rebuilt from absolute indices (taps that clamp onto the same D sample
// add up), which also makes out-of-range D tiles (computed from clamped pixels) inert.
#include <type_traits>

#include "hb_device.hpp"
#include "hb_host.hpp"

#ifndef HB_PYR_NS
#define HB_PYR_NS 2           // 32-column output blocks per wave strip
#endif
#ifndef HB_PYR_WAVES
#define HB_PYR_WAVES 5400     // aim for about this many interior wave tasks per launch
#endif

namespace hb {

struct PyrArgs {
    const half_t* in;
    float* res;
    half_t* down;      // may be null
    int H, W, Hd, Wd;
    int64_t in_pitch, res_pitch, down_pitch;
    // Task list of one launch (wave tasks).  Row steps are 32 output rows high.
    // Border tasks come first, each one 32-column block wide (the general path): the row steps above
    // r0 and from r1 on, one step per task, over all nblk blocks; then the blocks left of the interior
    // (nbl of them) and right of it (from block bR on) over the row steps [r0, r1) in chunks of
    // kPyrBorderSteps.  Interior tasks follow: nci strips of 32*NS columns starting at column 32*nbl,
    // each cut into nseg segments of `steps` row steps out of [r0, r1).
    int nblk, rowsteps;
    int nbl, bR, nci, r0, r1;
    int steps, nseg, nchunk;
    int ntop, nbot, nborder;

    __host__ __device__ int count() const { return nborder + nci * nseg; }
};
constexpr int kPyrBorderSteps = 4;

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
// Weight of D[dabs] in output xabs when the D index is clamped to [0, n-1]: the plain phase weight,
// plus, on the first and last D sample, the weights of the neighbours that clamp onto it.
__device__ __forceinline__ float upw_clamped(int dabs, int xabs, int n) {
    const int q = xabs >> 1, ph = xabs & 1;
    float s = (dabs >= 0 && dabs < n) ? upw(ph, dabs - q) : 0.f;
    if (dabs == 0 || dabs == n - 1) {
#pragma unroll
        for (int delta = -1; delta <= 1; ++delta) {
            const int d = q + delta;
            if ((dabs == 0 && d < 0) || (dabs == n - 1 && d > n - 1)) s += upw(ph, delta);
        }
    }
    return s;
}

// Sum of the taps t < j of [1,4,6,4,1]/16.
__device__ __forceinline__ float w5_prefix(int j) {
    return j <= 0 ? 0.f : j == 1 ? 0.0625f : j == 2 ? 0.3125f : j == 3 ? 0.6875f : j == 4 ? 0.9375f : 1.f;
}
// Weight of pixel u in D sample n when the pixel index 2n + t - 2 (t = 0..4) is clamped to [0, len-1]:
// the plain tap, plus, on the first and last pixel, the taps that clamp onto it.
__device__ __forceinline__ half_t down_tap_clamped(int n, int u, int len) {
    float s = (u >= 0 && u < len) ? (float)w5(u - 2 * n + 2) : 0.f;
    if (u == 0) s += w5_prefix(2 - 2 * n);                         // taps with 2n + t - 2 < 0
    if (u == len - 1) s += 1.f - w5_prefix(len + 2 - 2 * n);       // taps with 2n + t - 2 > len - 1
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

// Row-direction coefficient fragments of the border path (B operands; lane c = D row).
struct PyrCoef {
    half8 dy32;        // A_down, slots = rows 0..31 of the window (chained order)
    half8 d16;         // A_down for rows 32..35, in slots 8g + (0..3); zero in 8g + (4..7)
};

// One border task: a strip of NS blocks, nsteps output steps, anywhere in the image (D grid shift 8).
template <int NS, bool STREAM>
__device__ __forceinline__ void pyr_task(const PyrArgs& p, const PyrCoef& k, int X0, int R0, int nsteps, int c, int g) {
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

    // per D column tile, a pixel window moved inside the row and A_down fragments with the
    // column clamp folded in
    int wsx[NT];
    half8 fdx32[NT], fdx16[NT];
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

    half8 fux[NS][2];                                     // up-x fragments with the D column clamp folded in
#pragma unroll
    for (int t = 0; t < NS; ++t)
#pragma unroll
        for (int h = 0; h < 2; ++h) fux[t][h] = up_fragment_clamped(Dx0 + 16 * t, X0 + 32 * t + 16 * h, p.Wd, c, g);

    half8 win32[NT], nxt32[NT];
    half4 win16[NT], nxt16[NT];
    auto load_rows = [&](int r, half8 (&a32)[NT], half4 (&a16)[NT]) {
        const half_t* row = p.in + (int64_t)clampi(y00 + 16 * r + c, 0, p.H - 1) * p.in_pitch;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            a32[t] = *reinterpret_cast<const half8_u*>(row + wsx[t] + 8 * g);
            a16[t] = *reinterpret_cast<const half4_u*>(row + wsx[t] + 32 + 4 * g);
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
            acc = mfma16x16x32(win32[t], fdx32[t], acc);
            acc = mfma16x16x32(join(win16[t], z4), fdx16[t], acc);
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
                    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
                    acc = mfma16x16x32(join(D[t], D[t + 1]), fux[t][h], acc);
                    U1[1][t][h] = to_half4(acc);
                }
            if (q >= 1) {
                // pass 4: up along y for output rows R0 + 32 (q-1) + (0..31), then the residual
                const int Rq = R0 + 32 * (q - 1);
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2) {
                    const half8 b = up_fragment_clamped(M0 + 16 * (q - 1), Rq + 16 * h2, p.Hd, c, g);
                    const int yo = Rq + 16 * h2 + c;
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
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            win32[t] = nxt32[t];
            win16[t] = nxt16[t];
        }
    }
}

// ---------------------------------------------------------------------------
// Interior tasks.
//
// Coefficient fragments of the interior path (D grid shift 7, image column tiles of 32 pixels
// starting 16 left of the strip).  The two halves of a chained K = 32 operand live in one
// register quadruple that is filled alternately (tile r goes to half r % 2), so every second
// use sees the halves in swapped order and takes the fragment built for that order: no
// register is ever copied to line operands up.
struct PyrFastCoef {
    half8 dxa, dxb;    // A_down over image column tiles j and j + 1 (slot = pixel)
    half8 dy32;        // A_down over image row tiles r-2 | r-1 (chained slot order)
    half8 dy16;        // A_down for rows 32..35 in slots 8g + (0..3), zero in 8g + (4..7)
    half8 up[2];       // phase matrix of the first / second 16 outputs, operand halves (older | newer)
    half8 upsw[2];     // same for halves (newer | older)
    half8 sel[2];      // 0/1 selection (A operand): output column m <- tile pixel 16 + m / pixel m
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kBufFlags = 0x00020000;                     // raw buffer, 32-bit data format

__device__ __forceinline__ half4 lo4(half8 v) { return __builtin_shufflevector(v, v, 0, 1, 2, 3); }
__device__ __forceinline__ half4 hi4(half8 v) { return __builtin_shufflevector(v, v, 4, 5, 6, 7); }

constexpr int kPyrStashTile = 1024;                       // bytes per parked fragment: 64 lanes x 16
template <int NS>
struct PyrStash { static constexpr int kSlot = (NS + 1) * kPyrStashTile, kBytes = 3 * kSlot; };

// One interior task: a strip of NS blocks, nsteps (even) output steps, no image border in reach.
// Image row tile r holds rows R0 - 16 + 16 r + (0..15); image column tile j holds pixels
// X0 - 16 + 32 j + (0..31).  Tile loads are buffer loads: a wave-uniform descriptor of the
// task's footprint, one per-lane offset for the whole task, the row tile as scalar offset.
template <int NS, bool STREAM, bool DOWN>
__device__ __forceinline__ void pyr_fast_task(const PyrArgs& p, const PyrFastCoef& k, float* patch, char* stash,
                                              int X0, int R0, int nsteps, int lane) {
    constexpr int NT = NS + 1;                            // D column tiles per strip
    constexpr int NC = NS + 2;                            // image column tiles per strip
    constexpr int NB = 4;                                 // register ring of image row tiles (3 ahead)
    constexpr int NW = 2 * NS;                            // 16-column output tiles per row tile
    const int c = lane & 15, g = lane >> 4;
    const int Dx0 = X0 / 2 - 7, M0 = R0 / 2 - 7;          // first D column / row of tile 0

    // descriptors end with the image: an access past the last pixel would return zero / be dropped
    const int64_t in_left = ((int64_t)(p.H - 1 - (R0 - 16)) * p.in_pitch + (p.W - (X0 - 16))) * 2;
    const int64_t out_left = ((int64_t)(p.H - 1 - R0) * p.res_pitch + (p.W - X0)) * 4;
    const __amdgpu_buffer_rsrc_t rin = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<half_t*>(p.in + (int64_t)(R0 - 16) * p.in_pitch + (X0 - 16)), 0,
        (int)(in_left < 0x7fffffff ? in_left : 0x7fffffff), kBufFlags);
    const __amdgpu_buffer_rsrc_t rout = __builtin_amdgcn_make_buffer_rsrc(
        p.res + (int64_t)R0 * p.res_pitch + X0, 0, (int)(out_left < 0x7fffffff ? out_left : 0x7fffffff), kBufFlags);
    const uint32_t ivoff = (uint32_t)c * (uint32_t)p.in_pitch * 2u + 16u * g;
    // The last image column tile only feeds its first three pixels into a product (A_down of the last
    // D column); all four lanes of a row read its first eight pixels, so that a strip touches no
    // pixel beyond 24 past its last output.
    const uint32_t ivoff_last = (uint32_t)c * (uint32_t)p.in_pitch * 2u + 64u * (NC - 1);
    const uint32_t itile = 32u * (uint32_t)p.in_pitch;    // bytes per image row tile
    const uint32_t ovoff = ((uint32_t)g * (uint32_t)p.res_pitch + 4u * c) * 4u;
    const uint32_t orow4 = 16u * (uint32_t)p.res_pitch;   // bytes per four output rows
    const int ntiles = 2 * nsteps + 3;

    half8 W[NB][NC];                                      // image row tiles in flight / in use
    half8 TP[2][NT];                                      // row-filtered tiles: TP[a] = tiles (4i+2a | 4i+2a+1)
    half8 UP[NS][2];                                      // -(up-x results) of D row tiles (even q | odd q)
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int t = 0; t < NT; ++t) TP[a][t] = half8{0, 0, 0, 0, 0, 0, 0, 0};   // (finite: zero weights meet these)
#pragma unroll
    for (int t = 0; t < NS; ++t)
#pragma unroll
        for (int h = 0; h < 2; ++h) UP[t][h] = half8{0, 0, 0, 0, 0, 0, 0, 0};

    auto load_tile = [&](int r, half8 (&w)[NC]) {
        const uint32_t soff = (uint32_t)min(r, ntiles - 1) * itile;   // past the end: the last tile again
#pragma unroll
        for (int j = 0; j < NC - 1; ++j)
            w[j] = __builtin_bit_cast(half8, __builtin_amdgcn_raw_buffer_load_b128(rin, ivoff + 64u * j, soff, 0));
        w[NC - 1] = __builtin_bit_cast(half8, __builtin_amdgcn_raw_buffer_load_b128(rin, ivoff_last, soff, 0));
    };
    int sslot = 0;                                        // stash slot of the current tile: r % 3
    char* const mystash = stash + 16 * lane;

    // One image row tile.  S = r % 4 (compile time): ring slot of the tile, half of TP it fills.
    auto tile = [&](auto Stag, int r, __amdgpu_buffer_rsrc_t rdst) {
        constexpr int S = decltype(Stag)::value;
        // (no instruction may move between tiles: a product hoisted from a later tile would wait for
        // loads that are meant to stay in flight)
        __builtin_amdgcn_sched_barrier(0);
        load_tile(r + 3, W[(S + 3) % NB]);
        const half8 (&w)[NC] = W[S];
        // pass 1: down along x, all D column tiles
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
            acc = mfma16x16x32(w[t], k.dxa, acc);
            acc = mfma16x16x32(w[t + 1], k.dxb, acc);
            const half4 h = to_half4(acc);
            TP[S >> 1][t] = (S & 1) ? join(lo4(TP[S >> 1][t]), h) : join(h, hi4(TP[S >> 1][t]));
        }
        if constexpr ((S & 1) == 0) {
            const int q = r / 2 - 1;                      // D row tile completed by image tiles r-2 .. r
            constexpr int QO = (S == 0);                  // q is odd for S = 0, even for S = 2
            // pass 2: down along y (lane c = D row, four D columns)
            half4 D[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                floatx4 acc = {0.f, 0.f, 0.f, 0.f};
                acc = mfma16x16x32(TP[(S >> 1) ^ 1][t], k.dy32, acc);
                acc = mfma16x16x32(TP[S >> 1][t], k.dy16, acc);   // upper half: older rows, zero weights
                D[t] = to_half4(acc);
            }
            if constexpr (DOWN) {
                // each task writes the D samples under its own outputs
                const int m = M0 + 16 * q + c;
                if (m >= R0 / 2 && m < R0 / 2 + 16 * nsteps) {
                    half_t* drow = p.down + (int64_t)m * p.down_pitch;
#pragma unroll
                    for (int t = 0; t < NT; ++t)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int n = Dx0 + 16 * t + 4 * g + v;
                            if (n >= X0 / 2 && n < X0 / 2 + 16 * NS) drow[n] = D[t][v];
                        }
                }
            }
            // pass 3: up along x (lane c = output column, four D rows), sign flipped
#pragma unroll
            for (int t = 0; t < NS; ++t) {
                const half8 dd = join(D[t], D[t + 1]);
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
                    acc = mfma16x16x32(dd, k.up[h], acc);
                    const half4 u = to_half4(-acc);
                    UP[t][h] = QO ? join(lo4(UP[t][h]), u) : join(u, hi4(UP[t][h]));
                }
            }
            {
                // pass 4: parked pixels (tiles r-3, r-2) minus up along y, output rows 32 (q-1) + (0..31)
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2) {
                    const int sl = (sslot + h2 >= 3) ? sslot + h2 - 3 : sslot + h2;
                    const char* park = mystash + sl * PyrStash<NS>::kSlot;
                    half8 px[NT];
#pragma unroll
                    for (int j = 0; j < NT; ++j) px[j] = *reinterpret_cast<const half8*>(park + j * kPyrStashTile);
                    const half8 b = QO ? k.up[h2] : k.upsw[h2];
                    floatx4 rv[NW];
#pragma unroll
                    for (int t = 0; t < NS; ++t)
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
                            acc = mfma16x16x32(k.sel[h], px[t + h], acc);
                            acc = mfma16x16x32(UP[t][h], b, acc);
                            rv[2 * t + h] = acc;
                        }
                    // rows through the wave-private patch: 256-byte runs of one row per 16 lanes
#pragma unroll
                    for (int w2 = 0; w2 < NW; ++w2)
                        *reinterpret_cast<floatx4*>(patch + c * RowPatch<NW>::kPitch + 16 * w2 + 4 * g) = rv[w2];
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                    const uint32_t so = (uint32_t)(8 * (q - 1) + 4 * h2) * orow4;
#pragma unroll
                    for (int s4 = 0; s4 < 4; ++s4) {
                        const floatx4 v = *reinterpret_cast<const floatx4*>(patch + (4 * s4 + g) * RowPatch<NW>::kPitch + 4 * c);
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), rdst, ovoff,
                                                               so + (uint32_t)s4 * orow4, STREAM ? 2 : 0);
                    }
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                }
            }
        }
        // park this tile's fragments that lie under the outputs (read back three tiles later)
        {
            char* park = mystash + sslot * PyrStash<NS>::kSlot;
#pragma unroll
            for (int j = 0; j < NT; ++j) *reinterpret_cast<half8*>(park + j * kPyrStashTile) = w[j];
            sslot = (sslot == 2) ? 0 : sslot + 1;
        }
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;

    // Tiles run in rounds of four (ring slots 0..3); slots 0 and 2 complete a D row tile and store the
    // 32 output rows above it.  The first round has nothing to store yet: its stores go through a
    // descriptor of zero length, which the hardware drops.  Every round thereby issues the same
    // sequence of memory instructions, and so does the start-up below (loads, eight dropped stores,
    // loads): the compiler's counted waits then leave three tiles in flight instead of falling back
    // to the shortest path through the code.
    const __amdgpu_buffer_rsrc_t rnull = __builtin_amdgcn_make_buffer_rsrc(p.res, 0, 0, kBufFlags);
    load_tile(0, W[0]);
    load_tile(1, W[1]);
#pragma unroll
    for (int i = 0; i < 8; ++i)
        __builtin_amdgcn_raw_buffer_store_b128(u32x4{0u, 0u, 0u, 0u}, rnull, ovoff, 0, 0);
    load_tile(2, W[2]);
    for (int r = 0; r < ntiles; r += 4) {                 // tiles 0 .. 2 nsteps + 2, one spare at the end
        const __amdgpu_buffer_rsrc_t rdst = (r == 0) ? rnull : rout;
        tile(I0{}, r, rdst);
        tile(I1{}, r + 1, rdst);
        tile(I2{}, r + 2, rdst);
        tile(I3{}, r + 3, rdst);
    }
}

template <bool STREAM, bool DOWN>
__global__ void __launch_bounds__(256, 2) pyr_mfma_kernel(PyrArgs p) {
    constexpr int NS = HB_PYR_NS;
    const int lane = threadIdx.x & 63;
    const int c = lane & 15, g = lane >> 4;

    __shared__ __attribute__((aligned(16))) float s_patch[4][RowPatch<2 * NS>::kFloats];
    __shared__ __attribute__((aligned(16))) char s_stash[4][PyrStash<NS>::kBytes];

    // (of every 32 workgroups an XCD takes four neighbours: the waves in flight still sweep down the
    // image as one band, and neighbouring strips meet in one L2.  8192 x 8192: 91.4 us, plain launch
    // order 93.9, one contiguous eighth of the tasks per XCD, i.e. eight separate bands, 97)
    const int wgpos = xcd_blocked(blockIdx.x, gridDim.x, 4);
    const int wave = __builtin_amdgcn_readfirstlane(wgpos * 4 + (threadIdx.x >> 6));
    const int nwaves = (gridDim.x * blockDim.x) >> 6;
    const int ntasks = p.count();
    for (int task = wave; task < ntasks; task += nwaves) {
        if (task >= p.nborder) {
            PyrFastCoef k;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                k.dxa[i] = w5(8 * g + i - 2 * c);
                k.dxb[i] = w5(32 + 8 * g + i - 2 * c);
                k.dy32[i] = w5(krow32(g, i) - 2 * c);
                k.dy16[i] = (i < 4) ? w5(32 + 4 * g + i - 2 * c) : (half_t)0;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    k.up[h][i] = (half_t)upw(c & 1, krow32(g, i) - 7 - 8 * h - (c >> 1));
                    k.upsw[h][i] = (half_t)upw(c & 1, krow32(g, i ^ 4) - 7 - 8 * h - (c >> 1));
                }
                k.sel[0][i] = (half_t)((8 * g + i == 16 + c) ? 1.f : 0.f);
                k.sel[1][i] = (half_t)((8 * g + i == c) ? 1.f : 0.f);
            }
            const int id = task - p.nborder;
            const int seg = id / p.nci, ct = id - seg * p.nci;
            const int rs = p.r0 + seg * p.steps;
            pyr_fast_task<NS, STREAM, DOWN>(p, k, s_patch[threadIdx.x >> 6], s_stash[threadIdx.x >> 6],
                                            32 * (p.nbl + NS * ct), 32 * rs, min(p.steps, p.r1 - rs), lane);
        } else {
            PyrCoef k;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                k.dy32[i] = w5(krow32(g, i) - 2 * c);
                k.d16[i] = (i < 4) ? w5(32 + 4 * g + i - 2 * c) : (half_t)0;
            }
            int rs, blk, nst = 1;                         // one 32-column block, nst row steps
            if (task < p.ntop) {
                rs = task / p.nblk, blk = task - rs * p.nblk;
            } else if (task < p.ntop + p.nbot) {
                const int id = task - p.ntop;
                rs = id / p.nblk, blk = id - rs * p.nblk, rs += p.r1;
            } else {
                const int id = task - p.ntop - p.nbot;
                const int bi = id / p.nchunk, ch = id - bi * p.nchunk;
                blk = bi < p.nbl ? bi : p.bR + (bi - p.nbl);
                rs = p.r0 + kPyrBorderSteps * ch;
                nst = min(kPyrBorderSteps, p.r1 - rs);
            }
            pyr_task<1, STREAM>(p, k, 32 * blk, 32 * rs, nst, c, g);
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
    constexpr int SW = 32 * HB_PYR_NS;                    // interior strip width
    a.nblk = ceil_div(W, 32);
    a.rowsteps = ceil_div(H, 32);
    // interior: a task reads pixels from 16 before its first output to 32 past its last one (24 along
    // x), in both directions; then no up pass reads a clamped D index either.  One border block on
    // the left; on the right whatever the strips leave.
    a.nbl = 1;
    a.nci = (W - 32 - 32 >= SW) ? (W - 32 - 32) / SW : 0;
    a.bR = a.nbl + HB_PYR_NS * a.nci;
    a.r0 = 1;
    a.r1 = (H - 64 >= 0) ? (H - 64) / 32 + 1 : 0;        // last interior step e: 32 e + 32 + 32 <= H
    if ((a.r1 - a.r0) & 1) --a.r1;                        // interior tasks take two row steps per round
    // a task's footprint must stay below 2 GiB from its first row (32-bit buffer offsets)
    const int64_t rowbytes = in_pitch * 2 > res_pitch * 4 ? in_pitch * 2 : res_pitch * 4;
    const int64_t maxrows = (((int64_t)1 << 31) - 1) / rowbytes;
    // the interior path reads with 16-byte buffer loads: rows must start on 4-byte boundaries
    const bool dword_rows = (in_pitch % 2 == 0) && (reinterpret_cast<uintptr_t>(in) % 4 == 0);
    if (!dword_rows || maxrows < 2 * 32 + 64 || a.nci <= 0 || a.r1 <= a.r0) {   // no interior: everything is "top"
        a.nci = 0;
        a.nbl = a.bR = a.nblk;
        a.r0 = a.r1 = a.rowsteps;
    }
    const int nr = a.r1 - a.r0;
    int steps = 2 * (int)(((int64_t)nr * a.nci + 2 * HB_PYR_WAVES - 1) / (2 * HB_PYR_WAVES));
    if ((int64_t)32 * steps + 64 > maxrows) steps = (int)((maxrows - 64) / 64) * 2;
    a.steps = steps < 2 ? 2 : steps;
    a.nseg = a.nci > 0 ? ceil_div(nr, a.steps) : 0;
    a.nchunk = ceil_div(nr, kPyrBorderSteps);
    a.ntop = a.r0 * a.nblk;
    a.nbot = (a.rowsteps - a.r1) * a.nblk;
    a.nborder = a.ntop + a.nbot + (nr > 0 ? (a.nbl + a.nblk - a.bR) * a.nchunk : 0);
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
    const dim3 grid(min(ceil_div(a.count(), 4), kMaxStreamBlocks));
    const bool stream_stores = (int64_t)H * W * 4 <= kStreamStoreMaxBytes;
    if (a.down) {
        if (stream_stores) hipLaunchKernelGGL((pyr_mfma_kernel<true, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((pyr_mfma_kernel<false, true>), grid, dim3(256), 0, st, a);
    } else {
        if (stream_stores) hipLaunchKernelGGL((pyr_mfma_kernel<true, false>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((pyr_mfma_kernel<false, false>), grid, dim3(256), 0, st, a);
    }
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
