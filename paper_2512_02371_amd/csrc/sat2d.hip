// hb_sat2d: summed-area table.  Per 64 x 64 tile the table is L * X * U (L, U triangular
// all-ones); between tiles it needs carries, as the tiled recursive filter of Sec. V-D
// (tile, then fix up): three launches,
//   1 sums    per tile: row sums (X * 1) and column sums (1^T * X)                    read 2 B/px
//   2 scan    exclusive scans of those sums along the tile grid                       (tiny)
//   3 apply   per tile: row prefix X * U on the matrix units seeded with the row carry,
//             column prefix with the column carry, store                              read 2 + write 4 B/px
// so that  S[i][j] = P(i0-1, j) + sum_{y=i0..i} ( R(y) + sum_{x=j0..j} in[y][x] )
// with R(y) = sum of row y left of the tile and P(i0-1, j) the table value above the tile.
//
// MFMA formulation of the apply pass, transposed so that a lane ends with four consecutive
// columns of one row:
//   Z'[m][n] = sum_k Ut[m][k] * Xt[k][n] + R[n]      m = column, n = row, k = pixel in a 32-block
//   Ut[m][k] = 1 for k <= m (+16 for the second 16 columns), so one 16-byte pixel load feeds both
//   halves; a third product with the all-ones matrix yields the block's row totals in every lane,
//   which advance the row carry.  The 0/1 coefficients and fp16 pixels make every product exact;
//   sums are fp32.  The column prefix runs over the 16 rows that sit in the 16 lanes of a DPP row
//   (four shifted adds), the column carry is the prefix value of the last row.
//   The sums pass uses the same operands: X * 1 for row sums; X * [I|0], X * [0|I] copy the pixels
//   into accumulator layout (exactly), whose stacked pairs times the all-ones matrix give column
//   sums.  No cross-lane traffic in that pass at all.
#include <atomic>

#include "hb_device.hpp"
#include "hb_host.hpp"

namespace hb {

constexpr int kSatTile = 64;
constexpr int kMaxDevices = 64;

struct SatArgs {
    const half_t* in;
    float* out;
    int H, W;
    int64_t in_pitch, out_pitch;
    int nb, ns;            // 64-column strips, 64-row segments
    int Hs, Ws;            // H, W rounded up to whole tiles (workspace row lengths)
    // all tables keep the scanned index innermost, so that a scan is one coalesced wave access
    float* rs;             // [Hs][nb]  row sums per (row, strip)
    float* cs;             // [Ws][ns]  column sums per (column, segment)
    float* tot;            // [nb][ns]  tile totals per (strip, segment)
    float* rcarry;         // [Hs][nb]  exclusive scan of rs over strips
    float* ccarry;         // [Ws][ns]  exclusive scan of cs over segments
    float* es;             // [nb][ns]  exclusive scan of tot over segments
};

// Eight pixels row[xs .. xs+7], zero where the row or the column is outside the image.
__device__ __forceinline__ half8 load8_zero(const half_t* in, int64_t pitch, int y, int xs, int H, int W) {
    half8 r = {0, 0, 0, 0, 0, 0, 0, 0};
    if (y < H) {
        const half_t* row = in + (int64_t)y * pitch;
        if (xs + 8 <= W) {
            r = *reinterpret_cast<const half8_u*>(row + xs);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (xs + i < W) r[i] = row[xs + i];
        }
    }
    return r;
}

__device__ __forceinline__ half8 ones8() { return half8{1, 1, 1, 1, 1, 1, 1, 1}; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}


// ---------------------------------------------------------------------------
// 1  sums
__global__ void __launch_bounds__(256) sat_sums_mfma_kernel(SatArgs p) {
    const int lane = threadIdx.x & 63;
    const int c = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane((blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    if (wave >= p.nb * p.ns) return;
    const int s = wave / p.nb, b = wave - s * p.nb;
    const int y0 = kSatTile * s, x0 = kSatTile * b;

    half8 sel[2];                                         // B[k][n] = (k == 16 half + n)
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int i = 0; i < 8; ++i) sel[h][i] = (half_t)((8 * g + i == 16 * h + c) ? 1.f : 0.f);
    const half8 one = ones8();

    half8 X[4][2];                                        // all eight loads of the tile in flight at once
    if (y0 + kSatTile <= p.H && x0 + kSatTile <= p.W) {
        const half_t* src = p.in + (int64_t)y0 * p.in_pitch + x0;
        const uint32_t off = ((uint32_t)c * (uint32_t)p.in_pitch + 8u * g) * 2u;
#pragma unroll
        for (int rt = 0; rt < 4; ++rt)
#pragma unroll
            for (int blk = 0; blk < 2; ++blk)
                X[rt][blk] = ldg8(src + (int64_t)(16 * rt) * p.in_pitch, off + 64u * blk);   // 64-bit base per 16 rows
    } else {
#pragma unroll
        for (int rt = 0; rt < 4; ++rt)
#pragma unroll
            for (int blk = 0; blk < 2; ++blk)
                X[rt][blk] = load8_zero(p.in, p.in_pitch, y0 + 16 * rt + c, x0 + 32 * blk + 8 * g, p.H, p.W);
    }

    // Row tiles in pairs: row sums (X * 1), pixel copies in accumulator layout (X * [I|0], X * [0|I]),
    // whose stacked pairs times the all-ones matrix add up the column sums.
    floatx4 colsum[2][2];
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int h = 0; h < 2; ++h) colsum[blk][h] = floatx4{0.f, 0.f, 0.f, 0.f};
    float tile_total = 0.f;
#pragma unroll
    for (int rp = 0; rp < 2; ++rp) {
        half4 T[2][2][2];                                 // pixel copies of row tiles 2 rp, 2 rp + 1
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int rt = 2 * rp + u;
            floatx4 rowsum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int blk = 0; blk < 2; ++blk) {
                rowsum = mfma16x16x32(X[rt][blk], one, rowsum);              // [m = row][n]: row totals in every column
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    floatx4 t = {0.f, 0.f, 0.f, 0.f};
                    T[u][blk][h] = to_half4(mfma16x16x32(X[rt][blk], sel[h], t));   // [m = row][n = column]
                }
            }
            // lane (c, g) holds the sums of rows 4g + v, the same in every c: lanes c < 4 write row 4g + c
            const float mine = c == 0 ? rowsum[0] : c == 1 ? rowsum[1] : c == 2 ? rowsum[2] : rowsum[3];
            if (c < 4) p.rs[(int64_t)(y0 + 16 * rt + 4 * g + c) * p.nb + b] = mine;
            tile_total += rowsum[0] + rowsum[1] + rowsum[2] + rowsum[3];     // used from lanes c = 0 only
        }
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                colsum[blk][h] = mfma16x16x32(join(T[0][blk][h], T[1][blk][h]), one, colsum[blk][h]);   // [m = column][n]
    }
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const floatx4 cs = colsum[blk][h];
            const float mine = c == 0 ? cs[0] : c == 1 ? cs[1] : c == 2 ? cs[2] : cs[3];
            if (c < 4) p.cs[(int64_t)(x0 + 32 * blk + 16 * h + 4 * g + c) * p.ns + s] = mine;
        }
    // tile total: the four lane groups' partial row-sum totals
    tile_total = (c == 0) ? tile_total : 0.f;
    tile_total = wave_sum(tile_total);
    if (lane == 0) p.tot[(int64_t)b * p.ns + s] = tile_total;
}

// ---------------------------------------------------------------------------
// 2  scans.  One wave per line, one lane per element, 64 elements at a time with a running carry:
// waves [0, Hs): image row y, exclusive scan of rs[y][.] over strips;
// waves [Hs, Hs + Ws): image column x, exclusive scan of cs[x][.] over segments;
// waves [Hs + Ws, Hs + Ws + nb): strip b, exclusive scan of tot[b][.] over segments (what lies
// above-left of a tile is the sum of these over the strips to its left).
__device__ __forceinline__ void wave_exclusive_scan_line(const float* __restrict__ src, float* __restrict__ dst,
                                                         int n, int lane) {
    float carry = 0.f;
    for (int i0 = 0; i0 < n; i0 += 64) {
        const int i = i0 + lane;
        const float v = (i < n) ? src[i] : 0.f;
        float x = v;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const float t = __shfl_up(x, off, 64);
            if (lane >= off) x += t;
        }
        if (i < n) dst[i] = carry + x - v;
        carry += __shfl(x, 63, 64);
    }
}

__global__ void __launch_bounds__(256) sat_scan_kernel(SatArgs p) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    if (wave < p.Hs) {
        wave_exclusive_scan_line(p.rs + (int64_t)wave * p.nb, p.rcarry + (int64_t)wave * p.nb, p.nb, lane);
    } else if (wave < p.Hs + p.Ws) {
        const int x = wave - p.Hs;
        wave_exclusive_scan_line(p.cs + (int64_t)x * p.ns, p.ccarry + (int64_t)x * p.ns, p.ns, lane);
    } else if (wave < p.Hs + p.Ws + p.nb) {
        const int b = wave - p.Hs - p.Ws;
        wave_exclusive_scan_line(p.tot + (int64_t)b * p.ns, p.es + (int64_t)b * p.ns, p.ns, lane);
    }
}

// ---------------------------------------------------------------------------
// 3  apply
__device__ __forceinline__ float dpp_row_shr(float v, int n) {
    // lane i of each 16-lane row receives lane i - n of the same row, 0 where there is none
    int r;
    switch (n) {
        case 1: r = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x111, 0xf, 0xf, true); break;
        case 2: r = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x112, 0xf, 0xf, true); break;
        case 4: r = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x114, 0xf, 0xf, true); break;
        default: r = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x118, 0xf, 0xf, true); break;
    }
    return __builtin_bit_cast(float, r);
}

// Table row above the tile: P(i0 - 1, x0 + lane) = everything above-left of the tile plus the
// prefix over this strip's columns of the column carries.
__device__ __forceinline__ float sat_row_above(const SatArgs& p, int s, int b, int lane) {
    float above = 0.f;
    for (int b0 = 0; b0 < b; b0 += 64)
        if (b0 + lane < b) above += p.es[(int64_t)(b0 + lane) * p.ns + s];
    above = wave_sum(above);
    float colp = p.ccarry[(int64_t)(kSatTile * b + lane) * p.ns + s];
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const float t = __shfl_up(colp, off, 64);
        if (lane >= off) colp += t;
    }
    return colp + above;
}

template <bool STREAM>
__global__ void __launch_bounds__(256) sat_apply_mfma_kernel(SatArgs p) {
    __shared__ __attribute__((aligned(16))) float s_patch[4][RowPatch<4>::kFloats];
    const int lane = threadIdx.x & 63;
    const int c = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane((blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    if (wave >= p.nb * p.ns) return;
    const int s = wave / p.nb, b = wave - s * p.nb;
    const int y0 = kSatTile * s, x0 = kSatTile * b;
    const bool full = (y0 + kSatTile <= p.H) && (x0 + kSatTile <= p.W);

    // all eight pixel loads and the four row carries of the tile go out first
    half8 X[4][2];
    float r0[4];
    if (full) {
        const half_t* src = p.in + (int64_t)y0 * p.in_pitch + x0;
        const uint32_t off = ((uint32_t)c * (uint32_t)p.in_pitch + 8u * g) * 2u;
#pragma unroll
        for (int rt = 0; rt < 4; ++rt)
#pragma unroll
            for (int blk = 0; blk < 2; ++blk)
                X[rt][blk] = ldg8(src + (int64_t)(16 * rt) * p.in_pitch, off + 64u * blk);   // 64-bit base per 16 rows
    } else {
#pragma unroll
        for (int rt = 0; rt < 4; ++rt)
#pragma unroll
            for (int blk = 0; blk < 2; ++blk)
                X[rt][blk] = load8_zero(p.in, p.in_pitch, y0 + 16 * rt + c, x0 + 32 * blk + 8 * g, p.H, p.W);
    }
#pragma unroll
    for (int rt = 0; rt < 4; ++rt) r0[rt] = p.rcarry[(int64_t)(y0 + 16 * rt + c) * p.nb + b];

    // A operands: Ut[m][k] = (k <= m + 16 half): lane (c = m, g) holds k = 8g .. 8g+7
    half8 tri[2];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int i = 0; i < 8; ++i) tri[h][i] = (half_t)((8 * g + i <= c + 16 * h) ? 1.f : 0.f);
    const half8 one = ones8();

    const float colp = sat_row_above(p, s, b, lane);
    floatx4 ccar[4];                                      // lane (c, g): columns 16 t + 4g + v
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) ccar[t][v] = __shfl(colp, 16 * t + 4 * g + v, 64);

#pragma unroll
    for (int rt = 0; rt < 4; ++rt) {
        floatx4 rc = {r0[rt], r0[rt], r0[rt], r0[rt]};    // row carry of row c, the same in all four columns
        floatx4 acc[4];
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
            acc[2 * blk] = mfma16x16x32(tri[0], X[rt][blk], rc);      // [m = column][n = row]: lane c = row, columns 4g + v
            acc[2 * blk + 1] = mfma16x16x32(tri[1], X[rt][blk], rc);
            rc = mfma16x16x32(one, X[rt][blk], rc);                   // row carry advanced by the block's row totals
        }
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float x = acc[t][v];                      // inclusive prefix over the 16 rows of the DPP row
                x += dpp_row_shr(x, 1);
                x += dpp_row_shr(x, 2);
                x += dpp_row_shr(x, 4);
                x += dpp_row_shr(x, 8);
                x += ccar[t][v];
                acc[t][v] = x;
                ccar[t][v] = __shfl(x, (lane & 48) | 15, 64);         // value of the last row = next column carry
            }
        if (full) {
            store_rows_via_lds<4, STREAM>(s_patch[threadIdx.x >> 6], p.out + (int64_t)(y0 + 16 * rt) * p.out_pitch + x0,
                                          (uint32_t)p.out_pitch, acc, lane);
        } else {
            const int y = y0 + 16 * rt + c;
            if (y < p.H) {
                float* orow = p.out + (int64_t)y * p.out_pitch;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int xo = x0 + 16 * t + 4 * g;
                    if (xo < p.W) store4_mask(orow, xo, p.W, acc[t]);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// One launch for images whose tiles are all resident at once: the image is read ONCE.
//
// A workgroup of TR x TC waves owns a region of TR x TC tiles.  Before the grid-wide wait every
// wave loads its tile and turns it into the tile's LOCAL table Lt (row prefix on the matrix units,
// column prefix over the lanes), which stays in registers.  For a pixel (i, j) of a tile with
// origin (i0, j0)
//     S[i][j] = Lt[i-i0][j-j0] + R[i] + C[j] + A
//     R[i] = sum over the tiles to the left, in the same tile row, of the LAST COLUMN of their local table at row i
//     C[j] = sum over the tiles above, in the same tile column, of the LAST ROW of their local table at column j
//     A    = sum of everything above-left of the tile
// so what a tile has to publish is the last row and last column of its local table.  The
// workgroup adds those up over its region (prefixes restart at every tile border) and publishes
// RS[region column][row], CS[region row][column] and TOT[region]; one grid-wide wait; then it adds
// up the table lines of the regions to its left and above (coalesced 1 KB lines, few of them
// because regions are large), finishes R, C and A of its tiles through LDS, and what is left per
// pixel after the wait is two additions and the store.  The heavy arithmetic sits before the wait,
// where it overlaps with the loads of the other waves.
//
// Grid-wide wait.  Arrival is a two-level count (up to 16 leaf counters, one root, each on its own
// 128-byte line: arrivals at one address are served one after the other by the memory side); the
// last arrival raises eight copies of a `go` word and workgroup w polls copy w % 8.  Table data and
// the words of the wait are written and read with agent-scope accesses (they bypass the per-XCD L2,
// so no cache write-back or invalidation is needed; a write-back per workgroup costs ~20 ns each,
// one after the other).  The wait is BOUNDED: after `wait_limit` polls a workgroup stops waiting.
// It has already arrived, so the count still completes when the last workgroup gets to run; a
// workgroup that stopped waiting marks its region in `todo`, raises `late` and leaves, unless `go`
// came up meanwhile.  Every workgroup that passes the wait reads `late` (raised before `go` by
// construction, see below) and, if it is set, claims marked regions one by one, reloads their
// pixels and finishes them.  So every wave exits whatever the residency, and every region is
// finished by someone:
//   late workgroup: store todo[r], late; wait for the stores; load go.  go == 0 -> leave.
//   finisher:       observes go == 1; then loads late and todo.
//   go is raised once, after the late workgroup's load returned 0, hence after its stores were
//   performed at the memory side: the finisher's loads see them.
// The host uses this kernel only when the grid fits on the device at once (occupancy query), so the
// bounded wait ends by `go` unless other work holds compute units for longer than the limit.
#ifndef HB_SAT_POLL_SLEEP
#define HB_SAT_POLL_SLEEP 3                               // s_sleep units (64 clocks each) between two polls of `go`
#endif
struct SatSync {
    static constexpr int kLine = 32;                      // words per 128 bytes
    static constexpr int kLeaves = 16, kGo = 8, kMaxRegions = 1024;
    unsigned leaf[kLeaves * kLine];
    unsigned root[kLine];
    unsigned go[kGo * kLine];
    unsigned late[kLine];
    unsigned todo[kMaxRegions];                           // 0 idle, 1 waiting for a finisher, 2 claimed
#ifdef HB_SAT_TIMING
    unsigned long long stamp[kMaxRegions][8];             // measurement builds only: phase time stamps per workgroup
#endif
};
#ifdef HB_SAT_TIMING
#define SAT_STAMP(S, wg, i) do { if (threadIdx.x == 0) (S)->stamp[wg][i] = wall_clock64(); } while (0)
#else
#define SAT_STAMP(S, wg, i) do { } while (0)
#endif

struct SatFusedArgs {
    const half_t* in;
    float* out;
    int H, W;
    int64_t in_pitch, out_pitch;
    int nsw, nbw;          // regions down, across
    int Hr, Wr;            // H, W rounded up to whole regions
    float* RS;             // [nbw][Hr]  row y: sum over the columns of region column bw of the rows from its tile row's top to y
    float* CS;             // [nsw][Wr]  column x: sum over the rows of region row sw of the columns from its tile column's left to x
    float* TOT;            // [nsw][nbw] region totals
    SatSync* sync;
    int wait_limit;
};

__device__ __forceinline__ unsigned ld_agent(const unsigned* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(unsigned* p, unsigned v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ldf_agent(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void stf_agent(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// all earlier stores of this lane performed, and no memory access moved across this point
__device__ __forceinline__ void stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__global__ void __launch_bounds__(256) sat_sync_clear_kernel(SatSync* s) {
    unsigned* w = reinterpret_cast<unsigned*>(s);
    constexpr int kWords = (SatSync::kLeaves + 1 + SatSync::kGo + 1) * SatSync::kLine + SatSync::kMaxRegions;
    for (int i = threadIdx.x; i < kWords; i += 256) w[i] = 0u;
}

template <int TR, int TC>
struct SatFusedLds {
    static constexpr int kWaves = TR * TC;
    static constexpr int kRH = kSatTile * TR, kRW = kSatTile * TC;
    // (members that are accessed 16 bytes at a time come first and are sized in multiples of 16 bytes:
    // a misaligned 16-byte LDS access is split and runs at a fraction of the rate)
    float patch[kWaves][RowPatch<4>::kFloats];            // store patches
    union {
        struct { float r[kWaves][kRH]; float c[kWaves][kRW]; } part;    // per-wave partial sums of table lines
        struct { float row[kWaves][kSatTile]; float col[kWaves][kSatTile]; } term;   // R and C + A of every wave's tile
    } u;
    float lastrow[TR][TC][kSatTile];                      // per tile: last row of its local table
    float lastcol[TR][TC][kSatTile];                      // per tile: last column of its local table (prefix over its rows of the row sums)
    float Rc[kRH];                                        // per region row: the RS lines of the regions to the left, added up
    float Cc[kRW];                                        // per region column: the CS lines of the regions above, added up
    float Apart[kWaves];
    float A;                                              // sum of everything above-left of the region
    int ctl;
};
static_assert(RowPatch<4>::kFloats % 4 == 0, "patches stay 16-byte aligned");

// Before the wait, per wave: load the tile and build its local table in registers; its last row,
// last column (and so its total) go to LDS.  Lt[rt][t]: lane (c, g) holds row 16 rt + c, columns 16 t + 4 g + v.
template <int TR, int TC>
__device__ __forceinline__ void sat_fused_local(const SatFusedArgs& p, SatFusedLds<TR, TC>& L,
                                                int y0, int x0, int ts, int tb, int lane, floatx4 (&Lt)[4][4]) {
    const int c = lane & 15, g = lane >> 4;
    half8 X[4][2];
    if (y0 + kSatTile <= p.H && x0 + kSatTile <= p.W) {
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) {
            const half_t* src = p.in + (int64_t)(y0 + 16 * rt) * p.in_pitch + x0;       // 64-bit base per 16 rows
            const uint32_t off = ((uint32_t)c * (uint32_t)p.in_pitch + 8u * g) * 2u;
#pragma unroll
            for (int blk = 0; blk < 2; ++blk) X[rt][blk] = ldg8(src, off + 64u * blk);
        }
    } else {
#pragma unroll
        for (int rt = 0; rt < 4; ++rt)
#pragma unroll
            for (int blk = 0; blk < 2; ++blk)
                X[rt][blk] = load8_zero(p.in, p.in_pitch, y0 + 16 * rt + c, x0 + 32 * blk + 8 * g, p.H, p.W);
    }
    half8 tri[2];                                         // Ut[m][k] = (k <= m + 16 half)
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int i = 0; i < 8; ++i) tri[h][i] = (half_t)((8 * g + i <= c + 16 * h) ? 1.f : 0.f);
    const half8 one = ones8();
    floatx4 ccar[4];                                      // running column sums: lane (c, g), columns 16 t + 4 g + v
#pragma unroll
    for (int t = 0; t < 4; ++t) ccar[t] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int rt = 0; rt < 4; ++rt) {
        const floatx4 zero = {0.f, 0.f, 0.f, 0.f};
        Lt[rt][0] = mfma16x16x32(tri[0], X[rt][0], zero);             // [m = column][n = row]: lane c = row, columns 4g + v
        Lt[rt][1] = mfma16x16x32(tri[1], X[rt][0], zero);
        const floatx4 left = mfma16x16x32(one, X[rt][0], zero);       // the row's total over the first 32 columns
        Lt[rt][2] = mfma16x16x32(tri[0], X[rt][1], left);
        Lt[rt][3] = mfma16x16x32(tri[1], X[rt][1], left);
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float x = Lt[rt][t][v];                   // inclusive prefix over the 16 rows of the DPP row
                x += dpp_row_shr(x, 1);
                x += dpp_row_shr(x, 2);
                x += dpp_row_shr(x, 4);
                x += dpp_row_shr(x, 8);
                x += ccar[t][v];
                Lt[rt][t][v] = x;
                ccar[t][v] = __shfl(x, (lane & 48) | 15, 64);         // value of the last row = next column carry
            }
        if (g == 3) L.lastcol[ts][tb][16 * rt + c] = Lt[rt][3][3];    // column 63 of row 16 rt + c
    }
    if (c == 0) {
#pragma unroll
        for (int t = 0; t < 4; ++t) *reinterpret_cast<floatx4*>(&L.lastrow[ts][tb][16 * t + 4 * g]) = ccar[t];
    }
}

// After the wait, for the whole workgroup (every wave's local table in Lt): carries, two additions per pixel, store.
template <int TR, int TC, bool STREAM>
__device__ __forceinline__ void sat_fused_finish(const SatFusedArgs& p, SatFusedLds<TR, TC>& L,
                                                 int sw, int bw, int wv, int lane, floatx4 (&Lt)[4][4]) {
    using LT = SatFusedLds<TR, TC>;
    constexpr int kWaves = LT::kWaves, kRH = LT::kRH, kRW = LT::kRW, kThreads = 64 * kWaves;
    const int c = lane & 15, g = lane >> 4;
    const int ts = wv / TC, tb = wv - ts * TC;
    const int I0 = kRH * sw, J0 = kRW * bw;
    const int tid = wv * 64 + lane;

    // table lines of the regions to the left (RS) and above (CS): wave w takes lines w, w + kWaves, ...
    {
        float ar[kRH / 64], ac[kRW / 64];
#pragma unroll
        for (int k = 0; k < kRH / 64; ++k) ar[k] = 0.f;
#pragma unroll
        for (int k = 0; k < kRW / 64; ++k) ac[k] = 0.f;
        for (int b2 = wv; b2 < bw; b2 += kWaves) {
            const float* line = p.RS + (int64_t)b2 * p.Hr + I0;
#pragma unroll
            for (int k = 0; k < kRH / 64; ++k) ar[k] += ldf_agent(line + 64 * k + lane);
        }
        for (int s2 = wv; s2 < sw; s2 += kWaves) {
            const float* line = p.CS + (int64_t)s2 * p.Wr + J0;
#pragma unroll
            for (int k = 0; k < kRW / 64; ++k) ac[k] += ldf_agent(line + 64 * k + lane);
        }
        float a = 0.f;
        for (int i = tid; i < sw * bw; i += kThreads) {
            const int s2 = i / bw, b2 = i - s2 * bw;
            a += ldf_agent(p.TOT + (int64_t)s2 * p.nbw + b2);
        }
#pragma unroll
        for (int k = 0; k < kRH / 64; ++k) L.u.part.r[wv][64 * k + lane] = ar[k];
#pragma unroll
        for (int k = 0; k < kRW / 64; ++k) L.u.part.c[wv][64 * k + lane] = ac[k];
        a = wave_sum(a);
        if (lane == 0) L.Apart[wv] = a;
    }
    __syncthreads();
    if (tid < kRH) {
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) v += L.u.part.r[w][tid];
        L.Rc[tid] = v;
    } else if (tid < kRH + kRW) {
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) v += L.u.part.c[w][tid - kRH];
        L.Cc[tid - kRH] = v;
    }
    if (tid == kThreads - 1) {
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) v += L.Apart[w];
        L.A = v;
    }
    __syncthreads();

    // this wave's tile: R for row `lane`, C + A for column `lane`
    float R = L.Rc[kSatTile * ts + lane];
    for (int b2 = 0; b2 < tb; ++b2) R += L.lastcol[ts][b2][lane];
    float C = L.Cc[kSatTile * tb + lane];
    for (int t2 = 0; t2 < ts; ++t2) C += L.lastrow[t2][tb][lane];
    float A = L.A;
    for (int k = 0; k < tb; ++k) A += L.Cc[kSatTile * k + kSatTile - 1];      // above the region, tile columns to the left
    for (int k = 0; k < ts; ++k) A += L.Rc[kSatTile * k + kSatTile - 1];      // left of the region, tile rows above
    for (int t2 = 0; t2 < ts; ++t2)
        for (int b2 = 0; b2 < tb; ++b2) A += L.lastrow[t2][b2][kSatTile - 1]; // inside the region, tiles above-left
    L.u.term.row[wv][lane] = R;                           // (the parts were last read before the barrier above)
    L.u.term.col[wv][lane] = C + A;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    SAT_STAMP(p.sync, sw * p.nbw + bw, 4);

    const int y0 = I0 + kSatTile * ts, x0 = J0 + kSatTile * tb;
    const bool full = (y0 + kSatTile <= p.H) && (x0 + kSatTile <= p.W);
    if (y0 >= p.H || x0 >= p.W) return;                   // tile outside the image: nothing to store (no barrier follows)
    floatx4 ct[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) ct[t] = *reinterpret_cast<const floatx4*>(&L.u.term.col[wv][16 * t + 4 * g]);
#pragma unroll
    for (int rt = 0; rt < 4; ++rt) {
        const float r = L.u.term.row[wv][16 * rt + c];
        floatx4 acc[4];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[t][v] = Lt[rt][t][v] + (r + ct[t][v]);
        if (full) {
            store_rows_via_lds<4, STREAM>(L.patch[wv], p.out + (int64_t)(y0 + 16 * rt) * p.out_pitch + x0,
                                          (uint32_t)p.out_pitch, acc, lane);
        } else {
            const int y = y0 + 16 * rt + c;
            if (y < p.H) {
                float* orow = p.out + (int64_t)y * p.out_pitch;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int xo = x0 + 16 * t + 4 * g;
                    if (xo < p.W) store4_mask(orow, xo, p.W, acc[t]);
                }
            }
        }
    }
}

extern __shared__ __attribute__((aligned(16))) unsigned char s_sat_fused_lds[];

template <int TR, int TC, bool STREAM>
__global__ void __launch_bounds__(64 * TR * TC) sat_fused_kernel(SatFusedArgs p) {
    using LT = SatFusedLds<TR, TC>;
    constexpr int kWaves = LT::kWaves, kRH = LT::kRH, kRW = LT::kRW;
    LT& L = *reinterpret_cast<LT*>(s_sat_fused_lds);
    const int nwg = p.nsw * p.nbw;
    const int wg = blockIdx.x;
    SatSync* S = p.sync;

    // The first turn of this loop is the workgroup's own region (local tables, publish, arrive, wait,
    // finish).  Further turns run only in a finisher, on regions whose workgroups stopped waiting
    // (reload, local tables, finish).  `region` and `own` are the same in every lane.
    int region = wg;
    bool own = true;
    SAT_STAMP(S, wg, 0);
    for (;;) {
        // Lane-derived values (LDS addresses, per-lane offsets, the 0/1 operand fragments) are made to
        // look new in every turn: hoisted out of the loop they would stay live through it all, about
        // ninety registers, and push the kernel over the 128 its 16 waves per compute unit allow.
        int tid = threadIdx.x;
        asm volatile("" : "+v"(tid));
        const int lane = tid & 63;
        const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
        const int ts = wv / TC, tb = wv - ts * TC;
        const int sw = region / p.nbw, bw = region - sw * p.nbw;
        floatx4 Lt[4][4];
        sat_fused_local<TR, TC>(p, L, kRH * sw + kSatTile * ts, kRW * bw + kSatTile * tb, ts, tb, lane, Lt);
        __syncthreads();
        unsigned late = 0u;
        if (own) {
            SAT_STAMP(S, wg, 1);
            // publish the region's sums: the tiles' last columns added across a tile row, last rows down a tile column
            if (tid < kRH) {
                const int t2 = tid >> 6, y = tid & 63;
                float v = 0.f;
#pragma unroll
                for (int b2 = 0; b2 < TC; ++b2) v += L.lastcol[t2][b2][y];
                stf_agent(p.RS + (int64_t)bw * p.Hr + kRH * sw + tid, v);
            } else if (tid < kRH + kRW) {
                const int x = tid - kRH, b2 = x >> 6;
                float v = 0.f;
#pragma unroll
                for (int t2 = 0; t2 < TR; ++t2) v += L.lastrow[t2][b2][x & 63];
                stf_agent(p.CS + (int64_t)sw * p.Wr + kRW * bw + x, v);
            }
            if (tid == 64 * kWaves - 1) {
                float v = 0.f;
#pragma unroll
                for (int t2 = 0; t2 < TR; ++t2)
#pragma unroll
                    for (int b2 = 0; b2 < TC; ++b2) v += L.lastrow[t2][b2][kSatTile - 1];
                stf_agent(p.TOT + wg, v);
            }
            stores_done();
            __syncthreads();
            SAT_STAMP(S, wg, 2);
            // arrive, then wait (bounded) for the others
            if (tid == 0) {
                const int nleaf = nwg < SatSync::kLeaves ? nwg : SatSync::kLeaves;
                const int lf = wg % nleaf;
                const int leaf_target = (nwg - lf + nleaf - 1) / nleaf;
                const unsigned old = __hip_atomic_fetch_add(&S->leaf[SatSync::kLine * lf], 1u, __ATOMIC_RELAXED,
                                                            __HIP_MEMORY_SCOPE_AGENT);
                if ((int)old + 1 == leaf_target) {
                    const unsigned r = __hip_atomic_fetch_add(&S->root[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if ((int)r + 1 == nleaf) {
#pragma unroll
                        for (int i = 0; i < SatSync::kGo; ++i) st_agent(&S->go[SatSync::kLine * i], 1u);
                    }
                }
                const unsigned* mygo = &S->go[SatSync::kLine * (wg & (SatSync::kGo - 1))];
                int state = 1;                            // 1 passed, 0 leave
                int polls = 0;
                while (ld_agent(mygo) == 0u) {
                    if (++polls > p.wait_limit) { state = 0; break; }
                    __builtin_amdgcn_s_sleep(HB_SAT_POLL_SLEEP);
                }
                if (state == 0) {                         // stop waiting: hand the region to a finisher
                    st_agent(&S->todo[wg], 1u);
                    st_agent(&S->late[0], 1u);
                    stores_done();
                    if (ld_agent(mygo) != 0u) {           // the count completed meanwhile: finish it here after all
                        unsigned expect = 1u;             // (a finisher may have claimed it too: both write the same values)
                        __hip_atomic_compare_exchange_strong(&S->todo[wg], &expect, 2u, __ATOMIC_RELAXED,
                                                             __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        state = 1;
                    }
                }
                L.ctl = state;
            }
            __syncthreads();
            if (L.ctl == 0) return;
            if (tid == 0) late = ld_agent(&S->late[0]);   // in flight during the finish step
            SAT_STAMP(S, wg, 3);
        }

        sat_fused_finish<TR, TC, STREAM>(p, L, sw, bw, wv, lane, Lt);

        __syncthreads();
        if (own) {
            SAT_STAMP(S, wg, 5);
            if (tid == 0) L.ctl = (int)late;
            __syncthreads();
            if (__builtin_amdgcn_readfirstlane(L.ctl) == 0) return;   // nobody stopped waiting: done
            own = false;
            __syncthreads();
        }
        // finisher duty: wave 0 looks for a marked region and claims it
        if (tid < 64) {
            int found = -1;
            for (int r0 = 0; r0 < nwg && found < 0; r0 += 64) {
                const int r = r0 + lane;
                const bool marked = r < nwg && ld_agent(&S->todo[r]) == 1u;
                unsigned long long m = __ballot(marked);
                while (m && found < 0) {
                    const int cand = r0 + __builtin_ctzll(m);
                    m &= m - 1;
                    int won = 0;
                    if (lane == 0) {
                        unsigned expect = 1u;
                        won = __hip_atomic_compare_exchange_strong(&S->todo[cand], &expect, 2u, __ATOMIC_RELAXED,
                                                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ? 1 : 0;
                    }
                    if (__shfl(won, 0, 64)) found = cand;
                }
            }
            if (lane == 0) L.ctl = found;
        }
        __syncthreads();
        region = __builtin_amdgcn_readfirstlane(L.ctl);
        if (region < 0) return;
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// Vector-ALU twin of passes 1 and 3: the tile goes through LDS, threads add.
__global__ void __launch_bounds__(256) sat_sums_valu_kernel(SatArgs p) {
    __shared__ float s_px[kSatTile][kSatTile + 1];
    const int s = blockIdx.x / p.nb, b = blockIdx.x - s * p.nb;
    const int y0 = kSatTile * s, x0 = kSatTile * b;
    for (int idx = threadIdx.x; idx < kSatTile * 8; idx += 256) {
        const int r = idx >> 3, ch = idx & 7;
        const half8 v = load8_zero(p.in, p.in_pitch, y0 + r, x0 + 8 * ch, p.H, p.W);
#pragma unroll
        for (int i = 0; i < 8; ++i) s_px[r][8 * ch + i] = (float)v[i];
    }
    __syncthreads();
    if (threadIdx.x < 64) {
        float a = 0.f;
        for (int x = 0; x < kSatTile; ++x) a += s_px[threadIdx.x][x];
        p.rs[(int64_t)(y0 + threadIdx.x) * p.nb + b] = a;
        a = wave_sum(a);
        if (threadIdx.x == 0) p.tot[(int64_t)b * p.ns + s] = a;
    } else if (threadIdx.x < 128) {
        const int x = threadIdx.x - 64;
        float a = 0.f;
        for (int y = 0; y < kSatTile; ++y) a += s_px[y][x];
        p.cs[(int64_t)(x0 + x) * p.ns + s] = a;
    }
}

__global__ void __launch_bounds__(256) sat_apply_valu_kernel(SatArgs p) {
    __shared__ float s_t[kSatTile][kSatTile + 1];
    __shared__ float s_above[kSatTile];
    const int s = blockIdx.x / p.nb, b = blockIdx.x - s * p.nb;
    const int y0 = kSatTile * s, x0 = kSatTile * b;
    for (int idx = threadIdx.x; idx < kSatTile * 8; idx += 256) {
        const int r = idx >> 3, ch = idx & 7;
        const half8 v = load8_zero(p.in, p.in_pitch, y0 + r, x0 + 8 * ch, p.H, p.W);
#pragma unroll
        for (int i = 0; i < 8; ++i) s_t[r][8 * ch + i] = (float)v[i];
    }
    if (threadIdx.x < 64) {
        // table row above the tile, as in the MFMA kernel
        s_above[threadIdx.x] = sat_row_above(p, s, b, threadIdx.x);
    }
    __syncthreads();
    if (threadIdx.x < 64) {                               // row prefix, seeded with the row carry
        const int r = threadIdx.x;
        float a = p.rcarry[(int64_t)(y0 + r) * p.nb + b];
        for (int x = 0; x < kSatTile; ++x) {
            a += s_t[r][x];
            s_t[r][x] = a;
        }
    }
    __syncthreads();
    if (threadIdx.x < 64) {                               // column prefix, seeded with the table row above
        const int x = threadIdx.x;
        float a = s_above[x];
        for (int y = 0; y < kSatTile; ++y) {
            a += s_t[y][x];
            s_t[y][x] = a;
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < kSatTile * 16; idx += 256) {
        const int r = idx >> 4, q = idx & 15;
        const int y = y0 + r, xo = x0 + 4 * q;
        if (y >= p.H || xo >= p.W) continue;
        floatx4 v = {s_t[r][4 * q], s_t[r][4 * q + 1], s_t[r][4 * q + 2], s_t[r][4 * q + 3]};
        store4_mask(p.out + (int64_t)y * p.out_pitch, xo, p.W, v);
    }
}

static size_t sat_workspace_floats(int H, int W) {
    const size_t nb = (size_t)ceil_div(W, kSatTile), ns = (size_t)ceil_div(H, kSatTile);
    return 2 * (nb * ns * kSatTile) + 2 * (ns * nb * kSatTile) + 2 * ns * nb;   // rs, rcarry, cs, ccarry, tot, es
}

// Region shapes of the one-launch kernel: 2 x 2 tiles (128 x 128 pixels, 256 threads) for small
// images, 4 x 4 tiles (256 x 256 pixels, 1024 threads: fewer arrivals at the grid-wide wait, fewer
// table lines per region) once that still gives 128 regions or more.  0: more regions than the
// wait's bookkeeping holds; the three-launch path serves those.
static int sat_fused_shape(int H, int W) {
    const int64_t ra = (int64_t)ceil_div(H, 128) * ceil_div(W, 128), rb = (int64_t)ceil_div(H, 256) * ceil_div(W, 256);
    if (rb >= 128) return rb <= SatSync::kMaxRegions ? 4 : 0;
    return ra <= SatSync::kMaxRegions ? 2 : 4;            // rb < 128 here
}
// floats of the one-launch tables (RS, CS, TOT), rounded up to 64, for region edge `t` tiles
static size_t sat_fused_table_floats(int H, int W, int t) {
    const size_t e = (size_t)kSatTile * t, nsw = (size_t)ceil_div(H, (int)e), nbw = (size_t)ceil_div(W, (int)e);
    const size_t n = nbw * nsw * e + nsw * nbw * e + nsw * nbw;
    return (n + 63) & ~(size_t)63;
}
static size_t sat_fused_bytes(int H, int W) {
    const int t = sat_fused_shape(H, W);
    return t ? sat_fused_table_floats(H, W, t) * sizeof(float) + sizeof(SatSync) : 0;
}

static hb_status sat_prepare(SatArgs& a, const hb_half* in, float* out, int H, int W,
                             int64_t in_pitch, int64_t out_pitch, void* ws, size_t ws_bytes) {
    hb_status st = check_image(in, out, H, W, in_pitch, out_pitch);
    if (st != HB_OK) return st;
    if (!ws || !aligned_to(ws, 256) || ws_bytes < hb_sat2d_workspace_size(H, W)) return HB_ERR_WORKSPACE;
    a.in = reinterpret_cast<const half_t*>(in);
    a.out = out;
    a.H = H;
    a.W = W;
    a.in_pitch = in_pitch;
    a.out_pitch = out_pitch;
    a.nb = ceil_div(W, kSatTile);
    a.ns = ceil_div(H, kSatTile);
    a.Hs = a.ns * kSatTile;
    a.Ws = a.nb * kSatTile;
    float* f = reinterpret_cast<float*>(ws);
    a.rs = f;
    a.rcarry = a.rs + (size_t)a.nb * a.Hs;
    a.cs = a.rcarry + (size_t)a.nb * a.Hs;
    a.ccarry = a.cs + (size_t)a.ns * a.Ws;
    a.tot = a.ccarry + (size_t)a.ns * a.Ws;
    a.es = a.tot + (size_t)a.ns * a.nb;
    return HB_OK;
}

// The one-launch tables follow the three-launch tables in the workspace (both sized by hb_sat2d_workspace_size).
static void sat_prepare_fused(SatFusedArgs& f, const SatArgs& a, void* ws, int t, int wait_limit) {
    const int e = kSatTile * t;
    f.in = a.in;
    f.out = a.out;
    f.H = a.H;
    f.W = a.W;
    f.in_pitch = a.in_pitch;
    f.out_pitch = a.out_pitch;
    f.nsw = ceil_div(a.H, e);
    f.nbw = ceil_div(a.W, e);
    f.Hr = f.nsw * e;
    f.Wr = f.nbw * e;
    float* base = reinterpret_cast<float*>(ws) + ((sat_workspace_floats(a.H, a.W) + 63) & ~(size_t)63);
    f.RS = base;
    f.CS = f.RS + (size_t)f.nbw * f.Hr;
    f.TOT = f.CS + (size_t)f.nsw * f.Wr;
    f.sync = reinterpret_cast<SatSync*>(base + sat_fused_table_floats(a.H, a.W, t));
    f.wait_limit = wait_limit;
}

}  // namespace hb

extern "C" size_t hb_sat2d_workspace_size(int H, int W) {
    if (H < 1 || W < 1) return 0;
    return ((hb::sat_workspace_floats(H, W) + 63) & ~(size_t)63) * sizeof(float) + hb::sat_fused_bytes(H, W);
}

// Scratch of hb_sat2d_noalloc: the carry tables live in this array instead of a caller's workspace.
// In host code the array's name is only a handle, not a device address: the address is looked up
// once per device (every GPU holds its own copy of the array) and kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[HB_SAT2D_NOALLOC_SCRATCH_BYTES];

namespace hb {

// Polls a workgroup of the one-launch kernel spends in its grid-wide wait before it hands its region
// to a finisher (a poll is a quarter of a microsecond of sleep plus one memory round trip).
constexpr int kSatDefaultWaitLimit = 1 << 14;
static std::atomic<int> g_sat_wait_limit{kSatDefaultWaitLimit};

// Workgroups of each one-launch kernel shape the current device holds at once (0: query failed).
struct SatCapacity { int shape2 = -1, shape4 = -1; };
static SatCapacity g_sat_capacity[kMaxDevices];
static std::mutex g_sat_mu;

template <int T, bool STREAM>
static hb_status sat_fused_launch(const SatFusedArgs& f, hipStream_t st) {
    auto kernel = sat_fused_kernel<T, T, STREAM>;
    const size_t lds = sizeof(SatFusedLds<T, T>);
    hb_status s = allow_dynamic_lds(reinterpret_cast<const void*>(kernel), lds);
    if (s != HB_OK) return s;
    hipLaunchKernelGGL(sat_sync_clear_kernel, dim3(1), dim3(256), 0, st, f.sync);
    hipLaunchKernelGGL(kernel, dim3(f.nsw * f.nbw), dim3(64 * T * T), lds, st, f);
    return launch_status();
}

template <int T>
static int sat_fused_capacity_query() {
    auto kernel = sat_fused_kernel<T, T, true>;
    const size_t lds = sizeof(SatFusedLds<T, T>);
    if (allow_dynamic_lds(reinterpret_cast<const void*>(kernel), lds) != HB_OK) return 0;
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, 64 * T * T, lds) != hipSuccess) return 0;
    const int ncu = device_num_cu();
    return ncu > 0 && per_cu > 0 ? per_cu * ncu : 0;
}

// 0 when the grid of shape `t` cannot be resident at once on the current device.
static int sat_fused_capacity(int t) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
    std::lock_guard<std::mutex> lock(g_sat_mu);
    SatCapacity& c = g_sat_capacity[dev];
    if (t == 2) {
        if (c.shape2 < 0) c.shape2 = sat_fused_capacity_query<2>();
        return c.shape2;
    }
    if (c.shape4 < 0) c.shape4 = sat_fused_capacity_query<4>();
    return c.shape4;
}

static hb_status sat_launch_mfma(const SatArgs& a, void* ws, hipStream_t st) {
    const bool stream_stores = (int64_t)a.H * a.W * 4 <= kStreamStoreMaxBytes;
    const int t = sat_fused_shape(a.H, a.W);
    if (t) {
        SatFusedArgs f;
        sat_prepare_fused(f, a, ws, t, g_sat_wait_limit.load());
        if (f.nsw * f.nbw <= sat_fused_capacity(t)) {
            if (t == 2) return stream_stores ? sat_fused_launch<2, true>(f, st) : sat_fused_launch<2, false>(f, st);
            return stream_stores ? sat_fused_launch<4, true>(f, st) : sat_fused_launch<4, false>(f, st);
        }
    }
    const int ntiles = a.nb * a.ns;
    hipLaunchKernelGGL(sat_sums_mfma_kernel, dim3(ceil_div(ntiles, 4)), dim3(256), 0, st, a);
    hipLaunchKernelGGL(sat_scan_kernel, dim3(ceil_div(a.Hs + a.Ws + a.nb, 4)), dim3(256), 0, st, a);
    if (stream_stores)
        hipLaunchKernelGGL((sat_apply_mfma_kernel<true>), dim3(ceil_div(ntiles, 4)), dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL((sat_apply_mfma_kernel<false>), dim3(ceil_div(ntiles, 4)), dim3(256), 0, st, a);
    return launch_status();
}

static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mu;

static hb_status sat_scratch_address(void** ptr) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return HB_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return HB_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return HB_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return HB_OK;
}

}  // namespace hb

extern "C" int hb_sat2d_set_wait_limit(int polls) {
    const int prev = hb::g_sat_wait_limit.load();
    hb::g_sat_wait_limit.store(polls > 0 ? polls : (polls == 0 ? hb::kSatDefaultWaitLimit : 0));
    return prev;
}

extern "C" hb_status hb_sat2d(const hb_half* in, float* out, int H, int W,
                              int64_t in_pitch, int64_t out_pitch,
                              void* workspace, size_t workspace_bytes, hb_stream stream) {
    using namespace hb;
    SatArgs a;
    hb_status s = sat_prepare(a, in, out, H, W, in_pitch, out_pitch, workspace, workspace_bytes);
    if (s != HB_OK) return s;
    return sat_launch_mfma(a, workspace, reinterpret_cast<hipStream_t>(stream));
}

extern "C" hb_status hb_sat2d_noalloc(const hb_half* in, float* out, int H, int W,
                                      int64_t in_pitch, int64_t out_pitch, hb_stream stream) {
    using namespace hb;
    hb_status s = check_image(in, out, H, W, in_pitch, out_pitch);
    if (s != HB_OK) return s;
    if (hb_sat2d_workspace_size(H, W) > (size_t)HB_SAT2D_NOALLOC_SCRATCH_BYTES) return HB_ERR_UNSUPPORTED;
    void* ws = nullptr;
    s = sat_scratch_address(&ws);
    if (s != HB_OK) return s;
    SatArgs a;
    s = sat_prepare(a, in, out, H, W, in_pitch, out_pitch, ws, (size_t)HB_SAT2D_NOALLOC_SCRATCH_BYTES);
    if (s != HB_OK) return s;
    return sat_launch_mfma(a, ws, reinterpret_cast<hipStream_t>(stream));
}

extern "C" hb_status hb_sat2d_valu(const hb_half* in, float* out, int H, int W,
                                   int64_t in_pitch, int64_t out_pitch,
                                   void* workspace, size_t workspace_bytes, hb_stream stream) {
    using namespace hb;
    SatArgs a;
    hb_status s = sat_prepare(a, in, out, H, W, in_pitch, out_pitch, workspace, workspace_bytes);
    if (s != HB_OK) return s;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const int ntiles = a.nb * a.ns;
    hipLaunchKernelGGL(sat_sums_valu_kernel, dim3(ntiles), dim3(256), 0, st, a);
    hipLaunchKernelGGL(sat_scan_kernel, dim3(ceil_div(a.Hs + a.Ws + a.nb, 4)), dim3(256), 0, st, a);
    hipLaunchKernelGGL(sat_apply_valu_kernel, dim3(ntiles), dim3(256), 0, st, a);
    return launch_status();
}
