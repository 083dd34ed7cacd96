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
#include "hb_device.hpp"
#include "hb_host.hpp"

namespace hb {

constexpr int kSatTile = 64;

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
                X[rt][blk] = ldg8(src, off + 2u * (16u * rt * (uint32_t)p.in_pitch + 32u * blk));
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
                X[rt][blk] = ldg8(src, off + 2u * (16u * rt * (uint32_t)p.in_pitch + 32u * blk));
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

}  // namespace hb

extern "C" size_t hb_sat2d_workspace_size(int H, int W) {
    if (H < 1 || W < 1) return 0;
    return hb::sat_workspace_floats(H, W) * sizeof(float);
}

// Scratch of hb_sat2d_noalloc: the carry tables live in this array instead of a caller's workspace.
// In host code the array's name is only a handle, not a device address: the address is looked up
// once per device (every GPU holds its own copy of the array) and kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[HB_SAT2D_NOALLOC_SCRATCH_BYTES];

namespace hb {

static hb_status sat_launch_mfma(const SatArgs& a, hipStream_t st) {
    const int ntiles = a.nb * a.ns;
    hipLaunchKernelGGL(sat_sums_mfma_kernel, dim3(ceil_div(ntiles, 4)), dim3(256), 0, st, a);
    hipLaunchKernelGGL(sat_scan_kernel, dim3(ceil_div(a.Hs + a.Ws + a.nb, 4)), dim3(256), 0, st, a);
    if ((int64_t)a.H * a.W * 4 <= kStreamStoreMaxBytes)
        hipLaunchKernelGGL((sat_apply_mfma_kernel<true>), dim3(ceil_div(ntiles, 4)), dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL((sat_apply_mfma_kernel<false>), dim3(ceil_div(ntiles, 4)), dim3(256), 0, st, a);
    return launch_status();
}

constexpr int kMaxDevices = 64;
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

extern "C" hb_status hb_sat2d(const hb_half* in, float* out, int H, int W,
                              int64_t in_pitch, int64_t out_pitch,
                              void* workspace, size_t workspace_bytes, hb_stream stream) {
    using namespace hb;
    SatArgs a;
    hb_status s = sat_prepare(a, in, out, H, W, in_pitch, out_pitch, workspace, workspace_bytes);
    if (s != HB_OK) return s;
    return sat_launch_mfma(a, reinterpret_cast<hipStream_t>(stream));
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
    return sat_launch_mfma(a, reinterpret_cast<hipStream_t>(stream));
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
