// hb_dct_denoise: transform-domain coring on overlapping windowed 16 x 16 tiles, and its
// vector-ALU twin (Sec. V-E): window, DCT down the columns and along the rows, small bins set to
// zero, the two inverse transforms, window again; the overlapping tiles are blended and the
// windowing undone.
//
// As in the paper the four 16 x 16 matrix products of a tile and the coring between them are fused.
// The paper keeps the blend as a second launch; here the matrix-unit path blends inside the same
// kernel (a workgroup owns a patch of the output and accumulates its tiles in LDS), which saves
// writing and re-reading 1 KB per tile; the vector-ALU twin keeps the two-launch structure with the
// tiles in the workspace.  The products run on the matrix units in
// fp32 (v_mfma_f32_16x16x4_f32, four instructions per product): DCT coefficients reach 16 times the
// pixel range, so fp16 intermediates would cost about 1e-3 of absolute accuracy per rounding, and the
// products are far too small for the precision to matter for speed.  A product leaves its result
// with a lane owning four ROWS of one column while the next product needs that matrix as an operand
// indexed the other way round, so each of the three hand-overs goes through a wave-private 16 x 17
// LDS tile.
#include <math.h>

#include "hb_device.hpp"
#include "hb_host.hpp"

namespace hb {

constexpr int kDctWaves = 4;                  // waves per workgroup
constexpr int kDctPitch = 17;                 // floats per row of an LDS tile (conflict-free both ways)

struct DctArgs {
    const half_t* in;
    float* out;
    float* tiles;                             // workspace: [C][nty][ntx][16][16] windowed reconstructions
    int C, H, W, nty, ntx;
    int64_t in_pitch, in_plane, out_pitch, out_plane;
    float threshold;
    float d[256];                             // D[u][i], orthonormal DCT-II, row-major
    float w[16];                              // sine window
};

__device__ __forceinline__ void dct_wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// acc (lane (c, g): rows 4g + j of column c) -> LDS tile [row][column]
__device__ __forceinline__ void dct_put(float* tile, const floatx4& acc, int c, int g) {
#pragma unroll
    for (int j = 0; j < 4; ++j) tile[(4 * g + j) * kDctPitch + c] = acc[j];
}

__device__ __forceinline__ void dct_tile_origin(const DctArgs& p, int64_t t, int& plane, int& y0, int& x0) {
    const int per_plane = p.nty * p.ntx;
    plane = (int)(t / per_plane);
    const int r = (int)(t - (int64_t)plane * per_plane);
    y0 = 8 * (r / p.ntx);
    x0 = 8 * (r % p.ntx);
}

// ---------------------------------------------------------------------------
// The matrix-unit path in ONE launch: transform, core, transform back AND blend.  A workgroup owns a
// 64 x 64 patch of the output and runs every tile that overlaps it (up to 9 x 9; the tiles on the rim
// are run by the neighbouring patch as well, 1.27x the products), adding the windowed reconstructions
// into an fp32 image of the patch in LDS instead of writing 1 KB per tile to memory and reading it
// back.  Tiles overlap their neighbours at stride 8, tiles at stride 16 do not: the tiles are taken in
// four rounds by the parity of their (row, column) index, within a round the waves add to disjoint
// pixels with plain loads and stores, and the order of the four additions into a pixel is fixed.
constexpr int kDfPatch = 64;
constexpr int kDfPitch = kDfPatch + 4;        // rows 4 apart fall into different banks
constexpr int kDfWaves = 8;
constexpr int kDfRegion = kDfPatch + 16;      // pixels under the tiles of a patch, per axis
constexpr int kDfPxPitch = kDfRegion + 8;     // 88 halves: 16 consecutive rows fall into 16 different banks

__global__ void __launch_bounds__(64 * kDfWaves) dct_fused_mfma_kernel(DctArgs p) {
    __shared__ float s_tile[kDfWaves][16 * kDctPitch];
    __shared__ __attribute__((aligned(16))) float s_acc[kDfPatch * kDfPitch];
    __shared__ __attribute__((aligned(16))) half_t s_px[kDfRegion * kDfPxPitch];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int c = lane & 15, g = lane >> 4;
    float* tile = s_tile[wv];
    float dlk[4], dkl[4], win[4], wout[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        dlk[kk] = p.d[c * 16 + 4 * kk + g];
        dkl[kk] = p.d[(4 * kk + g) * 16 + c];
        win[kk] = p.w[c] * p.w[4 * kk + g];
        wout[kk] = p.w[4 * g + kk] * p.w[c];
    }
    const int npx = (p.W + kDfPatch - 1) / kDfPatch, npy = (p.H + kDfPatch - 1) / kDfPatch;
    // every XCD takes one contiguous run of the patches: the 8-pixel rims that neighbouring patches share
    // (whole 128-byte lines in memory) are fetched into one L2 once (measured reads 1.05x the image
    // instead of 2.9x)
    int wg = xcd_contiguous(blockIdx.x, gridDim.x);
    const int pc = wg % npx;
    wg /= npx;
    const int pr = wg % npy, plane = wg / npy;
    const int py0 = kDfPatch * pr, px0 = kDfPatch * pc;
    for (int i = threadIdx.x; i < kDfPatch * kDfPitch; i += 64 * kDfWaves) s_acc[i] = 0.f;
    // the pixels under every tile of the patch: rows py0 - 8 .. py0 + 71, columns px0 - 8 .. px0 + 71
    // (what lies outside the image is under no tile and is never read)
    {
        const half_t* plane_px = p.in + (int64_t)plane * p.in_plane;
        for (int i = threadIdx.x; i < kDfRegion * (kDfRegion / 8); i += 64 * kDfWaves) {
            const int r = i / (kDfRegion / 8), ch = i - r * (kDfRegion / 8);
            const int y = py0 - 8 + r, x = px0 - 8 + 8 * ch;
            if (y >= 0 && y < p.H && x >= 0 && x < p.W)       // W is a multiple of 8: whole chunks
                *reinterpret_cast<half8*>(&s_px[r * kDfPxPitch + 8 * ch]) =
                    *reinterpret_cast<const half8_u*>(plane_px + (int64_t)y * p.in_pitch + x);
        }
    }
    // tiles (ty, tx), origin (8 ty, 8 tx), that overlap the patch
    const int ty_lo = max(py0 / 8 - 1, 0), ty_hi = min(py0 / 8 + kDfPatch / 8 - 1, p.nty - 1);
    const int tx_lo = max(px0 / 8 - 1, 0), tx_hi = min(px0 / 8 + kDfPatch / 8 - 1, p.ntx - 1);
    __syncthreads();
    for (int round = 0; round < 4; ++round) {
        const int ty0 = ty_lo + ((ty_lo ^ (round >> 1)) & 1), tx0 = tx_lo + ((tx_lo ^ round) & 1);
        const int ny = ty0 <= ty_hi ? (ty_hi - ty0) / 2 + 1 : 0, nx = tx0 <= tx_hi ? (tx_hi - tx0) / 2 + 1 : 0;
        for (int i = wv; i < ny * nx; i += kDfWaves) {
            const int ty = ty0 + 2 * (i / nx), tx = tx0 + 2 * (i % nx);
            // lane (c = row, g) reads pixels (row, 4 kk + g)
            const half_t* src = &s_px[(8 * ty - py0 + 8 + c) * kDfPxPitch + 8 * tx - px0 + 8 + g];
            float px[4];
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) px[kk] = (float)src[4 * kk] * win[kk];
            // Q = T D^T
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) acc = mfma16x16x4f32(px[kk], dlk[kk], acc);
            dct_put(tile, acc, c, g);
            dct_wave_sync();
            // Y = D Q
            float b[4];
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) b[kk] = tile[(4 * kk + g) * kDctPitch + c];
            acc = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) acc = mfma16x16x4f32(dlk[kk], b[kk], acc);
            // coring: lane (c = v, g) holds Y[4g + j][v]; the DC bin always stays
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (fabsf(acc[j]) < p.threshold && !(c == 0 && g == 0 && j == 0)) acc[j] = 0.f;
            dct_wave_sync();
            dct_put(tile, acc, c, g);
            dct_wave_sync();
            // R = D^T Y
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) b[kk] = tile[(4 * kk + g) * kDctPitch + c];
            acc = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) acc = mfma16x16x4f32(dkl[kk], b[kk], acc);
            dct_wave_sync();
            dct_put(tile, acc, c, g);
            dct_wave_sync();
            // rec = R D
            float a[4];
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) a[kk] = tile[c * kDctPitch + 4 * kk + g];
            acc = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) acc = mfma16x16x4f32(a[kk], dkl[kk], acc);
            dct_wave_sync();
            // lane (c = col, g) holds rec[4g + j][col]: window again, add the part inside the patch
            const int xx = 8 * tx + c - px0;
            if (xx >= 0 && xx < kDfPatch) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int yy = 8 * ty + 4 * g + j - py0;
                    if (yy >= 0 && yy < kDfPatch) s_acc[yy * kDfPitch + xx] += acc[j] * wout[j];
                }
            }
        }
        __syncthreads();
    }
    // out = sum of the windowed reconstructions / sum of the squared windows of the tiles covering the pixel
    // (the tiles covering a pixel are a product set, so the denominator is a product of two 1-D sums)
    for (int idx = threadIdx.x; idx < kDfPatch * (kDfPatch / 4); idx += 64 * kDfWaves) {
        const int r = idx / (kDfPatch / 4), q4 = idx - r * (kDfPatch / 4);
        const int y = py0 + r, x = px0 + 4 * q4;
        if (y >= p.H || x >= p.W) continue;
        float dy = 0.f;
        for (int ty = y / 8 - 1; ty <= y / 8; ++ty)
            if (ty >= 0 && ty < p.nty) dy += p.w[y - 8 * ty] * p.w[y - 8 * ty];
        const floatx4 v = *reinterpret_cast<const floatx4*>(&s_acc[r * kDfPitch + 4 * q4]);
        floatx4 o;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float dx = 0.f;
            for (int tx = (x + q) / 8 - 1; tx <= (x + q) / 8; ++tx)
                if (tx >= 0 && tx < p.ntx) dx += p.w[x + q - 8 * tx] * p.w[x + q - 8 * tx];
            o[q] = v[q] / (dy * dx);
        }
        *reinterpret_cast<floatx4_u*>(p.out + (int64_t)plane * p.out_plane + (int64_t)y * p.out_pitch + x) = o;
    }
}

// Vector-ALU twin: the same four products as plain dot products over LDS tiles.
// out[i][j] = sum_k A[i * ai + k * ak] * B[k * bk + j * bj], lane (c, g) computes rows 4g + jj of column c.
__device__ __forceinline__ void dct_mm_valu(const float* A, int ai, int ak, const float* B, int bk, int bj,
                                            floatx4& acc, int c, int g) {
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
        float s = 0.f;
        for (int k = 0; k < 16; ++k) s = fmaf(A[(4 * g + jj) * ai + k * ak], B[k * bk + c * bj], s);
        acc[jj] = s;
    }
}

__global__ void __launch_bounds__(64 * kDctWaves) dct_transform_valu_kernel(DctArgs p) {
    __shared__ float s_tile[kDctWaves][2][16 * kDctPitch];
    __shared__ float s_d[16 * kDctPitch];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int c = lane & 15, g = lane >> 4;
    for (int i = threadIdx.x; i < 256; i += 64 * kDctWaves) s_d[(i >> 4) * kDctPitch + (i & 15)] = p.d[i];
    __syncthreads();
    float* ta = s_tile[wv][0];
    float* tb = s_tile[wv][1];
    const int64_t ntiles = (int64_t)p.C * p.nty * p.ntx;
    const int64_t stride = (int64_t)gridDim.x * kDctWaves;
    for (int64_t t = (int64_t)blockIdx.x * kDctWaves + wv; t < ntiles; t += stride) {
        int plane, y0, x0;
        dct_tile_origin(p, t, plane, y0, x0);
        const half_t* src = p.in + (int64_t)plane * p.in_plane + (int64_t)y0 * p.in_pitch + x0;
        floatx4 acc;
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = (float)src[(int64_t)(4 * g + j) * p.in_pitch + c] * p.w[4 * g + j] * p.w[c];
        dct_put(ta, acc, c, g);                                       // T [row][col]
        dct_wave_sync();
        dct_mm_valu(ta, kDctPitch, 1, s_d, 1, kDctPitch, acc, c, g);  // Q[r][v] = sum_col T[r][col] D[v][col]
        dct_put(tb, acc, c, g);
        dct_wave_sync();
        dct_mm_valu(s_d, kDctPitch, 1, tb, kDctPitch, 1, acc, c, g);  // Y[u][v] = sum_r D[u][r] Q[r][v]
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (fabsf(acc[j]) < p.threshold && !(c == 0 && g == 0 && j == 0)) acc[j] = 0.f;
        dct_put(ta, acc, c, g);
        dct_wave_sync();
        dct_mm_valu(s_d, 1, kDctPitch, ta, kDctPitch, 1, acc, c, g);  // R[r][v] = sum_u D[u][r] Y[u][v]
        dct_put(tb, acc, c, g);
        dct_wave_sync();
        dct_mm_valu(tb, kDctPitch, 1, s_d, kDctPitch, 1, acc, c, g);  // rec[r][col] = sum_v R[r][v] D[v][col]
        float* dst = p.tiles + t * 256;
#pragma unroll
        for (int j = 0; j < 4; ++j) dst[(4 * g + j) * 16 + c] = acc[j] * p.w[4 * g + j] * p.w[c];
        dct_wave_sync();
    }
}

// 2  blend: out = sum over the (up to four) tiles covering a pixel of their windowed
// reconstruction, divided by the sum of their squared windows.  A thread owns four consecutive pixels.
__global__ void __launch_bounds__(256) dct_blend_kernel(DctArgs p) {
    // a workgroup covers 16 rows x 64 columns: the 64-byte rows of a tile it reads share their
    // cache lines with the rows above and below, which the same workgroup reads as well
    const int bx_n = (p.W + 63) / 64, by_n = (p.H + 15) / 16;
    int wg = blockIdx.x;
    const int bx = wg % bx_n;
    wg /= bx_n;
    const int by = wg % by_n, plane = wg / by_n;
    const int y = 16 * by + (threadIdx.x >> 4), x = 64 * bx + 4 * (threadIdx.x & 15);
    if (y >= p.H || x >= p.W) return;
    floatx4 num = {0.f, 0.f, 0.f, 0.f}, den = {0.f, 0.f, 0.f, 0.f};
    for (int ty = y / 8 - 1; ty <= y / 8; ++ty) {
        if (ty < 0 || ty >= p.nty) continue;
        const int r = y - 8 * ty;
        for (int tx = x / 8 - 1; tx <= x / 8; ++tx) {
            if (tx < 0 || tx >= p.ntx) continue;
            const int cc = x - 8 * tx;
            const float* tile = p.tiles + (((int64_t)plane * p.nty + ty) * p.ntx + tx) * 256;
            const floatx4 v = *reinterpret_cast<const floatx4*>(tile + r * 16 + cc);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float ww = p.w[r] * p.w[cc + q];
                num[q] += v[q];
                den[q] += ww * ww;
            }
        }
    }
    float* dst = p.out + (int64_t)plane * p.out_plane + (int64_t)y * p.out_pitch + x;
#pragma unroll
    for (int q = 0; q < 4; ++q) dst[q] = num[q] / den[q];
}

static hb_status dct_run(bool valu, const hb_half* in, float* out, int C, int H, int W,
                         int64_t in_pitch, int64_t in_plane, int64_t out_pitch, int64_t out_plane,
                         float threshold, void* workspace, size_t workspace_bytes, hb_stream stream) {
    if (!in || !out) return HB_ERR_INVALID_ARG;
    if (C < 1 || H < 16 || W < 16 || (H & 7) || (W & 7)) return HB_ERR_INVALID_ARG;
    if (in_pitch < W || out_pitch < W) return HB_ERR_INVALID_ARG;
    if (C > 1 && (in_plane < (int64_t)H * in_pitch || out_plane < (int64_t)H * out_pitch)) return HB_ERR_INVALID_ARG;
    if (!aligned_to(in, 2) || !aligned_to(out, 4)) return HB_ERR_INVALID_ARG;
    if (!(threshold >= 0.f)) return HB_ERR_INVALID_ARG;                // also rejects NaN
    if (C > 65535 || (int64_t)C * H * W > ((int64_t)1 << 40)) return HB_ERR_UNSUPPORTED;
    const size_t need = hb_dct_denoise_workspace_size(C, H, W);
    if (!workspace || workspace_bytes < need || !aligned_to(workspace, 256)) return HB_ERR_WORKSPACE;

    DctArgs a;
    a.in = reinterpret_cast<const half_t*>(in);
    a.out = out;
    a.tiles = reinterpret_cast<float*>(workspace);
    a.C = C;
    a.H = H;
    a.W = W;
    a.nty = H / 8 - 1;
    a.ntx = W / 8 - 1;
    a.in_pitch = in_pitch;
    a.in_plane = in_plane;
    a.out_pitch = out_pitch;
    a.out_plane = out_plane;
    a.threshold = threshold;
    const double pi = 3.14159265358979323846;
    for (int u = 0; u < 16; ++u)
        for (int i = 0; i < 16; ++i)
            a.d[u * 16 + i] = (float)(u == 0 ? 0.25 : sqrt(2.0 / 16.0) * cos(pi * (2.0 * i + 1.0) * u / 32.0));
    for (int i = 0; i < 16; ++i) a.w[i] = (float)sin(pi * (i + 0.5) / 16.0);

    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const int64_t ntiles = (int64_t)C * a.nty * a.ntx;
    const int64_t wgs = (ntiles + kDctWaves - 1) / kDctWaves;
    const unsigned blocks = (unsigned)(wgs < 4096 ? wgs : 4096);     // waves stride over the tiles
    if (!valu) {
        // one launch: tiles and blend fused, the workspace stays unused
        const int64_t patches = (int64_t)C * ceil_div(H, kDfPatch) * ceil_div(W, kDfPatch);
        if (patches > 0x7fffffff) return HB_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(dct_fused_mfma_kernel, dim3((unsigned)patches), dim3(64 * kDfWaves), 0, st, a);
        return launch_status();
    }
    hipLaunchKernelGGL(dct_transform_valu_kernel, dim3(blocks), dim3(64 * kDctWaves), 0, st, a);
    const int64_t bblocks = (int64_t)C * ((H + 15) / 16) * ((W + 63) / 64);
    if (bblocks > 0x7fffffff) return HB_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(dct_blend_kernel, dim3((unsigned)bblocks), dim3(256), 0, st, a);
    return launch_status();
}

}  // namespace hb

extern "C" size_t hb_dct_denoise_workspace_size(int C, int H, int W) {
    if (C < 1 || H < 16 || W < 16 || (H & 7) || (W & 7)) return 0;
    return (size_t)C * (size_t)(H / 8 - 1) * (size_t)(W / 8 - 1) * 256 * sizeof(float);
}

extern "C" hb_status hb_dct_denoise(const hb_half* in, float* out, int C, int H, int W,
                                    int64_t in_pitch, int64_t in_plane, int64_t out_pitch, int64_t out_plane,
                                    float threshold, void* workspace, size_t workspace_bytes, hb_stream stream) {
    return hb::dct_run(false, in, out, C, H, W, in_pitch, in_plane, out_pitch, out_plane, threshold, workspace,
                       workspace_bytes, stream);
}

extern "C" hb_status hb_dct_denoise_valu(const hb_half* in, float* out, int C, int H, int W,
                                         int64_t in_pitch, int64_t in_plane, int64_t out_pitch, int64_t out_plane,
                                         float threshold, void* workspace, size_t workspace_bytes, hb_stream stream) {
    return hb::dct_run(true, in, out, C, H, W, in_pitch, in_plane, out_pitch, out_plane, threshold, workspace,
                       workspace_bytes, stream);
}
