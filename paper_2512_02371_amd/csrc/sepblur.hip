// hb_sepblur: separable 2-D blur as two chained Toeplitz products per tile
// (Sec. V-A), and its vector-ALU twin.
//
// MFMA formulation.  A wave owns a 64-column strip and walks down it in steps of
// 16 rows.
//   row pass     T1[m][n] = sum_k P[m][k] * Bx[k][n]     m = image row, n = column, k = pixel
//                Bx[k][n] = taps_x[32*delta + k - (16*par + n) + anchor_x]
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
// independently.
#include "hb_device.hpp"
#include "hb_host.hpp"

namespace hb {

struct SepArgs {
    const half_t* in;
    float* out;
    int H, W;
    int64_t in_pitch, out_pitch;
    int Tx, ax, Ty, ay;
    int dmin;          // first neighbouring 32-pixel block a 32-column output block reads
    int nct;           // 64-column strips
    int steps;         // 16-row steps per task
    int nseg;          // row segments per strip
    int ntasks;        // nct * nseg
    int vec_in, vec_out;
    Taps tx, ty;
};

__device__ __forceinline__ half_t sep_tap(uint16_t b) { return __builtin_bit_cast(half_t, b); }

template <int ND, int NT>
__global__ void __launch_bounds__(256) sepblur_mfma_kernel(SepArgs p) {
    constexpr int NK = (NT + 1) / 2;          // K = 32 chunks of the column pass
    __shared__ half_t s_tx[HB_MAX_TAPS], s_ty[HB_MAX_TAPS];
    if (threadIdx.x < HB_MAX_TAPS) {
        s_tx[threadIdx.x] = sep_tap(p.tx.v[threadIdx.x]);
        s_ty[threadIdx.x] = sep_tap(p.ty.v[threadIdx.x]);
    }
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int c = lane & 15, g = lane >> 4;

    half8 coefx[2][ND];                       // B operand of the row pass
#pragma unroll
    for (int par = 0; par < 2; ++par)
#pragma unroll
        for (int d = 0; d < ND; ++d)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                int t = 32 * (p.dmin + d) + 8 * g + i - (16 * par + c) + p.ax;
                coefx[par][d][i] = (t >= 0 && t < p.Tx) ? s_tx[t] : (half_t)0;
            }
    half8 coefy[NK];                          // B operand of the column pass, chained slot order
#pragma unroll
    for (int j = 0; j < NK; ++j)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            int t = 32 * j + krow32(g, i) - c;
            coefy[j][i] = (t >= 0 && t < p.Ty) ? s_ty[t] : (half_t)0;
        }

    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int nwaves = (gridDim.x * blockDim.x) >> 6;
    for (int task = wave; task < p.ntasks; task += nwaves) {
        const int seg = task / p.nct, ct = task - seg * p.nct;
        const int x0 = 64 * ct;
        const int Y0 = seg * p.steps * 16;
        const int nsteps = min(p.steps, (p.H - Y0 + 15) / 16);

        half4 hist[NT][4];                    // row-filtered tiles q .. q+NT-1, four 16-column tiles each
#pragma unroll
        for (int q = 0; q < NT; ++q)
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) hist[q][t4] = half4{0, 0, 0, 0};

        // tile q covers image rows Y0 - ay + 16 q + (0..15)
        for (int q = 0; q < nsteps + NT - 1; ++q) {
            const int yr = clampi(Y0 - p.ay + 16 * q + c, 0, p.H - 1);
            const half_t* row = p.in + (int64_t)yr * p.in_pitch;
            half8 blk[ND + 1];
#pragma unroll
            for (int j = 0; j <= ND; ++j)
                blk[j] = load8_clamp(row, x0 + 32 * (p.dmin + j) + 8 * g, p.W, p.vec_in);
#pragma unroll
            for (int u = 0; u < NT - 1; ++u)
#pragma unroll
                for (int t4 = 0; t4 < 4; ++t4) hist[u][t4] = hist[u + 1][t4];
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int par = 0; par < 2; ++par) {
                    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int d = 0; d < ND; ++d) acc = mfma16x16x32(blk[tb + d], coefx[par][d], acc);
                    hist[NT - 1][2 * tb + par] = to_half4(acc);
                }
            const int s = q - (NT - 1);       // output step completed by this tile
            if (s < 0) continue;
            const int yo = Y0 + 16 * s + c;
            float* orow = p.out + (int64_t)yo * p.out_pitch;
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) {
                floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < NK; ++j) {
                    const half4 lo = hist[2 * j][t4];
                    const half4 hi = (2 * j + 1 < NT) ? hist[2 * j + 1][t4] : half4{0, 0, 0, 0};
                    acc = mfma16x16x32(join(lo, hi), coefy[j], acc);
                }
                const int xo = x0 + 16 * t4 + 4 * g;
                if (yo < p.H && xo < p.W) store4_mask(orow, xo, p.W, acc, p.vec_out);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Vector-ALU twin: 32 x 64 output tile per workgroup; pixels with halo in LDS,
// row pass to an fp16 LDS intermediate, column pass from it.
constexpr int kVTH = 32, kVTW = 64;
constexpr int kVRows = kVTH + HB_MAX_TAPS - 1;          // 95
constexpr int kVPxPitch = kVTW + 64 + 64 + 8;           // 200
constexpr int kVTmpPitch = kVTW + 4;                    // 68

__global__ void __launch_bounds__(256) sepblur_valu_kernel(SepArgs p) {
    __shared__ half_t s_px[kVRows * kVPxPitch];
    __shared__ half_t s_tmp[kVRows * kVTmpPitch];
    __shared__ float s_kx[HB_MAX_TAPS], s_ky[HB_MAX_TAPS];
    if (threadIdx.x < HB_MAX_TAPS) {
        s_kx[threadIdx.x] = (float)sep_tap(p.tx.v[threadIdx.x]);
        s_ky[threadIdx.x] = (float)sep_tap(p.ty.v[threadIdx.x]);
    }
    const int nctv = (p.W + kVTW - 1) / kVTW;
    const int rt = blockIdx.x / nctv, ct = blockIdx.x - rt * nctv;
    const int x0 = ct * kVTW, y0 = rt * kVTH;
    const int lead = 8 * ((p.ax + 7) / 8);
    const int nch = (kVTW + lead + (p.Tx - 1 - p.ax) + 7) / 8;
    const int nrows = kVTH + p.Ty - 1;
    for (int idx = threadIdx.x; idx < nrows * nch; idx += 256) {
        const int r = idx / nch, ch = idx - r * nch;
        const half_t* row = p.in + (int64_t)clampi(y0 - p.ay + r, 0, p.H - 1) * p.in_pitch;
        *reinterpret_cast<half8*>(&s_px[r * kVPxPitch + 8 * ch]) =
            load8_clamp(row, x0 - lead + 8 * ch, p.W, p.vec_in);
    }
    __syncthreads();
    const int off = lead - p.ax;
    for (int idx = threadIdx.x; idx < nrows * (kVTW / 4); idx += 256) {
        const int r = idx / (kVTW / 4), cg = idx - r * (kVTW / 4);
        const half_t* src = &s_px[r * kVPxPitch + 4 * cg + off];
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int u = 0; u < p.Tx + 3; ++u) {
            const float v = (float)src[u];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int t = u - q;
                if (t >= 0 && t < p.Tx) acc[q] = fmaf(s_kx[t], v, acc[q]);
            }
        }
        *reinterpret_cast<half4*>(&s_tmp[r * kVTmpPitch + 4 * cg]) = to_half4(acc);
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < kVTH * (kVTW / 4); idx += 256) {
        const int r = idx / (kVTW / 4), cg = idx - r * (kVTW / 4);
        const int y = y0 + r, x = x0 + 4 * cg;
        if (y >= p.H || x >= p.W) continue;
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int t = 0; t < p.Ty; ++t) {
            const half4 v = *reinterpret_cast<const half4*>(&s_tmp[(r + t) * kVTmpPitch + 4 * cg]);
            const float k = s_ky[t];
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q] = fmaf(k, (float)v[q], acc[q]);
        }
        store4_mask(p.out + (int64_t)y * p.out_pitch, x, p.W, acc, p.vec_out);
    }
}

static hb_status sep_prepare(SepArgs& a, const hb_half* in, float* out, int H, int W,
                             int64_t in_pitch, int64_t out_pitch,
                             const hb_half* tx, int ntx, int ax, const hb_half* ty, int nty, int ay) {
    hb_status s = check_image(in, out, H, W, in_pitch, out_pitch);
    if (s != HB_OK) return s;
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
    a.dmin = floor_div(-ax, 32);
    a.nct = ceil_div(W, 64);
    const int rowsteps = ceil_div(H, 16);
    // enough tasks to fill the chip, few enough that the (NT-1)-tile warm-up stays small
    int steps = (int)(((int64_t)rowsteps * a.nct) / 4096);
    steps = steps < 1 ? 1 : (steps > 16 ? 16 : steps);
    a.steps = steps;
    a.nseg = ceil_div(rowsteps, steps);
    a.ntasks = a.nct * a.nseg;
    a.vec_in = aligned_to(in, 16) && (in_pitch % 8 == 0);
    a.vec_out = aligned_to(out, 16) && (out_pitch % 4 == 0);
    a.tx = pack_taps(tx, ntx);
    a.ty = pack_taps(ty, nty);
    return HB_OK;
}

template <int ND>
static void sep_launch_nt(int nt, int blocks, hipStream_t st, const SepArgs& a) {
    switch (nt) {
        case 1: hipLaunchKernelGGL((sepblur_mfma_kernel<ND, 1>), dim3(blocks), dim3(256), 0, st, a); break;
        case 2: hipLaunchKernelGGL((sepblur_mfma_kernel<ND, 2>), dim3(blocks), dim3(256), 0, st, a); break;
        case 3: hipLaunchKernelGGL((sepblur_mfma_kernel<ND, 3>), dim3(blocks), dim3(256), 0, st, a); break;
        case 4: hipLaunchKernelGGL((sepblur_mfma_kernel<ND, 4>), dim3(blocks), dim3(256), 0, st, a); break;
        default: hipLaunchKernelGGL((sepblur_mfma_kernel<ND, 5>), dim3(blocks), dim3(256), 0, st, a); break;
    }
}

}  // namespace hb

extern "C" hb_status hb_sepblur(const hb_half* in, float* out, int H, int W,
                                int64_t in_pitch, int64_t out_pitch,
                                const hb_half* taps_x_host, int ntaps_x, int anchor_x,
                                const hb_half* taps_y_host, int ntaps_y, int anchor_y, hb_stream stream) {
    using namespace hb;
    SepArgs a;
    hb_status s = sep_prepare(a, in, out, H, W, in_pitch, out_pitch, taps_x_host, ntaps_x, anchor_x,
                              taps_y_host, ntaps_y, anchor_y);
    if (s != HB_OK) return s;
    const int dmax = floor_div(31 - anchor_x + ntaps_x - 1, 32);
    const int nd = dmax - a.dmin + 1;
    const int nt = (ntaps_y + 30) / 16;
    const int blocks = min(ceil_div(a.ntasks, 4), kMaxStreamBlocks);
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    switch (nd) {
        case 1: sep_launch_nt<1>(nt, blocks, st, a); break;
        case 2: sep_launch_nt<2>(nt, blocks, st, a); break;
        case 3: sep_launch_nt<3>(nt, blocks, st, a); break;
        case 4: sep_launch_nt<4>(nt, blocks, st, a); break;
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
