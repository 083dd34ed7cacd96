// hb_resize: separable resampling by a non-integer factor with precomputed banded matrices, and
// its vector-ALU twin (Sec. V-C); hb_lanczos3_matrix builds such a matrix on the host.
//
// Each axis is one sparse matrix: row o holds `band` coefficients for the input samples
// start[o] .. start[o] + band - 1.  As in the paper the matrix is treated as block-sparse: the 16
// rows of an aligned group share one starting index (the smallest of theirs, moved to an even
// sample) and the band is widened to cover all of them, at the price of some multiplications by
// zero.  A group of 16 outputs is then a dense 16 x (32 NK) coefficient block, and 16 image rows
// times that block is NK products of the usual kind: the image operand is 8 consecutive samples of
// one row per lane, straight from memory.
//
// One kernel does both axes.  It contracts over the memory-contiguous index of its input and writes
// its result TRANSPOSED, Z[o][r] = sum_j X[r][start[o] + j] coef[o][j]: the horizontal pass turns the
// image into T^T[xo][y] (rounded to fp16, kept in the workspace), so the vertical pass finds its
// contraction index y contiguous again and its transposed result is the output in its natural
// orientation.  The accumulators leave with a lane owning four consecutive r of one o, which is four
// consecutive elements of a row of Z.
#include <math.h>

#include "hb_device.hpp"
#include "hb_host.hpp"

namespace hb {

constexpr int kRzTiles = 4;                   // 16-row tiles of X per wave (64 rows r)
constexpr int kRzWaves = 2;                   // waves per workgroup: 2 strips of 64 rows, one group of 16 outputs (measured: 1, 4, 8 are slower)
constexpr int kRzMaxChunks = HB_RESIZE_MAX_SPAN / 32;

struct BandArgs {
    const half_t* x;                          // [planes][rows][len], row pitch x_pitch, plane stride x_plane
    void* z;                                  // [planes][nout][rows] transposed result, fp16 or fp32
    const int* start;                         // device: nout first input indices
    const half_t* coef;                       // device: nout x band coefficients
    int rows, len, nout, band, planes;
    int64_t x_pitch, x_plane, z_pitch, z_plane;
    int ngroups, nruns;                       // groups of 16 outputs; runs of kRzWaves strips per plane
};

// Sixteen rows of 64 floats from the accumulators (lane (c, g): row c, columns 16 w + 4 g ..) to
// fp16 rows in memory, through the wave's LDS patch so that a row leaves as one 128-byte run.
template <int NW>
__device__ __forceinline__ void rz_store_rows_half(float* patch, half_t* dst, uint32_t pitch_elems,
                                                   const floatx4 (&acc)[NW], int lane) {
    const int c = lane & 15, g = lane >> 4;
#pragma unroll
    for (int w = 0; w < NW; ++w)
        *reinterpret_cast<floatx4*>(patch + c * RowPatch<NW>::kPitch + 16 * w + 4 * g) = acc[w];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    constexpr int kLanesPerRow = 4 * NW, kRowsPerPass = 64 / kLanesPerRow;
    const int rr = lane / kLanesPerRow, xq = lane - rr * kLanesPerRow;
#pragma unroll
    for (int s = 0; s < 16 / kRowsPerPass; ++s) {
        const int row = s * kRowsPerPass + rr;
        const floatx4 v = *reinterpret_cast<const floatx4*>(patch + row * RowPatch<NW>::kPitch + 4 * xq);
        const half4 h = {(half_t)v[0], (half_t)v[1], (half_t)v[2], (half_t)v[3]};
        *reinterpret_cast<half4_u*>(dst + (size_t)row * pitch_elems + 4 * xq) = h;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <bool OUT_HALF>
__global__ void __launch_bounds__(64 * kRzWaves) band_mfma_kernel(BandArgs p) {
    constexpr int NW = kRzTiles;
    // The coefficient block and, once the products are done, the waves' store patches share one piece
    // of LDS: with both resident a compute unit held too few workgroups to cover the grid in one round.
    constexpr int kFragBytes = kRzMaxChunks * 64 * 16, kPatchBytes = kRzWaves * RowPatch<NW>::kFloats * 4;
    __shared__ __attribute__((aligned(16))) char s_mem[kFragBytes > kPatchBytes ? kFragBytes : kPatchBytes];
    half8* s_frag = reinterpret_cast<half8*>(s_mem);
    float* s_patch = reinterpret_cast<float*>(s_mem);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    // neighbouring groups read neighbouring pieces of the same rows: walk them back to back inside one XCD
    int wg = xcd_contiguous(blockIdx.x, gridDim.x);
    const int grp = wg % p.ngroups;
    wg /= p.ngroups;
    const int run = wg % p.nruns, plane = wg / p.nruns;
    const int o0 = 16 * grp;

    // geometry of the group: first sample (even) and number of 32-sample chunks.  Lane column c
    // reads the start of output o0 + c; the minimum and maximum over the 16 columns come from four
    // butterfly steps inside each row of 16 lanes, so every lane ends up with the same numbers.
    // A start below -band (above len - 1) reads nothing but the first (last) sample, and so does
    // -band (len - 1): clamping it there changes no result and bounds the span by the image.
    const int o = o0 + c;
    const bool live = o < p.nout;
    const int st = live ? clampi(p.start[o], -p.band, p.len - 1) : 0;
    int lo = live ? st : 0x7fffffff, hi = live ? st + p.band : -0x7fffffff;
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) {
        lo = min(lo, __shfl_xor(lo, off, 64));
        hi = max(hi, __shfl_xor(hi, off, 64));
    }
    const int first = lo & ~1, nk_all = (hi - first + 31) / 32;

    const int r0 = 64 * (kRzWaves * run + wv);            // this wave's strip of rows
    const bool active = r0 < p.rows;
    const half_t* xpl = p.x + (size_t)plane * p.x_plane;
    const uint32_t rowbytes = (uint32_t)p.x_pitch * 2u;
    uint32_t rowoff[NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) rowoff[w] = (uint32_t)min(r0 + 16 * w + c, p.rows - 1) * rowbytes;

    auto load_chunk = [&](int kk, half8 (&d)[NW]) {
        const int xs = first + 32 * kk;                   // uniform
        if (xs >= 0 && xs + 32 <= p.len) {
#pragma unroll
            for (int w = 0; w < NW; ++w) d[w] = ldg8(xpl, rowoff[w] + 2u * (uint32_t)(xs + 8 * g));
        } else {
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int x = clampi(xs + 8 * g + i, 0, p.len - 1);
                    d[w][i] = *reinterpret_cast<const half_t*>(reinterpret_cast<const char*>(xpl) + (rowoff[w] + 2u * (uint32_t)x));
                }
        }
    };
    floatx4 acc[NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) acc[w] = floatx4{0.f, 0.f, 0.f, 0.f};
    half8 bufa[NW], bufb[NW];
    // The coefficient block holds kRzMaxChunks chunks; a group that spans more (a very large factor,
    // or starts that jump inside the group) takes several rounds of block + products.
    for (int base = 0; base < nk_all; base += kRzMaxChunks) {
        const int nk = min(nk_all - base, kRzMaxChunks);
        if (base) __syncthreads();                        // every wave is done with the previous block
        // the first window chunk is requested before the coefficient block is built
        if (active) load_chunk(base, bufa);

        // coefficient block, B-operand layout: lane (c = o, g) holds B[8g + i][o] = coef[o][first + 32 kk + 8g + i - start[o]];
        // wave wv builds chunks wv, wv + kRzWaves, ...
        for (int kk = wv; kk < nk; kk += kRzWaves) {
            half8 f;
#pragma unroll
            for (int i = 0; i < 8; ++i) f[i] = (half_t)0;
            if (live) {
                const int t0 = first + 32 * (base + kk) + 8 * g - st;
                const half_t* row = p.coef + (size_t)o * p.band;
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (t0 + i >= 0 && t0 + i < p.band) f[i] = row[t0 + i];
            }
            s_frag[kk * 64 + lane] = f;
        }
        __syncthreads();

        // two window buffers used alternately: the next chunk is in flight while this one is multiplied
        auto use_chunk = [&](int kk, const half8 (&d)[NW]) {
            const half8 f = s_frag[kk * 64 + lane];
#pragma unroll
            for (int w = 0; w < NW; ++w) acc[w] = mfma16x16x32(d[w], f, acc[w]);
        };
        for (int kk = 0; active && kk < nk; kk += 2) {
            if (kk + 1 < nk) load_chunk(base + kk + 1, bufb);
            use_chunk(kk, bufa);
            if (kk + 1 >= nk) break;
            if (kk + 2 < nk) load_chunk(base + kk + 2, bufa);
            use_chunk(kk + 1, bufb);
        }
    }
    __syncthreads();                                      // every wave is done with the coefficient block
    if (!active) return;

    // D[m = r][n = o]: lane (c = o, g) holds rows r0 + 16 w + 4 g .. + 3 = four consecutive elements of Z's row o
    float* patch = s_patch + wv * RowPatch<NW>::kFloats;
    const bool whole = o0 + 16 <= p.nout && r0 + 64 <= p.rows;
    if (OUT_HALF) {
        half_t* z = reinterpret_cast<half_t*>(p.z) + (size_t)plane * p.z_plane;
        if (whole) {
            rz_store_rows_half<NW>(patch, z + (size_t)o0 * p.z_pitch + r0, (uint32_t)p.z_pitch, acc, lane);
        } else if (o0 + c < p.nout) {
            half_t* row = z + (size_t)(o0 + c) * p.z_pitch;
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int r = r0 + 16 * w + 4 * g + j;
                    if (r < p.rows) row[r] = (half_t)acc[w][j];
                }
        }
    } else {
        float* z = reinterpret_cast<float*>(p.z) + (size_t)plane * p.z_plane;
        if (whole) {
            store_rows_via_lds<NW, true>(patch, z + (size_t)o0 * p.z_pitch + r0, (uint32_t)p.z_pitch, acc, lane);
        } else if (o0 + c < p.nout) {
            float* row = z + (size_t)(o0 + c) * p.z_pitch;
#pragma unroll
            for (int w = 0; w < NW; ++w) store4_mask(row, r0 + 16 * w + 4 * g, p.rows, acc[w]);
        }
    }
}

// Vector-ALU twin of one pass.  A workgroup takes one group of 16 outputs and 64 rows of X: the samples
// the group reads (from its smallest start on, 256 at a time, every index clamped) are staged in LDS
// with coalesced row loads; a thread owns one output o and four rows, reads a coefficient once and
// uses it for its four rows; the four results are consecutive elements of row o of the transposed Z.
constexpr int kRzvChunk = 256;                // staged samples per row and round
constexpr int kRzvPitch = kRzvChunk + 8;      // halves

template <bool OUT_HALF>
__global__ void __launch_bounds__(256) band_valu_kernel(BandArgs p) {
    __shared__ __attribute__((aligned(16))) half_t s_x[64 * kRzvPitch];
    const int tid = threadIdx.x;
    int wg = blockIdx.x;
    const int grp = wg % p.ngroups;
    wg /= p.ngroups;
    const int nblk = (p.rows + 63) / 64;
    const int blk = wg % nblk, plane = wg / nblk;
    const int r0 = 64 * blk;
    const int o = 16 * grp + (tid & 15), rq = tid >> 4;
    const bool live = o < p.nout;
    const int st = live ? clampi(p.start[o], -p.band, p.len - 1) : 0;   // same samples as the unclamped start
    int lo = live ? st : 0x7fffffff, hi = live ? st + p.band : -0x7fffffff;
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) {
        lo = min(lo, __shfl_xor(lo, off, 64));
        hi = max(hi, __shfl_xor(hi, off, 64));
    }
    const half_t* xpl = p.x + (size_t)plane * p.x_plane;
    const half_t* k = p.coef + (size_t)(live ? o : 0) * p.band;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int base = lo; base < hi; base += kRzvChunk) {
        const int n = min(kRzvChunk, hi - base);          // samples of this round
        const int nch = (n + 7) / 8;
        if (base != lo) __syncthreads();                  // everyone is done with the previous round
        for (int idx = tid; idx < 64 * nch; idx += 256) {
            const int r = idx / nch, ch = idx - r * nch;
            const half_t* row = xpl + (size_t)min(r0 + r, p.rows - 1) * p.x_pitch;
            *reinterpret_cast<half8*>(&s_x[r * kRzvPitch + 8 * ch]) = load8_clamp(row, base + 8 * ch, p.len);
        }
        __syncthreads();
        if (live) {
            const int j0 = max(0, base - st), j1 = min(p.band, base + n - st);
            for (int j = j0; j < j1; ++j) {
                const float c = (float)k[j];
                const half_t* src = &s_x[4 * rq * kRzvPitch + (st + j - base)];
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[q] = fmaf(c, (float)src[q * kRzvPitch], acc[q]);
            }
        }
    }
    if (!live) return;
    const int r = r0 + 4 * rq;
    if (OUT_HALF) {
        half_t* z = reinterpret_cast<half_t*>(p.z) + (size_t)plane * p.z_plane + (size_t)o * p.z_pitch;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (r + q < p.rows) z[r + q] = (half_t)acc[q];
    } else {
        float* z = reinterpret_cast<float*>(p.z) + (size_t)plane * p.z_plane + (size_t)o * p.z_pitch;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (r + q < p.rows) z[r + q] = acc[q];
    }
}

static int64_t rz_pitch(int H) { return ((int64_t)H + 7) & ~(int64_t)7; }

static hb_status resize_run(bool valu, const hb_half* in, float* out, void* workspace, size_t workspace_bytes,
                            int C, int H, int W, int Ho, int Wo,
                            int64_t in_pitch, int64_t in_plane, int64_t out_pitch, int64_t out_plane,
                            const int32_t* start_y, const hb_half* coef_y, int band_y,
                            const int32_t* start_x, const hb_half* coef_x, int band_x, hb_stream stream) {
    if (!in || !out || !start_y || !coef_y || !start_x || !coef_x) return HB_ERR_INVALID_ARG;
    if (C < 1 || H < 1 || W < 1 || Ho < 1 || Wo < 1) return HB_ERR_INVALID_ARG;
    if (band_y < 1 || band_x < 1 || band_y > HB_RESIZE_MAX_SPAN || band_x > HB_RESIZE_MAX_SPAN) return HB_ERR_INVALID_ARG;
    if (in_pitch < W || out_pitch < Wo) return HB_ERR_INVALID_ARG;
    if (C > 1 && (in_plane < (int64_t)H * in_pitch || out_plane < (int64_t)Ho * out_pitch)) return HB_ERR_INVALID_ARG;
    if (!aligned_to(in, 2) || !aligned_to(out, 4) || !aligned_to(start_y, 4) || !aligned_to(start_x, 4) ||
        !aligned_to(coef_y, 2) || !aligned_to(coef_x, 2))
        return HB_ERR_INVALID_ARG;
    const int64_t hp = rz_pitch(H);
    // lanes address the rows of a plane with 32-bit byte offsets
    if ((int64_t)H * in_pitch >= ((int64_t)1 << 31) || (int64_t)Wo * hp >= ((int64_t)1 << 31) ||
        (int64_t)Ho * out_pitch >= ((int64_t)1 << 30) || C > 65535)
        return HB_ERR_UNSUPPORTED;
    const size_t need = hb_resize_workspace_size(C, H, Wo);
    if (!workspace || workspace_bytes < need || !aligned_to(workspace, 256)) return HB_ERR_WORKSPACE;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);

    BandArgs a;
    // horizontal: image rows y, contraction over x, result T^T[xo][y] in fp16
    a.x = reinterpret_cast<const half_t*>(in);
    a.z = workspace;
    a.start = start_x;
    a.coef = reinterpret_cast<const half_t*>(coef_x);
    a.rows = H;
    a.len = W;
    a.nout = Wo;
    a.band = band_x;
    a.planes = C;
    a.x_pitch = in_pitch;
    a.x_plane = in_plane;
    a.z_pitch = hp;
    a.z_plane = (int64_t)Wo * hp;
    BandArgs b;
    // vertical: rows of T^T, contraction over y, result out[yo][xo] in fp32
    b.x = reinterpret_cast<const half_t*>(workspace);
    b.z = out;
    b.start = start_y;
    b.coef = reinterpret_cast<const half_t*>(coef_y);
    b.rows = Wo;
    b.len = H;
    b.nout = Ho;
    b.band = band_y;
    b.planes = C;
    b.x_pitch = hp;
    b.x_plane = (int64_t)Wo * hp;
    b.z_pitch = out_pitch;
    b.z_plane = out_plane;
    for (BandArgs* q : {&a, &b}) {
        q->ngroups = ceil_div(q->nout, 16);
        q->nruns = ceil_div(q->rows, 64 * kRzWaves);
        if (valu) {
            const int64_t blocks = (int64_t)q->planes * q->ngroups * ceil_div(q->rows, 64);
            if (blocks > 0x7fffffff) return HB_ERR_UNSUPPORTED;
            if (q == &a) hipLaunchKernelGGL(band_valu_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, st, *q);
            else hipLaunchKernelGGL(band_valu_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, st, *q);
        } else {
            const int64_t blocks = (int64_t)q->planes * q->ngroups * q->nruns;
            if (blocks > 0x7fffffff) return HB_ERR_UNSUPPORTED;
            if (q == &a) hipLaunchKernelGGL(band_mfma_kernel<true>, dim3((unsigned)blocks), dim3(64 * kRzWaves), 0, st, *q);
            else hipLaunchKernelGGL(band_mfma_kernel<false>, dim3((unsigned)blocks), dim3(64 * kRzWaves), 0, st, *q);
        }
        const hb_status s = launch_status();
        if (s != HB_OK) return s;
    }
    return HB_OK;
}

}  // namespace hb

extern "C" size_t hb_resize_workspace_size(int C, int H, int Wo) {
    if (C < 1 || H < 1 || Wo < 1) return 0;
    return (size_t)C * (size_t)Wo * (size_t)hb::rz_pitch(H) * sizeof(uint16_t);
}

extern "C" hb_status hb_resize(const hb_half* in, float* out, void* workspace, size_t workspace_bytes,
                               int C, int H, int W, int Ho, int Wo,
                               int64_t in_pitch, int64_t in_plane, int64_t out_pitch, int64_t out_plane,
                               const int32_t* start_y, const hb_half* coef_y, int band_y,
                               const int32_t* start_x, const hb_half* coef_x, int band_x, hb_stream stream) {
    return hb::resize_run(false, in, out, workspace, workspace_bytes, C, H, W, Ho, Wo, in_pitch, in_plane, out_pitch,
                          out_plane, start_y, coef_y, band_y, start_x, coef_x, band_x, stream);
}

extern "C" hb_status hb_resize_valu(const hb_half* in, float* out, void* workspace, size_t workspace_bytes,
                                    int C, int H, int W, int Ho, int Wo,
                                    int64_t in_pitch, int64_t in_plane, int64_t out_pitch, int64_t out_plane,
                                    const int32_t* start_y, const hb_half* coef_y, int band_y,
                                    const int32_t* start_x, const hb_half* coef_x, int band_x, hb_stream stream) {
    return hb::resize_run(true, in, out, workspace, workspace_bytes, C, H, W, Ho, Wo, in_pitch, in_plane, out_pitch,
                          out_plane, start_y, coef_y, band_y, start_x, coef_x, band_x, stream);
}

extern "C" int hb_lanczos3_band(int n_in, int n_out) {
    if (n_in < 1 || n_out < 1 || n_out > n_in) return 0;
    return (int)floor(6.0 * (double)n_in / (double)n_out) + 1;
}

extern "C" hb_status hb_lanczos3_matrix(int n_in, int n_out, int32_t* start_host, hb_half* coef_host) {
    const int band = hb_lanczos3_band(n_in, n_out);
    if (band == 0 || !start_host || !coef_host) return HB_ERR_INVALID_ARG;
    if (band > HB_RESIZE_MAX_SPAN) return HB_ERR_UNSUPPORTED;
    const double pi = 3.14159265358979323846, scale = (double)n_in / (double)n_out;
    double w[HB_RESIZE_MAX_SPAN];
    for (int o = 0; o < n_out; ++o) {
        const double centre = (o + 0.5) * scale - 0.5;
        const int first = (int)ceil(centre - 3.0 * scale);
        double sum = 0.0;
        for (int j = 0; j < band; ++j) {
            const double x = ((double)(first + j) - centre) / scale;
            double v = 0.0;
            if (fabs(x) < 3.0) v = x == 0.0 ? 1.0 : (sin(pi * x) / (pi * x)) * (sin(pi * x / 3.0) / (pi * x / 3.0));
            w[j] = v;
            sum += v;
        }
        start_host[o] = first;
        for (int j = 0; j < band; ++j) coef_host[(size_t)o * band + j] = hb::float_to_half_bits((float)(w[j] / sum));
    }
    return HB_OK;
}
