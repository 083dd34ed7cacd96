// hb_conv2d: single-channel 2-D convolution with an arbitrary (non-separable) kernel, and its
// vector-ALU twin (Sec. V-A, 2-D form: O(x, y) = sum_{rx, ry} I(x + rx, y + ry) K(rx, ry)).
//
// MFMA formulation: the serial loop over the kernel rows r_y of Sec. V-A.  For every r_y the
// contribution is a row-wise FIR with taps K(., r_y), i.e. one Toeplitz product per tile as in
// hb_fir1d (transposed: D[m][n] = sum_k A_ry[m][k] P[k][n], m = output column, n = image row in a
// 16-row group, k = pixel in the window).  The kh Toeplitz fragments per 32-pixel window chunk are
// built once per workgroup into LDS.
//
// The image operand P of a product lives in registers, one image row per lane column n, so the
// straightforward loop (rows shifted down by r_y for every r_y) would fetch a new operand for every
// product.  Instead the kernel keeps the INPUT rows fixed: a wave walks down a strip of 64 columns
// one group of 16 input rows at a time, loads that group's windows once, and multiplies them with
// all kh Toeplitz matrices.  The product for kernel row r_y holds, in lane column n, the contribution
// of input row r to output row r - r_y + anchor_y: the whole product tile is the output tile moved by
// r_y rows.  With the input groups placed at rows 16 G - anchor_y, kernel row b < 16 applied to input
// group G and kernel row b + 16 applied to input group G + 1 are moved by the same b rows relative
// to output group G, so their products are accumulated in one tile by the matrix unit (the second
// product takes the first as its addend) and the tile is then added into the accumulators of output
// groups G (rows n >= b) and G - 1 (rows n < b) with two lane-shifted additions inside each row of
// 16 lanes (DPP row shifts; lanes shifted out of the row are not written).  Two output groups are
// open at a time; the older one is complete after every step and is stored.  The lane-shifted
// additions are what bounds the kernel (they issue at half the rate of plain additions), which is
// why sharing one shift between two kernel rows matters.
//
// The clamp along x needs no folded fragments here: the Toeplitz matrix is indexed by the window
// position, so a strip whose windows reach over the left or right image border only loads its
// windows pixel by pixel with the column clamped (once per 16 input rows, shared by all kh
// products); the products themselves are the same.
#include "hb_device.hpp"
#include "hb_host.hpp"
#include "walk2d.hpp"

namespace hb {

struct Conv2dArgs {
    const half_t* in;
    float* out;
    int H, W;
    int64_t in_pitch, out_pitch;
    int kh, kw, ay, ax;
    // matrix kernel: nstrips strips of 64 columns; a task = one strip x seg_len output row groups;
    // ngroups = output row groups of the image
    int nstrips, ngroups, seg_len, nseg, ntasks;
    uint16_t taps[HB_MAX_TAPS_CONV2D * HB_MAX_TAPS_CONV2D];   // kh x kw, row-major
};

// ---------------------------------------------------------------------------
// Matrix-unit kernel.  NK = 32-pixel chunks of a tile's window (16 + kw - 1 pixels from x0 - ax on,
// one more when the window is moved to an even pixel); KH16 = kernel rows in units of 16 (the
// fragment table is padded with zero rows up to 16 KH16).
template <int NK, int KH16, bool STREAM>
__global__ void __launch_bounds__(kC2Threads) conv2d_mfma_kernel(Conv2dArgs p) {
    constexpr int NW = kC2Tiles;
    constexpr int KR = 16 * KH16;
    extern __shared__ __attribute__((aligned(16))) char s_dyn[];
    // [KR][NK][64 lanes] fragments, then one row patch per wave
    half8* s_frag = reinterpret_cast<half8*>(s_dyn);
    float* s_patch = reinterpret_cast<float*>(s_dyn + (size_t)KR * NK * 1024);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int e = p.ax & 1;
    const int aw = p.ax + e;                  // window start, left of the tile (even pixel)

    // Toeplitz fragments, A-operand layout: lane (c, g) holds A[c][32 kk + 8g + i] = K(32 kk + 8g + i - c - e, ry)
    for (int idx = tid; idx < KR * NK * 64; idx += kC2Threads) {
        const int l = idx & 63, kk = (idx >> 6) % NK, ry = idx / (64 * NK);
        const int t0 = 32 * kk + 8 * (l >> 4) - (l & 15) - e;
        half8 f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int t = t0 + i;
            f[i] = (ry < p.kh && t >= 0 && t < p.kw) ? __builtin_bit_cast(half_t, p.taps[ry * p.kw + t]) : (half_t)0;
        }
        s_frag[idx] = f;
    }
    __syncthreads();

    // plain launch order: with every XCD on one contiguous run of the tasks the halo windows meet in one
    // L2 (reads 1.25x the image instead of 1.57x) but the kernel measured 7 % slower at 4096 x 4096
    const int task = blockIdx.x * (kC2Threads / 64) + wv;
    if (task >= p.ntasks) return;
    const int sg = task / p.nstrips, ct = task - sg * p.nstrips;
    const int x0 = 16 * NW * ct;
    const int q0 = sg * p.seg_len, q1 = min(q0 + p.seg_len, p.ngroups);   // output groups of this task
    float* patch = s_patch + wv * RowPatch<NW>::kFloats;
    const uint32_t rowbytes = (uint32_t)p.in_pitch * 2u;
    // windows of the strip: pixels x0 - aw .. x0 - aw + 32 NK + 47; inside the row for interior strips
    const bool inside = x0 - aw >= 0 && x0 - aw + 32 * NK + 48 <= p.W;
    const bool whole = x0 + 16 * NW <= p.W;                // all 64 output columns exist
    const half_t* src = p.in + (x0 - aw);                 // uniform; lanes add row * pitch + 8g
    float* dst = p.out + x0;

    auto load_group = [&](int G, half8 (&d)[NW][NK]) {
        // input rows 16 G - anchor_y + c, clamped into the image
        const int yr = clampi(16 * G - p.ay + c, 0, p.H - 1);
        if (inside) {
            const uint32_t off = (uint32_t)yr * rowbytes + 16u * g;
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) d[w][kk] = ldg8(src, off + 2u * (16u * w + 32u * kk));
        } else {
            // pixel by pixel, column clamped; 32-bit byte offsets from the image base
            const uint32_t rowoff = (uint32_t)yr * rowbytes;
            const int xs = x0 - aw + 8 * g;
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int kk = 0; kk < NK; ++kk)
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int x = clampi(xs + 16 * w + 32 * kk + i, 0, p.W - 1);
                        d[w][kk][i] = *reinterpret_cast<const half_t*>(reinterpret_cast<const char*>(p.in) + (rowoff + 2u * (uint32_t)x));
                    }
        }
    };
    auto store_group = [&](int Q, const floatx4 (&acc)[NW]) {
        const int y0 = 16 * Q;
        if (whole && y0 + 16 <= p.H) {
            store_rows_via_lds<NW, STREAM>(patch, dst + (int64_t)y0 * p.out_pitch, (uint32_t)p.out_pitch, acc, lane);
        } else if (y0 + c < p.H) {
            float* row = p.out + (int64_t)(y0 + c) * p.out_pitch;
#pragma unroll
            for (int w = 0; w < NW; ++w) store4_mask(row, x0 + 16 * w + 4 * g, p.W, acc[w]);
        }
    };

    floatx4 ring[2][NW], done[NW];            // open groups G - 1 and G; the group completed by the previous step
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        ring[0][w] = floatx4{0.f, 0.f, 0.f, 0.f};
        ring[1][w] = floatx4{0.f, 0.f, 0.f, 0.f};
        done[w] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
    half8 wa[NW][NK], wb[NW][NK], wc[NW][NK];
    load_group(q0, wa);
    load_group(q0 + 1, wb);
    // Output group Q takes its rows n >= b parts in step Q and its rows n < b parts in step Q + 1:
    // steps q0 .. q1 complete the groups q0 .. q1 - 1.
#pragma unroll 1
    for (int G = q0; G <= q1; ++G) {
        // The finished group leaves before this step's loads are issued: loads and stores share one
        // counter, and a wait for the loads would otherwise also wait for the write
        // acknowledgements of stores issued just before it.
        if (G - 2 >= q0) store_group(G - 2, done);
        load_group(G + 2, wc);                // clamped rows: always inside the image
        // The fragment reads do not depend on G; left alone the compiler lifts all of them out of
        // the loop and spills.  An opaque copy of the lane index keeps them inside.
        int fl = lane;
        asm volatile("" : "+v"(fl));
        c2_step<NK, KH16 == 2>(s_frag, fl, p.kh, p.kh - 16, wa, wb, ring);
        // ring[0] = group G - 1 is complete: no later input group reaches it
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            done[w] = ring[0][w];
            ring[0][w] = ring[1][w];
            ring[1][w] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) {
                wa[w][kk] = wb[w][kk];
                wb[w][kk] = wc[w][kk];
            }
        }
    }
    if (q1 > q0) store_group(q1 - 1, done);
}

// ---------------------------------------------------------------------------
// Vector-ALU kernel: a 16 x 128 output tile per workgroup.  The tile and its halo are staged in LDS
// as fp32 with both indices clamped (the definition's border rule verbatim).  A thread owns 8
// consecutive outputs of one row: for every kernel row it reads the 8 + KWP - 1 pixels under them
// once (16-byte LDS reads) and slides the taps over them in registers, 8 FMAs per tap read.
// KWP = kernel width rounded up to 8, 16 or 32; the taps beyond kw are zeros.
constexpr int kC2vW = 128;
constexpr int kC2vRows = 16 + HB_MAX_TAPS_CONV2D - 1;                 // 47
constexpr int kC2vPitch = kC2vW + HB_MAX_TAPS_CONV2D;                  // 160 floats

template <int KWP>
__global__ void __launch_bounds__(256) conv2d_valu_kernel(Conv2dArgs p) {
    __shared__ __attribute__((aligned(16))) float s_px[kC2vRows * kC2vPitch];
    __shared__ float s_k[HB_MAX_TAPS_CONV2D * KWP];
    for (int i = threadIdx.x; i < p.kh * KWP; i += 256) {
        const int ry = i / KWP, t = i - ry * KWP;
        s_k[i] = t < p.kw ? (float)__builtin_bit_cast(half_t, p.taps[ry * p.kw + t]) : 0.f;
    }
    const int nt = (p.W + kC2vW - 1) / kC2vW;
    const int rg = blockIdx.x / nt, tc = blockIdx.x - rg * nt;
    const int x0 = kC2vW * tc, y0 = 16 * rg;
    const int nrows = 16 + p.kh - 1;
    for (int idx = threadIdx.x; idx < nrows * kC2vPitch; idx += 256) {
        const int r = idx / kC2vPitch, cc = idx - r * kC2vPitch;
        float v = 0.f;                                    // columns only zero taps can reach stay zero
        if (cc < kC2vW + p.kw - 1) {
            const int y = clampi(y0 + r - p.ay, 0, p.H - 1), x = clampi(x0 + cc - p.ax, 0, p.W - 1);
            v = (float)p.in[(int64_t)y * p.in_pitch + x];
        }
        s_px[idx] = v;
    }
    __syncthreads();

    const int r = threadIdx.x >> 4, xl = 8 * (threadIdx.x & 15);
    const int y = y0 + r;
    if (y >= p.H || x0 + xl >= p.W) return;
    float acc[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] = 0.f;
    for (int ry = 0; ry < p.kh; ++ry) {
        float w[KWP + 8];
        const floatx4* src = reinterpret_cast<const floatx4*>(&s_px[(r + ry) * kC2vPitch + xl]);
#pragma unroll
        for (int i = 0; i < (KWP + 8) / 4; ++i) {
            const floatx4 v = src[i];
            w[4 * i] = v[0];
            w[4 * i + 1] = v[1];
            w[4 * i + 2] = v[2];
            w[4 * i + 3] = v[3];
        }
        const float* k = &s_k[ry * KWP];
#pragma unroll
        for (int t = 0; t < KWP; ++t) {
            const float kv = k[t];
#pragma unroll
            for (int q = 0; q < 8; ++q) acc[q] = fmaf(kv, w[t + q], acc[q]);
        }
    }
    float* row = p.out + (int64_t)y * p.out_pitch;
    store4_mask(row, x0 + xl, p.W, floatx4{acc[0], acc[1], acc[2], acc[3]});
    store4_mask(row, x0 + xl + 4, p.W, floatx4{acc[4], acc[5], acc[6], acc[7]});
}

static hb_status conv2d_prepare(Conv2dArgs& a, const hb_half* in, float* out, int H, int W,
                                int64_t in_pitch, int64_t out_pitch,
                                const hb_half* taps_host, int kh, int kw, int ay, int ax) {
    hb_status s = check_image(in, out, H, W, in_pitch, out_pitch);
    if (s != HB_OK) return s;
    // lanes address rows with 32-bit byte offsets from the image base
    if ((int64_t)H * in_pitch >= ((int64_t)1 << 31) || (int64_t)H * out_pitch >= ((int64_t)1 << 30)) return HB_ERR_UNSUPPORTED;
    if (!taps_host) return HB_ERR_INVALID_ARG;
    if (kh < 1 || kh > HB_MAX_TAPS_CONV2D || kw < 1 || kw > HB_MAX_TAPS_CONV2D) return HB_ERR_INVALID_ARG;
    if (ay < 0 || ay >= kh || ax < 0 || ax >= kw) return HB_ERR_INVALID_ARG;
    a.in = reinterpret_cast<const half_t*>(in);
    a.out = out;
    a.H = H;
    a.W = W;
    a.in_pitch = in_pitch;
    a.out_pitch = out_pitch;
    a.kh = kh;
    a.kw = kw;
    a.ay = ay;
    a.ax = ax;
    memset(a.taps, 0, sizeof(a.taps));
    memcpy(a.taps, taps_host, sizeof(uint16_t) * (size_t)kh * (size_t)kw);
    a.ngroups = ceil_div(H, 16);
    a.nstrips = a.seg_len = a.nseg = a.ntasks = 0;
    return HB_OK;
}

static hb_status conv2d_launch_valu(const Conv2dArgs& a, hipStream_t st) {
    const int64_t blocks = (int64_t)a.ngroups * ceil_div(a.W, kC2vW);
    if (blocks > 0x7fffffff) return HB_ERR_UNSUPPORTED;
    if (a.kw <= 8) hipLaunchKernelGGL(conv2d_valu_kernel<8>, dim3((unsigned)blocks), dim3(256), 0, st, a);
    else if (a.kw <= 16) hipLaunchKernelGGL(conv2d_valu_kernel<16>, dim3((unsigned)blocks), dim3(256), 0, st, a);
    else hipLaunchKernelGGL(conv2d_valu_kernel<32>, dim3((unsigned)blocks), dim3(256), 0, st, a);
    return launch_status();
}

}  // namespace hb

extern "C" hb_status hb_conv2d(const hb_half* in, float* out, int H, int W,
                               int64_t in_pitch, int64_t out_pitch,
                               const hb_half* taps_host, int kh, int kw, int anchor_y, int anchor_x,
                               hb_stream stream) {
    using namespace hb;
    Conv2dArgs a;
    hb_status s = conv2d_prepare(a, in, out, H, W, in_pitch, out_pitch, taps_host, kh, kw, anchor_y, anchor_x);
    if (s != HB_OK) return s;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const int e = anchor_x & 1;
    const int nk = ceil_div(15 + kw + e, 32);                // 1 or 2
    const int kh16 = ceil_div(kh, 16);
    a.nstrips = ceil_div(W, 16 * kC2Tiles);
    // One task per wave: a strip times a run of output row groups.  Every task walks
    // (kernel rows / 16) extra input groups, so runs are as long as filling the chip allows.
    const int waves = num_cu() * (kC2Threads / 64);
    int len = (int)(((int64_t)a.nstrips * a.ngroups + waves - 1) / waves);
    if (len < 2) len = a.ngroups < 2 ? a.ngroups : 2;
    a.seg_len = len;
    a.nseg = ceil_div(a.ngroups, len);
    const int64_t ntasks = (int64_t)a.nstrips * a.nseg;
    if (ntasks > 0x7fffffff / 2) return HB_ERR_UNSUPPORTED;
    a.ntasks = (int)ntasks;
    const size_t lds = (size_t)(16 * kh16) * nk * 1024 + (kC2Threads / 64) * RowPatch<kC2Tiles>::kFloats * sizeof(float);
    const int blocks = ceil_div(a.ntasks, kC2Threads / 64);
    const bool ss = (int64_t)H * W * 4 <= kStreamStoreMaxBytes;
#define HB_C2_LAUNCH(N, K, S)                                                                         \
    {                                                                                                 \
        if (allow_dynamic_lds(reinterpret_cast<const void*>(&conv2d_mfma_kernel<N, K, S>), lds) != HB_OK) \
            return HB_ERR_HIP;                                                                        \
        hipLaunchKernelGGL((conv2d_mfma_kernel<N, K, S>), dim3(blocks), dim3(kC2Threads), lds, st, a); \
    }
#define HB_C2_PICK(N, K) { if (ss) HB_C2_LAUNCH(N, K, true) else HB_C2_LAUNCH(N, K, false) }
    if (nk == 1 && kh16 == 1) HB_C2_PICK(1, 1)
    else if (nk == 1) HB_C2_PICK(1, 2)
    else if (kh16 == 1) HB_C2_PICK(2, 1)
    else HB_C2_PICK(2, 2)
#undef HB_C2_PICK
#undef HB_C2_LAUNCH
    return launch_status();
}

extern "C" hb_status hb_conv2d_valu(const hb_half* in, float* out, int H, int W,
                                    int64_t in_pitch, int64_t out_pitch,
                                    const hb_half* taps_host, int kh, int kw, int anchor_y, int anchor_x,
                                    hb_stream stream) {
    using namespace hb;
    Conv2dArgs a;
    hb_status s = conv2d_prepare(a, in, out, H, W, in_pitch, out_pitch, taps_host, kh, kw, anchor_y, anchor_x);
    if (s != HB_OK) return s;
    return conv2d_launch_valu(a, reinterpret_cast<hipStream_t>(stream));
}
