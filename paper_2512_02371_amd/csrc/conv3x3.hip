// hb_conv3x3: 64 -> 64 channel 3x3 convolution (stride 1, zero padding 1, NHWC) as an implicit
// GEMM on the matrix units (Sec. V-A 2-D form summed over channels; the conv layer of Sec. IV
// without bias and activation), and its vector-ALU twin.
//
// MFMA formulation, transposed so that a lane ends with consecutive output channels of one pixel:
//   O'[m][n] = sum_k Wt[m][k] * X[k][n]     m = output channel, n = pixel, k = (tap, input channel)
// with v_mfma_f32_32x32x16_f16: 32 channels x 32 pixels per product, K = 16 input channels.
//   A (coefficients): the 9 x 64 x 32 weights of one 32-channel tile live in the registers of a
//     wave for the whole kernel (36 K-steps x 8 halves per lane = 144 registers), gathered once.
//   B (pixels): a workgroup stages an (8+2) x (32+2) pixel tile of all 64 input channels in LDS in
//     the image's own order (pixel-major, 128 bytes per pixel), with the eight 16-byte channel
//     pieces of a pixel permuted by an XOR with bits 1..3 of the pixel index: a tile row then
//     arrives as contiguous 1 KB copies, and the 16-byte reads of 16 consecutive pixels at one
//     channel piece still fall into 64 different banks for every tap shift (the overlapped view of
//     Eq. 1: the three horizontal taps read the same LDS row at pixel offsets 0, 1, 2).  Pixels
//     outside the image arrive as zeros, which is the zero padding.
//   A workgroup has 8 waves, two per SIMD, so that one wave's LDS reads hide behind the other's
//   products: wave (q, j) owns output rows 2q, 2q+1 of the tile and channel tile j, i.e. 2 x 36
//   products per tile.  fp32 accumulators are rounded to fp16 (RNE) and leave through a small
//   wave-private LDS stage as 16-byte pieces.  There are three tile buffers: the tile after the
//   next is requested (global memory straight into LDS) before a wave starts multiplying.
// Workgroups are persistent (one per compute unit) and walk over the tiles.
#include "hb_device.hpp"
#include "hb_host.hpp"

namespace hb {

constexpr int kCvC = 64;                 // channels in and out
constexpr int kCvTY = 8, kCvTX = 32;     // output tile (rows x pixels) per workgroup step
constexpr int kCvRows = kCvTY + 2, kCvPx = kCvTX + 2;
constexpr int kCvLdsHalves = kCvRows * 4 * kCvPx * 16;

struct ConvArgs {
    const half_t* in;
    const half_t* w;
    half_t* out;
    int N, H, W;
    int tiles_x, tiles_y;      // per image
    int ntiles;                // N * tiles_y * tiles_x
};

// LDS layout of the vector-ALU twin: [row][16-channel chunk][8-channel half][pixel][8 channels].
__device__ __forceinline__ int cv_lds_index(int r, int kc, int half, int px) {
    return (((r * 4 + kc) * 2 + half) * kCvPx + px) * 8;
}

// LDS layout of the MFMA kernel, in 16-byte slots: pixel-major, channel piece cp of pixel px in slot
// cp ^ ((px >> 1) & 7) of the pixel's eight.
constexpr int kCvRowSlots = kCvPx * 8;                    // 272 slots = 4352 bytes per staged row
__device__ __forceinline__ int cv_slot(int r, int px, int cp) {
    return (r * kCvPx + px) * 8 + (cp ^ ((px >> 1) & 7));
}

// A staged tile is 2720 slots.  It is filled by buffer loads that write LDS directly (64 lanes x
// 16 bytes = 1 KB of consecutive LDS per instruction = 8 whole pixels, whose 128 bytes are
// contiguous in memory): no register holds a pixel on its way in.  43 such loads make a tile; wave
// w issues those numbered w, w + 8, ...: six for waves 0..2, five for the others.  Slots past the
// tile and pixels outside the image are requested beyond the end of the buffer descriptor, which
// makes the hardware deliver zeros: that is the zero padding of the convolution.
constexpr int kCvThreads = 512;
constexpr int kCvPieces = kCvRows * kCvRowSlots;                             // 2720
constexpr int kCvLoads = (kCvPieces + 63) / 64;                              // 43 per tile
constexpr int kCvDma = (kCvLoads + 7) / 8;                                   // at most 6 per wave
constexpr int kCvBufHalves = kCvLoads * 64 * 8;                              // 22016 halves = 43 KB, three of them
constexpr uint32_t kCvOutside = 0x80000000u;              // offset beyond any descriptor used here

struct CvTile {
    int n, y0, x0;
};
__device__ __forceinline__ CvTile cv_tile(const ConvArgs& p, int tile) {
    CvTile t;
    t.n = tile / (p.tiles_x * p.tiles_y);
    const int rem = tile - t.n * (p.tiles_x * p.tiles_y);
    const int ty = rem / p.tiles_x;
    t.y0 = ty * kCvTY;
    t.x0 = (rem - ty * p.tiles_x) * kCvTX;
    return t;
}
// whole staged tile inside the image?
__device__ __forceinline__ bool cv_interior(const ConvArgs& p, const CvTile& t) {
    return t.y0 >= 1 && t.y0 + kCvTY + 1 <= p.H && t.x0 >= 1 && t.x0 + kCvTX + 1 <= p.W;
}

// One LDS-direct load: 64 lanes x 16 bytes from base + voff (per lane) to 1 KB of LDS at lds_addr
// (wave-uniform).  Written as assembly so that the compiler keeps no book on it: it would make
// LDS reads of the other tile buffers wait for these loads, which are meant to stay in flight
// for two tiles.  The waits that order them are explicit in cv_step.
typedef uint32_t u32x4s __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void cv_dma16(u32x4s rsrc, uint32_t lds_addr, uint32_t voff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds_addr), "v"(voff), "s"(rsrc) : "memory");
}
__device__ __forceinline__ uint32_t cv_lds_addr(const half_t* p) {
    return (uint32_t)(size_t)(__attribute__((address_space(3))) const void*)p;
}

// A value the compiler must take as new: what is computed from it is computed again where it is
// used, instead of being kept in registers (or spilled) across the whole tile loop.
__device__ __forceinline__ int cv_fresh(int v) {
    asm volatile("" : "+v"(v));
    return v;
}

// Requests the staged tile of `t` into `buf` (this wave's share): 6 loads in waves 0..2, 5 in the others.
// Load number wv + 8 i fills slots 64 (wv + 8 i) + lane.
__device__ __forceinline__ void cv_request(const ConvArgs& p, const CvTile& t, half_t* buf, int wv, int lane) {
    // the descriptor starts at the (possibly virtual) pixel (y0-1, x0-1); lanes outside the image never
    // reach memory
    const uint64_t org = (uint64_t)(p.in + (((int64_t)t.n * p.H + (t.y0 - 1)) * p.W + (t.x0 - 1)) * kCvC);
    const u32x4s rs = {(uint32_t)org, (uint32_t)(org >> 32) & 0xffffu, 0x7fffffffu, 0x00020000u};
    const bool inside = cv_interior(p, t);                // uniform
    const uint32_t lds0 = cv_lds_addr(buf) + 1024u * wv;
    lane = cv_fresh(lane);
#pragma unroll
    for (int i = 0; i < kCvDma; ++i) {
        if (wv + 8 * i >= kCvLoads) break;                // uniform
        const int slot = 64 * (wv + 8 * i) + lane;
        const int r = (slot * 241) >> 16;                 // slot / 272 for slot < 2752
        const int px = (slot - r * kCvRowSlots) >> 3;
        const int cp = (lane & 7) ^ ((px >> 1) & 7);      // channel piece held by this slot
        uint32_t off = (uint32_t)(((r * p.W + px) * kCvC + 8 * cp) * 2);
        bool ok = slot < kCvPieces;
        if (!inside) {
            const int y = t.y0 - 1 + r, x = t.x0 - 1 + px;
            ok = ok && y >= 0 && y < p.H && x >= 0 && x < p.W;
        }
        cv_dma16(rs, lds0 + 8192u * i, ok ? off : kCvOutside);
    }
}

// Two output rows (2 x 32 pixels) x 32 channels from the staged tile.  The four staged rows under
// the two output rows are read once per (channel chunk, horizontal tap) and serve both rows:
// 48 reads for 72 products, in 12 groups of 4 reads + 6 products.  The reads of a group are issued
// kCvAhead groups before its products (the scheduling barriers pin that order), so that an LDS
// read has the time of 6 * kCvAhead products to return.
#ifndef HB_CONV_AHEAD
#define HB_CONV_AHEAD 1
#endif
constexpr int kCvAhead = HB_CONV_AHEAD;
__device__ __forceinline__ void cv_rows(const half_t* buf, const half8 (&wf)[36], int ro, int c32, int h,
                                        floatx16 (&acc)[2]) {
    // byte offset of (staged row ro, pixel c32 + kx) and the piece permutation there, per tap shift kx;
    // group 3 kc + kx reads channel piece 2 kc + h, which sits in slot (2 kc) ^ (h ^ s)
    c32 = cv_fresh(c32);
    const char* cbuf = reinterpret_cast<const char*>(buf);
    int apx[3], sw[3];
#pragma unroll
    for (int kx = 0; kx < 3; ++kx) {
        const int px = c32 + kx;
        apx[kx] = (ro * kCvPx + px) * 128;
        sw[kx] = 16 * (h ^ ((px >> 1) & 7));
    }
    half8 b[kCvAhead + 1][4];
    auto read_group = [&](int grp, half8 (&dst)[4]) {
        const int kc = grp / 3, kx = grp - 3 * kc;
        const char* a = cbuf + (apx[kx] + ((32 * kc) ^ sw[kx]));
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) dst[rr] = *reinterpret_cast<const half8*>(a + rr * (kCvRowSlots * 16));
    };
#pragma unroll
    for (int g0 = 0; g0 < kCvAhead; ++g0) {
        read_group(g0, b[g0]);
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
    }
#pragma unroll
    for (int grp = 0; grp < 12; ++grp) {
        const int kc = grp / 3, kx = grp - 3 * kc;
        if (grp + kCvAhead < 12) {
            read_group(grp + kCvAhead, b[(grp + kCvAhead) % (kCvAhead + 1)]);
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
        }
        const half8 (&bb)[4] = b[grp % (kCvAhead + 1)];
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            if (rr <= 2) acc[0] = mfma32x32x16(wf[(3 * rr + kx) * 4 + kc], bb[rr], acc[0]);
            if (rr >= 1) acc[1] = mfma32x32x16(wf[(3 * (rr - 1) + kx) * 4 + kc], bb[rr], acc[1]);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 6, 0);
    }
}

// The accumulators hold, per lane, one pixel and 16 scattered channels: stored as they are, one store
// instruction would touch 64 different 128-byte lines with 8 bytes each.  Each of the two output rows
// passes through a wave-private LDS stage (32 pixels x 32 channels of fp16, 80-byte pixel pitch:
// conflict-free 16-byte reads) and leaves as 16-byte pieces, four consecutive lanes per pixel: a store
// instruction then writes the 64 contiguous bytes of this wave's channel tile for 16 pixels.
constexpr int kCvStagePitch = 40;                         // halves per pixel in the stage
constexpr int kCvStageHalves = 32 * kCvStagePitch;        // 2560 bytes per wave
__device__ __forceinline__ void cv_store_rows(const ConvArgs& p, const CvTile& t, int ro, int j, int lane,
                                              const floatx16 (&acc)[2], half_t* stage) {
    const int c32 = lane & 31, h = lane >> 5;
    const int spx = lane >> 2, piece = lane & 3;
#pragma unroll
    for (int row = 0; row < 2; ++row) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            half4 v4;
#pragma unroll
            for (int r = 0; r < 4; ++r) v4[r] = (half_t)acc[row][4 * q + r];
            *reinterpret_cast<half4*>(stage + c32 * kCvStagePitch + 8 * q + 4 * h) = v4;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int y = t.y0 + ro + row;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int px = spx + 16 * half, x = t.x0 + px;
            const half8 v = *reinterpret_cast<const half8*>(stage + px * kCvStagePitch + 8 * piece);
            if (y < p.H && x < p.W)
                *reinterpret_cast<half8*>(p.out + (((int64_t)t.n * p.H + y) * p.W + x) * kCvC + 32 * j + 8 * piece) = v;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

// One tile: request the tile after the next into the third buffer, multiply this one, meet, store.
// The three buffers are distinct LDS arrays at every call site, so the reads of `cur` do not wait for
// loads into another buffer.  A request has two tile times to land: at the meeting point a wave waits
// for all its memory instructions but the kCvDma newest (the request just made; loads and stores
// retire in order), i.e. for its share of the NEXT tile and for the previous tile's stores.
__device__ __forceinline__ void cv_step(const ConvArgs& p, int lane, const half8 (&wf)[36],
                                        const half_t* cur, half_t* far, half_t* stage, int tile, int stride,
                                        int wv, int ro, int j, int c32, int h) {
    const CvTile t = cv_tile(p, tile);
    const bool req = tile + 2 * stride < p.ntiles;        // uniform
    if (req) cv_request(p, cv_tile(p, tile + 2 * stride), far, wv, lane);
    __builtin_amdgcn_sched_barrier(0);                    // the requests go out before the first product
    floatx16 acc[2];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[u][v] = 0.f;
    cv_rows(cur, wf, ro, c32, h, acc);
    __builtin_amdgcn_sched_barrier(0);
    static_assert(kCvLoads == 43, "the counted waits below are written for 6 / 5 loads per request");
    if (!req) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else if (wv < 3) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
    // The barrier instruction is written out: the compiler would put a wait for ALL memory
    // instructions in front of one it emits itself, and the newest request must stay in flight.
    // This wave's LDS reads have been consumed by its products by now (lgkmcnt(0) states it).
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // next buffer complete, this one released
    cv_store_rows(p, t, ro, j, lane, acc, stage);         // in flight during the next tile's products
}

__global__ void __launch_bounds__(kCvThreads) conv3x3_mfma_kernel(ConvArgs p) {
    __shared__ __attribute__((aligned(16))) half_t s_a[kCvBufHalves];
    __shared__ __attribute__((aligned(16))) half_t s_b[kCvBufHalves];
    __shared__ __attribute__((aligned(16))) half_t s_c[kCvBufHalves];
    __shared__ __attribute__((aligned(16))) half_t s_stage[8][kCvStageHalves];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c32 = lane & 31, h = lane >> 5;
    const int j = wv >> 2;                                // channel tile of this wave
    const int ro = 2 * (wv & 3);                          // its two output rows inside the tile

    int tile = blockIdx.x;
    if (tile >= p.ntiles) return;

    // coefficient fragments: wf[s] lane (c32, h) = w[tap][16 kc + 8h + i][32 j + c32], s = 4 tap + kc.
    // The 72 KB of weights pass through LDS once, taps 0..4 through one buffer and 5..8 through
    // another (coalesced 16-byte copies in, 2-byte gathers out: lanes of a half-wave read 32
    // consecutive halves, no bank conflict).
    half8 wf[36];
    constexpr int kTapHalves = kCvC * kCvC;
    for (int i = tid; i < 5 * kTapHalves / 8; i += kCvThreads)
        reinterpret_cast<half8*>(s_a)[i] = reinterpret_cast<const half8*>(p.w)[i];
    for (int i = tid; i < 4 * kTapHalves / 8; i += kCvThreads)
        reinterpret_cast<half8*>(s_b)[i] = reinterpret_cast<const half8*>(p.w + 5 * kTapHalves)[i];
    __syncthreads();
#pragma unroll
    for (int s = 0; s < 36; ++s) {
        const int tap = s >> 2;
        const half_t* src = tap < 5 ? s_a + tap * kTapHalves : s_b + (tap - 5) * kTapHalves;
#pragma unroll
        for (int i = 0; i < 8; ++i) wf[s][i] = src[(16 * (s & 3) + 8 * h + i) * kCvC + 32 * j + c32];
    }
    __syncthreads();

    const int stride = gridDim.x;
    cv_request(p, cv_tile(p, tile), s_a, wv, lane);
    if (tile + stride < p.ntiles) cv_request(p, cv_tile(p, tile + stride), s_b, wv, lane);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    while (true) {
        cv_step(p, lane, wf, s_a, s_c, s_stage[wv], tile, stride, wv, ro, j, c32, h);
        if ((tile += stride) >= p.ntiles) break;
        cv_step(p, lane, wf, s_b, s_a, s_stage[wv], tile, stride, wv, ro, j, c32, h);
        if ((tile += stride) >= p.ntiles) break;
        cv_step(p, lane, wf, s_c, s_b, s_stage[wv], tile, stride, wv, ro, j, c32, h);
        if ((tile += stride) >= p.ntiles) break;
    }
}

// ---------------------------------------------------------------------------
// Vector-ALU twin: one thread per output pixel and 32 output channels, fp32 FMAs; pixels from the
// same LDS tile, weights through uniform (scalar) loads.
__global__ void __launch_bounds__(512) conv3x3_valu_kernel(ConvArgs p) {
    __shared__ __attribute__((aligned(16))) half_t s_in[kCvLdsHalves];
    const int tid = threadIdx.x;
    const int tile = blockIdx.x;
    const int n = tile / (p.tiles_x * p.tiles_y);
    const int rem = tile - n * (p.tiles_x * p.tiles_y);
    const int ty = rem / p.tiles_x, tx = rem - ty * p.tiles_x;
    const int y0 = ty * kCvTY, x0 = tx * kCvTX;
    const half_t* img = p.in + (int64_t)n * p.H * p.W * kCvC;
    for (int idx = tid; idx < kCvRows * kCvPx * 8; idx += 512) {
        const int piece = idx & 7;
        const int pr = idx >> 3;
        const int r = pr / kCvPx, px = pr - r * kCvPx;
        const int y = y0 - 1 + r, x = x0 - 1 + px;
        half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
        if (y >= 0 && y < p.H && x >= 0 && x < p.W)
            v = *reinterpret_cast<const half8*>(img + ((int64_t)y * p.W + x) * kCvC + 8 * piece);
        *reinterpret_cast<half8*>(&s_in[cv_lds_index(r, piece >> 1, piece & 1, px)]) = v;
    }
    __syncthreads();
    const int cohalf = __builtin_amdgcn_readfirstlane(tid >> 8);   // waves 0-3: channels 0..31, waves 4-7: 32..63
    const int pid = tid & 255;
    const int ro = pid >> 5, xi = pid & 31;
    float acc[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = 0.f;
    for (int tap = 0; tap < 9; ++tap) {
        const int ky = tap / 3, kx = tap - 3 * ky;
        for (int kc = 0; kc < 4; ++kc) {
            const half8 a = *reinterpret_cast<const half8*>(&s_in[cv_lds_index(ro + ky, kc, 0, xi + kx)]);
            const half8 b = *reinterpret_cast<const half8*>(&s_in[cv_lds_index(ro + ky, kc, 1, xi + kx)]);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float xv = (float)(i < 8 ? a[i] : b[i - 8]);
                const half_t* wrow = p.w + ((tap * kCvC) + 16 * kc + i) * kCvC + 32 * cohalf;   // uniform
#pragma unroll
                for (int co = 0; co < 32; ++co) acc[co] = fmaf(xv, (float)wrow[co], acc[co]);
            }
        }
    }
    const int y = y0 + ro, x = x0 + xi;
    if (y < p.H && x < p.W) {
        half_t* o = p.out + (((int64_t)n * p.H + y) * p.W + x) * kCvC + 32 * cohalf;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            half8 v8;
#pragma unroll
            for (int r = 0; r < 8; ++r) v8[r] = (half_t)acc[8 * q + r];
            *reinterpret_cast<half8*>(o + 8 * q) = v8;
        }
    }
}

static hb_status conv_prepare(ConvArgs& a, const hb_half* in, const hb_half* w, hb_half* out,
                              int N, int H, int W, int Cin, int Cout) {
    if (!in || !w || !out) return HB_ERR_INVALID_ARG;
    if (N < 1 || H < 1 || W < 1 || Cin < 1 || Cout < 1) return HB_ERR_INVALID_ARG;
    if (!aligned_to(in, 16) || !aligned_to(w, 16) || !aligned_to(out, 16)) return HB_ERR_INVALID_ARG;
    if (Cin != kCvC || Cout != kCvC) return HB_ERR_UNSUPPORTED;
    const int64_t tiles = (int64_t)N * ceil_div(H, kCvTY) * ceil_div(W, kCvTX);
    if (tiles > 0x7fffffff || (int64_t)N * H * W > ((int64_t)1 << 40)) return HB_ERR_UNSUPPORTED;
    if ((int64_t)W * kCvRows * kCvC * 2 >= ((int64_t)1 << 30)) return HB_ERR_UNSUPPORTED;   // 32-bit tile offsets
    a.in = reinterpret_cast<const half_t*>(in);
    a.w = reinterpret_cast<const half_t*>(w);
    a.out = reinterpret_cast<half_t*>(out);
    a.N = N;
    a.H = H;
    a.W = W;
    a.tiles_x = ceil_div(W, kCvTX);
    a.tiles_y = ceil_div(H, kCvTY);
    a.ntiles = (int)tiles;
    return HB_OK;
}

}  // namespace hb

extern "C" hb_status hb_conv3x3(const hb_half* in_nhwc, const hb_half* w_hwio, hb_half* out_nhwc,
                                int N, int H, int W, int Cin, int Cout, hb_stream stream) {
    using namespace hb;
    ConvArgs a;
    hb_status s = conv_prepare(a, in_nhwc, w_hwio, out_nhwc, N, H, W, Cin, Cout);
    if (s != HB_OK) return s;
    const int blocks = min(a.ntiles, kNumCU);
    hipLaunchKernelGGL(conv3x3_mfma_kernel, dim3(blocks), dim3(kCvThreads), 0,
                       reinterpret_cast<hipStream_t>(stream), a);
    return launch_status();
}

extern "C" hb_status hb_conv3x3_valu(const hb_half* in_nhwc, const hb_half* w_hwio, hb_half* out_nhwc,
                                     int N, int H, int W, int Cin, int Cout, hb_stream stream) {
    using namespace hb;
    ConvArgs a;
    hb_status s = conv_prepare(a, in_nhwc, w_hwio, out_nhwc, N, H, W, Cin, Cout);
    if (s != HB_OK) return s;
    hipLaunchKernelGGL(conv3x3_valu_kernel, dim3(a.ntiles), dim3(512), 0, reinterpret_cast<hipStream_t>(stream), a);
    return launch_status();
}
