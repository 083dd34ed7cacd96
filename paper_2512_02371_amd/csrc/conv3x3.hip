// hb_conv3x3: 64 -> 64 channel 3x3 convolution (stride 1, zero padding 1, NHWC) as an implicit
// GEMM on the matrix units (Sec. V-A 2-D form summed over channels; the conv layer of Sec. IV
// without bias and activation), and its vector-ALU twin.
//
// MFMA formulation, transposed so that a lane ends with consecutive output channels of one pixel:
//   O'[m][n] = sum_k Wt[m][k] * X[k][n]     m = output channel, n = pixel, k = (tap, input channel)
// with v_mfma_f32_32x32x16_f16: 32 channels x 32 pixels per product, K = 16 input channels.
//   A (coefficients): the 9 x 64 x 32 weights of one 32-channel tile live in the registers of a
//     wave for the whole kernel (36 K-steps x 8 halves per lane = 144 registers), gathered once.
//   B (pixels): a workgroup walks DOWN a column of 8 x 32 pixel tiles.  The image rows it needs
//     (34 pixels x 64 channels each, with the one-pixel halo) stream through a ring of 26 rows in
//     LDS: a tile reads 10 of them, the 8 new rows of the next tile have landed, those of the tile
//     after that are in flight, and the two halo rows between vertically adjacent tiles are
//     fetched once.  Rows arrive by buffer loads that write LDS directly, in the image's own order
//     (pixel-major, 128 bytes per pixel) with the eight 16-byte channel pieces of a pixel permuted
//     by an XOR with bits 1..3 of the pixel index: a row is a few contiguous 1 KB copies, and the
//     16-byte reads of 16 consecutive pixels at one channel piece still fall into 64 different
//     banks for every tap shift (the overlapped view of Eq. 1: the three horizontal taps read the
//     same LDS row at pixel offsets 0, 1, 2).  Pixels outside the image arrive as zeros (requested
//     beyond the end of the buffer descriptor), which is the zero padding.
//   A workgroup has 8 waves, two per SIMD, so that one wave's LDS reads hide behind the other's
//   products: wave (q, j) owns output rows 2q, 2q+1 of the tile and channel tile j, i.e. 2 x 36
//   products per tile.  fp32 accumulators are rounded to fp16 (RNE) into a stage shared by the
//   workgroup and leave as whole 128-byte pixels (1 KB per store instruction).
#include "hb_device.hpp"
#include "hb_host.hpp"

namespace hb {

constexpr int kCvC = 64;                 // channels in and out
constexpr int kCvTY = 8, kCvTX = 32;     // output tile (rows x pixels) per workgroup step
constexpr int kCvRows = kCvTY + 2, kCvPx = kCvTX + 2;
constexpr int kCvLdsHalves = kCvRows * 4 * kCvPx * 16;    // tile of the vector-ALU twin

struct ConvArgs {
    const half_t* in;
    const half_t* w;
    half_t* out;
    int N, H, W;
    int tiles_x, tiles_y;      // per image
    int ntiles;                // N * tiles_y * tiles_x
    int seg_len, nseg;         // MFMA kernel: tiles per column segment, segments per column
};

// LDS layout of the vector-ALU twin: [row][16-channel chunk][8-channel half][pixel][8 channels].
__device__ __forceinline__ int cv_lds_index(int r, int kc, int half, int px) {
    return (((r * 4 + kc) * 2 + half) * kCvPx + px) * 8;
}

// LDS ring of the MFMA kernel: kCvRing rows of 34 pixels x 128 bytes; channel piece cp (16 bytes) of
// pixel px sits in slot cp ^ ((px >> 1) & 7) of the pixel's eight.
constexpr int kCvThreads = 512;
constexpr int kCvRing = 26;                               // 10 in use + 8 landed + 8 in flight
constexpr int kCvRowBytes = kCvPx * 128;                  // 4352
constexpr int kCvRowSlots = kCvPx * 8;                    // 272 16-byte slots
constexpr int kCvRowLoads = (kCvRowSlots + 63) / 64;      // 5 loads per row, the last one 16 lanes wide
constexpr int kCvRingBytes = kCvRing * kCvRowBytes;       // 113152
constexpr uint32_t kCvOutside = 0x80000000u;              // offset beyond any descriptor used here
// Output stage: 8 rows x 32 pixels x 64 channels of fp16, 144-byte pixel pitch (conflict-free reads).
constexpr int kCvStagePitch = 144;
constexpr int kCvStageBytes = kCvTY * kCvTX * kCvStagePitch;   // 36864

// A value the compiler must take as new: what is computed from it is computed again where it is
// used, instead of being kept in registers (or spilled) across the whole tile loop.
__device__ __forceinline__ int cv_fresh(int v) {
    asm volatile("" : "+v"(v));
    return v;
}

// One LDS-direct load: the active lanes copy 16 bytes each from base + voff (per lane) to LDS at
// lds_addr + 16 * lane (lds_addr wave-uniform).  Written as assembly so that the compiler keeps no
// book on it: it would make LDS reads of other ring rows wait for these loads, which are meant to
// stay in flight for two tiles.  The waits that order them are explicit in the tile loop.
typedef uint32_t u32x4s __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void cv_dma16(u32x4s rsrc, uint32_t lds_addr, uint32_t voff) {
    uint32_t m0_before;                                   // M0 cannot be named as clobbered: it is put back
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tbuffer_load_dwordx4 %2, %3, 0 offen lds\n\t"
                 "s_mov_b32 m0, %0"
                 : "=&s"(m0_before) : "s"(lds_addr), "v"(voff), "s"(rsrc) : "memory");
}
__device__ __forceinline__ uint32_t cv_lds_addr(const void* p) {
    return (uint32_t)(size_t)(__attribute__((address_space(3))) const void*)p;
}

// Per-lane byte offsets of the kCvRowLoads loads of a row, from the row's pixel x0-1: slot 64 c + lane
// holds channel piece (lane & 7) ^ ((px >> 1) & 7) of pixel px = 8 c + lane / 8.  Pixels left or right
// of the image get an offset beyond the descriptor (they arrive as zeros).
struct CvRowOff {
    uint32_t off[kCvRowLoads];
};
__device__ __forceinline__ CvRowOff cv_row_offsets(const ConvArgs& p, int x0, int lane) {
    CvRowOff d;
#pragma unroll
    for (int c = 0; c < kCvRowLoads; ++c) {
        const int px = 8 * c + (lane >> 3);
        const int cp = (lane & 7) ^ ((px >> 1) & 7);
        const int x = x0 - 1 + px;
        d.off[c] = (x >= 0 && x < p.W) ? (uint32_t)(px * 128 + 16 * cp) : kCvOutside;
    }
    return d;
}

// Requests image row y, pixels x0-1 .. x0+32, of image n into ring row `rrow`: kCvRowLoads loads by
// the calling wave.  A row outside the image gets a descriptor of length zero: it arrives as zeros.
__device__ __forceinline__ void cv_request_row(const ConvArgs& p, const CvRowOff& d, int n, int y, int x0,
                                               char* ring, int rrow, int lane) {
    const bool yok = y >= 0 && y < p.H;                   // uniform
    // the descriptor starts at the (possibly virtual) pixel (y, x0-1); lanes outside the image never
    // reach memory
    const uint64_t org = (uint64_t)(p.in + (((int64_t)n * p.H + (yok ? y : 0)) * p.W + (x0 - 1)) * kCvC);
    const u32x4s rs = {(uint32_t)org, (uint32_t)(org >> 32) & 0xffffu, yok ? 0x7fffffffu : 0u, 0x00020000u};
    const uint32_t lds0 = cv_lds_addr(ring) + (uint32_t)(rrow * kCvRowBytes);
#pragma unroll
    for (int c = 0; c < kCvRowLoads - 1; ++c) cv_dma16(rs, lds0 + 1024u * c, d.off[c]);
    if (lane < kCvRowSlots - 64 * (kCvRowLoads - 1))      // the row ends after 272 slots
        cv_dma16(rs, lds0 + 1024u * (kCvRowLoads - 1), d.off[kCvRowLoads - 1]);
}

// Two output rows (2 x 32 pixels) x 32 channels from four ring rows (byte offsets row[0..3] from the
// ring base, wave-uniform).  The four rows under the two output rows are read once per (channel
// chunk, horizontal tap) and serve both output rows: 48 reads for 72 products, in 12 groups of
// 4 reads + 6 products.  The reads of a group are issued kCvAhead groups before its products (the
// scheduling barriers pin that order), so that an LDS read has the time of 6 * kCvAhead products.
#ifndef HB_CONV_AHEAD
#define HB_CONV_AHEAD 1
#endif
constexpr int kCvAhead = HB_CONV_AHEAD;
// Lane part of the LDS byte address of group grp = 3 kc + kx: pixel c32 + kx, channel piece 2 kc + h,
// which sits in slot (2 kc) ^ (h ^ s) of the pixel (s = the pixel's permutation).  The twelve values
// are formed once per kernel: every instruction between two products costs the matrix pipe issue time.
__device__ __forceinline__ int cv_lane_part(int grp, int c32, int h) {
    const int kc = grp / 3, kx = grp - 3 * kc;
    const int px = c32 + kx;
    return px * 128 + ((32 * kc) ^ (16 * (h ^ ((px >> 1) & 7))));
}
__device__ __forceinline__ void cv_rows(const char* ring, const int (&row)[4], const half8 (&wf)[36], const int (&L)[12],
                                        floatx16 (&acc)[2]) {
    half8 b[kCvAhead + 1][4];
    auto read_group = [&](int grp, half8 (&dst)[4]) {
        const int a = L[grp];
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) dst[rr] = *reinterpret_cast<const half8*>(ring + (a + row[rr]));
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

__global__ void __launch_bounds__(kCvThreads) conv3x3_mfma_kernel(ConvArgs p) {
    __shared__ __attribute__((aligned(16))) char s_ring[kCvRingBytes];
    __shared__ __attribute__((aligned(16))) char s_stage[kCvStageBytes];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c32 = lane & 31, h = lane >> 5;
    const int j = wv >> 2;                                // channel tile of this wave
    const int ro = 2 * (wv & 3);                          // its two output rows inside the tile

    // task = column segment: image n, tile column cx, tile rows ty0 .. ty0 + len - 1
    const int task = blockIdx.x;
    const int per_img = p.tiles_x * p.nseg;
    const int n = task / per_img;
    const int sg = (task - n * per_img) / p.tiles_x, cx = task - n * per_img - sg * p.tiles_x;
    const int ty0 = sg * p.seg_len;
    const int len = min(p.seg_len, p.tiles_y - ty0);
    const int x0 = cx * kCvTX;
    const int ys = ty0 * kCvTY - 1;                       // image row held by ring row 0 at the start

    const CvRowOff d = cv_row_offsets(p, x0, lane);

    // start-up, part 1: rows 0..9 of the first tile go out before anything else (waves 0, 1 take two
    // rows each) and land in ring rows 0..9 while the weights are staged
    if (wv < 2) cv_request_row(p, d, n, ys + wv, x0, s_ring, wv, lane);
    cv_request_row(p, d, n, ys + 2 + wv, x0, s_ring, 2 + wv, lane);

    // coefficient fragments: wf[s] lane (c32, h) = w[tap][16 kc + 8h + i][32 j + c32], s = 4 tap + kc.
    // The weights arrive with the output channel innermost; a fragment wants eight consecutive INPUT
    // channels per lane.  They pass through LDS once, transposed on the way in: coalesced 16-byte
    // reads of eight output channels, 4-byte writes to [tap][co][ci] with a 144-byte pitch per
    // (tap, co), so that each fragment is one conflict-free 16-byte read.  Taps 0..6 use ring rows
    // 10..25 (free until the second tile's rows are requested), taps 7, 8 the output stage.
    half8 wf[36];
    {
        constexpr int kWPitch = 144;                      // bytes per (tap, output channel): 64 ci + pad
        constexpr int kWTap = kCvC * kWPitch;             // 9216 bytes per tap
        constexpr int kTapsInRing = 7;
        static_assert(kTapsInRing * kWTap <= (kCvRing - 10) * kCvRowBytes, "taps 0..6 must fit ring rows 10..25");
        static_assert((9 - kTapsInRing) * kWTap <= kCvStageBytes, "taps 7, 8 must fit the output stage");
        char* const wring = s_ring + 10 * kCvRowBytes;
        // a thread takes the same eight output channels of TWO neighbouring input channels and writes
        // eight 4-byte pairs; with the input-channel pair as the fastest lane index the 64 writes of an
        // instruction fall into 64 different banks (2-byte writes, one input channel at a time, took
        // twice the instructions and met two lanes in every bank word)
        for (int i = tid; i < 9 * (kCvC / 2) * (kCvC / 8); i += kCvThreads) {
            const int cip = i & 31, cog = (i >> 5) & 7, tap = i >> 8;
            const half8 v0 = reinterpret_cast<const half8*>(p.w)[(tap * kCvC + 2 * cip) * 8 + cog];      // w[tap][2 cip][8 cog ..]
            const half8 v1 = reinterpret_cast<const half8*>(p.w)[(tap * kCvC + 2 * cip + 1) * 8 + cog];
            char* dst = (tap < kTapsInRing ? wring + tap * kWTap : s_stage + (tap - kTapsInRing) * kWTap) +
                        8 * cog * kWPitch + 4 * cip;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                typedef half_t half2v __attribute__((ext_vector_type(2)));
                *reinterpret_cast<half2v*>(dst + e * kWPitch) = half2v{v0[e], v1[e]};
            }
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < 36; ++s) {
            const int tap = s >> 2;
            const char* src = tap < kTapsInRing ? wring + tap * kWTap : s_stage + (tap - kTapsInRing) * kWTap;
            wf[s] = *reinterpret_cast<const half8*>(src + (32 * j + c32) * kWPitch + 2 * (16 * (s & 3) + 8 * h));
        }
        __syncthreads();
    }

    // output: a descriptor over image n; thread t stores pieces t, t + 512, ... of the 8 x 32 x 8 pieces
    // of a tile (8 lanes per pixel): row (t >> 8) + 2 i, pixel (t >> 3) & 31, piece t & 7
    const int64_t obytes = (int64_t)p.H * p.W * kCvC * 2;     // < 2 GiB (host check)
    const __amdgpu_buffer_rsrc_t orsrc = __builtin_amdgcn_make_buffer_rsrc(
        p.out + (int64_t)n * p.H * p.W * kCvC, 0, (int)obytes, 0x00020000);
    const int opx = (tid >> 3) & 31, opiece = tid & 7, orow0 = tid >> 8;
    const uint32_t ovoff = (x0 + opx < p.W) ? (uint32_t)(((orow0 * p.W + x0 + opx) * kCvC + 8 * opiece) * 2) : kCvOutside;
    const char* sread = s_stage + (orow0 * kCvTX + opx) * kCvStagePitch + 16 * opiece;
    char* swrite = s_stage + (ro * kCvTX + c32) * kCvStagePitch + (32 * j + 4 * h) * 2;

    // start-up, part 2: the 8 new rows of the second tile, now that ring rows 10..17 are free
    // (only the first tile's rows have to be there now: everything but this wave's newest request)
    if (len > 1) {
        cv_request_row(p, d, n, ys + 10 + wv, x0, s_ring, 10 + wv, lane);
        asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
    } else {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __syncthreads();

    int L[12];
#pragma unroll
    for (int grp = 0; grp < 12; ++grp) L[grp] = cv_lane_part(grp, c32, h);
    int rb = 0;                                           // ring row of the tile's first row: 8 k mod 26
    for (int k = 0; k < len; ++k) {
        // the rows of tile k + 2 take the ring rows that tile k - 1 has released
        const bool req = k + 2 < len;                     // uniform
        if (req) {
            int rr2 = rb + 18 + wv;
            if (rr2 >= kCvRing) rr2 -= kCvRing;
            cv_request_row(p, d, n, ys + 8 * k + 18 + wv, x0, s_ring, rr2, lane);
        }
        __builtin_amdgcn_sched_barrier(0);                // the requests go out before the first product
        int row[4];
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            int r = rb + ro + rr;
            if (r >= kCvRing) r -= kCvRing;
            row[rr] = r * kCvRowBytes;
        }
        floatx16 acc[2];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[u][v] = 0.f;
        cv_rows(s_ring, row, wf, L, acc);
        __builtin_amdgcn_sched_barrier(0);
        // accumulators -> stage: lane (c32, h) holds channels 32 j + 8 q + 4 h + (0..3) of pixel c32
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                half4 v4;
#pragma unroll
                for (int r = 0; r < 4; ++r) v4[r] = (half_t)acc[u][4 * q + r];
                *reinterpret_cast<half4*>(swrite + u * (kCvTX * kCvStagePitch) + 16 * q) = v4;
            }
        // Meeting point.  A wave waits for all its memory instructions but the newest request (loads
        // and stores retire in order): its row of the NEXT tile has landed, the previous tile's
        // stores are done.  The barrier instructions are written out: the compiler would put a wait
        // for ALL memory instructions in front of one it emits itself.
        static_assert(kCvRowLoads == 5, "the counted wait below is written for five loads per request");
        if (req) asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // next rows complete, this tile's rows released, stage written
        // stage -> memory: 8 lanes per pixel, 1 KB per store instruction; rows below the image fall
        // behind the end of the descriptor and are dropped
        const uint32_t osoff = (uint32_t)((ty0 + k) * kCvTY) * (uint32_t)(p.W * kCvC * 2);
#pragma unroll
        for (int i = 0; i < kCvTY * kCvTX * 8 / kCvThreads; ++i) {
            const half8 v = *reinterpret_cast<const half8*>(sread + 2 * i * (kCvTX * kCvStagePitch));
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4s, v), orsrc, ovoff,
                                                   osoff + (uint32_t)(2 * i) * (uint32_t)(p.W * kCvC * 2), 0);
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // stage read, free for the next tile
        rb += 8;
        if (rb >= kCvRing) rb -= kCvRing;
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
    if ((int64_t)H * W * kCvC * 2 >= ((int64_t)1 << 31)) return HB_ERR_UNSUPPORTED;   // 32-bit offsets inside an image
    a.in = reinterpret_cast<const half_t*>(in);
    a.w = reinterpret_cast<const half_t*>(w);
    a.out = reinterpret_cast<half_t*>(out);
    a.N = N;
    a.H = H;
    a.W = W;
    a.tiles_x = ceil_div(W, kCvTX);
    a.tiles_y = ceil_div(H, kCvTY);
    a.ntiles = (int)tiles;
    // column segments of the MFMA kernel: about one per compute unit, at least 4 tiles long
    const int want = ceil_div(num_cu(), N * a.tiles_x);
    int len = ceil_div(a.tiles_y, want);
    if (len < 4) len = a.tiles_y < 4 ? a.tiles_y : 4;
    a.seg_len = len;
    a.nseg = ceil_div(a.tiles_y, len);
    return HB_OK;
}

}  // namespace hb

extern "C" hb_status hb_conv3x3(const hb_half* in_nhwc, const hb_half* w_hwio, hb_half* out_nhwc,
                                int N, int H, int W, int Cin, int Cout, hb_stream stream) {
    using namespace hb;
    ConvArgs a;
    hb_status s = conv_prepare(a, in_nhwc, w_hwio, out_nhwc, N, H, W, Cin, Cout);
    if (s != HB_OK) return s;
    const int64_t blocks = (int64_t)N * a.tiles_x * a.nseg;
    if (blocks > 0x7fffffff) return HB_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(conv3x3_mfma_kernel, dim3((unsigned)blocks), dim3(kCvThreads), 0,
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
