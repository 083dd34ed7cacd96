// Device-side building blocks shared by the gfx950 kernels: vector types, MFMA
// wrappers with their operand-to-lane maps, edge-aware row loads and stores.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hb_host.hpp"

namespace hb {

typedef _Float16 half_t;
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// ---------------------------------------------------------------------------
// Operand-to-lane maps on a 64-lane wave (lane = 16*g + c for the 16-wide shapes).
//
// v_mfma_f32_16x16x32_f16   D[16x16] += A[16x32] * B[32x16]
//   A: lane (c, g) holds A[c][8g .. 8g+7]        (8 halves)
//   B: lane (c, g) holds B[8g .. 8g+7][c]        (8 halves)
//   D: lane (c, g) holds D[4g .. 4g+3][c]        (4 floats)
// v_mfma_f32_16x16x16_f16   D[16x16] += A[16x16] * B[16x16]
//   A: lane (c, g) holds A[c][4g .. 4g+3];  B: lane (c, g) holds B[4g .. 4g+3][c];  D as above
// v_mfma_f32_16x16x4_f32    D[16x16] += A[16x4] * B[4x16]
//   A: lane (c, g) holds A[c][g];  B: lane (c, g) holds B[g][c];  D as above
// v_mfma_f32_32x32x16_f16   D[32x32] += A[32x16] * B[16x32]      (lane = 32*h + c)
//   A: lane (c, h) holds A[c][8h .. 8h+7];  B: lane (c, h) holds B[8h .. 8h+7][c]
//   D: lane (c, h) holds D[8q + 4h + r][c] in register 4q + r  (q, r = 0..3)
//
// Because a D fragment holds, per lane, a run of the ROW index for a fixed column,
// a D fragment rounded to fp16 is already a valid A or B fragment of a following
// product that contracts over that row index: no transpose, no LDS round trip.
// Two stacked 16-row D fragments t = 0, 1 form one K = 32 operand whose k-slot
// 8g + i stands for row 16*(i/4) + 4g + (i%4); the coefficient operand is built
// with the same slot order (see krow32 below), which leaves the sum unchanged.
// ---------------------------------------------------------------------------

// These wrappers are the only matrix products the kernels can issue (a test scans the sources for
// builtins used anywhere else).  For 16 x 16 fp16 products there is ONE shape, K = 32: a
// 16x16x16 product issued straight after a 16x16x32 on the same accumulator once gave a wrong
// first tile, so an accumulator chain never mixes the two; operands with K = 16 are padded with
// zeros.  The K = 16 instruction exists only inside the self-check kernel of util.hip.
__device__ __forceinline__ floatx4 mfma16x16x32(half8 a, half8 b, floatx4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ floatx4 mfma16x16x4f32(float a, float b, floatx4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ floatx16 mfma32x32x16(half8 a, half8 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

// Row (within a 32-row window made of two stacked 16-row D fragments) that k-slot
// 8g + i of a chained K = 32 operand stands for.
__device__ __forceinline__ int krow32(int g, int i) { return 16 * (i >> 2) + 4 * g + (i & 3); }

// Two D fragments (rows 0..15 and 16..31 of a window), rounded to fp16 (RNE), as
// one K = 32 operand in the slot order of krow32.
__device__ __forceinline__ half8 chain2(floatx4 lo, floatx4 hi) {
    half8 r;
    r[0] = (half_t)lo[0]; r[1] = (half_t)lo[1]; r[2] = (half_t)lo[2]; r[3] = (half_t)lo[3];
    r[4] = (half_t)hi[0]; r[5] = (half_t)hi[1]; r[6] = (half_t)hi[2]; r[7] = (half_t)hi[3];
    return r;
}
__device__ __forceinline__ half4 to_half4(floatx4 v) {
    half4 r;
    r[0] = (half_t)v[0]; r[1] = (half_t)v[1]; r[2] = (half_t)v[2]; r[3] = (half_t)v[3];
    return r;
}
__device__ __forceinline__ half8 join(half4 lo, half4 hi) {
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// Vector types with element alignment only: gfx950 under HSA runs with unaligned
// access enabled, so a 16-byte access needs no more than the alignment of its elements.
typedef half8 half8_u __attribute__((aligned(2)));
typedef half4 half4_u __attribute__((aligned(2)));
typedef floatx4 floatx4_u __attribute__((aligned(4)));

// Eight consecutive pixels row[xs .. xs+7] with the column index clamped to [0, W-1].
// One 16-byte load (any 2-byte aligned address) when the run lies inside the row.
__device__ __forceinline__ half8 load8_clamp(const half_t* __restrict__ row, int xs, int W) {
    if (xs >= 0 && xs + 8 <= W) {
        return *reinterpret_cast<const half8_u*>(row + xs);
    }
    half8 r;
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = row[clampi(xs + i, 0, W - 1)];
    return r;
}

// Four consecutive pixels row[xs .. xs+3], clamped like load8_clamp.
__device__ __forceinline__ half4 load4_clamp(const half_t* __restrict__ row, int xs, int W) {
    if (xs >= 0 && xs + 4 <= W) {
        return *reinterpret_cast<const half4_u*>(row + xs);
    }
    half4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = row[clampi(xs + i, 0, W - 1)];
    return r;
}

// Store four consecutive floats at row[x .. x+3], dropping columns >= W.
__device__ __forceinline__ void store4_mask(float* __restrict__ row, int x, int W, floatx4 v) {
    if (x + 4 <= W) {
        *reinterpret_cast<floatx4_u*>(row + x) = v;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (x + i < W) row[x + i] = v[i];
    }
}

// Accesses through a wave-uniform base plus a 32-bit per-lane BYTE offset: the form the
// hardware addresses with a scalar base register and one vector offset register.
__device__ __forceinline__ half8 ldg8(const half_t* base, uint32_t byte_off) {
    return *reinterpret_cast<const half8_u*>(reinterpret_cast<const char*>(base) + byte_off);
}
__device__ __forceinline__ half4 ldg4(const half_t* base, uint32_t byte_off) {
    return *reinterpret_cast<const half4_u*>(reinterpret_cast<const char*>(base) + byte_off);
}
// Output stores.  STREAM = true marks the lines non-temporal (written once, not read back by the
// kernel).  With the coalesced row stores below, streaming stores measured faster at every output
// size tried (64 MB to 256 MB per call); the limit stays as a switch for measurements.
template <bool STREAM>
__device__ __forceinline__ void stg4(float* base, uint32_t byte_off, floatx4 v) {
    floatx4_u* q = reinterpret_cast<floatx4_u*>(reinterpret_cast<char*>(base) + byte_off);
    if (STREAM) __builtin_nontemporal_store(v, q); else *q = v;
}
// Outputs up to this many megabytes per call are written with streaming stores.
#ifndef HB_STREAM_STORE_MAX_MB
#define HB_STREAM_STORE_MAX_MB (1 << 20)
#endif
constexpr int64_t kStreamStoreMaxBytes = (int64_t)HB_STREAM_STORE_MAX_MB << 20;

// Accumulator tiles leave the MFMA with a lane owning four columns of ONE row and the 16 lanes
// of a quarter-wave owning 16 DIFFERENT rows, so a store instruction would touch each row with
// 16-byte pieces only.  Passing the NW tiles (16 rows x 16*NW floats) through a wave-private LDS
// patch turns that into stores of 16 consecutive lanes x 16 bytes = one 256-byte run of one row.
// The patch has a row pitch of 16*NW + 4 floats: both the accumulator-layout writes and the
// row-major reads are bank-conflict free.  Only the owning wave touches its patch and LDS serves
// one wave's instructions in order, so no workgroup barrier is needed.
template <int NW>
struct RowPatch {
    static constexpr int kPitch = 16 * NW + 4;
    static constexpr int kFloats = 16 * kPitch;
};
template <int NW, bool STREAM>
__device__ __forceinline__ void store_rows_via_lds(float* patch, float* dst, uint32_t pitch_elems,
                                                   const floatx4 (&acc)[NW], int lane) {
    const int c = lane & 15, g = lane >> 4;
#pragma unroll
    for (int w = 0; w < NW; ++w)
        *reinterpret_cast<floatx4*>(patch + c * RowPatch<NW>::kPitch + 16 * w + 4 * g) = acc[w];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    constexpr int kLanesPerRow = 4 * NW;                  // 16-byte pieces in a row of the patch
    constexpr int kRowsPerPass = 64 / kLanesPerRow;
    const int rr = lane / kLanesPerRow, xq = lane - rr * kLanesPerRow;
#pragma unroll
    for (int s = 0; s < 16 / kRowsPerPass; ++s) {
        const int row = s * kRowsPerPass + rr;
        const floatx4 v = *reinterpret_cast<const floatx4*>(patch + row * RowPatch<NW>::kPitch + 4 * xq);
        stg4<STREAM>(dst, ((uint32_t)row * pitch_elems + 4u * xq) * 4u, v);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Workgroups are handed to the 8 XCDs (each with its own L2) round-robin by workgroup id.
// This maps a workgroup id to a position such that every XCD works through one contiguous
// eighth of the positions, in order: neighbouring tasks, which share halo pixels, then meet
// in the same L2 at about the same time instead of each fetching the halo from memory.
#ifndef HB_XCD_CONTIGUOUS
#define HB_XCD_CONTIGUOUS 1
#endif
__device__ __forceinline__ int xcd_contiguous(int wg, int nwg) {
    if (!HB_XCD_CONTIGUOUS) return wg;
    const int per = nwg >> 3;                             // positions per XCD (remainder handled below)
    if (wg >= per * 8) return wg;                         // tail workgroups keep their place
    return (wg & 7) * per + (wg >> 3);
}

// The same idea at a finer grain: of every 8 G consecutive workgroup ids, XCD x (which receives
// ids x, x + 8, ...) takes G consecutive positions.  Neighbours still meet in one L2, while the chip
// as a whole sweeps through the tasks in launch order, as it does with the plain order.
__device__ __forceinline__ int xcd_blocked(int wg, int nwg, int G) {
    const int span = 8 * G, first = (wg / span) * span;
    if (first + span > nwg) return wg;                    // tail workgroups keep their place
    const int r = wg - first;
    return first + (r & 7) * G + (r >> 3);
}

// Toeplitz fragment = eight consecutive entries of the zero-padded tap table that travels in the
// kernel arguments (see TapsT): one 16-byte load at a 2-byte aligned address.
__device__ __forceinline__ half8 tap_run(const uint16_t* tab, int t0) {
    return *reinterpret_cast<const half8_u*>(tab + kTapPad + t0);
}
__device__ __forceinline__ half_t tap_at(const uint16_t* tab, int t) {
    return __builtin_bit_cast(half_t, tab[kTapPad + t]);
}

// ---------------------------------------------------------------------------
// Clamp-to-edge folded into the coefficient matrix.
//
// Clamping the input index is linear in the pixels: every tap that would read left of
// pixel 0 reads pixel 0 instead, so its weight moves onto the matrix row of pixel 0 (and
// likewise for the last pixel).  A border tile therefore keeps the in-bounds, aligned
// 16-byte window loads of an interior tile (the window is shifted to lie inside the row)
// and only swaps the Toeplitz fragment for a folded one built from absolute indices.
// Sums of fp16 taps are not fp16 numbers, so a folded fragment is carried as hi + lo
// (two products), which keeps the border as accurate as the interior.
//
// Tables (FoldTablesT, filled on the host): kf[t] = taps as fp32, pfx[i] = sum of taps t < i.
// Weight of pixel u in output x: sum of taps[t] over t with clamp(x + t - anchor, 0, n-1) == u.
template <class FT>
__device__ __forceinline__ float folded_tap(const FT& ft, int ntaps, int anchor, int n, int x, int u) {
    float v = 0.f;
    const int t = u - x + anchor;
    if (t >= 0 && t < ntaps) v = ft.kf[t];
    if (u == 0) v += ft.pfx[clampi(anchor - x, 0, ntaps)];                 // taps that read left of 0
    if (u == n - 1) {
        const int t0 = clampi(n - x + anchor, 0, ntaps);                   // first tap that reads past n-1
        v += ft.pfx[ntaps] - ft.pfx[t0];
    }
    return v;
}
// Folded fragment (natural slot order: slot 8g + i = window pixel 32*kk + 8g + i) for the 16
// outputs xbase + c and the window starting at absolute pixel ws.
template <class FT>
__device__ __forceinline__ void folded_fragment(const FT& ft, int ntaps, int anchor, int n,
                                                int xbase, int ws, int kk, int c, int g,
                                                half8& hi, half8& lo) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float v = folded_tap(ft, ntaps, anchor, n, xbase + c, ws + 32 * kk + 8 * g + i);
        hi[i] = (half_t)v;
        lo[i] = (half_t)(v - (float)hi[i]);
    }
}

}  // namespace hb
