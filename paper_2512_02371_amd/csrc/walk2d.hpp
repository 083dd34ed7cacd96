// The row-walking machinery shared by the 2-D kernels with arbitrary taps (hb_conv2d, hb_down2,
// hb_up2): a wave keeps the windows of 16 input rows in registers, multiplies them with the Toeplitz
// fragments of all kernel rows (fragments come from an LDS table laid out [row][chunk][lane]), and
// adds every product tile, moved by its kernel row's shift b, into two open groups of 16 output
// rows with lane-shifted additions (DPP row shifts inside each row of 16 lanes).
#pragma once
#include "hb_device.hpp"

namespace hb {

constexpr int kC2Tiles = 4;                   // 16-column tiles per wave strip
constexpr int kC2Threads = 512;               // 8 waves share one fragment table

// acc[c] += d[c + SH] for the lanes c of each row of 16 with 0 <= c + SH < 16 (SH in -15..15).
template <int SH>
__device__ __forceinline__ float c2_shift_add(float acc, float d) {
    if constexpr (SH == 0) {
        return acc + d;
    } else {
        constexpr int ctrl = SH > 0 ? 0x100 + SH : 0x110 - SH;        // row_shl:SH / row_shr:-SH
        const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, d), ctrl, 0xf, 0xf, true);
        return acc + __builtin_bit_cast(float, moved);
    }
}

// Adds a product tile moved by B rows into tile W of the two open output groups
// ring[1] = group G (rows n >= B) and ring[0] = group G - 1 (rows n < B).
template <int B, int W>
__device__ __forceinline__ void c2_add_tile(const floatx4& d, floatx4 (&ring)[2][kC2Tiles]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        ring[1][W][j] = c2_shift_add<B>(ring[1][W][j], d[j]);
        if constexpr (B != 0) ring[0][W][j] = c2_shift_add<B - 16>(ring[0][W][j], d[j]);
    }
}

// The fragments of kernel rows B (and, with UP, B + 16): [0][kk] lower row, [1][kk] upper row.
template <int NK, bool UP>
__device__ __forceinline__ void c2_read_frags(const half8* s_frag, int lane, int b, half8 (&f)[2][NK]) {
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) {
        f[0][kk] = s_frag[(b * NK + kk) * 64 + lane];
        if (UP) f[1][kk] = s_frag[((b + 16) * NK + kk) * 64 + lane];
    }
}

// The product tiles of two neighbouring strip tiles W, W + 1 for the shift of `f`: lower kernel row
// times input group G, plus (UP) upper kernel row times input group G + 1.  The two tiles' products
// alternate, so no product waits for the one it accumulates onto.
template <int NK, bool UP, int W>
__device__ __forceinline__ void c2_products(const half8 (&f)[2][NK], const half8 (&x0)[kC2Tiles][NK],
                                            const half8 (&x1)[kC2Tiles][NK], floatx4& da, floatx4& db) {
    da = floatx4{0.f, 0.f, 0.f, 0.f};
    db = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) {
        da = mfma16x16x32(f[0][kk], x0[W][kk], da);
        db = mfma16x16x32(f[0][kk], x0[W + 1][kk], db);
    }
    if (UP) {
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) {
            da = mfma16x16x32(f[1][kk], x1[W][kk], da);
            db = mfma16x16x32(f[1][kk], x1[W + 1][kk], db);
        }
    }
}

// A block of four shifts B4 .. B4+3 is 8 pairs of tiles: pair P = (shift B4 + P / 2, tiles 2 (P % 2)
// and 2 (P % 2) + 1).  The products of pair P + 1 are interleaved with the additions of pair P, so
// the vector ALU adds two tiles while the matrix unit multiplies the next two.
template <int NK, bool UP, int B4, int P>
__device__ __forceinline__ void c2_pairs(const half8* s_frag, int lane, const half8 (&x0)[kC2Tiles][NK],
                                         const half8 (&x1)[kC2Tiles][NK], floatx4 (&ring)[2][kC2Tiles],
                                         const half8 (&frag)[2][NK], const half8 (&ahead_in)[2][NK],
                                         const floatx4& da, const floatx4& db) {
    constexpr int b = B4 + P / 2, w = 2 * (P % 2);
    half8 ahead[2][NK];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) ahead[u][kk] = ahead_in[u][kk];
    // first pair of a shift: request the next shift's fragments
    if constexpr (w == 0 && b + 1 < B4 + 4) c2_read_frags<NK, UP>(s_frag, lane, b + 1, ahead);
    if constexpr (P + 1 < 8) {
        constexpr int w1 = 2 * ((P + 1) % 2);
        half8 fnext[2][NK];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) fnext[u][kk] = w1 == 0 ? ahead[u][kk] : frag[u][kk];
        floatx4 na, nb;
        c2_products<NK, UP, w1>(fnext, x0, x1, na, nb);
        c2_add_tile<b, w>(da, ring);
        c2_add_tile<b, w + 1>(db, ring);
        // One product, then its share of the additions, so that both units stay busy.  (Products
        // issued back to back block the wave's instruction stream until the matrix unit is free.)
        constexpr int nprod = 2 * NK * (UP ? 2 : 1), nadd = b ? 16 : 8;
#pragma unroll
        for (int i = 0; i < nprod; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, nadd / nprod, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        c2_pairs<NK, UP, B4, P + 1>(s_frag, lane, x0, x1, ring, fnext, ahead, na, nb);
    } else {
        c2_add_tile<b, w>(da, ring);
        c2_add_tile<b, w + 1>(db, ring);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Four shifts B4 .. B4+3 of one step.
template <int NK, bool UP, int B4>
__device__ __forceinline__ void c2_rows4(const half8* s_frag, int lane, const half8 (&x0)[kC2Tiles][NK],
                                         const half8 (&x1)[kC2Tiles][NK], floatx4 (&ring)[2][kC2Tiles]) {
    static_assert(kC2Tiles == 4, "pairs of tiles");
    half8 frag[2][NK];
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) frag[1][kk] = half8{};
    c2_read_frags<NK, UP>(s_frag, lane, B4, frag);
    floatx4 da, db;
    c2_products<NK, UP, 0>(frag, x0, x1, da, db);
    c2_pairs<NK, UP, B4, 0>(s_frag, lane, x0, x1, ring, frag, frag, da, db);
}

// One step of the walk: two sources of 16 input rows each (windows x0 and x1) against the fragment
// table rows b (applied to x0) and b + 16 (applied to x1) for every shift b < 16, in blocks of four
// shifts.  Blocks at or beyond nrows are skipped and the x1 half of a block is left out when the
// block lies at or beyond nup (uniform branches); single table rows beyond the counts inside a block
// hold zero fragments.  HASUP = false compiles no x1 half at all.
template <int NK, bool HASUP, int B4 = 0>
__device__ __forceinline__ void c2_step(const half8* s_frag, int lane, int nrows, int nup,
                                        const half8 (&x0)[kC2Tiles][NK], const half8 (&x1)[kC2Tiles][NK],
                                        floatx4 (&ring)[2][kC2Tiles]) {
    if constexpr (B4 < 16) {
        if (B4 < nrows) {
            if (HASUP && B4 < nup) c2_rows4<NK, true, B4>(s_frag, lane, x0, x1, ring);
            else c2_rows4<NK, false, B4>(s_frag, lane, x0, x1, ring);
        }
        c2_step<NK, HASUP, B4 + 4>(s_frag, lane, nrows, nup, x0, x1, ring);
    } else {
        // Pin the sums here: otherwise the additions are sunk below the caller's store and every
        // shifted product stays live (and is spilled) until then.
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int w = 0; w < kC2Tiles; ++w)
#pragma unroll
                for (int j = 0; j < 4; ++j) asm volatile("" : "+v"(ring[r][w][j]));
    }
}

}  // namespace hb
