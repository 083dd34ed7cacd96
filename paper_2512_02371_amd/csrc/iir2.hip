// hb_iir2: second-order recursive filter Y_t = X_t + alpha Y_{t-1} + beta Y_{t-2} over long signals,
// and its vector-ALU twin (Sec. V-D).
//
// The paper tiles the signal, runs the filter on every tile in parallel and fixes the tiles up with
// the contribution of their predecessors; inside a tile it trades the serial recursion for a
// convolution on the matrix units plus a dilated recursion.  Here the part inside a tile is taken
// one step further: the filter restricted to a block of 32 samples with zero initial state is the
// lower-triangular Toeplitz matrix of its impulse response, T(i, j) = h_{i-j}, so 16 blocks are one
// product T * X^T (K = 32) per half of the outputs, and the recursion survives only as the
// propagation of a two-number state (Y_{t-1}, Y_{t-2}) from block to block: the state after a block
// is M32 * (state before) + (last two local outputs), M32 the 32nd power of the companion matrix.
// Three launches, like the summed-area table: (1) local products, end state of every 512-sample
// tile; (2) scan of the tile states along the signal; (3) local products again, block states from
// the true tile state, outputs = local outputs + response of the block's initial state.
//
// The impulse response is not an fp16 number: T is split into a rounded part and the rounded
// remainder (two products), which leaves a relative coefficient error of about 2^-22.
#include <math.h>

#include "hb_device.hpp"
#include "hb_host.hpp"

namespace hb {

constexpr int kIirBlock = 32;                 // samples per block (the K of one product)
constexpr int kIirTile = 16 * kIirBlock;      // samples per wave tile: 16 blocks

struct IirArgs {
    const half_t* in;
    float* out;
    int C, ntiles, chunk;                     // chunk = tiles per lane in the scan
    int64_t T, in_pitch, out_pitch;
    float* end;                               // [C][ntiles][2] state after each tile if it started from zero
    float* start;                             // [C][ntiles][2] true state before each tile
    float m32[4], m512[4], mwave[4];          // state maps over a block, a tile, a wave's tiles in the scan (row-major 2x2)
    float mpow[6][4];                         // ... and over 2^j lanes' tiles, j = 0..5
    float bpow[4][4];                         // state map over 2^j blocks, j = 0..3 (in-tile scan)
    float bsel[16][4];                        // state map over b blocks, b = 0..15
    float ca[kIirBlock], cb[kIirBlock];       // response of output i to the initial state (Y_-1, Y_-2)
    uint16_t thi[kIirBlock], tlo[kIirBlock];  // impulse response h_0..h_31 as rounded fp16 + rounded remainder
    float alpha, beta;
};

struct State2 {
    float a, b;                               // (Y_{t-1}, Y_{t-2})
};

__device__ __forceinline__ State2 iir_step(const float (&m)[4], State2 s, float l1, float l0) {
    return State2{fmaf(m[0], s.a, fmaf(m[1], s.b, l1)), fmaf(m[2], s.a, fmaf(m[3], s.b, l0))};
}

// A-operand fragment of the triangular Toeplitz matrix for output rows 16 hh + c: lane (c, g) holds
// T(16 hh + c, 8g + i) = h_{16 hh + c - 8g - i} (0 above the diagonal).
__device__ __forceinline__ half8 iir_fragment(const uint16_t (&t)[kIirBlock], int hh, int lane) {
    const int d0 = 16 * hh + (lane & 15) - 8 * (lane >> 4);
    half8 f;
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = (d0 - i >= 0 && d0 - i < kIirBlock) ? __builtin_bit_cast(half_t, t[d0 - i]) : (half_t)0;
    return f;
}

// The 512 samples of a tile as the B operand X^T: lane (c = block, g) holds samples 32 c + 8 g .. + 7
// (zeros past the end of the signal).
__device__ __forceinline__ half8 iir_load_tile(const half_t* sig, int64_t t0, int64_t T, int lane) {
    const int64_t t = t0 + 32 * (lane & 15) + 8 * (lane >> 4);
    if (t + 8 <= T) return *reinterpret_cast<const half8_u*>(sig + t);
    half8 r;
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = t + i < T ? sig[t + i] : (half_t)0;
    return r;
}

// value of lane (c - SH) of the same row of 16 lanes, 0 for c < SH
template <int SH>
__device__ __forceinline__ float iir_row_shr(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x110 + SH, 0xf, 0xf, true));
}

// The last two local outputs (Y_31, Y_30) of the tile's 16 blocks sit in elements 3 and 2 of the
// upper-half accumulator, lanes 48 .. 63 (lane 48 + b for block b).  They are copied to every row
// of 16 lanes, and an inclusive scan in four doubling steps (the left half of a merge carried
// across the right half's 2^j blocks by the matching power of the block map) leaves in lane column
// b the state after block b of a tile that started from zero.  The elements are first copied into
// plain registers behind an opaque statement: a lane read straight out of an element of the
// accumulator vector was compiled into a read of element 0.
__device__ __forceinline__ State2 iir_scan_blocks(const IirArgs& p, const floatx4& d1, int lane) {
    float y31 = d1[3], y30 = d1[2];
    asm volatile("" : "+v"(y31), "+v"(y30));
    State2 v{__shfl(y31, 48 + (lane & 15), 64), __shfl(y30, 48 + (lane & 15), 64)};
    const int c = lane & 15;
    {
        const float la = iir_row_shr<1>(v.a), lb = iir_row_shr<1>(v.b);
        if (c >= 1) v = iir_step(p.bpow[0], State2{la, lb}, v.a, v.b);
    }
    {
        const float la = iir_row_shr<2>(v.a), lb = iir_row_shr<2>(v.b);
        if (c >= 2) v = iir_step(p.bpow[1], State2{la, lb}, v.a, v.b);
    }
    {
        const float la = iir_row_shr<4>(v.a), lb = iir_row_shr<4>(v.b);
        if (c >= 4) v = iir_step(p.bpow[2], State2{la, lb}, v.a, v.b);
    }
    {
        const float la = iir_row_shr<8>(v.a), lb = iir_row_shr<8>(v.b);
        if (c >= 8) v = iir_step(p.bpow[3], State2{la, lb}, v.a, v.b);
    }
    return v;
}

// 1  end state of every tile started from zero
__global__ void __launch_bounds__(256) iir2_state_mfma_kernel(IirArgs p) {
    const int lane = threadIdx.x & 63;
    const half8 fhi = iir_fragment(p.thi, 1, lane), flo = iir_fragment(p.tlo, 1, lane);
    const int64_t total = (int64_t)p.C * p.ntiles, nwaves = (int64_t)gridDim.x * 4;
    // waves stride over the tiles: the fragments above are built once per wave
    for (int64_t w = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6; w < total; w += nwaves) {
        const int ch = (int)(w / p.ntiles), tile = (int)(w - (int64_t)ch * p.ntiles);
        const half8 x = iir_load_tile(p.in + (int64_t)ch * p.in_pitch, (int64_t)tile * kIirTile, p.T, lane);
        floatx4 d1 = {0.f, 0.f, 0.f, 0.f};
        d1 = mfma16x16x32(fhi, x, d1);
        d1 = mfma16x16x32(flo, x, d1);
        const State2 s = iir_scan_blocks(p, d1, lane);        // lane column 15: the state after the last block
        if (lane == 15) {
            float* e = p.end + 2 * w;
            e[0] = s.a;
            e[1] = s.b;
        }
    }
}

// 2  true state before every tile: one workgroup of 16 waves per channel, a lane owns `chunk`
// consecutive tiles.  Lanes are scanned in doubling steps, waves chained serially; only the last
// lanes may own fewer tiles, and nothing depends on what follows them.
constexpr int kIirScanWaves = 16;

__device__ __forceinline__ State2 iir_scan_tiles(const IirArgs& p, const float* e, float* st, int lo, int hi, State2 s) {
    // Eight tiles at a time: their end states are requested together, then chained.  Whole groups
    // move as 16-byte pieces (two tiles each): with a lane stride of `chunk` tiles every piece of a
    // load instruction lies in another cache line, so fewer, wider instructions matter.
    for (int t0 = lo; t0 < hi; t0 += 8) {
        float ea[8], eb[8], sa[8], sb[8];
        const bool whole = t0 + 8 <= hi;
        if (whole) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const floatx4 v = *reinterpret_cast<const floatx4_u*>(e + 2 * (t0 + 2 * k));
                ea[2 * k] = v[0];
                eb[2 * k] = v[1];
                ea[2 * k + 1] = v[2];
                eb[2 * k + 1] = v[3];
            }
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                ea[k] = t0 + k < hi ? e[2 * (t0 + k)] : 0.f;
                eb[k] = t0 + k < hi ? e[2 * (t0 + k) + 1] : 0.f;
            }
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            sa[k] = s.a;
            sb[k] = s.b;
            if (t0 + k < hi) s = iir_step(p.m512, s, ea[k], eb[k]);
        }
        if (st) {
            if (whole) {
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    *reinterpret_cast<floatx4_u*>(st + 2 * (t0 + 2 * k)) = floatx4{sa[2 * k], sb[2 * k], sa[2 * k + 1], sb[2 * k + 1]};
            } else {
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    if (t0 + k < hi) {
                        st[2 * (t0 + k)] = sa[k];
                        st[2 * (t0 + k) + 1] = sb[k];
                    }
            }
        }
    }
    return s;
}

__global__ void __launch_bounds__(64 * kIirScanWaves) iir2_scan_kernel(IirArgs p) {
    __shared__ float s_tot[kIirScanWaves][2];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, ch = blockIdx.x;
    const float* e = p.end + 2 * (int64_t)ch * p.ntiles;
    float* st = p.start + 2 * (int64_t)ch * p.ntiles;
    const int lo = (int)min((int64_t)threadIdx.x * p.chunk, (int64_t)p.ntiles), hi = min(lo + p.chunk, p.ntiles);
    const State2 q = iir_scan_tiles(p, e, nullptr, lo, hi, State2{0.f, 0.f});   // the lane's tiles applied to a zero state
    // Inclusive scan over the lanes of a wave in six doubling steps: after step j a lane holds the
    // effect of up to 2^(j+1) lanes ending with itself; the left half of a merge is carried across
    // the 2^j lanes of the right half by the matching power of the lane map.
    auto scan_lanes = [&](State2 v) {
#pragma unroll
        for (int j = 0; j < 6; ++j) {
            const float la = __shfl_up(v.a, 1 << j, 64), lb = __shfl_up(v.b, 1 << j, 64);
            if (lane >= (1 << j)) v = iir_step(p.mpow[j], State2{la, lb}, v.a, v.b);
        }
        return v;
    };
    const State2 incl = scan_lanes(q);                                // lanes 0..l applied to a zero state
    if (lane == 63) {
        s_tot[wv][0] = incl.a;                                        // the wave's tiles applied to a zero state
        s_tot[wv][1] = incl.b;
    }
    __syncthreads();
    State2 ws{0.f, 0.f};                                              // state before the wave's first tile
    for (int w = 0; w < wv; ++w) ws = iir_step(p.mwave, ws, s_tot[w][0], s_tot[w][1]);
    // the wave's start enters through lane 0; the scan then gives the state AFTER every lane
    const State2 q0 = lane == 0 ? iir_step(p.mpow[0], ws, q.a, q.b) : q;
    const State2 after = scan_lanes(q0);
    const float pa = __shfl_up(after.a, 1, 64), pb = __shfl_up(after.b, 1, 64);
    const State2 mine = lane == 0 ? ws : State2{pa, pb};              // state before the lane's first tile
    iir_scan_tiles(p, e, st, lo, hi, mine);
}

// 3  outputs
__global__ void __launch_bounds__(256) iir2_apply_mfma_kernel(IirArgs p) {
    __shared__ __attribute__((aligned(16))) float s_patch[4 * RowPatch<2>::kFloats];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int c = lane & 15, g = lane >> 4;
    half8 fhi[2], flo[2];
    float ra[2][4], rb[2][4];                 // response of the lane's outputs i = 16 hh + 4 g + j to the block's state
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
        fhi[hh] = iir_fragment(p.thi, hh, lane);
        flo[hh] = iir_fragment(p.tlo, hh, lane);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            ra[hh][j] = p.ca[16 * hh + 4 * g + j];
            rb[hh][j] = p.cb[16 * hh + 4 * g + j];
        }
    }
    float bsel[4];                            // state map over the c blocks before the lane's block
#pragma unroll
    for (int i = 0; i < 4; ++i) bsel[i] = p.bsel[c][i];
    const int64_t total = (int64_t)p.C * p.ntiles, nwaves = (int64_t)gridDim.x * 4;
    // waves stride over the tiles: fragments and responses above are built once per wave
    for (int64_t w = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6; w < total; w += nwaves) {
        const int ch = (int)(w / p.ntiles), tile = (int)(w - (int64_t)ch * p.ntiles);
        const int64_t t0 = (int64_t)tile * kIirTile;
        const half8 x = iir_load_tile(p.in + (int64_t)ch * p.in_pitch, t0, p.T, lane);
        floatx4 d[2];
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            d[hh] = floatx4{0.f, 0.f, 0.f, 0.f};
            d[hh] = mfma16x16x32(fhi[hh], x, d[hh]);
            d[hh] = mfma16x16x32(flo[hh], x, d[hh]);
        }
        // state before block c = (tile state carried across c blocks) + (blocks 0 .. c-1 from zero)
        const float* st = p.start + 2 * w;
        const State2 incl = iir_scan_blocks(p, d[1], lane);
        const State2 mine = iir_step(bsel, State2{st[0], st[1]}, iir_row_shr<1>(incl.a), iir_row_shr<1>(incl.b));
        // lane (c = block, g) holds outputs i = 16 hh + 4 g + j of its block: add the response to the block's state
#pragma unroll
        for (int hh = 0; hh < 2; ++hh)
#pragma unroll
            for (int j = 0; j < 4; ++j) d[hh][j] += ra[hh][j] * mine.a + rb[hh][j] * mine.b;
        float* dst = p.out + (int64_t)ch * p.out_pitch + t0;
        if (t0 + kIirTile <= p.T) {
            // the tile is 16 rows (blocks) of 32 consecutive samples
            store_rows_via_lds<2, true>(s_patch + wv * RowPatch<2>::kFloats, dst, kIirBlock, d, lane);
        } else {
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int i = 32 * c + 16 * hh + 4 * g + j;
                    if (t0 + i < p.T) dst[i] = d[hh][j];
                }
        }
    }
}

// Vector-ALU twin of launches 1 and 3: a lane owns one block of 32 samples and runs the recursion
// itself; a wave covers four tiles.  WRITE = false: end states of the tiles started from zero;
// WRITE = true: outputs, every block started from its true state.
template <bool WRITE>
__global__ void __launch_bounds__(256) iir2_blocks_valu_kernel(IirArgs p) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6;
    const int groups = (p.ntiles + 3) / 4;                // waves per channel
    if (wave >= (int64_t)p.C * groups) return;
    const int ch = (int)(wave / groups), tile0 = 4 * (int)(wave - (int64_t)ch * groups);
    const half_t* sig = p.in + (int64_t)ch * p.in_pitch;
    const int64_t t0 = (int64_t)tile0 * kIirTile + (int64_t)kIirBlock * lane;
    // local pass from a zero state: the block's last two outputs
    float y1 = 0.f, y2 = 0.f;
    for (int i = 0; i < kIirBlock; ++i) {
        const float xv = t0 + i < p.T ? (float)sig[t0 + i] : 0.f;
        const float y = fmaf(p.alpha, y1, fmaf(p.beta, y2, xv));
        y2 = y1;
        y1 = y;
    }
    // state before every block, tile by tile
    State2 mine{0.f, 0.f};
    for (int q = 0; q < 4; ++q) {
        const int tile = tile0 + q;
        if (tile >= p.ntiles) break;
        State2 s{0.f, 0.f};
        if (WRITE) {
            const float* st = p.start + 2 * ((int64_t)ch * p.ntiles + tile);
            s = State2{st[0], st[1]};
        }
        for (int b = 0; b < 16; ++b) {
            if (lane == 16 * q + b) mine = s;
            const float l1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, y1), 16 * q + b));
            const float l0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, y2), 16 * q + b));
            s = iir_step(p.m32, s, l1, l0);
        }
        if (!WRITE && lane == 0) {
            float* e = p.end + 2 * ((int64_t)ch * p.ntiles + tile);
            e[0] = s.a;
            e[1] = s.b;
        }
    }
    if (WRITE) {
        // a lane's 32 outputs pass through a patch of LDS that belongs to its wave (pitch 33: the
        // lanes' writes and the rows read back fall into distinct banks) and leave as runs of 64
        // consecutive samples per store instruction, instead of 64 single samples 128 bytes apart
        __shared__ float s_y[4][64 * (kIirBlock + 1)];
        float* const yb = s_y[threadIdx.x >> 6];
        float* dst = p.out + (int64_t)ch * p.out_pitch;
        y1 = mine.a;
        y2 = mine.b;
        for (int i = 0; i < kIirBlock; ++i) {
            const float xv = t0 + i < p.T ? (float)sig[t0 + i] : 0.f;
            const float y = fmaf(p.alpha, y1, fmaf(p.beta, y2, xv));
            yb[lane * (kIirBlock + 1) + i] = y;
            y2 = y1;
            y1 = y;
        }
        const int64_t w0 = (int64_t)tile0 * kIirTile;     // first sample of the wave's four tiles
        for (int r = 0; r < kIirBlock; ++r) {
            const int64_t t = w0 + 64 * r + lane;
            if (t < p.T) dst[t] = yb[(2 * r + (lane >> 5)) * (kIirBlock + 1) + (lane & 31)];
        }
    }
}

// ---------------------------------------------------------------------------
// host: coefficient tables in double

struct Mat2 {
    double v[4];
};
static Mat2 mat2_mul(const Mat2& x, const Mat2& y) {
    return Mat2{{x.v[0] * y.v[0] + x.v[1] * y.v[2], x.v[0] * y.v[1] + x.v[1] * y.v[3],
                 x.v[2] * y.v[0] + x.v[3] * y.v[2], x.v[2] * y.v[1] + x.v[3] * y.v[3]}};
}
static Mat2 mat2_pow(Mat2 m, int64_t n) {
    Mat2 r{{1.0, 0.0, 0.0, 1.0}};
    while (n > 0) {
        if (n & 1) r = mat2_mul(r, m);
        m = mat2_mul(m, m);
        n >>= 1;
    }
    return r;
}

// sum of |h[i]|, i < T, of the filter's impulse response: the factor by which the filter can magnify a
// rounding error made at one sample.  The recurrence runs until the response has died away (both
// state values below 1e-12 of the sum so far), for at most kIirGainSamples samples; a response
// still alive there is taken to stay at its recent size for the rest of the signal.
constexpr int64_t kIirGainSamples = 1 << 16;
constexpr double kIirMaxGain = 16384.0;                   // 2^-24 * gain <= 1e-3
static double iir2_abs_gain(double al, double be, int64_t T) {
    double h1 = 0.0, h2 = 0.0, sum = 0.0, recent = 0.0;
    const int64_t n = T < kIirGainSamples ? T : kIirGainSamples;
    for (int64_t i = 0; i < n; ++i) {
        const double h = i == 0 ? 1.0 : al * h1 + be * h2;
        h2 = h1;
        h1 = h;
        sum += fabs(h);
        if (!(sum < 1.0e300)) return INFINITY;
        recent = fabs(h1) > fabs(h2) ? fabs(h1) : fabs(h2);
        if (i >= 2 && recent < 1.0e-12 * sum) return sum;
    }
    return sum + (double)(T - n) * recent;
}

static hb_status iir2_run(bool valu, const hb_half* in, float* out, int C, int64_t T, int64_t in_pitch, int64_t out_pitch,
                          float alpha, float beta, void* workspace, size_t workspace_bytes, hb_stream stream) {
    if (!in || !out) return HB_ERR_INVALID_ARG;
    if (C < 1 || T < 1 || in_pitch < T || out_pitch < T) return HB_ERR_INVALID_ARG;
    if (!aligned_to(in, 2) || !aligned_to(out, 4)) return HB_ERR_INVALID_ARG;
    if (!(fabsf(alpha) <= 4.f) || !(fabsf(beta) <= 4.f)) return HB_ERR_INVALID_ARG;     // also rejects NaN
    if (C > 65535 || T > ((int64_t)1 << 40)) return HB_ERR_UNSUPPORTED;
    const int64_t ntiles64 = (T + kIirTile - 1) / kIirTile;
    if (ntiles64 * C > ((int64_t)1 << 30)) return HB_ERR_UNSUPPORTED;
    const size_t need = hb_iir2_workspace_size(C, T);
    if (!workspace || workspace_bytes < need || !aligned_to(workspace, 256)) return HB_ERR_WORKSPACE;

    IirArgs a;
    a.in = reinterpret_cast<const half_t*>(in);
    a.out = out;
    a.C = C;
    a.T = T;
    a.in_pitch = in_pitch;
    a.out_pitch = out_pitch;
    a.ntiles = (int)ntiles64;
    a.chunk = (a.ntiles + 64 * kIirScanWaves - 1) / (64 * kIirScanWaves);
    a.end = reinterpret_cast<float*>(workspace);
    a.start = a.end + 2 * (size_t)C * a.ntiles;
    a.alpha = alpha;
    a.beta = beta;
    const double al = alpha, be = beta;
    if (!(iir2_abs_gain(al, be, T) <= kIirMaxGain)) return HB_ERR_UNSUPPORTED;
    // impulse response and the response to the initial state, 32 samples each
    double h[kIirBlock], ca[kIirBlock], cb[kIirBlock];
    for (int i = 0; i < kIirBlock; ++i) {
        h[i] = i == 0 ? 1.0 : al * h[i - 1] + (i >= 2 ? be * h[i - 2] : 0.0);
        const double ca1 = i >= 1 ? ca[i - 1] : 1.0, ca2 = i >= 2 ? ca[i - 2] : (i == 1 ? 1.0 : 0.0);
        const double cb1 = i >= 1 ? cb[i - 1] : 0.0, cb2 = i >= 2 ? cb[i - 2] : (i == 1 ? 0.0 : 1.0);
        ca[i] = al * ca1 + be * ca2;
        cb[i] = al * cb1 + be * cb2;
    }
    for (int i = 0; i < kIirBlock; ++i) {
        if (!(fabs(h[i]) < 3.0e4) || !(fabs(ca[i]) < 1.0e30) || !(fabs(cb[i]) < 1.0e30)) return HB_ERR_UNSUPPORTED;
        a.thi[i] = float_to_half_bits((float)h[i]);
        a.tlo[i] = float_to_half_bits((float)(h[i] - (double)half_bits_to_float(a.thi[i])));
        a.ca[i] = (float)ca[i];
        a.cb[i] = (float)cb[i];
    }
    const Mat2 m32{{ca[31], cb[31], ca[30], cb[30]}};
    const Mat2 m512 = mat2_pow(m32, 16), mchunk = mat2_pow(m512, a.chunk), mwave = mat2_pow(mchunk, 64);
    for (int i = 0; i < 4; ++i) {
        if (!(fabs(m512.v[i]) < 1.0e30) || !(fabs(mwave.v[i]) < 1.0e30)) return HB_ERR_UNSUPPORTED;
        a.m32[i] = (float)m32.v[i];
        a.m512[i] = (float)m512.v[i];
        a.mwave[i] = (float)mwave.v[i];
    }
    for (int j = 0; j < 4; ++j) {
        const Mat2 bp = mat2_pow(m32, (int64_t)1 << j);
        for (int i = 0; i < 4; ++i) a.bpow[j][i] = (float)bp.v[i];
    }
    for (int b = 0; b < 16; ++b) {
        const Mat2 bs = mat2_pow(m32, b);
        for (int i = 0; i < 4; ++i) {
            if (!(fabs(bs.v[i]) < 1.0e30)) return HB_ERR_UNSUPPORTED;
            a.bsel[b][i] = (float)bs.v[i];
        }
    }
    for (int j = 0; j < 6; ++j) {
        const Mat2 mp = mat2_pow(mchunk, (int64_t)1 << j);
        for (int i = 0; i < 4; ++i) {
            if (!(fabs(mp.v[i]) < 1.0e30)) return HB_ERR_UNSUPPORTED;
            a.mpow[j][i] = (float)mp.v[i];
        }
    }

    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const int64_t waves = (int64_t)C * (valu ? (a.ntiles + 3) / 4 : a.ntiles);
    int64_t wgs = (waves + 3) / 4;
    if (!valu && wgs > 8 * num_cu()) wgs = 8 * num_cu();          // the matrix kernels' waves stride over the tiles
    const unsigned blocks = (unsigned)wgs;
    if (valu) hipLaunchKernelGGL(iir2_blocks_valu_kernel<false>, dim3(blocks), dim3(256), 0, st, a);
    else hipLaunchKernelGGL(iir2_state_mfma_kernel, dim3(blocks), dim3(256), 0, st, a);
    hipLaunchKernelGGL(iir2_scan_kernel, dim3(C), dim3(64 * kIirScanWaves), 0, st, a);
    if (valu) hipLaunchKernelGGL(iir2_blocks_valu_kernel<true>, dim3(blocks), dim3(256), 0, st, a);
    else hipLaunchKernelGGL(iir2_apply_mfma_kernel, dim3(blocks), dim3(256), 0, st, a);
    return launch_status();
}

}  // namespace hb

extern "C" size_t hb_iir2_workspace_size(int C, int64_t T) {
    if (C < 1 || T < 1) return 0;
    const size_t ntiles = (size_t)((T + hb::kIirTile - 1) / hb::kIirTile);
    return 2 * 2 * sizeof(float) * (size_t)C * ntiles;
}

extern "C" double hb_iir2_abs_gain(float alpha, float beta, int64_t T) {
    if (T < 1 || !(fabsf(alpha) <= 4.f) || !(fabsf(beta) <= 4.f)) return -1.0;
    return hb::iir2_abs_gain(alpha, beta, T);
}

extern "C" hb_status hb_iir2(const hb_half* in, float* out, int C, int64_t T, int64_t in_pitch, int64_t out_pitch,
                             float alpha, float beta, void* workspace, size_t workspace_bytes, hb_stream stream) {
    return hb::iir2_run(false, in, out, C, T, in_pitch, out_pitch, alpha, beta, workspace, workspace_bytes, stream);
}

extern "C" hb_status hb_iir2_valu(const hb_half* in, float* out, int C, int64_t T, int64_t in_pitch, int64_t out_pitch,
                                  float alpha, float beta, void* workspace, size_t workspace_bytes, hb_stream stream) {
    return hb::iir2_run(true, in, out, C, T, in_pitch, out_pitch, alpha, beta, workspace, workspace_bytes, stream);
}
