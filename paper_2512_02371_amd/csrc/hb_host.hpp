// Host-side helpers shared by the C-ABI entry points: argument checks that run
// before any HIP call, launch-status mapping, and launch geometry constants.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <map>
#include <mutex>
#include <utility>

#include "hb.h"

namespace hb {

// Filter taps as they travel inside the kernel arguments: a zero-padded fp16 table (entry
// kTapPad + t holds taps[t] for 0 <= t < ntaps and zero for every other t in
// [-kTapPad, MAXT + 48)), from which a Toeplitz fragment is eight consecutive entries,
// and, for the border tiles, the taps and their running sums in fp32.  MAXT is the largest tap
// count of the entry point (hb_fir1d: 256, hb_sepblur: 64 per axis).
constexpr int kTapPad = 16;
template <int MAXT>
struct TapsT {
    uint16_t tab[kTapPad + MAXT + 48];
};
template <int MAXT>
struct FoldTablesT {
    float kf[MAXT];          // taps as fp32, zero beyond ntaps
    float pfx[MAXT + 1];     // pfx[i] = sum of taps t < i
};
using Taps = TapsT<HB_MAX_TAPS>;
using FoldTables = FoldTablesT<HB_MAX_TAPS>;

// Streaming kernels launch one short-lived wave per task (the dispatcher keeps the memory
// pipes fed best that way); beyond this many 256-thread workgroups every wave walks a
// strided list of tasks instead.  The number of compute units (MI355X: 256, 4 SIMDs each) is
// read from the device, see num_cu().
constexpr int kMaxStreamBlocks = 1 << 20;

// Tasks form an nct x nseg grid.  Those in the rectangle [c0, c1) x [s0, s1) touch no image
// border and take a lean code path (plain loads, unmasked stores); the others take a
// border-aware path that is written for small register use rather than speed, so that it
// does not lower the occupancy of the kernel that holds both.
struct TaskGrid {
    int nct, nseg;
    int c0, c1, s0, s1;
    __host__ __device__ int count() const { return nct * nseg; }
    __device__ bool interior(int seg, int ct) const { return ct >= c0 && ct < c1 && seg >= s0 && seg < s1; }
};

// Interior range [lo, hi) of the n task indices t whose footprint
// [t*step - before, t*step + after) lies inside [0, extent); lo = hi = 0 when empty.
inline void interior_range(int n, int step, int before, int after, int extent, int& lo, int& hi) {
    lo = before <= 0 ? 0 : (before + step - 1) / step;
    hi = extent - after < 0 ? 0 : (extent - after) / step + 1;
    if (hi > n) hi = n;
    if (hi <= lo) lo = hi = 0;
}

inline bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

inline hb_status check_image(const void* in, const void* out, int H, int W,
                             int64_t in_pitch, int64_t out_pitch) {
    if (!in || !out) return HB_ERR_INVALID_ARG;
    if (H < 1 || W < 1) return HB_ERR_INVALID_ARG;
    if (in_pitch < W || out_pitch < W) return HB_ERR_INVALID_ARG;
    if (!aligned_to(in, 2) || !aligned_to(out, 4)) return HB_ERR_INVALID_ARG;
    // lanes address a 16-row group with 32-bit byte offsets from a 64-bit group base
    if (in_pitch > ((int64_t)1 << 26) || out_pitch > ((int64_t)1 << 26)) return HB_ERR_UNSUPPORTED;
    return HB_OK;
}

inline hb_status check_taps(const hb_half* taps, int ntaps, int anchor, int max_taps = HB_MAX_TAPS) {
    if (!taps) return HB_ERR_INVALID_ARG;
    if (ntaps < 1 || ntaps > max_taps) return HB_ERR_INVALID_ARG;
    if (anchor < 0 || anchor >= ntaps) return HB_ERR_INVALID_ARG;
    return HB_OK;
}

inline float half_bits_to_float(uint16_t h) {
    const uint32_t sign = (uint32_t)(h >> 15) << 31;
    int e = (h >> 10) & 0x1f;
    uint32_t f = h & 0x3ff, bits;
    if (e == 0) {
        if (f == 0) {
            bits = sign;
        } else {                                          // subnormal: renormalise
            e = 1;
            while (!(f & 0x400)) { f <<= 1; --e; }
            bits = sign | ((uint32_t)(e + 112) << 23) | ((f & 0x3ff) << 13);
        }
    } else if (e == 31) {
        bits = sign | 0x7f800000u | (f << 13);
    } else {
        bits = sign | ((uint32_t)(e + 112) << 23) | (f << 13);
    }
    float out;
    memcpy(&out, &bits, sizeof(out));
    return out;
}

// float -> fp16 bit pattern, round to nearest even (finite inputs of moderate size only).
inline uint16_t float_to_half_bits(float v) {
    uint32_t b;
    memcpy(&b, &v, sizeof(b));
    const uint32_t sign = (b >> 16) & 0x8000u;
    const int32_t e = (int32_t)((b >> 23) & 0xff) - 127 + 15;
    uint32_t m = b & 0x7fffffu;
    if (e >= 31) return (uint16_t)(sign | 0x7c00u);                       // overflow -> inf
    if (e <= 0) {                                                         // subnormal or zero
        if (e < -10) return (uint16_t)sign;
        m |= 0x800000u;
        const int shift = 14 - e;
        uint32_t h = m >> shift;
        const uint32_t rest = m & ((1u << shift) - 1), halfway = 1u << (shift - 1);
        if (rest > halfway || (rest == halfway && (h & 1))) ++h;
        return (uint16_t)(sign | h);
    }
    uint32_t h = ((uint32_t)e << 10) | (m >> 13);
    const uint32_t rest = m & 0x1fffu;
    if (rest > 0x1000u || (rest == 0x1000u && (h & 1))) ++h;             // may carry into the exponent: still right
    return (uint16_t)(sign | h);
}

template <int MAXT = HB_MAX_TAPS>
inline TapsT<MAXT> pack_taps(const hb_half* taps, int ntaps) {
    TapsT<MAXT> t;
    memset(&t, 0, sizeof(t));
    memcpy(t.tab + kTapPad, taps, sizeof(uint16_t) * (size_t)ntaps);
    return t;
}

template <int MAXT = HB_MAX_TAPS>
inline FoldTablesT<MAXT> pack_fold_tables(const hb_half* taps, int ntaps) {
    FoldTablesT<MAXT> ft;
    memset(&ft, 0, sizeof(ft));
    float run = 0.f;
    for (int i = 0; i <= MAXT; ++i) {
        ft.pfx[i] = run;
        if (i < ntaps) {
            ft.kf[i] = half_bits_to_float(taps[i]);
            run += ft.kf[i];
        }
    }
    return ft;
}

inline hb_status launch_status() { return hipGetLastError() == hipSuccess ? HB_OK : HB_ERR_HIP; }

// Raises a kernel's dynamic LDS limit to `bytes`.  The runtime call costs about ten microseconds of
// host time, so it is made once per kernel and device (and again only for a larger size).
inline hb_status allow_dynamic_lds(const void* kernel, size_t bytes) {
    static std::mutex mu;
    static std::map<std::pair<const void*, int>, size_t> raised;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return HB_ERR_HIP;
    std::lock_guard<std::mutex> lock(mu);
    size_t& have = raised[std::make_pair(kernel, dev)];
    if (have >= bytes) return HB_OK;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) return HB_ERR_HIP;
    have = bytes;
    return HB_OK;
}

// Compute units of the current device (0 if the query fails), read once per device.
inline int device_num_cu() {
    static std::mutex mu;
    static std::map<int, int> known;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    std::lock_guard<std::mutex> lock(mu);
    auto it = known.find(dev);
    if (it != known.end()) return it->second;
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) n = 0;
    known[dev] = n;
    return n;
}

// Compute units used for launch geometry: the device's count, 256 (MI355X) if it cannot be read.
inline int num_cu() {
    const int n = device_num_cu();
    return n > 0 ? n : 256;
}

inline int floor_div(int a, int b) { return a >= 0 ? a / b : -((-a + b - 1) / b); }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

}  // namespace hb
