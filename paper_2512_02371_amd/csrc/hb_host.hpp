// Host-side helpers shared by the C-ABI entry points: argument checks that run
// before any HIP call, launch-status mapping, and launch geometry constants.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "hb.h"

namespace hb {

// Filter taps as they travel inside the kernel arguments (fp16 bits, zero padded).
struct Taps {
    uint16_t v[HB_MAX_TAPS];
};

// MI355X: 256 compute units, 4 SIMDs each.  Streaming kernels launch at most this
// many 256-thread workgroups and let every wave walk a strided list of tasks.
constexpr int kNumCU = 256;
constexpr int kMaxStreamBlocks = kNumCU * 8;

inline bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

inline hb_status check_image(const void* in, const void* out, int H, int W,
                             int64_t in_pitch, int64_t out_pitch) {
    if (!in || !out) return HB_ERR_INVALID_ARG;
    if (H < 1 || W < 1) return HB_ERR_INVALID_ARG;
    if (in_pitch < W || out_pitch < W) return HB_ERR_INVALID_ARG;
    if (!aligned_to(in, 2) || !aligned_to(out, 4)) return HB_ERR_INVALID_ARG;
    // rows are addressed with 32-bit element offsets inside a row and 64-bit row bases
    if ((int64_t)H * in_pitch > ((int64_t)1 << 40) || (int64_t)H * out_pitch > ((int64_t)1 << 40))
        return HB_ERR_UNSUPPORTED;
    return HB_OK;
}

inline hb_status check_taps(const hb_half* taps, int ntaps, int anchor) {
    if (!taps) return HB_ERR_INVALID_ARG;
    if (ntaps < 1 || ntaps > HB_MAX_TAPS) return HB_ERR_INVALID_ARG;
    if (anchor < 0 || anchor >= ntaps) return HB_ERR_INVALID_ARG;
    return HB_OK;
}

inline Taps pack_taps(const hb_half* taps, int ntaps) {
    Taps t;
    memset(&t, 0, sizeof(t));
    memcpy(t.v, taps, sizeof(uint16_t) * (size_t)ntaps);
    return t;
}

inline hb_status launch_status() { return hipGetLastError() == hipSuccess ? HB_OK : HB_ERR_HIP; }

inline int floor_div(int a, int b) { return a >= 0 ? a / b : -((-a + b - 1) / b); }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

}  // namespace hb
