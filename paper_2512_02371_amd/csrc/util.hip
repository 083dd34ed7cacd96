// Status strings, the streaming-copy bandwidth reference and the MFMA
// operand-layout self-check.
#include "hb_device.hpp"
#include "hb_host.hpp"

namespace hb {

__global__ void __launch_bounds__(256) copy_f16_f32_kernel(const half_t* __restrict__ in,
                                                           float* __restrict__ out, int64_t n) {
    const int64_t nvec = n >> 3;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += stride) {
        const half8 v = reinterpret_cast<const half8*>(in)[i];
        floatx4 a = {(float)v[0], (float)v[1], (float)v[2], (float)v[3]};
        floatx4 b = {(float)v[4], (float)v[5], (float)v[6], (float)v[7]};
        reinterpret_cast<floatx4*>(out)[2 * i] = a;
        reinterpret_cast<floatx4*>(out)[2 * i + 1] = b;
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 7)) {
        const int64_t i = (nvec << 3) + threadIdx.x;
        out[i] = (float)in[i];
    }
}

// One MFMA on dense row-major operands, gathered and scattered through the
// operand-to-lane maps documented in hb_device.hpp.
__global__ void __launch_bounds__(64) mfma_probe_kernel(int which, const void* Av, const void* Bv, float* D) {
    const int lane = threadIdx.x;
    if (which == 0) {          // 16x16x32 f16
        const half_t* A = (const half_t*)Av; const half_t* B = (const half_t*)Bv;
        const int c = lane & 15, g = lane >> 4;
        half8 a, b;
        for (int i = 0; i < 8; ++i) { a[i] = A[c * 32 + 8 * g + i]; b[i] = B[(8 * g + i) * 16 + c]; }
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
        acc = mfma16x16x32(a, b, acc);
        for (int v = 0; v < 4; ++v) D[(4 * g + v) * 16 + c] = acc[v];
    } else if (which == 1) {   // 16x16x16 f16
        const half_t* A = (const half_t*)Av; const half_t* B = (const half_t*)Bv;
        const int c = lane & 15, g = lane >> 4;
        half4 a, b;
        for (int i = 0; i < 4; ++i) { a[i] = A[c * 16 + 4 * g + i]; b[i] = B[(4 * g + i) * 16 + c]; }
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
        acc = mfma16x16x16(a, b, acc);
        for (int v = 0; v < 4; ++v) D[(4 * g + v) * 16 + c] = acc[v];
    } else if (which == 2) {   // 32x32x16 f16
        const half_t* A = (const half_t*)Av; const half_t* B = (const half_t*)Bv;
        const int c = lane & 31, h = lane >> 5;
        half8 a, b;
        for (int i = 0; i < 8; ++i) { a[i] = A[c * 16 + 8 * h + i]; b[i] = B[(8 * h + i) * 32 + c]; }
        floatx16 acc;
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
        acc = mfma32x32x16(a, b, acc);
        for (int q = 0; q < 4; ++q)
            for (int r = 0; r < 4; ++r) D[(8 * q + 4 * h + r) * 32 + c] = acc[4 * q + r];
    } else {                   // 16x16x4 f32
        const float* A = (const float*)Av; const float* B = (const float*)Bv;
        const int c = lane & 15, g = lane >> 4;
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
        acc = mfma16x16x4f32(A[c * 4 + g], B[g * 16 + c], acc);
        for (int v = 0; v < 4; ++v) D[(4 * g + v) * 16 + c] = acc[v];
    }
}

}  // namespace hb

extern "C" const char* hb_status_string(hb_status s) {
    switch (s) {
        case HB_OK: return "HB_OK";
        case HB_ERR_INVALID_ARG: return "HB_ERR_INVALID_ARG";
        case HB_ERR_UNSUPPORTED: return "HB_ERR_UNSUPPORTED";
        case HB_ERR_WORKSPACE: return "HB_ERR_WORKSPACE";
        case HB_ERR_HIP: return "HB_ERR_HIP";
    }
    return "HB_ERR_UNKNOWN";
}

extern "C" hb_status hb_copy_f16_f32(const hb_half* in, float* out, int64_t n, hb_stream stream) {
    using namespace hb;
    if (!in || !out || n < 1) return HB_ERR_INVALID_ARG;
    if (!aligned_to(in, 16) || !aligned_to(out, 16)) return HB_ERR_INVALID_ARG;
    const int64_t nvec = (n + 7) >> 3;
    const int blocks = (int)((nvec + 255) / 256 < kMaxStreamBlocks * 4 ? (nvec + 255) / 256 : kMaxStreamBlocks * 4);
    hipLaunchKernelGGL(copy_f16_f32_kernel, dim3(blocks), dim3(256), 0, reinterpret_cast<hipStream_t>(stream),
                       reinterpret_cast<const half_t*>(in), out, n);
    return launch_status();
}

extern "C" hb_status hb_mfma_probe(int which, const void* A, const void* B, float* D, hb_stream stream) {
    using namespace hb;
    if (!A || !B || !D || which < 0 || which > 3) return HB_ERR_INVALID_ARG;
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(1), dim3(64), 0, reinterpret_cast<hipStream_t>(stream), which, A, B, D);
    return launch_status();
}
