// Status strings, the streaming-copy bandwidth reference and the MFMA
// operand-layout self-check.
#include "hb_device.hpp"
#include "hb_host.hpp"

namespace hb {

// The bandwidth reference: out[i] = (float) in[i].  Shaped the way the memory system of this chip
// takes a 2 B in + 4 B out stream best (measured): short-lived waves that request everything they
// read before they convert anything, 8-byte loads so that lane l of a store instruction writes the
// 16 bytes at 16 l (every store instruction is 1 KB of consecutive bytes: whole 128-byte lines,
// which is what the streaming, non-temporal stores want), and one wave per 2048 elements in plain
// launch order, so that the waves in flight sweep a compact window of both arrays.
#ifndef HB_COPY_VEC
#define HB_COPY_VEC 2
#endif
constexpr int kCopyVec = HB_COPY_VEC;                     // 8-byte loads (16-byte stores) per lane
__global__ void __launch_bounds__(256) copy_f16_f32_kernel(const half_t* __restrict__ in,
                                                           float* __restrict__ out, int64_t n) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t e0 = wave * (256 * kCopyVec);           // first element of this wave's chunk
    if (e0 + 256 * kCopyVec <= n) {
        half4 v[kCopyVec];
#pragma unroll
        for (int i = 0; i < kCopyVec; ++i) v[i] = *reinterpret_cast<const half4*>(in + e0 + 256 * i + 4 * lane);
#pragma unroll
        for (int i = 0; i < kCopyVec; ++i) {
            const floatx4 f = {(float)v[i][0], (float)v[i][1], (float)v[i][2], (float)v[i][3]};
            __builtin_nontemporal_store(f, reinterpret_cast<floatx4*>(out + e0 + 256 * i + 4 * lane));
        }
    } else {
        for (int64_t i = e0 + lane; i < n && i < e0 + 256 * kCopyVec; i += 64) out[i] = (float)in[i];
    }
}

// The K = 16 product lives here only: the stage kernels have no way to issue it.
__device__ __forceinline__ floatx4 probe_mfma16x16x16(half4 a, half4 b, floatx4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x16f16(a, b, c, 0, 0, 0);
}

// One MFMA on dense row-major operands, gathered and scattered through the
// operand-to-lane maps documented in hb_device.hpp; which = 4 chains a K = 32 and a K = 16
// product on one accumulator, back to back (the order the stage kernels avoid).
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
        acc = probe_mfma16x16x16(a, b, acc);
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
    } else if (which == 4) {   // D = A32 B32 + A16 B16: A = [16 x 32 | 16 x 16], B = [32 x 16 | 16 x 16], each part dense
        const half_t* A = (const half_t*)Av; const half_t* B = (const half_t*)Bv;
        const int c = lane & 15, g = lane >> 4;
        half8 a, b;
        half4 a2, b2;
        for (int i = 0; i < 8; ++i) { a[i] = A[c * 32 + 8 * g + i]; b[i] = B[(8 * g + i) * 16 + c]; }
        for (int i = 0; i < 4; ++i) { a2[i] = A[512 + c * 16 + 4 * g + i]; b2[i] = B[512 + (4 * g + i) * 16 + c]; }
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
        __builtin_amdgcn_sched_barrier(0);
        acc = mfma16x16x32(a, b, acc);
        acc = probe_mfma16x16x16(a2, b2, acc);
        __builtin_amdgcn_sched_barrier(0);
        for (int v = 0; v < 4; ++v) D[(4 * g + v) * 16 + c] = acc[v];
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
    const int64_t waves = (n + 256 * kCopyVec - 1) / (256 * kCopyVec);
    const int64_t blocks = (waves + 3) / 4;
    if (blocks > 0x7fffffff) return HB_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(copy_f16_f32_kernel, dim3((unsigned)blocks), dim3(256), 0, reinterpret_cast<hipStream_t>(stream),
                       reinterpret_cast<const half_t*>(in), out, n);
    return launch_status();
}

extern "C" hb_status hb_mfma_probe(int which, const void* A, const void* B, float* D, hb_stream stream) {
    using namespace hb;
    if (!A || !B || !D || which < 0 || which > 4) return HB_ERR_INVALID_ARG;
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(1), dim3(64), 0, reinterpret_cast<hipStream_t>(stream), which, A, B, D);
    return launch_status();
}
