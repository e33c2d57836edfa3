// Measurement aid of libsage: a kernel that does nothing but issue the matrix instructions the attention
// kernel uses, back to back on independent accumulators, so that the benchmark can state the attention
// kernel's throughput against the matrix-pipe rate this GPU actually sustains (besides the published peak).
// Not part of the method; no step of the forward pass calls it.
#include "../../include/sage.h"
#include "sage_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kAcc = 8;  // independent accumulators per wavefront (no instruction waits for the one before it)

// kind 0: v_mfma_i32_16x16x64_i8            (S = Q^ K^T)
// kind 1: v_mfma_f32_16x16x128_f8f6f4, FP8  (O += P^ V^)
// kind 2: v_mfma_f32_16x16x32_fp8_fp8       (the older FP8 form, for comparison)
// kind 3: two of kind 0 per one of kind 1   (the attention kernel's own mix: equal operation counts)
template <int KIND>
__global__ __launch_bounds__(256, 4) void mfma_rate_kernel(int iters, float *sink) {
#if defined(__HIP_DEVICE_COMPILE__)
    const int lane = threadIdx.x & 63;
    // operands that are neither zero nor uniform (an all-zero operand would flatter the clock)
    v8i a8, b8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a8[i] = 0x38302820 + 0x01010101 * ((lane + i) & 7);   // FP8 bytes around 0.5 .. 1
        b8[i] = 0x30383028 + 0x01010101 * ((lane * 3 + i) & 7);
    }
    const v4i a4 = {a8[0], a8[1], a8[2], a8[3]}, b4 = {b8[0], b8[1], b8[2], b8[3]};
    const long a2 = ((long)a8[0] << 32) | (unsigned)a8[1], b2 = ((long)b8[0] << 32) | (unsigned)b8[1];
    v4i ci[kAcc];
    v4f cf[kAcc];
#pragma unroll
    for (int k = 0; k < kAcc; ++k) {
        ci[k] = v4i{0, 0, 0, 0};
        cf[k] = v4f{0.f, 0.f, 0.f, 0.f};
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < kAcc; ++k) {
            if constexpr (KIND == 0) {
                ci[k] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a4, b4, ci[k], 0, 0, 0);
            } else if constexpr (KIND == 1) {
                cf[k] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, b8, cf[k], 0, 0, 0, 0, 0, 0);
            } else if constexpr (KIND == 2) {
                cf[k] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(a2, b2, cf[k], 0, 0, 0);
            } else {
                ci[k] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a4, b4, ci[k], 0, 0, 0);
                ci[(k + 4) % kAcc] = __builtin_amdgcn_mfma_i32_16x16x64_i8(b4, a4, ci[(k + 4) % kAcc], 0, 0, 0);
                cf[k] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, b8, cf[k], 0, 0, 0, 0, 0, 0);
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < kAcc; ++k)
#pragma unroll
        for (int i = 0; i < 4; ++i) s += cf[k][i] + (float)ci[k][i];
    if (s == 12345.678f) sink[0] = s;  // keeps the loop alive; practically never true
#endif
}

}  // namespace

extern "C" int sage_diag_mfma_rate(int kind, int iters, int workgroups, float *sink, double *ops_per_launch,
                                   void *stream) {
    if (kind < 0 || kind > 3 || iters < 1 || iters > (1 << 24) || workgroups < 1 || workgroups > (1 << 20) || !sink ||
        !ops_per_launch)
        return SAGE_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    (void)hipGetLastError();
    const double per_iter[4] = {kAcc * 32768.0, kAcc * 65536.0, kAcc * 16384.0, kAcc * (2 * 32768.0 + 65536.0)};
    *ops_per_launch = per_iter[kind] * iters * 4.0 /* wavefronts */ * workgroups;
    switch (kind) {
        case 0: mfma_rate_kernel<0><<<workgroups, 256, 0, s>>>(iters, sink); break;
        case 1: mfma_rate_kernel<1><<<workgroups, 256, 0, s>>>(iters, sink); break;
        case 2: mfma_rate_kernel<2><<<workgroups, 256, 0, s>>>(iters, sink); break;
        default: mfma_rate_kernel<3><<<workgroups, 256, 0, s>>>(iters, sink); break;
    }
    return hipGetLastError() == hipSuccess ? SAGE_OK : SAGE_EHIP;
}

extern "C" int sage_diag_quant_kv_path(int path, long long wait_ticks) {
    if (path < 0 || path > 2) return SAGE_EINVAL;
    sage::set_quant_kv_path(path, wait_ticks);
    return SAGE_OK;
}
