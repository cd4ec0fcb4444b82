// Measurement aid: a register-only loop of the block-scaled FP4 matrix-core instruction that the
// GEMM uses (v_mfma_scale_f32_32x32x64_f8f6f4, both operands FP4), with no memory traffic at all.
// Timed by the caller, it gives the rate the matrix cores of this machine sustain under its power
// limit -- which depends strongly on the operand bits -- as the ceiling against which the GEMM's
// rate can be read besides the published peak.
#include "common.h"

namespace adahop {

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t mix(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x7feb352dU;
    x ^= x >> 15;
    x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}

// One workgroup of four waves per launch slot; every wave runs iters x 16 independent instructions
// (a 4 x 4 arrangement of accumulators over 4 + 4 operand fragments, as in the GEMM).  idle_sleeps > 0 puts
// that many short sleeps after every 16 instructions: under a power limit the clock rises when the matrix
// cores idle part of the time, so the rate falls by much less than the duty cycle.
__global__ __launch_bounds__(256) void k_probe_mfma(int random_operands, int idle_sleeps, int iters, float *sink)
{
    v16f acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    v8i a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const uint32_t s = threadIdx.x * 64 + i * 8 + q + blockIdx.x * 7919u;
            a[i][q] = q < 4 ? (int)(random_operands ? mix(s + 1) : 0x22222222u) : 0;
            b[i][q] = q < 4 ? (int)(random_operands ? mix(s + 40) : 0x22222222u) : 0;
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i * 4 + j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[i], b[j], acc[i * 4 + j], 4, 4, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
        for (int g = 0; g < idle_sleeps; ++g) __builtin_amdgcn_s_sleep(8); // an idle stretch after every 16 instructions
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    if (s == 123.456f) sink[0] = s; // keeps the loop alive; practically never true
}

} // namespace

} // namespace adahop

using namespace adahop;

extern "C" int adahop_probe_mfma_rate(int random_operands, int idle_sleeps, int workgroups, int iters, float *sink,
                                      void *stream)
{
    if (idle_sleeps < 0 || idle_sleeps > 64) return ADAHOP_E_INVALID_ARG;
    if (workgroups < 1 || workgroups > 65536 || iters < 1 || iters > (1 << 24) || !sink) return ADAHOP_E_INVALID_ARG;
    hipLaunchKernelGGL(k_probe_mfma, dim3((unsigned)workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                       random_operands, idle_sleeps, iters, sink);
    return check_launch();
}
