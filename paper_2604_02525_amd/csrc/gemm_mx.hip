// Block-scaled FP4 GEMM on the CDNA4 matrix cores (the MXFP4 term of paper Eq. 4 / 5 / 7 / 8), with
// the K-channel outlier product fused in front of it as BF16 matrix-core iterations on the same
// accumulators.
//
//   C[m, n] = sum_t Ag[m, t] Bg[n, t]                                   (bf16, optional, t < kpad)
//           + sum_blk 2^(sa[m,blk]-127) 2^(sb[n,blk]-127) sum_{i<32} a[m,32blk+i] b[n,32blk+i]
//
// Instruction used: v_mfma_scale_f32_32x32x64_f8f6f4 with both operands FP4.  Operand layout, as
// this file relies on it: lane l supplies, for row (A) / column (B) l % 32, the 32 consecutive
// K-elements of MX block l / 32 of the 64-wide K step as 16 packed bytes (element 2t in the low
// nibble of byte t), plus that block's E8M0 scale in a byte of the scale register.  The 32x32 fp32
// accumulator is the usual one: register r of lane l is C[8*(r/4) + 4*(l/32) + r%4][l % 32].
// v_mfma_f32_32x32x16_bf16 uses the same accumulator layout; lane l supplies K-elements
// 8*(l/32) .. +7 of row / column l % 32.
#include "common.h"

namespace adahop {

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

__device__ __forceinline__ v16f mfma_fp4(uint4 a, uint4 b, v16f c, int sa, int sb)
{
    v8i av = {(int)a.x, (int)a.y, (int)a.z, (int)a.w, 0, 0, 0, 0};
    v8i bv = {(int)b.x, (int)b.y, (int)b.z, (int)b.w, 0, 0, 0, 0};
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, bv, c, 4, 4, 0, sa, 0, sb);
}

__device__ __forceinline__ v16f mfma_bf16(uint4 a, uint4 b, v16f c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
}

// ------------------------------------------------------------------------------------------------
// Generic kernel: any M, N, any K % 32 == 0.  Workgroup tile 128x128, four waves as 2x2, each wave
// 64x64 (2x2 matrix-core tiles), operands read straight from global memory with bounds checks.
// It is the reference for the layout assumptions above and the fallback for ragged shapes.
// ------------------------------------------------------------------------------------------------
template <bool ACCUMULATE>
__global__ __launch_bounds__(256) void k_gemm_mx_generic(int64_t M, int64_t N, int64_t K,
                                                         const uint8_t *__restrict__ a_codes,
                                                         const uint8_t *__restrict__ a_scales,
                                                         const uint8_t *__restrict__ b_codes,
                                                         const uint8_t *__restrict__ b_scales, float *__restrict__ C,
                                                         int64_t ldc, const uint16_t *__restrict__ Ag,
                                                         const uint16_t *__restrict__ Bg, int kpad)
{
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int l32 = lane & 31, h = lane >> 5;
    const int64_t m0 = (int64_t)blockIdx.y * 128 + (w >> 1) * 64;
    const int64_t n0 = (int64_t)blockIdx.x * 128 + (w & 1) * 64;
    const int64_t rowA[2] = {m0 + l32, m0 + 32 + l32};
    const int64_t rowB[2] = {n0 + l32, n0 + 32 + l32};

    v16f acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    for (int t0 = 0; t0 < kpad; t0 += 16) {
        uint4 a[2], b[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            a[i] = rowA[i] < M ? *reinterpret_cast<const uint4 *>(Ag + rowA[i] * kpad + t0 + h * 8) : make_uint4(0, 0, 0, 0);
            b[i] = rowB[i] < N ? *reinterpret_cast<const uint4 *>(Bg + rowB[i] * kpad + t0 + h * 8) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = mfma_bf16(a[i], b[j], acc[i][j]);
    }

    const int64_t KB = K >> 5;
    for (int64_t kb = 0; kb < KB; kb += 2) {
        const int64_t blk = kb + h;
        const bool kok = blk < KB;
        uint4 a[2], b[2];
        int sa[2], sb[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const bool oka = kok && rowA[i] < M;
            const bool okb = kok && rowB[i] < N;
            a[i] = oka ? *reinterpret_cast<const uint4 *>(a_codes + rowA[i] * (K >> 1) + blk * 16) : make_uint4(0, 0, 0, 0);
            b[i] = okb ? *reinterpret_cast<const uint4 *>(b_codes + rowB[i] * (K >> 1) + blk * 16) : make_uint4(0, 0, 0, 0);
            sa[i] = oka ? (int)a_scales[rowA[i] * KB + blk] : 127;
            sb[i] = okb ? (int)b_scales[rowB[i] * KB + blk] : 127;
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = mfma_fp4(a[i], b[j], acc[i][j], sa[i], sb[j]);
    }

#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int64_t col = n0 + j * 32 + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = m0 + i * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
                if (row < M && col < N) {
                    float *p = C + row * ldc + col;
                    if constexpr (ACCUMULATE)
                        *p = *p + acc[i][j][r];
                    else
                        *p = acc[i][j][r];
                }
            }
        }
}

} // namespace

int launch_gemm_mx(int64_t M, int64_t N, int64_t K, const uint8_t *a_codes, const uint8_t *a_scales,
                   const uint8_t *b_codes, const uint8_t *b_scales, float *C, int64_t ldc, const uint16_t *Ag,
                   const uint16_t *Bg, int kpad, hipStream_t st)
{
    if (M == 0 || N == 0) return ADAHOP_OK;
    dim3 grid((unsigned)ceil_div(N, 128), (unsigned)ceil_div(M, 128));
    hipLaunchKernelGGL((k_gemm_mx_generic<false>), grid, dim3(256), 0, st, M, N, K, a_codes, a_scales, b_codes,
                       b_scales, C, ldc, Ag, Bg, kpad);
    return check_launch();
}

int launch_oe_k_accumulate(int64_t M, int64_t N, const uint16_t *Ag, const uint16_t *Bg, int kpad, float *C,
                           int64_t ldc, hipStream_t st)
{
    if (M == 0 || N == 0 || kpad == 0) return ADAHOP_OK;
    dim3 grid((unsigned)ceil_div(N, 128), (unsigned)ceil_div(M, 128));
    hipLaunchKernelGGL((k_gemm_mx_generic<true>), grid, dim3(256), 0, st, M, N, (int64_t)0, nullptr, nullptr, nullptr,
                       nullptr, C, ldc, Ag, Bg, kpad);
    return check_launch();
}

} // namespace adahop
