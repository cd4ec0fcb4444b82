// Outer Hadamard Transform, the comparison strategy of paper Eq. 6 (gfx950):
//
//     C_OHT = H_m^T ( Q(H_m A) * Q(B H_n) ) H_n^T
//
// with block-diagonal normalised Sylvester matrices of size B on both outer dimensions.  Two kernels:
//   k_oht_quant    one operand, logical [outer, K]: every block of B consecutive OUTER indices is
//                  transformed (for every K index), then every 32 consecutive K-elements of a row are
//                  quantised to MXFP4.  H_m A for A; (B H_n)^T = H_n B^T for B given as [N, K].
//   k_oht_inverse  C <- H^T C H^T in place, fp32: the rotations after the product.
// The paper's point about this strategy -- transforms along the outer dimensions plus inverse rotations
// of the whole output cost extra data movement -- is what these kernels let one measure.
//
// Numerics as for the inner transform: fp32 butterflies in ascending stride order (x + y to the lower
// index, x - y to the upper), one fp32 multiply by (float)(1/sqrt(B)), an exactly zero result stored as
// +0; then amax, E8M0 scale = biased exponent of amax minus 2, E2M1 round-to-nearest-even, saturating.
#include "common.h"

namespace adahop {

namespace {

// Tiles are kept small in the direction that is not transformed: several workgroups then share a compute unit and
// one's loads and stores overlap another's butterflies (a workgroup runs its phases one after the other).
constexpr int OHT_TK = 64;             // K-columns of an operand tile
constexpr int OHT_TN = 128;            // columns of a C tile (>= the largest block: a row's blocks lie inside a tile)
constexpr int OHT_KP = OHT_TK + 1;     // LDS pitches (floats): odd, so that column walks hit distinct banks
constexpr int OHT_NP = OHT_TN + 1;

template <int B> __device__ __forceinline__ float oht_norm();
template <> __device__ __forceinline__ float oht_norm<32>() { return 0x1.6a09e6p-3f; }
template <> __device__ __forceinline__ float oht_norm<64>() { return 0.125f; }
template <> __device__ __forceinline__ float oht_norm<128>() { return 0x1.6a09e6p-4f; }

// v <- (1/sqrt(B)) H_B v on B values spaced `stride` floats apart in LDS, the work of one vector shared by P
// threads (part = 0 .. P-1) in two passes with a workgroup barrier between them: first every thread runs the
// strides 1 .. B/(2P) on its own chunk of B/P consecutive values, then the strides B/P .. B/2 on the values of equal
// position in the P chunks.  Every value still sees the strides in ascending order with x + y to the lower and
// x - y to the upper index, so the result is that of the plain butterfly network, bit for bit.  All threads of the
// workgroup must call it (live = false: no memory access, barrier only).
// gout != nullptr: the results go to gout[index * gstride] (global memory) instead of back into LDS.
template <int B, int P>
__device__ __forceinline__ void fwht_lds_split(float *p, int stride, int part, bool live, float *gout = nullptr,
                                               int64_t gstride = 0)
{
    constexpr int CH = B / P, G = CH / P;
    if (live) {
        float v[CH];
        float *q = p + part * CH * stride;
#pragma unroll
        for (int i = 0; i < CH; ++i) v[i] = q[i * stride];
#pragma unroll
        for (int h = 1; h < CH; h *= 2)
#pragma unroll
            for (int i = 0; i < CH; i += 2 * h)
#pragma unroll
                for (int j = i; j < i + h; ++j) {
                    const float a = v[j], b = v[j + h];
                    v[j] = a + b;
                    v[j + h] = a - b;
                }
#pragma unroll
        for (int i = 0; i < CH; ++i) q[i * stride] = v[i];
    }
    __syncthreads();
    if (live) {
        const float c = oht_norm<B>();
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float *q = p + (part * G + g) * stride;
            float u[P];
#pragma unroll
            for (int j = 0; j < P; ++j) u[j] = q[j * CH * stride];
#pragma unroll
            for (int h = 1; h < P; h *= 2)
#pragma unroll
                for (int i = 0; i < P; i += 2 * h)
#pragma unroll
                    for (int j = i; j < i + h; ++j) {
                        const float a = u[j], b = u[j + h];
                        u[j] = a + b;
                        u[j + h] = a - b;
                    }
#pragma unroll
            for (int j = 0; j < P; ++j) {
                const float r = __builtin_fmaf(u[j], c, 0.0f); // "+ 0": an exact zero becomes +0
                if (gout)
                    gout[(int64_t)(j * CH + part * G + g) * gstride] = r;
                else
                    q[j * CH * stride] = r;
            }
        }
    }
}

__device__ __forceinline__ int e8m0_code(float amax)
{
    const int s = (int)((__float_as_uint(amax) >> 23) & 0xffu) - 2;
    return s < 0 ? 0 : s;
}

// Workgroup = B outer rows x OHT_TK K-columns.  grid (ceil(K / OHT_TK), outer / B).
template <int B>
__global__ __launch_bounds__(256) void k_oht_quant(const uint16_t *__restrict__ x, int64_t outer, int64_t K, int64_t ld,
                                                   int k_contig, uint8_t *__restrict__ codes,
                                                   uint8_t *__restrict__ scales)
{
    extern __shared__ float tile[]; // [B][OHT_KP]
    const int tid = threadIdx.x;
    const int64_t k0 = (int64_t)blockIdx.x * OHT_TK, o0 = (int64_t)blockIdx.y * B;

    // 1. load, 16 bytes per lane along whichever axis is contiguous in memory
    if (k_contig) {
        for (int idx = tid; idx < B * (OHT_TK / 8); idx += 256) {
            const int r = idx / (OHT_TK / 8), c8 = idx % (OHT_TK / 8);
            const int64_t kk = k0 + c8 * 8;
            if (kk < K) { // K % 32 == 0: a chunk of 8 is inside or outside as a whole
                const uint4 q = load_once16(x + (o0 + r) * ld + kk);
                float *t = tile + r * OHT_KP + c8 * 8;
                t[0] = bf16_lo(q.x), t[1] = bf16_hi(q.x), t[2] = bf16_lo(q.y), t[3] = bf16_hi(q.y);
                t[4] = bf16_lo(q.z), t[5] = bf16_hi(q.z), t[6] = bf16_lo(q.w), t[7] = bf16_hi(q.w);
            }
        }
    } else {
        for (int idx = tid; idx < OHT_TK * (B / 8); idx += 256) {
            const int c = idx / (B / 8), r8 = idx % (B / 8);
            const int64_t kk = k0 + c;
            if (kk < K) {
                const uint4 q = load_once16(x + kk * ld + o0 + r8 * 8);
                float *t = tile + (r8 * 8) * OHT_KP + c;
                t[0 * OHT_KP] = bf16_lo(q.x), t[1 * OHT_KP] = bf16_hi(q.x), t[2 * OHT_KP] = bf16_lo(q.y);
                t[3 * OHT_KP] = bf16_hi(q.y), t[4 * OHT_KP] = bf16_lo(q.z), t[5 * OHT_KP] = bf16_hi(q.z);
                t[6 * OHT_KP] = bf16_lo(q.w), t[7 * OHT_KP] = bf16_hi(q.w);
            }
        }
    }
    __syncthreads();
    // 2. transform along the outer index: four threads (one of each wave) per K-column
    fwht_lds_split<B, 256 / OHT_TK>(tile + tid % OHT_TK, OHT_KP, tid / OHT_TK, k0 + tid % OHT_TK < K);
    __syncthreads();
    // 3. quantise along K: one lane per 16 consecutive K-elements of a row, two lanes per MX block
    for (int idx = tid; idx < B * (OHT_TK / 16); idx += 256) {
        const int r = idx / (OHT_TK / 16), ch = idx % (OHT_TK / 16);
        const int64_t kk = k0 + ch * 16;
        const bool live = kk < K; // both lanes of an MX block are live together (K % 32 == 0)
        float w[16];
        float m = 0.0f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            w[i] = live ? tile[r * OHT_KP + ch * 16 + i] : 0.0f;
            m = fmaxf(m, fabsf(w[i]));
        }
        m = fmaxf(m, __shfl_xor(m, 1));
        if (live) {
            const int s = e8m0_code(m);
            const float X = __uint_as_float((uint32_t)s << 23);
            uint32_t c0 = 0, c1 = 0;
            c0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c0, w[0], w[1], X, 0);
            c0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c0, w[2], w[3], X, 1);
            c0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c0, w[4], w[5], X, 2);
            c0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c0, w[6], w[7], X, 3);
            c1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c1, w[8], w[9], X, 0);
            c1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c1, w[10], w[11], X, 1);
            c1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c1, w[12], w[13], X, 2);
            c1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c1, w[14], w[15], X, 3);
            *reinterpret_cast<uint2 *>(codes + (o0 + r) * (K >> 1) + (kk >> 1)) = make_uint2(c0, c1);
            if ((ch & 1) == 0) scales[(o0 + r) * (K >> 5) + (kk >> 5)] = (uint8_t)s;
        }
    }
}

// Workgroup = B rows x OHT_TN columns of C (OHT_TN / B blocks side by side), transformed along both axes in LDS.
// grid (ceil(N / OHT_TN), M / B).  M % B == 0, N % B == 0.
// VEC: C is 16-byte aligned with ldc % 4 == 0, rows are read as float4 (N % B == 0 makes every float4 whole).
// (A persistent variant that keeps the next tile on its way in registers while the butterflies run was measured:
// 1.08 against 1.12 ms for block 128 and 0.78 against 0.68 ms for block 32 on 16384 x 28672 -- the registers it
// needs cost the occupancy that hides the same latency here.)
template <int B, bool VEC>
__global__ __launch_bounds__(256) void k_oht_inverse(float *__restrict__ C, int64_t M, int64_t N, int64_t ldc)
{
    extern __shared__ float tile[]; // [B][OHT_NP]
    const int tid = threadIdx.x;
    const int64_t n0 = (int64_t)blockIdx.x * OHT_TN, m0 = (int64_t)blockIdx.y * B;
    if constexpr (VEC) {
#pragma unroll 4
        for (int idx = tid; idx < B * (OHT_TN / 4); idx += 256) {
            const int r = idx / (OHT_TN / 4), c4 = idx % (OHT_TN / 4);
            if (n0 + 4 * c4 < N) {
                const float4 q = *reinterpret_cast<const float4 *>(C + (m0 + r) * ldc + n0 + 4 * c4);
                float *t = tile + r * OHT_NP + 4 * c4;
                t[0] = q.x, t[1] = q.y, t[2] = q.z, t[3] = q.w;
            }
        }
    } else {
        for (int idx = tid; idx < B * OHT_TN; idx += 256) {
            const int r = idx / OHT_TN, c = idx % OHT_TN;
            if (n0 + c < N) tile[r * OHT_NP + c] = C[(m0 + r) * ldc + n0 + c];
        }
    }
    __syncthreads();
    {   // H^T from the right: two threads per (row, B-wide column block); there are B * (OHT_TN / B) such pairs
        const int u = tid % OHT_TN, r = u % B, seg = u / B;
        fwht_lds_split<B, 256 / OHT_TN>(tile + r * OHT_NP + seg * B, 1, tid / OHT_TN, n0 + seg * B < N);
    }
    __syncthreads();
    // H^T from the left: along the rows of every column, two threads per column; the results leave for memory from
    // the registers (a wave writes 256 consecutive bytes of a row)
    fwht_lds_split<B, 256 / OHT_TN>(tile + tid % OHT_TN, OHT_NP, tid / OHT_TN, n0 + tid % OHT_TN < N,
                                    C + m0 * ldc + n0 + tid % OHT_TN, ldc);
}

template <int B> constexpr size_t oht_quant_lds() { return (size_t)B * OHT_KP * sizeof(float); }
template <int B> constexpr size_t oht_inverse_lds() { return (size_t)B * OHT_NP * sizeof(float); }

template <int B> int allow_oht_lds()
{
    int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_oht_quant<B>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)oht_quant_lds<B>()));
    if (rc != ADAHOP_OK) return rc;
    rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_oht_inverse<B, true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)oht_inverse_lds<B>()));
    if (rc != ADAHOP_OK) return rc;
    return check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_oht_inverse<B, false>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)oht_inverse_lds<B>()));
}

template <int B> int launch_quant(const adahop_operand_t &x, uint8_t *codes, uint8_t *scales, hipStream_t st)
{
    const int rc = configure_oht(); // more LDS than a launch may ask for by default (B = 128): allowed once per device
    if (rc != ADAHOP_OK) return rc;
    const dim3 grid((unsigned)ceil_div(x.K, OHT_TK), (unsigned)(x.outer / B));
    hipLaunchKernelGGL(k_oht_quant<B>, grid, dim3(256), oht_quant_lds<B>(), st, static_cast<const uint16_t *>(x.data), x.outer,
                       x.K, x.ld, x.k_contig, codes, scales);
    return check_launch();
}

template <int B, bool VEC> int launch_inverse_as(float *C, int64_t M, int64_t N, int64_t ldc, hipStream_t st)
{
    const int rc = configure_oht();
    if (rc != ADAHOP_OK) return rc;
    const dim3 grid((unsigned)ceil_div(N, OHT_TN), (unsigned)(M / B));
    hipLaunchKernelGGL((k_oht_inverse<B, VEC>), grid, dim3(256), oht_inverse_lds<B>(), st, C, M, N, ldc);
    return check_launch();
}

template <int B> int launch_inverse(float *C, int64_t M, int64_t N, int64_t ldc, hipStream_t st)
{
    return aligned(C, 16) && ldc % 4 == 0 ? launch_inverse_as<B, true>(C, M, N, ldc, st)
                                          : launch_inverse_as<B, false>(C, M, N, ldc, st);
}

} // namespace

// Every OHT kernel instance, once per device (host-side calls, nothing queued).
int configure_oht()
{
    static device_once_t once;
    int dev = 0;
    int rc = check_hip(hipGetDevice(&dev));
    if (rc != ADAHOP_OK || !once.need(dev)) return rc;
    if ((rc = allow_oht_lds<32>()) != ADAHOP_OK || (rc = allow_oht_lds<64>()) != ADAHOP_OK ||
        (rc = allow_oht_lds<128>()) != ADAHOP_OK)
        return rc;
    once.mark(dev);
    return ADAHOP_OK;
}

bool valid_oht_block(int b) { return b == 32 || b == 64 || b == 128; }

// x.outer % b == 0 and valid_oht_block(b) are the caller's to check.
int launch_oht_quantize(const adahop_operand_t &x, int b, uint8_t *codes, uint8_t *scales, hipStream_t st)
{
    switch (b) {
    case 32: return launch_quant<32>(x, codes, scales, st);
    case 64: return launch_quant<64>(x, codes, scales, st);
    default: return launch_quant<128>(x, codes, scales, st);
    }
}

int launch_oht_inverse(float *C, int64_t M, int64_t N, int64_t ldc, int b, hipStream_t st)
{
    if (M == 0 || N == 0) return ADAHOP_OK;
    switch (b) {
    case 32: return launch_inverse<32>(C, M, N, ldc, st);
    case 64: return launch_inverse<64>(C, M, N, ldc, st);
    default: return launch_inverse<128>(C, M, N, ldc, st);
    }
}

} // namespace adahop
