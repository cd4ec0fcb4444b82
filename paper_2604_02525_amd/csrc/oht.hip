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
// grid (ceil(N / OHT_TN), M / B).  M % B == 0, N % B == 0.  Any alignment of C and any ldc: the kernel for rows that
// are not 16-byte aligned; aligned rows take k_oht_inverse_reg below.
template <int B>
__global__ __launch_bounds__(256) void k_oht_inverse(float *__restrict__ C, int64_t M, int64_t N, int64_t ldc)
{
    extern __shared__ float tile[]; // [B][OHT_NP]
    const int tid = threadIdx.x;
    const int64_t n0 = (int64_t)blockIdx.x * OHT_TN, m0 = (int64_t)blockIdx.y * B;
    for (int idx = tid; idx < B * OHT_TN; idx += 256) {
        const int r = idx / OHT_TN, c = idx % OHT_TN;
        if (n0 + c < N) tile[r * OHT_NP + c] = C[(m0 + r) * ldc + n0 + c];
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

// The value of lane (own lane ^ M) for M = 1, 2, 4, 8 (inside a row of 16 lanes: DPP) and 16 (between neighbouring
// rows: the row swap of this chip), combined with the own value into the butterfly of stride M over lanes:
// x + y on the lane with bit M clear, x - y (x the lower lane's value) on the lane with bit M set.  `sign` is +1 on
// the lower lane and -1 on the upper one: sign * own + partner is that sum or difference with a single rounding.
template <int M> __device__ __forceinline__ float lane_butterfly(float own, float sign)
{
    const int x = (int)__float_as_uint(own);
    if constexpr (M == 16) {
        typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
        // .x: the even row's value in both rows of a pair, .y: the odd row's
        const u32x2 r = __builtin_amdgcn_permlane16_swap((unsigned)x, (unsigned)x, false, false);
        return __builtin_fmaf(sign, __uint_as_float(r.y), __uint_as_float(r.x));
    } else {
        int p;
        if constexpr (M == 1) p = __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xf, 0xf, true);      // quad_perm [1,0,3,2]
        else if constexpr (M == 2) p = __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xf, 0xf, true); // quad_perm [2,3,0,1]
        else if constexpr (M == 4) {
            p = __builtin_amdgcn_update_dpp(0, x, 0x104, 0xf, 0x5, false); // lanes 0-3, 8-11 of a row: from lane + 4
            p = __builtin_amdgcn_update_dpp(p, x, 0x114, 0xf, 0xa, false); // lanes 4-7, 12-15: from lane - 4
        } else {
            p = __builtin_amdgcn_update_dpp(0, x, 0x108, 0xf, 0x3, false); // lanes 0-7: from lane + 8
            p = __builtin_amdgcn_update_dpp(p, x, 0x118, 0xf, 0xc, false); // lanes 8-15: from lane - 8
        }
        return __builtin_fmaf(sign, own, __uint_as_float((uint32_t)p));
    }
}

template <int M, int B> __device__ __forceinline__ void lane_step(float4 &v, int lane)
{
    if constexpr (4 * M < B) { // the stride 4 M (in floats) lies inside a block of B
        const float sign = (lane & M) ? -1.0f : 1.0f;
        v.x = lane_butterfly<M>(v.x, sign);
        v.y = lane_butterfly<M>(v.y, sign);
        v.z = lane_butterfly<M>(v.z, sign);
        v.w = lane_butterfly<M>(v.w, sign);
    }
}

// The same rotation with the butterflies in registers (C 16-byte aligned, ldc % 4 == 0).  A lane holds four
// consecutive columns of B / 8 rows (row = 8 it + 2 wave + lane / 32): the right-hand transform of a row's block of B
// columns runs inside the float4 (strides 1, 2) and over the B / 4 neighbouring lanes (strides 4 .. B / 2).  The tile
// then goes through LDS once, and comes back with a lane holding B / 2 rows of one column (column = 32 wave +
// lane % 32, rows from (B / 2) (lane / 32)): strides 1 .. B / 4 of the left-hand transform are in registers, the last
// one is between the two halves of the wave.  Every value sees the strides in ascending order with x + y to the lower
// and x - y to the upper index and one multiply by 1/sqrt(B) per transform: the result is that of k_oht_inverse,
// bit for bit.  On 16384 x 28672 with block 128 it takes 0.73 ms (5.1 TB/s read + written) against 1.13 ms with both
// transforms through LDS (five barriers and 512 KB of LDS traffic per tile instead of one and 128 KB); a persistent
// variant of the LDS kernel that kept the next tile on its way in registers had brought 4 % for block 128 and lost
// 15 % for block 32.
template <int B>
__global__ __launch_bounds__(256) void k_oht_inverse_reg(float *__restrict__ C, int64_t M, int64_t N, int64_t ldc)
{
    extern __shared__ float tile[]; // [B][OHT_NP]
    constexpr int ROWS = B / 8, CH = B / 2;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, half = lane >> 5, c4 = lane & 31;
    const int64_t n0 = (int64_t)blockIdx.x * OHT_TN, m0 = (int64_t)blockIdx.y * B;
    const float c = oht_norm<B>();
    {
        const bool live = n0 + 4 * c4 < N; // N % B == 0: a block of B columns is inside or outside as a whole
        const float *src = C + (m0 + 2 * w + half) * ldc + n0 + 4 * c4;
        float4 v[ROWS];
#pragma unroll
        for (int it = 0; it < ROWS; ++it)
            v[it] = live ? *reinterpret_cast<const float4 *>(src + (int64_t)(8 * it) * ldc) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int it = 0; it < ROWS; ++it) {
            float4 q = v[it];
            const float a0 = q.x + q.y, a1 = q.x - q.y, a2 = q.z + q.w, a3 = q.z - q.w;
            q = make_float4(a0 + a2, a1 + a3, a0 - a2, a1 - a3);
            lane_step<1, B>(q, lane);
            lane_step<2, B>(q, lane);
            lane_step<4, B>(q, lane);
            lane_step<8, B>(q, lane);
            lane_step<16, B>(q, lane);
            float *t = tile + (8 * it + 2 * w + half) * OHT_NP + 4 * c4;
            t[0] = __builtin_fmaf(q.x, c, 0.0f); // "+ 0": an exact zero becomes +0
            t[1] = __builtin_fmaf(q.y, c, 0.0f);
            t[2] = __builtin_fmaf(q.z, c, 0.0f);
            t[3] = __builtin_fmaf(q.w, c, 0.0f);
        }
    }
    __syncthreads();
    {
        const int col = 32 * w + c4;
        const bool live = n0 + col < N;
        float u[CH];
        const float *t = tile + (CH * half) * OHT_NP + col;
#pragma unroll
        for (int i = 0; i < CH; ++i) u[i] = t[i * OHT_NP];
#pragma unroll
        for (int h = 1; h < CH; h *= 2)
#pragma unroll
            for (int i = 0; i < CH; i += 2 * h)
#pragma unroll
                for (int j = i; j < i + h; ++j) {
                    const float a = u[j], b = u[j + h];
                    u[j] = a + b;
                    u[j + h] = a - b;
                }
        typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
        const float sign = half ? -1.0f : 1.0f;
        float *dst = C + (m0 + CH * half) * ldc + n0 + col;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            // .x: the lower half's value in both halves of the wave, .y: the upper half's
            const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(u[i]), __float_as_uint(u[i]), false, false);
            const float y = __builtin_fmaf(sign, __uint_as_float(r.y), __uint_as_float(r.x));
            if (live) dst[(int64_t)i * ldc] = __builtin_fmaf(y, c, 0.0f);
        }
    }
}

template <int B> constexpr size_t oht_quant_lds() { return (size_t)B * OHT_KP * sizeof(float); }
template <int B> constexpr size_t oht_inverse_lds() { return (size_t)B * OHT_NP * sizeof(float); }

template <int B> int allow_oht_lds()
{
    int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_oht_quant<B>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)oht_quant_lds<B>()));
    if (rc != ADAHOP_OK) return rc;
    rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_oht_inverse_reg<B>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)oht_inverse_lds<B>()));
    if (rc != ADAHOP_OK) return rc;
    return check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_oht_inverse<B>),
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

template <int B> int launch_inverse(float *C, int64_t M, int64_t N, int64_t ldc, hipStream_t st)
{
    const int rc = configure_oht();
    if (rc != ADAHOP_OK) return rc;
    const dim3 grid((unsigned)ceil_div(N, OHT_TN), (unsigned)(M / B));
    if (aligned(C, 16) && ldc % 4 == 0)
        hipLaunchKernelGGL(k_oht_inverse_reg<B>, grid, dim3(256), oht_inverse_lds<B>(), st, C, M, N, ldc);
    else
        hipLaunchKernelGGL(k_oht_inverse<B>, grid, dim3(256), oht_inverse_lds<B>(), st, C, M, N, ldc);
    return check_launch();
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
