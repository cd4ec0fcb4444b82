// Fused residual masking -> block Hadamard transform -> OCP-MX FP4 quantisation (gfx950).
//
// What is computed (paper Eq. 5 applied to one operand, App. F items 1-2): for every row of the
// logical [outer, K] operand, entries flagged by the masks become 0, every block of B consecutive
// K-elements is multiplied by the normalised Sylvester Hadamard matrix, and every 32 consecutive
// K-elements are quantised to E2M1 with one shared E8M0 scale.
//
// Numerics are fixed so that the packed bytes are reproducible: fp32 butterflies in ascending
// stride order (x+y to the lower index, x-y to the upper), one fp32 multiply by (float)(1/sqrt(B)),
// amax on those fp32 values, scale = biased exponent of amax minus 2, round-to-nearest-even to E2M1
// with saturation at 6.  The file is compiled with -ffp-contract=off.
//
// Two kernels, one per storage order of the operand:
//   k_quant_kc  K contiguous: a lane owns 8 consecutive K-elements (one 16-byte load); strides
//               1,2,4 are register butterflies, strides 8..B/2 exchange lanes (DPP / swizzle).
//               Reads and writes are fully coalesced.  HBM-bound: 2 + 1/2 + 1/32 bytes / element.
//   k_quant_ks  K strided (outer contiguous): a lane owns two neighbouring columns and one MX block
//               (32 K-elements) of each, so strides 1..16 are register butterflies with no lane
//               traffic; strides 32..B/2 pair whole MX blocks held by different waves of the
//               workgroup and go through LDS.  Loads are coalesced along `outer`.
#include "common.h"

namespace adahop {

namespace {

__device__ __forceinline__ int e8m0_of_amax(float amax)
{
    int e = (int)((__float_as_uint(amax) >> 23) & 0xffu);
    int s = e - 2;
    return s < 0 ? 0 : s; // zero and subnormal amax -> 0
}

// E2M1 code of v / 2^(s-127): sign in bit 3, magnitude index 0..7, RNE, saturating.
__device__ __forceinline__ uint32_t e2m1_code(float v, int s)
{
    float q = ldexpf(v, 127 - s);
    float a = fabsf(q);
    uint32_t m = (uint32_t)(a > 0.25f) + (uint32_t)(a >= 0.75f) + (uint32_t)(a > 1.25f) + (uint32_t)(a >= 1.75f) +
                 (uint32_t)(a > 2.5f) + (uint32_t)(a >= 3.5f) + (uint32_t)(a > 5.0f);
    return m | ((__float_as_uint(v) >> 28) & 8u);
}

template <int B> __device__ __forceinline__ float hadamard_norm();
template <> __device__ __forceinline__ float hadamard_norm<32>() { return 0x1.6a09e6p-3f; }
template <> __device__ __forceinline__ float hadamard_norm<64>() { return 0.125f; }
template <> __device__ __forceinline__ float hadamard_norm<128>() { return 0x1.6a09e6p-4f; }
template <> __device__ __forceinline__ float hadamard_norm<256>() { return 0.0625f; }

// Value held by lane (lane ^ XM); XM in {1, 2, 4, 8, 16}.
template <int XM> __device__ __forceinline__ float lane_xor(float v)
{
    int i = __float_as_int(v);
    if constexpr (XM == 1)
        i = __builtin_amdgcn_mov_dpp(i, 0xB1, 0xf, 0xf, true); // quad_perm [1,0,3,2]
    else if constexpr (XM == 2)
        i = __builtin_amdgcn_mov_dpp(i, 0x4E, 0xf, 0xf, true); // quad_perm [2,3,0,1]
    else
        i = __builtin_amdgcn_ds_swizzle(i, (XM << 10) | 0x1f); // bit mode: and 0x1f, or 0, xor XM
    return __int_as_float(i);
}

template <int XM, int B> __device__ __forceinline__ void lane_stage(float (&v)[8], int lane)
{
    if constexpr (8 * XM < B) {
        const bool upper = (lane & XM) != 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float p = lane_xor<XM>(v[i]);
            v[i] = upper ? p - v[i] : v[i] + p;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// K-contiguous operand.  One lane = 8 consecutive K-elements; 4 lanes = one MX block; B/8 lanes =
// one transform block.  FLAT = 0: blockIdx.x is the row, blockIdx.y*256+tid the 8-element chunk.
// FLAT = 1 (short rows): chunks of all rows are numbered consecutively.
// ------------------------------------------------------------------------------------------------
template <int B, int FLAT>
__global__ __launch_bounds__(256) void k_quant_kc(const uint16_t *__restrict__ x, int64_t outer, int64_t K,
                                                  int64_t ld, const uint8_t *__restrict__ zero_outer,
                                                  const uint8_t *__restrict__ zero_k,
                                                  uint8_t *__restrict__ codes, uint8_t *__restrict__ scales)
{
    const uint32_t cpr = (uint32_t)(K >> 3);
    int64_t row;
    uint32_t chunk;
    bool active;
    if constexpr (FLAT) {
        const uint32_t c = blockIdx.x * 256u + threadIdx.x;
        const uint32_t r = c / cpr;
        row = r;
        chunk = c - r * cpr;
        active = row < outer;
    } else {
        row = blockIdx.x;
        chunk = blockIdx.y * 256u + threadIdx.x;
        active = chunk < cpr;
    }
    const int lane = threadIdx.x & 63;
    const int64_t kk = (int64_t)chunk * 8;

    uint4 raw = make_uint4(0, 0, 0, 0);
    if (active) {
        raw = *reinterpret_cast<const uint4 *>(x + row * ld + kk);
        if (zero_outer && zero_outer[row]) raw = make_uint4(0, 0, 0, 0);
    }
    float v[8] = {bf16_lo(raw.x), bf16_hi(raw.x), bf16_lo(raw.y), bf16_hi(raw.y),
                  bf16_lo(raw.z), bf16_hi(raw.z), bf16_lo(raw.w), bf16_hi(raw.w)};
    if (zero_k && active) {
        const uint64_t zm = *reinterpret_cast<const uint64_t *>(zero_k + kk);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if ((zm >> (8 * i)) & 0xffu) v[i] = 0.0f;
    }

    if constexpr (B > 0) {
#pragma unroll
        for (int h = 1; h < 8; h *= 2)
#pragma unroll
            for (int i = 0; i < 8; i += 2 * h)
#pragma unroll
                for (int j = i; j < i + h; ++j) {
                    float a = v[j], b = v[j + h];
                    v[j] = a + b;
                    v[j + h] = a - b;
                }
        lane_stage<1, B>(v, lane);
        lane_stage<2, B>(v, lane);
        lane_stage<4, B>(v, lane);
        lane_stage<8, B>(v, lane);
        lane_stage<16, B>(v, lane);
        const float c = hadamard_norm<B>();
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = v[i] * c;
    }

    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(v[i]));
    amax = fmaxf(amax, lane_xor<1>(amax));
    amax = fmaxf(amax, lane_xor<2>(amax));
    const int s = e8m0_of_amax(amax);

    uint32_t packed = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) packed |= e2m1_code(v[i], s) << (4 * i);

    if (active) {
        *reinterpret_cast<uint32_t *>(codes + row * (K >> 1) + (kk >> 1)) = packed;
        if ((lane & 3) == 0) scales[row * (K >> 5) + (kk >> 5)] = (uint8_t)s;
    }
}

// ------------------------------------------------------------------------------------------------
// K-strided operand: element (o, kk) at x[kk*ld + o].  Workgroup = NW waves; wave w owns MX block
// (blockIdx.y*NW + w) of 128 columns (two per lane).
// ------------------------------------------------------------------------------------------------
template <int B> struct ks_cfg {
    static constexpr int NCH = (B <= 32) ? 1 : B / 32; // MX blocks per transform block
    static constexpr int NW = (NCH > 4) ? NCH : 4;     // waves per workgroup
};

template <int B>
__global__ __launch_bounds__(ks_cfg<B>::NW * 64) void k_quant_ks(const uint16_t *__restrict__ x, int64_t outer,
                                                                  int64_t K, int64_t ld,
                                                                  const uint8_t *__restrict__ zero_outer,
                                                                  const uint8_t *__restrict__ zero_k,
                                                                  uint8_t *__restrict__ codes,
                                                                  uint8_t *__restrict__ scales)
{
    constexpr int NCH = ks_cfg<B>::NCH;
    constexpr int NW = ks_cfg<B>::NW;
    extern __shared__ float2 xchg[]; // [NW][32][64], only touched when NCH > 1

    const int w = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63;
    const int64_t o = ((int64_t)blockIdx.x * 64 + lane) * 2;
    const int64_t blk = (int64_t)blockIdx.y * NW + w;
    const bool valid = (blk < (K >> 5)) && (o < outer);
    const bool valid1 = valid && (o + 1 < outer);

    float2 v[32];
    {
        bool z0 = false, z1 = false;
        if (zero_outer && valid) {
            z0 = zero_outer[o] != 0;
            z1 = valid1 ? (zero_outer[o + 1] != 0) : true;
        }
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            uint32_t pair = 0;
            if (valid) {
                const int64_t kk = blk * 32 + i;
                pair = *reinterpret_cast<const uint32_t *>(x + kk * ld + o);
                if (zero_k && zero_k[kk]) pair = 0;
            }
            v[i].x = z0 ? 0.0f : bf16_lo(pair);
            v[i].y = (z1 || !valid1) ? 0.0f : bf16_hi(pair);
        }
    }

    if constexpr (B > 0) {
#pragma unroll
        for (int h = 1; h < 32; h *= 2)
#pragma unroll
            for (int i = 0; i < 32; i += 2 * h)
#pragma unroll
                for (int j = i; j < i + h; ++j) {
                    float2 a = v[j], b = v[j + h];
                    v[j].x = a.x + b.x;
                    v[j].y = a.y + b.y;
                    v[j + h].x = a.x - b.x;
                    v[j + h].y = a.y - b.y;
                }
        if constexpr (NCH > 1) {
            const int c = w % NCH; // index of this MX block inside its transform block
#pragma unroll
            for (int d = 1; d < NCH; d *= 2) {
#pragma unroll
                for (int i = 0; i < 32; ++i) xchg[(w * 32 + i) * 64 + lane] = v[i];
                __syncthreads();
                const int pw = w ^ d;
                const bool upper = (c & d) != 0;
#pragma unroll
                for (int i = 0; i < 32; ++i) {
                    const float2 p = xchg[(pw * 32 + i) * 64 + lane];
                    v[i].x = upper ? p.x - v[i].x : v[i].x + p.x;
                    v[i].y = upper ? p.y - v[i].y : v[i].y + p.y;
                }
                __syncthreads();
            }
        }
        const float cn = hadamard_norm<(B >= 32 ? B : 32)>();
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            v[i].x = v[i].x * cn;
            v[i].y = v[i].y * cn;
        }
    }

    float ax = 0.0f, ay = 0.0f;
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        ax = fmaxf(ax, fabsf(v[i].x));
        ay = fmaxf(ay, fabsf(v[i].y));
    }
    const int sx = e8m0_of_amax(ax), sy = e8m0_of_amax(ay);
    uint32_t px[4] = {0, 0, 0, 0}, py[4] = {0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        px[i >> 3] |= e2m1_code(v[i].x, sx) << (4 * (i & 7));
        py[i >> 3] |= e2m1_code(v[i].y, sy) << (4 * (i & 7));
    }
    if (valid) {
        *reinterpret_cast<uint4 *>(codes + o * (K >> 1) + blk * 16) = make_uint4(px[0], px[1], px[2], px[3]);
        scales[o * (K >> 5) + blk] = (uint8_t)sx;
    }
    if (valid1) {
        *reinterpret_cast<uint4 *>(codes + (o + 1) * (K >> 1) + blk * 16) = make_uint4(py[0], py[1], py[2], py[3]);
        scales[(o + 1) * (K >> 5) + blk] = (uint8_t)sy;
    }
}

template <int B>
int launch_kc(const adahop_operand_t &x, const uint8_t *zo, const uint8_t *zk, uint8_t *codes, uint8_t *scales,
              hipStream_t st)
{
    const uint16_t *d = static_cast<const uint16_t *>(x.data);
    const int64_t cpr = x.K / 8;
    if (cpr >= 128) {
        dim3 grid((unsigned)x.outer, (unsigned)ceil_div(cpr, 256));
        hipLaunchKernelGGL((k_quant_kc<B, 0>), grid, dim3(256), 0, st, d, x.outer, x.K, x.ld, zo, zk, codes, scales);
    } else {
        dim3 grid((unsigned)ceil_div(x.outer * cpr, 256));
        hipLaunchKernelGGL((k_quant_kc<B, 1>), grid, dim3(256), 0, st, d, x.outer, x.K, x.ld, zo, zk, codes, scales);
    }
    return check_launch();
}

template <int B>
int launch_ks(const adahop_operand_t &x, const uint8_t *zo, const uint8_t *zk, uint8_t *codes, uint8_t *scales,
              hipStream_t st)
{
    constexpr int NW = ks_cfg<B>::NW;
    constexpr int NCH = ks_cfg<B>::NCH;
    const size_t lds = NCH > 1 ? (size_t)NW * 32 * 64 * sizeof(float2) : 0;
    if (lds > 48 * 1024) {
        int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_quant_ks<B>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        if (rc != ADAHOP_OK) return rc;
    }
    dim3 grid((unsigned)ceil_div(x.outer, 128), (unsigned)ceil_div(x.K / 32, NW));
    hipLaunchKernelGGL((k_quant_ks<B>), grid, dim3(NW * 64), lds, st, static_cast<const uint16_t *>(x.data),
                       x.outer, x.K, x.ld, zo, zk, codes, scales);
    return check_launch();
}

} // namespace

int launch_iht_quantize(const adahop_operand_t &x, int b, const uint8_t *zo, const uint8_t *zk, uint8_t *codes,
                        uint8_t *scales, hipStream_t st)
{
    if (x.outer == 0 || x.K == 0) return ADAHOP_OK;
#define ADAHOP_DISPATCH(BB)                                                              \
    case BB:                                                                             \
        return x.k_contig ? launch_kc<BB>(x, zo, zk, codes, scales, st)                  \
                          : launch_ks<BB>(x, zo, zk, codes, scales, st);
    switch (b) {
        ADAHOP_DISPATCH(0)
        ADAHOP_DISPATCH(32)
        ADAHOP_DISPATCH(64)
        ADAHOP_DISPATCH(128)
        ADAHOP_DISPATCH(256)
    default:
        return ADAHOP_E_INVALID_ARG;
    }
#undef ADAHOP_DISPATCH
}

} // namespace adahop
