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
// with saturation at 6; a transformed value that is exactly zero is stored as +0.  The file is
// compiled with -ffp-contract=off.
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

// ---- optional stochastic rounding of the elements (the paper cites it as prior work for unbiased
// gradient quantisation).  Random bits: Philox4x32 with 10 rounds (Salmon et al., SC'11), key = the two
// halves of the caller's seed, counter = (row, K index / 8, 0, 0): one block serves the 8 consecutive
// K-elements of a group, element j taking half j (word j / 2, low half for even j).
struct sr_key_t {
    uint32_t k0, k1;
};

__device__ __forceinline__ uint4 philox4x32_10(uint32_t c0, uint32_t c1, sr_key_t key)
{
    uint32_t c2 = 0, c3 = 0, k0 = key.k0, k1 = key.k1;
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return make_uint4(c0, c1, c2, c3);
}

// E2M1 code of v / 2^(s-127) rounded stochastically with the 16-bit draw r16: up to the next magnitude
// iff r16 / 65536 < (|q| - lo) / (hi - lo); |q| >= 6 saturates; sign as in e2m1_code.
__device__ __forceinline__ uint32_t e2m1_code_sr(float v, int s, uint32_t r16)
{
    const float a = fabsf(ldexpf(v, 127 - s));
    const uint32_t idx = (uint32_t)(a >= 0.5f) + (uint32_t)(a >= 1.0f) + (uint32_t)(a >= 1.5f) + (uint32_t)(a >= 2.0f) +
                         (uint32_t)(a >= 3.0f) + (uint32_t)(a >= 4.0f);
    const float lo = idx < 4 ? 0.5f * (float)idx : (float)(idx - 2);       // 0, .5, 1, 1.5, 2, 3, 4
    const float inv_step = idx < 4 ? 2.0f : (idx < 6 ? 1.0f : 0.5f);       // steps .5, 1, 2: exact scaling
    const float frac = (a - lo) * inv_step;
    const uint32_t up = (float)r16 * 0x1p-16f < frac ? 1u : 0u;
    const uint32_t m = a >= 6.0f ? 7u : idx + up;
    return m | ((__float_as_uint(v) >> 28) & 8u);
}

// Packed codes of 8 consecutive K-elements (first in the low nibble) starting at K index kk of row `row`.
__device__ __forceinline__ uint32_t pack8_sr(const float (&w)[8], int s, sr_key_t key, int64_t row, int64_t kk)
{
    const uint4 r = philox4x32_10((uint32_t)row, (uint32_t)(kk >> 3), key);
    const uint32_t word[4] = {r.x, r.y, r.z, r.w};
    uint32_t packed = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) packed |= e2m1_code_sr(w[i], s, (word[i >> 1] >> (16 * (i & 1))) & 0xffffu) << (4 * i);
    return packed;
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
template <int B, int FLAT, bool SR>
__global__ __launch_bounds__(256) void k_quant_kc(const uint16_t *__restrict__ x, int64_t outer, int64_t K,
                                                  int64_t ld, const uint8_t *__restrict__ zero_outer,
                                                  const uint8_t *__restrict__ zero_k,
                                                  uint8_t *__restrict__ codes, uint8_t *__restrict__ scales,
                                                  sr_key_t key)
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
        raw = load_once16(x + row * ld + kk);
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
        for (int i = 0; i < 8; ++i) v[i] = __builtin_fmaf(v[i], c, 0.0f); // exact zeros become +0
    }

    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(v[i]));
    amax = fmaxf(amax, lane_xor<1>(amax));
    amax = fmaxf(amax, lane_xor<2>(amax));
    const int s = e8m0_of_amax(amax);

    uint32_t packed = 0;
    if constexpr (SR) {
        packed = pack8_sr(v, s, key, row, kk);
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) packed |= e2m1_code(v[i], s) << (4 * i);
    }

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

template <int B, bool SR>
__global__ __launch_bounds__(ks_cfg<B>::NW * 64) void k_quant_ks(const uint16_t *__restrict__ x, int64_t outer,
                                                                  int64_t K, int64_t ld,
                                                                  const uint8_t *__restrict__ zero_outer,
                                                                  const uint8_t *__restrict__ zero_k,
                                                                  uint8_t *__restrict__ codes,
                                                                  uint8_t *__restrict__ scales, sr_key_t key)
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
                pair = load_once4(x + kk * ld + o);
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
            v[i].x = __builtin_fmaf(v[i].x, cn, 0.0f); // exact zeros become +0
            v[i].y = __builtin_fmaf(v[i].y, cn, 0.0f);
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
    if constexpr (SR) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            float wx[8], wy[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                wx[i] = v[8 * g + i].x;
                wy[i] = v[8 * g + i].y;
            }
            px[g] = pack8_sr(wx, sx, key, o, blk * 32 + 8 * g);
            py[g] = pack8_sr(wy, sy, key, o + 1, blk * 32 + 8 * g);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            px[i >> 3] |= e2m1_code(v[i].x, sx) << (4 * (i & 7));
            py[i >> 3] |= e2m1_code(v[i].y, sy) << (4 * (i & 7));
        }
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

// ================================================================================================
// Fast kernels for K % 256 == 0.  Both quantisers are bound by vector-ALU work long before HBM unless
// the per-element instruction count is kept near 12, so these kernels
//   - let the hardware convert: v_cvt_scalef32_pk_fp4_f32 rounds two fp32 values / 2^(s-127) to E2M1
//     (nearest even, saturating, first value in the low nibble) in one instruction;
//   - do every cross-lane butterfly as ONE fused multiply-add whose first operand comes through DPP:
//     w <- partner * t + w with t = +1 on the lower lane of the pair and -1 on the upper one.  That
//     yields L+U on the lower lane and -(L-U) on the upper lane; the stray sign is not fixed up but
//     tracked (it only depends on the lane) and folded into the final 1/sqrt(B) multiply.  Negation
//     commutes with rounding, so the stored bits are exactly those of the plain butterflies.
//
// Work split: 16 lanes (one DPP row) own 256 consecutive K-elements of one row; a lane holds two
// groups of 8 consecutive elements, 128 apart (chunk c of each half).  Strides 1, 2, 4 are register
// butterflies inside a group, strides 8..64 pair lanes, stride 128 pairs the lane's two groups.  A
// gfx9 DPP row offers the lane exchanges xor 1, xor 2 (quad_perm), xor 7 (row_half_mirror) and xor 8
// (row_ror:8) but not xor 4, so chunk c sits on lane (c0 ^ c2, c1 ^ c2, c2, c3): flipping chunk bit 2
// then is the xor-7 exchange.
// ================================================================================================
template <int CTRL> __device__ __forceinline__ float dpp_get(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

struct lane_plan_t {
    int chunk;     // which 8-element chunk (0..15) of each 128-element half this lane owns
    float t[4];    // multiplier of the partner value in cross-lane stage b
    float fin;     // sign left over from the stages times 1/sqrt(B)
};

template <int B> __device__ __forceinline__ lane_plan_t make_plan(int lane)
{
    constexpr int NS = B >= 128 ? 4 : (B == 64 ? 3 : (B == 32 ? 2 : 0));
    const int r = lane & 15, r2 = (r >> 2) & 1;
    lane_plan_t p;
    p.chunk = ((r ^ r2) & 1) | ((r ^ (r2 << 1)) & 2) | (r & 12);
    float sign = 1.0f;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const bool upper = b < NS && ((p.chunk >> b) & 1);
        p.t[b] = upper ? -1.0f : 1.0f;
        if (upper) sign = -sign;
    }
    if constexpr (B > 0)
        p.fin = sign * hadamard_norm<B>();
    else
        p.fin = 1.0f;
    return p;
}

// One cross-lane butterfly stage on all 16 values of the lane: w <- partner(w) * t + w, the partner
// being the lane of the DPP row whose chunk index differs in bit STAGE.  Written as assembly because
// the compiler does not fold the DPP move into the multiply-add (it emits a move, wait states and a
// separate v_fmac per value, doubling the cost of the stage).  The leading s_nop covers the two wait
// states a DPP read needs after a vector write of the same register; inside the block each
// instruction reads a register last written 16 instructions earlier.
#define ADAHOP_FMAC_DPP16(CTRL)                                                                        \
    asm volatile("s_nop 1\n\t"                                                                        \
                 "v_fmac_f32_dpp %0, %0, %16 " CTRL "\n\tv_fmac_f32_dpp %1, %1, %16 " CTRL "\n\t"     \
                 "v_fmac_f32_dpp %2, %2, %16 " CTRL "\n\tv_fmac_f32_dpp %3, %3, %16 " CTRL "\n\t"     \
                 "v_fmac_f32_dpp %4, %4, %16 " CTRL "\n\tv_fmac_f32_dpp %5, %5, %16 " CTRL "\n\t"     \
                 "v_fmac_f32_dpp %6, %6, %16 " CTRL "\n\tv_fmac_f32_dpp %7, %7, %16 " CTRL "\n\t"     \
                 "v_fmac_f32_dpp %8, %8, %16 " CTRL "\n\tv_fmac_f32_dpp %9, %9, %16 " CTRL "\n\t"     \
                 "v_fmac_f32_dpp %10, %10, %16 " CTRL "\n\tv_fmac_f32_dpp %11, %11, %16 " CTRL "\n\t" \
                 "v_fmac_f32_dpp %12, %12, %16 " CTRL "\n\tv_fmac_f32_dpp %13, %13, %16 " CTRL "\n\t" \
                 "v_fmac_f32_dpp %14, %14, %16 " CTRL "\n\tv_fmac_f32_dpp %15, %15, %16 " CTRL "\n\t" \
                 "s_nop 1"                                                                            \
                 : "+v"(w0[0]), "+v"(w0[1]), "+v"(w0[2]), "+v"(w0[3]), "+v"(w0[4]), "+v"(w0[5]), "+v"(w0[6]),   \
                   "+v"(w0[7]), "+v"(w1[0]), "+v"(w1[1]), "+v"(w1[2]), "+v"(w1[3]), "+v"(w1[4]), "+v"(w1[5]),   \
                   "+v"(w1[6]), "+v"(w1[7])                                                            \
                 : "v"(t))

template <int STAGE> __device__ __forceinline__ void cross_stage(float (&w0)[8], float (&w1)[8], float t)
{
    if constexpr (STAGE == 0)
        ADAHOP_FMAC_DPP16("quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf");
    else if constexpr (STAGE == 1)
        ADAHOP_FMAC_DPP16("quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf");
    else if constexpr (STAGE == 2)
        ADAHOP_FMAC_DPP16("row_half_mirror row_mask:0xf bank_mask:0xf");
    else
        ADAHOP_FMAC_DPP16("row_ror:8 row_mask:0xf bank_mask:0xf");
}

// Transform (B > 0) and quantise the lane's two groups; returns the packed codes of each group and
// the scale code of the MX block each group belongs to (identical on the 4 lanes of the block).
// SR: elements rounded stochastically; the groups start at K indices kk0 and kk1 of row `row`.
template <int B, bool SR>
__device__ __forceinline__ void transform_quantize16(float (&w0)[8], float (&w1)[8], const lane_plan_t &p,
                                                     uint32_t &codes0, uint32_t &codes1, int &s0, int &s1,
                                                     sr_key_t key, int64_t row, int64_t kk0, int64_t kk1)
{
    if constexpr (B > 0) {
#pragma unroll
        for (int h = 1; h < 8; h *= 2)
#pragma unroll
            for (int i = 0; i < 8; i += 2 * h)
#pragma unroll
                for (int j = i; j < i + h; ++j) {
                    float a = w0[j], b = w0[j + h];
                    w0[j] = a + b;
                    w0[j + h] = a - b;
                    a = w1[j], b = w1[j + h];
                    w1[j] = a + b;
                    w1[j + h] = a - b;
                }
        cross_stage<0>(w0, w1, p.t[0]);                        // stride 8: chunk bit 0
        cross_stage<1>(w0, w1, p.t[1]);                        // stride 16: chunk bit 1
        if constexpr (B >= 64) cross_stage<2>(w0, w1, p.t[2]); // stride 32: chunk bit 2
        if constexpr (B >= 128) cross_stage<3>(w0, w1, p.t[3]); // stride 64: chunk bit 3
        if constexpr (B == 256) {
#pragma unroll
            for (int i = 0; i < 8; ++i) { // stride 128: the lane's two groups (same leftover sign)
                const float a = w0[i], b = w1[i];
                w0[i] = a + b;
                w1[i] = a - b;
            }
        }
        // the "+ 0" turns an exactly zero result into +0 whatever sign the lane carries (and changes
        // nothing else): transformed zeros are stored unsigned
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            w0[i] = __builtin_fmaf(w0[i], p.fin, 0.0f);
            w1[i] = __builtin_fmaf(w1[i], p.fin, 0.0f);
        }
    }
    float m0 = 0.0f, m1 = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        m0 = fmaxf(m0, fabsf(w0[i]));
        m1 = fmaxf(m1, fabsf(w1[i]));
    }
    m0 = fmaxf(m0, dpp_get<0xB1>(m0)); // the MX block = chunks 4q..4q+3 = the lane's quad
    m1 = fmaxf(m1, dpp_get<0xB1>(m1));
    m0 = fmaxf(m0, dpp_get<0x4E>(m0));
    m1 = fmaxf(m1, dpp_get<0x4E>(m1));
    s0 = e8m0_of_amax(m0);
    s1 = e8m0_of_amax(m1);
    if constexpr (SR) {
        codes0 = pack8_sr(w0, s0, key, row, kk0);
        codes1 = pack8_sr(w1, s1, key, row, kk1);
        return;
    }
    const float x0 = __uint_as_float((uint32_t)s0 << 23), x1 = __uint_as_float((uint32_t)s1 << 23);
    codes0 = 0;
    codes1 = 0;
    codes0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes0, w0[0], w0[1], x0, 0);
    codes0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes0, w0[2], w0[3], x0, 1);
    codes0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes0, w0[4], w0[5], x0, 2);
    codes0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes0, w0[6], w0[7], x0, 3);
    codes1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes1, w1[0], w1[1], x1, 0);
    codes1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes1, w1[2], w1[3], x1, 1);
    codes1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes1, w1[4], w1[5], x1, 2);
    codes1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes1, w1[6], w1[7], x1, 3);
}

__device__ __forceinline__ void apply_k_mask(float (&w)[8], uint64_t zm)
{
#pragma unroll
    for (int i = 0; i < 8; ++i)
        if ((zm >> (8 * i)) & 0xffu) w[i] = 0.0f;
}

// Of 8 consecutive K-elements (raw bf16 in r), all go to slot[pos1] of the row's copy, pos1 being position + 1 for an
// extracted element and 0 for one that stays: slot 0 takes what is not extracted and is never read, so that no
// store needs a condition of its own (eight predicated stores cost three times the instructions).
constexpr int KC_GATHER_SLOT0 = 7; // index of slot 0 in the LDS array: the copy proper starts 16-byte aligned behind it

__device__ __forceinline__ void scatter_extracted(uint4 r, uint4 pos, uint16_t *slot)
{
    const uint32_t e[4] = {r.x, r.y, r.z, r.w}, q[4] = {pos.x, pos.y, pos.z, pos.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        slot[q[j] & 0xffffu] = (uint16_t)e[j];
        slot[q[j] >> 16] = (uint16_t)(e[j] >> 16);
    }
}

// The raw bf16 pairs with the extracted elements (pos1 != 0) cleared to +0: per 16-bit half, min(pos1, 1) - 1 is
// 0xffff for an element that stays and 0 for an extracted one.
__device__ __forceinline__ uint4 clear_extracted(uint4 r, uint4 pos)
{
    const uint32_t ones = 0x00010001u;
    auto keep = [&](uint32_t q) { // (the compiler's own code for this is a compare and a select per half)
        uint32_t t;
        asm("v_pk_min_u16 %0, %1, %2\n\tv_pk_sub_u16 %0, %0, %2" : "=&v"(t) : "v"(q), "v"(ones));
        return t;
    };
    return make_uint4(r.x & keep(pos.x), r.y & keep(pos.y), r.z & keep(pos.z), r.w & keep(pos.w));
}

// k0: start of the lane group's 256 K-elements (a multiple of 256).  sm: optional second copy of the scales in
// the order the tiled GEMM kernel reads them, [K/256][sm.rows][8].
__device__ __forceinline__ void store_codes_scales(uint8_t *codes, uint8_t *scales, int64_t row, int64_t K, int64_t k0,
                                                   int chunk, uint32_t c0, uint32_t c1, int s0, int s1, scales_sm_t sm)
{
    uint8_t *crow = codes + row * (K >> 1) + ((k0 + chunk * 8) >> 1);
    *reinterpret_cast<uint32_t *>(crow) = c0;
    *reinterpret_cast<uint32_t *>(crow + 64) = c1;
    if ((chunk & 3) == 0) {
        uint8_t *srow = scales + row * (K >> 5) + ((k0 + chunk * 8) >> 5);
        srow[0] = (uint8_t)s0;
        srow[4] = (uint8_t)s1;
        if (sm.out && row < sm.rows) {
            uint8_t *q = sm.out + ((k0 >> 8) * sm.rows + row) * 8 + (chunk >> 2);
            q[0] = (uint8_t)s0;
            q[4] = (uint8_t)s1;
        }
    }
}

// K-contiguous operand: 16 lanes per 256 K-elements of a row.  FLAT as in k_quant_kc.
template <int B, int FLAT, bool SR>
__global__ __launch_bounds__(256) void k_quant_kc16(const uint16_t *__restrict__ x, int64_t outer, int64_t K,
                                                    int64_t ld, const uint8_t *__restrict__ zero_outer,
                                                    const uint8_t *__restrict__ zero_k,
                                                    uint8_t *__restrict__ codes, uint8_t *__restrict__ scales,
                                                    sr_key_t key, scales_sm_t sm)
{
    const uint32_t upr = (uint32_t)(K >> 8); // 256-element units per row
    int64_t row;
    uint32_t unit;
    bool active;
    if constexpr (FLAT) {
        const uint32_t u = (blockIdx.x * 256u + threadIdx.x) >> 4;
        const uint32_t r = u / upr;
        row = r;
        unit = u - r * upr;
        active = row < outer;
    } else {
        row = blockIdx.x;
        unit = (blockIdx.y * 256u + threadIdx.x) >> 4;
        active = unit < upr;
    }
    const lane_plan_t plan = make_plan<B>(threadIdx.x & 63);
    const int64_t k0 = (int64_t)unit * 256, kk = k0 + plan.chunk * 8;

    uint4 r0 = make_uint4(0, 0, 0, 0), r1 = make_uint4(0, 0, 0, 0);
    if (active) { // the row's mask byte travels with the data (1 % of the rows are read for nothing) instead of ahead of it
        const uint16_t *src = x + row * ld + kk;
        r0 = load_once16(src);
        r1 = load_once16(src + 128);
        if (zero_outer && zero_outer[row]) r0 = r1 = make_uint4(0, 0, 0, 0);
    }
    float w0[8] = {bf16_lo(r0.x), bf16_hi(r0.x), bf16_lo(r0.y), bf16_hi(r0.y),
                   bf16_lo(r0.z), bf16_hi(r0.z), bf16_lo(r0.w), bf16_hi(r0.w)};
    float w1[8] = {bf16_lo(r1.x), bf16_hi(r1.x), bf16_lo(r1.y), bf16_hi(r1.y),
                   bf16_lo(r1.z), bf16_hi(r1.z), bf16_lo(r1.w), bf16_hi(r1.w)};
    if (zero_k && active) {
        const uint64_t z0 = *reinterpret_cast<const uint64_t *>(zero_k + kk);
        const uint64_t z1 = *reinterpret_cast<const uint64_t *>(zero_k + kk + 128);
        apply_k_mask(w0, z0);
        apply_k_mask(w1, z1);
    }
    uint32_t c0, c1;
    int s0, s1;
    transform_quantize16<B, SR>(w0, w1, plan, c0, c1, s0, s1, key, row, kk, kk + 128);
    if (active) store_codes_scales(codes, scales, row, K, k0, plan.chunk, c0, c1, s0, s1, sm);
}

// The same with the extracted K-channels copied out on the way (Eq. 7 with S a set of K-channels).  One workgroup
// takes a whole row, 4096 K-elements per pass.  In place of the byte mask it reads a 16-bit table, position in the
// index list + 1 for an extracted channel and 0 for the others, with the operand (one more coalesced load, no
// dependent look-ups); the extracted elements it meets go to those positions of a copy of the row's extracted part
// in LDS, which leaves for memory at the end in whole 16-byte pieces; they are cleared in the raw bf16 pairs with three
// packed 16-bit instructions per pair.
// (Two variants were measured on 16384 x 28672 at 1 % and made the quantiser half again as slow, more than the
// separate gather kernel costs: 2-byte stores straight into the copy, and a look-up of the position in a 32-bit
// table under the branch that an extracted element takes -- a chain of dependent loads in nearly every wave.
// What the kernel costs over the plain one, 10 .. 20 %, is not its instructions: with a fifth fewer of them, and
// with the next pass's loads issued ahead, it took the same time; without the table loads 4 .. 37 us of the 14 .. 50
// go away, most on the 57 KB table of K = 28672, which every workgroup reads whole.)
constexpr int KC_GATHER_MAX_KPAD = 4096;

template <int B, bool SR>
__global__ __launch_bounds__(256) void k_quant_kc16_gather(const uint16_t *__restrict__ x, int64_t K, int64_t ld,
                                                           uint8_t *__restrict__ codes, uint8_t *__restrict__ scales,
                                                           sr_key_t key, scales_sm_t sm, k_gather_t gk)
{
    __shared__ __attribute__((aligned(16))) uint16_t lds[8 + KC_GATHER_MAX_KPAD];
    uint16_t *slot = lds + KC_GATHER_SLOT0, *part = lds + 8; // part[t] = slot[t + 1]
    const uint32_t upr = (uint32_t)(K >> 8);
    const int64_t row = blockIdx.x;
    const lane_plan_t plan = make_plan<B>(threadIdx.x & 63);
    for (int p = gk.k + threadIdx.x; p < gk.kpad; p += 256) part[p] = 0;
    for (uint32_t u0 = 0; u0 < upr; u0 += 16) {
        const uint32_t unit = u0 + (threadIdx.x >> 4);
        const bool active = unit < upr;
        const int64_t k0 = (int64_t)unit * 256, kk = k0 + plan.chunk * 8;
        uint4 r0 = make_uint4(0, 0, 0, 0), r1 = r0, p0 = r0, p1 = r0;
        if (active) {
            const uint16_t *src = x + row * ld + kk;
            r0 = load_once16(src);
            r1 = load_once16(src + 128);
            p0 = *reinterpret_cast<const uint4 *>(gk.pos1 + kk);
            p1 = *reinterpret_cast<const uint4 *>(gk.pos1 + kk + 128);
        }
        if (p0.x | p0.y | p0.z | p0.w) scatter_extracted(r0, p0, slot);
        if (p1.x | p1.y | p1.z | p1.w) scatter_extracted(r1, p1, slot);
        r0 = clear_extracted(r0, p0);
        r1 = clear_extracted(r1, p1);
        float w0[8] = {bf16_lo(r0.x), bf16_hi(r0.x), bf16_lo(r0.y), bf16_hi(r0.y),
                       bf16_lo(r0.z), bf16_hi(r0.z), bf16_lo(r0.w), bf16_hi(r0.w)};
        float w1[8] = {bf16_lo(r1.x), bf16_hi(r1.x), bf16_lo(r1.y), bf16_hi(r1.y),
                       bf16_lo(r1.z), bf16_hi(r1.z), bf16_lo(r1.w), bf16_hi(r1.w)};
        uint32_t c0, c1;
        int s0, s1;
        transform_quantize16<B, SR>(w0, w1, plan, c0, c1, s0, s1, key, row, kk, kk + 128);
        if (active) store_codes_scales(codes, scales, row, K, k0, plan.chunk, c0, c1, s0, s1, sm);
    }
    __syncthreads();
    uint16_t *dst = gk.out + row * gk.kpad;
    for (int p = threadIdx.x * 8; p < gk.kpad; p += 256 * 8)
        *reinterpret_cast<uint4 *>(dst + p) = *reinterpret_cast<const uint4 *>(part + p);
}

// ------------------------------------------------------------------------------------------------
// K-strided operand (element (o, kk) at x[kk*ld + o]), K % 256 == 0.  A workgroup takes a tile of 256 K-rows x 64
// columns: coalesced 16-byte loads (8 columns of one K-row per lane) go to LDS as they are, and the LDS
// transposing read of gfx950 (ds_read_b64_tr_b16) hands every lane 4 consecutive K-elements of one column per
// instruction -- the transposition costs a quarter of an LDS instruction per element.
//
// The transposing read works on groups of 16 lanes: lane s supplies the address of 4 consecutive 16-bit elements
// (a piece of one K-row), and lane n of the group receives, as element j, the element n % 4 of the piece that lane
// 4 j + n / 4 supplied.  With lane s pointing at K-row 64 (s % 4) + 4 t + s / 4 of 4 neighbouring columns, lane n
// receives K-rows 64 (n / 4) + 4 t .. + 3 of column n % 4: after 16 reads (t = 0 .. 15) a group of 16 lanes holds
// 4 columns x 256 K, lane n the 64 consecutive K-elements [64 m, 64 m + 64), m = n / 4, of its column.
//
// Work split, then: strides 1 .. 32 of the transform are butterflies inside a lane's 64 registers, stride 64 pairs
// the lanes m and m ^ 1, stride 128 m and m ^ 2 of a column.  A gfx9 DPP row offers lane ^ 8 (row_ror:8) and lane ^ 7
// (row_half_mirror) but not lane ^ 4, so the K-rows with bit 6 set are stored in LDS with every aligned group of 4
// columns reversed: lane n then holds column 3 - n % 4 when m is odd, and lane n ^ 7 is its stride-64 partner in
// the same column.  The two MX blocks of a lane lie entirely in its registers (no cross-lane maximum).
//
// (A variant with 128 columns per workgroup, 256-byte pieces of the operand's K-rows, runs at the same speed: the
// kernel is bound by its vector instructions, about 15 per element, as much as by memory.)
//
// LDS layout: K-row kk at row index 4 (kk % 64) + kk / 64, 144 bytes per row (128 of data).  The 16 pieces of one
// transposing read of a half wave (two groups: 16 bytes per row) then start 4 banks apart and cover the 64 banks
// exactly once; the 16-byte writes of a 16-lane group go to two rows whose banks do not overlap either.
// ------------------------------------------------------------------------------------------------
constexpr int KS_COLS = 64, KT_PITCH = 144;
constexpr unsigned KS_GROUP = 32, KS_GROUP_FROM = 200; // column tiles that walk the K-blocks together; from how many on

typedef short v4s __attribute__((ext_vector_type(4)));

#define ADAHOP_FMAC_DPP16_AT(W, O, CTRL, T)                                                                    \
    asm volatile("s_nop 1\n\t"                                                                                \
                 "v_fmac_f32_dpp %0, %0, %16 " CTRL "\n\tv_fmac_f32_dpp %1, %1, %16 " CTRL "\n\t"             \
                 "v_fmac_f32_dpp %2, %2, %16 " CTRL "\n\tv_fmac_f32_dpp %3, %3, %16 " CTRL "\n\t"             \
                 "v_fmac_f32_dpp %4, %4, %16 " CTRL "\n\tv_fmac_f32_dpp %5, %5, %16 " CTRL "\n\t"             \
                 "v_fmac_f32_dpp %6, %6, %16 " CTRL "\n\tv_fmac_f32_dpp %7, %7, %16 " CTRL "\n\t"             \
                 "v_fmac_f32_dpp %8, %8, %16 " CTRL "\n\tv_fmac_f32_dpp %9, %9, %16 " CTRL "\n\t"             \
                 "v_fmac_f32_dpp %10, %10, %16 " CTRL "\n\tv_fmac_f32_dpp %11, %11, %16 " CTRL "\n\t"         \
                 "v_fmac_f32_dpp %12, %12, %16 " CTRL "\n\tv_fmac_f32_dpp %13, %13, %16 " CTRL "\n\t"         \
                 "v_fmac_f32_dpp %14, %14, %16 " CTRL "\n\tv_fmac_f32_dpp %15, %15, %16 " CTRL "\n\t"         \
                 "s_nop 1"                                                                                    \
                 : "+v"(W[O + 0]), "+v"(W[O + 1]), "+v"(W[O + 2]), "+v"(W[O + 3]), "+v"(W[O + 4]), "+v"(W[O + 5]),    \
                   "+v"(W[O + 6]), "+v"(W[O + 7]), "+v"(W[O + 8]), "+v"(W[O + 9]), "+v"(W[O + 10]), "+v"(W[O + 11]),  \
                   "+v"(W[O + 12]), "+v"(W[O + 13]), "+v"(W[O + 14]), "+v"(W[O + 15])                             \
                 : "v"(T))

// w <- partner(w) * t + w on all 64 values of the lane; XOR7: the partner is lane ^ 7, else lane ^ 8.
template <bool XOR7> __device__ __forceinline__ void cross_stage64(float (&w)[64], float t)
{
#pragma unroll
    for (int o = 0; o < 64; o += 16) {
        if constexpr (XOR7)
            ADAHOP_FMAC_DPP16_AT(w, o, "row_half_mirror row_mask:0xf bank_mask:0xf", t);
        else
            ADAHOP_FMAC_DPP16_AT(w, o, "row_ror:8 row_mask:0xf bank_mask:0xf", t);
    }
}

__device__ __forceinline__ uint32_t rot16(uint32_t v) { return __builtin_amdgcn_alignbit(v, v, 16); }

template <int B, bool SR>
__global__ __launch_bounds__(256) void k_quant_ks16(const uint16_t *__restrict__ x, int64_t outer, int64_t K,
                                                    int64_t ld, const uint8_t *__restrict__ zero_outer,
                                                    const uint8_t *__restrict__ zero_k,
                                                    uint8_t *__restrict__ codes, uint8_t *__restrict__ scales,
                                                    sr_key_t key, scales_sm_t sm, unsigned group)
{
    __shared__ __attribute__((aligned(16))) uint8_t tile[256 * KT_PITCH];
    __shared__ uint8_t kmask[256];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    // Workgroups start in the order of their linear index, x fastest.  Taken as it is, that order runs all column
    // tiles of one K-block before the next K-block: the workgroups in flight together then write 128-byte pieces of
    // thousands of different output rows.  Instead the index walks KS_GROUP neighbouring column tiles through all
    // K-blocks before it moves to the next group: the reads still come in pieces of KS_GROUP x 128 bytes of a K-row, and
    // an output row is written in one go.  Measured: operands with rows of 28672 elements (448 column tiles: the
    // about 1000 workgroups in flight span two K-blocks, 300 bytes of an output row) 292 -> 237 us ([16384][28672])
    // and 133 -> 122 us ([8192][28672]); 384, 320 and 224 column tiles 11 .. 13 % faster; 256 column tiles 7 % faster
    // or 5 % slower by K; with 192 column tiles and fewer the plain order is as fast or up to 10 % faster and is kept
    // (group == 0).
    unsigned bx = blockIdx.x, by = blockIdx.y;
    if (group) {
        const uint64_t nx = gridDim.x, ny = gridDim.y, L = by * nx + bx, full = nx / group * group;
        if (L < full * ny) {
            const uint64_t r = L % (group * ny);
            bx = (unsigned)(L / (group * ny) * group + r % group);
            by = (unsigned)(r / group);
        } else { // the last, narrower group
            const uint64_t r = L - full * ny, wdt = nx - full;
            bx = (unsigned)(full + r % wdt);
            by = (unsigned)(r / wdt);
        }
    }
    const int64_t o0 = (int64_t)bx * KS_COLS, k0 = (int64_t)by * 256;

    // ---- global -> LDS: a pass is 32 K-rows x 64 columns; lane: 8 columns (cg) of one of the wave's 8 rows.  A group
    // of 16 lanes takes two rows two apart (their banks do not overlap: consecutive K-rows are 16 banks apart).
    {
        const int cg = lane & 7, q = lane >> 4;
        const int rw = w * 8 + (q >> 1) * 4 + (q & 1) + 2 * ((lane >> 3) & 1);
        const int64_t oc = o0 + cg * 8;
        const bool ok = oc < outer;
        uint32_t cm[4] = {~0u, ~0u, ~0u, ~0u}; // keeps the columns that are not masked out
        if (zero_outer && ok) {
            // the 8 mask bytes of the lane's columns in one load where that is possible (eight dependent byte loads
            // at the head of every workgroup cost the masked call a third more time)
            uint64_t z = 0;
            if ((reinterpret_cast<uintptr_t>(zero_outer) & 7) == 0 && oc + 8 <= outer) {
                z = *reinterpret_cast<const uint64_t *>(zero_outer + oc);
            } else {
#pragma unroll
                for (int c = 0; c < 8; ++c)
                    if (oc + c < outer && zero_outer[oc + c]) z |= (uint64_t)1 << (8 * c);
            }
#pragma unroll
            for (int c = 0; c < 8; ++c)
                if ((z >> (8 * c)) & 0xffu) cm[c >> 1] &= (c & 1) ? 0x0000ffffu : 0xffff0000u;
        }
        uint4 v[8];
        // K-mask: one byte of the tile's 256 per thread, loaded ahead of the data and handed round through LDS (eight
        // byte loads per lane, one for each of its K-rows, made the masked call 15 % slower than the plain one)
        uint8_t my_kz = 0;
        if (zero_k) my_kz = zero_k[k0 + tid];
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int64_t kk = k0 + it * 32 + rw;
            v[it] = ok ? load_once16(x + kk * ld + oc) : make_uint4(0, 0, 0, 0);
        }
        uint32_t zk = 0; // bit it: the lane's K-row of pass it is masked out
        if (zero_k) {    // (uniform: a kernel argument)
            kmask[tid] = my_kz;
            __syncthreads();
#pragma unroll
            for (int it = 0; it < 8; ++it) zk |= (kmask[it * 32 + rw] ? 1u : 0u) << it;
        }
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int row = it * 32 + rw; // K-row within the tile; bit 6 = bit 1 of it
            const uint32_t kz = ((zk >> it) & 1u) ? 0u : ~0u;
            uint4 u = make_uint4(v[it].x & cm[0] & kz, v[it].y & cm[1] & kz, v[it].z & cm[2] & kz, v[it].w & cm[3] & kz);
            if (it & 2) u = make_uint4(rot16(u.y), rot16(u.x), rot16(u.w), rot16(u.z)); // groups of 4 columns reversed
            *reinterpret_cast<uint4 *>(tile + (4 * (row & 63) + (row >> 6)) * KT_PITCH + cg * 16) = u;
        }
    }
    __syncthreads();

    // ---- LDS -> registers, transposed: wave w takes columns [16 w, 16 w + 16)
    const int n = lane & 15, g = lane >> 4, m = n >> 2, e = n & 3;
    float wv[64];
    {
        // as the supplier of addresses this lane is s = n: K-row 64 (s % 4) + 4 t + s / 4, i.e. row index 16 t + 4 (s / 4) + s % 4
        const uint8_t *src = tile + (4 * (n >> 2) + (n & 3)) * KT_PITCH + 32 * w + 8 * g;
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            const v4s d = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) v4s *)(src + t * 16 * KT_PITCH));
#pragma unroll
            for (int j = 0; j < 4; ++j) wv[4 * t + j] = bf16_one((uint16_t)d[j]);
        }
    }
    const int col = 16 * w + 4 * g + ((m & 1) ? 3 - e : e);
    const int64_t o = o0 + col;
    const bool active = o < outer;

    // ---- transform
    if constexpr (B > 0) {
        constexpr int HMAX = B >= 64 ? 32 : 16;
#pragma unroll
        for (int h = 1; h <= HMAX; h *= 2)
#pragma unroll
            for (int i = 0; i < 64; i += 2 * h)
#pragma unroll
                for (int j = i; j < i + h; ++j) {
                    const float a = wv[j], b = wv[j + h];
                    wv[j] = a + b;
                    wv[j + h] = a - b;
                }
        float sign = 1.0f;
        if constexpr (B >= 128) { // stride 64: lanes m and m ^ 1 of the column (lane ^ 7)
            const bool upper = (m & 1) != 0;
            cross_stage64<true>(wv, upper ? -1.0f : 1.0f);
            if (upper) sign = -sign;
        }
        if constexpr (B == 256) { // stride 128: lanes m and m ^ 2 (lane ^ 8)
            const bool upper = (m & 2) != 0;
            cross_stage64<false>(wv, upper ? -1.0f : 1.0f);
            if (upper) sign = -sign;
        }
        // the sign left over from the stages goes into the normalisation; "+ 0" stores exact zeros unsigned
        const float fin = sign * hadamard_norm<B>();
#pragma unroll
        for (int i = 0; i < 64; ++i) wv[i] = __builtin_fmaf(wv[i], fin, 0.0f);
    }

    // ---- the lane's two MX blocks
    uint32_t c[8];
    int sc[2];
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
        float amax = 0.0f;
#pragma unroll
        for (int i = 0; i < 32; ++i) amax = fmaxf(amax, fabsf(wv[32 * blk + i]));
        const int s = e8m0_of_amax(amax);
        sc[blk] = s;
        if constexpr (SR) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float t8[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) t8[i] = wv[32 * blk + 8 * q + i];
                c[4 * blk + q] = pack8_sr(t8, s, key, o, k0 + 64 * m + 32 * blk + 8 * q);
            }
        } else {
            const float X = __uint_as_float((uint32_t)s << 23);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint32_t p = 0;
                const float *v8 = wv + 32 * blk + 8 * q;
                p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, v8[0], v8[1], X, 0);
                p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, v8[2], v8[3], X, 1);
                p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, v8[4], v8[5], X, 2);
                p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, v8[6], v8[7], X, 3);
                c[4 * blk + q] = p;
            }
        }
    }
    if (active) {
        uint8_t *crow = codes + o * (K >> 1) + ((k0 + 64 * m) >> 1);
        *reinterpret_cast<uint4 *>(crow) = make_uint4(c[0], c[1], c[2], c[3]);
        *reinterpret_cast<uint4 *>(crow + 16) = make_uint4(c[4], c[5], c[6], c[7]);
    }
    // The column's 8 scale bytes of this tile sit in the four lanes m = 0 .. 3 of the column, which are 4 apart in
    // the row of 16 lanes: the lane m = 0 collects them (two DPP shifts) and stores them at once.  Byte stores, four
    // per lane, were three quarters of the kernel's write requests.
    // (Lanes with odd m hold the columns of their quad in reverse order: they take their neighbour's bytes first.)
    const uint32_t own = (uint32_t)sc[0] | ((uint32_t)sc[1] << 8);
    const uint32_t mirrored = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)own, 0x1B /* quad_perm:[3,2,1,0] */, 0xf, 0xf, true);
    const uint32_t mine = (m & 1) ? mirrored : own;
    const uint32_t pair = mine | ((uint32_t)__builtin_amdgcn_update_dpp(0, (int)mine, 0x104 /* row_shl:4 */, 0xf, 0xf, true) << 16);
    const uint32_t upper = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)pair, 0x108 /* row_shl:8 */, 0xf, 0xf, true);
    if (active && m == 0) {
        uint8_t *srow = scales + o * (K >> 5) + (k0 >> 5);
        if ((reinterpret_cast<uintptr_t>(srow) & 7) == 0) {
            *reinterpret_cast<uint2 *>(srow) = make_uint2(pair, upper);
        } else { // the canonical array has no alignment rule
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                srow[i] = (uint8_t)(pair >> (8 * i));
                srow[4 + i] = (uint8_t)(upper >> (8 * i));
            }
        }
        if (sm.out && o < sm.rows)
            *reinterpret_cast<uint2 *>(sm.out + ((k0 >> 8) * sm.rows + o) * 8) = make_uint2(pair, upper);
    }
}

template <int B, bool SR>
int launch_kc(const adahop_operand_t &x, const uint8_t *zo, const uint8_t *zk, uint8_t *codes, uint8_t *scales,
              sr_key_t key, scales_sm_t sm, k_gather_t gk, hipStream_t st)
{
    const uint16_t *d = static_cast<const uint16_t *>(x.data);
    if (x.K % 256 == 0) {
        const int64_t tpr = x.K / 16; // threads per row
        if (gk.out) {
            hipLaunchKernelGGL((k_quant_kc16_gather<B, SR>), dim3((unsigned)x.outer), dim3(256), 0, st, d, x.K, x.ld, codes,
                               scales, key, sm, gk);
            return check_launch();
        }
        if (tpr >= 128) {
            dim3 grid((unsigned)x.outer, (unsigned)ceil_div(tpr, 256));
            hipLaunchKernelGGL((k_quant_kc16<B, 0, SR>), grid, dim3(256), 0, st, d, x.outer, x.K, x.ld, zo, zk, codes,
                               scales, key, sm);
        } else {
            dim3 grid((unsigned)ceil_div(x.outer * tpr, 256));
            hipLaunchKernelGGL((k_quant_kc16<B, 1, SR>), grid, dim3(256), 0, st, d, x.outer, x.K, x.ld, zo, zk, codes,
                               scales, key, sm);
        }
        return check_launch();
    }
    const int64_t cpr = x.K / 8;
    if (cpr >= 128) {
        dim3 grid((unsigned)x.outer, (unsigned)ceil_div(cpr, 256));
        hipLaunchKernelGGL((k_quant_kc<B, 0, SR>), grid, dim3(256), 0, st, d, x.outer, x.K, x.ld, zo, zk, codes, scales,
                           key);
    } else {
        dim3 grid((unsigned)ceil_div(x.outer * cpr, 256));
        hipLaunchKernelGGL((k_quant_kc<B, 1, SR>), grid, dim3(256), 0, st, d, x.outer, x.K, x.ld, zo, zk, codes, scales,
                           key);
    }
    return check_launch();
}

template <int B> constexpr size_t ks_lds_bytes()
{
    return ks_cfg<B>::NCH > 1 ? (size_t)ks_cfg<B>::NW * 32 * 64 * sizeof(float2) : 0;
}

template <int B> int allow_ks_lds()
{
    if (ks_lds_bytes<B>() <= 48 * 1024) return ADAHOP_OK;
    int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_quant_ks<B, false>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)ks_lds_bytes<B>()));
    if (rc != ADAHOP_OK) return rc;
    return check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_quant_ks<B, true>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)ks_lds_bytes<B>()));
}

template <int B, bool SR>
int launch_ks(const adahop_operand_t &x, const uint8_t *zo, const uint8_t *zk, uint8_t *codes, uint8_t *scales,
              sr_key_t key, scales_sm_t sm, hipStream_t st)
{
    if (iht_quantize_writes_scales_sm(x)) {
        dim3 grid((unsigned)ceil_div(x.outer, KS_COLS), (unsigned)(x.K / 256));
        const unsigned group = grid.x > KS_GROUP_FROM ? KS_GROUP : 0u;
        hipLaunchKernelGGL((k_quant_ks16<B, SR>), grid, dim3(256), 0, st, static_cast<const uint16_t *>(x.data), x.outer,
                           x.K, x.ld, zo, zk, codes, scales, key, sm, group);
        return check_launch();
    }
    constexpr int NW = ks_cfg<B>::NW;
    constexpr int NCH = ks_cfg<B>::NCH;
    const size_t lds = ks_lds_bytes<B>();
    if (lds > 48 * 1024) { // more LDS than a launch may ask for by default: allowed once per device
        const int rc = configure_quantizers();
        if (rc != ADAHOP_OK) return rc;
    }
    dim3 grid((unsigned)ceil_div(x.outer, 128), (unsigned)ceil_div(x.K / 32, NW));
    hipLaunchKernelGGL((k_quant_ks<B, SR>), grid, dim3(NW * 64), lds, st, static_cast<const uint16_t *>(x.data),
                       x.outer, x.K, x.ld, zo, zk, codes, scales, key);
    return check_launch();
}

template <bool SR>
int dispatch_block(const adahop_operand_t &x, int b, const uint8_t *zo, const uint8_t *zk, uint8_t *codes,
                   uint8_t *scales, sr_key_t key, scales_sm_t sm, k_gather_t gk, hipStream_t st)
{
#define ADAHOP_DISPATCH(BB)                                                                  \
    case BB:                                                                                 \
        return x.k_contig ? launch_kc<BB, SR>(x, zo, zk, codes, scales, key, sm, gk, st)     \
                          : launch_ks<BB, SR>(x, zo, zk, codes, scales, key, sm, st);
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

} // namespace

// The instances of the general K-strided quantiser that need more LDS than the default, once per device (host-side
// calls, nothing queued).
int configure_quantizers()
{
    static device_once_t once;
    int dev = 0;
    int rc = check_hip(hipGetDevice(&dev));
    if (rc != ADAHOP_OK || !once.need(dev)) return rc;
    if ((rc = allow_ks_lds<0>()) != ADAHOP_OK || (rc = allow_ks_lds<32>()) != ADAHOP_OK || (rc = allow_ks_lds<64>()) != ADAHOP_OK ||
        (rc = allow_ks_lds<128>()) != ADAHOP_OK || (rc = allow_ks_lds<256>()) != ADAHOP_OK)
        return rc;
    once.mark(dev);
    return ADAHOP_OK;
}

// The kernels for K % 256 == 0 (K / 256 is a grid dimension of the K-strided one) are the ones that also write
// the stage-major copy of the scales.
bool iht_quantize_writes_scales_sm(const adahop_operand_t &x) { return x.K % 256 == 0 && x.K / 256 <= 65535; }

// sr_seed: NULL for round-to-nearest-even, else the seed of the stochastic rounding of the elements.
// sm: NULL, or where a stage-major copy of the scales goes; honoured by the kernels for K % 256 == 0 only,
// which is also the only case in which the tiled GEMM kernel asks for it.
// A whole row per workgroup pays from 4096 K-elements on (one pass of all its lanes); the copy is staged in LDS.
bool iht_quantize_gathers_k(const adahop_operand_t &x, int kpad)
{
    return x.k_contig && x.K % 4096 == 0 && kpad <= KC_GATHER_MAX_KPAD && kpad % 8 == 0 && x.outer <= 0x7fffffff;
}

// gather: NULL, or where the extracted channels are copied to and the table that names them (it must describe the
// same channels as zk); honoured only where iht_quantize_gathers_k holds and zk is given.
int launch_iht_quantize(const adahop_operand_t &x, int b, const uint8_t *zo, const uint8_t *zk, uint8_t *codes,
                        uint8_t *scales, hipStream_t st, const uint64_t *sr_seed, const scales_sm_t *sm,
                        const k_gather_t *gather)
{
    if (x.outer == 0 || x.K == 0) return ADAHOP_OK;
    const scales_sm_t smv = sm && iht_quantize_writes_scales_sm(x) ? *sm : scales_sm_t{nullptr, 0};
    const k_gather_t gk = gather && gather->out && zk && !zo && iht_quantize_gathers_k(x, gather->kpad)
                              ? *gather
                              : k_gather_t{nullptr, nullptr, 0, 0};
    if (sr_seed) {
        const sr_key_t key = {(uint32_t)*sr_seed, (uint32_t)(*sr_seed >> 32)};
        return dispatch_block<true>(x, b, zo, zk, codes, scales, key, smv, gk, st);
    }
    return dispatch_block<false>(x, b, zo, zk, codes, scales, sr_key_t{0, 0}, smv, gk, st);
}

} // namespace adahop
