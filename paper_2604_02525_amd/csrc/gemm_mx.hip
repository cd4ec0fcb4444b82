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


// ------------------------------------------------------------------------------------------------
// Tiled kernel for M % 256 == 0, N % 256 == 0, K % 256 == 0 (and kpad % 64 == 0).
//
// One workgroup (4 waves, 2x2) per 256x256 tile of C; each wave owns 128x128 = 4x4 matrix-core
// tiles, i.e. 256 fp32 accumulators per lane, and the workgroup is alone on its compute unit.
// A pipeline stage holds 128 bytes of K per row for the 256 A rows and the 256 B rows (64 KiB):
// either 256 FP4 K-elements (8 MX blocks) or 64 gathered bf16 K-channels.  Two stages are double
// buffered; global memory is copied straight into LDS (global_load_lds, 16 bytes per lane) while
// the matrix cores work on the other stage, with one barrier per stage.
//
// LDS layout of an operand slab: row r at r*128, its 16-byte chunk c stored at chunk position
// c ^ (r & 7), which makes both the DMA writes (8 rows x 8 chunks per wave instruction, linear in
// the lane id) and the 16-byte fragment reads (32 consecutive rows, same logical chunk) free of
// bank conflicts.
//
// K order: within a stage lane-half h of matrix-core step s takes chunk 4h+s (for FP4: MX block
// 4h+s), the same for A and B, so the four scale bytes a lane needs for a stage are one aligned
// dword of the canonical scale array and the step's byte is picked by the instruction's op_sel.
// ------------------------------------------------------------------------------------------------
constexpr int TM = 256, TN = 256, TKB = 128;
constexpr int STAGE_BYTES = (TM + TN) * TKB;

typedef __attribute__((address_space(1))) const void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

template <int S>
__device__ __forceinline__ void stage_step_fp4(const uint8_t *sA, const uint8_t *sB, int off, v16f (&acc)[4][4],
                                               const int (&sa)[4], const int (&sb)[4])
{
    uint4 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = *reinterpret_cast<const uint4 *>(sA + i * 4096 + off);
        b[i] = *reinterpret_cast<const uint4 *>(sB + i * 4096 + off);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v8i av = {(int)a[i].x, (int)a[i].y, (int)a[i].z, (int)a[i].w, 0, 0, 0, 0};
            v8i bv = {(int)b[j].x, (int)b[j].y, (int)b[j].z, (int)b[j].w, 0, 0, 0, 0};
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, bv, acc[i][j], 4, 4, S, sa[i], S, sb[j]);
        }
}

__device__ __forceinline__ void stage_step_bf16(const uint8_t *sA, const uint8_t *sB, int off, v16f (&acc)[4][4])
{
    uint4 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = *reinterpret_cast<const uint4 *>(sA + i * 4096 + off);
        b[i] = *reinterpret_cast<const uint4 *>(sB + i * 4096 + off);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = mfma_bf16(a[i], b[j], acc[i][j]);
}

template <bool OEK>
__global__ __launch_bounds__(256) void k_gemm_mx_tile256(int64_t K, const uint8_t *__restrict__ a_codes,
                                                         const uint8_t *__restrict__ a_scales,
                                                         const uint8_t *__restrict__ b_codes,
                                                         const uint8_t *__restrict__ b_scales, float *__restrict__ C,
                                                         int64_t ldc, const uint16_t *__restrict__ Ag,
                                                         const uint16_t *__restrict__ Bg, int kpad, int tiles_m,
                                                         int tiles_n, int group_m)
{
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, l32 = lane & 31, h = lane >> 5;

    // Workgroup -> tile.  Consecutive workgroup ids land on different XCDs (8 of them, each with its
    // own L2), so give every XCD a contiguous run of the tile sequence, and order that sequence in
    // bands of group_m tile rows so that concurrently running tiles share A and B panels.
    const int ntiles = tiles_m * tiles_n;
    int t = blockIdx.x;
    if (ntiles % 8 == 0) t = (t & 7) * (ntiles >> 3) + (t >> 3);
    const int band = group_m * tiles_n;
    const int first_m = (t / band) * group_m;
    const int gsz = min(group_m, tiles_m - first_m);
    const int tm = first_m + (t % band) % gsz;
    const int tn = (t % band) / gsz;
    const int64_t m0 = (int64_t)tm * TM, n0 = (int64_t)tn * TN;
    const int wm = w >> 1, wn = w & 1;

    // ---- copy engine: wave w moves rows [64w, 64w+64) of both slabs, 8 rows per instruction
    const int lrow = lane >> 3;
    const int lchunk = (lane & 7) ^ lrow;
    const int64_t pitch = K >> 1, gpitch = (int64_t)kpad * 2;
    const uint8_t *ga = a_codes + (m0 + w * 64 + lrow) * pitch + lchunk * 16;
    const uint8_t *gb = b_codes + (n0 + w * 64 + lrow) * pitch + lchunk * 16;
    const uint8_t *gga = reinterpret_cast<const uint8_t *>(Ag) + (m0 + w * 64 + lrow) * gpitch + lchunk * 16;
    const uint8_t *ggb = reinterpret_cast<const uint8_t *>(Bg) + (n0 + w * 64 + lrow) * gpitch + lchunk * 16;
    const int nbf = OEK ? (kpad >> 6) : 0, ntile = nbf + (int)(K >> 8);

    auto issue = [&](int tile, int stage) {
        uint8_t *sA = smem + stage * STAGE_BYTES + w * 64 * TKB;
        uint8_t *sB = sA + TM * TKB;
        const uint8_t *pa, *pb;
        int64_t rp;
        if (OEK && tile < nbf) {
            pa = gga + (int64_t)tile * TKB;
            pb = ggb + (int64_t)tile * TKB;
            rp = gpitch * 8;
        } else {
            pa = ga + (int64_t)(tile - nbf) * TKB;
            pb = gb + (int64_t)(tile - nbf) * TKB;
            rp = pitch * 8;
        }
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            __builtin_amdgcn_global_load_lds((gptr_t)(pa + g * rp), (lptr_t)(sA + g * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((gptr_t)(pb + g * rp), (lptr_t)(sB + g * 1024), 16, 0, 0);
        }
    };

    // ---- fragment reads
    const int rx = l32 & 7;
    const int off0 = ((4 * h + 0) ^ rx) * 16, off1 = ((4 * h + 1) ^ rx) * 16;
    const int off2 = ((4 * h + 2) ^ rx) * 16, off3 = ((4 * h + 3) ^ rx) * 16;
    const int a_row = (wm * 128 + l32) * TKB;
    const int b_row = TM * TKB + (wn * 128 + l32) * TKB;
    const int64_t KB = K >> 5;
    const uint8_t *psa = a_scales + (m0 + wm * 128 + l32) * KB + 4 * h;
    const uint8_t *psb = b_scales + (n0 + wn * 128 + l32) * KB + 4 * h;

    v16f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // scales of the stage after the current one are fetched while the current one is multiplied
    int sa[4] = {0, 0, 0, 0}, sb[4] = {0, 0, 0, 0}, sa_next[4] = {0, 0, 0, 0}, sb_next[4] = {0, 0, 0, 0};
    auto load_scales = [&](int fp_tile) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            sa_next[i] = *reinterpret_cast<const int *>(psa + (int64_t)i * 32 * KB + (int64_t)fp_tile * 8);
            sb_next[i] = *reinterpret_cast<const int *>(psb + (int64_t)i * 32 * KB + (int64_t)fp_tile * 8);
        }
    };

    issue(0, 0);
    if (nbf == 0) load_scales(0);
    int tile = 0;
    if constexpr (OEK) {
        // gathered K-channels first: BF16 matrix-core steps on the same accumulators
        for (; tile < nbf; ++tile) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            issue(tile + 1, (tile + 1) & 1); // the FP4 part has at least one stage, so tile + 1 < ntile
            if (tile + 1 >= nbf) load_scales(tile + 1 - nbf);
            const uint8_t *sA = smem + (tile & 1) * STAGE_BYTES + a_row;
            const uint8_t *sB = smem + (tile & 1) * STAGE_BYTES + b_row;
            stage_step_bf16(sA, sB, off0, acc);
            stage_step_bf16(sA, sB, off1, acc);
            stage_step_bf16(sA, sB, off2, acc);
            stage_step_bf16(sA, sB, off3, acc);
        }
    }
    for (; tile < ntile; ++tile) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            sa[i] = sa_next[i];
            sb[i] = sb_next[i];
        }
        if (tile + 1 < ntile) {
            issue(tile + 1, (tile + 1) & 1);
            load_scales(tile + 1 - nbf);
        }
        const uint8_t *sA = smem + (tile & 1) * STAGE_BYTES + a_row;
        const uint8_t *sB = smem + (tile & 1) * STAGE_BYTES + b_row;
        stage_step_fp4<0>(sA, sB, off0, acc, sa, sb);
        stage_step_fp4<1>(sA, sB, off1, acc, sa, sb);
        stage_step_fp4<2>(sA, sB, off2, acc, sa, sb);
        stage_step_fp4<3>(sA, sB, off3, acc, sa, sb);
    }

    float *crow = C + (m0 + wm * 128 + h * 4) * ldc + n0 + wn * 128 + l32;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                crow[(int64_t)(i * 32 + (r >> 2) * 8 + (r & 3)) * ldc + j * 32] = acc[i][j][r];
}

} // namespace

int launch_gemm_mx(int64_t M, int64_t N, int64_t K, const uint8_t *a_codes, const uint8_t *a_scales,
                   const uint8_t *b_codes, const uint8_t *b_scales, float *C, int64_t ldc, const uint16_t *Ag,
                   const uint16_t *Bg, int kpad, hipStream_t st)
{
    if (M == 0 || N == 0) return ADAHOP_OK;
    const bool tiled = M % TM == 0 && N % TN == 0 && K % 256 == 0 && kpad % 64 == 0 && aligned(a_scales, 4) &&
                       aligned(b_scales, 4) && (M / TM) * (N / TN) < (1 << 30);
    if (tiled) {
        static bool configured = false;
        if (!configured) {
            int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_mx_tile256<false>),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, 2 * STAGE_BYTES));
            if (rc != ADAHOP_OK) return rc;
            rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_mx_tile256<true>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 2 * STAGE_BYTES));
            if (rc != ADAHOP_OK) return rc;
            configured = true;
        }
        const int tiles_m = (int)(M / TM), tiles_n = (int)(N / TN);
        const int group_m = tiles_m < 8 ? tiles_m : 8;
        const dim3 grid((unsigned)(tiles_m * tiles_n));
        if (kpad > 0)
            hipLaunchKernelGGL((k_gemm_mx_tile256<true>), grid, dim3(256), 2 * STAGE_BYTES, st, K, a_codes, a_scales,
                               b_codes, b_scales, C, ldc, Ag, Bg, kpad, tiles_m, tiles_n, group_m);
        else
            hipLaunchKernelGGL((k_gemm_mx_tile256<false>), grid, dim3(256), 2 * STAGE_BYTES, st, K, a_codes, a_scales,
                               b_codes, b_scales, C, ldc, Ag, Bg, kpad, tiles_m, tiles_n, group_m);
        return check_launch();
    }
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
