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
//
// Pipeline.  A stage holds 128 bytes of K per row for the 256 A rows and the 256 B rows -- 256 FP4
// K-elements (8 MX blocks, four matrix-core steps) or 64 gathered bf16 K-channels -- plus the 8 scale
// bytes per row: 68 KiB.  Two stages rotate in LDS and global memory is copied straight into LDS
// (global_load_lds): whole 128-byte lines per row, which is what the vector L1 moves fastest.  The
// one barrier per stage sits before the last matrix-core step of the stage: by then every wave has
// read its last fragments of the stage, so that buffer is refilled at once (the copy for stage t+2
// runs during the last step of stage t and all of stage t+1), and the next stage has landed, so its
// first fragments are read while the last step still runs.
//
// LDS layout of an operand slab: row r at r*128, its 16-byte chunk c at chunk position
// c ^ ((r / 2) & 7).  The LDS has 64 four-byte banks and serves a 16-byte-per-lane read 16 lanes at a
// time; 16 consecutive rows of one logical chunk then cover all 64 banks exactly once, and the DMA
// writes (8 rows x 8 chunks per wave instruction, linear in the lane id) are conflict-free too.
//
// K order: within a stage lane-half h of matrix-core step s takes chunk 4h+s (for FP4: MX block
// 4h+s), the same for A and B, so the four scale bytes a lane needs for a stage are one aligned
// dword and the step's byte is picked by the instruction's op_sel.
//
// Scales reach LDS by DMA as well, so the main loop has no register-targeted global loads and only
// waits where the kernel says so.  Fetching 8 bytes per row from the canonical [rows, K/32] array
// would cost one cache-line request per row and stage -- as many requests as the codes need -- so a
// small pre-pass (k_stage_major_scales) first rewrites the scales stage-major, [K/256][rows][8],
// where the 256 rows of a slab are 2 KiB contiguous.
// ------------------------------------------------------------------------------------------------
constexpr int TM = 256, TN = 256, TKB = 128, NSTAGE = 2;
constexpr int SLAB_BYTES = (TM + TN) * TKB;             // codes (or gathered bf16) of one stage
constexpr int STAGE_BYTES = SLAB_BYTES + (TM + TN) * 8; // + 8 scale bytes per row
constexpr int TILED_LDS_BYTES = NSTAGE * STAGE_BYTES;

// out[s][row][0..7] = in[row][8s .. 8s+7]   (8-byte units; KB8 = K/256 units per row)
__global__ __launch_bounds__(256) void k_stage_major_scales(const uint64_t *__restrict__ in, uint64_t *__restrict__ out,
                                                            int64_t rows, int64_t KB8)
{
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (g >= rows * KB8) return;
    const int64_t s = g / rows, r = g - s * rows; // consecutive threads: consecutive rows (coalesced writes)
    out[g] = in[r * KB8 + s];
}

// Copies from global memory straight into LDS: lane i's 16 bytes land at lds_addr + 16 i (lds_addr
// wave-uniform).  Inline assembly on purpose: with the builtin the compiler's wait-count pass makes
// every later LDS read wait for ALL outstanding copies (it cannot tell that they target the other
// stage), which serialises the copies with the matrix-core work.  The kernel waits for the copies
// itself (s_waitcnt vmcnt(0) before the stage barrier).  M0 is written here and used by nothing else
// in these kernels (no dynamic register indexing, no other DMA).
__device__ __forceinline__ void dma16(const void *g, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_addr) : "memory");
}

__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}

struct frags_t {
    uint4 a[4], b[4];
};

// Fragments of one matrix-core step for this lane: rows l32 (+32 i) of the wave's A and B slabs.
__device__ __forceinline__ void read_frags(const uint8_t *sA, const uint8_t *sB, int off, frags_t &f)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f.a[i] = *reinterpret_cast<const uint4 *>(sA + i * 32 * TKB + off);
        f.b[i] = *reinterpret_cast<const uint4 *>(sB + i * 32 * TKB + off);
    }
}

struct scales_t {
    int a[4], b[4];
};

__device__ __forceinline__ void read_scales(const uint8_t *sSa, const uint8_t *sSb, scales_t &sc)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        sc.a[i] = *reinterpret_cast<const int *>(sSa + i * 32 * 8);
        sc.b[i] = *reinterpret_cast<const int *>(sSb + i * 32 * 8);
    }
}

template <int S> __device__ __forceinline__ void mma_fp4(const frags_t &f, v16f (&acc)[4][4], const scales_t &sc)
{
#ifdef ADAHOP_DBG_NO_MMA
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j][S] += __int_as_float((f.a[i].x ^ f.b[j].y ^ sc.a[i] ^ sc.b[j]) & 0x3fffffff);
    return;
#endif
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v8i av = {(int)f.a[i].x, (int)f.a[i].y, (int)f.a[i].z, (int)f.a[i].w, 0, 0, 0, 0};
            v8i bv = {(int)f.b[j].x, (int)f.b[j].y, (int)f.b[j].z, (int)f.b[j].w, 0, 0, 0, 0};
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, bv, acc[i][j], 4, 4, S, sc.a[i], S, sc.b[j]);
        }
}

__device__ __forceinline__ void mma_bf16(const frags_t &f, v16f (&acc)[4][4])
{
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = mfma_bf16(f.a[i], f.b[j], acc[i][j]);
}

// Keeps the instruction scheduler from moving LDS reads and matrix-core instructions across this
// point (one wave per SIMD: the order written here is what hides the LDS latency).
#define ADAHOP_PIN() __builtin_amdgcn_sched_barrier(0)

// BF16 = true: the stage loop over the gathered bf16 K-channels; false: the FP4 stages.  The two
// loops run back to back on one pipeline: `stage` counts over both.
template <bool OEK>
__global__ __launch_bounds__(256) void k_gemm_mx_tile256(int64_t K, const uint8_t *__restrict__ a_codes,
                                                         const uint8_t *__restrict__ a_scales_sm,
                                                         const uint8_t *__restrict__ b_codes,
                                                         const uint8_t *__restrict__ b_scales_sm, int64_t M, int64_t N,
                                                         float *__restrict__ C, int64_t ldc,
                                                         const uint16_t *__restrict__ Ag,
                                                         const uint16_t *__restrict__ Bg, int kpad, int tiles_m,
                                                         int tiles_n, int group_m)
{
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

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

    // ---- copy engine: wave w moves rows [64w, 64w+64) of both slabs, 8 rows per instruction.
    // Lane i of instruction g writes LDS row 8g + i/8, chunk position i%8, which must hold logical
    // chunk (i%8) ^ ((row/2) & 7) = (i%8) ^ (4*(g&1) + i/16).
    const int lrow = lane >> 3;
    const int c_even = ((lane & 7) ^ (lane >> 4)) * 16, c_odd = c_even ^ 64;
    const int64_t pitch = K >> 1, gpitch = (int64_t)kpad * 2;
    const uint8_t *ga = a_codes + (m0 + w * 64 + lrow) * pitch;
    const uint8_t *gb = b_codes + (n0 + w * 64 + lrow) * pitch;
    const uint8_t *gga = reinterpret_cast<const uint8_t *>(Ag) + (m0 + w * 64 + lrow) * gpitch;
    const uint8_t *ggb = reinterpret_cast<const uint8_t *>(Bg) + (n0 + w * 64 + lrow) * gpitch;
    // scales (stage-major): waves 0,1 move the two 1 KiB halves of the A slab's scales, waves 2,3 of B's
    const uint8_t *gs = (w < 2 ? a_scales_sm + (m0 + w * 128) * 8 : b_scales_sm + (n0 + (w - 2) * 128) * 8) + lane * 16;
    const int64_t s_stride = (w < 2 ? M : N) * 8;
    const int nbf = OEK ? (kpad >> 6) : 0, nstage = nbf + (int)(K >> 8);
    const uint32_t smem_base = __builtin_amdgcn_readfirstlane(lds_address(smem));

    auto issue = [&](int stage) {
#ifdef ADAHOP_DBG_NO_DMA
        return;
#endif
        const uint32_t sbase = smem_base + (stage & 1) * STAGE_BYTES;
        const uint32_t sA = sbase + w * 64 * TKB, sB = sA + TM * TKB;
        const uint8_t *pa, *pb;
        int64_t rp;
        const bool bf = OEK && stage < nbf;
        if (bf) {
            pa = gga + (int64_t)stage * TKB;
            pb = ggb + (int64_t)stage * TKB;
            rp = gpitch * 8;
        } else {
            pa = ga + (int64_t)(stage - nbf) * TKB;
            pb = gb + (int64_t)(stage - nbf) * TKB;
            rp = pitch * 8;
        }
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            const int co = (g & 1) ? c_odd : c_even;
            dma16(pa + g * rp + co, sA + g * 1024);
            dma16(pb + g * rp + co, sB + g * 1024);
        }
        if (!bf) dma16(gs + (int64_t)(stage - nbf) * s_stride, sbase + SLAB_BYTES + w * 1024);
    };

    // ---- fragment reads: row l32 (+32 i) of the wave's slab, logical chunk 4h + s
    const int rx = (l32 >> 1) & 7;
    const int off0 = ((4 * h + 0) ^ rx) * 16, off1 = ((4 * h + 1) ^ rx) * 16;
    const int off2 = ((4 * h + 2) ^ rx) * 16, off3 = ((4 * h + 3) ^ rx) * 16;
    const int a_row = (wm * 128 + l32) * TKB;
    const int b_row = TM * TKB + (wn * 128 + l32) * TKB;
    const int sa_row = SLAB_BYTES + (wm * 128 + l32) * 8 + 4 * h;
    const int sb_row = SLAB_BYTES + TM * 8 + (wn * 128 + l32) * 8 + 4 * h;

    v16f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    frags_t f0, f1;
    scales_t sc, sc_next;
#pragma unroll
    for (int i = 0; i < 4; ++i) sc.a[i] = sc.b[i] = sc_next.a[i] = sc_next.b[i] = 0;

    // prologue: both buffers filled, stage 0 landed, its first fragments read
    issue(0);
    if (nstage > 1) {
        issue(1);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(16) : "memory"); // stage 1 (>= 16 copies) may still fly
    } else {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __syncthreads();
    read_frags(smem + a_row, smem + b_row, off0, f0);
    if (!(OEK && nbf > 0)) read_scales(smem + sa_row, smem + sb_row, sc);

    // Everything of a stage except its last matrix-core step, then the hand-over to the next stage.
    auto hand_over = [&](int stage) {
        if (stage + 1 < nstage) {
            asm volatile("s_waitcnt vmcnt(0)\n\ts_waitcnt lgkmcnt(0)" ::: "memory"); // next stage landed; my reads done
            __syncthreads();
            if (stage + 2 < nstage) issue(stage + 2); // refills the buffer just released
            const uint8_t *sn = smem + ((stage + 1) & 1) * STAGE_BYTES;
            read_frags(sn + a_row, sn + b_row, off0, f0);
            if (!(OEK && stage + 1 < nbf)) read_scales(sn + sa_row, sn + sb_row, sc_next);
        }
    };

    int stage = 0;
    if constexpr (OEK) {
        for (; stage < nbf; ++stage) {
            const uint8_t *st = smem + (stage & 1) * STAGE_BYTES;
            read_frags(st + a_row, st + b_row, off1, f1);
            ADAHOP_PIN();
            mma_bf16(f0, acc);
            ADAHOP_PIN();
            read_frags(st + a_row, st + b_row, off2, f0);
            ADAHOP_PIN();
            mma_bf16(f1, acc);
            ADAHOP_PIN();
            read_frags(st + a_row, st + b_row, off3, f1);
            ADAHOP_PIN();
            mma_bf16(f0, acc);
            ADAHOP_PIN();
            hand_over(stage);
            ADAHOP_PIN();
            mma_bf16(f1, acc);
            ADAHOP_PIN();
            sc = sc_next;
        }
    }
    for (; stage < nstage; ++stage) {
        const uint8_t *st = smem + (stage & 1) * STAGE_BYTES;
        read_frags(st + a_row, st + b_row, off1, f1);
        ADAHOP_PIN();
        mma_fp4<0>(f0, acc, sc);
        ADAHOP_PIN();
        read_frags(st + a_row, st + b_row, off2, f0);
        ADAHOP_PIN();
        mma_fp4<1>(f1, acc, sc);
        ADAHOP_PIN();
        read_frags(st + a_row, st + b_row, off3, f1);
        ADAHOP_PIN();
        mma_fp4<2>(f0, acc, sc);
        ADAHOP_PIN();
        hand_over(stage);
        ADAHOP_PIN();
        mma_fp4<3>(f1, acc, sc);
        ADAHOP_PIN();
        sc = sc_next;
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

size_t gemm_mx_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    return align_up((size_t)M * (K / 32), 256) + align_up((size_t)N * (K / 32), 256);
}

int launch_gemm_mx(int64_t M, int64_t N, int64_t K, const uint8_t *a_codes, const uint8_t *a_scales,
                   const uint8_t *b_codes, const uint8_t *b_scales, float *C, int64_t ldc, const uint16_t *Ag,
                   const uint16_t *Bg, int kpad, void *workspace, hipStream_t st)
{
    if (M == 0 || N == 0) return ADAHOP_OK;
    const bool tiled = M % TM == 0 && N % TN == 0 && K % 256 == 0 && kpad % 64 == 0 && aligned(a_scales, 8) &&
                       aligned(b_scales, 8) && (M / TM) * (N / TN) < (1 << 30);
    if (tiled) {
        static bool configured = false;
        if (!configured) {
            int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_mx_tile256<false>),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, TILED_LDS_BYTES));
            if (rc != ADAHOP_OK) return rc;
            rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_mx_tile256<true>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, TILED_LDS_BYTES));
            if (rc != ADAHOP_OK) return rc;
            configured = true;
        }
        // scales, stage-major, in the caller's workspace
        uint8_t *a_sm = static_cast<uint8_t *>(workspace);
        uint8_t *b_sm = a_sm + align_up((size_t)M * (K / 32), 256);
        const int64_t KB8 = K / 256;
        hipLaunchKernelGGL(k_stage_major_scales, dim3((unsigned)ceil_div(M * KB8, 256)), dim3(256), 0, st,
                           reinterpret_cast<const uint64_t *>(a_scales), reinterpret_cast<uint64_t *>(a_sm), M, KB8);
        hipLaunchKernelGGL(k_stage_major_scales, dim3((unsigned)ceil_div(N * KB8, 256)), dim3(256), 0, st,
                           reinterpret_cast<const uint64_t *>(b_scales), reinterpret_cast<uint64_t *>(b_sm), N, KB8);
        int rc = check_launch();
        if (rc != ADAHOP_OK) return rc;
        const int tiles_m = (int)(M / TM), tiles_n = (int)(N / TN);
        const int group_m = tiles_m < 8 ? tiles_m : 8;
        const dim3 grid((unsigned)(tiles_m * tiles_n));
        if (kpad > 0)
            hipLaunchKernelGGL((k_gemm_mx_tile256<true>), grid, dim3(256), TILED_LDS_BYTES, st, K, a_codes, a_sm, b_codes,
                               b_sm, M, N, C, ldc, Ag, Bg, kpad, tiles_m, tiles_n, group_m);
        else
            hipLaunchKernelGGL((k_gemm_mx_tile256<false>), grid, dim3(256), TILED_LDS_BYTES, st, K, a_codes, a_sm,
                               b_codes, b_sm, M, N, C, ldc, Ag, Bg, kpad, tiles_m, tiles_n, group_m);
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
