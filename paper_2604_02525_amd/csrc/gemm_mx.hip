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
#include "gemm_mx_common.h"

#include <cmath>

#include <type_traits>

namespace adahop {

namespace {

// fp32 -> bf16 bits, round to nearest even (finite values and infinities).
__device__ __forceinline__ uint32_t bf16_bits(float x)
{
    const uint32_t u = __float_as_uint(x);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// Output element types of C: float, or bf16 held as its 16 bits.
__device__ __forceinline__ void store_c(float *p, float v) { *p = v; }
__device__ __forceinline__ void store_c(uint16_t *p, float v) { *p = (uint16_t)bf16_bits(v); }
__device__ __forceinline__ float load_c(const float *p) { return *p; }
__device__ __forceinline__ float load_c(const uint16_t *p) { return bf16_one(*p); }

// ------------------------------------------------------------------------------------------------
// Generic kernel: any M, N, any K % 32 == 0.  Workgroup tile 128x128, four waves as 2x2, each wave
// 64x64 (2x2 matrix-core tiles), operands read straight from global memory with bounds checks.
// It is the reference for the layout assumptions above and the fallback for ragged shapes.
// ------------------------------------------------------------------------------------------------
template <bool ACCUMULATE, typename OUT>
__global__ __launch_bounds__(256) void k_gemm_mx_generic(int64_t M, int64_t N, int64_t K,
                                                         const uint8_t *__restrict__ a_codes,
                                                         const uint8_t *__restrict__ a_scales,
                                                         const uint8_t *__restrict__ b_codes,
                                                         const uint8_t *__restrict__ b_scales, OUT *__restrict__ C,
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
                    OUT *p = C + row * ldc + col;
                    if constexpr (ACCUMULATE)
                        store_c(p, load_c(p) + acc[i][j][r]);
                    else
                        store_c(p, acc[i][j][r]);
                }
            }
        }
}


// ------------------------------------------------------------------------------------------------
// Tiled kernel for M % 256 == 0, N % 256 == 0, K % 256 == 0 (and kpad % 64 == 0).
//
// A workgroup (4 waves, 2x2) computes 256x256 tiles of C, one after the other; each wave owns 128x128 =
// 4x4 matrix-core tiles, i.e. 256 fp32 accumulators per lane, and the workgroup is alone on its compute
// unit (see k_gemm_mx_tile256 for the walk over the tiles).
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
// would cost one cache-line request per row and stage -- as many requests as the codes need -- so the
// kernel reads a stage-major copy, [K/256][rows][8], where the 256 rows of a slab are 2 KiB contiguous:
// written by the quantiser beside the canonical scales, or by a small pre-pass (k_stage_major_scales).
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

struct frags_t {
    uint4 a[4], b[4];
};

struct scales_t {
    int a[4], b[4];
};

// Where the copies of one tile come from: wave-uniform bases of its stage 0 (see k_gemm_mx_tile256).
struct copy_src_t {
    const uint8_t *ga, *gb, *gga, *ggb, *gs;
};

// Everything one wave keeps across stages and tiles.
struct tile_state_t {
    v16f acc[4][4];
    frags_t f0, f1;
    scales_t sc, scn;
    // fragment reads: byte offsets inside a stage buffer
    int a_row, b_row, sa_row, sb_row, off[4];
    // copy engine (see k_gemm_mx_tile256)
    copy_src_t cur, nxt;                     // the tile being computed and the one after it
    int n;                                   // stages per tile
    uint32_t lrow, c_even, c_odd, vs;        // per-lane: row within an 8-row group, byte of its chunk in even / odd
                                             // groups, offset of the scale copy
    uint32_t pitch, gpitch;                  // bytes between rows of the codes / of the gathered bf16 operands
    int64_t s_stride;
    uint32_t lds_w;                          // LDS address of this wave's 64 rows of the A slab, buffer 0
    uint32_t lds_s;                          // LDS address of this wave's 1 KiB of scales, buffer 0
    int nbf;
};

__device__ __forceinline__ void read_frags(const uint8_t *buf, const tile_state_t &t, int s, frags_t &f)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f.a[i] = *reinterpret_cast<const uint4 *>(buf + t.a_row + i * 32 * TKB + t.off[s]);
        f.b[i] = *reinterpret_cast<const uint4 *>(buf + t.b_row + i * 32 * TKB + t.off[s]);
    }
}

// Item 0..3: A fragment of tile row item; 4..7: B fragment of tile column item - 4.
__device__ __forceinline__ void read_frag_item(const uint8_t *buf, const tile_state_t &t, int s, int item, frags_t &f)
{
    if (item < 4)
        f.a[item] = *reinterpret_cast<const uint4 *>(buf + t.a_row + item * 32 * TKB + t.off[s]);
    else
        f.b[item - 4] = *reinterpret_cast<const uint4 *>(buf + t.b_row + (item - 4) * 32 * TKB + t.off[s]);
}

__device__ __forceinline__ void read_scales(const uint8_t *buf, const tile_state_t &t, scales_t &sc)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        sc.a[i] = *reinterpret_cast<const int *>(buf + t.sa_row + i * 32 * 8);
        sc.b[i] = *reinterpret_cast<const int *>(buf + t.sb_row + i * 32 * 8);
    }
}

// Matrix-core instructions q0 .. q1-1 (of 16: instruction q is tile row q / 4, column q % 4) of step S.
// ZC: the very first step of a tile -- the accumulator input is the constant 0, which starts the tile
// without 256 register writes per lane to clear the accumulators.
template <bool BF, int S, bool ZC>
__device__ __forceinline__ void mma_some(const frags_t &f, tile_state_t &t, int q0, int q1)
{
    const v16f zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int q = q0; q < q1; ++q) {
        const int i = q >> 2, j = q & 3;
        const v16f c = ZC ? zero : t.acc[i][j];
        if constexpr (BF) {
            t.acc[i][j] = mfma_bf16(f.a[i], f.b[j], c);
        } else {
            v8i av = {(int)f.a[i].x, (int)f.a[i].y, (int)f.a[i].z, (int)f.a[i].w, 0, 0, 0, 0};
            v8i bv = {(int)f.b[j].x, (int)f.b[j].y, (int)f.b[j].z, (int)f.b[j].w, 0, 0, 0, 0};
            t.acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, bv, c, 4, 4, S, t.sc.a[i], S, t.sc.b[j]);
        }
    }
}

// Copies d0 .. d1-1 of the 17 copies of one stage: copy 2g + o (g < 8) is row group g of slab o
// (0 = A, 1 = B), copy 16 the scales.  TBF: the stage is one of the gathered-bf16 stages, whose
// operands have their own row pitch; such a stage has no scales and copy 16 is skipped.
// `stage` is the stage's index within its tile (it decides the addresses), `buf` the LDS buffer (0 / 1).
template <bool TBF, int D0, int D1>
__device__ __forceinline__ void issue_copies(const tile_state_t &t, const copy_src_t &src, int stage, int buf)
{
    const uint32_t boff = buf * STAGE_BYTES;
    const int cs = stage - t.nbf;                      // index among the FP4 stages
    const uint32_t rp = TBF ? t.gpitch : t.pitch;      // row pitch of this stage's operands
    const uint8_t *pa = TBF ? src.gga + (int64_t)stage * TKB : src.ga + (int64_t)cs * TKB;
    const uint8_t *pb = TBF ? src.ggb + (int64_t)stage * TKB : src.gb + (int64_t)cs * TKB;
    // row group g starts 8 g rows further: a wave-uniform term that goes into the base address
    const uint32_t v_even = t.lrow * rp + t.c_even, v_odd = t.lrow * rp + t.c_odd;
#pragma unroll
    for (int d = D0; d < D1; ++d) {
        if (d == 16) {
            if constexpr (!TBF) dma16(src.gs + (int64_t)cs * t.s_stride, t.vs, t.lds_s + boff);
        } else {
            const int g = d >> 1;
            const uint32_t vo = (g & 1) ? v_odd : v_even;
            const int64_t goff = (int64_t)(8 * g) * rp;
            if (d & 1)
                dma16(pb + goff, vo, t.lds_w + boff + TM * TKB + g * 1024);
            else
                dma16(pa + goff, vo, t.lds_w + boff + g * 1024);
        }
    }
}

// The copy path of a compute unit moves about 1 KiB per 16 .. 22 cycles, so the 68 copies of a stage
// (4 waves x 17) keep it busy for most of a stage; waves that issue copies faster than that block,
// and their matrix-core instructions with them.  The copies of a stage are therefore spread over
// SPREAD matrix-core steps (4 slots per step, one after each row of instructions): the last step of
// the stage that released the buffer and the first SPREAD - 1 steps of the following stage.
constexpr int SPS = 16;                         // copy slots per matrix-core step: one after every 16 / SPS instructions
constexpr int SPREAD = 3, NSLOT = SPS * SPREAD; // the stage body wires up at most three steps
static_assert(SPREAD >= 1 && SPREAD <= 3 && 16 % SPS == 0, "copy slots are placed in the last and the first two steps");
constexpr int slot_lo(int k) { return 17 * k / NSLOT; }

template <bool TBF, int K>
__device__ __forceinline__ void issue_slot(const tile_state_t &t, const copy_src_t &src, int stage, int buf)
{
    if constexpr (K < NSLOT) issue_copies<TBF, slot_lo(K), slot_lo(K + 1)>(t, src, stage, buf);
}

// The 16 matrix-core instructions of step S on fragments f, and between them
//   - the copy slots SLOT0 .. SLOT0 + SPS - 1 of stage `which` of the tile behind `src`, into LDS buffer
//     `wbuf` (COND: whether that stage exists);
//   - the eight fragment reads of step RS of buffer rbuf into rf (RS < 0: none), one at a time behind
//     the first instructions, and after them the scales of that buffer (RSC).
// A wave issues in order, so a burst of LDS or copy instructions keeps it from feeding the matrix
// cores; single instructions fit into the shadow of the matrix-core instruction before them.
template <bool BF, int S, bool COND, bool TBF, int SLOT0, int RS, bool RSC, bool ZC = false, int U = 0>
__device__ __forceinline__ void mma_and_copies(const frags_t &f, tile_state_t &t, const copy_src_t &src, int which,
                                               int wbuf, const uint8_t *rbuf, frags_t &rf)
{
    constexpr int PER = 16 / SPS;                 // matrix-core instructions per unit
    constexpr int RUNITS = SPS < 8 ? SPS : 8;     // units that carry fragment reads
    constexpr int RPU = 8 / RUNITS;               // fragment reads per such unit
    if constexpr (U < SPS) {
        mma_some<BF, S, ZC>(f, t, U * PER, (U + 1) * PER);
        ADAHOP_PIN();
        if constexpr (RS >= 0 && U < RUNITS) {
#pragma unroll
            for (int r = 0; r < RPU; ++r) read_frag_item(rbuf, t, RS, U * RPU + r, rf);
            ADAHOP_PIN();
        }
        if constexpr (RSC && U == RUNITS) {
            read_scales(rbuf, t, t.scn);
            ADAHOP_PIN();
        }
        if constexpr (COND) {
            issue_slot<TBF, SLOT0 + U>(t, src, which, wbuf);
            ADAHOP_PIN();
        }
        mma_and_copies<BF, S, COND, TBF, SLOT0, RS, RSC, ZC, U + 1>(f, t, src, which, wbuf, rbuf, rf);
    }
}

// One pipeline stage: four matrix-core steps on the fragments of LDS buffer f % 2, f counting the stages
// of all tiles of the workgroup; l is the stage's index within its tile.
//   BF:       this stage holds gathered bf16 K-channels (else FP4 codes and scales).
//   BF1, BF2: the same for the next stage and the one after it (they decide what the copies fetch).
//   N1, N2:   that stage belongs to the NEXT tile of this workgroup (the pipeline runs on across tiles:
//             the last two stages of a tile already fetch the first two of the following one).
//   HAS_NEXT: a next stage exists.  Its copies were begun during the previous stage (or the
//             prologue) and continue during the first steps of this one.  Before the last step,
//             wait until it has landed and every wave has read its last fragments of this stage
//             (one barrier), then read its first fragments while the last step runs.
//   ISSUE:    the stage after the next exists -- its copies go into the buffer just released,
//             starting between the instructions of the last step.
//   ZC:       first stage of a tile: its first step starts the accumulators from 0.
// The body has no branches, so the order written here is the order that runs.
template <bool BF, bool BF1, bool BF2, bool HAS_NEXT, bool ISSUE, bool N1 = false, bool N2 = false, bool ZC = false>
__device__ __forceinline__ void run_stage(tile_state_t &t, const uint8_t *smem, int l, int f)
{
    const uint8_t *st = smem + (f & 1) * STAGE_BYTES;
    const uint8_t *sn = smem + ((f + 1) & 1) * STAGE_BYTES;
    const copy_src_t &src1 = N1 ? t.nxt : t.cur, &src2 = N2 ? t.nxt : t.cur;
    const int l1 = N1 ? l + 1 - t.n : l + 1, l2 = N2 ? l + 2 - t.n : l + 2;
    const int b1 = (f + 1) & 1, b2 = f & 1;
    // step j computes on the fragments read during step j - 1 and reads those of step j + 1
    mma_and_copies<BF, 0, HAS_NEXT, BF1, SPS, 1, false, ZC>(t.f0, t, src1, l1, b1, st, t.f1);
    mma_and_copies<BF, 1, HAS_NEXT, BF1, 2 * SPS, 2, false>(t.f1, t, src1, l1, b1, st, t.f0);
    mma_and_copies<BF, 2, false, false, 0, 3, false>(t.f0, t, src1, 0, 0, st, t.f1);
    if constexpr (HAS_NEXT) {
        asm volatile("s_waitcnt vmcnt(0)\n\ts_waitcnt lgkmcnt(0)" ::: "memory"); // next stage landed; my reads done
        __syncthreads();
    }
    mma_and_copies<BF, 3, ISSUE, BF2, 0, (HAS_NEXT ? 0 : -1), (HAS_NEXT && !BF1)>(t.f1, t, src2, l2, b2, sn, t.f0);
    if constexpr (HAS_NEXT && !BF1) t.sc = t.scn;
}

// All stages of one tile, f0 being the running stage count at its start.  The last two stages fetch the
// first two stages of the tile behind t.nxt.  (After its last tile a workgroup names that tile once more:
// the fetched stages are never used, and the loop needs no second variant of its body.)
// NBFC: 0 = no gathered bf16 stages; 1, 2 = that many; 3 = three or more.  A compile-time class, so that
// the body of the tile loop is one straight sequence of stages (branches that each start the accumulators
// make the register allocator spill them).
template <int NBFC> __device__ __forceinline__ void run_tile(tile_state_t &t, const uint8_t *smem, int f0)
{
    const int n = t.n;
    int l = 1;
    if constexpr (NBFC == 0) {
        run_stage<false, false, false, true, true, false, false, true>(t, smem, 0, f0);
    } else if constexpr (NBFC == 1) {
        run_stage<true, false, false, true, true, false, false, true>(t, smem, 0, f0);
    } else if constexpr (NBFC == 2) {
        run_stage<true, true, false, true, true, false, false, true>(t, smem, 0, f0);
        run_stage<true, false, false, true, true>(t, smem, 1, f0 + 1);
        l = 2;
    } else {
        run_stage<true, true, true, true, true, false, false, true>(t, smem, 0, f0);
        for (; l + 2 < t.nbf; ++l) run_stage<true, true, true, true, true>(t, smem, l, f0 + l);
        run_stage<true, true, false, true, true>(t, smem, l, f0 + l);
        run_stage<true, false, false, true, true>(t, smem, l + 1, f0 + l + 1);
        l += 2;
    }
    for (; l + 2 < n; ++l) run_stage<false, false, false, true, true>(t, smem, l, f0 + l);
    // the two stages that reach into the next tile: its stage 0 is a bf16 stage iff there are any, its
    // stage 1 iff there are two or more
    run_stage<false, false, (NBFC >= 1), true, true, false, true>(t, smem, l, f0 + l);
    run_stage<false, (NBFC >= 1), (NBFC >= 2), true, true, true, true>(t, smem, l + 1, f0 + l + 1);
}

// The accumulators of a finished tile -> C.  The two stage buffers may already hold the next tile, so the
// bf16 path, which has to transpose through LDS, uses a small patch private to the wave beyond them; LDS
// operations of one wave execute in order, so the patch needs no barrier.  For bf16 the host side
// guarantees a 16-byte aligned C and ldc % 8 == 0.
constexpr int PATCH_BYTES = 5120;                                  // per wave
constexpr int KERNEL_LDS_BYTES = TILED_LDS_BYTES + 4 * PATCH_BYTES; // 159744 of the 163840 of a compute unit

template <typename OUT>
__device__ __forceinline__ void store_tile(tile_state_t &t, uint8_t *smem, OUT *__restrict__ C, int64_t ldc, int64_t m0,
                                           int64_t n0, int w, int lane)
{
    const int l32 = lane & 31, h = lane >> 5, wm = w >> 1, wn = w & 1;
    if constexpr (sizeof(OUT) == 4) {
        // fp32: straight from the accumulator registers, 128-byte row segments (staging through LDS as below
        // and storing whole rows, 16 bytes per lane, was measured and is no faster)
        float *crow = C + (m0 + wm * 128 + h * 4) * ldc + n0 + wn * 128 + l32;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    __builtin_nontemporal_store(t.acc[i][j][r],
                                                &crow[(int64_t)(i * 32 + (r >> 2) * 8 + (r & 3)) * ldc + j * 32]);
    } else {
        // bf16: a lane converts two consecutive accumulator rows into one packed pair, trades pairs with its
        // neighbour and keeps, as one dword, two adjacent columns of one row (even lane: the low halves =
        // rows 0, 2 of each four; odd lane: the high halves = rows 1, 3).  One patch = 32 rows x 64 columns
        // (two accumulator tiles side by side: 128-byte row segments), pitch 144 bytes.
        constexpr int BP = 144;
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        OUT *cbase = C + (m0 + wm * 128) * ldc + n0 + wn * 128;
        typedef float f2 __attribute__((ext_vector_type(2)));
        typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
        uint8_t *patch = smem + TILED_LDS_BYTES + w * PATCH_BYTES;
        const int odd = lane & 1;
        // byte selector over {neighbour's pair (bytes 4-7), own pair (bytes 0-3)}
        const uint32_t sel = odd ? 0x03020706u : 0x05040100u;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int jp = 0; jp < 2; ++jp) {
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                    for (int r = 0; r < 16; r += 2) {
                        const v16f &a = t.acc[i][jp * 2 + jj];
                        const f2 pair = {a[r], a[r + 1]};
                        const uint32_t p = __builtin_bit_cast(uint32_t, __builtin_convertvector(pair, bf2)); // RNE
                        const uint32_t q = __builtin_amdgcn_update_dpp(0, p, 0xB1, 0xF, 0xF, true); // lane ^ 1's pair
                        const int row = (r >> 2) * 8 + h * 4 + (r & 3) + odd;
                        *reinterpret_cast<uint32_t *>(patch + row * BP + (jj * 32 + (l32 & ~1)) * 2) =
                            __builtin_amdgcn_perm(q, p, sel);
                    }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int prow = q * 8 + (lane >> 3);
                    const u32x4 v = *reinterpret_cast<const u32x4 *>(patch + prow * BP + (lane & 7) * 16);
                    __builtin_nontemporal_store(
                        v, reinterpret_cast<u32x4 *>(cbase + (int64_t)(i * 32 + prow) * ldc + jp * 64 + (lane & 7) * 8));
                }
            }
    }
}

// Persistent kernel: the grid has one workgroup per compute unit (or per tile, if there are fewer), and a
// workgroup walks the tile sequence with the stride of the grid.  The stage pipeline of a tile runs over
// the gathered bf16 K-channels first (OEK), then over the FP4 stages, and on into the next tile: while a
// tile's accumulators are stored, the first two stages of the next one are already in LDS or on the way.
// Host side guarantees K >= 512 (two FP4 stages), so that every bf16 stage has two successors and the
// last two stages of a tile are FP4 stages, and at least three stages per tile (K >= 768 when there are
// no bf16 stages).
template <bool OEK, typename OUT>
__global__ __launch_bounds__(256) void k_gemm_mx_tile256(int64_t K, const uint8_t *__restrict__ a_codes,
                                                         const uint8_t *__restrict__ a_scales_sm,
                                                         const uint8_t *__restrict__ b_codes,
                                                         const uint8_t *__restrict__ b_scales_sm, int64_t M, int64_t N,
                                                         OUT *__restrict__ C, int64_t ldc,
                                                         const uint16_t *__restrict__ Ag,
                                                         const uint16_t *__restrict__ Bg, int kpad, int tiles_m,
                                                         int tiles_n, int group_m, int order)
{
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w >> 1, wn = w & 1;
    const int ntiles = tiles_m * tiles_n;
    const int grid = (int)gridDim.x;

    // Position v of the walk -> tile.  Consecutive workgroup ids land on different XCDs (8 of them, each
    // with its own L2) and the grid is a multiple of 8 whenever it is smaller than the tile count, so v % 8
    // is the XCD of every tile of a workgroup.  The operand with more tiles is the "major" one (order bit 1: B,
    // else A); the other is what the XCDs share.
    //   order bit 0 clear: every XCD gets a contiguous run of the tile sequence, ordered in bands of group_m major
    //     tiles (rows of tiles for A), so that the 32 tiles an XCD runs at a time share 8 + 4 panels, and an XCD keeps
    //     its bands of the major operand to itself.
    //   order bit 0 set (host side: a grid of 256, major tiles % 8 == 0, minor tiles % 32 == 0): the 256 tiles that run
    //     at a time are 8 major x 32 minor tiles -- XCD x takes minor tiles 4x .. 4x+3 of them -- and the walk sweeps the
    //     groups of 32 minor tiles before it moves to the next band of 8.  For a major operand of which the XCD-contiguous
    //     order would keep more in use than stays in the Infinity Cache: a band of it is fetched from HBM once.
    auto tile_origin = [&](int v, int64_t &m0, int64_t &n0) {
        const bool b_major = (order & 2) != 0;
        const int t_major = b_major ? tiles_n : tiles_m, t_minor = b_major ? tiles_m : tiles_n;
        int major, minor;
        if (order & 1) {
            const int x = v & 7, s = (v >> 3) & 31, round = v >> 8, groups = t_minor >> 5;
            major = (round / groups) * 8 + (s & 7);
            minor = (round % groups) * 32 + 4 * x + (s >> 3);
        } else {
            int tix = v;
            if (ntiles % 8 == 0) tix = (v & 7) * (ntiles >> 3) + (v >> 3);
            const int gm = min(group_m, t_major);
            const int band = gm * t_minor;
            const int first = (tix / band) * gm;
            const int gsz = min(gm, t_major - first);
            major = first + (tix % band) % gsz;
            minor = (tix % band) / gsz;
        }
        m0 = (int64_t)(b_major ? minor : major) * TM;
        n0 = (int64_t)(b_major ? major : minor) * TN;
    };

    tile_state_t t;
    // ---- copy engine: wave w moves rows [64w, 64w+64) of both slabs, 8 rows per instruction.
    // Lane i of instruction g writes LDS row 8g + i/8, chunk position i%8, which must hold logical
    // chunk (i%8) ^ ((row/2) & 7) = (i%8) ^ (4*(g&1) + i/16).
    t.lrow = lane >> 3;
    t.c_even = ((lane & 7) ^ (lane >> 4)) * 16;
    t.c_odd = t.c_even ^ 64;
    t.pitch = (uint32_t)(K >> 1);
    t.gpitch = (uint32_t)kpad * 2;
    t.vs = lane * 16;
    t.s_stride = (w < 2 ? M : N) * 8;
    {
        const uint32_t smem_base = __builtin_amdgcn_readfirstlane(lds_address(smem));
        t.lds_w = smem_base + w * 64 * TKB;
        t.lds_s = smem_base + SLAB_BYTES + w * 1024;
    }
    t.nbf = OEK ? (kpad >> 6) : 0;
    t.n = t.nbf + (int)(K >> 8);
    auto tile_source = [&](int64_t m0, int64_t n0) {
        const int64_t pitch = t.pitch, gpitch = t.gpitch;
        copy_src_t c;
        c.ga = uniform_ptr(a_codes + (m0 + w * 64) * pitch);
        c.gb = uniform_ptr(b_codes + (n0 + w * 64) * pitch);
        c.gga = uniform_ptr(reinterpret_cast<const uint8_t *>(Ag) + (m0 + w * 64) * gpitch);
        c.ggb = uniform_ptr(reinterpret_cast<const uint8_t *>(Bg) + (n0 + w * 64) * gpitch);
        // scales (stage-major): waves 0,1 move the two 1 KiB halves of the A slab's scales, waves 2,3 of B's
        c.gs = uniform_ptr(w < 2 ? a_scales_sm + (m0 + w * 128) * 8 : b_scales_sm + (n0 + (w - 2) * 128) * 8);
        return c;
    };

    // ---- fragment reads: row l32 (+32 i) of the wave's slab, logical chunk 4h + s
    {
        const int rx = (l32 >> 1) & 7;
#pragma unroll
        for (int s = 0; s < 4; ++s) t.off[s] = ((4 * h + s) ^ rx) * 16;
        t.a_row = (wm * 128 + l32) * TKB;
        t.b_row = TM * TKB + (wn * 128 + l32) * TKB;
        t.sa_row = SLAB_BYTES + (wm * 128 + l32) * 8 + 4 * h;
        t.sb_row = SLAB_BYTES + TM * 8 + (wn * 128 + l32) * 8 + 4 * h;
    }

#pragma unroll
    for (int i = 0; i < 4; ++i) t.sc.a[i] = t.sc.b[i] = t.scn.a[i] = t.scn.b[i] = 0;

    int v = blockIdx.x;
    int64_t m0, n0;
    tile_origin(v, m0, n0);
    t.cur = tile_source(m0, n0);
    t.nxt = t.cur;

    // prologue: stage 0 of the first tile copied and landed, the first slots of its stage 1 under way
    // (the rest of stage 1 follows during stage 0, as in every later stage), first fragments of stage 0 read.
    constexpr int PRO = slot_lo(SPS); // copies of the slots that fall into the step before a stage
    if constexpr (OEK) {
        issue_copies<true, 0, 17>(t, t.cur, 0, 0);
        if (t.nbf > 1)
            issue_copies<true, 0, PRO>(t, t.cur, 1, 1);
        else
            issue_copies<false, 0, PRO>(t, t.cur, 1, 1);
    } else {
        issue_copies<false, 0, 17>(t, t.cur, 0, 0);
        issue_copies<false, 0, PRO>(t, t.cur, 1, 1);
    }
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PRO) : "memory");
    __syncthreads();
    read_frags(smem, t, 0, t.f0);
    if constexpr (!OEK) read_scales(smem, t, t.sc);

    auto walk = [&](auto nbfc) {
        for (int f = 0;; f += t.n) {
            const int vn = v + grid;
            const bool more = vn < ntiles; // same for the whole workgroup
            int64_t m0n, n0n;
            tile_origin(more ? vn : v, m0n, n0n);
            t.nxt = tile_source(m0n, n0n);
            run_tile<decltype(nbfc)::value>(t, smem, f);
            store_tile(t, smem, C, ldc, m0, n0, w, lane);
            if (!more) break;
            v = vn;
            m0 = m0n;
            n0 = n0n;
            t.cur = t.nxt;
        }
    };
    if constexpr (!OEK)
        walk(std::integral_constant<int, 0>{});
    else if (t.nbf == 1)
        walk(std::integral_constant<int, 1>{});
    else if (t.nbf == 2)
        walk(std::integral_constant<int, 2>{});
    else
        walk(std::integral_constant<int, 3>{});
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); // the copies begun for a tile that does not follow
}

} // namespace


size_t gemm_mx_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    return align_up((size_t)M * (K / 32), 256) + align_up((size_t)N * (K / 32), 256);
}

// Which part of the product the tiled kernel takes: whole 256x256 tiles (rows [0, Mi), columns [0, Ni)), or
// nothing.  At least three pipeline stages are needed (64 gathered channels or 256 K-elements each, two of
// them FP4 stages); the bf16 epilogue stores 16 bytes per lane.
static std::atomic<int> g_kernel_choice{0};
static std::atomic<int> g_force_walk{-1}; // -1: the order of the tile walk chosen by shape; 0 .. 3: forced

void gemm_mx_force_kernel(int which)
{
    g_kernel_choice.store(which <= 2 ? which : 0);
    g_force_walk.store(which >= 3 ? which - 3 : -1);
}

// Which tiled kernel takes a product (fp32 C, no gathered K-channels; otherwise always the 256 x 256 kernel).  The
// 256 x 128 kernel with two accumulator sets hides the C stores behind the next tile but moves 1.5 times the operand
// bytes per flop from L2 into LDS and out of LDS; measured on MI355X it wins where the stores are a large part of a
// tile's time -- K = 2048: 1.2x; K = 4096: 1.04 .. 1.13x up to about 90 M elements of C, 0.97x at 8192 x 12288 -- and
// loses 4 .. 15 % from K = 8192 on, except where the 256 x 256 tiles fill the last round of the compute units badly
// (14336 x 4096: 896 tiles on 256 units, 3.5 rounds; 1.1x with 7 rounds of the smaller tiles).
static bool takes_dual_kernel(int64_t M, int64_t N, int64_t K, int kpad, int c_bf16)
{
    if (c_bf16 || kpad > 0 || !gemm_mx_dual_eligible(M, N, K)) return false;
    const int forced = g_kernel_choice.load();
    if (forced == 1) return false;
    if (forced == 2) return true;
    if (K <= 2048) return true;
    if (K <= 4096) return M * N <= (int64_t)8192 * 11008;
    const double units = 256.0, t256 = (double)(M / 256) * (double)(N / 256), t128 = (double)(M / 256) * (double)(N / 128);
    if (t256 < 1.0) return true; // N in [128, 256): only the smaller tile exists
    const double waste256 = std::ceil(t256 / units) * units / t256, waste128 = std::ceil(t128 / units) * units / t128;
    return waste256 >= 1.10 && waste128 + 0.08 <= waste256;
}

void gemm_mx_tiled_part(int64_t M, int64_t N, int64_t K, int kpad, const uint8_t *a_scales, const uint8_t *b_scales,
                        const void *C, int64_t ldc, int c_bf16, int64_t *Mi, int64_t *Ni)
{
    const bool fast_c = !c_bf16 || (aligned(C, 16) && ldc % 8 == 0);
    const bool fast_k = fast_c && K % 256 == 0 && K >= (kpad > 0 ? 512 : 768) && kpad % 64 == 0 &&
                        aligned(a_scales, 8) && aligned(b_scales, 8);
    const int64_t tn = fast_k && takes_dual_kernel(M, N, K, kpad, c_bf16) ? 128 : TN;
    *Mi = fast_k ? M / TM * TM : 0;
    *Ni = fast_k ? N / tn * tn : 0;
    if (*Mi == 0 || *Ni == 0 || (*Mi / TM) * (*Ni / tn) >= (1 << 30)) *Mi = *Ni = 0;
}

uint8_t *gemm_mx_scales_sm(void *workspace, int64_t M, int64_t K, int which)
{
    uint8_t *a_sm = static_cast<uint8_t *>(workspace);
    return which == 0 ? a_sm : a_sm + align_up((size_t)M * (K / 32), 256);
}

// Once per device: the compute-unit count, and for every instance of the tiled kernel the LDS size (more than a
// launch may ask for by default).  Host-side calls, nothing queued.
int configure_gemm_mx(int *ncu_out)
{
    static device_once_t once;
    static std::atomic<int> cu_count[64];
    int dev = 0;
    int rc = check_hip(hipGetDevice(&dev));
    if (rc != ADAHOP_OK) return rc;
    int ncu = dev >= 0 && dev < 64 ? cu_count[dev].load(std::memory_order_relaxed) : 0;
    if (once.need(dev) || ncu == 0) {
        rc = check_hip(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
        if (rc != ADAHOP_OK) return rc;
        const void *kernels[4] = {reinterpret_cast<const void *>(&k_gemm_mx_tile256<false, float>),
                                  reinterpret_cast<const void *>(&k_gemm_mx_tile256<true, float>),
                                  reinterpret_cast<const void *>(&k_gemm_mx_tile256<false, uint16_t>),
                                  reinterpret_cast<const void *>(&k_gemm_mx_tile256<true, uint16_t>)};
        for (const void *f : kernels) {
            rc = check_hip(hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, KERNEL_LDS_BYTES));
            if (rc != ADAHOP_OK) return rc;
        }
        if (dev >= 0 && dev < 64) cu_count[dev].store(ncu, std::memory_order_relaxed);
        once.mark(dev);
    }
    if (ncu_out) *ncu_out = ncu;
    return ADAHOP_OK;
}

namespace {

template <typename OUT>
int launch_gemm_mx_t(int64_t M, int64_t N, int64_t K, const uint8_t *a_codes, const uint8_t *a_scales,
                     const uint8_t *b_codes, const uint8_t *b_scales, OUT *C, int64_t ldc, const uint16_t *Ag,
                     const uint16_t *Bg, int kpad, void *workspace, int sm_ready, hipStream_t st)
{
    if (M == 0 || N == 0) return ADAHOP_OK;
    auto generic = [&](int64_t m, int64_t n, const uint8_t *ac, const uint8_t *as, const uint8_t *bc, const uint8_t *bs,
                       OUT *c, const uint16_t *ag, const uint16_t *bg) {
        dim3 grid((unsigned)ceil_div(n, 128), (unsigned)ceil_div(m, 128));
        hipLaunchKernelGGL((k_gemm_mx_generic<false, OUT>), grid, dim3(256), 0, st, m, n, K, ac, as, bc, bs, c, ldc, ag, bg,
                           kpad);
        return check_launch();
    };
    // The tiled kernel takes the whole 256x256 tiles; ragged edges (and shapes it cannot take at all) go to
    // the bounds-checked kernel.
    int64_t Mi, Ni;
    gemm_mx_tiled_part(M, N, K, kpad, a_scales, b_scales, C, ldc, sizeof(OUT) == 2, &Mi, &Ni);
    if (Mi == 0) return generic(M, N, a_codes, a_scales, b_codes, b_scales, C, Ag, Bg);

    int ncu = 0;
    const int rc0 = configure_gemm_mx(&ncu); // once per device: the compute-unit count and the kernels' LDS size
    if (rc0 != ADAHOP_OK) return rc0;
    ncu = ncu / 8 * 8; // keep a workgroup's tiles on one XCD
    if (ncu < 8) ncu = 8;
    // scales of the tiled part, stage-major, in the caller's workspace (sm_ready bit 0 / 1: the quantiser of A / B
    // has already written them there)
    uint8_t *a_sm = gemm_mx_scales_sm(workspace, M, K, 0), *b_sm = gemm_mx_scales_sm(workspace, M, K, 1);
    const int64_t KB8 = K / 256;
    if (!(sm_ready & 1))
        hipLaunchKernelGGL(k_stage_major_scales, dim3((unsigned)ceil_div(Mi * KB8, 256)), dim3(256), 0, st,
                           reinterpret_cast<const uint64_t *>(a_scales), reinterpret_cast<uint64_t *>(a_sm), Mi, KB8);
    if (!(sm_ready & 2))
        hipLaunchKernelGGL(k_stage_major_scales, dim3((unsigned)ceil_div(Ni * KB8, 256)), dim3(256), 0, st,
                           reinterpret_cast<const uint64_t *>(b_scales), reinterpret_cast<uint64_t *>(b_sm), Ni, KB8);
    int rc = check_launch();
    if (rc != ADAHOP_OK) return rc;
    const int tiles_m = (int)(Mi / TM), tiles_n = (int)(Ni / TN);
    const int group_m = 8;
    // one workgroup per compute unit walks the tiles (each workgroup fills a compute unit's LDS and registers)
    const int ntiles = tiles_m * tiles_n;
    const dim3 grid((unsigned)(ntiles < ncu ? ntiles : ncu));
    // The order of the walk (see the kernel), as measured on MI355X with the same flops each:
    //  - bands along the operand with more tiles, in XCD-contiguous runs.  The XCDs keep their bands of it to
    //    themselves and share the other one, which is smaller and stays in the 256 MB Infinity Cache:
    //    8192 x 28672 x 16384 takes 1.60 ms in bands of B against 1.74 ms in bands of A (each panel of the 235 MB B is
    //    then asked for by four XCDs at once, before the cache has it), and 28672 x 8192 x 16384 1.60 against 1.70 ms
    //    the other way round; 8192 x 16384 x 28672: 1.64 (bands of B) against 1.72 ms;
    //  - in such runs the eight XCDs work on up to 64 bands' worth of major tiles at a time and come back to them
    //    once per round: when that much of a packed A does not stay in the cache (and B would), bands of A swept over
    //    all of B fetch A from HBM once instead -- 16384 x 8192 x 28672 (235 MB of A in use at a time): 1.65 against
    //    1.69 .. 1.79 ms by machine.  (The mirrored sweep, bands of B over A, exists and gives the same bits but is
    //    not chosen: on the mirrored shape the contiguous runs are faster, 1.64 against 1.72 ms.)
    constexpr int64_t STAYS = 192ll << 20;
    const bool b_major = tiles_n > tiles_m;
    const int64_t a_in_use = (int64_t)(tiles_m < 64 ? tiles_m : 64) * TM * (K / 2);
    const bool sweep_a = !b_major && a_in_use > STAYS && Ni * (K / 2) <= STAYS && grid.x == 256 && tiles_m % 8 == 0 &&
                         tiles_n % 32 == 0;
    int order = b_major ? 2 : sweep_a ? 1 : 0;
    const int forced = g_force_walk.load();
    if (forced >= 0) {
        const bool fb = (forced & 2) != 0;
        const bool ok = !(forced & 1) || (grid.x == 256 && (fb ? tiles_n : tiles_m) % 8 == 0 && (fb ? tiles_m : tiles_n) % 32 == 0);
        order = ok ? forced : (forced & 2);
    }
    if constexpr (sizeof(OUT) == 4) {
        if (takes_dual_kernel(M, N, K, kpad, 0)) {
            rc = launch_gemm_mx_dual(Mi, Ni, K, a_codes, a_sm, b_codes, b_sm, reinterpret_cast<float *>(C), ldc, st);
            goto edges;
        }
    }
    if (kpad > 0)
        hipLaunchKernelGGL((k_gemm_mx_tile256<true, OUT>), grid, dim3(256), KERNEL_LDS_BYTES, st, K, a_codes, a_sm, b_codes,
                           b_sm, Mi, Ni, C, ldc, Ag, Bg, kpad, tiles_m, tiles_n, group_m, order);
    else
        hipLaunchKernelGGL((k_gemm_mx_tile256<false, OUT>), grid, dim3(256), KERNEL_LDS_BYTES, st, K, a_codes, a_sm, b_codes,
                           b_sm, Mi, Ni, C, ldc, Ag, Bg, kpad, tiles_m, tiles_n, group_m, order);
    rc = check_launch();
edges:
    if (rc != ADAHOP_OK) return rc;
    if (Mi < M) { // bottom strip: rows [Mi, M), all columns
        rc = generic(M - Mi, N, a_codes + Mi * (K / 2), a_scales + Mi * (K / 32), b_codes, b_scales, C + Mi * ldc,
                     Ag ? Ag + Mi * kpad : nullptr, Bg);
        if (rc != ADAHOP_OK) return rc;
    }
    if (Ni < N) // right strip: rows [0, Mi), columns [Ni, N)
        rc = generic(Mi, N - Ni, a_codes, a_scales, b_codes + Ni * (K / 2), b_scales + Ni * (K / 32), C + Ni, Ag,
                     Bg ? Bg + Ni * kpad : nullptr);
    return rc;
}

} // namespace

int launch_gemm_mx(int64_t M, int64_t N, int64_t K, const uint8_t *a_codes, const uint8_t *a_scales,
                   const uint8_t *b_codes, const uint8_t *b_scales, void *C, int64_t ldc, int c_bf16, const uint16_t *Ag,
                   const uint16_t *Bg, int kpad, void *workspace, hipStream_t st, int sm_ready)
{
    if (c_bf16)
        return launch_gemm_mx_t(M, N, K, a_codes, a_scales, b_codes, b_scales, static_cast<uint16_t *>(C), ldc, Ag, Bg,
                                kpad, workspace, sm_ready, st);
    return launch_gemm_mx_t(M, N, K, a_codes, a_scales, b_codes, b_scales, static_cast<float *>(C), ldc, Ag, Bg, kpad,
                            workspace, sm_ready, st);
}

int launch_oe_k_accumulate(int64_t M, int64_t N, const uint16_t *Ag, const uint16_t *Bg, int kpad, float *C,
                           int64_t ldc, hipStream_t st)
{
    if (M == 0 || N == 0 || kpad == 0) return ADAHOP_OK;
    dim3 grid((unsigned)ceil_div(N, 128), (unsigned)ceil_div(M, 128));
    hipLaunchKernelGGL((k_gemm_mx_generic<true, float>), grid, dim3(256), 0, st, M, N, (int64_t)0, nullptr, nullptr, nullptr,
                       nullptr, C, ldc, Ag, Bg, kpad);
    return check_launch();
}

} // namespace adahop
