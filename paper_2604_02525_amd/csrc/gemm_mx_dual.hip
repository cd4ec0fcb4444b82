// Block-scaled FP4 GEMM (the MXFP4 term of paper Eq. 4 / 5 / 7 / 8), variant for products whose C traffic is
// large next to their matrix-core time (short and medium K): 256 x 128 tiles of C and TWO accumulator sets per
// wave, so that the C stores of a finished tile are issued between the matrix-core instructions of the next one
// instead of holding the matrix cores up.
//
//   C[m, n] = sum_blk 2^(sa[m,blk]-127) 2^(sb[n,blk]-127) sum_{i<32} a[m,32blk+i] b[n,32blk+i]       (fp32 C)
//
// Same instruction, operand layout and LDS slab layout as the 256 x 256 kernel (gemm_mx.hip).  Differences:
//   - a workgroup (4 waves, 2 x 2) computes a 256 x 128 tile; a wave owns 128 x 64 = 4 x 2 matrix-core tiles,
//     128 fp32 accumulators per lane and set; tile t of a workgroup accumulates into set t % 2;
//   - while tile t is computed, the 128 stores per lane of tile t - 1 (the other set) are issued one after a
//     matrix-core instruction each, during the first 8 pipeline stages of tile t (16 stores per stage: one
//     32 x 32 accumulator tile); the product therefore needs K >= 2048 (8 stages of 256 K-elements);
//   - a stage is 256 K-elements of the 256 A rows and 128 B rows (48 KiB) plus their scales (3 KiB); THREE
//     stages rotate in LDS, copies run two to three stages ahead of the matrix cores.  A wave waits for its
//     own copies with a counted wait: vector memory operations of a wave complete in the order issued, so
//     "at most X outstanding" with X = the number of copies and stores issued after the last copy of the
//     stage that is needed next means that stage has landed, without waiting for the younger copies or for
//     the C stores;
//   - one barrier per stage, before its last matrix-core step, as in the 256 x 256 kernel: every wave has read
//     its last fragments of the stage by then (so its buffer may be refilled: it is the target of the copies
//     three stages ahead) and the next stage has landed.
#include "common.h"
#include "gemm_mx_common.h"

namespace adahop {

namespace {

namespace dual {

constexpr int TM = 256, TN = 128, TKB = 128, NBUF = 3;
constexpr int A_SLAB = TM * TKB, B_SLAB = TN * TKB;
constexpr int SA_OFF = A_SLAB + B_SLAB, SB_OFF = SA_OFF + TM * 8, STAGE_BYTES = SB_OFF + TN * 8;
constexpr int LDS_BYTES = NBUF * STAGE_BYTES; // 156672 of the 163840 of a compute unit
constexpr int NCOPY = 13;                     // copies per wave and stage: 8 of A, 4 of B, 1 of scales
constexpr int PART1 = 4;                      // of which issued in the last step of a stage, the rest in the next three
constexpr int STORE_STAGES = 8;               // stages of a tile that carry the stores of the previous tile
constexpr int STORES_PER_STAGE = 16;

struct frags_t {
    uint4 a[4], b[2];
};

struct scales_t {
    int a[4], b[2];
};

// Wave-uniform bases of this wave's share of stage 0 of a tile.
struct src_t {
    const uint8_t *ga, *gb, *gs;
};

struct state_t {
    v16f acc[2][4][2];
    frags_t f0, f1;
    scales_t sc, scn;
    int a_row, b_row, sa_row, sb_row, off[4]; // fragment reads: byte offsets inside a stage buffer
    // copy cursor: the stage being fetched, two to three stages ahead of the one being computed
    const uint8_t *pa, *pb, *ps;
    int left;          // stages of the cursor's tile that are not yet completely issued
    uint32_t cbuf;     // byte offset of the cursor's LDS buffer
    src_t nxt;         // the tile after the cursor's
    int n;             // stages per tile
    uint32_t v_even, v_odd, vs, pitch;
    int64_t s_stride;
    uint32_t lds_a, lds_b, lds_s; // LDS addresses, in buffer 0, of the rows this wave copies
};

__device__ __forceinline__ uint32_t next_buf(uint32_t off) { return off == (NBUF - 1) * STAGE_BYTES ? 0u : off + STAGE_BYTES; }

// Copies D0 .. D1-1 of the cursor's stage: 0..7 row groups of A (8 rows each), 8..11 row groups of B, 12 scales.
template <int D0, int D1> __device__ __forceinline__ void issue(const state_t &t)
{
#pragma unroll
    for (int d = D0; d < D1; ++d) {
        if (d < 8) {
            dma16(t.pa + (int64_t)(8 * d) * t.pitch, (d & 1) ? t.v_odd : t.v_even, t.lds_a + t.cbuf + d * 1024);
        } else if (d < 12) {
            const int g = d - 8;
            dma16(t.pb + (int64_t)(8 * g) * t.pitch, (g & 1) ? t.v_odd : t.v_even, t.lds_b + t.cbuf + g * 1024);
        } else {
            dma16(t.ps, t.vs, t.lds_s + t.cbuf);
        }
    }
}

// Moves the cursor to the next stage (of the same tile, or stage 0 of the tile behind t.nxt).  Written with selects
// on scalar values, not a branch: a branch would end the basic block in the middle of a tile, and the compiler then
// sinks the matrix-core instructions of the finished block, whose results are only used later, down into the next
// block -- out of the places between the copies, reads and stores that they were written into.
__device__ __forceinline__ const uint8_t *pick(bool c, const uint8_t *a, const uint8_t *b)
{
    return reinterpret_cast<const uint8_t *>(c ? reinterpret_cast<uintptr_t>(a) : reinterpret_cast<uintptr_t>(b));
}

__device__ __forceinline__ void advance(state_t &t)
{
    const bool wrap = t.left == 1;
    t.pa = pick(wrap, t.nxt.ga, t.pa + TKB);
    t.pb = pick(wrap, t.nxt.gb, t.pb + TKB);
    t.ps = pick(wrap, t.nxt.gs, t.ps + t.s_stride);
    t.left = wrap ? t.n : t.left - 1;
    t.cbuf = next_buf(t.cbuf);
}

// Item 0..3: A fragment of tile row item; 4, 5: B fragment of tile column item - 4.
__device__ __forceinline__ void read_item(const uint8_t *buf, const state_t &t, int s, int item, frags_t &f)
{
    if (item < 4)
        f.a[item] = *reinterpret_cast<const uint4 *>(buf + t.a_row + item * 32 * TKB + t.off[s]);
    else
        f.b[item - 4] = *reinterpret_cast<const uint4 *>(buf + t.b_row + (item - 4) * 32 * TKB + t.off[s]);
}

__device__ __forceinline__ void read_scales(const uint8_t *buf, const state_t &t, scales_t &sc)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) sc.a[i] = *reinterpret_cast<const int *>(buf + t.sa_row + i * 32 * 8);
#pragma unroll
    for (int j = 0; j < 2; ++j) sc.b[j] = *reinterpret_cast<const int *>(buf + t.sb_row + j * 32 * 8);
}

// Store r of accumulator tile ST (tile row ST / 2, column ST % 2) of set SET; cprev is the lane's pointer to
// C[tile row 4 * (lane / 32)][lane % 32] of the wave's 128 x 64 part of that tile.
template <int SET, int ST> __device__ __forceinline__ void store_one(const state_t &t, float *cprev, int64_t ldc, int r)
{
    constexpr int i = ST >> 1, j = ST & 1;
    __builtin_nontemporal_store(t.acc[SET][i][j][r], &cprev[(int64_t)(i * 32 + (r >> 2) * 8 + (r & 3)) * ldc + j * 32]);
}

// One matrix-core step (8 instructions on fragments f, step S of the stage, into set SET) and, one after each
// instruction: the fragment reads of step RS of buffer rbuf into rf (RS < 0: none; RSC: then the scales of that
// buffer), the copies C0 .. C1-1 of the cursor's stage, the stores R0 .. R1-1 of accumulator tile ST of the
// other set (ST < 0: none).  A wave issues in order and is alone on its SIMD: single instructions fit into the
// shadow of the matrix-core instruction before them, bursts would hold the matrix core up.  Written as a
// compile-time recursion over the instruction index Q (no loop: the order written is the order that runs).
template <int SET, int S, bool ZC, int RS, bool RSC, int C0, int C1, int ST, int R0, int R1, int Q = 0>
__device__ __forceinline__ void step(const frags_t &f, state_t &t, const uint8_t *rbuf, frags_t &rf, float *cprev,
                                     int64_t ldc)
{
    if constexpr (Q < 8) {
        constexpr int i = Q >> 1, j = Q & 1, NC = C1 - C0;
        const v16f zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
        const v16f c = ZC ? zero : t.acc[SET][i][j];
        v8i av = {(int)f.a[i].x, (int)f.a[i].y, (int)f.a[i].z, (int)f.a[i].w, 0, 0, 0, 0};
        v8i bv = {(int)f.b[j].x, (int)f.b[j].y, (int)f.b[j].z, (int)f.b[j].w, 0, 0, 0, 0};
        t.acc[SET][i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, bv, c, 4, 4, S, t.sc.a[i], S, t.sc.b[j]);
        ADAHOP_PIN();
        if constexpr (RS >= 0 && Q < 6) {
            read_item(rbuf, t, RS, Q, rf);
            ADAHOP_PIN();
        }
        if constexpr (RSC && Q == 6) {
            read_scales(rbuf, t, t.scn);
            ADAHOP_PIN();
        }
        if constexpr (NC > 0) {
            // NC copies spread over the 8 slots: slot Q carries copy k0 iff floor(Q NC / 8) < floor((Q + 1) NC / 8)
            constexpr int k0 = (Q * NC) / 8, k1 = ((Q + 1) * NC) / 8;
            if constexpr (k1 > k0) {
                issue<C0 + k0, C0 + k0 + 1>(t);
                ADAHOP_PIN();
            }
        }
        if constexpr (ST >= 0 && R0 + Q < R1 && Q < 6) {
            store_one<1 - SET, ST>(t, cprev, ldc, R0 + Q);
            ADAHOP_PIN();
        }
        step<SET, S, ZC, RS, RSC, C0, C1, ST, R0, R1, Q + 1>(f, t, rbuf, rf, cprev, ldc);
    }
}

// One pipeline stage: four matrix-core steps on the fragments of the LDS buffer at byte offset rb (advanced to
// the next buffer on return).  ST: the accumulator tile of the previous tile's set stored during this stage
// (-1: none).  ZC: first stage of a tile (its first step starts the accumulators from 0).
template <int SET, int ST, bool ZC>
__device__ __forceinline__ void run_stage(state_t &t, const uint8_t *smem, uint32_t &rb, float *cprev, int64_t ldc)
{
    const uint8_t *st = smem + rb;
    const uint32_t rn = next_buf(rb);
    const uint8_t *sn = smem + rn;
    // the copies of a stage: PART1 during the last step of the stage two before it (after that stage's barrier),
    // the rest during the first three steps of the stage before it
    step<SET, 0, ZC, 1, false, PART1, PART1 + 3, ST, 0, 6>(t.f0, t, st, t.f1, cprev, ldc);
    step<SET, 1, false, 2, false, PART1 + 3, PART1 + 6, ST, 6, 11>(t.f1, t, st, t.f0, cprev, ldc);
    step<SET, 2, false, 3, false, PART1 + 6, NCOPY, ST, 11, 16>(t.f0, t, st, t.f1, cprev, ldc);
    advance(t);
    // Younger than the last copy of the next stage: the NCOPY copies of the stage after it and this stage's stores.
    constexpr int X = NCOPY + (ST >= 0 ? STORES_PER_STAGE : 0);
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier" ::"n"(X) : "memory");
    step<SET, 3, false, 0, true, 0, PART1, -1, 0, 0>(t.f1, t, sn, t.f0, cprev, ldc);
    t.sc = t.scn;
    rb = rn;
}

template <int SET, int ST> __device__ __forceinline__ void store_stages(state_t &t, const uint8_t *smem, uint32_t &rb, float *cprev, int64_t ldc)
{
    if constexpr (ST < STORE_STAGES) {
        run_stage<SET, ST, ST == 0>(t, smem, rb, cprev, ldc);
        store_stages<SET, ST + 1>(t, smem, rb, cprev, ldc);
    }
}

// All stages of one tile into set SET; STORES: the other set holds a finished tile, whose stores go along.
template <int SET, bool STORES>
__device__ __forceinline__ void run_tile(state_t &t, const uint8_t *smem, uint32_t &rb, float *cprev, int64_t ldc)
{
    int l;
    if constexpr (STORES) {
        store_stages<SET, 0>(t, smem, rb, cprev, ldc);
        l = STORE_STAGES;
    } else {
        run_stage<SET, -1, true>(t, smem, rb, cprev, ldc);
        l = 1;
    }
    for (; l < t.n; ++l) run_stage<SET, -1, false>(t, smem, rb, cprev, ldc);
}

template <int SET> __device__ __forceinline__ void store_all(const state_t &t, float *c, int64_t ldc)
{
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                __builtin_nontemporal_store(t.acc[SET][i][j][r], &c[(int64_t)(i * 32 + (r >> 2) * 8 + (r & 3)) * ldc + j * 32]);
}

} // namespace dual

// Persistent kernel, one workgroup per compute unit walking the tile sequence with the stride of the grid.
// M % 256 == 0, N % 128 == 0, K % 256 == 0, K >= 2048 (host side).
__global__ __launch_bounds__(256) void k_gemm_mx_dual(int64_t K, const uint8_t *__restrict__ a_codes,
                                                      const uint8_t *__restrict__ a_scales_sm,
                                                      const uint8_t *__restrict__ b_codes,
                                                      const uint8_t *__restrict__ b_scales_sm, int64_t M, int64_t N,
                                                      float *__restrict__ C, int64_t ldc, int tiles_m, int tiles_n,
                                                      int group_m)
{
    using namespace dual;
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w >> 1, wn = w & 1;
    const int ntiles = tiles_m * tiles_n;
    const int grid = (int)gridDim.x;

    // position v of the walk -> tile (XCD-contiguous runs, bands of group_m tile rows; see the 256 x 256 kernel).
    // The XCDs advance through their bands at the same pace; each starts its bands at a different tile column
    // (an eighth of the width further per XCD), so that the C rows being written at any moment are spread over the
    // whole row width -- with a power-of-two leading dimension all rows of a tile column fall on the same few
    // memory channels, and eight XCDs storing the same columns at once queue up on them.
    auto tile_origin = [&](int v, int64_t &m0, int64_t &n0) {
        int tix = v, shift = 0;
        const int band = group_m * tiles_n;
        if (ntiles % 8 == 0) {
            tix = (v & 7) * (ntiles >> 3) + (v >> 3);
            // (only when an XCD's run consists of whole bands: a band shared by two XCDs must keep one column order)
            if ((ntiles >> 3) % band == 0) shift = (v & 7) * (tiles_n >> 3);
        }
        const int first_m = (tix / band) * group_m;
        const int gsz = min(group_m, tiles_m - first_m);
        int tn = (tix % band) / gsz + shift;
        if (tn >= tiles_n) tn -= tiles_n;
        m0 = (int64_t)(first_m + (tix % band) % gsz) * TM;
        n0 = (int64_t)tn * TN;
    };

    state_t t;
    // copy engine: wave w moves rows [64w, 64w+64) of the A slab and [32w, 32w+32) of the B slab, 8 rows per
    // instruction; lane i of a row group writes LDS row i/8, chunk position i%8, which holds logical chunk
    // (i%8) ^ ((row/2) & 7) = (i%8) ^ (4 * (group & 1) + i/16)
    t.pitch = (uint32_t)(K >> 1);
    {
        const uint32_t lrow = lane >> 3, c_even = ((lane & 7) ^ (lane >> 4)) * 16;
        t.v_even = lrow * t.pitch + c_even;
        t.v_odd = lrow * t.pitch + (c_even ^ 64);
    }
    t.vs = lane * 16;
    t.s_stride = (w < 2 ? M : N) * 8;
    {
        const uint32_t base = __builtin_amdgcn_readfirstlane(lds_address(smem));
        t.lds_a = base + w * 64 * TKB;
        t.lds_b = base + A_SLAB + w * 32 * TKB;
        t.lds_s = base + (w == 0 ? SA_OFF : (w == 1 ? SA_OFF + 1024 : SB_OFF)); // waves 2 and 3 both bring B's scales
    }
    t.n = (int)(K >> 8);
    auto tile_source = [&](int64_t m0, int64_t n0) {
        const int64_t pitch = t.pitch;
        src_t c;
        c.ga = uniform_ptr(a_codes + (m0 + w * 64) * pitch);
        c.gb = uniform_ptr(b_codes + (n0 + w * 32) * pitch);
        c.gs = uniform_ptr(w < 2 ? a_scales_sm + (m0 + w * 128) * 8 : b_scales_sm + n0 * 8);
        return c;
    };
    // fragment reads: row l32 (+32 i) of the wave's rows, logical chunk 4h + s
    {
        const int rx = (l32 >> 1) & 7;
#pragma unroll
        for (int s = 0; s < 4; ++s) t.off[s] = ((4 * h + s) ^ rx) * 16;
        t.a_row = (wm * 128 + l32) * TKB;
        t.b_row = A_SLAB + (wn * 64 + l32) * TKB;
        t.sa_row = SA_OFF + (wm * 128 + l32) * 8 + 4 * h;
        t.sb_row = SB_OFF + (wn * 64 + l32) * 8 + 4 * h;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) t.sc.a[i] = t.scn.a[i] = 0;
#pragma unroll
    for (int j = 0; j < 2; ++j) t.sc.b[j] = t.scn.b[j] = 0;

    int v = blockIdx.x;
    int64_t m0, n0;
    tile_origin(v, m0, n0);
    {
        const src_t cur = tile_source(m0, n0);
        t.pa = cur.ga;
        t.pb = cur.gb;
        t.ps = cur.gs;
        t.nxt = cur;
    }
    t.left = t.n;
    t.cbuf = 0;

    auto c_of = [&](int64_t mm, int64_t nn) { return C + (mm + wm * 128 + h * 4) * ldc + nn + wn * 64 + l32; };
    auto look_ahead = [&](bool &more, int64_t &m0n, int64_t &n0n) {
        const int vn = v + grid;
        more = vn < ntiles; // the same for the whole workgroup
        tile_origin(more ? vn : v, m0n, n0n);
        t.nxt = tile_source(m0n, n0n); // (after its last tile a workgroup names that tile once more: fetched, never used)
    };

    // prologue: stages 0 and 1 of the first tile and the first copies of stage 2 under way, stage 0 landed
    bool more;
    int64_t m0n, n0n;
    look_ahead(more, m0n, n0n);
    issue<0, NCOPY>(t);
    advance(t);
    issue<0, NCOPY>(t);
    advance(t);
    issue<0, PART1>(t);
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(NCOPY + PART1) : "memory");
    uint32_t rb = 0;
#pragma unroll
    for (int q = 0; q < 6; ++q) read_item(smem, t, 0, q, t.f0);
    read_scales(smem, t, t.sc);

    float *cprev = c_of(m0, n0);
    run_tile<0, false>(t, smem, rb, cprev, ldc);
    for (;;) {
        cprev = c_of(m0, n0); // the tile just finished, in set 0
        if (!more) {
            store_all<0>(t, cprev, ldc);
            break;
        }
        v += grid, m0 = m0n, n0 = n0n;
        look_ahead(more, m0n, n0n);
        run_tile<1, true>(t, smem, rb, cprev, ldc);
        cprev = c_of(m0, n0); // in set 1
        if (!more) {
            store_all<1>(t, cprev, ldc);
            break;
        }
        v += grid, m0 = m0n, n0 = n0n;
        look_ahead(more, m0n, n0n);
        run_tile<0, true>(t, smem, rb, cprev, ldc);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); // the copies begun for a tile that does not follow
}

} // namespace

bool gemm_mx_dual_eligible(int64_t M, int64_t N, int64_t K)
{
    return K % 256 == 0 && K >= 256 * dual::STORE_STAGES && M >= dual::TM && N >= dual::TN;
}

// Launches the kernel on rows [0, Mi), columns [0, Ni) (multiples of 256 and 128); scales stage-major over those rows.
// Once per device: the compute-unit count and the kernel's LDS size.  Host-side calls, nothing queued.
int configure_gemm_mx_dual(int *ncu_out)
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
        rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_mx_dual),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, dual::LDS_BYTES));
        if (rc != ADAHOP_OK) return rc;
        if (dev >= 0 && dev < 64) cu_count[dev].store(ncu, std::memory_order_relaxed);
        once.mark(dev);
    }
    if (ncu_out) *ncu_out = ncu;
    return ADAHOP_OK;
}

int launch_gemm_mx_dual(int64_t Mi, int64_t Ni, int64_t K, const uint8_t *a_codes, const uint8_t *a_sm,
                        const uint8_t *b_codes, const uint8_t *b_sm, float *C, int64_t ldc, hipStream_t st)
{
    int ncu = 0;
    int rc = configure_gemm_mx_dual(&ncu);
    if (rc != ADAHOP_OK) return rc;
    ncu = ncu / 8 * 8;
    if (ncu < 8) ncu = 8;
    const int tiles_m = (int)(Mi / dual::TM), tiles_n = (int)(Ni / dual::TN);
    const int ntiles = tiles_m * tiles_n;
    const int group_m = tiles_m < 4 ? tiles_m : 4; // the 32 tiles an XCD runs at a time: 4 x 8, a 1024 x 1024 block of C
    const dim3 grid((unsigned)(ntiles < ncu ? ntiles : ncu));
    hipLaunchKernelGGL(k_gemm_mx_dual, grid, dim3(256), dual::LDS_BYTES, st, K, a_codes, a_sm, b_codes, b_sm, Mi, Ni, C, ldc,
                       tiles_m, tiles_n, group_m);
    return check_launch();
}

} // namespace adahop
