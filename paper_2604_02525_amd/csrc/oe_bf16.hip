// The BF16 outlier products of Outlier Extraction (second term of paper Eq. 7 and Eq. 8) and the
// gather that feeds the K-channel form.  Operands are the ORIGINAL bf16 values, accumulated in fp32
// on the BF16 matrix cores (v_mfma_f32_32x32x16_bf16).
//
//   OE-row:  C[idx[t], n] = sum_kk A(idx[t], kk) B(n, kk)      for t < k, all n
//   OE-col:  C[m, idx[t]] = sum_kk A(m, kk) B(idx[t], kk)      for all m, t < k
//
// The extracted rows / columns of the residual are zero, so the MXFP4 product left exact zeros in
// these places of C and the sum of Eq. 7 / 8 is a plain overwrite.
#include "common.h"

#include <type_traits>

namespace adahop {

namespace {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

// ------------------------------------------------------------------------------------------------
// Row / column form.  With S the k extracted rows of the "short" operand (A for OE-row, B for
// OE-col) and L the other, "long" operand, both products are  P[t, l] = sum_kk S(idx[t], kk) L(l, kk),
// a skinny product: a few hundred rows against a whole operand, bound by reading L once.
//
//   1. k_gather_rows   copies the extracted rows into a K-contiguous staging matrix Sg, zero padded to
//                      whole 32-row matrix-core tiles;
//   2. k_oe_skinny     workgroup = (RT x 32 rows of Sg) x (256 rows of L) x (one slice of K), a wave = all the rows
//                      of Sg x 64 rows of L.  Stages of 64 K-elements travel memory -> registers -> LDS; two are
//                      on their way in registers while a third is multiplied from one LDS buffer and a fourth is
//                      being written into the other (one barrier per stage).  Sg and a K-contiguous L lie in LDS
//                      as [row][64 K]; a K-strided L lies there as it lies in memory, [K][256 rows], and the
//                      transposing LDS read hands the matrix cores their 8 consecutive K-elements of a row.  K
//                      is split over workgroups so that the chip is full although there are few tiles; every
//                      slice writes its own partial tile (no atomics: the result does not depend on scheduling);
//   3. k_oe_reduce     adds the slices in a fixed order and writes the rows / columns of C.
// ------------------------------------------------------------------------------------------------
constexpr int SK_LCOLS = 256;  // rows of L per workgroup
constexpr int SK_KSTAGE = 64;  // K-elements per pipeline stage
constexpr int SK_PITCH = 72;   // LDS row pitch in bf16 of the [row][64 K] layout (144 bytes: 16-byte fragment
                               // reads of 16 consecutive rows then cover the 64 banks exactly once)
constexpr int SK_TPITCH = 288; // pitch in bf16 of the [K][256 rows] layout (576 bytes: the four K-rows of one
                               // transposing read of 32 lanes start 16 banks apart)
constexpr int SK_L_ELEMS = SK_LCOLS * SK_PITCH; // = SK_KSTAGE * SK_TPITCH: either layout of a stage of L

typedef short v4s __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void k_gather_rows(const uint16_t *__restrict__ x, int64_t ld, int64_t K,
                                                     const int32_t *__restrict__ idx, int k, int rows_alloc,
                                                     uint16_t *__restrict__ out)
{ // K-contiguous source: one thread = 8 consecutive K-elements of one row
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x, per_row = K >> 3;
    if (g >= rows_alloc * per_row) return;
    const int64_t t = g / per_row, c = g - t * per_row;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (t < k) v = load_once16(x + (int64_t)idx[t] * ld + c * 8);
    *reinterpret_cast<uint4 *>(out + t * K + c * 8) = v;
}

// K-strided source (element (o, kk) at x[kk * ld + o]): a workgroup takes 64 K-rows x 64 extracted columns.  It reads
// with the extracted column as the fast index, so that a wave's 64 two-byte reads fall into one K-row of the source
// (one DRAM page, neighbouring sectors where the indices are close) instead of 64 rows, turns the tile in LDS and
// writes 128-byte runs along K.
__global__ __launch_bounds__(256) void k_gather_rows_strided(const uint16_t *__restrict__ x, int64_t ld, int64_t K,
                                                             const int32_t *__restrict__ idx, int k,
                                                             uint16_t *__restrict__ out)
{
    __shared__ uint16_t tile[64][66]; // [t][kk], 33-word pitch: the column writes below spread over the banks
    const int64_t kk0 = (int64_t)blockIdx.x * 64;
    const int t0 = blockIdx.y * 64, lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int t = t0 + lane;
    const int64_t col = t < k ? idx[t] : -1;
    uint16_t v[16]; // all 16 reads of a thread in flight at once: few workgroups, each bound by its round trips
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int64_t kk = kk0 + 4 * i + w;
        v[i] = (col >= 0 && kk < K) ? load_once2(x + kk * ld + col) : (uint16_t)0;
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) tile[lane][4 * i + w] = v[i];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int tt = 4 * i + w; // row of the tile; the wave's lanes run along K
        if (kk0 + lane < K) out[(int64_t)(t0 + tt) * K + kk0 + lane] = tile[tt][lane];
    }
}

template <int RT, bool LONG_KC>
__global__ __launch_bounds__(256, 1) void k_oe_skinny(const uint16_t *__restrict__ Sg, const uint16_t *__restrict__ L,
                                                      int64_t ldl, int64_t Lo, int64_t K, int stages_per_slice,
                                                      float *__restrict__ P, int64_t rows_all)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[]; // 2 x (stage of Sg, stage of L)
    constexpr int S_ELEMS = RT * 32 * SK_PITCH, BUF_ELEMS = S_ELEMS + SK_L_ELEMS;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
    const int64_t l0 = (int64_t)blockIdx.x * SK_LCOLS;
    const int nstage_all = (int)((K + SK_KSTAGE - 1) / SK_KSTAGE);
    const int s0 = blockIdx.y * stages_per_slice, s1 = min(s0 + stages_per_slice, nstage_all);
    Sg += (int64_t)blockIdx.z * RT * 32 * K;
    P += ((int64_t)blockIdx.y * rows_all + (int64_t)blockIdx.z * RT * 32) * Lo;

    // loader geometry.  [row][K] sources: 16-byte chunk c8 of rows r32 + 32 i.  K-strided L: chunk c32 (8 rows of
    // L) of K-rows k8 + 8 i, so that a wave reads two whole 512-byte pieces of K-rows.  Every address is a base that
    // is the same for the whole workgroup plus a 32-bit byte offset of the lane (the offsets stay below 2^31: at most
    // 256 rows of at most 2^21 elements).  Rows of L past the end are replaced by the last row (their results are
    // not stored); in a last stage of 32 K-elements the upper half reads the lower half again and the Sg side is
    // zero there.
    const int c8 = tid & 7, r32 = tid >> 3, c32 = tid & 31, k8 = tid >> 5;
    const int64_t last_row = Lo - 1 - l0; // >= 0
    const char *const Lb = reinterpret_cast<const char *>(L + (LONG_KC ? l0 * ldl : 0));
    const char *const Sb = reinterpret_cast<const char *>(Sg);
    const uint32_t voff_s = (uint32_t)(((int64_t)r32 * K + c8 * 8) * 2);
    uint32_t voff_l[LONG_KC ? 8 : 1];
    if constexpr (LONG_KC) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int64_t r = r32 + 32 * i;
            voff_l[i] = (uint32_t)(((r < last_row ? r : last_row) * ldl + c8 * 8) * 2);
        }
    } else {
        const int64_t l = l0 + 8 * c32, l_last = (Lo - 1) / 8 * 8; // whole 16-byte pieces: ld is a multiple of 8
        voff_l[0] = (uint32_t)(((int64_t)k8 * ldl) * 2) + (uint32_t)((l < l_last ? l : l_last) * 2);
    }

    // A stage past the end of the slice (the loop below works on pairs of stages) reads the slice's last stage
    // again with the Sg side cleared.  No branches: the loop body stays one block, which the interleaving of
    // memory and matrix-core instructions below relies on.
    // QUARTER = 0 .. 3: the quarter of a stage's loads / LDS writes that is slotted between the matrix-core
    // instructions of K-step QUARTER (rows of L 2 q and 2 q + 1 of the lane's eight, row tiles q and q + 4 of Sg);
    // QUARTER = -1: all of them.
    // (The clearing of the Sg side happens when the registers are written to LDS, stage_keep below: touching a
    // loaded value here would make the wave wait for the load it has just issued.)
    auto stage_keep = [&](int stage) -> uint32_t {
        const bool ghost = stage >= s1;
        const int64_t kk0 = (int64_t)(ghost ? s1 - 1 : stage) * SK_KSTAGE;
        return (ghost || (kk0 + SK_KSTAGE > K && c8 >= 4)) ? 0u : 0xffffffffu;
    };
    auto fetch = [&](int stage, uint4 (&fs)[RT], uint4 (&fl)[8], auto quarter) {
        constexpr int Q = decltype(quarter)::value;
        const bool ghost = stage >= s1;
        const int64_t kk0 = (int64_t)(ghost ? s1 - 1 : stage) * SK_KSTAGE;
        const bool half = kk0 + SK_KSTAGE > K; // K is a multiple of 32: the last stage may hold 32 K-elements
        const uint32_t back = half && c8 >= 4 ? 64u : 0u;
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            if (Q >= 0 && (i & 3) != Q) continue;
            fs[i] = *reinterpret_cast<const uint4 *>(Sb + ((int64_t)32 * i * K + kk0) * 2 + (voff_s - back));
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (Q >= 0 && (i >> 1) != Q) continue;
            if constexpr (LONG_KC)
                fl[i] = load_once16(Lb + kk0 * 2 + (voff_l[i] - back));
            else
                fl[i] = load_once16(Lb + (kk0 + (half ? (8 * i) & 31 : 8 * i)) * ldl * 2 + voff_l[0]);
        }
    };
    auto stash = [&](uint16_t *buf, const uint4 (&fs)[RT], const uint4 (&fl)[8], uint32_t keep, auto quarter) {
        constexpr int Q = decltype(quarter)::value;
        uint16_t *sS = buf, *sL = buf + S_ELEMS;
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            if (Q >= 0 && (i & 3) != Q) continue;
            *reinterpret_cast<uint4 *>(sS + (r32 + 32 * i) * SK_PITCH + c8 * 8) =
                make_uint4(fs[i].x & keep, fs[i].y & keep, fs[i].z & keep, fs[i].w & keep);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (Q >= 0 && (i >> 1) != Q) continue;
            if constexpr (LONG_KC)
                *reinterpret_cast<uint4 *>(sL + (r32 + 32 * i) * SK_PITCH + c8 * 8) = fl[i];
            else
                *reinterpret_cast<uint4 *>(sL + (k8 + 8 * i) * SK_TPITCH + 8 * c32) = fl[i];
        }
    };
    typedef std::integral_constant<int, -1> all_t;

    v16f acc[RT][2];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][c][r] = 0.0f;

    // As supplier of addresses for the transposing read, lane s of a group of 16 points at 4 consecutive rows of L
    // (4 (s % 4) ..) in K-row s / 4; lane n of the group then receives K-rows 0 .. 3 of row n.  The four groups of a
    // wave are (rows 0-15 | 16-31 of the 32-row tile) x (K-half h) as the matrix cores want them.
    const int tr_elem = ((lane & 15) >> 2) * SK_TPITCH + 64 * w + 16 * ((lane >> 4) & 1) + 4 * (lane & 3) + 8 * h * SK_TPITCH;

    // One stage: multiply from `cur`; meanwhile write the stage that has arrived in (fs, fl) into `oth` (every wave
    // left that buffer before the last barrier) and refill (fs, fl) with stage `next`.  A wave issues in order and
    // is alone on its SIMD, so whatever is issued in a burst keeps it from feeding the matrix core: the fragment
    // reads of K-step ks + 1, a quarter of the LDS writes and a quarter of the loads are slotted one by one between
    // the matrix-core instructions of K-step ks (scheduling groups), and a scheduling barrier after every K-step
    // keeps the compiler from reading a whole stage's fragments (128 registers) ahead.
    // (fs, fl) hold stage next - 2 on entry.
    auto stage_body = [&](const uint16_t *cur, uint16_t *oth, uint4 (&fs)[RT], uint4 (&fl)[8], int next) {
        const uint32_t keep = stage_keep(next - 2);
        const uint16_t *sS = cur, *sL = cur + S_ELEMS;
        uint4 a[2][RT];
        v8bf b[2][2];
        auto fragments = [&](int ks, uint4 (&fa)[RT], v8bf (&fb)[2]) {
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                if constexpr (LONG_KC) {
                    const uint4 v = *reinterpret_cast<const uint4 *>(sL + (64 * w + 32 * c + l32) * SK_PITCH + 16 * ks + 8 * h);
                    fb[c] = __builtin_bit_cast(v8bf, v);
                } else {
                    const uint16_t *q = sL + tr_elem + 16 * ks * SK_TPITCH + 32 * c;
                    const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s *)q);
                    const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) v4s *)(q + 4 * SK_TPITCH));
                    typedef short v8s __attribute__((ext_vector_type(8)));
                    const v8s both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    fb[c] = __builtin_bit_cast(v8bf, both);
                }
            }
#pragma unroll
            for (int i = 0; i < RT; ++i)
                fa[i] = *reinterpret_cast<const uint4 *>(sS + (32 * i + l32) * SK_PITCH + 16 * ks + 8 * h);
        };
        auto step = [&](auto ks_c) {
            constexpr int ks = decltype(ks_c)::value;
            constexpr int n_read = ks + 1 < SK_KSTAGE / 16 ? RT + (LONG_KC ? 2 : 4) : 0;
            constexpr int n_move = 2 + (ks < RT ? 1 : 0) + (ks + 4 < RT ? 1 : 0); // LDS writes = loads of this quarter
            if constexpr (ks + 1 < SK_KSTAGE / 16) fragments(ks + 1, a[(ks + 1) & 1], b[(ks + 1) & 1]);
            stash(oth, fs, fl, keep, ks_c);
            fetch(next, fs, fl, ks_c);
#pragma unroll
            for (int i = 0; i < RT; ++i)
#pragma unroll
                for (int c = 0; c < 2; ++c)
                    acc[i][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a[ks & 1][i]), b[ks & 1][c],
                                                                        acc[i][c], 0, 0, 0);
#pragma unroll
            for (int j = 0; j < 2 * RT; ++j) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                 // one matrix-core instruction
                if (j < n_read) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); // one LDS read
                if (j < n_move) {
                    __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);             // one LDS write
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);             // one load
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        fragments(0, a[0], b[0]);
        step(std::integral_constant<int, 0>());
        step(std::integral_constant<int, 1>());
        step(std::integral_constant<int, 2>());
        step(std::integral_constant<int, 3>());
    };
    static_assert(SK_KSTAGE == 64, "four K-steps per stage, one quarter of the data movement in each");

    // Register set (stage - s0) & 1 carries a stage from memory to LDS buffer (stage - s0) & 1.  While a stage is
    // multiplied, the next one is written into the other buffer and the two after that are in flight.
    uint4 ps[2][RT], pl[2][8];
    uint16_t *buf0 = smem, *buf1 = smem + BUF_ELEMS;
    fetch(s0, ps[0], pl[0], all_t());
    fetch(s0 + 1, ps[1], pl[1], all_t());
    stash(buf0, ps[0], pl[0], stage_keep(s0), all_t());
    fetch(s0 + 2, ps[0], pl[0], all_t());
    __syncthreads();
    for (int stage = s0; stage < s1; stage += 2) { // no branch around a multiply: the accumulators stay where they are
        stage_body(buf0, buf1, ps[1], pl[1], stage + 3);
        __syncthreads();
        stage_body(buf1, buf0, ps[0], pl[0], stage + 4);
        __syncthreads();
    }

#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int64_t l = l0 + 64 * w + 32 * c + l32;
        if (l < Lo) {
#pragma unroll
            for (int i = 0; i < RT; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    P[(int64_t)(32 * i + (r >> 2) * 8 + h * 4 + (r & 3)) * Lo + l] = acc[i][c][r];
        }
    }
}

// C[idx[t], l] (ROWS) or C[l, idx[t]] = sum over the K slices of P[s][t][l], in slice order.
// C holds float, or bf16 as its 16 bits (rounded to nearest even from the fp32 sum).
template <bool ROWS, typename OUT>
__global__ __launch_bounds__(256) void k_oe_reduce(const float *__restrict__ P, int nslice, int64_t rows_all, int64_t Lo,
                                                   const int32_t *__restrict__ idx, int k, OUT *__restrict__ C, int64_t ldc)
{
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (g >= (int64_t)k * Lo) return;
    const int64_t t = g / Lo, l = g - t * Lo;
    float s = 0.0f;
    for (int i = 0; i < nslice; ++i) s += P[((int64_t)i * rows_all + t) * Lo + l];
    const int64_t o = idx[t];
    OUT v;
    if constexpr (sizeof(OUT) == 4) {
        v = s;
    } else {
        const uint32_t u = __float_as_uint(s);
        v = (OUT)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
    }
    if (ROWS)
        C[o * ldc + l] = v;
    else
        C[l * ldc + o] = v;
}

// The same on 4 consecutive long-side indices per thread (Lo % 4 == 0; for ROWS also 16-byte / 8-byte aligned rows of
// C): 16-byte reads of the partials, and for ROWS one 16-byte (fp32) or 8-byte (bf16) store.
__device__ __forceinline__ uint16_t bf16_rne(float s)
{
    const uint32_t u = __float_as_uint(s);
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

template <bool ROWS, typename OUT>
__global__ __launch_bounds__(256) void k_oe_reduce4(const float *__restrict__ P, int nslice, int64_t rows_all, int64_t Lo,
                                                    const int32_t *__restrict__ idx, int k, OUT *__restrict__ C, int64_t ldc)
{
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x, per = Lo >> 2;
    if (g >= (int64_t)k * per) return;
    const int64_t t = g / per, l = (g - t * per) * 4;
    float4 s = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    for (int i = 0; i < nslice; ++i) {
        const float4 v = *reinterpret_cast<const float4 *>(P + ((int64_t)i * rows_all + t) * Lo + l);
        s.x += v.x, s.y += v.y, s.z += v.z, s.w += v.w;
    }
    const int64_t o = idx[t];
    if constexpr (ROWS) {
        if constexpr (sizeof(OUT) == 4) {
            *reinterpret_cast<float4 *>(C + o * ldc + l) = s;
        } else {
            const uint32_t lo = (uint32_t)bf16_rne(s.x) | ((uint32_t)bf16_rne(s.y) << 16);
            const uint32_t hi = (uint32_t)bf16_rne(s.z) | ((uint32_t)bf16_rne(s.w) << 16);
            *reinterpret_cast<uint2 *>(C + o * ldc + l) = make_uint2(lo, hi);
        }
    } else {
        const float e[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (sizeof(OUT) == 4)
                C[(l + j) * ldc + o] = e[j];
            else
                C[(l + j) * ldc + o] = bf16_rne(e[j]);
        }
    }
}

struct skinny_plan_t {
    int rt, groups, nslice, stages_per_slice;
    int64_t rows_all;
    size_t sg_bytes, p_bytes;
};

// Row tiles per workgroup from {2, 4, 6}; K slices so that up to one workgroup per compute unit exists, each
// with at least 8 stages.
skinny_plan_t plan_skinny(int64_t Lo, int64_t K, int k)
{
    skinny_plan_t p;
    const int tiles = (k + 31) / 32;
    p.groups = (tiles + 5) / 6; // every group of row tiles reads L once: as few as possible
    p.rt = 6;
    for (int rt = 4; rt >= 2; rt -= 2)
        if ((tiles + rt - 1) / rt == p.groups) p.rt = rt; // the same passes with less padding
    p.rows_all = (int64_t)p.groups * p.rt * 32;
    const int64_t nstage = ceil_div(K, SK_KSTAGE), wgs = ceil_div(Lo, SK_LCOLS) * p.groups;
    int64_t want = 256 / wgs; // one workgroup per compute unit is resident; never more than that many: a second,
                              // partly filled round costs more than idle compute units do
    if (want > nstage / 8) want = nstage / 8;
    if (want < 1) want = 1;
    p.stages_per_slice = (int)ceil_div(nstage, want);
    p.nslice = (int)ceil_div(nstage, p.stages_per_slice);
    p.sg_bytes = align_up((size_t)p.rows_all * K * 2, 256);
    p.p_bytes = align_up((size_t)p.nslice * p.rows_all * Lo * 4, 256);
    return p;
}

template <int RT, bool LONG_KC> constexpr size_t skinny_lds_bytes() { return 2 * (RT * 32 * SK_PITCH + SK_L_ELEMS) * sizeof(uint16_t); }

template <int RT, bool LONG_KC> int allow_skinny_lds()
{
    return check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_oe_skinny<RT, LONG_KC>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)skinny_lds_bytes<RT, LONG_KC>()));
}

template <int RT, bool LONG_KC>
int launch_skinny_as(dim3 grid, hipStream_t st, const uint16_t *Sg, const uint16_t *L, int64_t ldl, int64_t Lo, int64_t K,
                     int sps, float *P, int64_t rows_all)
{
    const int rc = configure_oe_rowcol(); // more LDS than a launch may ask for by default: allowed once per device
    if (rc != ADAHOP_OK) return rc;
    constexpr size_t lds = skinny_lds_bytes<RT, LONG_KC>();
    hipLaunchKernelGGL((k_oe_skinny<RT, LONG_KC>), grid, dim3(256), lds, st, Sg, L, ldl, Lo, K, sps, P, rows_all);
    return check_launch();
}

template <int RT>
int launch_skinny(bool long_kc, dim3 grid, hipStream_t st, const uint16_t *Sg, const uint16_t *L, int64_t ldl, int64_t Lo,
                  int64_t K, int sps, float *P, int64_t rows_all)
{
    return long_kc ? launch_skinny_as<RT, true>(grid, st, Sg, L, ldl, Lo, K, sps, P, rows_all)
                   : launch_skinny_as<RT, false>(grid, st, Sg, L, ldl, Lo, K, sps, P, rows_all);
}

// out[o, t] = x(o, idx[t]) for t < k, 0 for k <= t < kpad.  out is [outer, kpad] bf16.
__global__ __launch_bounds__(256) void k_gather_k(const uint16_t *__restrict__ x, int64_t ld, int k_contig,
                                                  int64_t outer, const int32_t *__restrict__ idx, int k, int kpad,
                                                  uint16_t *__restrict__ out)
{
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (g >= outer * kpad) return;
    int64_t o, t;
    if (k_contig) { // neighbouring threads: neighbouring t of one row
        o = g / kpad;
        t = g - o * kpad;
    } else {        // neighbouring threads: neighbouring rows of one t (coalesced reads)
        t = g / outer;
        o = g - t * outer;
    }
    uint16_t v = 0;
    if (t < k) {
        const int64_t kk = idx[t];
        v = load_once2(k_contig ? x + o * ld + kk : x + kk * ld + o);
    }
    out[o * kpad + t] = v;
}

// The same for a K-strided operand (x stored [K, outer]): 64 channels x 64 rows per workgroup through
// LDS, so that both the reads (along the rows of one channel) and the writes (along the channels of
// one row) are whole 128-byte segments, 16 bytes per lane.
__global__ __launch_bounds__(256) void k_gather_k_strided(const uint16_t *__restrict__ x, int64_t ld, int64_t outer,
                                                          const int32_t *__restrict__ idx, int k, int kpad,
                                                          uint16_t *__restrict__ out)
{
    constexpr int PITCH = 72; // elements: 144-byte rows, 16-byte aligned
    __shared__ __align__(16) uint16_t tile[64 * PITCH];
    const int row = threadIdx.x >> 3, seg = threadIdx.x & 7;
    const int64_t o0 = (int64_t)blockIdx.x * 64;
    const int t0 = blockIdx.y * 64;
    uint4 v[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int t = t0 + p * 32 + row;
        const int64_t o = o0 + seg * 8;
        v[p] = make_uint4(0u, 0u, 0u, 0u);
        if (t < k) {
            const uint16_t *src = x + (int64_t)idx[t] * ld + o;
            if (o + 7 < outer) {
                v[p] = load_once16(src);
            } else { // (the last, ragged segment of a channel)
                uint16_t e[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) e[q] = o + q < outer ? load_once2(src + q) : (uint16_t)0;
                v[p] = make_uint4(e[0] | (uint32_t)e[1] << 16, e[2] | (uint32_t)e[3] << 16, e[4] | (uint32_t)e[5] << 16,
                                  e[6] | (uint32_t)e[7] << 16);
            }
        }
    }
#pragma unroll
    for (int p = 0; p < 2; ++p) *reinterpret_cast<uint4 *>(&tile[(p * 32 + row) * PITCH + seg * 8]) = v[p];
    __syncthreads();
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int ol = p * 32 + row; // row of the output: one outer index, 8 channels per lane
        uint16_t e[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) e[q] = tile[(seg * 8 + q) * PITCH + ol];
        if (o0 + ol < outer)
            *reinterpret_cast<uint4 *>(out + (o0 + ol) * kpad + t0 + seg * 8) =
                make_uint4(e[0] | (uint32_t)e[1] << 16, e[2] | (uint32_t)e[3] << 16, e[4] | (uint32_t)e[5] << 16,
                           e[6] | (uint32_t)e[7] << 16);
    }
}

} // namespace

// The first K threads clear the entries of the channels that stay, the next k set those of the extracted ones:
// no entry is written twice.
__global__ __launch_bounds__(256) void k_positions(const int32_t *__restrict__ idx, int k, const uint8_t *__restrict__ mask,
                                                   int64_t K, uint16_t *__restrict__ pos1)
{
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (g < K) {
        if (!mask[g]) pos1[g] = 0;
    } else if (g < K + k) {
        pos1[idx[g - K]] = (uint16_t)(g - K + 1);
    }
}

int launch_k_positions(const int32_t *idx, int k, const uint8_t *mask, int64_t K, uint16_t *pos1, hipStream_t st)
{
    hipLaunchKernelGGL(k_positions, dim3((unsigned)ceil_div(K + k, 256)), dim3(256), 0, st, idx, k, mask, K, pos1);
    return check_launch();
}

int launch_gather_k(const adahop_operand_t &x, const int32_t *idx, int k, int kpad, uint16_t *out, hipStream_t st)
{
    const int64_t n = x.outer * kpad;
    if (n == 0) return ADAHOP_OK;
    if (!x.k_contig && kpad % 64 == 0) {
        const dim3 grid((unsigned)ceil_div(x.outer, 64), (unsigned)(kpad / 64));
        hipLaunchKernelGGL(k_gather_k_strided, grid, dim3(256), 0, st, static_cast<const uint16_t *>(x.data), x.ld,
                           x.outer, idx, k, kpad, out);
        return check_launch();
    }
    hipLaunchKernelGGL(k_gather_k, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, st,
                       static_cast<const uint16_t *>(x.data), x.ld, x.k_contig, x.outer, idx, k, kpad, out);
    return check_launch();
}

// Every instance of the row / column product kernel, once per device (host-side calls, nothing queued).
int configure_oe_rowcol()
{
    static device_once_t once;
    int dev = 0;
    int rc = check_hip(hipGetDevice(&dev));
    if (rc != ADAHOP_OK || !once.need(dev)) return rc;
    if ((rc = allow_skinny_lds<2, true>()) != ADAHOP_OK || (rc = allow_skinny_lds<2, false>()) != ADAHOP_OK ||
        (rc = allow_skinny_lds<4, true>()) != ADAHOP_OK || (rc = allow_skinny_lds<4, false>()) != ADAHOP_OK ||
        (rc = allow_skinny_lds<6, true>()) != ADAHOP_OK || (rc = allow_skinny_lds<6, false>()) != ADAHOP_OK)
        return rc;
    once.mark(dev);
    return ADAHOP_OK;
}

size_t oe_rowcol_workspace_bytes(int64_t M, int64_t N, int64_t K, int kind, int k)
{
    if (k <= 0) return 0;
    const skinny_plan_t p = plan_skinny(kind == ADAHOP_IHT_OE_ROW ? N : M, K, k);
    return p.sg_bytes + p.p_bytes;
}

int launch_oe_rowcol(const adahop_operand_t &A, const adahop_operand_t &B, int kind, const int32_t *idx, int k,
                     void *C, int64_t ldc, int c_bf16, void *workspace, hipStream_t st)
{
    const int64_t M = A.outer, N = B.outer, K = A.K;
    if (k == 0 || M == 0 || N == 0) return ADAHOP_OK;
    const bool rows = kind == ADAHOP_IHT_OE_ROW;
    const adahop_operand_t &S = rows ? A : B, &L = rows ? B : A;
    const int64_t Lo = L.outer;
    const skinny_plan_t p = plan_skinny(Lo, K, k);
    uint16_t *Sg = static_cast<uint16_t *>(workspace);
    float *P = reinterpret_cast<float *>(static_cast<char *>(workspace) + p.sg_bytes);

    if (S.k_contig)
        hipLaunchKernelGGL(k_gather_rows, dim3((unsigned)ceil_div(p.rows_all * (K >> 3), 256)), dim3(256), 0, st,
                           static_cast<const uint16_t *>(S.data), S.ld, K, idx, k, (int)p.rows_all, Sg);
    else // rows_all is a multiple of 64: whole tiles of extracted columns
        hipLaunchKernelGGL(k_gather_rows_strided, dim3((unsigned)ceil_div(K, 64), (unsigned)(p.rows_all / 64)), dim3(256), 0,
                           st, static_cast<const uint16_t *>(S.data), S.ld, K, idx, k, Sg);
    int rc = check_launch();
    if (rc != ADAHOP_OK) return rc;

    const dim3 grid((unsigned)ceil_div(Lo, SK_LCOLS), (unsigned)p.nslice, (unsigned)p.groups);
    const uint16_t *l = static_cast<const uint16_t *>(L.data);
    switch (p.rt) {
    case 2: rc = launch_skinny<2>(L.k_contig, grid, st, Sg, l, L.ld, Lo, K, p.stages_per_slice, P, p.rows_all); break;
    case 4: rc = launch_skinny<4>(L.k_contig, grid, st, Sg, l, L.ld, Lo, K, p.stages_per_slice, P, p.rows_all); break;
    default: rc = launch_skinny<6>(L.k_contig, grid, st, Sg, l, L.ld, Lo, K, p.stages_per_slice, P, p.rows_all); break;
    }
    if (rc != ADAHOP_OK) return rc;

    const unsigned rblocks = (unsigned)ceil_div((int64_t)k * Lo, 256);
    auto reduce = [&](auto *c) {
        typedef typename std::remove_pointer<decltype(c)>::type out_t;
        // four long-side indices per thread where rows of the partials (and, for rows of C, of C) are 16-byte pieces
        if (Lo % 4 == 0 && (!rows || (ldc % 4 == 0 && aligned(c, 4 * sizeof(out_t))))) {
            const unsigned b4 = (unsigned)ceil_div((int64_t)k * (Lo >> 2), 256);
            if (rows)
                hipLaunchKernelGGL((k_oe_reduce4<true, out_t>), dim3(b4), dim3(256), 0, st, P, p.nslice, p.rows_all, Lo, idx, k, c,
                                   ldc);
            else
                hipLaunchKernelGGL((k_oe_reduce4<false, out_t>), dim3(b4), dim3(256), 0, st, P, p.nslice, p.rows_all, Lo, idx, k,
                                   c, ldc);
            return;
        }
        if (rows)
            hipLaunchKernelGGL((k_oe_reduce<true, out_t>), dim3(rblocks), dim3(256), 0, st, P, p.nslice, p.rows_all, Lo, idx,
                               k, c, ldc);
        else // (a variant that turns 32 x 64 blocks in LDS so that a wave's stores fall into two rows of C was measured
             // and is slower, 42 against 33 us on 123 x 8192: the k x Lo partial-sector writes cost the same either way)
            hipLaunchKernelGGL((k_oe_reduce<false, out_t>), dim3(rblocks), dim3(256), 0, st, P, p.nslice, p.rows_all, Lo, idx,
                               k, c, ldc);
    };
    if (c_bf16)
        reduce(static_cast<uint16_t *>(C));
    else
        reduce(static_cast<float *>(C));
    return check_launch();
}

} // namespace adahop
