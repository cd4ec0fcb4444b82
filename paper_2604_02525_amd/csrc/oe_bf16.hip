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
//   2. k_oe_skinny     workgroup = (RT x 32 rows of Sg) x (128 rows of L) x (one slice of K); both
//                      operands go through LDS in a K-contiguous [row][64 K] layout, so a K-strided L
//                      is transposed on its way into LDS (16-bit scatter stores) while its global reads
//                      stay 16 bytes per lane; the next stage is fetched into registers while the
//                      matrix cores work on the current one.  K is split over workgroups so that the
//                      chip is full although there are few tiles; every slice writes its own partial
//                      tile (no atomics: the result does not depend on scheduling);
//   3. k_oe_reduce     adds the slices in a fixed order and writes the rows / columns of C.
// ------------------------------------------------------------------------------------------------
constexpr int SK_LCOLS = 128;  // rows of L per workgroup
constexpr int SK_KSTAGE = 64;  // K-elements per pipeline stage
constexpr int SK_PITCH = 72;   // LDS row pitch in bf16 (144 bytes: 16-byte fragment reads of 16
                               // consecutive rows then cover the 64 banks exactly once)

__global__ __launch_bounds__(256) void k_gather_rows(const uint16_t *__restrict__ x, int64_t ld, int k_contig, int64_t K,
                                                     const int32_t *__restrict__ idx, int k, int rows_alloc,
                                                     uint16_t *__restrict__ out)
{
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k_contig) { // one thread = 8 consecutive K-elements of one row
        const int64_t per_row = K >> 3;
        if (g >= rows_alloc * per_row) return;
        const int64_t t = g / per_row, c = g - t * per_row;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (t < k) v = load_once16(x + (int64_t)idx[t] * ld + c * 8);
        *reinterpret_cast<uint4 *>(out + t * K + c * 8) = v;
    } else {        // one thread = one element; neighbouring threads write neighbouring K
        if (g >= rows_alloc * K) return;
        const int64_t t = g / K, kk = g - t * K;
        out[g] = t < k ? load_once2(x + kk * ld + idx[t]) : (uint16_t)0;
    }
}

template <int RT, bool LONG_KC>
__global__ __launch_bounds__(256, 2) void k_oe_skinny(const uint16_t *__restrict__ Sg, const uint16_t *__restrict__ L,
                                                      int64_t ldl, int64_t Lo, int64_t K, int stages_per_slice,
                                                      float *__restrict__ P, int64_t rows_all)
{
    __shared__ __attribute__((aligned(16))) uint16_t sS[RT * 32 * SK_PITCH];
    __shared__ __attribute__((aligned(16))) uint16_t sL[SK_LCOLS * SK_PITCH];
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
    const int64_t l0 = (int64_t)blockIdx.x * SK_LCOLS;
    const int nstage_all = (int)((K + SK_KSTAGE - 1) / SK_KSTAGE);
    const int s0 = blockIdx.y * stages_per_slice, s1 = min(s0 + stages_per_slice, nstage_all);
    Sg += (int64_t)blockIdx.z * RT * 32 * K;
    P += ((int64_t)blockIdx.y * rows_all + (int64_t)blockIdx.z * RT * 32) * Lo;

    // loader geometry
    const int c8 = tid & 7, r32 = tid >> 3;           // K-contiguous: 16-byte chunk c8 of rows r32 + 32 i
    const int lane16 = lane & 15, grp = lane >> 4;    // K-strided: K offset lane16, 8 L-rows at 32 w + 8 grp
    uint4 ps[RT], pl[4];

    auto fetch = [&](int stage) {
        const int64_t kk0 = (int64_t)stage * SK_KSTAGE;
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            const int64_t kk = kk0 + c8 * 8;
            ps[i] = kk < K ? *reinterpret_cast<const uint4 *>(Sg + (int64_t)(r32 + 32 * i) * K + kk) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if constexpr (LONG_KC) {
                const int64_t kk = kk0 + c8 * 8, l = l0 + r32 + 32 * i;
                pl[i] = (kk < K && l < Lo) ? load_once16(L + l * ldl + kk) : make_uint4(0, 0, 0, 0);
            } else {
                const int64_t kk = kk0 + 16 * i + lane16, l = l0 + 32 * w + 8 * grp;
                pl[i] = (kk < K && l < Lo) ? load_once16(L + kk * ldl + l) : make_uint4(0, 0, 0, 0);
            }
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int i = 0; i < RT; ++i) *reinterpret_cast<uint4 *>(sS + (r32 + 32 * i) * SK_PITCH + c8 * 8) = ps[i];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if constexpr (LONG_KC) {
                *reinterpret_cast<uint4 *>(sL + (r32 + 32 * i) * SK_PITCH + c8 * 8) = pl[i];
            } else {
                uint16_t *d = sL + (32 * w + 8 * grp) * SK_PITCH + 16 * i + lane16;
                const uint32_t e[4] = {pl[i].x, pl[i].y, pl[i].z, pl[i].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    d[(2 * j) * SK_PITCH] = (uint16_t)(e[j] & 0xffffu);
                    d[(2 * j + 1) * SK_PITCH] = (uint16_t)(e[j] >> 16);
                }
            }
        }
    };

    v16f acc[RT];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;

    if (s0 < s1) {
        fetch(s0);
        stash();
    }
    __syncthreads();
    for (int stage = s0; stage < s1; ++stage) {
        const bool more = stage + 1 < s1;
        if (more) fetch(stage + 1);
#pragma unroll
        for (int ks = 0; ks < SK_KSTAGE / 16; ++ks) {
            const uint4 b = *reinterpret_cast<const uint4 *>(sL + (32 * w + l32) * SK_PITCH + 16 * ks + 8 * h);
#pragma unroll
            for (int i = 0; i < RT; ++i) {
                const uint4 a = *reinterpret_cast<const uint4 *>(sS + (32 * i + l32) * SK_PITCH + 16 * ks + 8 * h);
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), acc[i], 0, 0, 0);
            }
        }
        __syncthreads();
        if (more) stash();
        __syncthreads();
    }

    const int64_t l = l0 + 32 * w + l32;
    if (l < Lo) {
#pragma unroll
        for (int i = 0; i < RT; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) P[(int64_t)(32 * i + (r >> 2) * 8 + h * 4 + (r & 3)) * Lo + l] = acc[i][r];
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

struct skinny_plan_t {
    int rt, groups, nslice, stages_per_slice;
    int64_t rows_all;
    size_t sg_bytes, p_bytes;
};

// Row tiles per workgroup from {2, 4, 6, 8} with the least padding; K slices so that about two
// workgroups per compute unit exist, each with at least 8 stages.
skinny_plan_t plan_skinny(int64_t Lo, int64_t K, int k)
{
    skinny_plan_t p;
    const int tiles = (k + 31) / 32;
    p.rt = 8;
    p.groups = (tiles + 7) / 8;
    for (int rt = 6; rt >= 2; rt -= 2) {
        const int g = (tiles + rt - 1) / rt;
        if (g * rt < p.groups * p.rt || (g * rt == p.groups * p.rt && g < p.groups)) {
            p.rt = rt;
            p.groups = g;
        }
    }
    p.rows_all = (int64_t)p.groups * p.rt * 32;
    const int64_t nstage = ceil_div(K, SK_KSTAGE), wgs = ceil_div(Lo, SK_LCOLS) * p.groups;
    int64_t want = ceil_div(512, wgs);
    if (want > nstage / 8) want = nstage / 8;
    if (want < 1) want = 1;
    p.stages_per_slice = (int)ceil_div(nstage, want);
    p.nslice = (int)ceil_div(nstage, p.stages_per_slice);
    p.sg_bytes = align_up((size_t)p.rows_all * K * 2, 256);
    p.p_bytes = align_up((size_t)p.nslice * p.rows_all * Lo * 4, 256);
    return p;
}

template <int RT>
void launch_skinny(bool long_kc, dim3 grid, hipStream_t st, const uint16_t *Sg, const uint16_t *L, int64_t ldl, int64_t Lo,
                   int64_t K, int sps, float *P, int64_t rows_all)
{
    if (long_kc)
        hipLaunchKernelGGL((k_oe_skinny<RT, true>), grid, dim3(256), 0, st, Sg, L, ldl, Lo, K, sps, P, rows_all);
    else
        hipLaunchKernelGGL((k_oe_skinny<RT, false>), grid, dim3(256), 0, st, Sg, L, ldl, Lo, K, sps, P, rows_all);
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
// one row) are whole 128-byte segments.
__global__ __launch_bounds__(256) void k_gather_k_strided(const uint16_t *__restrict__ x, int64_t ld, int64_t outer,
                                                          const int32_t *__restrict__ idx, int k, int kpad,
                                                          uint16_t *__restrict__ out)
{
    __shared__ uint16_t tile[64][66];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int64_t o0 = (int64_t)blockIdx.x * 64;
    const int t0 = blockIdx.y * 64;
#pragma unroll 4
    for (int r = 0; r < 16; ++r) {
        const int t = t0 + ty * 16 + r;
        const int64_t o = o0 + tx;
        tile[ty * 16 + r][tx] = (t < k && o < outer) ? load_once2(x + (int64_t)idx[t] * ld + o) : (uint16_t)0;
    }
    __syncthreads();
#pragma unroll 4
    for (int r = 0; r < 16; ++r) {
        const int64_t o = o0 + ty * 16 + r;
        if (o < outer) out[o * kpad + t0 + tx] = tile[tx][ty * 16 + r];
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

    const int64_t gthreads = S.k_contig ? p.rows_all * (K >> 3) : p.rows_all * K;
    hipLaunchKernelGGL(k_gather_rows, dim3((unsigned)ceil_div(gthreads, 256)), dim3(256), 0, st,
                       static_cast<const uint16_t *>(S.data), S.ld, S.k_contig, K, idx, k, (int)p.rows_all, Sg);
    int rc = check_launch();
    if (rc != ADAHOP_OK) return rc;

    const dim3 grid((unsigned)ceil_div(Lo, SK_LCOLS), (unsigned)p.nslice, (unsigned)p.groups);
    const uint16_t *l = static_cast<const uint16_t *>(L.data);
    switch (p.rt) {
    case 2: launch_skinny<2>(L.k_contig, grid, st, Sg, l, L.ld, Lo, K, p.stages_per_slice, P, p.rows_all); break;
    case 4: launch_skinny<4>(L.k_contig, grid, st, Sg, l, L.ld, Lo, K, p.stages_per_slice, P, p.rows_all); break;
    case 6: launch_skinny<6>(L.k_contig, grid, st, Sg, l, L.ld, Lo, K, p.stages_per_slice, P, p.rows_all); break;
    default: launch_skinny<8>(L.k_contig, grid, st, Sg, l, L.ld, Lo, K, p.stages_per_slice, P, p.rows_all); break;
    }
    rc = check_launch();
    if (rc != ADAHOP_OK) return rc;

    const unsigned rblocks = (unsigned)ceil_div((int64_t)k * Lo, 256);
    auto reduce = [&](auto *c) {
        typedef typename std::remove_pointer<decltype(c)>::type out_t;
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
