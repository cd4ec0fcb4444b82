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

namespace adahop {

namespace {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

// Eight consecutive K-elements (kk .. kk+7) of row o of an operand, as packed bf16.
__device__ __forceinline__ uint4 load8(const uint16_t *__restrict__ d, int64_t ld, int k_contig, int64_t o, int64_t kk)
{
    if (k_contig) return *reinterpret_cast<const uint4 *>(d + o * ld + kk);
    uint32_t e[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) e[t] = d[(kk + t) * ld + o];
    return make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
}

// Workgroup tile 64x64 (four waves, one 32x32 matrix-core tile each).  ROWS: the tile's rows are
// gathered through idx (OE-row); else its columns are (OE-col).
template <bool ROWS>
__global__ __launch_bounds__(256) void k_oe_rowcol(const uint16_t *__restrict__ A, int64_t lda, int a_kc,
                                                   const uint16_t *__restrict__ B, int64_t ldb, int b_kc, int64_t M,
                                                   int64_t N, int64_t K, const int32_t *__restrict__ idx, int k,
                                                   float *__restrict__ C, int64_t ldc)
{
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int l32 = lane & 31, h = lane >> 5;
    const int64_t R = ROWS ? k : M, Cn = ROWS ? N : k;
    const int64_t r0 = (int64_t)blockIdx.y * 64 + (w >> 1) * 32;
    const int64_t c0 = (int64_t)blockIdx.x * 64 + (w & 1) * 32;
    const int64_t r = r0 + l32, c = c0 + l32;
    const bool rok = r < R, cok = c < Cn;
    const int64_t arow = rok ? (ROWS ? (int64_t)idx[r] : r) : 0;
    const int64_t brow = cok ? (ROWS ? c : (int64_t)idx[c]) : 0;

    v16f acc;
#pragma unroll
    for (int t = 0; t < 16; ++t) acc[t] = 0.0f;
    for (int64_t kk = 0; kk < K; kk += 16) {
        uint4 a = rok ? load8(A, lda, a_kc, arow, kk + h * 8) : make_uint4(0, 0, 0, 0);
        uint4 b = cok ? load8(B, ldb, b_kc, brow, kk + h * 8) : make_uint4(0, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), acc, 0, 0, 0);
    }
    if (!cok) return;
    const int64_t ocol = ROWS ? c : (int64_t)idx[c];
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        const int64_t rr = r0 + (t >> 2) * 8 + h * 4 + (t & 3);
        if (rr < R) {
            const int64_t orow = ROWS ? (int64_t)idx[rr] : rr;
            C[orow * ldc + ocol] = acc[t];
        }
    }
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
        v = k_contig ? x[o * ld + kk] : x[kk * ld + o];
    }
    out[o * kpad + t] = v;
}

} // namespace

int launch_gather_k(const adahop_operand_t &x, const int32_t *idx, int k, int kpad, uint16_t *out, hipStream_t st)
{
    const int64_t n = x.outer * kpad;
    if (n == 0) return ADAHOP_OK;
    hipLaunchKernelGGL(k_gather_k, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, st,
                       static_cast<const uint16_t *>(x.data), x.ld, x.k_contig, x.outer, idx, k, kpad, out);
    return check_launch();
}

int launch_oe_rowcol(const adahop_operand_t &A, const adahop_operand_t &B, int kind, const int32_t *idx, int k,
                     float *C, int64_t ldc, hipStream_t st)
{
    const int64_t M = A.outer, N = B.outer, K = A.K;
    if (k == 0 || M == 0 || N == 0) return ADAHOP_OK;
    const uint16_t *a = static_cast<const uint16_t *>(A.data);
    const uint16_t *b = static_cast<const uint16_t *>(B.data);
    if (kind == ADAHOP_IHT_OE_ROW) {
        dim3 grid((unsigned)ceil_div(N, 64), (unsigned)ceil_div(k, 64));
        hipLaunchKernelGGL((k_oe_rowcol<true>), grid, dim3(256), 0, st, a, A.ld, A.k_contig, b, B.ld, B.k_contig, M, N,
                           K, idx, k, C, ldc);
    } else {
        dim3 grid((unsigned)ceil_div(k, 64), (unsigned)ceil_div(M, 64));
        hipLaunchKernelGGL((k_oe_rowcol<false>), grid, dim3(256), 0, st, a, A.ld, A.k_contig, b, B.ld, B.k_contig, M,
                           N, K, idx, k, C, ldc);
    }
    return check_launch();
}

} // namespace adahop
