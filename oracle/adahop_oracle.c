/*
 * CPU oracle for the AdaHOP per-GEMM hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain statement of what the GPU path must compute.  It is used by
 * the tests, by the smoke check and by the benchmark's CPU-baseline leg, and by nothing else.
 * It shares no code, header, table or constant with the HIP library.
 *
 * What is implemented, and the passage each piece follows:
 *   - the three linear-layer products and the operand layouts they imply      (paper Eq. 1-3)
 *   - C ~= Q(A) Q(B)                                                          (paper Eq. 4)
 *   - block Inner Hadamard Transform along K, normalised Sylvester matrix     (paper Eq. 5,
 *     App. F item 2: "1D Hadamard transform" with a fixed block size)
 *   - Outlier Extraction: residual + extracted part, OE-Left / OE-Right       (paper Eq. 7-8,
 *     App. E "OE formulation"); the K-channel form is the same split applied to K indices
 *   - FOID: variance over the first 64 elements, top-r by variance           (App. F item 1)
 *   - Outer Hadamard Transform, the comparison strategy: block transform along the OUTER
 *     index of each operand before quantisation, inverse rotations of C afterwards  (paper Eq. 6)
 *   - optional stochastic rounding of the elements (the paper cites it as prior work for unbiased
 *     gradient quantisation, Sec. 2.1-2.2): between the two neighbouring E2M1 values with probability
 *     proportional to the distance, random bits from Philox4x32-10 keyed by a seed and counted by the
 *     element's (row, K) position
 *   - MXFP4: OCP Microscaling v1.0 -- E2M1 elements, one E8M0 scale per 32 elements along K,
 *     scale = 2^(floor(log2 amax) - 2), round-to-nearest-even, saturate to +-6.  The paper only
 *     names the format; these rules are the published OCP ones.
 *
 * Arithmetic: bf16 inputs are widened exactly to fp32.  The Hadamard butterflies are fp32
 * add/sub in ascending stride order followed by one fp32 multiply by (float)(1/sqrt(b)); this
 * order is part of the definition because it fixes the rounding.  All GEMMs accumulate in double.
 *
 * Build:  gcc -O2 -fopenmp -ffp-contract=off -shared -fPIC (see oracle/build.py).
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ bf16 and operand access */

static inline float bf16_bits_to_f32(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* A logical [outer, K] bf16 matrix.  k_contig = 1: element (o, kk) at data[o*ld + kk];
 * k_contig = 0: at data[kk*ld + o].  (Eq. 1-3 give both kinds: X and W are K-contiguous in the
 * forward product, W is K-strided in dgrad, G_Y and X are K-strided in wgrad.) */
static inline float op_at(const uint16_t *data, int64_t ld, int k_contig, int64_t o, int64_t kk)
{
    return bf16_bits_to_f32(k_contig ? data[o * ld + kk] : data[kk * ld + o]);
}

/* ------------------------------------------------------------------ Hadamard (Eq. 5) */

/* In-place v <- (1/sqrt(b)) * H_b v, H_b the Sylvester (natural-order) Hadamard matrix.
 * H_b is symmetric, so the same routine serves A*H (rows of A) and H^T*B (columns of B). */
void orc_fwht(float *v, int b)
{
    for (int h = 1; h < b; h *= 2) {
        for (int i = 0; i < b; i += 2 * h) {
            for (int j = i; j < i + h; ++j) {
                float x = v[j];
                float y = v[j + h];
                v[j] = x + y;
                v[j + h] = x - y;
            }
        }
    }
    float c = (float)(1.0 / sqrt((double)b));
    for (int j = 0; j < b; ++j) {
        v[j] = v[j] * c;
        /* Convention, chosen here (the paper is silent): a transformed value that is exactly zero is
         * stored as +0.  Mathematically (H v)_j = 0 has no sign.  The plain butterflies above would
         * give -0 only where every contributing input is -0 (round-to-nearest cancellation of
         * nonzero terms yields +0 in any order), so the rule changes the sign nibble of such
         * all-negative-zero blocks and nothing else; both zeros dequantise to 0, so no product
         * changes.  It is fixed so that the sign of a zero is defined by the value alone and an
         * implementation that tracks signs differently (e.g. negated intermediate sums) is not
         * forced to reproduce IEEE -0 propagation.  Pinned by test_sign_of_zero_rules. */
        if (v[j] == 0.0f) v[j] = 0.0f;
    }
}

/* ------------------------------------------------------------------ FOID (App. F item 1) */

/* axis = 0: score each outer index over its first min(64, K) K-elements.
 * axis = 1: score each K index over its first min(64, outer) outer elements.
 * Score = sum of squared deviations from the mean (the variance up to a constant factor, which
 * cannot change the ranking).  Sequential fp32 sum, then sequential fused multiply-add. */
void orc_foid_scores(const uint16_t *data, int64_t outer, int64_t K, int64_t ld, int k_contig,
                     int axis, float *scores)
{
    int64_t dim = axis == 0 ? outer : K;
    int64_t len = axis == 0 ? K : outer;
    int64_t L = len < 64 ? len : 64;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < dim; ++i) {
        float s = 0.0f;
        for (int64_t j = 0; j < L; ++j) {
            float x = axis == 0 ? op_at(data, ld, k_contig, i, j) : op_at(data, ld, k_contig, j, i);
            s = s + x;
        }
        float mean = s * (1.0f / (float)L);
        float v = 0.0f;
        for (int64_t j = 0; j < L; ++j) {
            float x = axis == 0 ? op_at(data, ld, k_contig, i, j) : op_at(data, ld, k_contig, j, i);
            float d = x - mean;
            v = fmaf(d, d, v);
        }
        scores[i] = v;
    }
}

typedef struct {
    float score;
    int32_t index;
} scored_t;

static int scored_cmp(const void *pa, const void *pb)
{
    const scored_t *a = (const scored_t *)pa, *b = (const scored_t *)pb;
    if (a->score > b->score) return -1;
    if (a->score < b->score) return 1;
    return a->index < b->index ? -1 : (a->index > b->index ? 1 : 0);
}

static int int32_cmp(const void *pa, const void *pb)
{
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return a < b ? -1 : (a > b ? 1 : 0);
}

/* The k largest scores; equal scores are ranked by ascending index.  idx comes back sorted
 * ascending; mask[i] = 1 for selected i, else 0. */
void orc_topk(const float *scores, int64_t dim, int64_t k, int32_t *idx, uint8_t *mask)
{
    scored_t *a = (scored_t *)malloc((size_t)(dim > 0 ? dim : 1) * sizeof *a);
    for (int64_t i = 0; i < dim; ++i) {
        a[i].score = scores[i];
        a[i].index = (int32_t)i;
    }
    qsort(a, (size_t)dim, sizeof *a, scored_cmp);
    memset(mask, 0, (size_t)dim);
    for (int64_t t = 0; t < k; ++t) {
        idx[t] = a[t].index;
        mask[a[t].index] = 1;
    }
    qsort(idx, (size_t)k, sizeof *idx, int32_cmp);
    free(a);
}

/* ------------------------------------------------------------------ MX quantisation (OCP MX) */

/* E8M0 code for a block whose largest magnitude is amax: 127 + floor(log2 amax) - 2, clamped
 * to [0, 254]; an all-zero block gets code 0. */
uint8_t orc_e8m0_from_amax(float amax)
{
    if (!(amax > 0.0f)) return 0;
    int e;
    (void)frexpf(amax, &e); /* amax = m * 2^e, m in [0.5, 1)  =>  floor(log2 amax) = e - 1 */
    int s = (e - 1) - 2 + 127;
    if (s < 0) s = 0;
    if (s > 254) s = 254;
    return (uint8_t)s;
}

/* E2M1 code (sign in bit 3, magnitude index 0..7 for {0, .5, 1, 1.5, 2, 3, 4, 6}) of q, rounded
 * to nearest, ties to the even magnitude index, magnitudes above 6 saturating to 6.  The sign
 * bit is copied from q even when the magnitude rounds to zero. */
uint8_t orc_e2m1_encode(float q)
{
    uint32_t u;
    memcpy(&u, &q, sizeof u);
    uint8_t sign = (uint8_t)((u >> 31) << 3);
    float a = fabsf(q);
    uint8_t m;
    if (a <= 0.25f) m = 0;
    else if (a < 0.75f) m = 1;
    else if (a <= 1.25f) m = 2;
    else if (a < 1.75f) m = 3;
    else if (a <= 2.5f) m = 4;
    else if (a < 3.5f) m = 5;
    else if (a <= 5.0f) m = 6;
    else m = 7;
    return (uint8_t)(sign | m);
}

static const double E2M1_VALUE[8] = {0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0};

static inline double e2m1_decode(uint8_t code)
{
    double m = E2M1_VALUE[code & 7];
    return (code & 8) ? -m : m;
}

/* Quantise one 32-element block: scale code to *scale, 16 packed bytes to codes
 * (element 2t in the low nibble of byte t, element 2t+1 in the high nibble). */
void orc_mx_quantize_block(const float *v, uint8_t *codes, uint8_t *scale)
{
    float amax = 0.0f;
    for (int i = 0; i < 32; ++i) {
        float a = fabsf(v[i]);
        if (a > amax) amax = a;
    }
    uint8_t s = orc_e8m0_from_amax(amax);
    float X = ldexpf(1.0f, (int)s - 127);
    for (int t = 0; t < 16; ++t) {
        uint8_t lo = orc_e2m1_encode(v[2 * t] / X);
        uint8_t hi = orc_e2m1_encode(v[2 * t + 1] / X);
        codes[t] = (uint8_t)(lo | (hi << 4));
    }
    *scale = s;
}

/* ------------------------------------------------------------------ stochastic rounding (optional) */

/* Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",
 * SC'11): a keyed bijection of 128-bit counters, used as a counter-based generator. */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0, out[1] = c1, out[2] = c2, out[3] = c3;
}

/* The 16 random bits of element (o, kk) of an operand under `seed`: Philox key = (low, high) half of the
 * seed, counter = (o, kk / 8, 0, 0); the 8 elements of that group take the eight 16-bit halves of the four
 * output words in order (element kk % 8 = j: word j / 2, low half if j is even). */
uint32_t orc_sr_bits(uint64_t seed, int64_t o, int64_t kk)
{
    uint32_t ctr[4] = {(uint32_t)o, (uint32_t)(kk / 8), 0u, 0u};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t w[4];
    orc_philox4x32_10(ctr, key, w);
    int j = (int)(kk % 8);
    return (w[j / 2] >> (16 * (j % 2))) & 0xffffu;
}

/* Stochastic rounding of q to E2M1 with the 16-bit uniform number r16: |q| >= 6 saturates; otherwise with
 * lo <= |q| < hi the neighbouring representable magnitudes, the result is hi with probability
 * (|q| - lo) / (hi - lo) -- taken as "r16 / 65536 < that fraction" -- else lo.  Sign bit as in the
 * deterministic encoder.  A representable |q| is never moved. */
uint8_t orc_e2m1_encode_sr(float q, uint32_t r16)
{
    uint32_t u;
    memcpy(&u, &q, sizeof u);
    uint8_t sign = (uint8_t)((u >> 31) << 3);
    float a = fabsf(q);
    if (a >= 6.0f) return (uint8_t)(sign | 7);
    int lo = 0;
    while (lo < 6 && (float)E2M1_VALUE[lo + 1] <= a) ++lo;
    float vlo = (float)E2M1_VALUE[lo], vhi = (float)E2M1_VALUE[lo + 1];
    float frac = (a - vlo) / (vhi - vlo);
    float draw = (float)r16 / 65536.0f;
    return (uint8_t)(sign | (uint8_t)(draw < frac ? lo + 1 : lo));
}

/* ------------------------------------------------------------------ mask -> IHT -> quantise */

/* The fp32 values that get quantised: row o of the operand with masked entries set to zero
 * (the OE residual, Eq. 7-8), then the block transform along K (iht_block = 0: no transform).
 * out is [outer, K] row-major. */
void orc_transform(const uint16_t *data, int64_t outer, int64_t K, int64_t ld, int k_contig,
                   int iht_block, const uint8_t *zero_outer, const uint8_t *zero_k, float *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < outer; ++o) {
        float *row = out + o * K;
        int row_zero = zero_outer && zero_outer[o];
        for (int64_t kk = 0; kk < K; ++kk) {
            float x = op_at(data, ld, k_contig, o, kk);
            if (row_zero || (zero_k && zero_k[kk])) x = 0.0f;
            row[kk] = x;
        }
        if (iht_block > 0)
            for (int64_t k0 = 0; k0 < K; k0 += iht_block)
                orc_fwht(row + k0, iht_block);
    }
}

/* codes: [outer, K/2], scales: [outer, K/32], both K-contiguous whatever the input layout. */
void orc_iht_quantize(const uint16_t *data, int64_t outer, int64_t K, int64_t ld, int k_contig,
                      int iht_block, const uint8_t *zero_outer, const uint8_t *zero_k,
                      uint8_t *codes, uint8_t *scales)
{
#pragma omp parallel
    {
        float *row = (float *)malloc((size_t)K * sizeof *row);
#pragma omp for schedule(static)
        for (int64_t o = 0; o < outer; ++o) {
            int row_zero = zero_outer && zero_outer[o];
            for (int64_t kk = 0; kk < K; ++kk) {
                float x = op_at(data, ld, k_contig, o, kk);
                if (row_zero || (zero_k && zero_k[kk])) x = 0.0f;
                row[kk] = x;
            }
            if (iht_block > 0)
                for (int64_t k0 = 0; k0 < K; k0 += iht_block)
                    orc_fwht(row + k0, iht_block);
            for (int64_t blk = 0; blk < K / 32; ++blk)
                orc_mx_quantize_block(row + 32 * blk, codes + o * (K / 2) + 16 * blk,
                                      scales + o * (K / 32) + blk);
        }
        free(row);
    }
}

/* As orc_iht_quantize, with the elements rounded stochastically (scales as before: amax rule). */
void orc_iht_quantize_sr(const uint16_t *data, int64_t outer, int64_t K, int64_t ld, int k_contig,
                         int iht_block, const uint8_t *zero_outer, const uint8_t *zero_k, uint64_t seed,
                         uint8_t *codes, uint8_t *scales)
{
    float *t = (float *)malloc((size_t)outer * (size_t)K * sizeof *t);
    orc_transform(data, outer, K, ld, k_contig, iht_block, zero_outer, zero_k, t);
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < outer; ++o) {
        for (int64_t blk = 0; blk < K / 32; ++blk) {
            const float *v = t + o * K + 32 * blk;
            float amax = 0.0f;
            for (int i = 0; i < 32; ++i) {
                float a = fabsf(v[i]);
                if (a > amax) amax = a;
            }
            uint8_t s = orc_e8m0_from_amax(amax);
            float X = ldexpf(1.0f, (int)s - 127);
            for (int i = 0; i < 32; i += 2) {
                uint8_t lo = orc_e2m1_encode_sr(v[i] / X, orc_sr_bits(seed, o, 32 * blk + i));
                uint8_t hi = orc_e2m1_encode_sr(v[i + 1] / X, orc_sr_bits(seed, o, 32 * blk + i + 1));
                codes[o * (K / 2) + 16 * blk + i / 2] = (uint8_t)(lo | (hi << 4));
            }
            scales[o * (K / 32) + blk] = s;
        }
    }
    free(t);
}

/* ------------------------------------------------------------------ OHT (Eq. 6), operand side */

/* The fp32 values that get quantised under the Outer Hadamard Transform: H_m A for the A operand,
 * (B H_n)^T = H_n B^T for B given as [N, K] -- in both cases the block transform runs along the
 * OUTER index: for every K index, every block of b consecutive outer indices is multiplied by the
 * normalised Sylvester matrix (same butterflies, same rounding order as the inner transform).
 * outer % b == 0.  out is [outer, K] row-major. */
void orc_oht_transform(const uint16_t *data, int64_t outer, int64_t K, int64_t ld, int k_contig, int b, float *out)
{
#pragma omp parallel
    {
        float *col = (float *)malloc((size_t)b * sizeof *col);
#pragma omp for schedule(static)
        for (int64_t kk = 0; kk < K; ++kk) {
            for (int64_t o0 = 0; o0 < outer; o0 += b) {
                for (int i = 0; i < b; ++i) col[i] = op_at(data, ld, k_contig, o0 + i, kk);
                orc_fwht(col, b);
                for (int i = 0; i < b; ++i) out[(o0 + i) * K + kk] = col[i];
            }
        }
        free(col);
    }
}

/* OHT-transformed operand -> MXFP4, MX blocks along K as everywhere (codes [outer, K/2], scales [outer, K/32]). */
void orc_oht_quantize(const uint16_t *data, int64_t outer, int64_t K, int64_t ld, int k_contig, int b,
                      uint8_t *codes, uint8_t *scales)
{
    float *t = (float *)malloc((size_t)outer * (size_t)K * sizeof *t);
    orc_oht_transform(data, outer, K, ld, k_contig, b, t);
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < outer; ++o)
        for (int64_t blk = 0; blk < K / 32; ++blk)
            orc_mx_quantize_block(t + o * K + 32 * blk, codes + o * (K / 2) + 16 * blk, scales + o * (K / 32) + blk);
    free(t);
}

/* ------------------------------------------------------------------ GEMMs in double */

/* Dequantise row o of a packed operand into dst[K] (value(code) * 2^(scale-127), exact). */
static void dequant_row(const uint8_t *codes, const uint8_t *scales, int64_t K, int64_t o, double *dst)
{
    for (int64_t kk = 0; kk < K; ++kk) {
        uint8_t byte = codes[o * (K / 2) + kk / 2];
        uint8_t code = (kk & 1) ? (uint8_t)(byte >> 4) : (uint8_t)(byte & 15);
        int s = scales[o * (K / 32) + kk / 32];
        dst[kk] = ldexp(e2m1_decode(code), s - 127);
    }
}

/* out[r, c] = sum_kk Ahat[rows[r], kk] * Bhat[cols[c], kk]  (Eq. 4 with the quantised operands
 * of Eq. 5 / 7 / 8).  rows / cols select which outputs are computed; NULL means 0..n-1. */
void orc_mx_gemm(int64_t K, const uint8_t *a_codes, const uint8_t *a_scales, const uint8_t *b_codes,
                 const uint8_t *b_scales, const int32_t *rows, int64_t nrows, const int32_t *cols,
                 int64_t ncols, double *out)
{
    double *Ah = (double *)malloc((size_t)(nrows * K) * sizeof *Ah);
    double *Bh = (double *)malloc((size_t)(ncols * K) * sizeof *Bh);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < nrows; ++r)
        dequant_row(a_codes, a_scales, K, rows ? rows[r] : r, Ah + r * K);
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < ncols; ++c)
        dequant_row(b_codes, b_scales, K, cols ? cols[c] : c, Bh + c * K);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < nrows; ++r)
        for (int64_t c = 0; c < ncols; ++c) {
            double acc = 0.0;
            for (int64_t kk = 0; kk < K; ++kk)
                acc += Ah[r * K + kk] * Bh[c * K + kk];
            out[r * ncols + c] = acc;
        }
    free(Ah);
    free(Bh);
}

/* Double-precision product on the original bf16 values:
 *   out[r, c] = sum over kk in ksel (or all K) of A'[rows[r], kk] * B'[cols[c], kk]
 * where A' / B' are A / B with the masked rows and K indices set to zero (NULL masks: nothing
 * zeroed).  With no masks and no ksel this is the exact product A*B (Eq. 4's left-hand side);
 * with ksel = S it is the K-channel outlier part A[:,S] B[S,:]; with rows restricted to S it is
 * A_out*B of Eq. 7; with cols restricted to S it is A*B_out of Eq. 8; with masks it is the
 * unquantised residual product. */
void orc_bf16_gemm(const uint16_t *a, int64_t a_ld, int a_k_contig, const uint16_t *b, int64_t b_ld,
                   int b_k_contig, int64_t K, const uint8_t *a_zero_outer, const uint8_t *b_zero_outer,
                   const uint8_t *zero_k, const int32_t *ksel, int64_t nk, const int32_t *rows,
                   int64_t nrows, const int32_t *cols, int64_t ncols, double *out)
{
    int64_t kn = ksel ? nk : K;
    double *Ad = (double *)malloc((size_t)(nrows * kn + 1) * sizeof *Ad);
    double *Bd = (double *)malloc((size_t)(ncols * kn + 1) * sizeof *Bd);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < nrows; ++r) {
        int64_t o = rows ? rows[r] : r;
        for (int64_t t = 0; t < kn; ++t) {
            int64_t kk = ksel ? ksel[t] : t;
            double x = (double)op_at(a, a_ld, a_k_contig, o, kk);
            if ((a_zero_outer && a_zero_outer[o]) || (zero_k && zero_k[kk])) x = 0.0;
            Ad[r * kn + t] = x;
        }
    }
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < ncols; ++c) {
        int64_t o = cols ? cols[c] : c;
        for (int64_t t = 0; t < kn; ++t) {
            int64_t kk = ksel ? ksel[t] : t;
            double x = (double)op_at(b, b_ld, b_k_contig, o, kk);
            if ((b_zero_outer && b_zero_outer[o]) || (zero_k && zero_k[kk])) x = 0.0;
            Bd[c * kn + t] = x;
        }
    }
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < nrows; ++r)
        for (int64_t c = 0; c < ncols; ++c) {
            double acc = 0.0;
            for (int64_t t = 0; t < kn; ++t)
                acc += Ad[r * kn + t] * Bd[c * kn + t];
            out[r * ncols + c] = acc;
        }
    free(Ad);
    free(Bd);
}

int orc_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
