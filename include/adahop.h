/*
 * adahop.h -- C ABI of the MI355X (gfx950) AdaHOP per-GEMM hot path.
 *
 * One GEMM of a linear layer, C[M,N] = A[M,K] * B[K,N] (paper Eq. 1-4), computed as
 *
 *     C = Q(A_res H) * Q(H^T B_res)            MXFP4, block-scaled FP4 matrix cores
 *       + (extracted rows / columns / K-channels of the original operands)   BF16 matrix cores
 *
 * with H the block-diagonal normalised Sylvester Hadamard matrix along K (paper Eq. 5), Q the OCP
 * MX quantiser (E2M1 elements, one E8M0 scale per 32 consecutive K-elements), and the extracted
 * part chosen by a 64-sample variance score (paper Eq. 7-8, App. F).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller; the library allocates nothing
 *     and never synchronises: work is queued on `stream` (a hipStream_t passed as void*, NULL =
 *     the default stream) and the call returns.  No data is kept between calls.  The only state is
 *     a per-device "configured" flag per kernel family: the first call on a device that reaches a
 *     family with a large LDS footprint sets the function attributes of all its kernels and reads
 *     the device's compute-unit count (host-side HIP calls, no allocation, no synchronisation).
 *     adahop_prepare_device() does this for every family at once; call it (or make the first
 *     calls) outside a stream capture.
 *   - Sizes: 1 <= outer <= 2^21 and 32 <= K <= 2^21 for every operand (M, N, K of a product
 *     alike), and outer * K < 2^35; anything larger is ADAHOP_E_INVALID_ARG.
 *   - Outputs are fully overwritten.  Inputs are not modified.
 *   - Return value: ADAHOP_OK, or a negative adahop_status_t.  Arguments are validated before any
 *     HIP call, so ADAHOP_E_INVALID_ARG / ADAHOP_E_WORKSPACE can be exercised without a GPU.
 *     After ADAHOP_E_HIP, adahop_last_hip_error() returns the hipError_t of the failed call.
 *   - B is always described as its transpose: a logical [N, K] matrix, so that both operands are
 *     "outer x K" and K is the contraction axis.
 */
#ifndef ADAHOP_H
#define ADAHOP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ADAHOP_OK = 0,
    ADAHOP_E_INVALID_ARG = -1, /* null pointer, bad enum, K % 32 != 0, K % iht_block != 0, bad k, ld too small, misaligned */
    ADAHOP_E_WORKSPACE = -2,   /* workspace pointer null / misaligned / too small */
    ADAHOP_E_HIP = -3          /* a HIP launch or API call failed */
} adahop_status_t;

/* Per-GEMM strategy (paper Sec. 4.2; the caller supplies what the paper's calibration would). */
typedef enum {
    ADAHOP_NONE = 0,       /* C = Q(A) Q(B)                                   (Eq. 4)            */
    ADAHOP_IHT = 1,        /* C = Q(A H) Q(H^T B)                             (Eq. 5)            */
    ADAHOP_IHT_OE_ROW = 2, /* OE-Left : top-k rows of A in BF16              (Eq. 7)            */
    ADAHOP_IHT_OE_COL = 3, /* OE-Right: top-k columns of B in BF16           (Eq. 8)            */
    ADAHOP_IHT_OE_K = 4,   /* top-k K-channels (of A) in BF16, removed from both residuals       */
    ADAHOP_OHT = 5         /* C = H^T ( Q(H A) Q(B H) ) H^T, outer transforms (Eq. 6): comparison */
} adahop_strategy_t;

/* A bf16 matrix operand, logical shape [outer, K].
 *   k_contig = 1: element (o, kk) is data[o * ld + kk]   (ld >= K)
 *   k_contig = 0: element (o, kk) is data[kk * ld + o]   (ld >= outer)
 * The three products of a linear layer (Eq. 1-3) use: forward  A = X (k_contig), B = W (k_contig);
 * dgrad  A = G_Y (k_contig), B = W stored [K, N] (k_contig = 0);  wgrad  A = G_Y stored [K, M] and
 * B = X stored [K, N] (both k_contig = 0).
 * Alignment: data must be 16-byte aligned and ld a multiple of 8 elements. */
typedef struct {
    const void *data; /* device pointer to bf16 */
    int64_t outer;
    int64_t K;
    int64_t ld;       /* leading dimension in elements */
    int k_contig;
} adahop_operand_t;

/* ---------------------------------------------------------------------------------------------
 * Quantisers.  Canonical packed layout, K-contiguous whatever the input layout:
 *   codes  uint8 [outer, K/2]   byte t of a row = code(kk = 2t) | code(kk = 2t+1) << 4
 *   scales uint8 [outer, K/32]  E8M0, biased by 127
 * E2M1 code: bit 3 = sign, bits 0..2 index {0, .5, 1, 1.5, 2, 3, 4, 6}; round to nearest even,
 * saturating at 6.  Scale = 127 + floor(log2(amax)) - 2, clamped to [0, 254]; 0 for an all-zero
 * block (OCP Microscaling v1.0; the paper names the format in Sec. 1 and App. F item 2).
 * Requires K % 32 == 0.
 * ------------------------------------------------------------------------------------------- */

/* Plain MX quantisation along K (the operand side of Eq. 4). */
int adahop_quantize_mx(const adahop_operand_t *x, uint8_t *codes, uint8_t *scales, void *stream);

/* Fused residual masking -> block Hadamard transform -> MX quantisation (Eq. 5 applied to one
 * operand; App. F items 1-2).  iht_block in {0, 32, 64, 128, 256}; 0 = no transform; K % iht_block
 * must be 0.  The transform is fp32: butterflies in ascending stride, then one multiply by
 * (float)(1/sqrt(iht_block)).
 * zero_outer (length outer) / zero_k (length K): optional device byte masks; a nonzero byte means
 * that whole row / that K index is treated as 0 (the Outlier Extraction residual).  NULL = none.
 * zero_k must be 8-byte aligned. */
int adahop_iht_quantize(const adahop_operand_t *x, int iht_block, const uint8_t *zero_outer,
                        const uint8_t *zero_k, uint8_t *codes, uint8_t *scales, void *stream);

/* ---------------------------------------------------------------------------------------------
 * FOID (App. F item 1): score = sum of squared deviations from the mean over the first
 * min(64, len) elements (fp32: sequential sum, mean = sum * (1/len), sequential fused
 * multiply-add), then the exact top-k by (score descending, index ascending).
 *   axis = 0: score every outer index over its first 64 K-elements        (dim = outer)
 *   axis = 1: score every K index over its first 64 outer elements        (dim = K)
 * idx_out  int32 [k]    selected indices, ascending
 * mask_out uint8 [dim]  1 where selected, else 0 (8-byte aligned; usable as zero_outer / zero_k)
 * scores_ws float [dim] scratch for the scores (left filled on return)
 * 0 <= k <= dim.
 * ------------------------------------------------------------------------------------------- */
int adahop_foid_topk(const adahop_operand_t *x, int axis, int k, int32_t *idx_out, uint8_t *mask_out,
                     float *scores_ws, void *stream);

/* adahop_foid_topk for callers that cannot allocate device memory or hand over a scratch buffer (code under
 * stream capture, tight serving loops, harnesses that forbid allocation): same arguments and results, but the
 * scores go to a fixed array inside the library's device image instead of scores_ws.  The call allocates
 * and frees nothing.
 *   - Limit: dim (outer for axis 0, K for axis 1) <= ADAHOP_FOID_NOALLOC_MAX_DIM; beyond it the call returns
 *     ADAHOP_E_WORKSPACE and queues nothing.  The array takes ADAHOP_FOID_NOALLOC_MAX_DIM * 4 bytes (1 MiB) on
 *     every GPU the library runs on, until the process ends.
 *   - The first call on a device looks up the array's device address (a host-side HIP call, no allocation);
 *     later calls on that device reuse it.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two
 *     threads) race on it and must be serialised by the caller.  Calls in sequence on one stream are safe; the
 *     array keeps the previous call's scores, and every entry a call reads is written by that call first, so
 *     nothing needs clearing. */
#define ADAHOP_FOID_NOALLOC_MAX_DIM 262144
int adahop_foid_topk_noalloc(const adahop_operand_t *x, int axis, int k, int32_t *idx_out, uint8_t *mask_out,
                             void *stream);

/* ---------------------------------------------------------------------------------------------
 * Block-scaled FP4 product on packed operands (the MXFP4 term of Eq. 4 / 5 / 7 / 8):
 *   C[m, n] = sum_blk 2^(sa[m,blk]-127) 2^(sb[n,blk]-127) sum_{i<32} a[m, 32 blk + i] b[n, 32 blk + i]
 * fp32 accumulation and output, C row-major with leading dimension ldc >= N.
 * codes / scales in the canonical layout above; codes 16-byte aligned, K % 32 == 0.
 * workspace: device scratch of at least adahop_gemm_mx_workspace_bytes(M, N, K) bytes, 256-byte
 * aligned (the kernel keeps a re-ordered copy of the scales there); contents undefined on return.
 * With K % 256 == 0 and K >= 768 the whole 256x256 tiles of C take the tiled, LDS-pipelined kernel
 * and only the ragged edges a slower bounds-checked kernel; any other K takes the latter throughout.
 * ------------------------------------------------------------------------------------------- */
size_t adahop_gemm_mx_workspace_bytes(int64_t M, int64_t N, int64_t K);
int adahop_gemm_mx(int64_t M, int64_t N, int64_t K, const uint8_t *a_codes, const uint8_t *a_scales,
                   const uint8_t *b_codes, const uint8_t *b_scales, float *C, int64_t ldc, void *workspace,
                   size_t workspace_bytes, void *stream);

/* The same product with C rounded to bf16 (round to nearest even from the fp32 accumulators; the
 * paper's kernels also emit bf16): C is bf16 [M, ldc], 2-byte aligned.  The tiled kernel needs
 * ldc % 8 == 0 and C 16-byte aligned; otherwise the bounds-checked kernel runs. */
int adahop_gemm_mx_bf16out(int64_t M, int64_t N, int64_t K, const uint8_t *a_codes, const uint8_t *a_scales,
                           const uint8_t *b_codes, const uint8_t *b_scales, uint16_t *C, int64_t ldc,
                           void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * The whole path (App. F: FOID -> IHT + quantise -> MXFP4 product + BF16 outlier product -> sum).
 * A is [M, K], B is [N, K] (operand sense), C is fp32 [M, N] with leading dimension ldc.
 *   strategy NONE: iht_block is ignored.  OE strategies with k == 0 behave as ADAHOP_IHT.
 *   k counts extracted rows of A (OE_ROW, k <= M), columns of B (OE_COL, k <= N) or K-channels
 *   (OE_K, k <= K; scored on A over its first 64 rows and removed from both operands).
 *   idx_inout int32 [k]: if use_given_idx != 0 the k distinct indices are read from it (any order),
 *   else FOID fills it (ascending).  May be NULL when k == 0.
 * The BF16 part uses the original bf16 values with fp32 accumulation and is added in fp32.
 * The workspace holds, at the offsets reported by adahop_gemm_workspace_layout(), the canonical
 * codes and scales of both operands, the extraction mask and the FOID scores, all left in place on
 * return so that a caller can inspect or reuse them -- except that with ADAHOP_IHT_OE_K the region of the
 * scores may come back holding a 16-bit table of the selected channels' positions instead (the quantisers
 * use it to copy those channels out).
 * ------------------------------------------------------------------------------------------- */
typedef struct {
    size_t a_codes, a_scales, b_codes, b_scales; /* byte offsets into the workspace */
    size_t mask;                                 /* uint8 [extracted dim]           */
    size_t scores;                               /* float [extracted dim]           */
    size_t gather_a, gather_b;                   /* scratch of the BF16 part        */
    size_t gemm;                                 /* scratch of the MXFP4 product    */
    size_t total;                                /* bytes required                  */
} adahop_ws_layout_t;

int adahop_gemm_workspace_layout(int64_t M, int64_t N, int64_t K, adahop_strategy_t strategy, int k,
                                 adahop_ws_layout_t *out);
size_t adahop_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, adahop_strategy_t strategy, int k);

int adahop_gemm(const adahop_operand_t *A, const adahop_operand_t *B, float *C, int64_t ldc,
                adahop_strategy_t strategy, int iht_block, int k, int32_t *idx_inout, int use_given_idx,
                void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * adahop_iht_quantize with stochastic rounding of the elements -- an option for gradient operands (the
 * paper cites it as prior work for unbiased MXFP4 gradient estimates, Sec. 2.1-2.2; AdaHOP itself rounds
 * to nearest).  Scales as before (amax rule).  An element q = v / 2^(s-127) with |q| >= 6 saturates;
 * otherwise, lo <= |q| < hi being its neighbouring E2M1 magnitudes, it becomes hi if
 * r / 65536 < (|q| - lo) / (hi - lo) and lo otherwise (a representable |q| never moves; sign kept), with r
 * the 16-bit draw of that element: Philox4x32-10, key = (low, high) 32 bits of seed, counter =
 * (outer index, K index / 8, 0, 0), element K index % 8 = j taking the low (j even) or high (j odd) half
 * of output word j / 2.  The result depends on (seed, position) only: not on layout, launch shape or k.
 * ------------------------------------------------------------------------------------------- */
int adahop_iht_quantize_sr(const adahop_operand_t *x, int iht_block, const uint8_t *zero_outer,
                           const uint8_t *zero_k, uint64_t seed, uint8_t *codes, uint8_t *scales, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Outer Hadamard Transform (paper Eq. 6), the strategy the paper compares against:
 *     C_OHT = H_m^T ( Q(H_m A) Q(B H_n) ) H_n^T
 * with block-diagonal normalised Sylvester matrices of size oht_block in {32, 64, 128} on both outer
 * dimensions (same butterfly order and rounding as the inner transform).
 *   adahop_oht_quantize: operand x, logical [outer, K], outer % oht_block == 0: every block of oht_block
 *     consecutive OUTER indices is transformed for every K index (H_m A for A; H_n B^T for B given as
 *     [N, K]), then rows are quantised along K to canonical codes [outer, K/2] / scales [outer, K/32].
 *   adahop_oht_inverse: C (float [M, ldc], M % oht_block == 0, N % oht_block == 0) <- H^T C H^T in place.
 * adahop_gemm / adahop_gemm_ex with strategy ADAHOP_OHT run both operands through adahop_oht_quantize,
 * the MXFP4 product and adahop_oht_inverse; iht_block is then the OHT block, k is ignored, C must be
 * float (c_bf16 = 0) and M, N multiples of the block: INVALID_ARG otherwise.  outer / oht_block (M / oht_block
 * for adahop_oht_inverse) must not exceed 65535.
 * ------------------------------------------------------------------------------------------- */
int adahop_oht_quantize(const adahop_operand_t *x, int oht_block, uint8_t *codes, uint8_t *scales, void *stream);
int adahop_oht_inverse(float *C, int64_t M, int64_t N, int64_t ldc, int oht_block, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Quantise-once operand reuse and bf16 output (the paper's layers share operands between products:
 * one activation feeds several projections, a weight is constant over the micro-batches of a step;
 * App. F runs IHT + quantisation per operand, so its result can be kept).
 *
 * adahop_pack_operand: the residual -> IHT -> MXFP4 step of the whole path for ONE operand, into
 * caller-owned canonical codes [outer, K/2] / scales [outer, K/32].  is_b: 0 if x will be the A
 * operand, 1 if B.  strategy / iht_block as in adahop_gemm.  The residual of x depends on the
 * extracted indices only for (OE_ROW, A), (OE_COL, B) and (OE_K, either); then idx int32 [k] (device,
 * distinct, in range) names them and mask_ws is device scratch of `outer` (row / column kinds) or K
 * (OE_K) bytes, 8-byte aligned; otherwise k, idx and mask_ws are ignored.
 *
 * adahop_gemm_ex: adahop_gemm with options.  opts may be NULL (then identical to adahop_gemm).
 *   a_codes / a_scales (b_...): if non-NULL, A (B) is taken as packed by adahop_pack_operand with the
 *     same strategy, iht_block, k and indices, and is not quantised again; the bf16 operand is still
 *     required (FOID and the BF16 outlier product read it).  If the residual of a packed operand
 *     depends on the indices (see above) and k > 0, use_given_idx must be set: INVALID_ARG otherwise.
 *     The workspace regions of an operand packed by the caller are left untouched.
 *   c_bf16: 0: C is float [M, ldc]; 1: C is bf16 [M, ldc] (2-byte aligned), every element the fp32
 *     result rounded to nearest even once (the K-channel product is added before the rounding, the
 *     row / column product overwrites its rows / columns).
 *   sr_a / sr_b with sr_seed_a / sr_seed_b: the elements of that operand are rounded stochastically as
 *     by adahop_iht_quantize_sr (ignored for an operand packed by the caller and under ADAHOP_OHT).
 * Workspace size and layout are those of adahop_gemm.
 * ------------------------------------------------------------------------------------------- */
typedef struct {
    const uint8_t *a_codes, *a_scales;
    const uint8_t *b_codes, *b_scales;
    int c_bf16;
    int sr_a, sr_b;                 /* nonzero: quantise that operand with stochastic rounding (below) */
    uint64_t sr_seed_a, sr_seed_b;  /* seeds of the two streams                                       */
} adahop_gemm_opts_t;

int adahop_pack_operand(const adahop_operand_t *x, int is_b, adahop_strategy_t strategy, int iht_block, int k,
                        const int32_t *idx, uint8_t *mask_ws, uint8_t *codes, uint8_t *scales, void *stream);
int adahop_gemm_ex(const adahop_operand_t *A, const adahop_operand_t *B, void *C, int64_t ldc,
                   adahop_strategy_t strategy, int iht_block, int k, int32_t *idx_inout, int use_given_idx,
                   const adahop_gemm_opts_t *opts, void *workspace, size_t workspace_bytes, void *stream);

/* The BF16 outlier product alone (second term of Eq. 7 / Eq. 8 / the K-channel form), for callers
 * that keep quantised operands across products and for tests.
 *   kind OE_ROW: C[idx[t], :]  = A[idx[t], :] * B          (overwrites those rows)
 *   kind OE_COL: C[:, idx[t]]  = A * B[:, idx[t]]          (overwrites those columns)
 *   kind OE_K  : C            += A[:, idx] * B[idx, :]     (accumulates)
 * idx int32 [k] device, distinct, in range.  gather_ws: device scratch of at least
 * adahop_oe_gather_bytes(M, N, K, kind, k) bytes, 256-byte aligned (the gathered rows / columns /
 * K-channels and, for OE_ROW and OE_COL, the partial products of the K slices); contents undefined
 * on return. */
size_t adahop_oe_gather_bytes(int64_t M, int64_t N, int64_t K, adahop_strategy_t kind, int k);
int adahop_oe_gemm_bf16(const adahop_operand_t *A, const adahop_operand_t *B, adahop_strategy_t kind,
                        const int32_t *idx, int k, float *C, int64_t ldc, void *gather_ws,
                        size_t gather_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Outlier-pattern detection of one tensor and the pattern-pair -> strategy table (paper Sec. 4.1,
 * 4.2, App. A) -- what the paper's 30-step calibration evaluates per tensor and per step; the
 * majority vote over the steps is adahop_vote_pattern below (host-side), the table
 * adahop_select_strategy.
 *
 * For the operand in its logical [outer, K] shape: v_outer[o] = variance of x[o, :], v_k[kk] =
 * variance of x[:, kk] (population variances, fp64), CV = std(v) / (mean(v) + 1e-12) for each vector,
 * CV^_outer = CV_outer / sqrt(2 / (K - 1)), CV^_k = CV_k / sqrt(2 / (outer - 1)), and
 *   ADAHOP_PATTERN_OUTER if CV^_outer / CV^_k > tau   (whole rows of A / whole columns of B stand out:
 *                                                      the paper's Row-wise for A, Column-wise for B)
 *   ADAHOP_PATTERN_K     if CV^_k / CV^_outer > tau   (whole K-channels: Column-wise for A, Row-wise for B)
 *   ADAHOP_PATTERN_NONE  otherwise.                    A ratio with a zero denominator counts as
 *                                                      infinite if its numerator is positive, else 0.
 * pattern_out: one device int32; stats_out: four device doubles (CV_outer, CV_k, CV^_outer, CV^_k).
 * Requires outer >= 2 and K >= 32.  workspace: adahop_detect_pattern_workspace_bytes(x) bytes, 256-byte
 * aligned, contents undefined on return.
 * ------------------------------------------------------------------------------------------- */
typedef enum { ADAHOP_PATTERN_NONE = 0, ADAHOP_PATTERN_OUTER = 1, ADAHOP_PATTERN_K = 2 } adahop_pattern_t;

size_t adahop_detect_pattern_workspace_bytes(const adahop_operand_t *x);
int adahop_detect_pattern(const adahop_operand_t *x, double tau, int32_t *pattern_out, double *stats_out,
                          void *workspace, size_t workspace_bytes, void *stream);

/* The calibrated pattern of a tensor from its per-step classifications (Sec. 4.1: the paper classifies every
 * tensor at each of 30 calibration steps and keeps the majority).  patterns: HOST array of n values of
 * adahop_pattern_t (what adahop_detect_pattern wrote, copied back by the caller).  Returns the class that
 * occurs most often; when several classes share the top count, ADAHOP_PATTERN_NONE.  Host-side, no GPU work.
 * Returns ADAHOP_E_INVALID_ARG (negative) for a null array, n < 1 or a value outside the enum. */
int adahop_vote_pattern(const int32_t *patterns, int n);

/* Strategy for the product of A and B from their patterns (Sec. 4.2; host-side, no GPU work):
 *   B outer-wise (the paper's RC, NC, CC)              -> ADAHOP_IHT_OE_COL  (OE-Right)
 *   else A outer-wise (RN; RR by the same argument)    -> ADAHOP_IHT_OE_ROW  (OE-Left)
 *   else (CN, NN, CR; NR)                              -> ADAHOP_IHT
 * level 2 (AdaHOP-Lv2) computes the CC pair (A K-wise, B outer-wise) fully in BF16: *full_bf16 is set
 * to 1 and the return value is ADAHOP_NONE; in every other case *full_bf16 = 0.  level must be 1 or 2;
 * returns ADAHOP_E_INVALID_ARG (as a negative value) on bad arguments. */
int adahop_select_strategy(adahop_pattern_t pattern_a, adahop_pattern_t pattern_b, int level, int *full_bf16);

/* hipError_t (as int) of the most recent failed HIP call on this thread, 0 if none. */
int adahop_last_hip_error(void);
const char *adahop_status_string(int status);
/* ABI version: bumped on any incompatible change. */
int adahop_abi_version(void);

/* One-time set-up of the current device for every kernel of the library (function attributes, compute-unit
 * count, address of the built-in scratch of adahop_foid_topk_noalloc): host-side HIP calls only, nothing is
 * queued or allocated.  Optional -- every entry point does the part it needs at its first call on a device --
 * but a caller that captures streams into graphs calls it once per device beforehand, so that no later call has
 * set-up left to do.  Returns ADAHOP_OK or ADAHOP_E_HIP. */
int adahop_prepare_device(void);

/* =============================================================================================
 * DIAGNOSTICS -- not part of the method and not needed by a user of the product path.
 * =============================================================================================
 * Measurement aid: launches `workgroups` x 4 waves that each run
 * iters x 16 block-scaled FP4 matrix-core instructions (32x32x64, 131072 flop each) on register
 * operands only -- constant bits, or pseudo-random bits if random_operands != 0 -- so that a caller
 * timing the launch obtains the rate the matrix cores sustain on this machine without any memory
 * traffic: 2 * 65536 * 16 * iters * 4 * workgroups flop.  idle_sleeps (0..64): that many short sleeps
 * after every 16 instructions, to see how the rate responds to idle stretches under the power limit.
 * sink: one device float (never written in practice).  Used by bench.py to report the power-limited
 * ceiling beside the published peak. */
int adahop_probe_mfma_rate(int random_operands, int idle_sleeps, int workgroups, int iters, float *sink,
                           void *stream);

/* Measurement aid: which tiled kernel the MXFP4 product uses from now on (process-wide).  0 = chosen by shape (the
 * default), 1 = always the 256 x 256 tile kernel, 2 = the 256 x 128 tile kernel with two accumulator sets wherever it
 * can run (fp32 C, K % 256 == 0, K >= 2048, no K-channel extraction).  3 .. 6 = kernel chosen by shape, and the
 * 256 x 256 kernel walks its tiles in a forced order: 3 = bands of A in XCD-contiguous runs, 4 = bands of A swept
 * over B, 5 / 6 = the same two with the roles of A and B exchanged (a sweep that the shape does not allow falls back
 * to the contiguous runs).  By default the bands run along the operand with more tiles, swept where more of it would
 * be in use at a time than stays in the Infinity Cache.  Results are the same up to fp32 summation order (3 .. 6: the
 * same bits).  Returns ADAHOP_E_INVALID_ARG for any other value. */
int adahop_debug_force_gemm_kernel(int which);

#ifdef __cplusplus
}
#endif
#endif /* ADAHOP_H */
