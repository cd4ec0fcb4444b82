// extern "C" entry points of the AdaHOP library: argument validation (before any HIP call),
// workspace layout, and the per-GEMM pipeline of paper App. F (FOID -> IHT + quantise -> MXFP4
// product + BF16 outlier product -> sum) queued on one stream.
#include "common.h"

namespace adahop {

static thread_local int g_last_hip_error = 0;
void set_last_hip_error(int e) { g_last_hip_error = e; }

// Largest operand extents.  They keep every launch legal: the second grid dimension of a launch may not exceed
// 65535, and the kernels put K / 256 (fast quantisers), K / 128 (general K-strided quantiser: K / 32 blocks over
// 4 waves) and stored rows / 256 (pattern detector) there.  The OHT kernels put outer / block there and check it
// themselves (oht_grid_ok).
static const int64_t MAX_OUTER = (int64_t)1 << 21;
static const int64_t MAX_K = (int64_t)1 << 21;

bool valid_iht_block(int b) { return b == 0 || b == 32 || b == 64 || b == 128 || b == 256; }

int validate_operand(const adahop_operand_t *x)
{
    if (!x || !x->data) return ADAHOP_E_INVALID_ARG;
    if (x->outer < 1 || x->K < 32 || x->outer > MAX_OUTER || x->K > MAX_K) return ADAHOP_E_INVALID_ARG;
    if (x->K % 32 != 0) return ADAHOP_E_INVALID_ARG;
    if (x->k_contig != 0 && x->k_contig != 1) return ADAHOP_E_INVALID_ARG;
    if (x->ld < (x->k_contig ? x->K : x->outer) || x->ld % 8 != 0) return ADAHOP_E_INVALID_ARG;
    if (!aligned(x->data, 16)) return ADAHOP_E_INVALID_ARG;
    if (x->outer * (x->K / 8) >= ((int64_t)1 << 32)) return ADAHOP_E_INVALID_ARG;
    return ADAHOP_OK;
}

// gathered K-channels are zero-padded to whole 64-channel pipeline stages of the GEMM
static int kpad_of(int k) { return (k + 63) / 64 * 64; }

static int extracted_dim(adahop_strategy_t s, int64_t M, int64_t N, int64_t K, int64_t *dim)
{
    switch (s) {
    case ADAHOP_NONE:
    case ADAHOP_OHT:
    case ADAHOP_IHT: *dim = 0; return ADAHOP_OK;
    case ADAHOP_IHT_OE_ROW: *dim = M; return ADAHOP_OK;
    case ADAHOP_IHT_OE_COL: *dim = N; return ADAHOP_OK;
    case ADAHOP_IHT_OE_K: *dim = K; return ADAHOP_OK;
    }
    return ADAHOP_E_INVALID_ARG;
}

} // namespace adahop

using namespace adahop;

extern "C" {

int adahop_abi_version(void) { return 1; }

int adahop_debug_force_gemm_kernel(int which)
{
    if (which < 0 || which > 6) return ADAHOP_E_INVALID_ARG;
    gemm_mx_force_kernel(which);
    return ADAHOP_OK;
}

int adahop_prepare_device(void)
{
    int rc;
    if ((rc = configure_gemm_mx(nullptr)) != ADAHOP_OK || (rc = configure_gemm_mx_dual(nullptr)) != ADAHOP_OK ||
        (rc = configure_oe_rowcol()) != ADAHOP_OK || (rc = configure_oht()) != ADAHOP_OK ||
        (rc = configure_quantizers()) != ADAHOP_OK || (rc = configure_foid()) != ADAHOP_OK)
        return rc;
    float *scores = nullptr;
    return foid_static_scores(&scores); // the address of the built-in score scratch, looked up once per device
}

int adahop_last_hip_error(void) { return g_last_hip_error; }

const char *adahop_status_string(int status)
{
    switch (status) {
    case ADAHOP_OK: return "ok";
    case ADAHOP_E_INVALID_ARG: return "invalid argument";
    case ADAHOP_E_WORKSPACE: return "workspace missing, misaligned or too small";
    case ADAHOP_E_HIP: return "HIP call failed (see adahop_last_hip_error)";
    default: return "unknown status";
    }
}

static int iht_quantize_checked(const adahop_operand_t *x, int iht_block, const uint8_t *zero_outer,
                                const uint8_t *zero_k, uint8_t *codes, uint8_t *scales, void *stream,
                                const uint64_t *sr_seed)
{
    int rc = validate_operand(x);
    if (rc != ADAHOP_OK) return rc;
    if (!codes || !scales || !valid_iht_block(iht_block)) return ADAHOP_E_INVALID_ARG;
    if (iht_block > 0 && x->K % iht_block != 0) return ADAHOP_E_INVALID_ARG;
    if (!aligned(codes, 16) || (zero_k && !aligned(zero_k, 8))) return ADAHOP_E_INVALID_ARG;
    return launch_iht_quantize(*x, iht_block, zero_outer, zero_k, codes, scales, static_cast<hipStream_t>(stream),
                               sr_seed);
}

int adahop_iht_quantize(const adahop_operand_t *x, int iht_block, const uint8_t *zero_outer, const uint8_t *zero_k,
                        uint8_t *codes, uint8_t *scales, void *stream)
{
    return iht_quantize_checked(x, iht_block, zero_outer, zero_k, codes, scales, stream, nullptr);
}

int adahop_iht_quantize_sr(const adahop_operand_t *x, int iht_block, const uint8_t *zero_outer,
                           const uint8_t *zero_k, uint64_t seed, uint8_t *codes, uint8_t *scales, void *stream)
{
    return iht_quantize_checked(x, iht_block, zero_outer, zero_k, codes, scales, stream, &seed);
}

int adahop_quantize_mx(const adahop_operand_t *x, uint8_t *codes, uint8_t *scales, void *stream)
{
    return adahop_iht_quantize(x, 0, nullptr, nullptr, codes, scales, stream);
}

int adahop_foid_topk(const adahop_operand_t *x, int axis, int k, int32_t *idx_out, uint8_t *mask_out, float *scores_ws,
                     void *stream)
{
    int rc = validate_operand(x);
    if (rc != ADAHOP_OK) return rc;
    if (axis != 0 && axis != 1) return ADAHOP_E_INVALID_ARG;
    const int64_t dim = axis == 0 ? x->outer : x->K;
    if (k < 0 || k > dim || !mask_out || !scores_ws || (k > 0 && !idx_out)) return ADAHOP_E_INVALID_ARG;
    if (!aligned(mask_out, 8) || !aligned(scores_ws, 4)) return ADAHOP_E_INVALID_ARG;
    return launch_foid_topk(*x, axis, k, idx_out, mask_out, scores_ws, static_cast<hipStream_t>(stream));
}

int adahop_foid_topk_noalloc(const adahop_operand_t *x, int axis, int k, int32_t *idx_out, uint8_t *mask_out,
                             void *stream)
{
    int rc = validate_operand(x);
    if (rc != ADAHOP_OK) return rc;
    if (axis != 0 && axis != 1) return ADAHOP_E_INVALID_ARG;
    const int64_t dim = axis == 0 ? x->outer : x->K;
    if (dim > ADAHOP_FOID_NOALLOC_MAX_DIM) return ADAHOP_E_WORKSPACE; // beyond the built-in scratch
    if (k < 0 || k > dim || !mask_out || (k > 0 && !idx_out) || !aligned(mask_out, 8)) return ADAHOP_E_INVALID_ARG;
    float *scores = nullptr;
    rc = foid_static_scores(&scores);
    if (rc != ADAHOP_OK) return rc;
    return launch_foid_topk(*x, axis, k, idx_out, mask_out, scores, static_cast<hipStream_t>(stream));
}

size_t adahop_gemm_mx_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (M < 1 || N < 1 || K < 32 || K % 32 != 0 || M > MAX_OUTER || N > MAX_OUTER || K > MAX_K) return 0;
    return gemm_mx_workspace_bytes(M, N, K);
}

static int gemm_mx_checked(int64_t M, int64_t N, int64_t K, const uint8_t *a_codes, const uint8_t *a_scales,
                           const uint8_t *b_codes, const uint8_t *b_scales, void *C, int64_t ldc, int c_bf16,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    if (M < 1 || N < 1 || K < 32 || K % 32 != 0 || M > MAX_OUTER || N > MAX_OUTER || K > MAX_K)
        return ADAHOP_E_INVALID_ARG;
    if (!a_codes || !a_scales || !b_codes || !b_scales || !C || ldc < N) return ADAHOP_E_INVALID_ARG;
    if (!aligned(a_codes, 16) || !aligned(b_codes, 16) || !aligned(C, c_bf16 ? 2 : 4)) return ADAHOP_E_INVALID_ARG;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < gemm_mx_workspace_bytes(M, N, K))
        return ADAHOP_E_WORKSPACE;
    return launch_gemm_mx(M, N, K, a_codes, a_scales, b_codes, b_scales, C, ldc, c_bf16, nullptr, nullptr, 0, workspace,
                          static_cast<hipStream_t>(stream));
}

int adahop_gemm_mx(int64_t M, int64_t N, int64_t K, const uint8_t *a_codes, const uint8_t *a_scales,
                   const uint8_t *b_codes, const uint8_t *b_scales, float *C, int64_t ldc, void *workspace,
                   size_t workspace_bytes, void *stream)
{
    return gemm_mx_checked(M, N, K, a_codes, a_scales, b_codes, b_scales, C, ldc, 0, workspace, workspace_bytes, stream);
}

int adahop_gemm_mx_bf16out(int64_t M, int64_t N, int64_t K, const uint8_t *a_codes, const uint8_t *a_scales,
                           const uint8_t *b_codes, const uint8_t *b_scales, uint16_t *C, int64_t ldc, void *workspace,
                           size_t workspace_bytes, void *stream)
{
    return gemm_mx_checked(M, N, K, a_codes, a_scales, b_codes, b_scales, C, ldc, 1, workspace, workspace_bytes, stream);
}


int adahop_gemm_workspace_layout(int64_t M, int64_t N, int64_t K, adahop_strategy_t strategy, int k,
                                 adahop_ws_layout_t *out)
{
    if (!out || M < 1 || N < 1 || K < 32 || K % 32 != 0 || M > MAX_OUTER || N > MAX_OUTER || K > MAX_K)
        return ADAHOP_E_INVALID_ARG;
    int64_t dim = 0;
    if (extracted_dim(strategy, M, N, K, &dim) != ADAHOP_OK) return ADAHOP_E_INVALID_ARG;
    if (k < 0 || (dim > 0 && k > dim)) return ADAHOP_E_INVALID_ARG;
    size_t off = 0;
    auto take = [&off](size_t bytes) {
        size_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    };
    out->a_codes = take((size_t)M * (K / 2));
    out->a_scales = take((size_t)M * (K / 32));
    out->b_codes = take((size_t)N * (K / 2));
    out->b_scales = take((size_t)N * (K / 32));
    out->mask = take((size_t)dim);
    out->scores = take((size_t)dim * sizeof(float));
    const bool oek = strategy == ADAHOP_IHT_OE_K && k > 0;
    const bool oerc = (strategy == ADAHOP_IHT_OE_ROW || strategy == ADAHOP_IHT_OE_COL) && k > 0;
    out->gather_a = take(oek ? (size_t)M * kpad_of(k) * 2 : oerc ? oe_rowcol_workspace_bytes(M, N, K, strategy, k) : 0);
    out->gather_b = take(oek ? (size_t)N * kpad_of(k) * 2 : 0);
    out->gemm = take(gemm_mx_workspace_bytes(M, N, K));
    out->total = off;
    return ADAHOP_OK;
}

size_t adahop_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, adahop_strategy_t strategy, int k)
{
    adahop_ws_layout_t l;
    if (adahop_gemm_workspace_layout(M, N, K, strategy, k, &l) != ADAHOP_OK) return 0;
    return l.total;
}

size_t adahop_oe_gather_bytes(int64_t M, int64_t N, int64_t K, adahop_strategy_t kind, int k)
{
    if (k <= 0 || M < 1 || N < 1 || K < 1) return 0;
    if (kind == ADAHOP_IHT_OE_ROW || kind == ADAHOP_IHT_OE_COL) return oe_rowcol_workspace_bytes(M, N, K, kind, k);
    if (kind != ADAHOP_IHT_OE_K) return 0;
    return align_up((size_t)M * kpad_of(k) * 2, 256) + align_up((size_t)N * kpad_of(k) * 2, 256);
}

static int validate_pair(const adahop_operand_t *A, const adahop_operand_t *B, const void *C, int64_t ldc,
                         size_t c_align = 4)
{
    int rc = validate_operand(A);
    if (rc != ADAHOP_OK) return rc;
    rc = validate_operand(B);
    if (rc != ADAHOP_OK) return rc;
    if (A->K != B->K || !C || ldc < B->outer || !aligned(C, c_align)) return ADAHOP_E_INVALID_ARG;
    return ADAHOP_OK;
}

int adahop_oe_gemm_bf16(const adahop_operand_t *A, const adahop_operand_t *B, adahop_strategy_t kind,
                        const int32_t *idx, int k, float *C, int64_t ldc, void *gather_ws, size_t gather_bytes,
                        void *stream)
{
    int rc = validate_pair(A, B, C, ldc);
    if (rc != ADAHOP_OK) return rc;
    int64_t dim = 0;
    if (extracted_dim(kind, A->outer, B->outer, A->K, &dim) != ADAHOP_OK || dim == 0) return ADAHOP_E_INVALID_ARG;
    if (k < 0 || k > dim || (k > 0 && !idx)) return ADAHOP_E_INVALID_ARG;
    if (k == 0) return ADAHOP_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t need = adahop_oe_gather_bytes(A->outer, B->outer, A->K, kind, k);
    if (!gather_ws || !aligned(gather_ws, 256) || gather_bytes < need) return ADAHOP_E_WORKSPACE;
    if (kind != ADAHOP_IHT_OE_K) return launch_oe_rowcol(*A, *B, kind, idx, k, C, ldc, 0, gather_ws, st);
    const int kpad = kpad_of(k);
    uint16_t *Ag = static_cast<uint16_t *>(gather_ws);
    uint16_t *Bg = reinterpret_cast<uint16_t *>(static_cast<char *>(gather_ws) + align_up((size_t)A->outer * kpad * 2, 256));
    rc = launch_gather_k(*A, idx, k, kpad, Ag, st);
    if (rc != ADAHOP_OK) return rc;
    rc = launch_gather_k(*B, idx, k, kpad, Bg, st);
    if (rc != ADAHOP_OK) return rc;
    return launch_oe_k_accumulate(A->outer, B->outer, Ag, Bg, kpad, C, ldc, st);
}

size_t adahop_detect_pattern_workspace_bytes(const adahop_operand_t *x)
{
    if (validate_operand(x) != ADAHOP_OK || x->outer < 2) return 0;
    return pattern_workspace_bytes(*x);
}

int adahop_detect_pattern(const adahop_operand_t *x, double tau, int32_t *pattern_out, double *stats_out,
                          void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = validate_operand(x);
    if (rc != ADAHOP_OK) return rc;
    if (x->outer < 2 || !(tau > 0.0) || !pattern_out || !stats_out || !aligned(stats_out, 8) || !aligned(pattern_out, 4))
        return ADAHOP_E_INVALID_ARG;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < pattern_workspace_bytes(*x)) return ADAHOP_E_WORKSPACE;
    return launch_detect_pattern(*x, tau, 1e-12, pattern_out, stats_out, workspace, static_cast<hipStream_t>(stream));
}

int adahop_vote_pattern(const int32_t *patterns, int n)
{
    if (!patterns || n < 1) return ADAHOP_E_INVALID_ARG;
    int count[3] = {0, 0, 0};
    for (int i = 0; i < n; ++i) {
        if (patterns[i] < ADAHOP_PATTERN_NONE || patterns[i] > ADAHOP_PATTERN_K) return ADAHOP_E_INVALID_ARG;
        ++count[patterns[i]];
    }
    int best = ADAHOP_PATTERN_NONE;
    for (int c = ADAHOP_PATTERN_OUTER; c <= ADAHOP_PATTERN_K; ++c)
        if (count[c] > count[best]) best = c;
    for (int c = ADAHOP_PATTERN_NONE; c <= ADAHOP_PATTERN_K; ++c)
        if (c != best && count[c] == count[best]) return ADAHOP_PATTERN_NONE; // no single most frequent class
    return best;
}

int adahop_select_strategy(adahop_pattern_t pattern_a, adahop_pattern_t pattern_b, int level, int *full_bf16)
{
    auto ok = [](int p) { return p == ADAHOP_PATTERN_NONE || p == ADAHOP_PATTERN_OUTER || p == ADAHOP_PATTERN_K; };
    if (!ok(pattern_a) || !ok(pattern_b) || (level != 1 && level != 2) || !full_bf16) return ADAHOP_E_INVALID_ARG;
    *full_bf16 = 0;
    if (pattern_b == ADAHOP_PATTERN_OUTER) {
        if (level == 2 && pattern_a == ADAHOP_PATTERN_K) {
            *full_bf16 = 1;
            return ADAHOP_NONE;
        }
        return ADAHOP_IHT_OE_COL;
    }
    if (pattern_a == ADAHOP_PATTERN_OUTER) return ADAHOP_IHT_OE_ROW;
    return ADAHOP_IHT;
}

// Which mask the residual of an operand needs under a strategy: 0 none, 1 over its outer index, 2 over K.
static int residual_mask_kind(adahop_strategy_t s, bool is_b)
{
    if (s == ADAHOP_IHT_OE_K) return 2;
    if (s == ADAHOP_IHT_OE_ROW && !is_b) return 1;
    if (s == ADAHOP_IHT_OE_COL && is_b) return 1;
    return 0;
}

int adahop_pack_operand(const adahop_operand_t *x, int is_b, adahop_strategy_t strategy, int iht_block, int k,
                        const int32_t *idx, uint8_t *mask_ws, uint8_t *codes, uint8_t *scales, void *stream)
{
    int rc = validate_operand(x);
    if (rc != ADAHOP_OK) return rc;
    if (strategy < ADAHOP_NONE || strategy > ADAHOP_OHT) return ADAHOP_E_INVALID_ARG;
    if (!codes || !scales || !aligned(codes, 16)) return ADAHOP_E_INVALID_ARG;
    if (strategy == ADAHOP_OHT) {
        if (!valid_oht_block(iht_block) || x->outer % iht_block != 0 || !oht_grid_ok(x->outer, iht_block))
            return ADAHOP_E_INVALID_ARG;
        return launch_oht_quantize(*x, iht_block, codes, scales, static_cast<hipStream_t>(stream));
    }
    const int b = strategy == ADAHOP_NONE ? 0 : iht_block;
    if (!valid_iht_block(b) || (b > 0 && x->K % b != 0)) return ADAHOP_E_INVALID_ARG;
    if (strategy != ADAHOP_NONE && b == 0) return ADAHOP_E_INVALID_ARG;
    const int kind = residual_mask_kind(strategy, is_b != 0);
    const int64_t dim = kind == 1 ? x->outer : x->K;
    const bool masked = kind != 0 && k != 0;
    if (masked && (k < 0 || k > dim || !idx || !mask_ws || !aligned(mask_ws, 8))) return ADAHOP_E_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (masked) {
        rc = launch_mask_from_idx(idx, k, mask_ws, dim, st);
        if (rc != ADAHOP_OK) return rc;
    }
    return launch_iht_quantize(*x, b, masked && kind == 1 ? mask_ws : nullptr, masked && kind == 2 ? mask_ws : nullptr,
                               codes, scales, st);
}

int adahop_oht_quantize(const adahop_operand_t *x, int oht_block, uint8_t *codes, uint8_t *scales, void *stream)
{
    int rc = validate_operand(x);
    if (rc != ADAHOP_OK) return rc;
    if (!valid_oht_block(oht_block) || x->outer % oht_block != 0 || !oht_grid_ok(x->outer, oht_block))
        return ADAHOP_E_INVALID_ARG;
    if (!codes || !scales || !aligned(codes, 16)) return ADAHOP_E_INVALID_ARG;
    return launch_oht_quantize(*x, oht_block, codes, scales, static_cast<hipStream_t>(stream));
}

int adahop_oht_inverse(float *C, int64_t M, int64_t N, int64_t ldc, int oht_block, void *stream)
{
    if (!C || !aligned(C, 4) || M < 1 || N < 1 || M > MAX_OUTER || N > MAX_OUTER || ldc < N) return ADAHOP_E_INVALID_ARG;
    if (!valid_oht_block(oht_block) || M % oht_block != 0 || N % oht_block != 0 || !oht_grid_ok(M, oht_block))
        return ADAHOP_E_INVALID_ARG;
    return launch_oht_inverse(C, M, N, ldc, oht_block, static_cast<hipStream_t>(stream));
}

static int gemm_whole_path(const adahop_operand_t *A, const adahop_operand_t *B, void *C, int64_t ldc,
                           adahop_strategy_t strategy, int iht_block, int k, int32_t *idx_inout, int use_given_idx,
                           const adahop_gemm_opts_t *opts, void *workspace, size_t workspace_bytes, void *stream)
{
    const int c_bf16 = opts ? opts->c_bf16 : 0;
    if (c_bf16 != 0 && c_bf16 != 1) return ADAHOP_E_INVALID_ARG;
    int rc = validate_pair(A, B, C, ldc, c_bf16 ? 2 : 4);
    if (rc != ADAHOP_OK) return rc;
    const int64_t M = A->outer, N = B->outer, K = A->K;
    int64_t dim = 0;
    if (extracted_dim(strategy, M, N, K, &dim) != ADAHOP_OK) return ADAHOP_E_INVALID_ARG;
    const bool oht = strategy == ADAHOP_OHT;
    const int b = strategy == ADAHOP_NONE ? 0 : iht_block;
    if (oht) {
        if (!valid_oht_block(b) || M % b != 0 || N % b != 0 || c_bf16 || !oht_grid_ok(M, b) || !oht_grid_ok(N, b))
            return ADAHOP_E_INVALID_ARG;
    } else {
        if (!valid_iht_block(b) || (b > 0 && K % b != 0)) return ADAHOP_E_INVALID_ARG;
        if (strategy != ADAHOP_NONE && b == 0) return ADAHOP_E_INVALID_ARG;
    }
    if (k < 0 || (dim > 0 && k > dim)) return ADAHOP_E_INVALID_ARG;
    const bool oe = dim > 0 && k > 0;
    if (oe && !idx_inout) return ADAHOP_E_INVALID_ARG;
    // operands packed by the caller: both arrays or neither, and a residual that depends on the extracted
    // indices can only be trusted when the caller also supplies those indices
    const bool a_given = opts && (opts->a_codes || opts->a_scales), b_given = opts && (opts->b_codes || opts->b_scales);
    if (a_given && (!opts->a_codes || !opts->a_scales || !aligned(opts->a_codes, 16))) return ADAHOP_E_INVALID_ARG;
    if (b_given && (!opts->b_codes || !opts->b_scales || !aligned(opts->b_codes, 16))) return ADAHOP_E_INVALID_ARG;
    const int a_kind = oe ? residual_mask_kind(strategy, false) : 0, b_kind = oe ? residual_mask_kind(strategy, true) : 0;
    if (!use_given_idx && ((a_given && a_kind) || (b_given && b_kind))) return ADAHOP_E_INVALID_ARG;
    adahop_ws_layout_t L;
    rc = adahop_gemm_workspace_layout(M, N, K, strategy, k, &L);
    if (rc != ADAHOP_OK) return rc;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < L.total) return ADAHOP_E_WORKSPACE;

    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    uint8_t *mask = reinterpret_cast<uint8_t *>(ws + L.mask);
    float *scores = reinterpret_cast<float *>(ws + L.scores);

    // 1. which rows / columns / K-channels leave the MXFP4 path (App. F item 1)
    if (oe) {
        const bool mask_used = (!a_given && a_kind) || (!b_given && b_kind);
        if (use_given_idx) {
            rc = mask_used ? launch_mask_from_idx(idx_inout, k, mask, dim, st) : ADAHOP_OK;
        } else if (strategy == ADAHOP_IHT_OE_ROW) {
            rc = launch_foid_topk(*A, 0, k, idx_inout, mask, scores, st);
        } else if (strategy == ADAHOP_IHT_OE_COL) {
            rc = launch_foid_topk(*B, 0, k, idx_inout, mask, scores, st);
        } else {
            rc = launch_foid_topk(*A, 1, k, idx_inout, mask, scores, st);
        }
        if (rc != ADAHOP_OK) return rc;
    }
    // 2. residual -> transform -> MXFP4 (App. F item 2), for the operands the caller has not packed
    const uint8_t *a_codes = a_given ? opts->a_codes : reinterpret_cast<uint8_t *>(ws + L.a_codes);
    const uint8_t *a_scales = a_given ? opts->a_scales : reinterpret_cast<uint8_t *>(ws + L.a_scales);
    const uint8_t *b_codes = b_given ? opts->b_codes : reinterpret_cast<uint8_t *>(ws + L.b_codes);
    const uint8_t *b_scales = b_given ? opts->b_scales : reinterpret_cast<uint8_t *>(ws + L.b_scales);
    // The tiled GEMM kernel reads the scales in a stage-major copy; the quantisers that run here write it
    // beside the canonical one, which saves the product its two re-ordering launches.
    const int kpad_planned = oe && strategy == ADAHOP_IHT_OE_K ? kpad_of(k) : 0;
    int64_t Mi = 0, Ni = 0;
    gemm_mx_tiled_part(M, N, K, kpad_planned, a_scales, b_scales, C, ldc, c_bf16, &Mi, &Ni);
    // K-channel extraction: a quantiser that runs here on a K-contiguous operand also copies the extracted channels
    // out (it has the row in registers); the position of a channel in the index list comes from a 16-bit table that
    // takes the place of the scores, which nobody reads after the selection.
    // Only for indices selected here, which are distinct: a repeated index in a caller's list would leave a position
    // of the copy unwritten, where the separate gather reads the channel twice.
    const bool oe_k = oe && strategy == ADAHOP_IHT_OE_K, fuse = oe_k && !use_given_idx;
    const bool a_gathers = fuse && !a_given && iht_quantize_gathers_k(*A, kpad_planned);
    const bool b_gathers = fuse && !b_given && iht_quantize_gathers_k(*B, kpad_planned);
    k_gather_t ga = {nullptr, nullptr, 0, 0}, gb = ga;
    if (a_gathers || b_gathers) {
        uint16_t *pos1 = reinterpret_cast<uint16_t *>(scores);
        rc = launch_k_positions(idx_inout, k, mask, K, pos1, st);
        if (rc != ADAHOP_OK) return rc;
        if (a_gathers) ga = k_gather_t{pos1, reinterpret_cast<uint16_t *>(ws + L.gather_a), k, kpad_planned};
        if (b_gathers) gb = k_gather_t{pos1, reinterpret_cast<uint16_t *>(ws + L.gather_b), k, kpad_planned};
    }
    int sm_ready = 0;
    if (!a_given) {
        uint8_t *c = reinterpret_cast<uint8_t *>(ws + L.a_codes), *s = reinterpret_cast<uint8_t *>(ws + L.a_scales);
        const scales_sm_t sm = {Mi > 0 && !oht ? gemm_mx_scales_sm(ws + L.gemm, M, K, 0) : nullptr, Mi};
        rc = oht ? launch_oht_quantize(*A, b, c, s, st)
                 : launch_iht_quantize(*A, b, a_kind == 1 ? mask : nullptr, a_kind == 2 ? mask : nullptr, c, s, st,
                                       opts && opts->sr_a ? &opts->sr_seed_a : nullptr, &sm, &ga);
        if (rc != ADAHOP_OK) return rc;
        if (sm.out && iht_quantize_writes_scales_sm(*A)) sm_ready |= 1;
    }
    if (!b_given) {
        uint8_t *c = reinterpret_cast<uint8_t *>(ws + L.b_codes), *s = reinterpret_cast<uint8_t *>(ws + L.b_scales);
        const scales_sm_t sm = {Ni > 0 && !oht ? gemm_mx_scales_sm(ws + L.gemm, M, K, 1) : nullptr, Ni};
        rc = oht ? launch_oht_quantize(*B, b, c, s, st)
                 : launch_iht_quantize(*B, b, b_kind == 1 ? mask : nullptr, b_kind == 2 ? mask : nullptr, c, s, st,
                                       opts && opts->sr_b ? &opts->sr_seed_b : nullptr, &sm, &gb);
        if (rc != ADAHOP_OK) return rc;
        if (sm.out && iht_quantize_writes_scales_sm(*B)) sm_ready |= 2;
    }
    // 3. MXFP4 product, with the K-channel BF16 product fused in front; 4. row / column BF16 product
    if (oe_k) {
        const int kpad = kpad_planned;
        uint16_t *Ag = reinterpret_cast<uint16_t *>(ws + L.gather_a), *Bg = reinterpret_cast<uint16_t *>(ws + L.gather_b);
        rc = a_gathers ? ADAHOP_OK : launch_gather_k(*A, idx_inout, k, kpad, Ag, st);
        if (rc != ADAHOP_OK) return rc;
        rc = b_gathers ? ADAHOP_OK : launch_gather_k(*B, idx_inout, k, kpad, Bg, st);
        if (rc != ADAHOP_OK) return rc;
        return launch_gemm_mx(M, N, K, a_codes, a_scales, b_codes, b_scales, C, ldc, c_bf16, Ag, Bg, kpad, ws + L.gemm, st,
                              sm_ready);
    }
    rc = launch_gemm_mx(M, N, K, a_codes, a_scales, b_codes, b_scales, C, ldc, c_bf16, nullptr, nullptr, 0, ws + L.gemm, st,
                        sm_ready);
    if (rc != ADAHOP_OK) return rc;
    if (oht) return launch_oht_inverse(static_cast<float *>(C), M, N, ldc, b, st); // the rotations after the product (Eq. 6)
    if (oe) rc = launch_oe_rowcol(*A, *B, strategy, idx_inout, k, C, ldc, c_bf16, ws + L.gather_a, st);
    return rc;
}

int adahop_gemm(const adahop_operand_t *A, const adahop_operand_t *B, float *C, int64_t ldc,
                adahop_strategy_t strategy, int iht_block, int k, int32_t *idx_inout, int use_given_idx,
                void *workspace, size_t workspace_bytes, void *stream)
{
    return gemm_whole_path(A, B, C, ldc, strategy, iht_block, k, idx_inout, use_given_idx, nullptr, workspace,
                           workspace_bytes, stream);
}

int adahop_gemm_ex(const adahop_operand_t *A, const adahop_operand_t *B, void *C, int64_t ldc,
                   adahop_strategy_t strategy, int iht_block, int k, int32_t *idx_inout, int use_given_idx,
                   const adahop_gemm_opts_t *opts, void *workspace, size_t workspace_bytes, void *stream)
{
    return gemm_whole_path(A, B, C, ldc, strategy, iht_block, k, idx_inout, use_given_idx, opts, workspace,
                           workspace_bytes, stream);
}

} // extern "C"
