// Fast Outlier Index Detection (paper App. F item 1): a variance score over the first 64 samples of
// every row / column / K-channel, then the exact top-k.
//
// Scores are evaluated in a fixed fp32 order (sequential sum, mean = sum * (1/L), sequential fused
// multiply-add of squared deviations) so the ranking is reproducible bit for bit; ties are broken
// towards the lower index.  The selection is a 4-pass radix select over the score bits (scores are
// non-negative, so their bit patterns order like the values) followed by an ordered compaction, all
// inside one workgroup: the candidate count is at most a few tens of thousands and the whole step
// is latency-bound.
#include "common.h"

namespace adahop {

namespace {

__global__ __launch_bounds__(256) void k_foid_scores(const uint16_t *__restrict__ x, int64_t ld, int k_contig,
                                                     int axis, int64_t dim, int L, float inv_L,
                                                     float *__restrict__ scores)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= dim) return;
    // sample j of scored index i: (o = i, kk = j) for axis 0, (o = j, kk = i) for axis 1
    const bool along_contig = (axis == 0) == (k_contig != 0);
    const int64_t base = along_contig ? i * ld : i;
    const int64_t step = along_contig ? 1 : ld;
    float s = 0.0f;
    for (int j = 0; j < L; ++j) s = s + bf16_one(x[base + j * step]);
    const float mean = s * inv_L;
    float v = 0.0f;
    for (int j = 0; j < L; ++j) {
        const float d = bf16_one(x[base + j * step]) - mean;
        v = __builtin_fmaf(d, d, v);
    }
    scores[i] = v;
}

constexpr int TOPK_THREADS = 1024;

__global__ __launch_bounds__(TOPK_THREADS) void k_topk(const float *__restrict__ scores, int dim, int k,
                                                       int32_t *__restrict__ idx, uint8_t *__restrict__ mask)
{
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sh_prefix, sh_remaining;
    __shared__ uint32_t scan_gt[TOPK_THREADS], scan_eq[TOPK_THREADS];
    const int tid = threadIdx.x;
    const uint32_t *keys = reinterpret_cast<const uint32_t *>(scores);

    if (k <= 0) {
        for (int i = tid; i < dim; i += TOPK_THREADS) mask[i] = 0;
        return;
    }

    // Radix select: after the 4 passes `prefix` is the key of the k-th largest score and
    // `remaining` is how many keys equal to it are still to be taken.
    uint32_t prefix = 0, pmask = 0, remaining = (uint32_t)k;
    for (int shift = 24; shift >= 0; shift -= 8) {
        for (int b = tid; b < 256; b += TOPK_THREADS) hist[b] = 0;
        __syncthreads();
        for (int i = tid; i < dim; i += TOPK_THREADS) {
            const uint32_t key = keys[i];
            if ((key & pmask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid == 0) {
            uint32_t cum = 0;
            int b = 255;
            for (; b > 0; --b) {
                if (cum + hist[b] >= remaining) break;
                cum += hist[b];
            }
            sh_prefix = prefix | ((uint32_t)b << shift);
            sh_remaining = remaining - cum;
        }
        __syncthreads();
        prefix = sh_prefix;
        remaining = sh_remaining;
        pmask |= 255u << shift;
        __syncthreads();
    }
    const uint32_t T = prefix;

    // Ordered compaction: thread t owns the contiguous index range [t*per, (t+1)*per).
    const int per = (dim + TOPK_THREADS - 1) / TOPK_THREADS;
    const int lo = tid * per;
    const int hi = min(dim, lo + per);
    uint32_t gt = 0, eq = 0;
    for (int i = lo; i < hi; ++i) {
        const uint32_t key = keys[i];
        gt += key > T;
        eq += key == T;
    }
    scan_gt[tid] = gt;
    scan_eq[tid] = eq;
    __syncthreads();
    for (int d = 1; d < TOPK_THREADS; d *= 2) {
        uint32_t a = 0, b = 0;
        if (tid >= d) {
            a = scan_gt[tid - d];
            b = scan_eq[tid - d];
        }
        __syncthreads();
        scan_gt[tid] += a;
        scan_eq[tid] += b;
        __syncthreads();
    }
    uint32_t gt_before = scan_gt[tid] - gt, eq_before = scan_eq[tid] - eq;
    for (int i = lo; i < hi; ++i) {
        const uint32_t key = keys[i];
        const bool is_gt = key > T;
        const bool is_eq = key == T;
        const bool sel = is_gt || (is_eq && eq_before < remaining);
        if (sel) idx[gt_before + min(eq_before, remaining)] = i;
        mask[i] = sel ? 1 : 0;
        gt_before += is_gt;
        eq_before += is_eq;
    }
}

__global__ __launch_bounds__(256) void k_fill_u8(uint8_t *p, int64_t n, uint8_t v)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

__global__ __launch_bounds__(256) void k_mark(const int32_t *__restrict__ idx, int k, uint8_t *mask)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t < k) mask[idx[t]] = 1;
}

} // namespace

int launch_foid_topk(const adahop_operand_t &x, int axis, int k, int32_t *idx, uint8_t *mask, float *scores,
                     hipStream_t st)
{
    const int64_t dim = axis == 0 ? x.outer : x.K;
    const int64_t len = axis == 0 ? x.K : x.outer;
    if (dim == 0) return ADAHOP_OK;
    const int L = (int)(len < 64 ? len : 64);
    const float inv_L = 1.0f / (float)L;
    hipLaunchKernelGGL(k_foid_scores, dim3((unsigned)ceil_div(dim, 256)), dim3(256), 0, st,
                       static_cast<const uint16_t *>(x.data), x.ld, x.k_contig, axis, dim, L, inv_L, scores);
    int rc = check_launch();
    if (rc != ADAHOP_OK) return rc;
    hipLaunchKernelGGL(k_topk, dim3(1), dim3(TOPK_THREADS), 0, st, scores, (int)dim, k, idx, mask);
    return check_launch();
}

int launch_mask_from_idx(const int32_t *idx, int k, uint8_t *mask, int64_t dim, hipStream_t st)
{
    if (dim == 0) return ADAHOP_OK;
    hipLaunchKernelGGL(k_fill_u8, dim3((unsigned)ceil_div(dim, 256)), dim3(256), 0, st, mask, dim, (uint8_t)0);
    int rc = check_launch();
    if (rc != ADAHOP_OK || k == 0) return rc;
    hipLaunchKernelGGL(k_mark, dim3((unsigned)ceil_div(k, 256)), dim3(256), 0, st, idx, k, mask);
    return check_launch();
}

} // namespace adahop
