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
    float s = 0.0f, v = 0.0f;
    if (L == 64) {
        // all 64 samples first (independent loads, in flight together), then the fixed-order arithmetic
        float e[64];
        if (along_contig) {
            const uint4 *p = reinterpret_cast<const uint4 *>(x + base); // ld % 8 == 0 and 16-byte aligned data
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const uint4 u = p[q];
                e[8 * q + 0] = bf16_lo(u.x); e[8 * q + 1] = bf16_hi(u.x);
                e[8 * q + 2] = bf16_lo(u.y); e[8 * q + 3] = bf16_hi(u.y);
                e[8 * q + 4] = bf16_lo(u.z); e[8 * q + 5] = bf16_hi(u.z);
                e[8 * q + 6] = bf16_lo(u.w); e[8 * q + 7] = bf16_hi(u.w);
            }
        } else {
#pragma unroll
            for (int j = 0; j < 64; ++j) e[j] = bf16_one(x[base + j * step]);
        }
#pragma unroll
        for (int j = 0; j < 64; ++j) s = s + e[j];
        const float mean = s * inv_L;
#pragma unroll
        for (int j = 0; j < 64; ++j) {
            const float d = e[j] - mean;
            v = __builtin_fmaf(d, d, v);
        }
    } else {
        for (int j = 0; j < L; ++j) s = s + bf16_one(x[base + j * step]);
        const float mean = s * inv_L;
        for (int j = 0; j < L; ++j) {
            const float d = bf16_one(x[base + j * step]) - mean;
            v = __builtin_fmaf(d, d, v);
        }
    }
    scores[i] = v;
}

constexpr int TOPK_THREADS = 1024, TOPK_WAVES = TOPK_THREADS / 64;

// hist[bin] += 1 for every lane with valid set.  The scores of ordinary rows share their high bytes,
// and per-key atomics on one bin would serialise; so the most frequent bins of the wave are added with
// one atomic each (up to two rounds), and whatever is left -- then spread over many bins -- with
// plain per-lane atomics.
__device__ __forceinline__ void wave_histogram(uint32_t *hist, bool valid, uint32_t bin)
{
    uint64_t todo = __ballot(valid);
#pragma unroll 1
    for (int round = 0; round < 2 && todo; ++round) {
        const int leader = __ffsll((long long)todo) - 1;
        const uint32_t b = __builtin_amdgcn_readlane(bin, leader);
        const uint64_t same = __ballot(valid && bin == b);
        if ((int)(threadIdx.x & 63) == leader) atomicAdd(&hist[b], (uint32_t)__popcll(same));
        todo &= ~same;
    }
    if ((todo >> (threadIdx.x & 63)) & 1) atomicAdd(&hist[bin], 1u);
}

__global__ __launch_bounds__(TOPK_THREADS) void k_topk(const float *__restrict__ scores, int dim, int k,
                                                       int32_t *__restrict__ idx, uint8_t *__restrict__ mask)
{
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sh_prefix, sh_remaining;
    __shared__ uint32_t wave_gt[TOPK_WAVES], wave_eq[TOPK_WAVES];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const uint32_t *keys = reinterpret_cast<const uint32_t *>(scores);

    if (k <= 0) {
        for (int i = tid; i < dim; i += TOPK_THREADS) mask[i] = 0;
        return;
    }

    // Radix select: after the 4 passes `prefix` is the key of the k-th largest score and
    // `remaining` is how many keys equal to it are still to be taken.
    uint32_t prefix = 0, pmask = 0, remaining = (uint32_t)k;
    const int dim_up = (dim + TOPK_THREADS - 1) / TOPK_THREADS * TOPK_THREADS; // whole waves stay in the loop
    for (int shift = 24; shift >= 0; shift -= 8) {
        for (int b = tid; b < 256; b += TOPK_THREADS) hist[b] = 0;
        __syncthreads();
        for (int i = tid; i < dim_up; i += TOPK_THREADS) {
            const uint32_t key = i < dim ? keys[i] : 0u;
            wave_histogram(hist, i < dim && (key & pmask) == prefix, (key >> shift) & 255u);
        }
        __syncthreads();
        // The digit of the k-th largest key: the highest bin b with (keys in bins above b) + hist[b] >=
        // remaining.  Wave 0 scans the 256 bins in parallel: lane l owns bins 255 - 4l .. 252 - 4l.
        if (w == 0) {
            uint32_t c[4], mine = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                c[j] = hist[255 - 4 * lane - j];
                mine += c[j];
            }
            uint32_t incl = mine; // inclusive scan over lanes = over descending bins
#pragma unroll
            for (int d = 1; d < 64; d *= 2) {
                const uint32_t up = __shfl_up(incl, d);
                if (lane >= d) incl += up;
            }
            uint32_t cum = incl - mine; // keys in bins above this lane's
            int found = -1;
            uint32_t cum_at = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (found < 0 && cum + c[j] >= remaining) {
                    found = 255 - 4 * lane - j;
                    cum_at = cum;
                }
                cum += c[j];
            }
            const uint64_t hit = __ballot(found >= 0);
            if (hit && lane == __ffsll((long long)hit) - 1) {
                sh_prefix = prefix | ((uint32_t)found << shift);
                sh_remaining = remaining - cum_at;
            }
        }
        __syncthreads();
        prefix = sh_prefix;
        remaining = sh_remaining;
        pmask |= 255u << shift;
        __syncthreads();
    }
    const uint32_t T = prefix;

    // Ordered compaction: wave w owns the contiguous index range [w*per, (w+1)*per), per a multiple
    // of 64, and walks it 64 consecutive keys at a time.
    const int per = ((dim + TOPK_WAVES - 1) / TOPK_WAVES + 63) / 64 * 64;
    const int lo = w * per, hi = min(dim, lo + per);
    uint32_t gt = 0, eq = 0;
    for (int i0 = lo; i0 < hi; i0 += 64) {
        const int i = i0 + lane;
        const uint32_t key = i < hi ? keys[i] : 0u;
        gt += (uint32_t)__popcll(__ballot(i < hi && key > T));
        eq += (uint32_t)__popcll(__ballot(i < hi && key == T));
    }
    if (lane == 0) {
        wave_gt[w] = gt;
        wave_eq[w] = eq;
    }
    __syncthreads();
    uint32_t gt_before = 0, eq_before = 0;
    for (int v = 0; v < w; ++v) {
        gt_before += wave_gt[v];
        eq_before += wave_eq[v];
    }
    const uint64_t below = ((uint64_t)1 << lane) - 1;
    for (int i0 = lo; i0 < hi; i0 += 64) {
        const int i = i0 + lane;
        const uint32_t key = i < hi ? keys[i] : 0u;
        const bool is_gt = i < hi && key > T, is_eq = i < hi && key == T;
        const uint64_t m_gt = __ballot(is_gt), m_eq = __ballot(is_eq);
        const uint32_t my_gt = gt_before + (uint32_t)__popcll(m_gt & below);
        const uint32_t my_eq = eq_before + (uint32_t)__popcll(m_eq & below);
        const bool sel = is_gt || (is_eq && my_eq < remaining);
        // selected entries before this one: every greater key, and the equal keys that were taken
        if (sel) idx[my_gt + min(my_eq, remaining)] = i;
        if (i < hi) mask[i] = sel ? 1 : 0;
        gt_before += (uint32_t)__popcll(m_gt);
        eq_before += (uint32_t)__popcll(m_eq);
    }
}

// The same selection for dim <= TOPK_REG_KEYS * 1024 with every key held in registers: wave w owns the
// contiguous index range [w*per, (w+1)*per) throughout and lane l its keys w*per + 64 j + l, loaded once (the
// general kernel reads all keys from memory in each of its six passes, one dependent load per iteration, which
// is what its run time consists of at these sizes).
constexpr int TOPK_REG_KEYS = 32;

// hist[bin] += 1 for every lane with valid set, hist being private to the wave: one combined add for the bin
// of the first valid lane (the scores of ordinary rows share their high bytes, so that bin usually takes most of
// the wave), plain per-lane adds for the rest (conflicts only among the lanes of this wave).
__device__ __forceinline__ void wave_histogram_private(uint32_t *hist, bool valid, uint32_t bin)
{
    const uint64_t todo = __ballot(valid);
    if (todo == 0) return;
    const int leader = __ffsll((long long)todo) - 1;
    const uint32_t b = __builtin_amdgcn_readlane(bin, leader);
    const uint64_t same = __ballot(valid && bin == b);
    if ((int)(threadIdx.x & 63) == leader) atomicAdd(&hist[b], (uint32_t)__popcll(same));
    if (valid && bin != b) atomicAdd(&hist[bin], 1u);
}

__global__ __launch_bounds__(TOPK_THREADS) void k_topk_reg(const float *__restrict__ scores, int dim, int k,
                                                           int32_t *__restrict__ idx, uint8_t *__restrict__ mask)
{
    __shared__ uint32_t hist[TOPK_WAVES + 1][256]; // one per wave, and their sum
    __shared__ uint32_t sh_prefix, sh_remaining;
    __shared__ uint32_t wave_gt[TOPK_WAVES], wave_eq[TOPK_WAVES];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const uint32_t *keys = reinterpret_cast<const uint32_t *>(scores);
    const int per = ((dim + TOPK_WAVES - 1) / TOPK_WAVES + 63) / 64 * 64; // <= 64 * TOPK_REG_KEYS
    const int lo = w * per, hi = min(dim, lo + per);

    if (k <= 0) {
        for (int i = tid; i < dim; i += TOPK_THREADS) mask[i] = 0;
        return;
    }
    uint32_t key[TOPK_REG_KEYS];
#pragma unroll
    for (int j = 0; j < TOPK_REG_KEYS; ++j) {
        const int i = lo + 64 * j + lane;
        key[j] = i < hi ? keys[i] : 0u;
    }
    const int nj = (per + 63) / 64; // the same for every wave

    uint32_t prefix = 0, pmask = 0, remaining = (uint32_t)k;
    uint32_t *total = hist[TOPK_WAVES];
    for (int shift = 24; shift >= 0; shift -= 8) {
#pragma unroll
        for (int q = 0; q < 4; ++q) hist[w][lane + 64 * q] = 0;
        // (each wave clears and fills its own histogram: no barrier needed in between)
#pragma unroll
        for (int j = 0; j < TOPK_REG_KEYS; ++j)
            if (j < nj)
                wave_histogram_private(hist[w], lo + 64 * j + lane < hi && (key[j] & pmask) == prefix,
                                       (key[j] >> shift) & 255u);
        __syncthreads();
        if (tid < 256) {
            uint32_t sum = 0;
#pragma unroll
            for (int v = 0; v < TOPK_WAVES; ++v) sum += hist[v][tid];
            total[tid] = sum;
        }
        __syncthreads();
        if (w == 0) { // the digit of the k-th largest key, as in k_topk
            uint32_t c[4], mine = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                c[j] = total[255 - 4 * lane - j];
                mine += c[j];
            }
            uint32_t incl = mine;
#pragma unroll
            for (int d = 1; d < 64; d *= 2) {
                const uint32_t up = __shfl_up(incl, d);
                if (lane >= d) incl += up;
            }
            uint32_t cum = incl - mine;
            int found = -1;
            uint32_t cum_at = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (found < 0 && cum + c[j] >= remaining) {
                    found = 255 - 4 * lane - j;
                    cum_at = cum;
                }
                cum += c[j];
            }
            const uint64_t hit = __ballot(found >= 0);
            if (hit && lane == __ffsll((long long)hit) - 1) {
                sh_prefix = prefix | ((uint32_t)found << shift);
                sh_remaining = remaining - cum_at;
            }
        }
        __syncthreads();
        prefix = sh_prefix;
        remaining = sh_remaining;
        pmask |= 255u << shift;
    }
    const uint32_t T = prefix;

    uint32_t gt = 0, eq = 0;
#pragma unroll
    for (int j = 0; j < TOPK_REG_KEYS; ++j) {
        const bool in = lo + 64 * j + lane < hi; // false for every lane once j >= nj
        gt += (uint32_t)__popcll(__ballot(in && key[j] > T));
        eq += (uint32_t)__popcll(__ballot(in && key[j] == T));
    }
    if (lane == 0) {
        wave_gt[w] = gt;
        wave_eq[w] = eq;
    }
    __syncthreads();
    uint32_t gt_before = 0, eq_before = 0;
    for (int v = 0; v < w; ++v) {
        gt_before += wave_gt[v];
        eq_before += wave_eq[v];
    }
    const uint64_t below = ((uint64_t)1 << lane) - 1;
#pragma unroll
    for (int j = 0; j < TOPK_REG_KEYS; ++j) {
        const int i = lo + 64 * j + lane;
        const bool in = i < hi;
        const bool is_gt = in && key[j] > T, is_eq = in && key[j] == T;
        const uint64_t m_gt = __ballot(is_gt), m_eq = __ballot(is_eq);
        const uint32_t my_gt = gt_before + (uint32_t)__popcll(m_gt & below);
        const uint32_t my_eq = eq_before + (uint32_t)__popcll(m_eq & below);
        const bool sel = is_gt || (is_eq && my_eq < remaining);
        if (sel) idx[my_gt + min(my_eq, remaining)] = i;
        if (in) mask[i] = sel ? 1 : 0;
        gt_before += (uint32_t)__popcll(m_gt);
        eq_before += (uint32_t)__popcll(m_eq);
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
    if (dim <= (int64_t)TOPK_REG_KEYS * TOPK_THREADS)
        hipLaunchKernelGGL(k_topk_reg, dim3(1), dim3(TOPK_THREADS), 0, st, scores, (int)dim, k, idx, mask);
    else
        hipLaunchKernelGGL(k_topk, dim3(1), dim3(TOPK_THREADS), 0, st, scores, (int)dim, k, idx, mask);
    return check_launch();
}

// ------------------------------------------------------------------------------------------------
// Score scratch that needs no allocation: a fixed array in the library's own device image, for the entry point
// that serves callers which cannot allocate.  Every GPU the library runs on holds its own copy (at its own
// address) until the process ends.  In host code the array's name is only a stand-in; the address that kernels
// and copies may use is asked for once per device, with that device current, and kept.
// ------------------------------------------------------------------------------------------------
static __device__ __align__(256) float scratch[ADAHOP_FOID_NOALLOC_MAX_DIM];

int foid_static_scores(float **out)
{
    static std::atomic<float *> per_device[64];
    int dev = 0;
    int rc = check_hip(hipGetDevice(&dev));
    if (rc != ADAHOP_OK) return rc;
    if (dev < 0 || dev >= 64) return ADAHOP_E_INVALID_ARG;
    float *ptr = per_device[dev].load(std::memory_order_acquire);
    if (!ptr) {
        rc = check_hip(hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch)));
        if (rc != ADAHOP_OK) return rc;
        if (!ptr) return ADAHOP_E_HIP;
        per_device[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return ADAHOP_OK;
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
