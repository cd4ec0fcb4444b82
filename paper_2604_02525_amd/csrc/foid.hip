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

// The same selection for dim <= TOPK_REG_KEYS * 1024 with every key held in registers: wave w owns the contiguous
// index range [w*per, (w+1)*per) throughout and lane l its keys w*per + 64 j + l, loaded once.
//
// One workgroup is all the parallelism there is, so the cost is the number of instructions per key.  A radix pass over
// all keys costs about 25 of them per key, and four are needed.  Instead:
//   1. every thread takes the maximum of its keys; the k-th largest of these 1024 maxima, cut down to its upper 16
//      bits (two radix passes over ONE value per thread), is a threshold T0 that at least k keys reach -- so the k
//      largest keys, and every key tied with the k-th, are among the keys >= T0 -- and that few others reach
//      (about 1.2 k of them for scores without structure);
//   2. the keys >= T0 are collected in LDS (one pass over the registers: a compare per key) and the radix select
//      runs over this short list (at most TOPK_CAND_PER_THREAD per thread);
//   3. the ordered compaction walks all keys once, as in k_topk.
// If k > 1024, or more than TOPK_CAND keys reach T0, the select runs over all register keys as before.
constexpr int TOPK_REG_KEYS = 32;
constexpr int TOPK_CAND_PER_THREAD = 4, TOPK_CAND = TOPK_CAND_PER_THREAD * TOPK_THREADS;

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

struct topk_shared_t {
    uint32_t hist[TOPK_WAVES + 1][256]; // one per wave, and their sum
    uint32_t prefix, remaining, count, whole_bin;
    uint32_t wave_gt[TOPK_WAVES], wave_eq[TOPK_WAVES];
    uint32_t cand[TOPK_CAND];
};

// Radix select over NK keys per thread (valid[j] says which exist), digits of 8 bits from bit 24 down to bit
// LAST_SHIFT: on return `prefix` holds the upper bits of the k-th largest key (k >= 1, at most the number of valid
// keys) and `remaining` how many keys with exactly these upper bits are among the k largest.  All threads call it.
// EARLY: stop at the first digit at which the k largest keys are exactly the keys of the found bin and of the bins
// above it (well separated outliers: usually the first or second digit): the remaining digits cannot change the
// selection then.  `prefix` then has zeros below that digit and `remaining` is UINT32_MAX, which says "every key
// >= prefix is selected"; returns true.
template <int NK, int LAST_SHIFT, bool EARLY = false>
__device__ __forceinline__ bool radix_select(topk_shared_t &sh, const uint32_t (&key)[NK], const bool (&valid)[NK], uint32_t k,
                                             uint32_t &prefix, uint32_t &remaining)
{
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    uint32_t pmask = 0;
    prefix = 0;
    remaining = k;
    uint32_t *total = sh.hist[TOPK_WAVES];
    for (int shift = 24; shift >= LAST_SHIFT; shift -= 8) {
#pragma unroll
        for (int q = 0; q < 4; ++q) sh.hist[w][lane + 64 * q] = 0;
        // (each wave clears and fills its own histogram: no barrier needed in between)
#pragma unroll
        for (int j = 0; j < NK; ++j) {
            const bool in = valid[j] && (key[j] & pmask) == prefix;
            if (__ballot(in)) wave_histogram_private(sh.hist[w], in, (key[j] >> shift) & 255u);
        }
        __syncthreads();
        if (tid < 256) {
            uint32_t sum = 0;
#pragma unroll
            for (int v = 0; v < TOPK_WAVES; ++v) sum += sh.hist[v][tid];
            total[tid] = sum;
        }
        __syncthreads();
        // The digit of the k-th largest key: the highest bin b with (keys in bins above b) + total[b] >= remaining.
        // Wave 0 scans the 256 bins in parallel: lane l owns bins 255 - 4l .. 252 - 4l.
        if (w == 0) {
            uint32_t c[4], mine = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                c[j] = total[255 - 4 * lane - j];
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
                sh.prefix = prefix | ((uint32_t)found << shift);
                sh.remaining = remaining - cum_at;
                sh.whole_bin = total[found] == remaining - cum_at ? 1u : 0u;
            }
        }
        __syncthreads();
        prefix = sh.prefix;
        remaining = sh.remaining;
        pmask |= 255u << shift;
        if (EARLY && shift > LAST_SHIFT && sh.whole_bin) { // (uniform: every thread reads the same word)
            remaining = 0xffffffffu;
            __syncthreads(); // the next use of the histograms and of sh.* must not overtake this read
            return true;
        }
    }
    return false;
}

__global__ __launch_bounds__(TOPK_THREADS) void k_topk_reg(const float *__restrict__ scores, int dim, int k,
                                                           int32_t *__restrict__ idx, uint8_t *__restrict__ mask)
{
    __shared__ topk_shared_t sh;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const uint32_t *keys = reinterpret_cast<const uint32_t *>(scores);
    const int per = ((dim + TOPK_WAVES - 1) / TOPK_WAVES + 63) / 64 * 64; // <= 64 * TOPK_REG_KEYS
    const int lo = w * per, hi = min(dim, lo + per);

    if (k <= 0) {
        for (int i = tid; i < dim; i += TOPK_THREADS) mask[i] = 0;
        return;
    }
    uint32_t key[TOPK_REG_KEYS];
    bool in[TOPK_REG_KEYS];
    uint32_t tmax = 0;
    bool any = false;
#pragma unroll
    for (int j = 0; j < TOPK_REG_KEYS; ++j) {
        const int i = lo + 64 * j + lane;
        in[j] = i < hi; // false for every lane once 64 j >= per
        key[j] = in[j] ? keys[i] : 0u;
        tmax = max(tmax, key[j]);
        any |= in[j];
    }
    if (tid == 0) sh.count = 0;

    // 1. threshold from the thread maxima (dim <= TOPK_CAND: every key is a candidate anyway)
    uint32_t T0 = 0;
    bool short_list = dim <= TOPK_CAND;
    if (!short_list && k <= TOPK_THREADS) {
        const uint32_t m[1] = {tmax};
        const bool mv[1] = {any};
        // threads that own at least one key (a wave's range may hold fewer than 64): with fewer than k of them there
        // is no k-th largest maximum and no threshold
        uint32_t have = 0;
        for (int v = 0; v < TOPK_WAVES; ++v) {
            const int n = min(dim, (v + 1) * per) - v * per;
            have += (uint32_t)max(0, min(n, 64));
        }
        if ((uint32_t)k <= have) {
            uint32_t p, r;
            radix_select<1, 16>(sh, m, mv, (uint32_t)k, p, r);
            T0 = p; // upper 16 bits of the k-th largest maximum, lower bits 0
            short_list = true;
        }
    }
    __syncthreads(); // sh.count = 0 is visible; the histograms are free again

    uint32_t T = 0, remaining = (uint32_t)k;
    bool selected = false;
    if (short_list) {
        // 2. collect the keys >= T0, in any order
#pragma unroll
        for (int j = 0; j < TOPK_REG_KEYS; ++j) {
            const bool c = in[j] && key[j] >= T0;
            const uint64_t m = __ballot(c);
            if (m) {
                uint32_t base = 0;
                const int leader = __ffsll((long long)m) - 1;
                if (lane == leader) base = atomicAdd(&sh.count, (uint32_t)__popcll(m));
                base = __builtin_amdgcn_readlane(base, leader);
                const uint32_t pos = base + (uint32_t)__popcll(m & (((uint64_t)1 << lane) - 1));
                if (c && pos < (uint32_t)TOPK_CAND) sh.cand[pos] = key[j];
            }
        }
        __syncthreads();
        const uint32_t count = sh.count;
        if (count <= (uint32_t)TOPK_CAND) {
            uint32_t ck[TOPK_CAND_PER_THREAD];
            bool cv[TOPK_CAND_PER_THREAD];
#pragma unroll
            for (int q = 0; q < TOPK_CAND_PER_THREAD; ++q) {
                const uint32_t i = (uint32_t)tid + (uint32_t)q * TOPK_THREADS;
                cv[q] = i < count;
                ck[q] = cv[q] ? sh.cand[i] : 0u;
            }
            // (stopped early, the threshold may lie below T0, where keys that are no candidates begin)
            if (radix_select<TOPK_CAND_PER_THREAD, 0, true>(sh, ck, cv, (uint32_t)k, T, remaining)) T = max(T, T0);
            selected = true;
        }
    }
    if (!selected) radix_select<TOPK_REG_KEYS, 0, true>(sh, key, in, (uint32_t)k, T, remaining); // the general way

    // 3. ordered compaction, as in k_topk
    uint32_t gt = 0, eq = 0;
#pragma unroll
    for (int j = 0; j < TOPK_REG_KEYS; ++j) {
        gt += (uint32_t)__popcll(__ballot(in[j] && key[j] > T));
        eq += (uint32_t)__popcll(__ballot(in[j] && key[j] == T));
    }
    if (lane == 0) {
        sh.wave_gt[w] = gt;
        sh.wave_eq[w] = eq;
    }
    __syncthreads();
    uint32_t gt_before = 0, eq_before = 0;
    for (int v = 0; v < w; ++v) {
        gt_before += sh.wave_gt[v];
        eq_before += sh.wave_eq[v];
    }
    const uint64_t below = ((uint64_t)1 << lane) - 1;
#pragma unroll
    for (int j = 0; j < TOPK_REG_KEYS; ++j) {
        const int i = lo + 64 * j + lane;
        const bool is_gt = in[j] && key[j] > T, is_eq = in[j] && key[j] == T;
        const uint64_t m_gt = __ballot(is_gt), m_eq = __ballot(is_eq);
        if ((m_gt | m_eq) == 0 && !__ballot(in[j])) continue; // past the end of the wave's range
        const uint32_t my_gt = gt_before + (uint32_t)__popcll(m_gt & below);
        const uint32_t my_eq = eq_before + (uint32_t)__popcll(m_eq & below);
        const bool sel = is_gt || (is_eq && my_eq < remaining);
        if (sel) idx[my_gt + min(my_eq, remaining)] = i;
        if (in[j]) mask[i] = sel ? 1 : 0;
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
