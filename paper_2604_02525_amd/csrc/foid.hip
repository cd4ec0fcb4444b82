// Fast Outlier Index Detection (paper App. F item 1): a variance score over the first 64 samples of
// every row / column / K-channel, then the exact top-k.
//
// Scores are evaluated in a fixed fp32 order (sequential sum, mean = sum * (1/L), sequential fused
// multiply-add of squared deviations) so the ranking is reproducible bit for bit; ties are broken
// towards the lower index.  The selection is a radix select over the score bits (scores are
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

// The same selection for dim <= TOPK_LDS_KEYS with every key staged in LDS once: wave w owns the contiguous index
// range [w*per, (w+1)*per) throughout.
//
// One workgroup is all the parallelism there is, and it runs every instruction of the kernel once or a few times
// only: what such a kernel costs is, first, the instruction lines it has to fetch (the cache is cold at every launch;
// a version of this kernel with the keys in registers and every loop unrolled spent most of its 12-18 us there) and,
// second, the number of passes over all keys.  So every pass is a rolled loop over keys in LDS, the select and the
// compaction exist once each (they run over a list described by a few numbers), and the passes over all keys are light:
//   1. every thread takes the maximum of the keys it loads; the k-th largest of these 1024 maxima, cut down to its
//      upper 16 bits (two radix passes over ONE value per thread), is a threshold T0 that at least k keys reach -- so
//      the k largest keys, and every key tied with the k-th, are among the keys >= T0 -- and that few others reach
//      (about 1.2 k of them for scores without structure).  With fewer than k threads that own a key the threshold
//      comes out as 0 and step 2 finds too many candidates, which is handled there;
//   2. the keys >= T0 are counted per wave and then copied, with their indices, to a list in index order (a compare
//      per key in each of the two passes);
//   3. radix select and ordered compaction run over this list (at most two entries per thread).
// If k > 1024, or more than TOPK_CAND keys reach T0, or there are no more keys than four per thread, the list is
// the keys themselves.
constexpr int TOPK_LDS_KEYS = 32768;
constexpr int TOPK_CAND = 2048, TOPK_DIRECT = 4 * TOPK_THREADS;

// hist[bin] += 1 for every lane with valid set: one combined add for the bin of the first valid lane (the scores of
// ordinary rows share their high bytes, so that bin usually takes most of the wave), plain per-lane adds for the rest.
__device__ __forceinline__ void wave_histogram_once(uint32_t *hist, bool valid, uint32_t bin)
{
    const uint64_t todo = __ballot(valid);
    if (todo == 0) return;
    const int leader = __ffsll((long long)todo) - 1;
    const uint32_t b = __builtin_amdgcn_readlane(bin, leader);
    const uint64_t same = __ballot(valid && bin == b);
    if ((int)(threadIdx.x & 63) == leader) atomicAdd(&hist[b], (uint32_t)__popcll(same));
    if (valid && bin != b) atomicAdd(&hist[bin], 1u);
}

// Inclusive sum over the lanes of a wave (all 64 active): four shifts within the rows of 16 lanes, then the row totals
// handed on to the following rows.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t v)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false); // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false); // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false); // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false); // row_shr:8
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false); // lane 15 of rows 0, 2 to rows 1, 3
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false); // lane 31 to rows 2, 3
    return v;
}

struct topk_shared_t { // behind the keys
    uint32_t hist[2][256];              // used in turn by the radix passes, each cleared again after its pass
    uint32_t cand[TOPK_CAND];           // first the 1024 thread maxima, then the keys >= T0 in index order
    uint16_t cand_i[TOPK_CAND];         // and their indices (< TOPK_LDS_KEYS)
    uint32_t prefix, remaining, whole_bin, unused;
    uint32_t wave_a[TOPK_WAVES], wave_b[TOPK_WAVES];
};
static_assert(TOPK_LDS_KEYS <= 65536, "candidate indices are kept in 16 bits");

constexpr int topk_per_wave(int n) { return ((n + TOPK_WAVES - 1) / TOPK_WAVES + 63) / 64 * 64; }
constexpr size_t topk_lds_bytes(int dim) { return (size_t)topk_per_wave(dim) * TOPK_WAVES * 4 + sizeof(topk_shared_t); }
static_assert(topk_lds_bytes(TOPK_LDS_KEYS) <= 160 * 1024, "keys, histograms and candidates share one compute unit's LDS");

__global__ __launch_bounds__(TOPK_THREADS) void k_topk_lds(const float *__restrict__ scores, int dim, int k,
                                                           int32_t *__restrict__ idx, uint8_t *__restrict__ mask)
{
    extern __shared__ __align__(16) uint32_t skeys[]; // per * TOPK_WAVES keys, then topk_shared_t
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6); // (a scalar: loop bounds derived from it are uniform)
    const uint32_t *keys = reinterpret_cast<const uint32_t *>(scores);
    const int per = topk_per_wave(dim); // <= TOPK_LDS_KEYS / TOPK_WAVES
    const int lo = w * per, hi = min(dim, lo + per);
    const int nslice = hi > lo ? (hi - lo + 63) / 64 : 0; // 64-key slices of this wave that hold keys
    topk_shared_t &sh = *reinterpret_cast<topk_shared_t *>(skeys + per * TOPK_WAVES);

    if (k <= 0) {
        for (int i = tid; i < dim; i += TOPK_THREADS) mask[i] = 0;
        return;
    }

    // 0. the wave's keys into LDS (a wave reads back only what it wrote itself: no barrier), the thread's maximum,
    // and the mask cleared (the selected entries are set at the end, many barriers later)
    uint32_t tmax = 0;
    if (((reinterpret_cast<uintptr_t>(keys) & 15) | (reinterpret_cast<uintptr_t>(mask) & 3)) == 0) {
        // 16 bytes per lane, all loads of the wave in flight together (per <= 2048 = 8 x 256)
        uint4 u[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int o = 256 * q + 4 * lane, i = lo + o; // (per is a multiple of 64, not of 256)
            u[q] = make_uint4(0u, 0u, 0u, 0u);
            if (o < per) {
                if (i + 3 < hi) {
                    u[q] = *reinterpret_cast<const uint4 *>(keys + i);
                    *reinterpret_cast<uint32_t *>(mask + i) = 0u;
                } else { // (one lane of one wave at most)
                    if (i < hi) u[q].x = keys[i], mask[i] = 0;
                    if (i + 1 < hi) u[q].y = keys[i + 1], mask[i + 1] = 0;
                    if (i + 2 < hi) u[q].z = keys[i + 2], mask[i + 2] = 0;
                }
            }
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int o = 256 * q + 4 * lane;
            if (o < per) {
                *reinterpret_cast<uint4 *>(skeys + lo + o) = u[q];
                tmax = max(max(tmax, u[q].x), max(max(u[q].y, u[q].z), u[q].w));
            }
        }
    } else {
#pragma unroll 4
        for (int i = lo + lane; i < hi; i += 64) {
            const uint32_t key = keys[i];
            mask[i] = 0;
            skeys[i] = key;
            tmax = max(tmax, key);
        }
    }

    // The list that the final select and the compaction run over: entries [c_lo, c_hi) of src are this wave's part
    // (in index order over the waves; c_n slices of 64), entry p standing for index p (the keys themselves) or
    // cand_i[p] (candidates).  Entries up to the end of the last slice may be read (and are ignored).
    const uint32_t *src = skeys;
    int c_lo = lo, c_hi = hi, c_n = nslice;
    bool direct = true;

    // 1./2. radix select, once over the thread maxima (gives T0) and once over the list: digits of 8 bits from bit 24
    // down to bit last_shift.  After a use `prefix` holds the upper bits of the k-th largest key and `remaining` how
    // many keys with exactly these upper bits are among the k largest.  Over the list it stops at the first digit at
    // which the k largest keys are exactly the keys of the found bin and of the bins above it (well separated
    // outliers: usually the first or second digit): the remaining digits cannot change the selection then; `prefix`
    // then has zeros below that digit and `remaining` is UINT32_MAX, which says "every key >= prefix is selected".
    bool maxima = dim > TOPK_DIRECT && k <= TOPK_THREADS;
    if (maxima) sh.cand[tid] = tmax;
    if (tid < 512) sh.hist[0][tid] = 0; // (both histograms)
    __syncthreads();
    int pass = 0;
    uint32_t T = 0, T0 = 0, remaining = (uint32_t)k;
    const uint64_t below = ((uint64_t)1 << lane) - 1;
    for (;;) {
        const uint32_t *from = maxima ? sh.cand : src;
        const int first = maxima ? tid : c_lo + lane;
        const int end = maxima ? 64 * (w + 1) : c_hi; // (the maxima: one per thread, the wave's own 64)
        const int n = maxima ? 1 : c_n;
        const int last_shift = maxima ? 16 : 0;
        uint32_t prefix = 0, pmask = 0;
        remaining = (uint32_t)k;
        for (int shift = 24; shift >= last_shift; shift -= 8) {
            uint32_t *hist = sh.hist[pass & 1]; // (all zeros: cleared two passes ago, or before the first)
            ++pass;
            for (int j = 0; j < n; j += 2) { // (two reads in flight; what lies past the list is ignored)
                const int i0 = first + 64 * j, i1 = i0 + 64;
                const uint32_t key0 = from[i0], key1 = from[i1];
                const bool in0 = i0 < end && (key0 & pmask) == prefix, in1 = i1 < end && (key1 & pmask) == prefix;
                if (__ballot(in0)) wave_histogram_once(hist, in0, (key0 >> shift) & 255u);
                if (__ballot(in1)) wave_histogram_once(hist, in1, (key1 >> shift) & 255u);
            }
            __syncthreads();
            // The digit of the k-th largest key: the highest bin b with (keys in bins above b) + count[b] >= remaining.
            // Wave 0 scans the 256 bins in parallel: lane l owns bins 255 - 4l .. 252 - 4l.
            if (w == 0) {
                const uint4 h = *reinterpret_cast<const uint4 *>(&hist[252 - 4 * lane]);
                const uint32_t c[4] = {h.w, h.z, h.y, h.x};
                const uint32_t mine = c[0] + c[1] + c[2] + c[3];
                uint32_t cum = wave_inclusive_sum(mine) - mine; // keys in bins above this lane's (lanes = descending bins)
                int found = -1;
                uint32_t cum_at = 0, c_at = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (found < 0 && cum + c[j] >= remaining) {
                        found = 255 - 4 * lane - j;
                        cum_at = cum;
                        c_at = c[j];
                    }
                    cum += c[j];
                }
                const uint64_t hit = __ballot(found >= 0);
                if (hit && lane == __ffsll((long long)hit) - 1) {
                    sh.prefix = prefix | ((uint32_t)found << shift);
                    sh.remaining = remaining - cum_at;
                    sh.whole_bin = c_at == remaining - cum_at ? 1u : 0u;
                }
            }
            __syncthreads();
            if (tid < 256) hist[tid] = 0; // for the pass after the next (barriers in between)
            prefix = sh.prefix;
            remaining = sh.remaining;
            pmask |= 255u << shift;
            const bool stop = !maxima && shift > last_shift && sh.whole_bin; // (uniform: every thread reads the same word)
            if (stop || shift == last_shift) __syncthreads(); // what comes next must not overtake these reads
            if (stop) {
                remaining = 0xffffffffu;
                break;
            }
        }
        if (!maxima) {
            // (stopped early over the candidates, the threshold may lie below T0, where keys that are no candidates begin)
            T = max(prefix, T0);
            break;
        }
        maxima = false;
        T0 = prefix; // upper 16 bits of the k-th largest maximum, lower bits 0
        // the keys >= T0: how many in this wave's part, in the parts before it, and in all
        // (four reads in flight; what lies past the wave's part is ignored)
        uint32_t mine = 0;
        for (int j = 0; j < nslice; j += 4) {
            uint32_t key[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) key[q] = skeys[lo + 64 * (j + q) + lane];
#pragma unroll
            for (int q = 0; q < 4; ++q)
                mine += (uint32_t)__popcll(__ballot(lo + 64 * (j + q) + lane < hi && key[q] >= T0));
        }
        if (lane == 0) sh.wave_a[w] = mine;
        __syncthreads();
        uint32_t pos = 0, count = 0;
        for (int v = 0; v < TOPK_WAVES; ++v) {
            const uint32_t c = sh.wave_a[v];
            pos += v < w ? c : 0u;
            count += c;
        }
        pos = __builtin_amdgcn_readfirstlane(pos);
        count = __builtin_amdgcn_readfirstlane(count);
        if (count <= (uint32_t)TOPK_CAND) {
            // copied in index order, with their indices
            for (int j = 0; j < nslice; j += 4) {
                uint32_t key[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) key[q] = skeys[lo + 64 * (j + q) + lane];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int i = lo + 64 * (j + q) + lane;
                    const bool c = i < hi && key[q] >= T0;
                    const uint64_t m = __ballot(c);
                    if (m) { // (most slices hold no candidate)
                        if (c) {
                            const uint32_t p = pos + (uint32_t)__popcll(m & below);
                            sh.cand[p] = key[q];
                            sh.cand_i[p] = (uint16_t)i;
                        }
                        pos += (uint32_t)__popcll(m);
                    }
                }
            }
            const int per_c = topk_per_wave((int)count);
            src = sh.cand;
            direct = false;
            c_lo = w * per_c;
            c_hi = min((int)count, c_lo + per_c);
            c_n = c_hi > c_lo ? (c_hi - c_lo + 63) / 64 : 0;
        }
        __syncthreads();
    }

    // 3. ordered compaction over the list
    uint32_t gt = 0, eq = 0;
#pragma unroll 2
    for (int j = 0; j < c_n; ++j) {
        const int i = c_lo + 64 * j + lane;
        const uint32_t key = src[i];
        gt += (uint32_t)__popcll(__ballot(i < c_hi && key > T));
        eq += (uint32_t)__popcll(__ballot(i < c_hi && key == T));
    }
    if (lane == 0) {
        sh.wave_a[w] = gt;
        sh.wave_b[w] = eq;
    }
    __syncthreads();
    uint32_t gt_before = 0, eq_before = 0;
    for (int v = 0; v < w; ++v) {
        gt_before += sh.wave_a[v];
        eq_before += sh.wave_b[v];
    }
#pragma unroll 2
    for (int j = 0; j < c_n; ++j) {
        const int i = c_lo + 64 * j + lane;
        const bool in = i < c_hi;
        const uint32_t key = src[i];
        const bool is_gt = in && key > T, is_eq = in && key == T;
        const uint64_t m_gt = __ballot(is_gt), m_eq = __ballot(is_eq);
        const uint32_t my_gt = gt_before + (uint32_t)__popcll(m_gt & below);
        const uint32_t my_eq = eq_before + (uint32_t)__popcll(m_eq & below);
        // selected entries before this one: every greater key, and the equal keys that were taken
        if (is_gt || (is_eq && my_eq < remaining)) {
            const int index = direct ? i : (int)sh.cand_i[i];
            idx[my_gt + min(my_eq, remaining)] = index;
            mask[index] = 1;
        }
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

// The one-workgroup selection keeps up to TOPK_LDS_KEYS keys in LDS: allowed once per device (host-side call).
int configure_foid()
{
    static device_once_t once;
    int dev = 0;
    int rc = check_hip(hipGetDevice(&dev));
    if (rc != ADAHOP_OK || !once.need(dev)) return rc;
    rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(k_topk_lds), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)topk_lds_bytes(TOPK_LDS_KEYS)));
    if (rc != ADAHOP_OK) return rc;
    once.mark(dev);
    return ADAHOP_OK;
}

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
    if (dim <= (int64_t)TOPK_LDS_KEYS) {
        rc = configure_foid(); // more LDS than a launch may ask for by default: allowed once per device
        if (rc != ADAHOP_OK) return rc;
        hipLaunchKernelGGL(k_topk_lds, dim3(1), dim3(TOPK_THREADS), topk_lds_bytes((int)dim), st, scores, (int)dim, k, idx,
                           mask);
    } else {
        hipLaunchKernelGGL(k_topk, dim3(1), dim3(TOPK_THREADS), 0, st, scores, (int)dim, k, idx, mask);
    }
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
