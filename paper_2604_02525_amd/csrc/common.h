// Shared host/device helpers of the AdaHOP HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "../../include/adahop.h"

namespace adahop {

// Records the hipError_t of a failed call for adahop_last_hip_error().
void set_last_hip_error(int e);

inline int check_hip(hipError_t e)
{
    if (e == hipSuccess) return ADAHOP_OK;
    set_last_hip_error((int)e);
    return ADAHOP_E_HIP;
}

inline int check_launch() { return check_hip(hipGetLastError()); }

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Argument checks shared by the entry points; all run before any HIP call.
int validate_operand(const adahop_operand_t *x);
bool valid_iht_block(int b);

// One-time set-up per device and kernel family: function attributes (LDS sizes above the default) for every
// instance of the family, and the compute-unit count for the persistent kernels.  Host-side calls only; the
// launchers call them, adahop_prepare_device calls them all.
int configure_gemm_mx(int *ncu_out);
int configure_gemm_mx_dual(int *ncu_out);
int configure_oe_rowcol();
int configure_oht();
int configure_quantizers();
int configure_foid();

// Launchers (one per kernel family); each validates nothing and returns a status.
// Stage-major copy of the scales for the tiled GEMM kernel (see gemm_mx_tiled_part): [K/256][rows][8].
struct scales_sm_t {
    uint8_t *out; // stage-major copy, or nullptr
    int64_t rows; // rows [0, rows) are written
};
// Whether launch_iht_quantize honours a scales_sm_t for this operand (only its kernels for K % 256 == 0 write the
// copy); a caller may tell the product that the copy is there only if this holds.
bool iht_quantize_writes_scales_sm(const adahop_operand_t &x);
// The extracted K-channels of an operand, copied out by the quantiser that reads the operand anyway (Eq. 7 with
// S a set of K-channels): out[o, pos1[c] - 1] = x(o, c) for every channel c with pos1[c] != 0, out[o, k .. kpad) = 0.
// out is [outer, kpad] bf16; pos1[c] = t + 1 for the channel c = idx[t], 0 for a channel that is not extracted.
struct k_gather_t {
    const uint16_t *pos1; // per K-channel, 16-byte aligned
    uint16_t *out;        // nullptr: no copy
    int k, kpad;
};
// Whether launch_iht_quantize honours a k_gather_t for this operand (K-contiguous, whole passes of a workgroup
// along K, a copy that fits its LDS staging).
bool iht_quantize_gathers_k(const adahop_operand_t &x, int kpad);
// pos1[c] = t + 1 where c = idx[t], 0 where mask[c] == 0 (mask as launch_foid_topk / launch_mask_from_idx leave it).
int launch_k_positions(const int32_t *idx, int k, const uint8_t *mask, int64_t K, uint16_t *pos1, hipStream_t st);
// sr_seed: NULL = round to nearest even; else the elements are rounded stochastically under that seed.
int launch_iht_quantize(const adahop_operand_t &x, int iht_block, const uint8_t *zero_outer,
                        const uint8_t *zero_k, uint8_t *codes, uint8_t *scales, hipStream_t st,
                        const uint64_t *sr_seed = nullptr, const scales_sm_t *sm = nullptr,
                        const k_gather_t *gather = nullptr);
int launch_foid_topk(const adahop_operand_t &x, int axis, int k, int32_t *idx, uint8_t *mask, float *scores,
                     hipStream_t st);
// Device address, on the current device, of the library's built-in score scratch (ADAHOP_FOID_NOALLOC_MAX_DIM floats).
int foid_static_scores(float **out);
int launch_mask_from_idx(const int32_t *idx, int k, uint8_t *mask, int64_t dim, hipStream_t st);
// OE-K operands for the fused prologue: Ag [M, kpad], Bg [N, kpad] bf16, K-contiguous, zero padded.
int launch_gemm_mx(int64_t M, int64_t N, int64_t K, const uint8_t *a_codes, const uint8_t *a_scales,
                   const uint8_t *b_codes, const uint8_t *b_scales, void *C, int64_t ldc, int c_bf16,
                   const uint16_t *Ag, const uint16_t *Bg, int kpad, void *workspace, hipStream_t st,
                   int sm_ready = 0);
size_t gemm_mx_workspace_bytes(int64_t M, int64_t N, int64_t K);
// The tiled kernel reads the scales in a stage-major copy, [K/256][rows][8] over the rows it takes.  A caller
// that quantises right before the product lets the quantiser write that copy as well (scales_sm_t above) and
// says so with sm_ready (bit 0: A, bit 1: B); otherwise launch_gemm_mx re-orders the canonical scales itself.
void gemm_mx_tiled_part(int64_t M, int64_t N, int64_t K, int kpad, const uint8_t *a_scales, const uint8_t *b_scales,
                        const void *C, int64_t ldc, int c_bf16, int64_t *Mi, int64_t *Ni);
uint8_t *gemm_mx_scales_sm(void *workspace, int64_t M, int64_t K, int which);
// The 256 x 128 kernel with two accumulator sets (gemm_mx_dual.hip): fp32 C, no gathered K-channels, K >= 2048.
bool gemm_mx_dual_eligible(int64_t M, int64_t N, int64_t K);
int launch_gemm_mx_dual(int64_t Mi, int64_t Ni, int64_t K, const uint8_t *a_codes, const uint8_t *a_sm,
                        const uint8_t *b_codes, const uint8_t *b_sm, float *C, int64_t ldc, hipStream_t st);
// Diagnostics: 0 = choose by shape, 1 = always the 256 x 256 kernel, 2 = the 256 x 128 kernel wherever it can run.
void gemm_mx_force_kernel(int which);
int launch_gather_k(const adahop_operand_t &x, const int32_t *idx, int k, int kpad, uint16_t *out, hipStream_t st);
// C is float[M, ldc], or bf16[M, ldc] when c_bf16 is set (here and in launch_oe_rowcol).
// Row / column outlier product; workspace of oe_rowcol_workspace_bytes() bytes, 256-byte aligned.
size_t oe_rowcol_workspace_bytes(int64_t M, int64_t N, int64_t K, int kind, int k);
int launch_oe_rowcol(const adahop_operand_t &A, const adahop_operand_t &B, int kind, const int32_t *idx, int k,
                     void *C, int64_t ldc, int c_bf16, void *workspace, hipStream_t st);
int launch_oe_k_accumulate(int64_t M, int64_t N, const uint16_t *Ag, const uint16_t *Bg, int kpad, float *C,
                           int64_t ldc, hipStream_t st);

// Outer Hadamard Transform strategy (paper Eq. 6): operand side and the rotations of C after the product.
bool valid_oht_block(int b);
// The OHT kernels put outer / b into the second grid dimension, which may not exceed 65535.
inline bool oht_grid_ok(int64_t outer, int b) { return b > 0 && outer / b <= 65535; }
int launch_oht_quantize(const adahop_operand_t &x, int b, uint8_t *codes, uint8_t *scales, hipStream_t st);
int launch_oht_inverse(float *C, int64_t M, int64_t N, int64_t ldc, int b, hipStream_t st);

size_t pattern_workspace_bytes(const adahop_operand_t &x);
int launch_detect_pattern(const adahop_operand_t &x, double tau, double eps, int32_t *pattern_out, double *stats_out,
                          void *workspace, hipStream_t st);

// One-time set-up per device (function attributes, device properties): the only state the library keeps.
// need(dev) is true until mark(dev) has been called for that device; devices numbered 64 and above are set
// up on every call.
struct device_once_t {
    std::atomic<uint64_t> done{0};
    bool need(int dev) const { return dev < 0 || dev >= 64 || !((done.load(std::memory_order_acquire) >> dev) & 1u); }
    void mark(int dev)
    {
        if (dev >= 0 && dev < 64) done.fetch_or((uint64_t)1 << dev, std::memory_order_release);
    }
};

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

#if defined(__HIPCC__)
// Loads of operand data that a kernel reads exactly once.  They are marked non-temporal (streaming) so that they
// do not displace what the caches hold for the kernels that follow -- above all the packed codes the quantisers
// write, which the product reads next: the product's own prefetch depth (two LDS stages) covers the latency of the
// memory-side cache, not that of HBM under its C-write load.
__device__ __forceinline__ uint4 load_once16(const void *p)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 v = __builtin_nontemporal_load(static_cast<const u32x4 *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint32_t load_once4(const void *p)
{
    return __builtin_nontemporal_load(static_cast<const uint32_t *>(p));
}
__device__ __forceinline__ uint16_t load_once2(const uint16_t *p) { return __builtin_nontemporal_load(p); }

__device__ __forceinline__ float bf16_lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }
__device__ __forceinline__ float bf16_one(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
#endif

} // namespace adahop
