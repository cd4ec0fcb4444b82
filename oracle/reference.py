"""Python face of the CPU oracle (ctypes over oracle/adahop_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module.  It
never touches the GPU library and the GPU library never touches it.

Operands are passed as the 2-D uint16 array of bf16 bit patterns *as stored* plus a flag:
k_contig=True means the array is [outer, K]; k_contig=False means it is [K, outer] (paper Eq. 1-3:
the forward product has both operands K-contiguous, dgrad has a K-strided B, wgrad has both K-strided).

The whole-path function `adahop_gemm` strings the steps together in the order of the paper's
pipeline (App. F: FOID -> IHT + quantise on the residual -> MXFP4 product + BF16 outlier product ->
sum), for the five strategies none / IHT / IHT+OE-row (Eq. 7) / IHT+OE-col (Eq. 8) / IHT+OE-K.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

NONE, IHT, IHT_OE_ROW, IHT_OE_COL, IHT_OE_K, OHT = range(6)

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        _lib.orc_e8m0_from_amax.restype = C.c_uint8
        _lib.orc_e8m0_from_amax.argtypes = [C.c_float]
        _lib.orc_e2m1_encode.restype = C.c_uint8
        _lib.orc_e2m1_encode.argtypes = [C.c_float]
        _lib.orc_num_threads.restype = C.c_int
        _lib.orc_e2m1_encode_sr.restype = C.c_uint8
        _lib.orc_e2m1_encode_sr.argtypes = [C.c_float, C.c_uint32]
        _lib.orc_sr_bits.restype = C.c_uint32
        _lib.orc_sr_bits.argtypes = [C.c_uint64, C.c_int64, C.c_int64]
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _i64(x):
    return C.c_int64(int(x))


def _operand(bits, k_contig):
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    assert bits.ndim == 2
    outer, K = (bits.shape if k_contig else bits.shape[::-1])
    return bits, outer, K, bits.shape[1]


def _mask(m, n):
    if m is None:
        return None
    m = np.ascontiguousarray(m, dtype=np.uint8)
    assert m.shape == (n,)
    return m


def _sel(s):
    return None if s is None else np.ascontiguousarray(s, dtype=np.int32)


def num_threads():
    return int(lib().orc_num_threads())


def fwht(v, b):
    """(1/sqrt(b)) H_b v on a length-b fp32 vector (Eq. 5, one block)."""
    v = np.array(v, dtype=np.float32, copy=True)
    assert v.shape == (b,)
    lib().orc_fwht(_p(v), C.c_int(b))
    return v


def e8m0_from_amax(amax):
    return int(lib().orc_e8m0_from_amax(C.c_float(float(amax))))


def e2m1_encode(q):
    return int(lib().orc_e2m1_encode(C.c_float(float(q))))


def foid_scores(bits, k_contig, axis):
    bits, outer, K, ld = _operand(bits, k_contig)
    out = np.empty(outer if axis == 0 else K, dtype=np.float32)
    lib().orc_foid_scores(_p(bits), _i64(outer), _i64(K), _i64(ld), C.c_int(int(k_contig)), C.c_int(axis), _p(out))
    return out


def topk(scores, k):
    scores = np.ascontiguousarray(scores, dtype=np.float32)
    idx = np.empty(k, dtype=np.int32)
    mask = np.empty(scores.shape[0], dtype=np.uint8)
    lib().orc_topk(_p(scores), _i64(scores.shape[0]), _i64(k), _p(idx), _p(mask))
    return idx, mask


def foid_topk(bits, k_contig, axis, k):
    return topk(foid_scores(bits, k_contig, axis), k)


def transform(bits, k_contig, iht_block, zero_outer=None, zero_k=None):
    """fp32 values that enter the quantiser: residual masking, then the block transform."""
    bits, outer, K, ld = _operand(bits, k_contig)
    zo, zk = _mask(zero_outer, outer), _mask(zero_k, K)
    out = np.empty((outer, K), dtype=np.float32)
    lib().orc_transform(_p(bits), _i64(outer), _i64(K), _i64(ld), C.c_int(int(k_contig)), C.c_int(iht_block),
                        _p(zo), _p(zk), _p(out))
    return out


def philox4x32_10(ctr, key):
    """One Philox4x32-10 block: ctr 4 x uint32, key 2 x uint32 -> 4 x uint32."""
    c = (C.c_uint32 * 4)(*[int(x) for x in ctr])
    k = (C.c_uint32 * 2)(*[int(x) for x in key])
    out = (C.c_uint32 * 4)()
    lib().orc_philox4x32_10(c, k, out)
    return [int(x) for x in out]


def sr_bits(seed, o, kk):
    """The 16 random bits that stochastic rounding uses for element (o, kk) under `seed`."""
    return int(lib().orc_sr_bits(C.c_uint64(int(seed)), _i64(o), _i64(kk)))


def e2m1_encode_sr(q, r16):
    return int(lib().orc_e2m1_encode_sr(C.c_float(q), C.c_uint32(int(r16))))


def iht_quantize(bits, k_contig, iht_block, zero_outer=None, zero_k=None, sr_seed=None):
    """Residual masking -> block transform -> MXFP4.  sr_seed: round the elements stochastically (Philox
    stream of that seed) instead of to nearest even."""
    bits, outer, K, ld = _operand(bits, k_contig)
    assert K % 32 == 0 and (iht_block == 0 or K % iht_block == 0)
    zo, zk = _mask(zero_outer, outer), _mask(zero_k, K)
    codes = np.empty((outer, K // 2), dtype=np.uint8)
    scales = np.empty((outer, K // 32), dtype=np.uint8)
    if sr_seed is not None:
        lib().orc_iht_quantize_sr(_p(bits), _i64(outer), _i64(K), _i64(ld), C.c_int(int(k_contig)),
                                  C.c_int(iht_block), _p(zo), _p(zk), C.c_uint64(int(sr_seed)), _p(codes), _p(scales))
        return codes, scales
    lib().orc_iht_quantize(_p(bits), _i64(outer), _i64(K), _i64(ld), C.c_int(int(k_contig)), C.c_int(iht_block),
                           _p(zo), _p(zk), _p(codes), _p(scales))
    return codes, scales


def quantize_mx(bits, k_contig):
    return iht_quantize(bits, k_contig, 0)


def mx_gemm(a_codes, a_scales, b_codes, b_scales, rows=None, cols=None):
    """Emulated MXFP4 product in double: out[r, c] = <dequant A[rows[r]], dequant B[cols[c]]>."""
    a_codes = np.ascontiguousarray(a_codes, dtype=np.uint8)
    b_codes = np.ascontiguousarray(b_codes, dtype=np.uint8)
    a_scales = np.ascontiguousarray(a_scales, dtype=np.uint8)
    b_scales = np.ascontiguousarray(b_scales, dtype=np.uint8)
    K = a_codes.shape[1] * 2
    assert b_codes.shape[1] * 2 == K
    rows, cols = _sel(rows), _sel(cols)
    nr = a_codes.shape[0] if rows is None else rows.shape[0]
    nc = b_codes.shape[0] if cols is None else cols.shape[0]
    out = np.empty((nr, nc), dtype=np.float64)
    lib().orc_mx_gemm(_i64(K), _p(a_codes), _p(a_scales), _p(b_codes), _p(b_scales), _p(rows), _i64(nr),
                      _p(cols), _i64(nc), _p(out))
    return out


def bf16_gemm(a_bits, a_k_contig, b_bits, b_k_contig, a_zero_outer=None, b_zero_outer=None, zero_k=None,
              ksel=None, rows=None, cols=None):
    """Double-precision product on the bf16 values themselves (see orc_bf16_gemm)."""
    a_bits, M, K, a_ld = _operand(a_bits, a_k_contig)
    b_bits, N, Kb, b_ld = _operand(b_bits, b_k_contig)
    assert K == Kb
    azo, bzo, zk = _mask(a_zero_outer, M), _mask(b_zero_outer, N), _mask(zero_k, K)
    ksel, rows, cols = _sel(ksel), _sel(rows), _sel(cols)
    nr = M if rows is None else rows.shape[0]
    nc = N if cols is None else cols.shape[0]
    nk = 0 if ksel is None else ksel.shape[0]
    out = np.empty((nr, nc), dtype=np.float64)
    lib().orc_bf16_gemm(_p(a_bits), _i64(a_ld), C.c_int(int(a_k_contig)), _p(b_bits), _i64(b_ld),
                        C.c_int(int(b_k_contig)), _i64(K), _p(azo), _p(bzo), _p(zk), _p(ksel), _i64(nk),
                        _p(rows), _i64(nr), _p(cols), _i64(nc), _p(out))
    return out


def exact_gemm(a_bits, a_k_contig, b_bits, b_k_contig, rows=None, cols=None):
    """A*B in double on the bf16 inputs: the quality reference (left-hand side of Eq. 4)."""
    return bf16_gemm(a_bits, a_k_contig, b_bits, b_k_contig, rows=rows, cols=cols)


def adahop_gemm(a_bits, a_k_contig, b_bits, b_k_contig, strategy, iht_block, k=0, idx=None, rows=None, cols=None,
                sr_seed_a=None, sr_seed_b=None):
    """The whole per-GEMM path.  A is logical [M, K], B is logical [N, K] (i.e. B^T), C is [M, N].

    rows / cols: optional index samples; C is returned on rows x cols only.
    idx: optional externally chosen extraction indices (else FOID picks them).
    sr_seed_a / sr_seed_b: stochastic rounding of that operand's elements with this seed.
    Returns dict(C, a_codes, a_scales, b_codes, b_scales, idx).
    """
    a_bits, M, K, _ = _operand(a_bits, a_k_contig)
    b_bits, N, _, _ = _operand(b_bits, b_k_contig)
    rows_a = np.arange(M, dtype=np.int32) if rows is None else _sel(rows)
    cols_a = np.arange(N, dtype=np.int32) if cols is None else _sel(cols)
    b_iht = 0 if strategy == NONE else iht_block
    a_zo = b_zo = zk = None
    sel = np.zeros(0, dtype=np.int32)
    if strategy in (IHT_OE_ROW, IHT_OE_COL, IHT_OE_K) and k > 0:
        dim = {IHT_OE_ROW: M, IHT_OE_COL: N, IHT_OE_K: K}[strategy]
        if idx is not None:
            sel = np.sort(_sel(idx))
            mask = np.zeros(dim, dtype=np.uint8)
            mask[sel] = 1
        elif strategy == IHT_OE_ROW:      # rows of A, scored over their first 64 K-elements
            sel, mask = foid_topk(a_bits, a_k_contig, 0, k)
        elif strategy == IHT_OE_COL:      # columns of B, scored over their first 64 K-elements
            sel, mask = foid_topk(b_bits, b_k_contig, 0, k)
        else:                             # K-channels, scored on A over its first 64 rows
            sel, mask = foid_topk(a_bits, a_k_contig, 1, k)
        if strategy == IHT_OE_ROW:
            a_zo = mask
        elif strategy == IHT_OE_COL:
            b_zo = mask
        else:
            zk = mask
    a_codes, a_scales = iht_quantize(a_bits, a_k_contig, b_iht, a_zo, zk, sr_seed=sr_seed_a)
    b_codes, b_scales = iht_quantize(b_bits, b_k_contig, b_iht, b_zo, zk, sr_seed=sr_seed_b)
    Cm = mx_gemm(a_codes, a_scales, b_codes, b_scales, rows_a, cols_a)
    if sel.size:
        if strategy == IHT_OE_ROW:        # C[S, :] += A[S, :] B   (Eq. 7)
            pos = np.nonzero(np.isin(rows_a, sel))[0]
            if pos.size:
                Cm[pos, :] += bf16_gemm(a_bits, a_k_contig, b_bits, b_k_contig, rows=rows_a[pos], cols=cols_a)
        elif strategy == IHT_OE_COL:      # C[:, S] += A B[:, S]   (Eq. 8)
            pos = np.nonzero(np.isin(cols_a, sel))[0]
            if pos.size:
                Cm[:, pos] += bf16_gemm(a_bits, a_k_contig, b_bits, b_k_contig, rows=rows_a, cols=cols_a[pos])
        else:                             # C += A[:, S] B[S, :]
            Cm += bf16_gemm(a_bits, a_k_contig, b_bits, b_k_contig, ksel=sel, rows=rows_a, cols=cols_a)
    return dict(C=Cm, a_codes=a_codes, a_scales=a_scales, b_codes=b_codes, b_scales=b_scales, idx=sel)


# ------------------------------------------------------------------------------------------------
# Outer Hadamard Transform (paper Eq. 6): the comparison strategy
# ------------------------------------------------------------------------------------------------
def hadamard_matrix(b):
    """Normalised Sylvester Hadamard matrix H_b (float64), by the doubling recursion H_2n = [[H, H], [H, -H]]."""
    H = np.ones((1, 1))
    while H.shape[0] < b:
        H = np.block([[H, H], [H, -H]])
    assert H.shape[0] == b, "b must be a power of two"
    return H / np.sqrt(float(b))


def oht_transform(bits, k_contig, block):
    """fp32 values that enter the quantiser under OHT: block transform along the OUTER index (H_m A; H_n B^T)."""
    bits, outer, K, ld = _operand(bits, k_contig)
    assert outer % block == 0
    out = np.empty((outer, K), dtype=np.float32)
    lib().orc_oht_transform(_p(bits), _i64(outer), _i64(K), _i64(ld), C.c_int(int(k_contig)), C.c_int(block), _p(out))
    return out


def oht_quantize(bits, k_contig, block):
    bits, outer, K, ld = _operand(bits, k_contig)
    assert K % 32 == 0 and outer % block == 0
    codes = np.empty((outer, K // 2), dtype=np.uint8)
    scales = np.empty((outer, K // 32), dtype=np.uint8)
    lib().orc_oht_quantize(_p(bits), _i64(outer), _i64(K), _i64(ld), C.c_int(int(k_contig)), C.c_int(block),
                           _p(codes), _p(scales))
    return codes, scales


def oht_inverse(Cq, block_m, block_n):
    """H_m^T Cq H_n^T with block-diagonal H (Eq. 6, the rotations after the product), in double, written as the
    two matrix products they are."""
    M, N = Cq.shape
    assert M % block_m == 0 and N % block_n == 0
    Hm = np.kron(np.eye(M // block_m), hadamard_matrix(block_m))
    Hn = np.kron(np.eye(N // block_n), hadamard_matrix(block_n))
    return Hm.T @ np.asarray(Cq, dtype=np.float64) @ Hn.T


def oht_gemm(a_bits, a_k_contig, b_bits, b_k_contig, block):
    """C_OHT = H_m^T ( Q(H_m A) Q(B H_n) ) H_n^T (Eq. 6) with block-diagonal transforms of size `block` on both
    outer dimensions.  Returns dict(C, a_codes, a_scales, b_codes, b_scales)."""
    a_codes, a_scales = oht_quantize(a_bits, a_k_contig, block)
    b_codes, b_scales = oht_quantize(b_bits, b_k_contig, block)
    Cq = mx_gemm(a_codes, a_scales, b_codes, b_scales)
    return dict(C=oht_inverse(Cq, block, block), Cq=Cq, a_codes=a_codes, a_scales=a_scales, b_codes=b_codes,
                b_scales=b_scales)


def round_to_bf16(x):
    """bf16 bit patterns (uint16) of a float64 array: each value rounded ONCE to the nearest number with an
    8-bit significand (exponent range of fp32, gradual underflow), ties to the even significand.

    The paper's kernels emit C in BF16 (App. F, last item); the library's optional bf16 output is compared
    with this rounding of the double-precision result.  Written from the definition of the format, not
    through an fp32 intermediate (which would round twice)."""
    x = np.asarray(x, dtype=np.float64)
    mag = np.abs(x)
    _, e = np.frexp(mag)                               # mag = m 2^e with m in [0.5, 1)
    e = np.maximum(e, -125)                            # below 2^-126 the spacing stays that of the smallest normal
    quantum = np.ldexp(1.0, e - 8)                     # spacing of 8-bit significands in [2^(e-1), 2^e)
    val = np.rint(mag / quantum) * quantum             # np.rint rounds half to even; the division is exact
    val = np.where(val >= np.ldexp(1.0, 128), np.inf, val)
    f32 = np.copysign(val, x).astype(np.float32)       # exact: val has at most 8 significant bits
    return (f32.view(np.uint32) >> 16).astype(np.uint16)


def bf16_to_double(bits):
    """Values of bf16 bit patterns (uint16 array) as float64 (exact)."""
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# ------------------------------------------------------------------------------------------------
# Outlier-pattern detection and strategy table (paper Sec. 4.1, 4.2, App. A)
# ------------------------------------------------------------------------------------------------
PATTERN_NONE, PATTERN_OUTER, PATTERN_K = range(3)


def _ratio(a, b):
    if b > 0.0:
        return a / b
    return float("inf") if a > 0.0 else 0.0


def detect_pattern(bits, k_contig, tau=2.0, eps=1e-12):
    """App. A on the operand in its logical [outer, K] shape, in float64 with numpy's var / std / mean
    (population forms): the variance of every outer index and of every K index, the coefficient of
    variation of each variance vector, each divided by its IID value sqrt(2 / (samples - 1)), and the
    class from the ratio of the two against tau.  "Outer-wise" is the paper's Row-wise for A (m x k)
    and Column-wise for B (k x n); "K-wise" is Column-wise for A and Row-wise for B.
    Returns (pattern, [CV_outer, CV_k, CVhat_outer, CVhat_k])."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    T = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    if not k_contig:
        T = T.T
    outer, K = T.shape
    v_outer = T.var(axis=1)
    v_k = T.var(axis=0)
    cv_outer = v_outer.std() / (v_outer.mean() + eps)
    cv_k = v_k.std() / (v_k.mean() + eps)
    hat_outer = cv_outer / np.sqrt(2.0 / (K - 1))
    hat_k = cv_k / np.sqrt(2.0 / (outer - 1))
    if _ratio(hat_outer, hat_k) > tau:
        p = PATTERN_OUTER
    elif _ratio(hat_k, hat_outer) > tau:
        p = PATTERN_K
    else:
        p = PATTERN_NONE
    return p, np.array([cv_outer, cv_k, hat_outer, hat_k])


def vote_pattern(patterns):
    """Sec. 4.1: the calibrated pattern of a tensor is the majority among its per-step classifications (the
    paper calibrates over 30 steps).  The class that occurs most often wins; when two or three classes share
    the top count no pattern dominates and the result is PATTERN_NONE (the paper does not say; NONE is the
    class that claims no structure, and it sends the pair to plain IHT)."""
    counts = [sum(1 for p in patterns if p == c) for c in (PATTERN_NONE, PATTERN_OUTER, PATTERN_K)]
    best = max(counts)
    winners = [c for c in (PATTERN_NONE, PATTERN_OUTER, PATTERN_K) if counts[c] == best]
    return winners[0] if len(winners) == 1 else PATTERN_NONE


def select_strategy(pattern_a, pattern_b, level=1):
    """Sec. 4.2: pairs whose outliers lie along K in both operands (CN, NN, CR) take IHT alone; outlier
    rows of A (RN) take OE-Left; outlier columns of B (RC, NC, CC) take OE-Right; AdaHOP-Lv2 computes CC
    fully in BF16.  The pairs the section does not list follow the same argument (RR like RN, NR like NN).
    Returns (strategy, full_bf16)."""
    if pattern_b == PATTERN_OUTER:
        if level == 2 and pattern_a == PATTERN_K:
            return NONE, True
        return IHT_OE_COL, False
    if pattern_a == PATTERN_OUTER:
        return IHT_OE_ROW, False
    return IHT, False
