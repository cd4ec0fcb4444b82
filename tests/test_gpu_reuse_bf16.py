"""GPU parity of the quantise-once / bf16-output variants of the whole path (run with -m gpu).

Bars.  Packed operands: codes and scales bit-exact against the oracle's residual -> IHT -> MXFP4 step; a
product that takes them must give exactly the bits of the product that quantises in the call (same kernels,
same inputs) and stay within 1e-3 relative Frobenius of the oracle.  bf16 output: every element is the fp32
accumulator rounded once, so it must equal the fp32 path's C rounded to bf16 bit for bit.  Against the
oracle's double-precision C the bar is that of a correct single rounding of a value within the fp32
accumulation error d of the oracle's: |C_gpu - C_oracle| <= half a bf16 step at that magnitude + d, with
d[i, j] = 2^-20 |A[i, :]|_2 |B[j, :]|_2 (the transform keeps those norms; a length-K fp32 accumulation of exact
products errs by about sqrt(K) 2^-24 |C|, and |C| is about |A_i| |B_j| / sqrt(K) for these inputs, so d is some
tens of times the expected error and still ~1/60 of half a step: a truncating or double rounding fails).
Where the unrounded values straddle a rounding boundary the bf16 results differ by one step -- expected for
about 2^8 * 1e-6 < 0.1 % of the elements; the test allows 1 %.  Relative Frobenius error <= 1e-3 as everywhere.
"""
import numpy as np
import pytest

from oracle import reference as orc
from paper_2604_02525_amd import inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def say(*a):
    print("[case]", *a, flush=True)


@pytest.fixture(scope="module")
def ah():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2604_02525_amd import binding
    binding.lib()
    return binding


def dev_op(ah, op):
    return ah.Operand.from_bits(op.bits, op.k_contig)


def host(t):
    return t.cpu().numpy()


def bits_of(t):
    return host(t.view(torch.int16)).view(np.uint16)


def ordered(bits):
    """bf16 bit patterns -> integers that are monotone in the value (one step = one representable number)."""
    b = bits.astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7fff), b)


def logical(op):
    """[outer, K] float64 values of an inputs.Operand."""
    v = orc.bf16_to_double(op.bits)
    return v if op.k_contig else v.T


def check_bf16_against_oracle(got_bits, ref_c, A, B, what):
    want = orc.round_to_bf16(ref_c)
    frac = float(np.mean(ordered(got_bits) != ordered(want)))
    v_got, v_want = orc.bf16_to_double(got_bits), orc.bf16_to_double(want)
    err = float(np.linalg.norm(v_got - v_want) / max(np.linalg.norm(v_want), 1e-300))
    d = 2.0 ** -20 * np.outer(np.linalg.norm(logical(A), axis=1), np.linalg.norm(logical(B), axis=1))
    big = np.maximum(np.abs(ref_c), np.abs(v_got))
    half_step = np.ldexp(0.5, np.frexp(big)[1] - 8)          # big in [2^(e-1), 2^e): numbers are 2^(e-8) apart
    excess = np.abs(v_got - ref_c) - half_step - d
    say(f"  {what}: {frac:.2e} of the elements differ from the rounded oracle, rel. Frobenius {err:.2e}, "
        f"worst |error| - half step - d = {excess.max():.2e}")
    assert excess.max() <= 0.0
    assert frac < 0.01
    assert err < 1e-3


def small_pair(kind, M=328, N=200, K=512):
    a_kc, b_kc = {"fwd": (True, True), "dgrad": (True, False), "wgrad": (False, False)}[kind]
    A_log = inputs.matrix(M, K, 1.0, 70, row_outliers=(5, 100.0, 100.0), col_outliers=(6, 50.0, 50.0))
    B_log = inputs.matrix(N, K, 0.02, 71, row_outliers=(4, 30.0, 30.0))
    A = inputs.Operand(A_log if a_kc else np.ascontiguousarray(A_log.T), a_kc)
    B = inputs.Operand(B_log if b_kc else np.ascontiguousarray(B_log.T), b_kc)
    return A, B


K_OF = {inputs.NONE: 0, inputs.IHT: 0, inputs.IHT_OE_ROW: 9, inputs.IHT_OE_COL: 7, inputs.IHT_OE_K: 21}


# ----------------------------------------------------------------------------- bf16 output

@pytest.mark.parametrize("kind", ["fwd", "wgrad"])
@pytest.mark.parametrize("strategy", [inputs.NONE, inputs.IHT, inputs.IHT_OE_ROW, inputs.IHT_OE_COL, inputs.IHT_OE_K])
def test_bf16_output_small_ragged(ah, strategy, kind):
    A, B = small_pair(kind)
    k = K_OF[strategy]
    say("bf16 output, small ragged", kind, inputs.STRATEGY_NAMES[strategy])
    dA, dB = dev_op(ah, A), dev_op(ah, B)
    c32 = ah.adahop_gemm(dA, dB, strategy, 128, k)["C"]
    out = ah.adahop_gemm(dA, dB, strategy, 128, k, c_bf16=True)
    torch.cuda.synchronize()
    assert out["C"].dtype == torch.bfloat16
    assert np.array_equal(bits_of(out["C"]), bits_of(c32.to(torch.bfloat16))), "not the fp32 result rounded once"
    ref = orc.adahop_gemm(A.bits, A.k_contig, B.bits, B.k_contig, strategy, 128, k)
    check_bf16_against_oracle(bits_of(out["C"]), ref["C"], A, B, "vs oracle")


@pytest.mark.parametrize("strategy,k", [(inputs.IHT, 0), (inputs.IHT_OE_K, 70), (inputs.IHT_OE_ROW, 6),
                                        (inputs.IHT_OE_COL, 3)])
@pytest.mark.parametrize("M,N", [(768, 512), (840, 600)])
def test_bf16_output_tiled_kernel(ah, strategy, k, M, N):
    """K % 256 == 0: the LDS-pipelined kernel writes the whole 256x256 tiles (packed column pairs), the
    bounds-checked kernel the ragged edges of the second shape."""
    K = 1024
    A = inputs.Operand(inputs.matrix(M, K, 1.0, 72, row_outliers=(4, 100.0, 100.0), col_outliers=(5, 50.0, 50.0)), True)
    B = inputs.Operand(np.ascontiguousarray(inputs.matrix(N, K, 0.02, 73).T), False)
    say("bf16 output, tiled", inputs.STRATEGY_NAMES[strategy], k, M, N)
    dA, dB = dev_op(ah, A), dev_op(ah, B)
    c32 = ah.adahop_gemm(dA, dB, strategy, 256, k)["C"]
    out = ah.adahop_gemm(dA, dB, strategy, 256, k, c_bf16=True)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(out["C"]), bits_of(c32.to(torch.bfloat16)))
    ref = orc.adahop_gemm(A.bits, A.k_contig, B.bits, B.k_contig, strategy, 256, k)
    check_bf16_against_oracle(bits_of(out["C"]), ref["C"], A, B, "vs oracle")


def test_bf16_output_odd_leading_dimension_and_untouched_padding(ah):
    """A ldc that is no multiple of 8 (or a C that is not 16-byte aligned) rules out the 16-byte stores of the
    tiled kernel: the bounds-checked kernel takes the whole product; the last case is a padded C that the tiled
    kernel does take.  Nothing outside [M, N] may be written."""
    M, N, K = 512, 512, 512
    A = inputs.Operand(inputs.matrix(M, K, 1.0, 74, col_outliers=(3, 40.0, 40.0)), True)
    B = inputs.Operand(inputs.matrix(N, K, 0.02, 75), True)
    dA, dB = dev_op(ah, A), dev_op(ah, B)
    ref = orc.adahop_gemm(A.bits, A.k_contig, B.bits, B.k_contig, inputs.IHT_OE_K, 128, 5)
    for ld, off in ((N + 1, 0), (N + 6, 1), (N + 6, 2), (N + 8, 8)):
        say("bf16 output with ldc", ld, "element offset", off)
        buf = torch.full((M * ld + 16,), -7.0, dtype=torch.bfloat16, device="cuda")
        Cv = buf[off:off + M * ld].view(M, ld)[:, :N]
        out = ah.adahop_gemm(dA, dB, inputs.IHT_OE_K, 128, 5, Cout=Cv)
        torch.cuda.synchronize()
        check_bf16_against_oracle(bits_of(out["C"].contiguous()), ref["C"], A, B, "vs oracle")
        pad = buf[off:off + M * ld].view(M, ld)[:, N:]
        assert bool((pad == -7.0).all()) and bool((buf[:off] == -7.0).all()) and bool((buf[off + M * ld:] == -7.0).all())


def test_gemm_mx_bf16out_on_packed_operands(ah):
    M, N, K = 520, 300, 768
    A = inputs.Operand(inputs.matrix(M, K, 1.0, 76), True)
    B = inputs.Operand(inputs.matrix(N, K, 0.02, 77), True)
    say("gemm_mx bf16 out")
    ac, asc = ah.adahop_quantize_mx(dev_op(ah, A))
    bc, bsc = ah.adahop_quantize_mx(dev_op(ah, B))
    c32 = ah.adahop_gemm_mx(ac, asc, bc, bsc)
    c16 = ah.adahop_gemm_mx(ac, asc, bc, bsc, c_bf16=True)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(c16), bits_of(c32.to(torch.bfloat16)))
    ref = orc.mx_gemm(host(ac), host(asc), host(bc), host(bsc))
    check_bf16_against_oracle(bits_of(c16), ref, A, B, "vs oracle")


# ----------------------------------------------------------------------------- quantise-once reuse

@pytest.mark.parametrize("kind", ["fwd", "dgrad", "wgrad"])
def test_pack_operand_matches_oracle_residual_quantiser(ah, kind):
    A, B = small_pair(kind)
    M, N, K = A.outer, B.outer, A.K
    rng = np.random.default_rng(11)
    for strategy, dim in ((inputs.NONE, 0), (inputs.IHT, 0), (inputs.IHT_OE_ROW, M), (inputs.IHT_OE_COL, N),
                          (inputs.IHT_OE_K, K)):
        k = K_OF[strategy]
        idx = rng.permutation(dim)[:k].astype(np.int32) if k else None
        idx_d = None if idx is None else torch.from_numpy(idx).cuda()
        mask = None
        if k:
            mask = np.zeros(dim, np.uint8)
            mask[idx] = 1
        for is_b, X in ((0, A), (1, B)):
            say("pack_operand", kind, inputs.STRATEGY_NAMES[strategy], "B" if is_b else "A")
            codes, scales = ah.adahop_pack_operand(dev_op(ah, X), is_b, strategy, 64, k, idx_d)
            torch.cuda.synchronize()
            zo = mask if (strategy, is_b) in ((inputs.IHT_OE_ROW, 0), (inputs.IHT_OE_COL, 1)) else None
            zk = mask if strategy == inputs.IHT_OE_K else None
            rc, rs = orc.iht_quantize(X.bits, X.k_contig, 0 if strategy == inputs.NONE else 64, zo, zk)
            assert np.array_equal(host(scales), rs)
            assert np.array_equal(host(codes), rc)


def test_activation_packed_once_feeds_several_projections(ah):
    """One X (A operand), three weights: pure IHT, then OE-K with the channels FOID picks on X."""
    T, d_in = 520, 1024
    X = inputs.Operand(inputs.matrix(T, d_in, 1.0, 80, col_outliers=(6, 30.0, 80.0)), True)
    Ws = [inputs.Operand(inputs.matrix(n, d_in, 0.02, 81 + i), True) for i, n in enumerate((256, 300, 768))]
    dX = dev_op(ah, X)
    for strategy, k in ((inputs.IHT, 0), (inputs.IHT_OE_K, 6)):
        idx_d = None
        if k:
            idx_d, _, _ = ah.adahop_foid_topk(dX, 1, k)
        packed = ah.adahop_pack_operand(dX, 0, strategy, 256, k, idx_d)
        for W in Ws:
            say("shared activation", inputs.STRATEGY_NAMES[strategy], "N =", W.outer)
            dW = dev_op(ah, W)
            plain = ah.adahop_gemm(dX, dW, strategy, 256, k, idx=idx_d)
            reuse = ah.adahop_gemm(dX, dW, strategy, 256, k, idx=idx_d, a_packed=packed)
            torch.cuda.synchronize()
            assert np.array_equal(host(packed[0]), host(plain["a_codes"]))
            assert np.array_equal(host(packed[1]), host(plain["a_scales"]))
            assert np.array_equal(host(reuse["C"]), host(plain["C"]))
            ref = orc.adahop_gemm(X.bits, True, W.bits, True, strategy, 256, k)
            if k:
                assert np.array_equal(np.sort(host(idx_d)), ref["idx"])
            err = np.linalg.norm(host(reuse["C"]).astype(np.float64) - ref["C"]) / np.linalg.norm(ref["C"])
            say(f"  vs oracle {err:.3e}")
            assert err < 1e-3


@pytest.mark.parametrize("strategy", [inputs.IHT_OE_ROW, inputs.IHT_OE_COL])
def test_weight_packed_once_over_microbatches(ah, strategy):
    """dgrad-like products G_X = G_Y W with one K-strided W (B operand) and several G_Y.  Under OE-row the
    residual of B does not depend on the extracted rows, so FOID may still run inside the call; under OE-col
    it does, so the caller passes the indices it packed with."""
    d_out, d_in = 512, 520
    W = inputs.Operand(inputs.matrix(d_out, d_in, 0.02, 90, col_outliers=(5, 30.0, 30.0)), False)   # [K, N] as stored
    dW = dev_op(ah, W)
    k = 5
    idx_d = None
    if strategy == inputs.IHT_OE_COL:
        idx_d, _, _ = ah.adahop_foid_topk(dW, 0, k)
    packed = ah.adahop_pack_operand(dW, 1, strategy, 128, k, idx_d)
    for i, T in enumerate((256, 328)):
        G = inputs.Operand(inputs.matrix(T, d_out, 1e-3, 91 + i, row_outliers=(4, 100.0, 100.0)), True)
        dG = dev_op(ah, G)
        say("shared weight", inputs.STRATEGY_NAMES[strategy], "T =", T)
        plain = ah.adahop_gemm(dG, dW, strategy, 128, k, idx=idx_d)
        reuse = ah.adahop_gemm(dG, dW, strategy, 128, k, idx=idx_d, b_packed=packed, c_bf16=True)
        torch.cuda.synchronize()
        assert np.array_equal(host(reuse["idx"]), host(plain["idx"]))
        assert np.array_equal(bits_of(reuse["C"]), bits_of(plain["C"].to(torch.bfloat16)))
        ref = orc.adahop_gemm(G.bits, True, W.bits, False, strategy, 128, k)
        assert np.array_equal(np.sort(host(reuse["idx"])), ref["idx"])
        check_bf16_against_oracle(bits_of(reuse["C"]), ref["C"], G, W, "vs oracle")


def test_packed_operand_that_depends_on_indices_needs_them(ah):
    A, B = small_pair("fwd")
    dA, dB = dev_op(ah, A), dev_op(ah, B)
    idx_d, _, _ = ah.adahop_foid_topk(dA, 0, 4)
    packed = ah.adahop_pack_operand(dA, 0, inputs.IHT_OE_ROW, 64, 4, idx_d)
    with pytest.raises(ah.AdahopError) as e:
        ah.adahop_gemm(dA, dB, inputs.IHT_OE_ROW, 64, 4, a_packed=packed)
    assert e.value.status == ah.ADAHOP_E_INVALID_ARG
