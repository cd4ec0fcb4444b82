"""Pins for the CPU oracle: every check here is against something other than the oracle itself --
the definition of the Sylvester matrix, exact algebraic identities, the OCP MX value table, brute
force, numpy's float64 routines, or closed forms.  No GPU.
"""
import os

import numpy as np
import pytest

from oracle import reference as orc
from paper_2604_02525_amd import inputs


# ----------------------------------------------------------------------------- helpers (test-side)

def bf16_bits(x):
    """fp32 array -> bf16 bit patterns (RNE), done with integer arithmetic on the fp32 bits."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)
    return r


def bits_to_f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def sylvester(n):
    """H_1 = [1];  H_2n = [[H, H], [H, -H]]  (integer entries)."""
    H = np.array([[1]], dtype=np.int64)
    while H.shape[0] < n:
        H = np.block([[H, H], [H, -H]])
    return H


def load_table(path):
    rows = []
    for line in open(path):
        line = line.strip()
        if line and not line.startswith("#"):
            rows.append(line.split())
    return rows


def e2m1_table(golden_dir):
    t = {int(c): float(v) for c, v in load_table(os.path.join(golden_dir, "e2m1_values.txt"))}
    assert len(t) == 16
    return t


def unpack_codes(codes):
    lo = codes & 15
    hi = codes >> 4
    return np.stack([lo, hi], axis=-1).reshape(codes.shape[0], -1)


def dequant(codes, scales, table):
    """Independent dequantiser: value table from the golden file, scale 2^(s-127)."""
    c = unpack_codes(codes)
    vals = np.vectorize(table.get)(c).astype(np.float64)
    s = np.repeat(scales.astype(np.int64), 32, axis=1)
    return vals * np.exp2((s - 127).astype(np.float64))


# ----------------------------------------------------------------------------- Hadamard

@pytest.mark.parametrize("b", [2, 4, 8, 16, 32, 64, 128, 256])
def test_sylvester_is_hadamard_and_fwht_matches_its_columns(b):
    H = sylvester(b)
    assert np.array_equal(H @ H.T, b * np.eye(b, dtype=np.int64))
    assert np.array_equal(H, H.T)
    c = np.float32(1.0 / np.sqrt(float(b)))
    for i in range(b):
        e = np.zeros(b, dtype=np.float32)
        e[i] = 1.0
        got = orc.fwht(e, b)
        assert np.array_equal(got, (H[:, i].astype(np.float32) * c)), (b, i)


@pytest.mark.parametrize("b", [32, 64, 128, 256])
def test_fwht_close_to_explicit_matrix_product(b):
    rng = np.random.default_rng(b)
    H = sylvester(b).astype(np.float64)
    for _ in range(8):
        x = rng.standard_normal(b).astype(np.float32)
        ref = H @ x.astype(np.float64) / np.sqrt(float(b))
        got = orc.fwht(x, b).astype(np.float64)
        assert np.max(np.abs(got - ref)) <= 16 * np.log2(b) * np.finfo(np.float32).eps * np.max(np.abs(ref))


def test_fwht_exact_on_integers_block_256():
    rng = np.random.default_rng(7)
    x = rng.integers(-64, 65, size=256).astype(np.float32)
    ref = sylvester(256) @ x.astype(np.int64)          # |ref| <= 256*64 = 2^14: exact in fp32
    got = orc.fwht(x, 256)
    assert np.array_equal(got.astype(np.float64), ref / 16.0)


def test_fwht_stage_order_is_ascending_stride():
    """With a value that rounds differently under the two textbook stage orders the result must be
    the ascending-stride one: ((x0+x1)+(x2+x3)), not ((x0+x2)+(x1+x3))."""
    x = np.array([1.0, 2.0 ** -24, 0.0, 2.0 ** -24], dtype=np.float32)
    f = np.float32
    asc0 = f(f(x[0] + x[1]) + f(x[2] + x[3]))      # h=1 first, then h=2
    desc0 = f(f(x[0] + x[2]) + f(x[1] + x[3]))     # h=2 first, then h=1
    assert asc0 != desc0                            # the probe does discriminate
    got = orc.fwht(x, 4)
    assert got[0] == f(asc0 * f(0.5))


@pytest.mark.parametrize("b", [32, 128, 256])
def test_iht_identity_without_quantisation(b):
    """(A H)(H^T B) = A B  (Eq. 5's remark), with the oracle's fp32 transform and no quantiser."""
    rng = np.random.default_rng(11 + b)
    M, N, K = 24, 40, 2 * b
    A = bf16_bits(rng.standard_normal((M, K)))
    Bt = bf16_bits(rng.standard_normal((N, K)) * 0.02)
    # B stored K-strided, as in dgrad: array [K, N]
    B_store = np.ascontiguousarray(Bt.T)
    Ah = orc.transform(A, True, b).astype(np.float64)
    Bh = orc.transform(B_store, False, b).astype(np.float64)
    exact = bits_to_f64(A) @ bits_to_f64(Bt).T
    got = Ah @ Bh.T
    assert np.linalg.norm(got - exact) / np.linalg.norm(exact) < 2e-6
    # and the oracle's exact product agrees with numpy's float64 matmul
    assert np.allclose(orc.exact_gemm(A, True, B_store, False), exact, rtol=1e-12, atol=1e-12)


def test_transform_is_per_block_and_respects_layout():
    """Block-diagonal I (x) H_b: each K-block only sees its own elements, in both layouts."""
    rng = np.random.default_rng(5)
    b, K, O = 32, 96, 3
    x = rng.standard_normal((O, K)).astype(np.float32)
    bits = bf16_bits(x)
    ref = np.empty((O, K))
    H = sylvester(b) / np.sqrt(float(b))
    xv = bits_to_f64(bits)
    for o in range(O):
        for k0 in range(0, K, b):
            ref[o, k0:k0 + b] = H @ xv[o, k0:k0 + b]
    for kc, store in ((True, bits), (False, np.ascontiguousarray(bits.T))):
        got = orc.transform(store, kc, b)
        assert np.allclose(got, ref, rtol=0, atol=1e-5)


# ----------------------------------------------------------------------------- E2M1 / E8M0

def test_e2m1_encode_brute_force_all_bf16(golden_dir):
    """Every finite bf16 bit pattern, at every power-of-two scaling that keeps it within the format's
    range, against an argmin over the 16 representable values with ties to the even code."""
    table = e2m1_table(golden_dir)
    mags = np.array([table[c] for c in range(8)])
    allbits = np.arange(65536, dtype=np.uint32)
    vals = (allbits << 16).astype(np.uint32).view(np.float32)
    finite = np.isfinite(vals)
    vals = vals[finite]
    checked = 0
    for v in vals:
        a = abs(float(v))
        if a == 0.0:
            scalings = [1.0]
        else:
            e = int(np.floor(np.log2(a)))
            if e < -120:
                continue
            # bring |v| into each binade from 2^-3 up to just below 8
            scalings = [2.0 ** (t - e) for t in (-3, -2, -1, 0, 1, 2)]
        for sc in scalings:
            q = np.float32(v) * np.float32(sc)
            aq = abs(float(q))
            if aq >= 8.0:
                continue
            d = np.abs(mags - aq)
            best = np.flatnonzero(d == d.min())
            m = int(best[0]) if len(best) == 1 else int([c for c in best if c % 2 == 0][0])
            if aq > 6.0:
                m = 7
            want = m | (8 if np.signbit(q) else 0)
            assert orc.e2m1_encode(q) == want, (float(q), want)
            checked += 1
    assert checked > 150000


def test_e2m1_ties_and_saturation(golden_dir):
    table = e2m1_table(golden_dir)
    for mid, want in load_table(os.path.join(golden_dir, "e2m1_ties.txt")):
        for sign in (1.0, -1.0):
            code = orc.e2m1_encode(sign * float(mid))
            assert abs(table[code]) == float(want)
            assert (code >> 3) == (1 if sign < 0 else 0)
    for big in (6.0, 6.5, 7.0, 7.999):
        assert table[orc.e2m1_encode(big)] == 6.0
        assert table[orc.e2m1_encode(-big)] == -6.0
    assert orc.e2m1_encode(-0.0) == 8 and orc.e2m1_encode(-0.1) == 8 and orc.e2m1_encode(0.1) == 0


def test_e8m0_rule(golden_dir):
    for amax, want in load_table(os.path.join(golden_dir, "e8m0_cases.txt")):
        assert orc.e8m0_from_amax(float.fromhex(amax)) == int(want), amax
    assert orc.e8m0_from_amax(0.0) == 0
    # closed form over many exponents and mantissas: amax = m 2^e, m in [1,2)  ->  e + 125
    for e in range(-100, 101, 7):
        for m in (1.0, 1.25, 1.999):
            assert orc.e8m0_from_amax(np.float32(m * 2.0 ** e)) == e + 125


def test_nibble_order_and_scale_layout(golden_dir):
    """Element 2t in the low nibble of byte t; one scale byte per 32 K-elements, K-contiguous."""
    K = 64
    x = np.zeros((2, K), dtype=np.float32)
    x[0, 0] = 6.0      # block 0: amax 6 -> scale 127, element 0 -> code 7
    x[0, 1] = -1.0     # element 1 -> code 10, high nibble of byte 0
    x[0, 33] = 3.0     # block 1: amax 3 -> scale 126 (X = 0.5), 3/0.5 = 6 -> code 7, high nibble of byte 16
    x[1, 62] = 0.5     # row 1 block 1: amax .5 -> X = 2^-3, .5/X = 4 -> code 6, low nibble of byte 31
    codes, scales = orc.quantize_mx(bf16_bits(x), True)
    assert codes.shape == (2, 32) and scales.shape == (2, 2)
    assert codes[0, 0] == (7 | (10 << 4))
    assert codes[0, 16] == (7 << 4)
    assert codes[1, 31] == 6
    assert scales.tolist() == [[127, 126], [0, 124]]
    expect_zero = np.ones_like(codes, dtype=bool)
    expect_zero[0, 0] = expect_zero[0, 16] = expect_zero[1, 31] = False
    assert np.all(codes[expect_zero] == 0)


def test_quantiser_round_trip_and_none_gemm_is_exact(golden_dir):
    """Blocks made of E2M1 values times a common power of two (with a 4 or 6 present) quantise to
    themselves, so strategy `none` must reproduce the exact product (numpy float64 matmul)."""
    table = e2m1_table(golden_dir)
    rng = np.random.default_rng(3)
    M, N, K = 16, 24, 128

    def make(rows):
        codes = rng.integers(0, 16, size=(rows, K))
        exps = rng.integers(-6, 7, size=(rows, K // 32))
        codes[:, ::32] = rng.choice([6, 7, 14, 15], size=(rows, K // 32))   # a 4 or a 6 per block
        vals = np.vectorize(table.get)(codes) * np.exp2(np.repeat(exps, 32, axis=1).astype(np.float64))
        return codes, exps, vals

    ca, ea, va = make(M)
    cb, eb, vb = make(N)
    A, Bt = bf16_bits(va), bf16_bits(vb)
    assert np.array_equal(bits_to_f64(A), va)            # all values are bf16-exact
    a_codes, a_scales = orc.quantize_mx(A, True)
    assert np.array_equal(unpack_codes(a_codes) & 7, ca & 7)
    nz = (ca & 7) != 0
    assert np.array_equal((unpack_codes(a_codes) >> 3)[nz], (ca >> 3)[nz])
    assert np.array_equal(a_scales.astype(np.int64), ea + 127)
    assert np.array_equal(dequant(a_codes, a_scales, table), va)
    # K-strided storage of B gives the same codes
    b_codes, b_scales = orc.quantize_mx(np.ascontiguousarray(Bt.T), False)
    b_codes2, b_scales2 = orc.quantize_mx(Bt, True)
    assert np.array_equal(b_codes, b_codes2) and np.array_equal(b_scales, b_scales2)
    res = orc.adahop_gemm(A, True, np.ascontiguousarray(Bt.T), False, orc.NONE, 0)
    assert np.allclose(res["C"], va @ vb.T, rtol=1e-13, atol=0)


@pytest.mark.parametrize("b", [32, 64, 128, 256])
def test_fused_closed_form_hadamard_rows(b, golden_dir):
    """A K-block equal to c * (row i of the +-1 Sylvester matrix) transforms to b*c*e_i exactly
    (integer butterflies), i.e. fl(fl(b c) * c_b) at position i and 0 elsewhere: one nonzero nibble
    per transform block, and the E8M0 code from the closed form."""
    table = e2m1_table(golden_dir)
    H = sylvester(b)
    cvals = [1.0, 0.75, 3.0, 0.0078125, 5.0]
    nblk = len(cvals)
    picks = [1, b - 1, b // 2, 3, 17 % b]
    x = np.concatenate([c * H[i] for c, i in zip(cvals, picks)]).astype(np.float32)[None, :]
    codes, scales = orc.iht_quantize(bf16_bits(x), True, b)
    dq = dequant(codes, scales, table)[0]
    cb = np.float32(1.0 / np.sqrt(float(b)))
    for t, (c, i) in enumerate(zip(cvals, picks)):
        blk = dq[t * b:(t + 1) * b]
        peak = float(np.float32(np.float32(b * c) * cb))
        nzpos = np.flatnonzero(blk)
        assert nzpos.tolist() == [i]
        e = int(np.floor(np.log2(peak)))
        s = scales[0, (t * b + i) // 32]
        assert s == e - 2 + 127
        # the value stored is the nearest E2M1 magnitude to peak / 2^(e-2) (6 when that exceeds 6)
        q = peak / 2.0 ** (e - 2)
        mags = np.array([table[c] for c in range(8)])
        d = np.abs(mags - q)
        best = [int(c) for c in np.flatnonzero(d == d.min())]
        pick = best[0] if len(best) == 1 else [c for c in best if c % 2 == 0][0]   # tie -> even code
        assert blk[i] == mags[pick] * 2.0 ** (e - 2)
        other = np.delete(scales[0, t * b // 32:(t + 1) * b // 32], i // 32)
        assert np.all(other == 0)
    assert nblk * b == x.shape[1]


def test_sign_of_zero_rules():
    """Without a transform the sign bit of a zero is the input's; a transformed value that is exactly
    zero is stored as +0: a convention (the paper is silent; H v = 0 has no sign).  Plain IEEE
    butterflies would keep -0 only for an all -0 block, which is the case planted here."""
    x = np.zeros((1, 64), dtype=np.float32)
    x[0, :32] = -0.0
    x[0, 32] = 1.0
    x[0, 33] = -1.0                      # cancels in the first butterfly of the transform
    bits = bf16_bits(x)
    assert bits[0, 0] == 0x8000
    codes, scales = orc.quantize_mx(bits, True)
    assert np.all(codes[0, :16] == 0x88) and scales[0, 0] == 0
    codes_t, _ = orc.iht_quantize(bits, True, 32)
    assert np.all(codes_t[0, :16] == 0)                       # all -0 block -> +0 codes
    t = orc.transform(bits, True, 32)[0]
    assert not np.any(np.signbit(t[t == 0]))


# ----------------------------------------------------------------------------- emulated GEMM

def test_mx_gemm_matches_numpy_on_independent_dequant(golden_dir):
    table = e2m1_table(golden_dir)
    rng = np.random.default_rng(9)
    M, N, K = 20, 12, 96
    a_codes = rng.integers(0, 256, size=(M, K // 2), dtype=np.uint8)
    b_codes = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    a_scales = rng.integers(110, 140, size=(M, K // 32), dtype=np.uint8)
    b_scales = rng.integers(110, 140, size=(N, K // 32), dtype=np.uint8)
    ref = dequant(a_codes, a_scales, table) @ dequant(b_codes, b_scales, table).T
    got = orc.mx_gemm(a_codes, a_scales, b_codes, b_scales)
    assert np.allclose(got, ref, rtol=1e-13, atol=1e-300)
    rows = np.array([3, 19, 0], dtype=np.int32)
    cols = np.array([11, 2], dtype=np.int32)
    assert np.allclose(orc.mx_gemm(a_codes, a_scales, b_codes, b_scales, rows, cols), ref[np.ix_(rows, cols)],
                       rtol=1e-13)


def test_mx_gemm_hand_case():
    """M=N=1, K=32: a = [6, -0.5, 0...] scale 2^1, b = [1.5, 4, 0...] scale 2^-2:
    (6*2)(1.5/4) + (-0.5*2)(4/4) = 4.5 - 1 = 3.5."""
    a = np.zeros((1, 16), dtype=np.uint8)
    b = np.zeros((1, 16), dtype=np.uint8)
    a[0, 0] = 7 | (9 << 4)
    b[0, 0] = 3 | (6 << 4)
    got = orc.mx_gemm(a, np.array([[128]], dtype=np.uint8), b, np.array([[125]], dtype=np.uint8))
    assert got.shape == (1, 1) and got[0, 0] == 3.5


# ----------------------------------------------------------------------------- OE

@pytest.mark.parametrize("kind", ["row", "col", "k"])
@pytest.mark.parametrize("layouts", [(True, True), (True, False), (False, False)])
def test_oe_split_identity_without_quantisation(kind, layouts):
    """A B = A_res B_res' + extracted part, exactly in double (App. E), for all three OE kinds."""
    rng = np.random.default_rng(21)
    M, N, K = 18, 22, 64
    A = bf16_bits(rng.standard_normal((M, K)))
    Bt = bf16_bits(rng.standard_normal((N, K)))
    a_store = A if layouts[0] else np.ascontiguousarray(A.T)
    b_store = Bt if layouts[1] else np.ascontiguousarray(Bt.T)
    exact = bits_to_f64(A) @ bits_to_f64(Bt).T
    assert np.allclose(orc.exact_gemm(a_store, layouts[0], b_store, layouts[1]), exact, rtol=1e-13)
    dim = {"row": M, "col": N, "k": K}[kind]
    sel = np.sort(rng.permutation(dim)[:5]).astype(np.int32)
    mask = np.zeros(dim, dtype=np.uint8)
    mask[sel] = 1
    kw = {"row": dict(a_zero_outer=mask), "col": dict(b_zero_outer=mask), "k": dict(zero_k=mask)}[kind]
    res = orc.bf16_gemm(a_store, layouts[0], b_store, layouts[1], **kw)
    if kind == "row":
        assert np.all(res[sel, :] == 0)
        out = np.zeros_like(res)
        out[sel, :] = orc.bf16_gemm(a_store, layouts[0], b_store, layouts[1], rows=sel)
        assert np.allclose(out[sel], exact[sel], rtol=1e-13)
    elif kind == "col":
        assert np.all(res[:, sel] == 0)
        out = np.zeros_like(res)
        out[:, sel] = orc.bf16_gemm(a_store, layouts[0], b_store, layouts[1], cols=sel)
    else:
        out = orc.bf16_gemm(a_store, layouts[0], b_store, layouts[1], ksel=sel)
        ref_part = bits_to_f64(A)[:, sel] @ bits_to_f64(Bt)[:, sel].T
        assert np.allclose(out, ref_part, rtol=1e-12, atol=1e-12)
    assert np.allclose(res + out, exact, rtol=1e-12, atol=1e-12)


def test_oe_row_residual_rows_have_zero_codes():
    g = inputs.Gemm("t", inputs.Operand(inputs.matrix(64, 128, 1.0, 77, row_outliers=(3, 100.0, 100.0)), True),
                    inputs.Operand(inputs.matrix(48, 128, 0.02, 78), True), orc.IHT_OE_ROW, 32, 3)
    res = orc.adahop_gemm(g.A.bits, True, g.B.bits, True, g.strategy, g.iht_block, g.k)
    S = res["idx"]
    assert len(S) == 3
    assert np.all(res["a_codes"][S] == 0) and np.all(res["a_scales"][S] == 0)
    # with the residual rows zero the MXFP4 part contributes nothing there: C[S] is the bf16 product
    exact = orc.exact_gemm(g.A.bits, True, g.B.bits, True)
    assert np.allclose(res["C"][S], exact[S], rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("b_k_contig", [True, False])
@pytest.mark.parametrize("a_k_contig", [True, False])
def test_oe_col_whole_path_against_numpy_pieces(a_k_contig, b_k_contig, golden_dir):
    """OE-Right (Eq. 8) through adahop_gemm, B in both storage orders: FOID must pick the planted columns of B
    (scored on B, over each column's first 64 K-elements), the residual of B -- and only of B -- loses exactly
    those columns, C[:, S] is the float64 product on the original values and every other column is the product
    of the two dequantised operands, all rebuilt here with numpy and the golden E2M1 table.  A carries amplified
    rows and K-channels of its own, so scoring A, masking A or adding into rows instead of columns would each
    fail one of the assertions."""
    table = e2m1_table(golden_dir)
    M, N, K, k = 40, 56, 128, 5
    A = inputs.matrix(M, K, 1.0, 91, row_outliers=(4, 60.0, 60.0), col_outliers=(3, 40.0, 40.0))
    Bt = inputs.matrix(N, K, 0.02, 92)                       # logical [N, K]: row n is column n of the paper's B
    planted = np.sort(np.random.default_rng(93).permutation(N)[:k]).astype(np.int32)
    bt = bits_to_f64(Bt)
    bt[planted] *= 32.0                                      # power of two: stays exactly representable
    Bt = bf16_bits(bt.astype(np.float32))
    a_store = A if a_k_contig else np.ascontiguousarray(A.T)
    b_store = Bt if b_k_contig else np.ascontiguousarray(Bt.T)
    res = orc.adahop_gemm(a_store, a_k_contig, b_store, b_k_contig, orc.IHT_OE_COL, 32, k)
    S = res["idx"]
    assert S.tolist() == planted.tolist()
    # residual: the extracted columns of B are gone from the MXFP4 operand, nothing is removed from A
    assert np.all(res["b_codes"][S] == 0) and np.all(res["b_scales"][S] == 0)
    rest = np.setdiff1d(np.arange(N), S)
    assert np.all(res["b_scales"][rest] != 0)
    ca, sa = orc.iht_quantize(a_store, a_k_contig, 32)
    assert np.array_equal(ca, res["a_codes"]) and np.array_equal(sa, res["a_scales"])
    Bres = Bt.copy()
    Bres[S] = 0
    cb, sb = orc.iht_quantize(Bres, True, 32)
    assert np.array_equal(cb, res["b_codes"]) and np.array_equal(sb, res["b_scales"])
    # C: extracted columns exact, the others the emulated MXFP4 product
    a64, b64 = bits_to_f64(A), bits_to_f64(Bt)
    assert np.allclose(res["C"][:, S], a64 @ b64[S].T, rtol=1e-12, atol=1e-14)
    emu = dequant(res["a_codes"], res["a_scales"], table) @ dequant(res["b_codes"], res["b_scales"], table).T
    assert np.all(emu[:, S] == 0)
    assert np.allclose(res["C"][:, rest], emu[:, rest], rtol=1e-12, atol=1e-14)
    # the quantised columns really differ from the exact ones (the test would not notice a BF16 product
    # written everywhere otherwise)
    assert np.linalg.norm(res["C"][:, rest] - (a64 @ b64[rest].T)) > 1e-3 * np.linalg.norm(a64 @ b64[rest].T)
    # sampled outputs: rows x cols selections address the same matrix
    rows = np.array([3, 17, 39], dtype=np.int32)
    cols = np.array([int(S[1]), int(rest[0]), int(S[4]), int(rest[7])], dtype=np.int32)
    sub = orc.adahop_gemm(a_store, a_k_contig, b_store, b_k_contig, orc.IHT_OE_COL, 32, k, rows=rows, cols=cols)
    assert np.allclose(sub["C"], res["C"][np.ix_(rows, cols)], rtol=1e-13, atol=1e-300)
    # caller-chosen indices take the place of FOID's
    given = np.array([int(rest[2]), int(S[0])], dtype=np.int32)
    alt = orc.adahop_gemm(a_store, a_k_contig, b_store, b_k_contig, orc.IHT_OE_COL, 32, 2, idx=given)
    assert alt["idx"].tolist() == sorted(given.tolist())
    assert np.all(alt["b_codes"][given] == 0) and np.any(alt["b_codes"][S[1]] != 0)
    assert np.allclose(alt["C"][:, given], a64 @ b64[given].T, rtol=1e-12, atol=1e-14)


def test_oe_row_whole_path_sampled_outputs(golden_dir):
    """OE-Left (Eq. 7) with a rows x cols sample: the sample addresses the same C, extracted rows in it carry the
    float64 product, the others the emulated MXFP4 product (numpy + golden table)."""
    table = e2m1_table(golden_dir)
    A = inputs.matrix(48, 96, 1.0, 95, row_outliers=(4, 100.0, 100.0))
    Bt = inputs.matrix(40, 96, 0.02, 96, row_outliers=(3, 30.0, 30.0))
    b_store = np.ascontiguousarray(Bt.T)
    full = orc.adahop_gemm(A, True, b_store, False, orc.IHT_OE_ROW, 32, 4)
    S = full["idx"]
    rows = np.array([int(S[2]), 0 if 0 not in S else 1, int(S[0]), 47 if 47 not in S else 46], dtype=np.int32)
    cols = np.array([39, 5, 12], dtype=np.int32)
    sub = orc.adahop_gemm(A, True, b_store, False, orc.IHT_OE_ROW, 32, 4, rows=rows, cols=cols)
    assert np.allclose(sub["C"], full["C"][np.ix_(rows, cols)], rtol=1e-13, atol=1e-300)
    a64, b64 = bits_to_f64(A), bits_to_f64(Bt)
    emu = dequant(full["a_codes"], full["a_scales"], table) @ dequant(full["b_codes"], full["b_scales"], table).T
    for r, row in enumerate(rows):
        want = (a64[row] @ b64.T)[cols] if row in S else emu[row, cols]
        assert np.allclose(sub["C"][r], want, rtol=1e-12, atol=1e-14)


def test_whole_path_matches_step_by_step_numpy(golden_dir):
    """adahop_gemm (OE-K, K-strided B) against the same pipeline assembled in the test from numpy
    pieces: Sylvester matrix product for the transform is replaced by the oracle's own codes (pinned
    above), everything downstream -- dequantise, product, outlier part, sum -- is numpy."""
    table = e2m1_table(golden_dir)
    A = inputs.matrix(40, 128, 1.0, 5, col_outliers=(4, 50.0, 50.0))
    Bt = inputs.matrix(24, 128, 0.02, 6)
    b_store = np.ascontiguousarray(Bt.T)
    res = orc.adahop_gemm(A, True, b_store, False, orc.IHT_OE_K, 64, 4)
    S = res["idx"]
    a64, b64 = bits_to_f64(A), bits_to_f64(Bt)
    ref = dequant(res["a_codes"], res["a_scales"], table) @ dequant(res["b_codes"], res["b_scales"], table).T
    ref += a64[:, S] @ b64[:, S].T
    assert np.allclose(res["C"], ref, rtol=1e-12, atol=1e-12)
    # the codes are those of the masked operand
    mask = np.zeros(128, dtype=np.uint8)
    mask[S] = 1
    A_res = A.copy()
    A_res[:, S] = 0
    c2, s2 = orc.iht_quantize(A_res, True, 64)
    assert np.array_equal(c2, res["a_codes"]) and np.array_equal(s2, res["a_scales"])


# ----------------------------------------------------------------------------- FOID

def test_foid_recall_of_planted_outliers_and_double_precision_ranking():
    rng = np.random.default_rng(31)
    rows, cols = 512, 256
    g = np.random.default_rng(1)
    x = g.standard_normal((rows, cols)).astype(np.float32)
    planted = np.sort(rng.permutation(rows)[:9])
    x[planted] *= 20.0                      # variance ratio 400
    bits = bf16_bits(x)
    for kc, store in ((True, bits), (False, np.ascontiguousarray(bits.T))):
        idx, mask = orc.foid_topk(store, kc, 0, 9)
        assert idx.tolist() == planted.tolist()
        assert mask.sum() == 9 and np.all(mask[planted] == 1)
        idx12, _ = orc.foid_topk(store, kc, 0, 12)
        assert set(planted.tolist()) <= set(idx12.tolist()) and np.all(np.diff(idx12) > 0)
        # double-precision variance over the first 64 elements ranks the same way
        scores = orc.foid_scores(store, kc, 0)
        v = bits_to_f64(bits)[:, :64]
        ref = ((v - v.mean(axis=1, keepdims=True)) ** 2).sum(axis=1)
        assert np.allclose(scores, ref, rtol=2e-5)
        order = np.argsort(-ref, kind="stable")
        gap_ok = ref[order[11]] * (1 - 1e-4) > ref[order[12]]
        if gap_ok:
            assert set(order[:12].tolist()) == set(idx12.tolist())
    # axis = 1: score K indices over the first 64 outer elements
    idxk, _ = orc.foid_topk(np.ascontiguousarray(bits.T), True, 1, 9)     # array [outer=cols, K=rows]
    assert idxk.tolist() == planted.tolist()


def test_topk_tie_break_is_lowest_index():
    scores = np.array([1.0, 5.0, 5.0, 0.5, 5.0, 7.0, 1.0], dtype=np.float32)
    idx, mask = orc.topk(scores, 3)
    assert idx.tolist() == [1, 2, 5] and mask.tolist() == [0, 1, 1, 0, 0, 1, 0]
    idx, _ = orc.topk(scores, 5)
    assert idx.tolist() == [0, 1, 2, 4, 5]
    idx, mask = orc.topk(scores, 0)
    assert idx.size == 0 and mask.sum() == 0


def test_foid_uses_only_first_64_samples():
    x = np.zeros((4, 256), dtype=np.float32)
    x[1, 100:] = 1000.0 * np.arange(156)          # huge, but outside the sampled window
    x[2, :64] = np.arange(64)
    s = orc.foid_scores(bf16_bits(x), True, 0)
    assert s[1] == 0.0 and s[2] > 0 and s[0] == 0.0


# ----------------------------------------------------------------------------- qualitative (paper)

def test_iht_helps_column_outlier_activations_config0():
    """Sec. 3.2 / Fig. 2: for a CN pair IHT lowers the product error relative to plain MXFP4."""
    g = inputs.config0()[0]
    exact = orc.exact_gemm(g.A.bits, True, g.B.bits, True)
    e = {}
    for s in (orc.NONE, orc.IHT):
        C = orc.adahop_gemm(g.A.bits, True, g.B.bits, True, s, 32)["C"]
        e[s] = np.mean((C - exact) ** 2)
    assert e[orc.IHT] < e[orc.NONE]


def test_oe_row_error_non_increasing_in_rank():
    """App. G: error falls with the extraction rank and flattens once the planted rows are out."""
    A = inputs.matrix(256, 256, 1.0, 41, row_outliers=(6, 100.0, 100.0))
    Bt = inputs.matrix(128, 256, 0.02, 42)
    exact = orc.exact_gemm(A, True, Bt, True)
    errs = []
    for k in (0, 2, 6, 12):
        C = orc.adahop_gemm(A, True, Bt, True, orc.IHT_OE_ROW, 32, k)["C"]
        errs.append(np.linalg.norm(C - exact))
    assert errs[0] > errs[1] > errs[2] >= errs[3] * 0.999
    assert errs[2] < 0.2 * errs[0]


# ----------------------------------------------------------------------------- pattern detection (App. A)

def _paper_letters_to_patterns(pair):
    """Paper letters (A is m x k, B is k x n) -> operand-sense patterns: for A, R = outer-wise and C = K-wise;
    for B (passed as [n, k]), C = outer-wise and R = K-wise."""
    a = {"R": orc.PATTERN_OUTER, "C": orc.PATTERN_K, "N": orc.PATTERN_NONE}[pair[0]]
    b = {"C": orc.PATTERN_OUTER, "R": orc.PATTERN_K, "N": orc.PATTERN_NONE}[pair[1]]
    return a, b


def test_strategy_table_matches_the_papers_section():
    names = {"IHT": (orc.IHT, False), "OE-LEFT": (orc.IHT_OE_ROW, False), "OE-RIGHT": (orc.IHT_OE_COL, False),
             "BF16": (orc.NONE, True)}
    rows = load_table(os.path.join(os.path.dirname(__file__), "golden", "strategy_table.txt"))
    assert len(rows) == 13
    for pair, level, want in rows:
        a, b = _paper_letters_to_patterns(pair)
        assert orc.select_strategy(a, b, int(level)) == names[want], (pair, level)


def test_calibration_vote_is_the_majority_with_ties_to_none():
    """Hand cases for the 30-step vote of Sec. 4.1."""
    N, O, K = orc.PATTERN_NONE, orc.PATTERN_OUTER, orc.PATTERN_K
    assert orc.vote_pattern([K] * 30) == K
    assert orc.vote_pattern([K] * 16 + [N] * 14) == K
    assert orc.vote_pattern([O] * 11 + [K] * 10 + [N] * 9) == O          # a plurality is enough
    assert orc.vote_pattern([O] * 15 + [K] * 15) == N                    # nothing dominates
    assert orc.vote_pattern([O] * 10 + [K] * 10 + [N] * 10) == N
    assert orc.vote_pattern([N] * 15 + [K] * 15) == N
    assert orc.vote_pattern([O]) == O


def test_pattern_closed_form_rank_one():
    """T[i, j] = a_i * s_j with s = +-1 alternating: every row has mean 0 and variance a_i^2 exactly, every
    column has the same variance var(a) -> CV of the column variances is 0 and CV_row = std(a^2) / mean(a^2).
    a = (1, 2, 1, 2, ...): a^2 in {1, 4}: mean 2.5, std 1.5 -> CV_row = 0.6 (up to the 1e-12 in the denominator)."""
    m, n = 64, 128
    a = np.where(np.arange(m) % 2 == 0, 1.0, 2.0)
    s = np.where(np.arange(n) % 2 == 0, 1.0, -1.0)
    T = bf16_bits(np.outer(a, s))
    p, st = orc.detect_pattern(T, True)
    assert abs(st[0] - 0.6) < 1e-9 and st[1] < 1e-12
    assert abs(st[2] - 0.6 / np.sqrt(2.0 / (n - 1))) < 1e-8
    assert p == orc.PATTERN_OUTER                       # a ratio with a zero denominator counts as infinite
    # the same matrix stored transposed is the same logical operand
    p2, st2 = orc.detect_pattern(np.ascontiguousarray(T.T), False)
    assert p2 == p and np.allclose(st2, st, rtol=1e-12, atol=1e-15)
    # and read as an [outer = n, K = m] operand the roles swap
    p3, st3 = orc.detect_pattern(np.ascontiguousarray(T.T), True)
    assert p3 == orc.PATTERN_K and abs(st3[1] - 0.6) < 1e-9


def test_pattern_iid_gives_unit_normalised_cv_and_planted_outliers_are_found():
    """App. A: for IID data both normalised CVs are about 1 (whatever the aspect ratio), hence class None;
    amplified rows give Row-wise, amplified columns Column-wise."""
    for rows, cols in ((512, 2048), (2048, 256)):
        p, st = orc.detect_pattern(inputs.matrix(rows, cols, 1.0, 77), True)
        assert p == orc.PATTERN_NONE and 0.8 < st[2] < 1.25 and 0.8 < st[3] < 1.25, st
    p, _ = orc.detect_pattern(inputs.matrix(512, 1024, 1.0, 78, row_outliers=(5, 100.0, 100.0)), True)
    assert p == orc.PATTERN_OUTER
    p, _ = orc.detect_pattern(inputs.matrix(512, 1024, 1.0, 79, col_outliers=(8, 50.0, 50.0)), True)
    assert p == orc.PATTERN_K


# ----------------------------------------------------------------------------- bf16 rounding of C

def test_round_to_bf16_matches_the_library_conversion_on_fp32_values():
    """Pin: for values that already are fp32 numbers a single rounding to bf16 is what torch's CPU conversion
    does (an independent library routine); covers normals, bf16-subnormals, both signs, overflow."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(123)
    x = (rng.standard_normal(400000) * np.exp(rng.uniform(-88.0, 88.0, 400000))).astype(np.float32)
    x = np.concatenate([x, np.float32([0.0, -0.0, 3.4e38, -3.4e38, 1e-40, -1e-40, 2.0 ** -133, 2.0 ** -134])])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(orc.round_to_bf16(x.astype(np.float64)), want)
    assert np.array_equal(orc.bf16_to_double(want[np.isfinite(x)]),
                          torch.from_numpy(want[np.isfinite(x)].view(np.int16)).view(torch.bfloat16).double().numpy())


def test_round_to_bf16_ties_and_single_rounding():
    """Pin from the format's definition: the midpoint of two neighbouring bf16 numbers goes to the one with the
    even significand, for every positive finite pair; a double just above a midpoint goes up although an fp32
    intermediate would land on the midpoint and go down."""
    b = np.arange(0, 0x7f7f, dtype=np.uint32)
    lo = (b << 16).view(np.float32).astype(np.float64)
    hi = ((b + 1) << 16).view(np.float32).astype(np.float64)
    want = np.where(b % 2 == 0, b, b + 1).astype(np.uint16)
    assert np.array_equal(orc.round_to_bf16((lo + hi) / 2), want)
    assert np.array_equal(orc.round_to_bf16(-(lo + hi) / 2), want | 0x8000)
    assert orc.round_to_bf16(np.array([1 + 2.0 ** -8]))[0] == 0x3f80
    assert orc.round_to_bf16(np.array([1 + 2.0 ** -8 + 2.0 ** -40]))[0] == 0x3f81
    assert orc.round_to_bf16(np.array([1 + 3 * 2.0 ** -8]))[0] == 0x3f82


# ----------------------------------------------------------------------------- Outer Hadamard Transform (Eq. 6)

@pytest.mark.parametrize("b", [32, 64, 128])
def test_oht_hadamard_matrix_is_the_library_sylvester_matrix(b):
    """Pin: scipy's Hadamard construction (a library routine) and exact orthogonality in integers."""
    import scipy.linalg
    H = orc.hadamard_matrix(b)
    assert np.array_equal(np.rint(H * np.sqrt(b)).astype(np.int64), scipy.linalg.hadamard(b))
    assert np.array_equal(sylvester(b) @ sylvester(b).T, b * np.eye(b, dtype=np.int64))
    assert np.allclose(H @ H.T, np.eye(b), atol=1e-14)


@pytest.mark.parametrize("b", [32, 64, 128])
def test_oht_transform_is_left_multiplication_by_block_hadamard(b):
    """H_m A mixes along the OUTER index (Lemma on mixing directions): compare with the explicit double
    product (I kron H_b) X built from scipy's matrix, and check that the storage order does not matter."""
    import scipy.linalg
    rng = np.random.default_rng(b)
    x = rng.standard_normal((2 * b, 96)).astype(np.float32)
    bits = bf16_bits(x)
    got = orc.oht_transform(bits, True, b)
    Hb = scipy.linalg.hadamard(b) / np.sqrt(b)
    want = np.kron(np.eye(2), Hb) @ bits_to_f64(bits)
    assert np.abs(got - want).max() <= 4e-7 * np.log2(b) * np.abs(want).max()
    assert np.array_equal(orc.oht_transform(np.ascontiguousarray(bits.T), False, b), got)
    # not the inner transform: a matrix that is constant along K and varies along outer must change
    ramp = bf16_bits(np.repeat(np.arange(2 * b, dtype=np.float32)[:, None], 32, axis=1))
    assert not np.array_equal(orc.oht_transform(ramp, True, b), bits_to_f64(ramp).astype(np.float32))
    assert np.array_equal(orc.transform(ramp, True, 32)[:, 1:], np.zeros((2 * b, 31), np.float32))


def test_oht_spreads_one_outlier_row_over_its_block_exactly():
    """Closed form for b = 64 (normalisation 1/8, exact): A zero except row r = u  =>  every row o of r's block
    becomes H[o, r] u / 8, rows of other blocks stay zero."""
    b, r = 64, 70
    u = bits_to_f64(bf16_bits(np.random.default_rng(1).standard_normal(64).astype(np.float32) * 40))
    x = np.zeros((3 * b, 64), dtype=np.float32)
    x[r] = u
    got = orc.oht_transform(bf16_bits(x), True, b).astype(np.float64)
    H = sylvester(b)
    want = np.zeros_like(got)
    want[b:2 * b] = H[:, r - b][:, None] * u[None, :] / 8.0
    assert np.array_equal(got, want)


def test_oht_identity_without_quantisation():
    """Eq. 6 with Q = identity: H_m^T (H_m A)(B H_n) H_n^T = A B (fp32 butterflies on the operand side)."""
    rng = np.random.default_rng(7)
    a = bf16_bits(rng.standard_normal((128, 160)).astype(np.float32))
    bt = bf16_bits((rng.standard_normal((64, 160)) * 0.02).astype(np.float32))
    for b in (32, 64):
        Ta = orc.oht_transform(a, True, b).astype(np.float64)
        Tb = orc.oht_transform(np.ascontiguousarray(bt.T), False, b).astype(np.float64)
        C = orc.oht_inverse(Ta @ Tb.T, b, b)
        exact = bits_to_f64(a) @ bits_to_f64(bt).T
        assert np.linalg.norm(C - exact) <= 1e-5 * np.linalg.norm(exact)
    # the inverse is a two-sided rotation: one side alone does not restore the product
    one_sided = np.kron(np.eye(128 // 64), orc.hadamard_matrix(64)).T @ (Ta @ Tb.T)
    assert np.linalg.norm(one_sided - exact) > 0.1 * np.linalg.norm(exact)


def test_oht_inverse_against_direct_sums():
    """Brute force on a tiny case: C[i, j] = sum_p sum_q H[p, i] Cq[p, q] H[q, j] within each block pair."""
    rng = np.random.default_rng(9)
    Cq = rng.standard_normal((64, 32))
    H = sylvester(32) / np.sqrt(32.0)
    want = np.zeros_like(Cq)
    for bi in range(2):
        blk = Cq[32 * bi:32 * bi + 32]
        for i in range(32):
            for j in range(32):
                want[32 * bi + i, j] = sum(H[p, i] * blk[p, q] * H[q, j] for p in range(32) for q in range(32))
    assert np.allclose(orc.oht_inverse(Cq, 32, 32), want, atol=1e-12)


def test_oht_quantize_closed_form_and_whole_strategy(golden_dir):
    """Columns of a 64-row block equal to c * (column i of the +-1 Sylvester matrix) transform to 8 c at row i and
    0 elsewhere (b = 64: integer butterflies, exact normalisation), so the packed operand is known in closed form:
    row i of the block holds 8 c along K, every other row is all-zero codes with scale code 0.  Then the whole
    strategy on such operands is exact: C_OHT = A B."""
    table = e2m1_table(golden_dir)
    b, K = 64, 64
    H = sylvester(b)
    cs = np.array([0.5, 0.25, 0.125, 0.0625] * (K // 4))           # 8c in {4, 2, 1, 0.5}: E2M1 values, amax 4
    hot = [5, 40]                                                  # hot row of block 0 / block 1
    x = np.zeros((2 * b, K), dtype=np.float32)
    for blk, i in enumerate(hot):
        x[blk * b:(blk + 1) * b] = H[:, i][:, None] * cs[None, :]
    bits = bf16_bits(x)
    codes, scales = orc.oht_quantize(bits, True, b)
    dq = dequant(codes, scales, table)
    want = np.zeros((2 * b, K))
    for blk, i in enumerate(hot):
        want[blk * b + i] = 8.0 * cs
    assert np.array_equal(dq, want)
    hot_rows = [blk * b + i for blk, i in enumerate(hot)]
    assert np.all(scales[hot_rows] == 127) and np.all(np.delete(scales, hot_rows, axis=0) == 0)
    assert np.all(np.delete(codes, hot_rows, axis=0) == 0)
    # whole strategy: both operands of this kind -> every quantisation is exact -> Eq. 6 returns A B
    out = orc.oht_gemm(bits, True, bits[:b], True, b)
    exact = bits_to_f64(bits) @ bits_to_f64(bits[:b]).T
    assert np.allclose(out["C"], exact, rtol=0, atol=1e-12 * np.abs(exact).max())


# ----------------------------------------------------------------------------- stochastic rounding (optional)

def test_philox_known_answers(golden_dir):
    rows = load_table(os.path.join(golden_dir, "philox4x32_10_kat.txt"))
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        assert orc.philox4x32_10(w[0:4], w[4:6]) == w[6:10]


def test_sr_bits_layout_and_uniformity():
    """Element (o, kk) takes half j = kk % 8 of the block with counter (o, kk / 8, 0, 0), key = the seed's halves;
    the 16-bit draws are uniform (mean, 16-bucket chi-square) and differ between seeds, rows and K indices."""
    seed = 0x0123456789abcdef
    for o, kk in ((0, 0), (5, 17), (1000, 8191), (3, 8)):
        w = orc.philox4x32_10([o, kk // 8, 0, 0], [seed & 0xffffffff, seed >> 32])
        j = kk % 8
        assert orc.sr_bits(seed, o, kk) == (w[j // 2] >> (16 * (j % 2))) & 0xffff
    draws = np.array([orc.sr_bits(7, o, kk) for o in range(40) for kk in range(512)])
    assert abs(draws.mean() - 32767.5) < 4 * 65536 / np.sqrt(12 * draws.size)
    counts = np.bincount(draws >> 12, minlength=16)
    chi2 = ((counts - draws.size / 16) ** 2 / (draws.size / 16)).sum()
    assert chi2 < 45.0                                   # 15 degrees of freedom: P(chi2 > 45) < 1e-4
    other = np.array([orc.sr_bits(8, o, kk) for o in range(40) for kk in range(512)])
    assert np.mean(draws == other) < 0.001
    assert len({orc.sr_bits(7, 0, kk) for kk in range(64)}) > 60


def test_sr_encoder_probability_is_the_distance_fraction(golden_dir):
    """Brute force over all 65536 draws: the number of draws that round q up equals ceil(frac * 65536) with frac
    the position of |q| between its E2M1 neighbours; representable values never move; |q| >= 6 saturates;
    the result is always one of the two neighbours and keeps the sign."""
    table = e2m1_table(golden_dir)
    grid = [table[c] for c in range(8)]
    all_draws = np.arange(65536)
    for q in (0.1, 0.25, 0.49, 0.5, 0.7, 1.3, 1.75, 2.0, 2.2, 3.9, 4.5, 5.999, 1e-6, 2.0 ** -20):
        for sign in (1.0, -1.0):
            lo = max(i for i in range(8) if grid[i] <= q)
            frac = (np.float32(q) - np.float32(grid[lo])) / np.float32(grid[lo + 1] - grid[lo])
            codes = np.array([orc.e2m1_encode_sr(sign * q, int(r)) for r in all_draws[::1 if q in (0.7, 4.5) else 97]])
            mags = codes & 7
            assert set(mags.tolist()) <= {lo, lo + 1}
            assert np.all((codes >> 3) == (0 if sign > 0 else 1))
            if q in (0.7, 4.5):
                assert int(np.sum(mags == lo + 1)) == int(np.ceil(float(frac) * 65536))
            if frac == 0:
                assert np.all(mags == lo)
    for q in (6.0, 6.5, 7.99, 1e9):
        assert orc.e2m1_encode_sr(q, 0) == 7 and orc.e2m1_encode_sr(-q, 65535) == 15


def test_sr_quantiser_is_unbiased_where_round_to_nearest_is_not(golden_dir):
    """Mean over seeds of the dequantised SR result converges to the transformed value (no saturation in this
    input); round-to-nearest keeps a systematic offset on the same data.  Scales do not depend on the rounding."""
    table = e2m1_table(golden_dir)
    x = np.full((4, 64), 2.6, dtype=np.float32)
    x[:, 0] = 4.0                                        # block amax 4 -> scale 1: 2.6 sits between 2 and 3
    x[:, 32] = 4.0
    bits = bf16_bits(x)
    truth = bits_to_f64(bits)
    rne_codes, rne_scales = orc.iht_quantize(bits, True, 0)
    rne = dequant(rne_codes, rne_scales, table)
    acc = np.zeros_like(truth)
    n = 400
    for seed in range(n):
        c, s = orc.iht_quantize(bits, True, 0, sr_seed=seed)
        assert np.array_equal(s, rne_scales)
        d = dequant(c, s, table)
        assert np.all((d == 2.0) | (d == 3.0) | (d == 4.0))
        acc += d
    mean = acc / n
    # per element the estimator has variance p(1-p) <= 1/4; averaged over 4*62 elements and n seeds
    assert abs((mean - truth)[truth < 4].mean()) < 4 * 0.5 / np.sqrt(n * 4 * 62)
    assert abs((rne - truth)[truth < 4].mean()) > 0.3    # nearest: every 2.6 (bf16: 2.59375) becomes 3


def test_sr_product_converges_to_the_unquantised_transformed_product():
    """E[Q_sr(A H) Q_sr(H^T B)] = (A H)(H^T B) = A B when nothing saturates: the error of the seed-averaged
    product falls like 1 / sqrt(n), well below the single-draw and the round-to-nearest errors."""
    rng = np.random.default_rng(3)
    a = bf16_bits(rng.uniform(-1, 1, (48, 128)).astype(np.float32))
    b = bf16_bits(rng.uniform(-1, 1, (40, 128)).astype(np.float32))
    exact = orc.exact_gemm(a, True, b, True)
    err = lambda c: np.linalg.norm(c - exact) / np.linalg.norm(exact)
    single = orc.adahop_gemm(a, True, b, True, orc.IHT, 32, sr_seed_a=1, sr_seed_b=2)["C"]
    acc = np.zeros_like(exact)
    n = 64
    for i in range(n):
        acc += orc.adahop_gemm(a, True, b, True, orc.IHT, 32, sr_seed_a=2 * i + 1, sr_seed_b=2 * i + 2)["C"]
    e1, en = err(single), err(acc / n)
    assert en < 2.0 * e1 / np.sqrt(n) + 0.02 * e1        # saturation in (6, 8) X blocks leaves a small floor
    assert en < 0.5 * err(orc.adahop_gemm(a, True, b, True, orc.IHT, 32)["C"])
