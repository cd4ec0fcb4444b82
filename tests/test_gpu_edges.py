"""Edge cases of the GPU path against the oracle (run with -m gpu): smallest shapes, everything extracted,
all-zero and extreme-magnitude operands, and operands at the documented size limits."""
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


def host(t):
    return t.cpu().numpy()


def bf16(x):
    return torch.from_numpy(np.asarray(x, dtype=np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def stored(logical, k_contig):
    """Device operand for logical [outer, K] bits; a K-strided array narrower than 8 is padded to ld = 8."""
    a = logical if k_contig else np.ascontiguousarray(logical.T)
    pad = (-a.shape[1]) % 8
    if pad:
        wide = np.zeros((a.shape[0], a.shape[1] + pad), dtype=np.uint16)
        wide[:, :a.shape[1]] = a
        return torch.from_numpy(wide.view(np.int16)).cuda()[:, :a.shape[1]], a
    return torch.from_numpy(a.view(np.int16)).cuda(), a


def whole(ah, A_log, B_log, a_kc, b_kc, strategy, b, k):
    ta, sa = stored(A_log, a_kc)
    tb, sb = stored(B_log, b_kc)
    out = ah.adahop_gemm(ah.Operand(ta, a_kc), ah.Operand(tb, b_kc), strategy, b, k)
    torch.cuda.synchronize()
    ref = orc.adahop_gemm(sa, a_kc, sb, b_kc, strategy, b, k)
    for name in ("a_scales", "b_scales", "a_codes", "b_codes"):
        assert np.array_equal(host(out[name]), ref[name]), name
    if k:
        assert np.array_equal(np.sort(host(out["idx"])), ref["idx"])
    got = host(out["C"]).astype(np.float64)
    den = max(np.linalg.norm(ref["C"]), 1e-300)
    assert np.linalg.norm(got - ref["C"]) / den < 1e-3 or np.array_equal(got, ref["C"])
    return got, ref


@pytest.mark.parametrize("layouts", [(True, True), (True, False), (False, False)])
def test_smallest_shapes(ah, layouts):
    rng = np.random.default_rng(1)
    for M, N, K, b in ((1, 1, 32, 32), (1, 9, 64, 32), (7, 1, 32, 0), (3, 5, 256, 256)):
        A = bf16(rng.standard_normal((M, K)))
        B = bf16(rng.standard_normal((N, K)) * 0.02)
        for strategy in ((inputs.NONE, inputs.IHT) if b else (inputs.NONE,)):
            say("smallest", (M, N, K), layouts, inputs.STRATEGY_NAMES[strategy])
            whole(ah, A, B, layouts[0], layouts[1], strategy, b, 0)


@pytest.mark.parametrize("layouts", [(True, True), (True, False), (False, True), (False, False)])
def test_smallest_shapes_with_extraction(ah, layouts):
    """One extracted row / column / K-channel (and all but one of them) on operands far smaller than any tile of the
    BF16 product kernels: a single workgroup whose loads past the last row repeat that row, a K of half a pipeline
    stage, a long side of one row."""
    rng = np.random.default_rng(4)
    for M, N, K in ((1, 1, 32), (1, 9, 64), (7, 1, 32), (3, 5, 256), (9, 17, 96), (260, 3, 160)):
        A = bf16(rng.standard_normal((M, K)) * np.where(rng.random((M, 1)) < 0.3, 50.0, 1.0))
        B = bf16(rng.standard_normal((N, K)) * 0.02)
        for strategy, dim in ((inputs.IHT_OE_ROW, M), (inputs.IHT_OE_COL, N), (inputs.IHT_OE_K, K)):
            for k in sorted({1, max(dim - 1, 1)}):
                say("smallest with extraction", (M, N, K), layouts, inputs.STRATEGY_NAMES[strategy], k)
                whole(ah, A, B, layouts[0], layouts[1], strategy, 32, k)


@pytest.mark.parametrize("layouts", [(True, True), (False, False)])
def test_everything_extracted_is_the_bf16_product(ah, layouts):
    """k equal to the whole extracted dimension: the residual is all zero (codes 0, scales 0) and C is the BF16 product
    of the original operands -- bf16 x bf16 with fp32 accumulation, compared with the exact product."""
    rng = np.random.default_rng(2)
    M, N, K = 40, 24, 96
    A = bf16(rng.standard_normal((M, K)))
    B = bf16(rng.standard_normal((N, K)))
    exact = orc.exact_gemm(A if layouts[0] else np.ascontiguousarray(A.T), layouts[0],
                           B if layouts[1] else np.ascontiguousarray(B.T), layouts[1])
    for strategy, k in ((inputs.IHT_OE_ROW, M), (inputs.IHT_OE_COL, N), (inputs.IHT_OE_K, K)):
        say("all extracted", inputs.STRATEGY_NAMES[strategy], layouts)
        got, ref = whole(ah, A, B, layouts[0], layouts[1], strategy, 32, k)
        masked = {inputs.IHT_OE_ROW: ("a",), inputs.IHT_OE_COL: ("b",), inputs.IHT_OE_K: ("a", "b")}[strategy]
        for side in masked:
            assert not ref[side + "_codes"].any() and not ref[side + "_scales"].any()
        assert np.linalg.norm(got - exact) / np.linalg.norm(exact) < 1e-5


def test_all_zero_and_signed_zero_operands(ah):
    M, N, K = 33, 17, 128
    Z = np.zeros((M, K), dtype=np.uint16)
    NZ = np.full((M, K), 0x8000, dtype=np.uint16)                        # -0.0 everywhere
    B = bf16(np.random.default_rng(3).standard_normal((N, K)))
    for name, A in (("zeros", Z), ("negative zeros", NZ)):
        for strategy, k in ((inputs.NONE, 0), (inputs.IHT, 0), (inputs.IHT_OE_ROW, 3), (inputs.IHT_OE_K, 5)):
            say(name, inputs.STRATEGY_NAMES[strategy])
            got, ref = whole(ah, A, B, True, True, strategy, 64, k)
            assert not got.any() and not ref["a_scales"].any()


@pytest.mark.parametrize("k_contig", [True, False])
@pytest.mark.parametrize("b", [0, 32, 256])
def test_extreme_magnitudes_quantise_bit_exact(ah, b, k_contig):
    """Blocks whose amax spans the whole bf16 range, from subnormals to the largest finite value: scale codes from 0
    to 252 (and the transform's sums stay finite: each 32-block holds one large value among tiny ones)."""
    rng = np.random.default_rng(4)
    outer, K = 96, 512
    x = rng.standard_normal((outer, K)).astype(np.float32) * 1e-3
    expo = rng.integers(-126, 120, size=(outer, K // 32))
    x[:, ::32] = np.ldexp(rng.uniform(1.0, 1.99, (outer, K // 32)).astype(np.float32), expo) * rng.choice([-1, 1], (outer, K // 32))
    x[0, :32] = np.float32(2.0 ** -133)                                  # a block of bf16 subnormals
    x[1, 0] = np.float32(3.38e38) if b == 0 else np.float32(1e30)        # near the largest finite bf16
    bits = bf16(x)
    t, s = stored(bits, k_contig)
    say("extreme magnitudes", b, k_contig)
    codes, scales = ah.adahop_iht_quantize(ah.Operand(t, k_contig), b)
    torch.cuda.synchronize()
    rc, rs = orc.iht_quantize(s, k_contig, b)
    assert np.array_equal(host(scales), rs) and np.array_equal(host(codes), rc)
    if b == 0:                                                            # (a transform spreads the large values over its block)
        assert rs.min() == 0 and rs.max() >= 240


def test_operands_at_the_size_limits(ah):
    """outer = 2^21 (the documented maximum) with the shortest K, and a long-K operand: every byte against the oracle;
    FOID over 2^21 indices."""
    rng = np.random.default_rng(5)
    outer = 1 << 21
    x = torch.randn((outer, 32), generator=torch.Generator().manual_seed(11)).to(torch.bfloat16)
    x[rng.integers(0, outer, 50)] *= 30.0
    bits = x.view(torch.int16).numpy().view(np.uint16)
    for kc, arr in ((True, bits), (False, np.ascontiguousarray(bits.T))):
        say("outer = 2^21", "K-contiguous" if kc else "K-strided")
        op = ah.Operand(torch.from_numpy(arr.view(np.int16)).cuda(), kc)
        codes, scales = ah.adahop_iht_quantize(op, 32)
        torch.cuda.synchronize()
        rc, rs = orc.iht_quantize(arr, kc, 32)
        assert np.array_equal(host(scales), rs) and np.array_equal(host(codes), rc)
        del codes, scales
        idx, mask, _ = ah.adahop_foid_topk(op, 0, 1000)
        torch.cuda.synchronize()
        ri, rm = orc.foid_topk(arr, kc, 0, 1000)
        assert np.array_equal(host(idx), ri) and np.array_equal(host(mask), rm)
        del op
    torch.cuda.empty_cache()
    K = 1 << 21
    y = torch.randn((24, K), generator=torch.Generator().manual_seed(12)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    for kc, arr in ((True, y), (False, np.ascontiguousarray(y.T))):
        say("K = 2^21", "K-contiguous" if kc else "K-strided")
        op = ah.Operand(torch.from_numpy(arr.view(np.int16)).cuda(), kc)
        codes, scales = ah.adahop_iht_quantize(op, 256)
        torch.cuda.synchronize()
        rc, rs = orc.iht_quantize(arr, kc, 256)
        assert np.array_equal(host(scales), rs) and np.array_equal(host(codes), rc)
        idx, mask, _ = ah.adahop_foid_topk(op, 1, 4096)                 # K-channels, scored over the first 24 rows
        torch.cuda.synchronize()
        ri, rm = orc.foid_topk(arr, kc, 1, 4096)
        assert np.array_equal(host(idx), ri) and np.array_equal(host(mask), rm)
    torch.cuda.empty_cache()
