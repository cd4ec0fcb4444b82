"""GPU parity of the stochastic-rounding option of the quantisers (run with -m gpu).

Both sides implement the same counter-based generator (Philox4x32-10 keyed by the seed, counted by the
element's position), so the bar is the usual one: codes and scales bit for bit, whatever the layout, the
transform block, the masks or the kernel the launcher picks (K % 256 == 0 takes the 16-wide kernels, other K
the general ones); the product within 1e-3 relative Frobenius of the oracle's.
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


def host(t):
    return t.cpu().numpy()


@pytest.mark.parametrize("k_contig", [True, False])
@pytest.mark.parametrize("b,outer,K", [(0, 70, 96), (32, 130, 160), (64, 67, 448), (128, 200, 512), (256, 131, 1024),
                                       (32, 300, 2048), (0, 9, 256)])
def test_sr_quantiser_bit_exact(ah, b, outer, K, k_contig):
    logical = inputs.matrix(outer, K, 1.0, 700 + b, row_outliers=(3, 60.0, 60.0), col_outliers=(4, 30.0, 30.0))
    stored = logical if k_contig else np.ascontiguousarray(logical.T)
    if stored.shape[1] % 8:
        wide = np.zeros((stored.shape[0], (stored.shape[1] + 7) // 8 * 8), dtype=np.uint16)
        wide[:, :stored.shape[1]] = stored
        t = torch.from_numpy(wide.view(np.int16)).cuda()[:, :stored.shape[1]]
    else:
        t = torch.from_numpy(stored.view(np.int16)).cuda()
    x = ah.Operand(t, k_contig)
    rng = np.random.default_rng(b + outer)
    zo = (rng.random(outer) < 0.05).astype(np.uint8)
    zk = (rng.random(K) < 0.05).astype(np.uint8)
    for seed, masks in ((1, False), (0xfedcba9876543210, True)):
        say("SR quantiser", b, outer, K, "K-contiguous" if k_contig else "K-strided", hex(seed), "masks" if masks else "")
        d_zo = torch.from_numpy(zo).cuda() if masks else None
        d_zk = torch.from_numpy(zk).cuda() if masks else None
        codes, scales = ah.adahop_iht_quantize(x, b, d_zo, d_zk, sr_seed=seed)
        torch.cuda.synchronize()
        rc, rs = orc.iht_quantize(stored, k_contig, b, zo if masks else None, zk if masks else None, sr_seed=seed)
        assert np.array_equal(host(scales), rs)
        assert np.array_equal(host(codes), rc)
    # a different seed changes codes but not scales; no seed is the deterministic quantiser
    c2, s2 = ah.adahop_iht_quantize(x, b, sr_seed=2)
    c0, s0 = ah.adahop_iht_quantize(x, b)
    c1, s1 = ah.adahop_iht_quantize(x, b, sr_seed=1)
    torch.cuda.synchronize()
    assert torch.equal(s2, s0) and torch.equal(s1, s0) and not torch.equal(c1, c2)
    r0, _ = orc.iht_quantize(stored, k_contig, b)
    assert np.array_equal(host(c0), r0)


@pytest.mark.parametrize("strategy,k", [(inputs.IHT, 0), (inputs.IHT_OE_ROW, 5), (inputs.IHT_OE_K, 9)])
def test_whole_path_with_stochastically_rounded_gradient_operand(ah, strategy, k):
    """dgrad-like product: the gradient (A) rounded stochastically, the weight (B, K-strided) to nearest."""
    T, d_out, d_in = 328, 512, 264
    G = inputs.Operand(inputs.matrix(T, d_out, 1e-3, 710, row_outliers=(4, 100.0, 100.0)), True)
    W = inputs.Operand(inputs.matrix(d_out, d_in, 0.02, 711), False)
    say("whole path, SR on A", inputs.STRATEGY_NAMES[strategy])
    dG, dW = ah.Operand.from_bits(G.bits, True), ah.Operand.from_bits(W.bits, False)
    out = ah.adahop_gemm(dG, dW, strategy, 128, k, sr_seed_a=77)
    torch.cuda.synchronize()
    ref = orc.adahop_gemm(G.bits, True, W.bits, False, strategy, 128, k, sr_seed_a=77)
    for name in ("a_scales", "b_scales", "a_codes", "b_codes"):
        assert np.array_equal(host(out[name]), ref[name]), name
    if k:
        assert np.array_equal(np.sort(host(out["idx"])), ref["idx"])
    err = np.linalg.norm(host(out["C"]).astype(np.float64) - ref["C"]) / np.linalg.norm(ref["C"])
    say(f"  vs oracle {err:.2e}")
    assert err < 1e-3
    det = ah.adahop_gemm(dG, dW, strategy, 128, k)
    torch.cuda.synchronize()
    assert torch.equal(det["b_codes"], out["b_codes"]) and not torch.equal(det["a_codes"], out["a_codes"])


def test_stochastic_rounding_in_the_quantiser_that_copies_k_channels(ah):
    """OE-K on K-contiguous operands with K a whole number of 4096-element passes takes the quantiser that also
    copies the extracted channels out; its stochastic-rounding instance must draw as every other quantiser does."""
    M, N, K, k, b = 136, 72, 4096, 37, 128
    A = inputs.Operand(inputs.matrix(M, K, 1.0, 720, col_outliers=(12, 40.0, 80.0)), True)
    B = inputs.Operand(inputs.matrix(N, K, 0.02, 721), True)
    say("whole path, SR on both operands, channels copied by the quantiser")
    dA, dB = ah.Operand.from_bits(A.bits, True), ah.Operand.from_bits(B.bits, True)
    out = ah.adahop_gemm(dA, dB, inputs.IHT_OE_K, b, k, sr_seed_a=5, sr_seed_b=6)
    torch.cuda.synchronize()
    ref = orc.adahop_gemm(A.bits, True, B.bits, True, inputs.IHT_OE_K, b, k, sr_seed_a=5, sr_seed_b=6)
    for name in ("a_scales", "b_scales", "a_codes", "b_codes"):
        assert np.array_equal(host(out[name]), ref[name]), name
    assert np.array_equal(np.sort(host(out["idx"])), ref["idx"])
    err = np.linalg.norm(host(out["C"]).astype(np.float64) - ref["C"]) / np.linalg.norm(ref["C"])
    say(f"  vs oracle {err:.2e}")
    assert err < 1e-3

