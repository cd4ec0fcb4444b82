"""GPU parity of the Outer Hadamard Transform strategy (paper Eq. 6) against the oracle (run with -m gpu).

Bars: packed codes and scales of H_m A / H_n B^T bit-exact; the rotations of C after the product and the whole
strategy within 1e-3 relative Frobenius of the oracle's double-precision result (observed ~1e-7: the GPU does
the rotations with fp32 butterflies).
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


def rel_fro(got, ref):
    return float(np.linalg.norm(got.astype(np.float64) - ref) / max(np.linalg.norm(ref), 1e-300))


def padded(bits, pad):
    """The stored array with `pad` extra elements per row (ld > width), as a device tensor view."""
    wide = np.zeros((bits.shape[0], bits.shape[1] + pad), dtype=np.uint16)
    wide[:, :bits.shape[1]] = bits
    return torch.from_numpy(wide.view(np.int16)).cuda()[:, :bits.shape[1]]


@pytest.mark.parametrize("k_contig", [True, False])
@pytest.mark.parametrize("b,outer,K", [(32, 96, 160), (64, 192, 416), (128, 256, 128), (128, 384, 1056), (32, 32, 32)])
def test_oht_quantize_bit_exact(ah, b, outer, K, k_contig):
    logical = inputs.matrix(outer, K, 1.0, 500 + b, row_outliers=(3, 60.0, 60.0), col_outliers=(2, 30.0, 30.0))
    stored = logical if k_contig else np.ascontiguousarray(logical.T)
    say("oht_quantize", b, outer, K, "K-contiguous" if k_contig else "K-strided")
    for pad in (0, 8):
        x = ah.Operand(padded(stored, pad), k_contig)
        codes, scales = ah.adahop_oht_quantize(x, b)
        torch.cuda.synchronize()
        rc, rs = orc.oht_quantize(stored, k_contig, b)
        assert np.array_equal(host(scales), rs)
        assert np.array_equal(host(codes), rc)


@pytest.mark.parametrize("b,M,N,pad", [(32, 64, 96, 0), (32, 96, 544, 5), (64, 192, 320, 0), (128, 256, 384, 3),
                                       (128, 128, 1280, 0)])
def test_oht_inverse_matches_double_rotations(ah, b, M, N, pad):
    rng = np.random.default_rng(b + M + N)
    Cq = (rng.standard_normal((M, N)) * np.exp(rng.uniform(-3, 3, (M, 1)))).astype(np.float32)
    say("oht_inverse", b, M, N, "ldc", N + pad)
    buf = torch.full((M, N + pad), 3.0, dtype=torch.float32, device="cuda")
    buf[:, :N] = torch.from_numpy(Cq).cuda()
    ah.adahop_oht_inverse(buf[:, :N], b)
    torch.cuda.synchronize()
    want = orc.oht_inverse(Cq, b, b)
    err = rel_fro(host(buf[:, :N]), want)
    say(f"  vs oracle {err:.2e}")
    assert err < 1e-5
    assert bool((buf[:, N:] == 3.0).all())


@pytest.mark.parametrize("b,M,N", [(32, 64, 160), (64, 128, 448), (128, 384, 640)])
def test_oht_inverse_same_bits_in_both_kernels(ah, b, M, N):
    """The rotation with butterflies in registers (16-byte aligned rows) and the one through LDS (any ldc) apply the
    same butterfly network: identical bits, including exact zeros (a block of equal values transforms to one
    nonzero and B - 1 zeros)."""
    rng = np.random.default_rng(b * 7 + N)
    Cq = (rng.standard_normal((M, N)) * np.exp(rng.uniform(-3, 3, (M, 1)))).astype(np.float32)
    Cq[:b, :b] = -1.25                      # exact cancellations
    Cq[b // 2, b:2 * b] = 0.0
    say("oht_inverse, both kernels", b, M, N)
    fast = torch.from_numpy(Cq).cuda()
    slow = torch.full((M, N + 1), 9.0, dtype=torch.float32, device="cuda")
    slow[:, :N] = torch.from_numpy(Cq).cuda()
    ah.adahop_oht_inverse(fast, b)
    ah.adahop_oht_inverse(slow[:, :N], b)
    torch.cuda.synchronize()
    assert np.array_equal(host(fast).view(np.uint32), host(slow[:, :N]).view(np.uint32))


@pytest.mark.parametrize("b,M,N,K,layouts", [(128, 256, 384, 512, (True, True)), (64, 320, 192, 160, (True, False)),
                                             (32, 512, 512, 1024, (False, False)), (128, 768, 512, 1024, (True, False))])
def test_oht_whole_strategy(ah, b, M, N, K, layouts):
    a_kc, b_kc = layouts
    A_log = inputs.matrix(M, K, 1.0, 600, row_outliers=(4, 50.0, 50.0))
    B_log = inputs.matrix(N, K, 0.02, 601, row_outliers=(3, 30.0, 30.0))          # rows of [N, K] = columns of B
    A = inputs.Operand(A_log if a_kc else np.ascontiguousarray(A_log.T), a_kc)
    B = inputs.Operand(B_log if b_kc else np.ascontiguousarray(B_log.T), b_kc)
    say("OHT strategy", b, M, N, K, layouts)
    dA, dB = ah.Operand.from_bits(A.bits, a_kc), ah.Operand.from_bits(B.bits, b_kc)
    out = ah.adahop_gemm(dA, dB, inputs.OHT, b)
    torch.cuda.synchronize()
    ref = orc.oht_gemm(A.bits, a_kc, B.bits, b_kc, b)
    for name in ("a_scales", "b_scales", "a_codes", "b_codes"):
        assert np.array_equal(host(out[name]), ref[name]), name
    err = rel_fro(host(out["C"]), ref["C"])
    exact = orc.exact_gemm(A.bits, a_kc, B.bits, b_kc)
    q_oht = rel_fro(host(out["C"]), exact)
    q_iht = rel_fro(host(ah.adahop_gemm(dA, dB, inputs.IHT, 32)["C"]), exact)     # inner transform, block 32
    q_none = rel_fro(host(ah.adahop_gemm(dA, dB, inputs.NONE, 0)["C"]), exact)
    say(f"  vs oracle {err:.2e}; error vs the exact product: OHT {q_oht:.3e}, IHT {q_iht:.3e}, none {q_none:.3e}")
    assert err < 1e-3
    assert np.isfinite(q_oht) and q_oht < 1.0
    # operands packed once with the OHT strategy give the same bits
    pa = ah.adahop_pack_operand(dA, 0, inputs.OHT, b)
    pb = ah.adahop_pack_operand(dB, 1, inputs.OHT, b)
    again = ah.adahop_gemm(dA, dB, inputs.OHT, b, a_packed=pa, b_packed=pb)
    torch.cuda.synchronize()
    assert np.array_equal(host(pa[0]), ref["a_codes"]) and np.array_equal(host(pb[1]), ref["b_scales"])
    assert np.array_equal(host(again["C"]), host(out["C"]))


def test_oht_argument_checks_on_device_operands(ah):
    A = ah.Operand.from_bits(inputs.matrix(96, 64, 1.0, 1), True)
    B = ah.Operand.from_bits(inputs.matrix(64, 64, 1.0, 2), True)
    for kwargs in (dict(iht_block=64), dict(iht_block=256), dict(iht_block=32, c_bf16=True)):   # 96 % 64, block, bf16 C
        with pytest.raises(ah.AdahopError) as e:
            ah.adahop_gemm(A, B, inputs.OHT, kwargs["iht_block"], c_bf16=kwargs.get("c_bf16", False))
        assert e.value.status == ah.ADAHOP_E_INVALID_ARG
