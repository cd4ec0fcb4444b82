"""The two tiled kernels of the MXFP4 product against the oracle's emulated product, each forced through the
diagnostics switch: the 256 x 256 tile kernel and the 256 x 128 tile kernel with two accumulator sets (C stores of a
tile issued during the next tile).  Shapes cover one tile, several tiles per workgroup (both accumulator sets, an odd
and an even count of tiles per workgroup), ragged edges that go to the bounds-checked kernel, tile counts whose
split over the eight XCDs does and does not fall on whole bands of the tile order, and stage counts from the minimum of
the two-set kernel (8) up.  Every element is compared (1e-5 relative Frobenius and the per-element
accumulation allowance of test_gpu_parity)."""
import numpy as np
import pytest

from oracle import reference as orc
from test_gpu_parity import ah, host, rel_fro, say  # noqa: F401  (ah is a fixture)

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

TILE256, DUAL = 1, 2


@pytest.fixture
def force(ah):
    yield lambda which: ah.adahop_debug_force_gemm_kernel(which)
    ah.adahop_debug_force_gemm_kernel(0)


def dequant_norms(codes, scales):
    table = np.array([0, .5, 1, 1.5, 2, 3, 4, 6, 0, .5, 1, 1.5, 2, 3, 4, 6], dtype=np.float64)   # magnitudes only
    mag2 = table[codes & 15] ** 2 + table[codes >> 4] ** 2                                        # per byte
    per_block = mag2.reshape(codes.shape[0], -1, 16).sum(axis=2)
    return np.sqrt((per_block * np.exp2(2.0 * (scales.astype(np.float64) - 127.0))).sum(axis=1))


@pytest.mark.parametrize("kernel", [TILE256, DUAL])
@pytest.mark.parametrize("shape", [(256, 128, 2048), (256, 256, 2048), (512, 384, 2304), (768, 1280, 4096),
                                   (300, 200, 2560), (1000, 650, 2048), (4352, 4096, 2048), (8448, 4224, 2048),
                                   (4096, 2176, 3072), (3584, 1024, 2048), (7168, 2048, 2048)])
def test_tiled_kernels_match_emulation(ah, force, kernel, shape):
    M, N, K = shape
    rng = np.random.default_rng(M + 3 * N + 7 * K)
    a_codes = rng.integers(0, 256, size=(M, K // 2), dtype=np.uint8)
    b_codes = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    a_scales = rng.integers(117, 137, size=(M, K // 32), dtype=np.uint8)
    b_scales = rng.integers(100, 120, size=(N, K // 32), dtype=np.uint8)
    say("tiled kernel", {TILE256: "256x256", DUAL: "256x128 two sets"}[kernel], shape)
    force(kernel)
    C = ah.adahop_gemm_mx(*(torch.from_numpy(t).cuda() for t in (a_codes, a_scales, b_codes, b_scales)))
    torch.cuda.synchronize()
    got = host(C).astype(np.float64)
    if M * N * K <= 4352 * 4096 * 2048:
        rows = cols = None
        ref = orc.mx_gemm(a_codes, a_scales, b_codes, b_scales)
    else:       # one row and one column in every 64-band: every tile, every wave's part of it
        rows = (np.arange(0, M, 64) + rng.integers(0, 64, (M + 63) // 64)).clip(max=M - 1).astype(np.int32)
        cols = (np.arange(0, N, 64) + rng.integers(0, 64, (N + 63) // 64)).clip(max=N - 1).astype(np.int32)
        ref = orc.mx_gemm(a_codes, a_scales, b_codes, b_scales, rows, cols)
        got = got[np.ix_(rows, cols)]
    err = rel_fro(got, ref)
    na, nb = dequant_norms(a_codes, a_scales), dequant_norms(b_codes, b_scales)
    bar = 2.0 ** -20 * np.outer(na if rows is None else na[rows], nb if cols is None else nb[cols])
    worst = float((np.abs(got - ref) / bar).max())
    say(f"  rel_fro {err:.2e}, worst element at {worst:.3f} of its allowance")
    assert err < 1e-5
    assert worst <= 1.0


@pytest.mark.parametrize("kernel", [TILE256, DUAL])
def test_tiled_kernels_single_nonzero_positions(ah, force, kernel):
    """One nonzero code per operand: the product lands in exactly one element of C with exactly the right value, for
    positions in different tiles, waves, accumulator tiles, pipeline stages and scale slots."""
    M, N, K = 768, 512, 2560
    force(kernel)
    rng = np.random.default_rng(kernel)
    for _ in range(12):
        m, n, ka = int(rng.integers(0, M)), int(rng.integers(0, N)), int(rng.integers(0, K))
        a_codes = np.zeros((M, K // 2), np.uint8)
        b_codes = np.zeros((N, K // 2), np.uint8)
        a_scales = np.full((M, K // 32), 127, np.uint8)
        b_scales = np.full((N, K // 32), 127, np.uint8)
        a_codes[m, ka // 2] = int(rng.integers(1, 16)) << (4 * (ka & 1))
        b_codes[n, ka // 2] = int(rng.integers(1, 16)) << (4 * (ka & 1))
        if (a_codes[m, ka // 2] >> (4 * (ka & 1))) & 7 == 0 or (b_codes[n, ka // 2] >> (4 * (ka & 1))) & 7 == 0:
            continue                                                       # a signed zero: nothing to find
        a_scales[m, ka // 32] = int(rng.integers(120, 135))
        b_scales[n, ka // 32] = int(rng.integers(120, 135))
        say("single nonzero", kernel, (m, n, ka))
        C = host(ah.adahop_gemm_mx(*(torch.from_numpy(t).cuda() for t in (a_codes, a_scales, b_codes, b_scales))))
        ref = orc.mx_gemm(a_codes, a_scales, b_codes, b_scales)
        assert np.count_nonzero(ref) == 1
        assert np.array_equal(C.astype(np.float64), ref)
