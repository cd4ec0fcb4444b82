"""The entry point that allocates nothing (adahop_foid_topk_noalloc) against adahop_foid_topk, through the C ABI:
indices and masks must be identical bit for bit, on two calls in a row that share the library's built-in
scratch -- the second on a smaller input, so stale scores of the first call lie beyond what it writes."""
import ctypes as C

import numpy as np
import pytest

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


def run_pair(ah, bits, k_contig, axis, k):
    x = ah.Operand.from_bits(bits, k_contig)
    dim = x.outer if axis == 0 else x.K
    ref_idx, ref_mask, _ = ah.adahop_foid_topk(x, axis, k)
    idx = torch.full((max(k, 1),), -1, dtype=torch.int32, device="cuda")
    mask = torch.full((dim,), 7, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    rc = ah.lib().adahop_foid_topk_noalloc(C.byref(x.c()), axis, k, idx.data_ptr(), mask.data_ptr(),
                                           torch.cuda.current_stream().cuda_stream)
    assert rc == ah.ADAHOP_OK
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(idx[:k], ref_idx), "indices differ from adahop_foid_topk"
    assert torch.equal(mask, ref_mask), "mask differs from adahop_foid_topk"
    return idx[:k].cpu().numpy()


def test_no_alloc_entry_matches_foid_topk_on_two_calls_in_a_row(ah):
    big = inputs.matrix(28672, 96, 1.0, 321, row_outliers=(40, 30.0, 60.0))
    small = inputs.matrix(3000, 160, 1.0, 322, row_outliers=(9, 30.0, 60.0), col_outliers=(5, 40.0, 40.0))
    say("no-alloc FOID, first call", big.shape, "axis 0, k = 287")
    first = run_pair(ah, big, True, 0, 287)
    assert len(np.unique(first)) == 287
    say("no-alloc FOID, second call on a smaller input", small.shape, "axis 0, k = 30")
    run_pair(ah, small, True, 0, 30)
    say("no-alloc FOID, K-strided operand and axis 1", small.shape)
    run_pair(ah, np.ascontiguousarray(small.T), False, 0, 12)
    run_pair(ah, small, True, 1, 5)
    run_pair(ah, small, True, 1, 0)


def test_no_alloc_entry_rejects_sizes_beyond_its_scratch(ah):
    x = ah.adahop_operand_t(0x10000, ah.FOID_NOALLOC_MAX_DIM + 8, 64, 64, 1)
    say("no-alloc FOID, dim beyond the limit")
    assert ah.lib().adahop_foid_topk_noalloc(C.byref(x), 0, 4, 0x10000, 0x10000, None) == ah.ADAHOP_E_WORKSPACE
    ok = ah.adahop_operand_t(0x10000, ah.FOID_NOALLOC_MAX_DIM, 64, 64, 1)
    assert ah.lib().adahop_foid_topk_noalloc(C.byref(ok), 2, 4, 0x10000, 0x10000, None) == ah.ADAHOP_E_INVALID_ARG
