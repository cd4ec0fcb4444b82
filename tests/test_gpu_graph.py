"""The whole path under HIP graph capture (run with -m gpu).

The library allocates nothing, clears memory with kernels only and queues everything on the caller's stream, so
a call can be captured into a graph and replayed -- what a launch-bound caller (small products, ~10 launches each)
wants.  Each replay runs on fresh input bytes written into the captured buffers, with eager work and
synchronisations between the replays, and is compared with the eager result bit for bit and with the oracle.
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


def test_prepare_device_is_idempotent(ah):
    """The one-time set-up a capturing caller makes beforehand: succeeds, also when repeated or when entry points
    have already done their own part."""
    ah.adahop_prepare_device()
    ah.adahop_prepare_device()


@pytest.mark.parametrize("strategy,k", [(inputs.IHT, 0), (inputs.IHT_OE_K, 6), (inputs.IHT_OE_ROW, 5), (inputs.IHT_OE_COL, 4)])
def test_whole_path_replays_from_a_graph(ah, strategy, k):
    M, N, K, b = 512, 384, 1024, 128
    def fresh(seed):
        A = inputs.matrix(M, K, 1.0, seed, row_outliers=(4, 80.0, 80.0), col_outliers=(5, 40.0, 40.0))
        B = inputs.matrix(N, K, 0.02, seed + 1, row_outliers=(3, 30.0, 30.0))
        return A, B
    A0, B0 = fresh(800)
    a_buf = torch.from_numpy(A0.view(np.int16)).cuda()
    b_buf = torch.from_numpy(B0.view(np.int16)).cuda()
    opA, opB = ah.Operand(a_buf, True), ah.Operand(b_buf, True)
    ws = torch.empty(ah.adahop_gemm_workspace_bytes(M, N, K, strategy, k), dtype=torch.uint8, device="cuda")
    Cg = torch.empty((M, N), dtype=torch.float32, device="cuda")
    idx = torch.zeros(max(k, 1), dtype=torch.int32, device="cuda")

    def call(Cout):
        import ctypes as C
        rc = ah.lib().adahop_gemm(C.byref(opA.c()), C.byref(opB.c()), Cout.data_ptr(), Cout.stride(0), strategy, b, k,
                                  idx.data_ptr(), 0, ws.data_ptr(), ws.numel(), ah._stream(None))
        assert rc == 0

    call(Cg)                                   # warm up outside the capture (one-time function attributes)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            call(Cg)
    torch.cuda.synchronize()
    for rep, seed in enumerate((810, 820, 830)):
        say("graph replay", inputs.STRATEGY_NAMES[strategy], rep)
        A, B = fresh(seed)
        a_buf.copy_(torch.from_numpy(A.view(np.int16)))
        b_buf.copy_(torch.from_numpy(B.view(np.int16)))
        Cg.fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = Cg.clone()
        got_idx = idx.clone()
        Ce = torch.empty_like(Cg)              # eager work between the replays
        call(Ce)
        torch.cuda.synchronize()
        assert torch.equal(got, Ce)
        assert torch.equal(got_idx, idx)
        ref = orc.adahop_gemm(A, True, B, True, strategy, b, k)
        if k:
            assert np.array_equal(np.sort(got_idx.cpu().numpy()[:k]), ref["idx"])
        err = np.linalg.norm(got.cpu().numpy().astype(np.float64) - ref["C"]) / np.linalg.norm(ref["C"])
        assert err < 1e-3
