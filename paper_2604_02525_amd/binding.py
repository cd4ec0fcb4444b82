"""Thin ctypes binding over libadahop.so (the C ABI of include/adahop.h).

Argument marshalling only: every step of the path runs in the HIP kernels behind the ABI.  PyTorch is
used for device memory (outputs and workspaces are torch tensors) and for the current stream.  There
is no CPU fallback: if the library is missing, loading fails loudly.
"""
import ctypes as C
import os

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libadahop.so")

ADAHOP_NONE, ADAHOP_IHT, ADAHOP_IHT_OE_ROW, ADAHOP_IHT_OE_COL, ADAHOP_IHT_OE_K, ADAHOP_OHT = range(6)
ADAHOP_OK, ADAHOP_E_INVALID_ARG, ADAHOP_E_WORKSPACE, ADAHOP_E_HIP = 0, -1, -2, -3
ADAHOP_PATTERN_NONE, ADAHOP_PATTERN_OUTER, ADAHOP_PATTERN_K = range(3)

EXPORTS = ["adahop_quantize_mx", "adahop_iht_quantize", "adahop_foid_topk", "adahop_foid_topk_noalloc", "adahop_gemm_mx",
           "adahop_gemm_mx_bf16out", "adahop_gemm_mx_workspace_bytes", "adahop_pack_operand", "adahop_gemm_ex",
           "adahop_oht_quantize", "adahop_oht_inverse", "adahop_iht_quantize_sr",
           "adahop_gemm_workspace_layout", "adahop_gemm_workspace_bytes", "adahop_gemm", "adahop_oe_gather_bytes",
           "adahop_oe_gemm_bf16", "adahop_detect_pattern_workspace_bytes", "adahop_detect_pattern",
           "adahop_select_strategy", "adahop_vote_pattern", "adahop_probe_mfma_rate", "adahop_debug_force_gemm_kernel", "adahop_prepare_device", "adahop_last_hip_error", "adahop_status_string",
           "adahop_abi_version"]


class AdahopError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().adahop_status_string(status).decode()
        if status == ADAHOP_E_HIP:
            msg += f" [hipError {lib().adahop_last_hip_error()}]"
        super().__init__(f"{where}: {msg} ({status})")


class adahop_operand_t(C.Structure):
    _fields_ = [("data", C.c_void_p), ("outer", C.c_int64), ("K", C.c_int64), ("ld", C.c_int64), ("k_contig", C.c_int)]


class adahop_gemm_opts_t(C.Structure):
    _fields_ = [("a_codes", C.c_void_p), ("a_scales", C.c_void_p), ("b_codes", C.c_void_p), ("b_scales", C.c_void_p),
                ("c_bf16", C.c_int), ("sr_a", C.c_int), ("sr_b", C.c_int), ("sr_seed_a", C.c_uint64),
                ("sr_seed_b", C.c_uint64)]


class adahop_ws_layout_t(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("a_codes", "a_scales", "b_codes", "b_scales", "mask", "scores",
                                          "gather_a", "gather_b", "gemm", "total")]


_lib = None


def lib():
    """Load libadahop.so (built in-tree by paper_2604_02525_amd/build.py); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        P, I64, I, SZ = C.c_void_p, C.c_int64, C.c_int, C.c_size_t
        OP = C.POINTER(adahop_operand_t)
        L.adahop_quantize_mx.argtypes = [OP, P, P, P]
        L.adahop_iht_quantize.argtypes = [OP, I, P, P, P, P, P]
        L.adahop_iht_quantize_sr.argtypes = [OP, I, P, P, C.c_uint64, P, P, P]
        L.adahop_foid_topk.argtypes = [OP, I, I, P, P, P, P]
        L.adahop_foid_topk_noalloc.argtypes = [OP, I, I, P, P, P]
        L.adahop_gemm_mx.argtypes = [I64, I64, I64, P, P, P, P, P, I64, P, SZ, P]
        L.adahop_gemm_mx_bf16out.argtypes = [I64, I64, I64, P, P, P, P, P, I64, P, SZ, P]
        L.adahop_pack_operand.argtypes = [OP, I, I, I, I, P, P, P, P, P]
        L.adahop_gemm_ex.argtypes = [OP, OP, P, I64, I, I, I, P, I, C.POINTER(adahop_gemm_opts_t), P, SZ, P]
        L.adahop_oht_quantize.argtypes = [OP, I, P, P, P]
        L.adahop_oht_inverse.argtypes = [P, I64, I64, I64, I, P]
        L.adahop_gemm_mx_workspace_bytes.argtypes = [I64, I64, I64]
        L.adahop_gemm_mx_workspace_bytes.restype = SZ
        L.adahop_gemm_workspace_layout.argtypes = [I64, I64, I64, I, I, C.POINTER(adahop_ws_layout_t)]
        L.adahop_gemm_workspace_bytes.argtypes = [I64, I64, I64, I, I]
        L.adahop_gemm_workspace_bytes.restype = SZ
        L.adahop_gemm.argtypes = [OP, OP, P, I64, I, I, I, P, I, P, SZ, P]
        L.adahop_oe_gather_bytes.argtypes = [I64, I64, I64, I, I]
        L.adahop_oe_gather_bytes.restype = SZ
        L.adahop_oe_gemm_bf16.argtypes = [OP, OP, I, P, I, P, I64, P, SZ, P]
        L.adahop_detect_pattern_workspace_bytes.argtypes = [OP]
        L.adahop_detect_pattern_workspace_bytes.restype = SZ
        L.adahop_detect_pattern.argtypes = [OP, C.c_double, P, P, P, SZ, P]
        L.adahop_select_strategy.argtypes = [I, I, I, C.POINTER(C.c_int)]
        L.adahop_vote_pattern.argtypes = [C.POINTER(C.c_int32), I]
        L.adahop_probe_mfma_rate.argtypes = [I, I, I, I, P, P]
        L.adahop_debug_force_gemm_kernel.argtypes = [I]
        L.adahop_status_string.restype = C.c_char_p
        L.adahop_status_string.argtypes = [I]
        for name in EXPORTS:
            getattr(L, name)          # AttributeError here means the library is stale: rebuild it
        _lib = L
    return _lib


def _check(status, where):
    if status != ADAHOP_OK:
        raise AdahopError(status, where)


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _ptr(t):
    return None if t is None else t.data_ptr()


def _hold(stream, *temporaries):
    """Temporaries allocated here are released when the Python call returns, while the kernels that use them may
    still be queued.  That is safe on torch's current stream (the allocator hands the block to later work of the
    same stream only).  For any other stream the block must be tied to it: a torch stream object is recorded on
    each temporary; a raw stream handle cannot be, so the caller then has to pass the buffers in."""
    if stream is None:
        return
    handle = getattr(stream, "cuda_stream", stream)
    if handle == torch.cuda.current_stream().cuda_stream:
        return
    live = [t for t in temporaries if t is not None]
    if not live:
        return
    if not hasattr(stream, "cuda_stream"):
        raise ValueError("a raw stream handle other than the current stream needs caller-owned workspaces "
                         "(pass workspace= / gather_ws=, or a torch.cuda.Stream)")
    for t in live:
        t.record_stream(stream)


class Operand:
    """A bf16 device matrix as stored plus the flag saying which of its axes is K.

    tensor: 2-D torch tensor on the GPU (bfloat16, or int16/uint16 bit patterns), row stride = ld,
    unit column stride.  k_contig=True: tensor is [outer, K]; False: tensor is [K, outer].
    """

    def __init__(self, tensor, k_contig):
        assert tensor.dim() == 2 and tensor.stride(1) == 1 and tensor.element_size() == 2
        self.tensor = tensor
        self.k_contig = bool(k_contig)
        self.outer, self.K = (tensor.shape if k_contig else tensor.shape[::-1])
        self.ld = tensor.stride(0)

    @classmethod
    def from_bits(cls, bits, k_contig, device="cuda"):
        """Upload a numpy uint16 array of bf16 bit patterns."""
        t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device)
        return cls(t, k_contig)

    def c(self):
        return adahop_operand_t(self.tensor.data_ptr(), self.outer, self.K, self.ld, int(self.k_contig))


def _u8(shape, device):
    return torch.empty(shape, dtype=torch.uint8, device=device)


def adahop_iht_quantize(x, iht_block, zero_outer=None, zero_k=None, codes=None, scales=None, stream=None,
                        sr_seed=None):
    """sr_seed: round the elements stochastically under that seed (adahop_iht_quantize_sr)."""
    dev = x.tensor.device
    codes = _u8((x.outer, x.K // 2), dev) if codes is None else codes
    scales = _u8((x.outer, x.K // 32), dev) if scales is None else scales
    if sr_seed is not None:
        _check(lib().adahop_iht_quantize_sr(C.byref(x.c()), iht_block, _ptr(zero_outer), _ptr(zero_k), int(sr_seed),
                                            _ptr(codes), _ptr(scales), _stream(stream)), "adahop_iht_quantize_sr")
        return codes, scales
    _check(lib().adahop_iht_quantize(C.byref(x.c()), iht_block, _ptr(zero_outer), _ptr(zero_k), _ptr(codes),
                                     _ptr(scales), _stream(stream)), "adahop_iht_quantize")
    return codes, scales


def adahop_quantize_mx(x, codes=None, scales=None, stream=None):
    dev = x.tensor.device
    codes = _u8((x.outer, x.K // 2), dev) if codes is None else codes
    scales = _u8((x.outer, x.K // 32), dev) if scales is None else scales
    _check(lib().adahop_quantize_mx(C.byref(x.c()), _ptr(codes), _ptr(scales), _stream(stream)), "adahop_quantize_mx")
    return codes, scales


def adahop_foid_topk(x, axis, k, stream=None):
    dev = x.tensor.device
    dim = x.outer if axis == 0 else x.K
    idx = torch.empty(max(k, 1), dtype=torch.int32, device=dev)
    mask = _u8((dim,), dev)
    scores = torch.empty(dim, dtype=torch.float32, device=dev)
    _check(lib().adahop_foid_topk(C.byref(x.c()), axis, k, _ptr(idx), _ptr(mask), _ptr(scores), _stream(stream)),
           "adahop_foid_topk")
    return idx[:k], mask, scores


FOID_NOALLOC_MAX_DIM = 262144


def adahop_foid_topk_noalloc(x, axis, k, idx, mask, stream=None):
    """adahop_foid_topk with the scores in the library's built-in scratch: idx (int32, at least k entries) and mask
    (uint8 [dim]) are the caller's; nothing is allocated here or in the library."""
    _check(lib().adahop_foid_topk_noalloc(C.byref(x.c()), axis, k, _ptr(idx), _ptr(mask), _stream(stream)),
           "adahop_foid_topk_noalloc")
    return idx[:k], mask


def adahop_gemm_mx_workspace_bytes(M, N, K):
    return int(lib().adahop_gemm_mx_workspace_bytes(M, N, K))


def adahop_gemm_mx(a_codes, a_scales, b_codes, b_scales, Cout=None, workspace=None, stream=None, c_bf16=False):
    """C = dequant(A) dequant(B)^T; Cout float32, or bfloat16 with c_bf16 (or a bfloat16 Cout)."""
    M, N, K = a_codes.shape[0], b_codes.shape[0], a_codes.shape[1] * 2
    assert b_codes.shape[1] * 2 == K
    if Cout is None:
        Cout = torch.empty((M, N), dtype=torch.bfloat16 if c_bf16 else torch.float32, device=a_codes.device)
    if workspace is None:
        workspace = _u8((adahop_gemm_mx_workspace_bytes(M, N, K),), a_codes.device)
        _hold(stream, workspace)
    fn, name = ((lib().adahop_gemm_mx_bf16out, "adahop_gemm_mx_bf16out") if Cout.element_size() == 2
                else (lib().adahop_gemm_mx, "adahop_gemm_mx"))
    _check(fn(M, N, K, _ptr(a_codes), _ptr(a_scales), _ptr(b_codes), _ptr(b_scales), _ptr(Cout), Cout.stride(0),
              _ptr(workspace), workspace.numel(), _stream(stream)), name)
    return Cout


def adahop_gemm_workspace_layout(M, N, K, strategy, k):
    L = adahop_ws_layout_t()
    _check(lib().adahop_gemm_workspace_layout(M, N, K, strategy, k, C.byref(L)), "adahop_gemm_workspace_layout")
    return L


def adahop_gemm_workspace_bytes(M, N, K, strategy, k):
    return int(lib().adahop_gemm_workspace_bytes(M, N, K, strategy, k))


def adahop_oht_quantize(x, oht_block, codes=None, scales=None, stream=None):
    """Block Hadamard transform along the OUTER index, then MXFP4 along K (operand side of paper Eq. 6)."""
    dev = x.tensor.device
    codes = _u8((x.outer, x.K // 2), dev) if codes is None else codes
    scales = _u8((x.outer, x.K // 32), dev) if scales is None else scales
    _check(lib().adahop_oht_quantize(C.byref(x.c()), oht_block, _ptr(codes), _ptr(scales), _stream(stream)),
           "adahop_oht_quantize")
    return codes, scales


def adahop_oht_inverse(Cmat, oht_block, stream=None):
    """Cmat (float32 [M, N], row stride ld) <- H^T Cmat H^T in place (the rotations after the product, Eq. 6)."""
    assert Cmat.dtype == torch.float32 and Cmat.dim() == 2 and Cmat.stride(1) == 1
    _check(lib().adahop_oht_inverse(_ptr(Cmat), Cmat.shape[0], Cmat.shape[1], Cmat.stride(0), oht_block,
                                    _stream(stream)), "adahop_oht_inverse")
    return Cmat


def adahop_pack_operand(x, is_b, strategy, iht_block, k=0, idx=None, codes=None, scales=None, stream=None):
    """Residual -> IHT -> MXFP4 of one operand as the whole path would do it; returns (codes, scales)."""
    dev = x.tensor.device
    codes = _u8((x.outer, x.K // 2), dev) if codes is None else codes
    scales = _u8((x.outer, x.K // 32), dev) if scales is None else scales
    mask_ws = _u8((max(x.outer, x.K),), dev) if k else None
    _hold(stream, mask_ws)
    _check(lib().adahop_pack_operand(C.byref(x.c()), int(bool(is_b)), strategy, iht_block, k, _ptr(idx), _ptr(mask_ws),
                                     _ptr(codes), _ptr(scales), _stream(stream)), "adahop_pack_operand")
    return codes, scales


def adahop_gemm(A, B, strategy, iht_block, k=0, idx=None, Cout=None, workspace=None, stream=None,
                a_packed=None, b_packed=None, c_bf16=False, sr_seed_a=None, sr_seed_b=None):
    """Whole path.  Returns dict(C, idx, workspace, layout, a_codes, a_scales, b_codes, b_scales, mask)
    where the codes / scales / mask entries are views into the workspace.  a_packed / b_packed: (codes,
    scales) from adahop_pack_operand; c_bf16 (or a bfloat16 Cout): bf16 output; sr_seed_a / sr_seed_b:
    stochastic rounding of that operand.  Any of these routes the call through adahop_gemm_ex."""
    dev = A.tensor.device
    M, N, K = A.outer, B.outer, A.K
    L = adahop_gemm_workspace_layout(M, N, K, strategy, k)
    if workspace is None:
        workspace = _u8((L.total,), dev)
    if Cout is None:
        Cout = torch.empty((M, N), dtype=torch.bfloat16 if c_bf16 else torch.float32, device=dev)
    c_bf16 = Cout.element_size() == 2
    use_given = idx is not None
    if idx is None:
        idx = torch.empty(max(k, 1), dtype=torch.int32, device=dev)
    if a_packed is None and b_packed is None and not c_bf16 and sr_seed_a is None and sr_seed_b is None:
        _check(lib().adahop_gemm(C.byref(A.c()), C.byref(B.c()), _ptr(Cout), Cout.stride(0), strategy, iht_block, k,
                                 _ptr(idx), int(use_given), _ptr(workspace), workspace.numel(), _stream(stream)),
               "adahop_gemm")
    else:
        ac, asc = a_packed if a_packed is not None else (None, None)
        bc, bsc = b_packed if b_packed is not None else (None, None)
        opts = adahop_gemm_opts_t(_ptr(ac), _ptr(asc), _ptr(bc), _ptr(bsc), int(c_bf16), int(sr_seed_a is not None),
                                  int(sr_seed_b is not None), int(sr_seed_a or 0), int(sr_seed_b or 0))
        _check(lib().adahop_gemm_ex(C.byref(A.c()), C.byref(B.c()), _ptr(Cout), Cout.stride(0), strategy, iht_block, k,
                                    _ptr(idx), int(use_given), C.byref(opts), _ptr(workspace), workspace.numel(),
                                    _stream(stream)), "adahop_gemm_ex")
    dim = {ADAHOP_IHT_OE_ROW: M, ADAHOP_IHT_OE_COL: N, ADAHOP_IHT_OE_K: K}.get(strategy, 0)
    view = lambda off, n, shape: workspace[off:off + n].view(shape)
    return dict(C=Cout, idx=idx[:k], workspace=workspace, layout=L,
                a_codes=view(L.a_codes, M * K // 2, (M, K // 2)), a_scales=view(L.a_scales, M * K // 32, (M, K // 32)),
                b_codes=view(L.b_codes, N * K // 2, (N, K // 2)), b_scales=view(L.b_scales, N * K // 32, (N, K // 32)),
                mask=view(L.mask, dim, (dim,)))


def adahop_oe_gather_bytes(M, N, K, kind, k):
    return int(lib().adahop_oe_gather_bytes(M, N, K, kind, k))


def adahop_oe_gemm_bf16(A, B, kind, idx, Cout, gather_ws=None, stream=None):
    k = int(idx.numel())
    need = adahop_oe_gather_bytes(A.outer, B.outer, A.K, kind, k)
    if gather_ws is None and need:
        gather_ws = _u8((need,), A.tensor.device)
        _hold(stream, gather_ws)
    _check(lib().adahop_oe_gemm_bf16(C.byref(A.c()), C.byref(B.c()), kind, _ptr(idx), k, _ptr(Cout), Cout.stride(0),
                                     _ptr(gather_ws), 0 if gather_ws is None else gather_ws.numel(), _stream(stream)),
           "adahop_oe_gemm_bf16")
    return Cout


def adahop_probe_mfma_rate(random_operands, workgroups, iters, sink, stream=None, idle_sleeps=0):
    """Measurement aid: register-only matrix-core loop; returns the flop count of the launch."""
    _check(lib().adahop_probe_mfma_rate(int(bool(random_operands)), int(idle_sleeps), workgroups, iters, _ptr(sink),
                                        _stream(stream)),
           "adahop_probe_mfma_rate")
    return 2.0 * 65536 * 16 * iters * 4 * workgroups


def adahop_prepare_device():
    """One-time set-up of the current device for every kernel (call before capturing streams into graphs)."""
    _check(lib().adahop_prepare_device(), "adahop_prepare_device")


def adahop_debug_force_gemm_kernel(which):
    """Measurement aid: 0 = kernel chosen by shape, 1 = 256 x 256 tiles, 2 = 256 x 128 tiles with two accumulator sets,
    3 .. 6 = kernel by shape with the order of the tile walk forced (bands of A: contiguous runs / swept over B; 5, 6: of B)."""
    _check(lib().adahop_debug_force_gemm_kernel(int(which)), "adahop_debug_force_gemm_kernel")


def adahop_detect_pattern(x, tau=2.0, workspace=None, stream=None):
    """Outlier pattern of one operand: returns (pattern int32[1], stats float64[4]) device tensors."""
    dev = x.tensor.device
    need = int(lib().adahop_detect_pattern_workspace_bytes(C.byref(x.c())))
    if workspace is None:
        workspace = _u8((max(need, 256),), dev)
        _hold(stream, workspace)
    pattern = torch.empty(1, dtype=torch.int32, device=dev)
    stats = torch.empty(4, dtype=torch.float64, device=dev)
    _check(lib().adahop_detect_pattern(C.byref(x.c()), float(tau), _ptr(pattern), _ptr(stats), _ptr(workspace),
                                       workspace.numel(), _stream(stream)), "adahop_detect_pattern")
    return pattern, stats


def adahop_vote_pattern(patterns):
    """Majority class of a sequence of per-step patterns (host-side)."""
    arr = (C.c_int32 * len(patterns))(*[int(p) for p in patterns])
    r = lib().adahop_vote_pattern(arr, len(patterns))
    if r < 0:
        raise AdahopError(r, "adahop_vote_pattern")
    return r


def adahop_select_strategy(pattern_a, pattern_b, level=1):
    """(strategy, full_bf16) for a product from the patterns of its operands (host-side table)."""
    flag = C.c_int(0)
    s = lib().adahop_select_strategy(int(pattern_a), int(pattern_b), int(level), C.byref(flag))
    if s < 0:
        raise AdahopError(s, "adahop_select_strategy")
    return s, bool(flag.value)
