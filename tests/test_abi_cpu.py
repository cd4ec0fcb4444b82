"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function that
include/adahop.h declares, and rejects bad arguments before touching HIP."""
import ctypes as C
import os
import re

import pytest

from paper_2604_02525_amd import binding as ah

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "adahop.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(adahop_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) >= 10
    L = ah.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(ah.EXPORTS) == names
    assert L.adahop_abi_version() == 1


FAKE = 0x10000  # non-null, 16-byte aligned, never dereferenced on these paths


def op(outer=64, K=128, ld=None, kc=1, data=FAKE):
    return ah.adahop_operand_t(data, outer, K, K if ld is None and kc else (outer if ld is None else ld), kc)


@pytest.mark.parametrize("bad", [
    dict(K=100), dict(K=0), dict(outer=0), dict(data=0), dict(data=FAKE + 2), dict(ld=120), dict(ld=132), dict(kc=2),
])
def test_quantize_rejects_bad_operands(bad):
    L = ah.lib()
    x = op(**bad)
    assert L.adahop_quantize_mx(C.byref(x), FAKE, FAKE, None) == ah.ADAHOP_E_INVALID_ARG
    assert L.adahop_iht_quantize(C.byref(x), 32, None, None, FAKE, FAKE, None) == ah.ADAHOP_E_INVALID_ARG


def test_iht_quantize_sr_rejects_what_the_deterministic_entry_rejects():
    L = ah.lib()
    x = op(K=192)
    f = lambda xx, b, zk, codes: L.adahop_iht_quantize_sr(None if xx is None else C.byref(xx), b, None, zk, 12345, codes,
                                                           FAKE, None)
    assert f(x, 48, None, FAKE) == ah.ADAHOP_E_INVALID_ARG
    assert f(x, 128, None, FAKE) == ah.ADAHOP_E_INVALID_ARG        # 192 % 128
    assert f(x, 64, FAKE + 4, FAKE) == ah.ADAHOP_E_INVALID_ARG     # mask alignment
    assert f(x, 64, None, None) == ah.ADAHOP_E_INVALID_ARG
    assert f(None, 64, None, FAKE) == ah.ADAHOP_E_INVALID_ARG
    assert f(op(K=100), 0, None, FAKE) == ah.ADAHOP_E_INVALID_ARG


def test_iht_quantize_rejects_bad_blocks_and_pointers():
    L = ah.lib()
    x = op(K=192)
    for b in (16, 48, 512, -32):
        assert L.adahop_iht_quantize(C.byref(x), b, None, None, FAKE, FAKE, None) == ah.ADAHOP_E_INVALID_ARG
    assert L.adahop_iht_quantize(C.byref(x), 128, None, None, FAKE, FAKE, None) == ah.ADAHOP_E_INVALID_ARG  # 192 % 128
    assert L.adahop_iht_quantize(C.byref(x), 64, None, None, None, FAKE, None) == ah.ADAHOP_E_INVALID_ARG
    assert L.adahop_iht_quantize(C.byref(x), 64, None, FAKE + 4, FAKE, FAKE, None) == ah.ADAHOP_E_INVALID_ARG  # mask align
    assert L.adahop_iht_quantize(None, 64, None, None, FAKE, FAKE, None) == ah.ADAHOP_E_INVALID_ARG


def test_foid_rejects_bad_arguments():
    L = ah.lib()
    x = op()
    assert L.adahop_foid_topk(C.byref(x), 2, 1, FAKE, FAKE, FAKE, None) == ah.ADAHOP_E_INVALID_ARG
    assert L.adahop_foid_topk(C.byref(x), 0, 65, FAKE, FAKE, FAKE, None) == ah.ADAHOP_E_INVALID_ARG
    assert L.adahop_foid_topk(C.byref(x), 1, 129, FAKE, FAKE, FAKE, None) == ah.ADAHOP_E_INVALID_ARG
    assert L.adahop_foid_topk(C.byref(x), 0, -1, FAKE, FAKE, FAKE, None) == ah.ADAHOP_E_INVALID_ARG
    assert L.adahop_foid_topk(C.byref(x), 0, 4, None, FAKE, FAKE, None) == ah.ADAHOP_E_INVALID_ARG


def test_gemm_mx_rejects_bad_arguments():
    L = ah.lib()
    need = L.adahop_gemm_mx_workspace_bytes(64, 64, 128)
    assert need >= 2 * 64 * 4 and need % 256 == 0
    ok = [64, 64, 128, FAKE, FAKE, FAKE, FAKE, FAKE, 64, FAKE, need, None]
    for pos, val in ((0, 0), (2, 48), (2, 0), (3, None), (7, None), (8, 63), (3, FAKE + 8)):
        a = list(ok)
        a[pos] = val
        assert L.adahop_gemm_mx(*a) == ah.ADAHOP_E_INVALID_ARG, (pos, val)
    for pos, val in ((9, None), (9, FAKE + 64), (10, need - 1)):
        a = list(ok)
        a[pos] = val
        assert L.adahop_gemm_mx(*a) == ah.ADAHOP_E_WORKSPACE, (pos, val)


def test_gemm_argument_and_workspace_checks():
    L = ah.lib()
    A, B = op(64, 256), op(32, 256)
    need = L.adahop_gemm_workspace_bytes(64, 32, 256, ah.ADAHOP_IHT_OE_K, 8)
    lay = ah.adahop_gemm_workspace_layout(64, 32, 256, ah.ADAHOP_IHT_OE_K, 8)
    assert need == lay.total and need % 256 == 0
    offs = [lay.a_codes, lay.a_scales, lay.b_codes, lay.b_scales, lay.mask, lay.scores, lay.gather_a, lay.gather_b,
            lay.gemm]
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs)
    assert lay.a_scales - lay.a_codes >= 64 * 128 and lay.gather_b - lay.gather_a >= 64 * 64 * 2
    call = lambda **kw: L.adahop_gemm(C.byref(kw.get("A", A)), C.byref(kw.get("B", B)), kw.get("C", FAKE),
                                      kw.get("ldc", 32), kw.get("s", ah.ADAHOP_IHT), kw.get("b", 64), kw.get("k", 0),
                                      kw.get("idx", FAKE), 0, kw.get("ws", FAKE), kw.get("wsb", need), None)
    assert call(B=op(32, 128)) == ah.ADAHOP_E_INVALID_ARG          # K mismatch
    assert call(ldc=31) == ah.ADAHOP_E_INVALID_ARG
    assert call(s=7) == ah.ADAHOP_E_INVALID_ARG
    assert call(b=48) == ah.ADAHOP_E_INVALID_ARG
    assert call(b=0) == ah.ADAHOP_E_INVALID_ARG                    # IHT strategies need a block
    assert call(s=ah.ADAHOP_IHT_OE_ROW, k=65) == ah.ADAHOP_E_INVALID_ARG
    assert call(s=ah.ADAHOP_IHT_OE_COL, k=33) == ah.ADAHOP_E_INVALID_ARG
    assert call(s=ah.ADAHOP_IHT_OE_K, k=8, idx=None) == ah.ADAHOP_E_INVALID_ARG
    assert call(ws=None) == ah.ADAHOP_E_WORKSPACE
    assert call(ws=FAKE + 16) == ah.ADAHOP_E_WORKSPACE
    assert call(s=ah.ADAHOP_IHT_OE_K, k=8, wsb=need - 1) == ah.ADAHOP_E_WORKSPACE
    assert L.adahop_gemm_workspace_bytes(64, 32, 100, ah.ADAHOP_IHT, 0) == 0


def test_gemm_mx_bf16out_rejects_bad_arguments():
    L = ah.lib()
    need = L.adahop_gemm_mx_workspace_bytes(64, 64, 128)
    ok = [64, 64, 128, FAKE, FAKE, FAKE, FAKE, FAKE + 2, 64, FAKE, need, None]   # bf16 C: 2-byte alignment is enough
    for pos, val in ((0, 0), (2, 48), (7, None), (7, FAKE + 1), (8, 63)):
        a = list(ok)
        a[pos] = val
        assert L.adahop_gemm_mx_bf16out(*a) == ah.ADAHOP_E_INVALID_ARG, (pos, val)
    a = list(ok)
    a[10] = need - 1
    assert L.adahop_gemm_mx_bf16out(*a) == ah.ADAHOP_E_WORKSPACE


def test_pack_operand_argument_checks():
    L = ah.lib()
    x = op(64, 256)
    f = lambda **kw: L.adahop_pack_operand(C.byref(kw.get("x", x)), kw.get("is_b", 0), kw.get("s", ah.ADAHOP_IHT),
                                           kw.get("b", 64), kw.get("k", 0), kw.get("idx", None), kw.get("mask", None),
                                           kw.get("codes", FAKE), kw.get("scales", FAKE), None)
    assert f(x=op(K=100)) == ah.ADAHOP_E_INVALID_ARG
    assert f(s=9) == ah.ADAHOP_E_INVALID_ARG
    assert f(b=48) == ah.ADAHOP_E_INVALID_ARG
    assert f(b=0) == ah.ADAHOP_E_INVALID_ARG
    assert f(codes=None) == ah.ADAHOP_E_INVALID_ARG
    assert f(codes=FAKE + 8) == ah.ADAHOP_E_INVALID_ARG
    # the residual of A depends on the indices under OE_ROW and OE_K, that of B under OE_COL and OE_K
    for s, is_b, dim in ((ah.ADAHOP_IHT_OE_ROW, 0, 64), (ah.ADAHOP_IHT_OE_COL, 1, 64), (ah.ADAHOP_IHT_OE_K, 0, 256),
                         (ah.ADAHOP_IHT_OE_K, 1, 256)):
        assert f(s=s, is_b=is_b, k=4, idx=None, mask=FAKE) == ah.ADAHOP_E_INVALID_ARG
        assert f(s=s, is_b=is_b, k=4, idx=FAKE, mask=None) == ah.ADAHOP_E_INVALID_ARG
        assert f(s=s, is_b=is_b, k=4, idx=FAKE, mask=FAKE + 4) == ah.ADAHOP_E_INVALID_ARG
        assert f(s=s, is_b=is_b, k=dim + 1, idx=FAKE, mask=FAKE) == ah.ADAHOP_E_INVALID_ARG
        assert f(s=s, is_b=is_b, k=-1, idx=FAKE, mask=FAKE) == ah.ADAHOP_E_INVALID_ARG


def test_gemm_ex_argument_checks():
    L = ah.lib()
    A, B = op(64, 256), op(32, 256)
    need = L.adahop_gemm_workspace_bytes(64, 32, 256, ah.ADAHOP_IHT_OE_K, 8)

    def call(opts, s=ah.ADAHOP_IHT, k=0, given=0, c=FAKE, ldc=32, wsb=need):
        o = None if opts is None else C.byref(ah.adahop_gemm_opts_t(*opts))
        return L.adahop_gemm_ex(C.byref(A), C.byref(B), c, ldc, s, 64, k, FAKE, given, o, FAKE, wsb, None)

    assert call(None, ldc=31) == ah.ADAHOP_E_INVALID_ARG                          # same checks as adahop_gemm
    assert call((None, None, None, None, 2)) == ah.ADAHOP_E_INVALID_ARG           # c_bf16 is 0 or 1
    assert call((None, None, None, None, 0), c=FAKE + 2) == ah.ADAHOP_E_INVALID_ARG   # float C: 4-byte aligned
    assert call((FAKE, None, None, None, 0)) == ah.ADAHOP_E_INVALID_ARG           # codes without scales
    assert call((None, None, None, FAKE, 0)) == ah.ADAHOP_E_INVALID_ARG
    assert call((FAKE + 8, FAKE, None, None, 0)) == ah.ADAHOP_E_INVALID_ARG       # codes 16-byte aligned
    # a packed operand whose residual depends on the indices needs the caller's indices
    assert call((FAKE, FAKE, None, None, 0), s=ah.ADAHOP_IHT_OE_ROW, k=4) == ah.ADAHOP_E_INVALID_ARG
    assert call((None, None, FAKE, FAKE, 0), s=ah.ADAHOP_IHT_OE_COL, k=4) == ah.ADAHOP_E_INVALID_ARG
    assert call((None, None, FAKE, FAKE, 0), s=ah.ADAHOP_IHT_OE_K, k=4) == ah.ADAHOP_E_INVALID_ARG
    assert call((FAKE, FAKE, FAKE, FAKE, 1), s=ah.ADAHOP_IHT_OE_K, k=8, given=1, wsb=need - 1) == ah.ADAHOP_E_WORKSPACE


def test_oht_argument_checks():
    L = ah.lib()
    x = op(64, 128)
    for b in (0, 16, 48, 256):
        assert L.adahop_oht_quantize(C.byref(x), b, FAKE, FAKE, None) == ah.ADAHOP_E_INVALID_ARG
    assert L.adahop_oht_quantize(C.byref(op(96, 128)), 64, FAKE, FAKE, None) == ah.ADAHOP_E_INVALID_ARG   # 96 % 64
    assert L.adahop_oht_quantize(C.byref(x), 32, None, FAKE, None) == ah.ADAHOP_E_INVALID_ARG
    assert L.adahop_oht_quantize(C.byref(x), 32, FAKE + 8, FAKE, None) == ah.ADAHOP_E_INVALID_ARG
    assert L.adahop_oht_quantize(C.byref(op(K=100)), 32, FAKE, FAKE, None) == ah.ADAHOP_E_INVALID_ARG
    inv = lambda c=FAKE, M=64, N=64, ldc=64, b=32: L.adahop_oht_inverse(c, M, N, ldc, b, None)
    assert inv(c=None) == ah.ADAHOP_E_INVALID_ARG
    assert inv(c=FAKE + 2) == ah.ADAHOP_E_INVALID_ARG
    assert inv(M=48) == ah.ADAHOP_E_INVALID_ARG
    assert inv(N=80) == ah.ADAHOP_E_INVALID_ARG
    assert inv(ldc=63) == ah.ADAHOP_E_INVALID_ARG
    assert inv(b=256) == ah.ADAHOP_E_INVALID_ARG
    assert inv(M=0) == ah.ADAHOP_E_INVALID_ARG
    # whole path: block, divisibility of M and N, float C only
    A, B = op(64, 256), op(96, 256)
    need = L.adahop_gemm_workspace_bytes(64, 96, 256, ah.ADAHOP_OHT, 0)
    assert need > 0
    g = lambda b, opts=None: L.adahop_gemm_ex(C.byref(A), C.byref(B), FAKE, 96, ah.ADAHOP_OHT, b, 0, None, 0,
                                              None if opts is None else C.byref(ah.adahop_gemm_opts_t(*opts)), FAKE, need,
                                              None)
    assert g(64) == ah.ADAHOP_E_INVALID_ARG            # 96 % 64
    assert g(256) == ah.ADAHOP_E_INVALID_ARG
    assert g(32, (None, None, None, None, 1)) == ah.ADAHOP_E_INVALID_ARG


def test_oe_gemm_argument_checks():
    L = ah.lib()
    A, B = op(64, 256), op(32, 256)
    f = lambda kind, idx, k, ws, wsb: L.adahop_oe_gemm_bf16(C.byref(A), C.byref(B), kind, idx, k, FAKE, 32, ws, wsb, None)
    assert f(ah.ADAHOP_IHT, FAKE, 4, None, 0) == ah.ADAHOP_E_INVALID_ARG
    assert f(ah.ADAHOP_IHT_OE_ROW, None, 4, None, 0) == ah.ADAHOP_E_INVALID_ARG
    assert f(ah.ADAHOP_IHT_OE_ROW, FAKE, 65, None, 0) == ah.ADAHOP_E_INVALID_ARG
    assert f(ah.ADAHOP_IHT_OE_K, FAKE, 4, None, 0) == ah.ADAHOP_E_WORKSPACE
    assert f(ah.ADAHOP_IHT_OE_K, FAKE, 0, None, 0) == ah.ADAHOP_OK      # nothing to do
    assert L.adahop_oe_gather_bytes(64, 32, 256, ah.ADAHOP_IHT_OE_K, 4) == 64 * 64 * 2 + 32 * 64 * 2


def test_status_strings():
    L = ah.lib()
    assert L.adahop_status_string(0) == b"ok"
    for s in (-1, -2, -3, -99):
        assert len(L.adahop_status_string(s)) > 3


def test_pattern_argument_checks_and_strategy_table():
    L = ah.lib()
    x = op(64, 256)
    need = L.adahop_detect_pattern_workspace_bytes(C.byref(x))
    assert need > 0 and need % 256 == 0
    f = lambda **kw: L.adahop_detect_pattern(C.byref(kw.get("x", x)), kw.get("tau", 2.0), kw.get("p", FAKE), kw.get("s", FAKE),
                                             kw.get("ws", FAKE), kw.get("wsb", need), None)
    assert f(x=op(1, 256)) == ah.ADAHOP_E_INVALID_ARG          # a variance vector needs two entries
    assert f(tau=0.0) == ah.ADAHOP_E_INVALID_ARG
    assert f(p=None) == ah.ADAHOP_E_INVALID_ARG
    assert f(s=None) == ah.ADAHOP_E_INVALID_ARG
    assert f(ws=None) == ah.ADAHOP_E_WORKSPACE
    assert f(wsb=need - 1) == ah.ADAHOP_E_WORKSPACE
    assert L.adahop_detect_pattern_workspace_bytes(C.byref(op(1, 256))) == 0
    # Sec. 4.2, in operand-sense patterns (outer-wise = the paper's R for A and C for B)
    N, O, K = ah.ADAHOP_PATTERN_NONE, ah.ADAHOP_PATTERN_OUTER, ah.ADAHOP_PATTERN_K
    assert ah.adahop_select_strategy(K, N) == (ah.ADAHOP_IHT, False)          # CN
    assert ah.adahop_select_strategy(N, N) == (ah.ADAHOP_IHT, False)          # NN
    assert ah.adahop_select_strategy(K, K) == (ah.ADAHOP_IHT, False)          # CR
    assert ah.adahop_select_strategy(O, N) == (ah.ADAHOP_IHT_OE_ROW, False)   # RN
    assert ah.adahop_select_strategy(O, O) == (ah.ADAHOP_IHT_OE_COL, False)   # RC
    assert ah.adahop_select_strategy(N, O) == (ah.ADAHOP_IHT_OE_COL, False)   # NC
    assert ah.adahop_select_strategy(K, O) == (ah.ADAHOP_IHT_OE_COL, False)   # CC, level 1
    assert ah.adahop_select_strategy(K, O, 2) == (ah.ADAHOP_NONE, True)       # CC, level 2: BF16
    assert ah.adahop_select_strategy(N, O, 2) == (ah.ADAHOP_IHT_OE_COL, False)
    with pytest.raises(ah.AdahopError):
        ah.adahop_select_strategy(3, N)
    with pytest.raises(ah.AdahopError):
        ah.adahop_select_strategy(N, N, 3)


def test_vote_pattern_matches_the_oracle_and_rejects_bad_input():
    """Host-side function: compared with the oracle on every multiset of up to 7 votes, plus the error paths."""
    import itertools
    from oracle import reference as orc
    L = ah.lib()
    for n in range(1, 8):
        for votes in itertools.combinations_with_replacement((0, 1, 2), n):
            assert ah.adahop_vote_pattern(list(votes)) == orc.vote_pattern(list(votes)), votes
    assert ah.adahop_vote_pattern([2] * 17 + [0] * 13) == ah.ADAHOP_PATTERN_K
    arr = (C.c_int32 * 3)(0, 3, 1)
    assert L.adahop_vote_pattern(arr, 3) == ah.ADAHOP_E_INVALID_ARG
    assert L.adahop_vote_pattern(arr, 0) == ah.ADAHOP_E_INVALID_ARG
    assert L.adahop_vote_pattern(None, 3) == ah.ADAHOP_E_INVALID_ARG


def test_size_limits_keep_every_launch_legal():
    """Operand extents beyond 2^21 are rejected up front (the second grid dimension of the K-strided quantisers,
    the pattern detector and the OHT kernels is K / 256, K / 128, stored rows / 256 and outer / block, and may not
    exceed 65535), so that no accepted shape can reach a launch that fails -- in particular the K = 2^24 operand for
    which the K-strided quantiser once dropped the stage-major scale copy the product then relied on."""
    L = ah.lib()
    big = 1 << 21
    q = lambda x: L.adahop_iht_quantize(C.byref(x), 256, None, None, FAKE, FAKE, None)
    for K in (1 << 24, big + 256):
        for kc in (1, 0):
            assert q(op(64, K, kc=kc)) == ah.ADAHOP_E_INVALID_ARG, (K, kc)
    assert q(op(big + 8, 256, kc=0)) == ah.ADAHOP_E_INVALID_ARG
    assert q(op(big, 1 << 15)) == ah.ADAHOP_E_INVALID_ARG                 # outer * K reaches 2^35
    assert L.adahop_gemm_mx_workspace_bytes(256, 256, 1 << 24) == 0
    assert L.adahop_gemm_mx_workspace_bytes(256, 256, big) == 2 * 256 * (big // 32)
    assert L.adahop_gemm_workspace_bytes(256, 256, 1 << 24, ah.ADAHOP_IHT, 0) == 0
    need = L.adahop_gemm_workspace_bytes(256, 256, big, ah.ADAHOP_IHT, 0)
    assert need > 0
    A = op(256, 1 << 24, kc=0)
    assert L.adahop_gemm(C.byref(A), C.byref(A), FAKE, 256, ah.ADAHOP_IHT, 256, 0, None, 0, FAKE, 1 << 40,
                         None) == ah.ADAHOP_E_INVALID_ARG
    assert L.adahop_foid_topk(C.byref(op(64, 1 << 24)), 1, 4, FAKE, FAKE, FAKE, None) == ah.ADAHOP_E_INVALID_ARG
    assert L.adahop_detect_pattern_workspace_bytes(C.byref(op(64, 1 << 24, kc=0))) == 0
    # OHT: outer / block is a grid dimension
    assert L.adahop_oht_quantize(C.byref(op(big, 32)), 32, FAKE, FAKE, None) == ah.ADAHOP_E_INVALID_ARG   # 65536 blocks
    assert L.adahop_oht_inverse(FAKE, big, 32, 32, 32, None) == ah.ADAHOP_E_INVALID_ARG
    assert L.adahop_pack_operand(C.byref(op(big, 32)), 0, ah.ADAHOP_OHT, 32, 0, None, None, FAKE, FAKE,
                                 None) == ah.ADAHOP_E_INVALID_ARG


def test_foid_noalloc_rejects_before_touching_the_gpu():
    L = ah.lib()
    f = lambda x, axis=0, k=4, idx=FAKE, mask=FAKE: L.adahop_foid_topk_noalloc(C.byref(x), axis, k, idx, mask, None)
    assert f(op(ah.FOID_NOALLOC_MAX_DIM + 8, 64)) == ah.ADAHOP_E_WORKSPACE        # beyond the built-in scratch
    assert f(op(64, ah.FOID_NOALLOC_MAX_DIM + 32), axis=1) == ah.ADAHOP_E_WORKSPACE
    assert f(op(), axis=2) == ah.ADAHOP_E_INVALID_ARG
    assert f(op(), k=65) == ah.ADAHOP_E_INVALID_ARG
    assert f(op(), idx=None) == ah.ADAHOP_E_INVALID_ARG
    assert f(op(), mask=FAKE + 4) == ah.ADAHOP_E_INVALID_ARG
    assert f(op(K=100)) == ah.ADAHOP_E_INVALID_ARG
