"""GPU-vs-oracle parity through the C ABI (run with -m gpu on an MI355X).

Bars: packed E2M1 codes, E8M0 scales, FOID indices and masks bit-exact.  GEMM outputs: within 1e-3
relative Frobenius error of the oracle's emulated-MXFP4 result, taken separately over the extracted
rows / columns (BF16 path, ~100x larger values) and over the rest, so that the large entries cannot
hide an error in the ordinary ones; and every compared element within
    |C_gpu[i, j] - C_oracle[i, j]| <= 2^-20 |A[i, :]|_2 |B[j, :]|_2.
Both sides sum the same exact products (E2M1 values times powers of two, or bf16 x bf16, are exact in
fp32); only the fp32 accumulation order of the GPU differs from the oracle's double sum.  A length-K
fp32 accumulation errs by about sqrt(K) 2^-24 |C| and |C| is about |A_i| |B_j| / sqrt(K) for these
inputs, so the allowance is some tens of times the expected error and, relative to a typical |C|,
sqrt(K) 2^-20 <= 1e-4: a wrong operand byte, scale or tile lands orders of magnitude above it.
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


def rel_fro(got, ref):
    return float(np.linalg.norm(got.astype(np.float64) - ref) / max(np.linalg.norm(ref), 1e-300))


def row_norms(op, sel=None):
    """2-norms of the logical rows (all of them, or those in sel) of an inputs.Operand, in float64."""
    bits = op.bits if op.k_contig else op.bits.T
    if sel is not None:
        bits = bits[np.asarray(sel, dtype=np.int64)]
    out = np.empty(bits.shape[0])
    for r0 in range(0, bits.shape[0], 1024):          # in slabs: a whole config operand in float64 is gigabytes
        v = (np.ascontiguousarray(bits[r0:r0 + 1024]).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        out[r0:r0 + 1024] = np.sqrt((v * v).sum(axis=1))
    return out


def check_c(got, ref, g, rows=None, cols=None, extracted=None, tol=1e-3):
    """The bars of the module docstring on C (got: what the GPU wrote, ref: the oracle's, both on rows x cols).
    extracted: the indices the strategy routed to BF16 (rows for OE-row, columns for OE-col)."""
    got = got.astype(np.float64)
    bar = 2.0 ** -20 * np.outer(row_norms(g.A, rows), row_norms(g.B, cols))
    excess = np.abs(got - ref) - bar
    worst = np.unravel_index(np.argmax(excess), excess.shape)
    assert excess[worst] <= 0.0, (f"element {worst} of the compared block: |{got[worst]} - {ref[worst]}| exceeds the "
                                  f"accumulation allowance {bar[worst]:.3e}")
    err = rel_fro(got, ref)
    assert err < tol
    parts = {}
    if extracted is not None and len(extracted):
        R = np.arange(ref.shape[0]) if rows is None else np.asarray(rows)
        Cc = np.arange(ref.shape[1]) if cols is None else np.asarray(cols)
        if g.strategy == inputs.IHT_OE_ROW:
            m = np.isin(R, extracted)
            split = ((got[m], ref[m]), (got[~m], ref[~m]))
        elif g.strategy == inputs.IHT_OE_COL:
            m = np.isin(Cc, extracted)
            split = ((got[:, m], ref[:, m]), (got[:, ~m], ref[:, ~m]))
        else:
            split = ()
        for name, (a, b) in zip(("extracted", "residual"), split):
            if a.size:
                parts[name] = rel_fro(a, b)
                assert parts[name] < tol, name
    return err, parts, float((np.abs(got - ref) / bar).max())


def rand_bits(rng, shape, scale=1.0):
    x = torch.from_numpy((rng.standard_normal(shape) * scale).astype(np.float32))
    return x.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def stored(bits_ok, k_contig, pad=0):
    """bits_ok is logical [outer, K]; return the array as stored (optionally with ld > width)."""
    a = bits_ok if k_contig else np.ascontiguousarray(bits_ok.T)
    pad += (-(a.shape[1] + pad)) % 8          # the ABI wants ld to be a multiple of 8 elements
    if pad:
        wide = np.zeros((a.shape[0], a.shape[1] + pad), dtype=a.dtype)
        wide[:, :a.shape[1]] = a
        return wide, a.shape[1]
    return a, a.shape[1]


# ----------------------------------------------------------------------------- quantisers

@pytest.mark.parametrize("k_contig", [True, False])
@pytest.mark.parametrize("b", [0, 32, 64, 128, 256])
def test_iht_quantize_bit_exact(ah, b, k_contig):
    rng = np.random.default_rng(100 + b + int(k_contig))
    for outer, K, pad, masks in ((77, 3 * max(b, 32), 0, False), (300, 4 * max(b, 32), 8, True),
                                 (130, 1280 if b != 256 else 1280, 0, True), (1, max(b, 32), 0, False)):
        if b and K % b:
            K = (K // b + 1) * b
        say("iht_quantize", dict(b=b, k_contig=k_contig, outer=outer, K=K, pad=pad, masks=masks))
        logical = rand_bits(rng, (outer, K))
        logical[rng.integers(0, outer), :] = 0                      # an all-zero row
        logical[:, 5] = rand_bits(rng, (outer,), 60.0)              # an outlier channel
        arr, width = stored(logical, k_contig, pad)
        t = torch.from_numpy(arr.view(np.int16)).cuda()
        x = ah.Operand(t[:, :width], k_contig)
        zo = zk = zo_d = zk_d = None
        if masks:
            zo = (rng.random(outer) < 0.1).astype(np.uint8)
            zk = (rng.random(K) < 0.05).astype(np.uint8)
            zo_d, zk_d = torch.from_numpy(zo).cuda(), torch.from_numpy(zk).cuda()
        codes, scales = ah.adahop_iht_quantize(x, b, zo_d, zk_d)
        torch.cuda.synchronize()
        rc, rs = orc.iht_quantize(arr[:, :width], k_contig, b, zo, zk)
        assert np.array_equal(host(scales), rs)
        assert np.array_equal(host(codes), rc)


@pytest.mark.parametrize("b", [256, 32])
def test_iht_quantize_k_strided_long_rows_bit_exact(ah, b):
    """K-strided operand with more than 256 tiles of 64 columns (the quantiser then starts its workgroups in groups of
    32 column tiles that walk the K-blocks together): a whole number of groups plus a narrower last one plus a ragged
    last tile, three K-blocks, with both masks."""
    outer, K = (8 * 32 + 21) * 64 + 40, 768
    rng = np.random.default_rng(300 + b)
    logical = rand_bits(rng, (outer, K))
    logical[:, 700] = rand_bits(rng, (outer,), 60.0)
    arr, width = stored(logical, False)
    x = ah.Operand(torch.from_numpy(arr.view(np.int16)).cuda()[:, :width], False)
    zo = (rng.random(outer) < 0.05).astype(np.uint8)
    zk = (rng.random(K) < 0.05).astype(np.uint8)
    say("iht_quantize, K-strided, long rows", dict(b=b, outer=outer, K=K))
    for masks in (False, True):
        codes, scales = ah.adahop_iht_quantize(x, b, torch.from_numpy(zo).cuda() if masks else None,
                                               torch.from_numpy(zk).cuda() if masks else None)
        torch.cuda.synchronize()
        rc, rs = orc.iht_quantize(arr[:, :width], False, b, zo if masks else None, zk if masks else None)
        assert np.array_equal(host(scales), rs)
        assert np.array_equal(host(codes), rc)


def test_quantize_mx_every_bf16_pattern_bit_exact(ah):
    """Every finite bf16 value, placed so that it lands in each E2M1 binade (and in the saturating
    range) relative to the block scale set by an anchor element."""
    allbits = np.arange(65536, dtype=np.uint32)
    vals = (allbits << 16).view(np.float32)
    keep = np.isfinite(vals) & (np.abs(vals) > 2.0 ** -100) & (np.abs(vals) < 2.0 ** 100)
    pats = allbits[keep].astype(np.uint16)
    v = vals[keep]
    e = np.floor(np.log2(np.abs(v))).astype(np.int64)
    blocks = []
    for shift in (-4, -3, -2, -1, 0, 1, 2):      # anchor = 2^(e - shift + 2): value/X falls in binade `shift`
        anchor = np.exp2((e - shift + 2).astype(np.float64)).astype(np.float32)
        anchor_bits = (anchor.view(np.uint32) >> 16).astype(np.uint16)
        blk = np.zeros((len(pats), 32), dtype=np.uint16)
        blk[:, 0] = anchor_bits
        blk[:, 7] = pats
        blk[:, 30] = pats ^ 0x8000
        blocks.append(blk)
    # value itself is the block maximum (exercises saturation: value / X in [4, 8))
    blk = np.zeros((len(pats), 32), dtype=np.uint16)
    blk[:, 3] = pats
    blocks.append(blk)
    logical = np.concatenate(blocks, axis=0)
    say("quantize_mx all bf16 patterns", logical.shape)
    for k_contig in (True, False):
        arr, width = stored(logical, k_contig)
        x = ah.Operand(torch.from_numpy(arr.view(np.int16)).cuda()[:, :width], k_contig)
        codes, scales = ah.adahop_quantize_mx(x)
        torch.cuda.synchronize()
        rc, rs = orc.quantize_mx(arr[:, :width], k_contig)
        assert np.array_equal(host(scales), rs)
        assert np.array_equal(host(codes), rc)


# ----------------------------------------------------------------------------- FOID

@pytest.mark.parametrize("k_contig", [True, False])
@pytest.mark.parametrize("axis", [0, 1])
def test_foid_topk_bit_exact(ah, axis, k_contig):
    rng = np.random.default_rng(7 + axis * 2 + int(k_contig))
    for outer, K, ks in ((200, 96, (0, 1, 7, 96)), (4100, 160, (41, 160)), (40, 2080, (13,)), (28672, 64, (574, 72))):
        logical = rand_bits(rng, (outer, K))
        dim = outer if axis == 0 else K
        hot = rng.permutation(dim)[:5]
        if axis == 0:
            logical[hot, :] = rand_bits(rng, (5, K), 30.0)
        else:
            logical[:, hot] = rand_bits(rng, (outer, 5), 30.0)
        dup = rng.permutation(dim)[:6]              # exact score ties: identical sample windows
        if axis == 0:
            logical[dup[1::2], :64] = logical[dup[0::2], :64]
        else:
            logical[:64, dup[1::2]] = logical[:64, dup[0::2]]
        arr, width = stored(logical, k_contig)
        x = ah.Operand(torch.from_numpy(arr.view(np.int16)).cuda()[:, :width], k_contig)
        ref_scores = orc.foid_scores(arr[:, :width], k_contig, axis)
        for k in ks:
            k = min(k, dim)
            say("foid_topk", dict(axis=axis, k_contig=k_contig, outer=outer, K=K, k=k))
            idx, mask, scores = ah.adahop_foid_topk(x, axis, k)
            torch.cuda.synchronize()
            assert np.array_equal(host(scores).view(np.uint32), ref_scores.view(np.uint32))
            ridx, rmask = orc.topk(ref_scores, k)
            assert np.array_equal(host(idx), ridx)
            assert np.array_equal(host(mask), rmask)


def test_topk_selection_paths_bit_exact(ah):
    """The exact top-k on score vectors chosen to take each way through the selection kernel: a short candidate list
    behind the threshold from the thread maxima; more candidates than the list holds (all scores equal, or equal in
    their upper 16 bits); k above the number of threads; fewer key-owning threads than k; k = dim; dims just above
    and below the list size; well separated outliers, with k at, below and above their number (the select stops
    early, also with a threshold below that of the candidate list).  Scores come from rows that are constant except for two entries, so that their fp32
    variance scores can be steered: x = (a, -a, 0, ...) scores 2 a^2 exactly."""
    rng = np.random.default_rng(77)
    cases = []
    for dim, ks, kind in ((28672, (287, 574, 1, 1024, 1025, 3000, 28672), "random"), (28672, (287, 5000), "equal"),
                          (28672, (300,), "two-level"), (4097, (41, 4097), "random"), (4096, (41, 1500), "random"),
                          (9000, (90, 1100), "few-big"), (32768, (328, 640), "random"), (1090, (1089, 1024, 70), "random"),
                          (16384, (164, 100, 165, 200), "separated"), (3000, (30, 29, 31), "separated"),
                          (4100, (1000, 820, 41), "random"), (8191, (81, 1024), "random"), (32767, (327,), "separated")):
        if kind == "random":
            a = np.abs(rng.standard_normal(dim)).astype(np.float32) + 0.5
        elif kind == "equal":
            a = np.full(dim, 1.5, dtype=np.float32)
        elif kind == "separated":            # 1 % of the scores far above the rest and spread over several leading
            a = rng.uniform(0.5, 1.5, dim).astype(np.float32)  # digits: the select stops at its first or second digit
            big = rng.permutation(dim)[:ks[0]]
            a[big] = rng.uniform(8.0, 64.0, ks[0]).astype(np.float32)
        elif kind == "two-level":            # upper 16 bits of every score equal; they differ further down
            a = (1.0 + rng.integers(0, 60, dim) * 2.0 ** -9).astype(np.float32)
        else:                                # a handful of large scores among many equal small ones
            a = np.full(dim, 0.25, dtype=np.float32)
            a[rng.permutation(dim)[:50]] = rng.uniform(8.0, 16.0, 50).astype(np.float32)
        cases.append((dim, ks, kind, a))
    for dim, ks, kind, a in cases:
        x = np.zeros((dim, 64), dtype=np.float32)
        x[:, 0], x[:, 1] = a, -a
        bits = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        op = ah.Operand.from_bits(bits, True)
        ref_scores = orc.foid_scores(bits, True, 0)
        for k in ks:
            say("top-k paths", dict(dim=dim, k=k, kind=kind))
            idx, mask, scores = ah.adahop_foid_topk(op, 0, k)
            torch.cuda.synchronize()
            assert np.array_equal(host(scores).view(np.uint32), ref_scores.view(np.uint32))
            ridx, rmask = orc.topk(ref_scores, k)
            assert np.array_equal(host(idx), ridx)
            assert np.array_equal(host(mask), rmask)


def test_topk_score_scratch_at_odd_addresses(ah):
    """Score scratch that is only 4-byte aligned, which is all the interface asks for (the selection kernel then
    loads and clears element by element), on sizes with a ragged last wave."""
    import ctypes as C
    rng = np.random.default_rng(78)
    for dim, k in ((5000, 50), (28671, 287), (130, 7)):
        bits = rand_bits(rng, (dim, 64))
        bits[rng.permutation(dim)[:k // 2], :] = rand_bits(rng, (k // 2, 64), 30.0)
        op = ah.Operand.from_bits(bits, True)
        ref_scores = orc.foid_scores(bits, True, 0)
        ridx, rmask = orc.topk(ref_scores, k)
        for s_off, m_off in ((1, 0), (3, 8), (2, 0)):
            say("top-k, scratch at odd addresses", dict(dim=dim, k=k, scores_offset=4 * s_off, mask_offset=m_off))
            scores = torch.zeros(dim + 8, dtype=torch.float32, device="cuda")
            mask = torch.full((dim + 16,), 7, dtype=torch.uint8, device="cuda")
            idx = torch.zeros(k, dtype=torch.int32, device="cuda")
            rc = ah.lib().adahop_foid_topk(C.byref(op.c()), 0, k, idx.data_ptr(), mask.data_ptr() + m_off,
                                           scores.data_ptr() + 4 * s_off, torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            assert rc == 0
            assert np.array_equal(host(scores)[s_off:s_off + dim].view(np.uint32), ref_scores.view(np.uint32))
            assert np.array_equal(host(idx), ridx)
            m = host(mask)
            assert np.array_equal(m[m_off:m_off + dim], rmask)
            assert (m[:m_off] == 7).all() and (m[m_off + dim:] == 7).all()      # nothing written around the mask


# ----------------------------------------------------------------------------- MXFP4 product

@pytest.mark.parametrize("shape", [(32, 32, 64), (128, 128, 256), (200, 136, 96), (257, 129, 32), (64, 384, 1056),
                                   (256, 256, 256), (512, 512, 512), (768, 1280, 2304), (2304, 512, 256),
                                   (300, 520, 512), (700, 256, 768), (256, 333, 1024)])
def test_gemm_mx_matches_emulation(ah, shape):
    M, N, K = shape
    rng = np.random.default_rng(M + N + K)
    a_codes = rng.integers(0, 256, size=(M, K // 2), dtype=np.uint8)
    b_codes = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    a_scales = rng.integers(117, 137, size=(M, K // 32), dtype=np.uint8)
    b_scales = rng.integers(100, 120, size=(N, K // 32), dtype=np.uint8)
    say("gemm_mx", shape)
    C = ah.adahop_gemm_mx(*(torch.from_numpy(t).cuda() for t in (a_codes, a_scales, b_codes, b_scales)))
    torch.cuda.synchronize()
    ref = orc.mx_gemm(a_codes, a_scales, b_codes, b_scales)
    err = rel_fro(host(C), ref)
    say("  rel_fro", err)
    assert err < 1e-3
    assert err < 1e-5        # what the arithmetic predicts; a layout mistake gives O(1)


def test_gemm_mx_single_nonzero_probes_operand_layout(ah):
    """One nonzero code per operand at a time: the product must land in exactly one output element
    with exactly the right value, for positions covering every lane group, nibble and scale slot."""
    M = N = 64
    K = 128
    for (m, ka, code_a, sa), (n, code_b, sb) in [((0, 0, 7, 127), (0, 2, 127)), ((33, 37, 3, 130), (5, 6, 120)),
                                                 ((63, 127, 15, 125), (63, 9, 129)), ((17, 64, 5, 127), (40, 12, 127)),
                                                 ((8, 95, 1, 127), (31, 1, 126))]:
        a_codes = np.zeros((M, K // 2), np.uint8)
        b_codes = np.zeros((N, K // 2), np.uint8)
        a_scales = np.full((M, K // 32), 127, np.uint8)
        b_scales = np.full((N, K // 32), 127, np.uint8)
        a_codes[m, ka // 2] = code_a << (4 * (ka & 1))
        b_codes[n, ka // 2] = code_b << (4 * (ka & 1))
        a_scales[m, ka // 32] = sa
        b_scales[n, ka // 32] = sb
        say("gemm_mx probe", (m, n, ka))
        C = host(ah.adahop_gemm_mx(*(torch.from_numpy(t).cuda() for t in (a_codes, a_scales, b_codes, b_scales))))
        ref = orc.mx_gemm(a_codes, a_scales, b_codes, b_scales)
        assert np.count_nonzero(ref) == 1
        assert np.array_equal(C.astype(np.float64), ref)


# ----------------------------------------------------------------------------- whole path

def run_whole(ah, g, rows=None, cols=None, given_idx=None, tol=1e-3):
    A, B = dev_op(ah, g.A), dev_op(ah, g.B)
    idx_d = None if given_idx is None else torch.from_numpy(np.asarray(given_idx, dtype=np.int32)).cuda()
    out = ah.adahop_gemm(A, B, g.strategy, g.iht_block, g.k, idx=idx_d)
    torch.cuda.synchronize()
    ref = orc.adahop_gemm(g.A.bits, g.A.k_contig, g.B.bits, g.B.k_contig, g.strategy, g.iht_block, g.k,
                          idx=given_idx, rows=rows, cols=cols)
    if g.strategy >= inputs.IHT_OE_ROW and g.k > 0:
        got_idx = np.sort(host(out["idx"]))
        assert np.array_equal(got_idx, ref["idx"]), "extraction indices differ"
        mask = np.zeros(out["mask"].numel(), np.uint8)
        mask[ref["idx"]] = 1
        assert np.array_equal(host(out["mask"]), mask)
    for name in ("a_scales", "b_scales", "a_codes", "b_codes"):
        assert np.array_equal(host(out[name]), ref[name]), name
    C = out["C"]
    if rows is not None:
        C = C[torch.from_numpy(np.asarray(rows, dtype=np.int64)).cuda()]
    if cols is not None:
        C = C[:, torch.from_numpy(np.asarray(cols, dtype=np.int64)).cuda()]
    got = host(C)
    err, parts, used = check_c(got, ref["C"], g, rows, cols, ref["idx"] if g.k > 0 else None, tol)
    exact = orc.exact_gemm(g.A.bits, g.A.k_contig, g.B.bits, g.B.k_contig, rows=rows, cols=cols)
    q = rel_fro(got, exact)
    say(f"  {g.name} {inputs.STRATEGY_NAMES[g.strategy]} b={g.iht_block} k={g.k} shape={g.shape}: "
        f"vs oracle {err:.3e} " + " ".join(f"{n} {v:.3e}" for n, v in parts.items()) +
        f", worst element at {used:.3f} of its allowance, vs exact product {q:.3e} "
        f"({got.shape[0]} x {got.shape[1]} elements compared)")
    return err, q


def test_config0_iht_and_none(ah):
    g = inputs.config0()[0]
    say("config0 IHT")
    _, q_iht = run_whole(ah, g)
    g.strategy = inputs.NONE
    say("config0 none")
    _, q_none = run_whole(ah, g)
    assert q_iht < q_none                      # CN pair: the transform must help (paper Sec. 3.2)


LAYOUTS = {"fwd": (True, True), "dgrad": (True, False), "wgrad": (False, False)}


@pytest.mark.parametrize("kind", ["fwd", "dgrad", "wgrad"])
@pytest.mark.parametrize("strategy", [inputs.IHT, inputs.IHT_OE_ROW, inputs.IHT_OE_COL, inputs.IHT_OE_K])
def test_whole_path_small_all_layouts(ah, strategy, kind):
    """Ragged M and N spanning several workgroup tiles; K spans several transform blocks."""
    M, N, K, b = 328, 200, 512, 128
    a_kc, b_kc = LAYOUTS[kind]
    A_log = inputs.matrix(M, K, 1.0, 50, row_outliers=(5, 100.0, 100.0), col_outliers=(6, 50.0, 50.0))
    B_log = inputs.matrix(N, K, 0.02, 51, row_outliers=(4, 30.0, 30.0))
    A = inputs.Operand(A_log if a_kc else np.ascontiguousarray(A_log.T), a_kc)
    B = inputs.Operand(B_log if b_kc else np.ascontiguousarray(B_log.T), b_kc)
    k = {inputs.IHT: 0, inputs.IHT_OE_ROW: 9, inputs.IHT_OE_COL: 7, inputs.IHT_OE_K: 21}[strategy]
    g = inputs.Gemm(f"small.{kind}", A, B, strategy, b, k)
    say("whole path", kind, inputs.STRATEGY_NAMES[strategy])
    run_whole(ah, g)
    if k:
        given = np.random.default_rng(5).permutation({inputs.IHT_OE_ROW: M, inputs.IHT_OE_COL: N,
                                                      inputs.IHT_OE_K: K}[strategy])[:k].astype(np.int32)
        say("whole path, caller-chosen indices", kind, inputs.STRATEGY_NAMES[strategy])
        run_whole(ah, g, given_idx=given)


@pytest.mark.parametrize("strategy,k", [(inputs.IHT, 0), (inputs.IHT_OE_K, 5), (inputs.IHT_OE_K, 70),
                                        (inputs.IHT_OE_ROW, 6), (inputs.IHT_OE_COL, 3)])
@pytest.mark.parametrize("M,N", [(768, 512), (840, 600)])
def test_whole_path_tile_aligned_shape(ah, strategy, k, M, N):
    """K a multiple of 256: the tiled GEMM kernel (LDS-staged, K-channel part fused) takes the whole 256x256
    tiles, the bounds-checked kernel the ragged edges of the second shape."""
    K = 1024
    A = inputs.Operand(inputs.matrix(M, K, 1.0, 60, row_outliers=(4, 100.0, 100.0), col_outliers=(5, 50.0, 50.0)), True)
    B = inputs.Operand(np.ascontiguousarray(inputs.matrix(N, K, 0.02, 61).T), False)
    g = inputs.Gemm("tiled", A, B, strategy, 256, k)
    say("tile-aligned whole path", inputs.STRATEGY_NAMES[strategy], k)
    run_whole(ah, g)


@pytest.mark.parametrize("strategy,k", [(inputs.IHT, 0), (inputs.IHT_OE_K, 5), (inputs.IHT_OE_K, 70), (inputs.IHT_OE_K, 150),
                                        (inputs.IHT_OE_ROW, 9)])
@pytest.mark.parametrize("M,N", [(4352, 4096), (4608, 3840)])
def test_more_tiles_than_compute_units(ah, strategy, k, M, N):
    """272 and 270 tiles of 256x256: some workgroups of the persistent kernel walk two tiles, with the stage pipeline
    running from one into the next (one, two and three gathered-bf16 stages per tile for the three OE-K ranks; an odd
    and an even number of stages per tile; a tile count that is and is not a multiple of 8).  C on a seeded sample of
    rows and columns that covers every tile row and tile column."""
    K = 768
    A = inputs.Operand(inputs.matrix(M, K, 1.0, 62, row_outliers=(6, 100.0, 100.0), col_outliers=(5, 50.0, 50.0)), True)
    B = inputs.Operand(inputs.matrix(N, K, 0.02, 63), True)
    g = inputs.Gemm("manytiles", A, B, strategy, 256, k)
    rng = np.random.default_rng(M + k)
    rows = np.unique(np.concatenate([np.arange(0, M, 256) + rng.integers(0, 256, M // 256), rng.integers(0, M, 16)]))
    cols = np.unique(np.concatenate([np.arange(0, N, 256) + rng.integers(0, 256, N // 256), rng.integers(0, N, 48)]))
    if strategy == inputs.IHT_OE_ROW:
        sel, _ = orc.foid_topk(A.bits, True, 0, k)
        rows = np.unique(np.concatenate([rows, sel[:4]]))
    say("more tiles than compute units", inputs.STRATEGY_NAMES[strategy], k, (M, N, K))
    run_whole(ah, g, rows=rows.astype(np.int32), cols=cols.astype(np.int32))


@pytest.mark.parametrize("M,N,K", [(4096, 8192, 768), (2048, 16384, 1024), (16384, 4096, 768), (8192, 8192, 768),
                                   (2304, 8192, 768)])
def test_every_order_of_the_tile_walk_gives_the_same_bits(ah, M, N, K):
    """The persistent 256 x 256 kernel walks its tiles in bands of A or of B, in XCD-contiguous runs or swept over the
    other operand (chosen by shape: the sweep only for operands larger than the Infinity Cache).  Forced each way on
    512 and 1024 tiles (two and four rounds of the 256 workgroups; two bands; two groups of 32 minor tiles; a shape
    whose sweep along B cannot run and falls back), every tile must be computed exactly once, with the same bits, and
    agree with the oracle on a sample that touches every tile."""
    rng = np.random.default_rng(M + N + K)
    a_codes = rng.integers(0, 256, size=(M, K // 2), dtype=np.uint8)
    b_codes = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    a_scales = rng.integers(117, 137, size=(M, K // 32), dtype=np.uint8)
    b_scales = rng.integers(100, 120, size=(N, K // 32), dtype=np.uint8)
    dev = [torch.from_numpy(t).cuda() for t in (a_codes, a_scales, b_codes, b_scales)]
    say("tile walk orders", (M, N, K))
    out = {}
    try:
        for which in (0, 3, 4, 5, 6):
            ah.adahop_debug_force_gemm_kernel(which)
            C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
            ah.adahop_gemm_mx(*dev, Cout=C)
            torch.cuda.synchronize()
            out[which] = host(C)
    finally:
        ah.adahop_debug_force_gemm_kernel(0)
    for which in (0, 4, 5, 6):
        assert np.array_equal(out[3].view(np.uint32), out[which].view(np.uint32)), which
    rows = np.arange(0, M, 256) + rng.integers(0, 256, M // 256)
    cols = np.arange(0, N, 256) + rng.integers(0, 256, N // 256)
    ref = orc.mx_gemm(a_codes[rows], a_scales[rows], b_codes[cols], b_scales[cols])
    err = rel_fro(out[4][np.ix_(rows, cols)], ref)
    say("  rel_fro", err)
    assert err < 1e-5


@pytest.mark.parametrize("a_kc,b_kc", [(True, True), (True, False), (False, True)])
@pytest.mark.parametrize("K,k", [(4096, 41), (8192, 5), (8192, 200)])
def test_oe_k_channels_copied_by_the_quantiser(ah, a_kc, b_kc, K, k):
    """K-contiguous operands whose K is a whole number of 4096-element passes: the quantiser that the whole path runs
    also copies the extracted channels out, where otherwise a gather kernel does.  With the indices handed back in,
    the path takes the gather kernels: both must give the same C bit for bit (same copy, same summation order), and
    the oracle's on a sample of rows.  (Operands with one K-strided side mix the two routes in one product.)"""
    M, N, b = 304, 264, 128
    A_log = inputs.matrix(M, K, 1.0, 70 + k, col_outliers=(max(k // 2, 3), 40.0, 80.0))
    B_log = inputs.matrix(N, K, 0.02, 71 + k)
    A = inputs.Operand(A_log if a_kc else np.ascontiguousarray(A_log.T), a_kc)
    B = inputs.Operand(B_log if b_kc else np.ascontiguousarray(B_log.T), b_kc)
    g = inputs.Gemm("kcopy", A, B, inputs.IHT_OE_K, b, k)
    say("K-channels copied by the quantiser", (M, N, K), k, a_kc, b_kc)
    rows = np.arange(0, M, 7, dtype=np.int32)
    run_whole(ah, g, rows=rows)
    dA, dB = dev_op(ah, A), dev_op(ah, B)
    first = ah.adahop_gemm(dA, dB, inputs.IHT_OE_K, b, k)
    c_first, idx = host(first["C"]), first["idx"].clone()
    second = ah.adahop_gemm(dA, dB, inputs.IHT_OE_K, b, k, idx=idx)
    assert np.array_equal(c_first, host(second["C"]))


def test_oe_k_zero_equals_iht(ah):
    g = inputs.config0()[0]
    A, B = dev_op(ah, g.A), dev_op(ah, g.B)
    say("k=0 equals IHT")
    c_iht = host(ah.adahop_gemm(A, B, inputs.IHT, 32)["C"])
    for s in (inputs.IHT_OE_ROW, inputs.IHT_OE_COL, inputs.IHT_OE_K):
        assert np.array_equal(host(ah.adahop_gemm(A, B, s, 32, 0)["C"]), c_iht)


@pytest.mark.parametrize("M,N,K,k_row,k_col,k_k", [(152, 88, 160, 37, 5, 19), (520, 264, 1088, 300, 70, 33)])
def test_oe_gemm_bf16_standalone(ah, M, N, K, k_row, k_col, k_k):
    """Second term of Eq. 7 / Eq. 8 / the K-channel form alone; the larger case needs several row-tile groups
    and several K slices of the row / column kernel."""
    rng = np.random.default_rng(3)
    for a_kc, b_kc in LAYOUTS.values():
        A_log, B_log = rand_bits(rng, (M, K)), rand_bits(rng, (N, K), 0.05)
        A = inputs.Operand(A_log if a_kc else np.ascontiguousarray(A_log.T), a_kc)
        B = inputs.Operand(B_log if b_kc else np.ascontiguousarray(B_log.T), b_kc)
        dA, dB = dev_op(ah, A), dev_op(ah, B)
        for kind, dim, k in ((inputs.IHT_OE_ROW, M, k_row), (inputs.IHT_OE_COL, N, k_col), (inputs.IHT_OE_K, K, k_k)):
            sel = np.sort(rng.permutation(dim)[:k]).astype(np.int32)
            base = rng.standard_normal((M, N)).astype(np.float32)
            C = torch.from_numpy(base.copy()).cuda()
            say("oe_gemm_bf16", dict(a_kc=a_kc, b_kc=b_kc, kind=kind, k=k))
            ah.adahop_oe_gemm_bf16(dA, dB, kind, torch.from_numpy(sel).cuda(), C)
            torch.cuda.synchronize()
            want = base.astype(np.float64)
            if kind == inputs.IHT_OE_ROW:
                want[sel, :] = orc.bf16_gemm(A.bits, a_kc, B.bits, b_kc, rows=sel)
            elif kind == inputs.IHT_OE_COL:
                want[:, sel] = orc.bf16_gemm(A.bits, a_kc, B.bits, b_kc, cols=sel)
            else:
                want += orc.bf16_gemm(A.bits, a_kc, B.bits, b_kc, ksel=sel)
            assert rel_fro(host(C), want) < 1e-5


# ----------------------------------------------------------------------------- pattern detection (App. A)

@pytest.mark.parametrize("shape", [(600, 1056), (256, 512), (1030, 288)])
@pytest.mark.parametrize("k_contig", [True, False])
def test_detect_pattern_matches_oracle(ah, shape, k_contig):
    """CV figures to 1e-9 relative and the class exactly, for plain, row-outlier and channel-outlier tensors in both
    storage orders; sizes span several 256 x 512 blocks with ragged tails."""
    outer, K = shape
    for seed, kw in ((1, {}), (2, dict(row_outliers=(5, 100.0, 100.0))), (3, dict(col_outliers=(6, 50.0, 50.0)))):
        logical = inputs.matrix(outer, K, 1.0, 9000 + seed, **kw)
        arr, width = stored(logical, k_contig)
        say("detect_pattern", shape, k_contig, kw)
        x = ah.Operand(torch.from_numpy(arr.view(np.int16)).cuda()[:, :width], k_contig)
        p, st = ah.adahop_detect_pattern(x)
        torch.cuda.synchronize()
        want_p, want_st = orc.detect_pattern(logical, True)
        assert int(host(p)[0]) == want_p
        assert np.allclose(host(st), want_st, rtol=1e-9, atol=1e-12), (host(st), want_st)
