"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.

Bar: codes, dialect IDs, exponents and dequantized values are bit-exact.  The
only tolerated difference is a dialect choice between two candidates whose
oracle scores agree to 1e-6 relative; such a block is reported (and its codes
are checked against the oracle run with the GPU's choice).  All scores are
exact integers on the GPU, so no such block is expected.
"""

import warnings

import numpy as np
import pytest
import torch

from fb4_inputs import DEFAULT_FORMATBOOK, E2M1_X2_FORMATBOOK, synth
from oracle import fb4_oracle as O

pytestmark = pytest.mark.gpu

SELECTORS = [("lut8", 1, 8), ("lut32", 1, 32), ("sse", 0, 8), ("lut16", 1, 16)]


@pytest.fixture(scope="module")
def F():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2603_02883_amd as F
    return F


@pytest.fixture(scope="module")
def luts(F):
    l = F.fb4_build_luts(DEFAULT_FORMATBOOK)
    yield l
    l.free()


def dev_bits(bits):
    return synth.bits_to_bf16(bits, "cuda")


def host_u8(t):
    return t.cpu().numpy()


def host_u16(t):
    return t.cpu().numpy().view(np.uint16)


def compare_quant(fbk, x_bits, cg, mg, cr, mr, sel, g, flags=0, token_group=None, sub=None, what="", block=32):
    """cg/mg from the GPU, cr/mr from the oracle (numpy)."""
    assert cg.shape == cr.shape and mg.shape == mr.shape
    if np.array_equal(mg, mr) and np.array_equal(cg, cr):
        return 0
    assert np.array_equal(mg >> 8, mr >> 8), what + ": shared exponents differ"
    bad = np.argwhere((mg & 0xFF) != (mr & 0xFF))
    ties = 0
    for r, b in bad[:64]:
        blk = x_bits[r, block * b:block * b + block]
        sub8 = None if (token_group is None or token_group[r] < 0) else sub[token_group[r]]
        cand, scores, did, e = O.block_scores(fbk, blk, selector=sel, num_groups=g, flags=flags, sub8=sub8)
        dg = int(mg[r, b] & 0xFF)
        assert dg in cand.tolist(), "%s: GPU chose DID %d outside the candidates at (%d,%d)" % (what, dg, r, b)
        sg = scores[cand.tolist().index(dg)]
        sr = scores[cand.tolist().index(int(mr[r, b] & 0xFF))]
        assert abs(sg - sr) <= 1e-6 * max(abs(sr), 1e-30), (
            "%s: dialect mismatch at row %d block %d: gpu %d (score %r) oracle %d (score %r)"
            % (what, r, b, dg, sg, int(mr[r, b] & 0xFF), sr))
        c1, _ = O.quantize(fbk[dg:dg + 1], blk[None, :], block=block, selector=O.SEL_SSE)
        assert np.array_equal(cg[r, block // 2 * b:block // 2 * (b + 1)], c1[0]), what + ": codes of a tied block"
        ties += 1
    assert len(bad) <= 64, what + ": %d dialect mismatches" % len(bad)
    if ties:
        warnings.warn("%s: %d argmin ties resolved differently (scores equal within 1e-6)" % (what, ties))
    ok = np.ones(mg.shape, dtype=bool)
    ok[bad[:, 0], bad[:, 1]] = False
    assert np.array_equal(cg.reshape(mg.shape + (block // 2,))[ok], cr.reshape(mr.shape + (block // 2,))[ok]), \
        what + ": codes differ"
    return ties


def run_quant(F, luts, x, sel, g, flags=0):
    o = F.opts(selector=sel, num_groups=g, flags=flags)
    c, m = F.fb4_quantize(luts, o, x)
    torch.cuda.synchronize()
    return host_u8(c), host_u16(m), c, m


# ----------------------------------------------------------------- configs
@pytest.mark.parametrize("name,sel,g", SELECTORS)
def test_cfg1_gaussian_outliers_full_tensor(F, luts, name, sel, g):
    x = synth.gaussian_outlier(device="cuda")                 # 1024 x 3072
    xb = synth.bf16_bits(x)
    cg, mg, c, m = run_quant(F, luts, x, sel, g)
    cr, mr = O.quantize(DEFAULT_FORMATBOOK, xb, selector=sel, num_groups=g)
    compare_quant(DEFAULT_FORMATBOOK, xb, cg, mg, cr, mr, sel, g, what="cfg1 " + name)
    for dt, odt in ((F.DTYPE_BF16, O.OUT_BF16), (F.DTYPE_F32, O.OUT_F32)):
        y = F.fb4_dequantize(luts, c, m, out_dtype=dt)
        torch.cuda.synchronize()
        yr = O.dequantize(DEFAULT_FORMATBOOK, cg, mg, out_dtype=odt)
        yg = synth.bf16_bits(y) if dt == F.DTYPE_BF16 else y.cpu().numpy().view(np.uint32)
        assert np.array_equal(yg, yr if dt == F.DTYPE_BF16 else yr.view(np.uint32))


@pytest.mark.parametrize("name,sel,g", SELECTORS)
def test_cfg2_vdit_activation_full_size(F, luts, name, sel, g):
    x = synth.vdit_activation(device="cuda")                  # 16384 x 3072, the benchmark workload
    xb = synth.bf16_bits(x)
    cg, mg, c, m = run_quant(F, luts, x, sel, g)
    cr, mr = O.quantize(DEFAULT_FORMATBOOK, xb, selector=sel, num_groups=g)
    compare_quant(DEFAULT_FORMATBOOK, xb, cg, mg, cr, mr, sel, g, what="cfg2 " + name)
    hist = np.bincount((mg & 0xFF).ravel(), minlength=32)
    assert (hist > 0).sum() >= 24                             # many dialects in use (App. B: no collapse)


@pytest.mark.parametrize("name,sel,g", [SELECTORS[0], SELECTORS[2]])
def test_cfg3_decomposition_of_salient_tokens(F, luts, name, sel, g):
    x = synth.vdit_activation(device="cuda")
    xb = synth.bf16_bits(x)
    sal = synth.salient_rows_from_attention(16384, frac=0.05, heads=24, seed=3, device="cuda")
    assert sal.size == 819 and (np.diff(sal) > 0).all()
    o = F.opts(selector=sel, num_groups=g)
    c1, m1 = F.fb4_quantize(luts, o, x)
    sal_d = torch.from_numpy(sal).cuda()
    c2, m2 = F.fb4_decompose(luts, o, x, c1, m1, sal_d)
    y = F.fb4_dequantize(luts, c1, m1, codes2=c2, meta2=m2, salient_rows=sal_d)
    yf = F.fb4_dequantize(luts, c1, m1, codes2=c2, meta2=m2, salient_rows=sal_d, out_dtype=F.DTYPE_F32)
    torch.cuda.synchronize()
    c1h, m1h = host_u8(c1), host_u16(m1)
    # oracle on the salient rows only (plane 1 of the other rows is covered by cfg2)
    c1r, m1r = O.quantize(DEFAULT_FORMATBOOK, xb[sal], selector=sel, num_groups=g)
    compare_quant(DEFAULT_FORMATBOOK, xb[sal], c1h[sal], m1h[sal], c1r, m1r, sel, g, what="cfg3 plane1 " + name)
    c2r, m2r = O.decompose(DEFAULT_FORMATBOOK, xb[sal], c1h[sal], m1h[sal], np.arange(sal.size, dtype=np.int32),
                           selector=sel, num_groups=g)
    compare_quant(DEFAULT_FORMATBOOK, xb[sal], host_u8(c2), host_u16(m2), c2r, m2r, sel, g, what="cfg3 plane2 " + name)
    # dequantize: salient rows = both planes, a sample of the other rows = plane 1
    rest = np.setdiff1d(np.arange(0, 16384, 37), sal)
    rows = np.sort(np.concatenate([sal, rest])).astype(np.int64)
    pos = np.searchsorted(rows, sal).astype(np.int32)
    yr = O.dequantize(DEFAULT_FORMATBOOK, c1h[rows], m1h[rows], codes2=host_u8(c2), meta2=host_u16(m2),
                      salient_rows=pos, out_dtype=O.OUT_BF16)
    assert np.array_equal(synth.bf16_bits(y)[rows], yr)
    yfr = O.dequantize(DEFAULT_FORMATBOOK, c1h[rows], m1h[rows], codes2=host_u8(c2), meta2=host_u16(m2),
                       salient_rows=pos, out_dtype=O.OUT_F32)
    assert np.array_equal(yf.cpu().numpy()[rows].view(np.uint32), yfr.view(np.uint32))
    # Sec. 3.3: the second plane shrinks the error of the salient rows
    xs = x[sal_d.long()].float()
    e1 = (xs - F.fb4_dequantize(luts, c1, m1, out_dtype=F.DTYPE_F32)[sal_d.long()]).pow(2).sum()
    e2 = (xs - yf[sal_d.long()]).pow(2).sum()
    assert float(e2) < 0.2 * float(e1)


@pytest.mark.parametrize("name,sel,g", SELECTORS)
def test_cfg4_seda_sub_formatbooks(F, luts, name, sel, g):
    x, comp = synth.mixture_activation(device="cuda")         # 16384 x 3072, 64 groups
    xb = synth.bf16_bits(x)
    sub = synth.seda_sub_formatbooks(DEFAULT_FORMATBOOK, n_groups=64, seed=4)
    tg = comp.copy()
    tg[::97] = -1                                             # a few rows on the full formatbook
    o = F.opts(selector=sel, num_groups=g)
    c, m = F.fb4_quantize_seda(luts, o, x, torch.from_numpy(tg).cuda(), torch.from_numpy(sub).cuda())
    torch.cuda.synchronize()
    cr, mr = O.quantize(DEFAULT_FORMATBOOK, xb, selector=sel, num_groups=g, token_group=tg, sub_formatbooks=sub)
    compare_quant(DEFAULT_FORMATBOOK, xb, host_u8(c), host_u16(m), cr, mr, sel, g, token_group=tg, sub=sub,
                  what="cfg4 " + name)
    did = host_u16(m) & 0xFF
    inside = (did[:, :, None] == sub[np.maximum(tg, 0)][:, None, :]).any(axis=2)
    assert inside[tg >= 0].all()                              # every DID from the row's sub-formatbook


def test_cfg5_large_ffn_activation_and_weight(F, luts):
    """The 65536 x 12288 tensor whole: every code, dialect and exponent of the online selector's first plane, the
    second plane of all 3276 salient rows, the decoded sum on those rows and on a band, and the exhaustive selector on
    a band of 4096 rows plus scattered rows (the oracle's exhaustive search over 805 M elements would take minutes)."""
    rows, cols = synth.CONFIG_SHAPES["cfg5"]
    x = synth.vdit_activation(rows=rows, cols=cols, seed=5, device="cuda", outlier_frac=0.01)
    sal = synth.salient_rows_from_attention(rows, frac=0.05, heads=24, seed=5, device="cuda", window=1024)
    assert sal.size == 3276
    sal_d = torch.from_numpy(sal).cuda()
    band = 8192                                                # rows per oracle call: bounds the host copies
    # ---- online selector, whole tensor, both planes in one pass (the second plane also as its own launch)
    o = F.opts(selector=1, num_groups=8)
    c1, m1, c2, m2 = F.fb4_quantize_decompose(luts, o, x, sal_d)
    c2b, m2b = F.fb4_decompose(luts, o, x, c1, m1, sal_d)
    y = F.fb4_dequantize(luts, c1, m1, codes2=c2, meta2=m2, salient_rows=sal_d)
    torch.cuda.synchronize()
    assert torch.equal(c2, c2b) and torch.equal(m2, m2b)
    del c2b, m2b
    for r0 in range(0, rows, band):
        xb = synth.bf16_bits(x[r0:r0 + band])
        cr, mr = O.quantize(DEFAULT_FORMATBOOK, xb, selector=1, num_groups=8)
        compare_quant(DEFAULT_FORMATBOOK, xb, host_u8(c1[r0:r0 + band]), host_u16(m1[r0:r0 + band]), cr, mr, 1, 8,
                      what="cfg5 lut8 rows %d.." % r0)
        if r0 == 3 * band:                                     # decode of one band, salient rows included
            in_band = (sal >= r0) & (sal < r0 + band)
            p0 = int(np.argmax(in_band))
            n_in = int(in_band.sum())
            c2h, m2h = host_u8(c2[p0:p0 + n_in]), host_u16(m2[p0:p0 + n_in])
            yr = O.dequantize(DEFAULT_FORMATBOOK, cr, mr, codes2=c2h, meta2=m2h, salient_rows=(sal[in_band] - r0).astype(np.int32))
            assert np.array_equal(synth.bf16_bits(y[r0:r0 + band]), yr)
            del yr
        del xb, cr, mr
    xs = synth.bf16_bits(x[sal_d.long()])
    c1s, m1s = host_u8(c1[sal_d.long()]), host_u16(m1[sal_d.long()])
    ident = np.arange(sal.size, dtype=np.int32)
    c2r, m2r = O.decompose(DEFAULT_FORMATBOOK, xs, c1s, m1s, ident, selector=1, num_groups=8)
    compare_quant(DEFAULT_FORMATBOOK, xs, host_u8(c2), host_u16(m2), c2r, m2r, 1, 8, what="cfg5 plane 2, all salient rows")
    yr = O.dequantize(DEFAULT_FORMATBOOK, c1s, m1s, codes2=c2r, meta2=m2r, salient_rows=ident)
    assert np.array_equal(synth.bf16_bits(y[sal_d.long()]), yr)
    # properties that hold at any size, checked on the whole tensor on the device
    mi = m1.view(torch.int16).to(torch.int32) & 0xFFFF
    assert int((mi & 0xFF).max()) < 32
    amax = x.view(rows, cols // 32, 32).abs().amax(dim=2).float()
    _, ex = torch.frexp(amax)                                  # amax = mant * 2^ex, mant in [0.5, 1)
    e = torch.where(amax > 0, ex - 1, torch.full_like(ex, -123)).clamp(-123, 127).to(torch.int32)
    assert torch.equal((mi >> 8) - 127, e)
    assert bool((y.float().abs() <= amax.repeat_interleave(32, dim=1) * 2.0).all())    # decoded values stay in range
    del c1, m1, c2, m2, y, mi, amax, ex, e
    torch.cuda.empty_cache()
    # ---- exhaustive selector: the band of rows 28672 .. 32767, scattered rows, and the salient rows' second plane
    o = F.opts(selector=0, num_groups=8)
    c1, m1 = F.fb4_quantize(luts, o, x)
    c2, m2 = F.fb4_decompose(luts, o, x, c1, m1, sal_d)
    torch.cuda.synchronize()
    rng = np.random.default_rng(55)
    sample = np.unique(np.concatenate([np.arange(28672, 32768), rng.integers(0, rows, 256), [0, rows - 1]])).astype(np.int64)
    idx = torch.from_numpy(sample).cuda()
    xs2 = synth.bf16_bits(x[idx])
    cr, mr = O.quantize(DEFAULT_FORMATBOOK, xs2, selector=0)
    compare_quant(DEFAULT_FORMATBOOK, xs2, host_u8(c1[idx]), host_u16(m1[idx]), cr, mr, 0, 8, what="cfg5 sse, 4354 rows")
    sub_sal = np.arange(0, sal.size, 8)                        # every eighth salient row
    sidx = torch.from_numpy(sal[sub_sal].astype(np.int64)).cuda()
    c1s, m1s = host_u8(c1[sidx]), host_u16(m1[sidx])
    c2r, m2r = O.decompose(DEFAULT_FORMATBOOK, xs[sub_sal], c1s, m1s, np.arange(sub_sal.size, dtype=np.int32), selector=0)
    pidx = torch.from_numpy(sub_sal).cuda()
    compare_quant(DEFAULT_FORMATBOOK, xs[sub_sal], host_u8(c2[pidx]), host_u16(m2[pidx]), c2r, m2r, 0, 8, what="cfg5 sse plane 2")
    del c1, m1, c2, m2
    torch.cuda.empty_cache()
    # the weight matrix of the layer goes through the same kernel (exhaustive selection, Sec. 3.3 / App. D)
    w = synth.weight_matrix(device="cuda")
    wb = synth.bf16_bits(w)
    cg, mg, _, _ = run_quant(F, luts, w, 0, 8)
    cr, mr = O.quantize(DEFAULT_FORMATBOOK, wb, selector=O.SEL_SSE)
    compare_quant(DEFAULT_FORMATBOOK, wb, cg, mg, cr, mr, 0, 8, what="cfg5 weight")


# -------------------------------------------------------------- edge cases
@pytest.mark.parametrize("name,sel,g", SELECTORS)
def test_degenerate_values(F, luts, name, sel, g):
    xb = synth.edge_case_tensor(cols=256)
    x = dev_bits(xb)
    o = F.opts(selector=sel, num_groups=g)
    c, m = F.fb4_quantize(luts, o, x)
    torch.cuda.synchronize()
    cr, mr = O.quantize(DEFAULT_FORMATBOOK, xb, selector=sel, num_groups=g)
    compare_quant(DEFAULT_FORMATBOOK, xb, host_u8(c), host_u16(m), cr, mr, sel, g, what="edge " + name)
    y = F.fb4_dequantize(luts, c, m)
    torch.cuda.synchronize()
    assert np.array_equal(synth.bf16_bits(y), O.dequantize(DEFAULT_FORMATBOOK, cr, mr))
    # decomposition of every row, including Inf/NaN/subnormal residuals
    sal = np.arange(xb.shape[0], dtype=np.int32)
    c2, m2 = F.fb4_decompose(luts, o, x, c, m, torch.from_numpy(sal).cuda())
    yy = F.fb4_dequantize(luts, c, m, codes2=c2, meta2=m2, salient_rows=torch.from_numpy(sal).cuda())
    torch.cuda.synchronize()
    c2r, m2r = O.decompose(DEFAULT_FORMATBOOK, xb, cr, mr, sal, selector=sel, num_groups=g)
    compare_quant(DEFAULT_FORMATBOOK, xb, host_u8(c2), host_u16(m2), c2r, m2r, sel, g, what="edge plane2 " + name)
    yyr = O.dequantize(DEFAULT_FORMATBOOK, cr, mr, codes2=c2r, meta2=m2r, salient_rows=sal)
    assert np.array_equal(synth.bf16_bits(yy), yyr)


@pytest.mark.parametrize("name,sel,g", SELECTORS)
def test_ragged_shapes_and_row_stride(F, luts, name, sel, g):
    rng = np.random.default_rng(12)
    for rows, cols, stride in ((37, 32 * 19, 32 * 19 + 8), (1, 32, 32), (5, 32 * 33, 32 * 40), (300, 64, 64)):
        big = synth.vdit_activation(rows=rows, cols=stride, seed=40 + cols % 7, device="cuda")
        x = big[:, :cols]                                     # non-contiguous view when stride > cols
        xb = synth.bf16_bits(big)[:, :cols]
        o = F.opts(selector=sel, num_groups=g)
        c, m = F.fb4_quantize(luts, o, x)
        torch.cuda.synchronize()
        cr, mr = O.quantize(DEFAULT_FORMATBOOK, np.ascontiguousarray(xb), selector=sel, num_groups=g)
        compare_quant(DEFAULT_FORMATBOOK, xb, host_u8(c), host_u16(m), cr, mr, sel, g,
                      what="ragged %dx%d %s" % (rows, cols, name))
        out = torch.full((rows, stride), 7.0, dtype=torch.bfloat16, device="cuda")
        F.fb4_dequantize(luts, c, m, out=out[:, :cols])
        torch.cuda.synchronize()
        assert np.array_equal(synth.bf16_bits(out)[:, :cols], O.dequantize(DEFAULT_FORMATBOOK, cr, mr))
        assert bool((out[:, cols:] == 7.0).all())             # padding untouched


@pytest.mark.parametrize("name,sel,g", SELECTORS)
def test_two_stage_selection(F, luts, name, sel, g):
    x = synth.vdit_activation(rows=512, cols=3072, seed=41, device="cuda")
    xb = synth.bf16_bits(x)
    cg, mg, _, _ = run_quant(F, luts, x, sel, g, flags=F.FLAG_TWO_STAGE)
    cr, mr = O.quantize(DEFAULT_FORMATBOOK, xb, selector=sel, num_groups=g, flags=O.FLAG_TWO_STAGE)
    compare_quant(DEFAULT_FORMATBOOK, xb, cg, mg, cr, mr, sel, g, flags=O.FLAG_TWO_STAGE, what="two-stage " + name)


@pytest.mark.parametrize("name,sel,g", SELECTORS)
def test_small_formatbooks(F, name, sel, g):
    x = synth.gaussian_outlier(rows=64, cols=1024, seed=42, device="cuda")
    xb = synth.bf16_bits(x)
    for fbk in (E2M1_X2_FORMATBOOK, DEFAULT_FORMATBOOK[:5], DEFAULT_FORMATBOOK[[0, 3, 9, 12, 17, 23, 31]]):
        l = F.fb4_build_luts(fbk)
        for flags in (0, F.FLAG_TWO_STAGE):
            cg, mg, c, m = run_quant(F, l, x, sel, g, flags=flags)
            cr, mr = O.quantize(fbk, xb, selector=sel, num_groups=g, flags=flags)
            compare_quant(fbk, xb, cg, mg, cr, mr, sel, g, flags=flags, what="small formatbook " + name)
        y = F.fb4_dequantize(l, c, m)
        torch.cuda.synchronize()
        assert np.array_equal(synth.bf16_bits(y), O.dequantize(fbk, cr, mr))
        l.free()


@pytest.mark.parametrize("name,sel,g", SELECTORS)
def test_seda_with_two_stage_decomposition_and_odd_tables(F, luts, name, sel, g):
    x, comp = synth.mixture_activation(rows=256, cols=32 * 21, seed=43, device="cuda", n_components=5)
    xb = synth.bf16_bits(x)
    sub = synth.seda_sub_formatbooks(DEFAULT_FORMATBOOK, n_groups=5, seed=43)
    sub[3] = [2, 2, 5, 9, 9, 30, 31, 31]                      # duplicates, ranges missing
    tg = comp.copy()
    tg[::9] = -1
    tg_d, sub_d = torch.from_numpy(tg).cuda(), torch.from_numpy(sub).cuda()
    for flags in (0, F.FLAG_TWO_STAGE):
        o = F.opts(selector=sel, num_groups=g, flags=flags)
        c, m = F.fb4_quantize_seda(luts, o, x, tg_d, sub_d)
        torch.cuda.synchronize()
        # the oracle wants ascending unique lists: give it the same sets, padded by repetition-free order
        cr = np.zeros_like(host_u8(c)); mr = np.zeros_like(host_u16(m))
        for grp in range(-1, 5):
            rows = np.nonzero(tg == grp)[0]
            if grp < 0:
                a, b = O.quantize(DEFAULT_FORMATBOOK, xb[rows], selector=sel, num_groups=g, flags=flags)
            else:
                a, b = _oracle_subset(xb[rows], sorted(set(sub[grp].tolist())), sel, g, flags)
            cr[rows], mr[rows] = a, b
        compare_quant(DEFAULT_FORMATBOOK, xb, host_u8(c), host_u16(m), cr, mr, sel, g, flags=flags,
                      what="seda odd %s flags %d" % (name, flags))
        # decomposition restricted to the same sub-formatbooks (App. D)
        sal = np.arange(0, 256, 7, dtype=np.int32)
        c2, m2 = F.fb4_decompose(luts, o, x, c, m, torch.from_numpy(sal).cuda(), token_group=tg_d,
                                 sub_formatbooks=sub_d)
        torch.cuda.synchronize()
        if flags == 0:
            keep = tg[sal] != 3                                # group 3's table is not a valid oracle input
            sal, c2, m2 = sal[keep], c2[torch.from_numpy(keep).cuda()], m2[torch.from_numpy(keep).cuda()]
            sub_ok = sub.copy()
            sub_ok[3] = sub[0]
            c2r, m2r = O.decompose(DEFAULT_FORMATBOOK, xb, host_u8(c), host_u16(m), sal, selector=sel,
                                   num_groups=g, token_group=tg, sub_formatbooks=sub_ok)
            compare_quant(DEFAULT_FORMATBOOK, xb[sal], host_u8(c2), host_u16(m2), c2r, m2r, sel, g,
                          what="seda decomposition " + name)


def _oracle_subset(xb, dids, sel, g, flags):
    """Oracle selection restricted to an arbitrary DID set: quantize with the
    formatbook cut down to those dialects and map the DIDs back."""
    fbk = DEFAULT_FORMATBOOK[dids]
    c, m = O.quantize(fbk, xb, selector=sel, num_groups=g, flags=flags)
    did = np.asarray(dids, dtype=np.uint16)[m & 0xFF]
    return c, (m & 0xFF00) | did


def test_seda_invalid_groups_and_dids_fall_back(F, luts):
    x = synth.gaussian_outlier(rows=32, cols=512, seed=44, device="cuda")
    xb = synth.bf16_bits(x)
    l5 = F.fb4_build_luts(DEFAULT_FORMATBOOK[:5])
    sub = np.array([[0, 1, 2, 3, 4, 4, 4, 4], [9, 9, 9, 9, 9, 9, 9, 9], [1, 40, 200, 3, 3, 3, 3, 3]], dtype=np.uint8)
    tg = np.array([0, 1, 2, 3, -1, -7, 99, 0] * 4, dtype=np.int32)
    o = F.opts(selector=F.SEL_LUT, num_groups=8)
    c, m = F.fb4_quantize_seda(l5, o, x, torch.from_numpy(tg).cuda(), torch.from_numpy(sub).cuda())
    torch.cuda.synchronize()
    fb5 = DEFAULT_FORMATBOOK[:5]
    cr = np.zeros_like(host_u8(c)); mr = np.zeros_like(host_u16(m))
    full = np.isin(tg, [1, 3, -1, -7, 99])                     # group 1 has no valid DID -> full formatbook
    cr[full], mr[full] = O.quantize(fb5, xb[full], selector=O.SEL_LUT)
    cr[tg == 0], mr[tg == 0] = O.quantize(fb5, xb[tg == 0], selector=O.SEL_LUT)   # all five dialects listed
    c13, m13 = O.quantize(fb5[[1, 3]], xb[tg == 2], selector=O.SEL_LUT)
    cr[tg == 2] = c13
    mr[tg == 2] = (m13 & 0xFF00) | np.array([1, 3], dtype=np.uint16)[m13 & 0xFF]
    assert np.array_equal(host_u16(m), mr) and np.array_equal(host_u8(c), cr)
    l5.free()


def test_empty_inputs_and_error_codes_with_a_real_handle(F, luts):
    o = F.opts()
    x = torch.zeros((0, 64), dtype=torch.bfloat16, device="cuda")
    c, m = F.fb4_quantize(luts, o, x)
    assert c.shape == (0, 32) and m.shape == (0, 2)
    x = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    c, m = F.fb4_quantize(luts, o, x)
    sal = torch.zeros(0, dtype=torch.int32, device="cuda")
    c2, m2 = F.fb4_decompose(luts, o, x, c, m, sal)
    assert c2.shape == (0, 32)
    y = F.fb4_dequantize(luts, c, m, codes2=c2, meta2=m2, salient_rows=sal)
    torch.cuda.synchronize()
    assert bool((y == 0).all())
    with pytest.raises(F.Fb4Error) as e:
        F.fb4_quantize(luts, o, torch.zeros((4, 48), dtype=torch.bfloat16, device="cuda"))
    assert e.value.code == F.ERR_UNSUPPORTED
    with pytest.raises(F.Fb4Error) as e:
        F.fb4_quantize(luts, F.opts(block=16, num_groups=32), x)        # more groups than elements
    assert e.value.code == F.ERR_INVALID_ARG
    # out-of-range salient rows leave their output rows untouched
    sal = torch.tensor([1, 77], dtype=torch.int32, device="cuda")
    c2 = torch.full((2, 32), 0x5A, dtype=torch.uint8, device="cuda")
    m2 = torch.zeros((2, 2), dtype=torch.int16, device="cuda")
    F.fb4_decompose(luts, o, x, c, m, sal, codes2=c2, meta2=m2)
    torch.cuda.synchronize()
    assert bool((c2[1] == 0x5A).all()) and bool((c2[0] == 0).all())


# ------------------------------------------------------------ block size 16
def _histogram_extreme_blocks(block, seed):
    """bf16 bit patterns [n][block] of blocks that drive the per-bin statistics of the matrix-core selectors to
    their limits: every element in one bin with the largest fractions (count = block, fraction sum at its
    maximum), every bin holding one element, alternating signs, a lone maximum over zeros, values just below
    and on bin and rounding boundaries, and exact ties between dialects."""
    rng = np.random.default_rng(seed)
    f32 = lambda v: (np.asarray(v, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)   # exact for these values
    blocks = []
    for top in (8.0, 9.5, 12.0, 15.9375):
        for scale in (1.0, 2.0 ** -9, 2.0 ** 20):
            # all other elements in ONE bin, with the largest fraction that bin can hold
            for b in (1, 2, 3, 7, 15, 16, 30, 31):
                hi = (b + 1) / 2.0
                v = np.full(block, hi, dtype=np.float64)
                # the largest bf16 below the bin's upper edge that is at most `top`
                cand = np.float32(min(hi, top))
                bits = cand.view(np.uint32) >> 16
                below = np.array([(int(bits) - 1) << 16], dtype=np.uint32).view(np.float32)[0]
                v[:] = below if hi <= top else top
                v[0] = top
                blocks.append(f32(v * scale))
                w = v.copy(); w[1::2] *= -1.0
                blocks.append(f32(w * scale))
            # one element per bin (block 32) / per second bin (block 16), smallest and largest fractions
            for frac in (0.0, 0.49609375):
                v = (np.arange(block) * (32 // block)) / 2.0 + frac
                v = np.minimum(v, top); v[-1] = top
                blocks.append(f32(rng.permutation(v) * scale))
            # a lone maximum over zeros; everything equal to the maximum; everything at a rounding boundary
            v = np.zeros(block); v[rng.integers(block)] = top; blocks.append(f32(v * scale))
            blocks.append(f32(np.full(block, top) * scale))
            for mid in (0.5, 1.5, 2.5, 4.5, 6.0, 7.5):
                v = np.full(block, mid); v[0] = top; blocks.append(f32(v * scale))
    return np.stack(blocks)


@pytest.mark.parametrize("block", [32, 16])
def test_matrix_core_selectors_at_the_limits_of_their_histograms(F, luts, block):
    """The exhaustive selector and the 32-group online selector score on the matrix cores from per-bin counts
    and fraction sums kept in byte fields: blocks that push every field to its limit, with and without the
    two-stage filter and SeDA lists, against the oracle."""
    fbk = DEFAULT_FORMATBOOK
    blk = _histogram_extreme_blocks(block, 91)
    per_row = 96 * 32 // block                       # blocks per row: rows of 3072 elements
    n = (len(blk) + per_row - 1) // per_row * per_row
    rng = np.random.default_rng(92)
    blk = np.concatenate([blk, blk[rng.integers(len(blk), size=n - len(blk))]])
    xb = blk[rng.permutation(n)].reshape(n // per_row, 3072)
    x = dev_bits(xb)
    sub = synth.seda_sub_formatbooks(fbk, n_groups=3, seed=93)
    tg = (np.arange(xb.shape[0]) % 4 - 1).astype(np.int32)      # -1, 0, 1, 2
    tg_d, sub_d = torch.from_numpy(tg).cuda(), torch.from_numpy(sub).cuda()
    for sel, g in ((F.SEL_SSE, 8),) + (((F.SEL_LUT, 32),) if block == 32 else ()):
        for flags in (0, F.FLAG_TWO_STAGE):
            o = F.opts(block=block, selector=sel, num_groups=g, flags=flags)
            c, m = F.fb4_quantize(luts, o, x)
            torch.cuda.synchronize()
            cr, mr = O.quantize(fbk, xb, block=block, selector=sel, num_groups=g, flags=flags)
            assert compare_quant(fbk, xb, host_u8(c), host_u16(m), cr, mr, sel, g, flags=flags, block=block,
                                 what="histogram limits sel %d flags %d" % (sel, flags)) == 0
            c, m = F.fb4_quantize_seda(luts, o, x, tg_d, sub_d)
            torch.cuda.synchronize()
            cr, mr = O.quantize(fbk, xb, block=block, selector=sel, num_groups=g, flags=flags, token_group=tg,
                                sub_formatbooks=sub)
            assert compare_quant(fbk, xb, host_u8(c), host_u16(m), cr, mr, sel, g, flags=flags, token_group=tg,
                                 sub=sub, block=block, what="histogram limits, SeDA, sel %d flags %d" % (sel, flags)) == 0


SELECTORS_B16 = [("lut8", 1, 8), ("lut16", 1, 16), ("sse", 0, 8)]


@pytest.mark.parametrize("name,sel,g", SELECTORS_B16)
def test_block16_all_entry_points(F, luts, name, sel, g):
    """Sec. 4.1 evaluates block sizes 16 and 32: the same pipeline with a scale and a dialect per 16 elements."""
    fbk = DEFAULT_FORMATBOOK
    for rows, cols, stride, seed in ((512, 3072, 3072, 46), (37, 16 * 21, 16 * 21 + 8, 47), (3, 16, 16, 48)):
        big = synth.vdit_activation(rows=rows, cols=stride, seed=seed, device="cuda")
        x = big[:, :cols]
        xb = np.ascontiguousarray(synth.bf16_bits(big)[:, :cols])
        for flags in (0, F.FLAG_TWO_STAGE):
            o = F.opts(block=16, selector=sel, num_groups=g, flags=flags)
            c, m = F.fb4_quantize(luts, o, x)
            torch.cuda.synchronize()
            assert m.shape == (rows, cols // 16)
            cr, mr = O.quantize(fbk, xb, block=16, selector=sel, num_groups=g, flags=flags)
            compare_quant(fbk, xb, host_u8(c), host_u16(m), cr, mr, sel, g, flags=flags, block=16,
                          what="block16 %dx%d %s flags %d" % (rows, cols, name, flags))
        # second plane of some rows, then both decodes
        sal = np.arange(0, rows, 3, dtype=np.int32)
        sal_d = torch.from_numpy(sal).cuda()
        c2, m2 = F.fb4_decompose(luts, o, x, c, m, sal_d)
        torch.cuda.synchronize()
        c2r, m2r = O.decompose(fbk, xb, host_u8(c), host_u16(m), sal, block=16, selector=sel, num_groups=g,
                               flags=flags)
        compare_quant(fbk, xb[sal], host_u8(c2), host_u16(m2), c2r, m2r, sel, g, flags=flags, block=16,
                      what="block16 plane2 " + name)
        for dt, odt in ((F.DTYPE_BF16, O.OUT_BF16), (F.DTYPE_F32, O.OUT_F32)):
            y = F.fb4_dequantize(luts, c, m, block=16, codes2=c2, meta2=m2, salient_rows=sal_d, out_dtype=dt)
            torch.cuda.synchronize()
            yr = O.dequantize(fbk, host_u8(c), host_u16(m), block=16, codes2=host_u8(c2), meta2=host_u16(m2),
                              salient_rows=sal, out_dtype=odt)
            yg = synth.bf16_bits(y) if dt == F.DTYPE_BF16 else y.cpu().numpy().view(np.uint32)
            assert np.array_equal(yg, yr if dt == F.DTYPE_BF16 else yr.view(np.uint32))


@pytest.mark.parametrize("name,sel,g", SELECTORS_B16)
def test_block16_seda_and_degenerate_values(F, luts, name, sel, g):
    x, comp = synth.mixture_activation(rows=256, cols=16 * 41, seed=49, device="cuda", n_components=5)
    xb = synth.bf16_bits(x)
    sub = synth.seda_sub_formatbooks(DEFAULT_FORMATBOOK, n_groups=5, seed=49)
    tg = comp.copy()
    tg[::9] = -1
    o = F.opts(block=16, selector=sel, num_groups=g)
    c, m = F.fb4_quantize_seda(luts, o, x, torch.from_numpy(tg).cuda(), torch.from_numpy(sub).cuda())
    torch.cuda.synchronize()
    cr, mr = O.quantize(DEFAULT_FORMATBOOK, xb, block=16, selector=sel, num_groups=g, token_group=tg,
                        sub_formatbooks=sub)
    compare_quant(DEFAULT_FORMATBOOK, xb, host_u8(c), host_u16(m), cr, mr, sel, g, token_group=tg, sub=sub,
                  block=16, what="block16 seda " + name)
    xe = synth.edge_case_tensor(cols=256)
    c, m = F.fb4_quantize(luts, o, dev_bits(xe))
    y = F.fb4_dequantize(luts, c, m, block=16)
    torch.cuda.synchronize()
    cr, mr = O.quantize(DEFAULT_FORMATBOOK, xe, block=16, selector=sel, num_groups=g)
    compare_quant(DEFAULT_FORMATBOOK, xe, host_u8(c), host_u16(m), cr, mr, sel, g, block=16,
                  what="block16 edge " + name)
    assert np.array_equal(synth.bf16_bits(y), O.dequantize(DEFAULT_FORMATBOOK, cr, mr, block=16))


@pytest.mark.parametrize("block", [32, 16])
def test_outputs_without_wide_alignment_and_many_seda_groups(F, luts, block):
    """Requests the streaming kernels do not serve (4-byte aligned codes, 2-byte aligned metadata, more SeDA
    groups than fit their LDS) take the generic kernels and give the same results."""
    rows, cols = 96, 1024
    x = synth.vdit_activation(rows=rows, cols=cols, seed=50, device="cuda")
    xb = synth.bf16_bits(x)
    o = F.opts(block=block)
    cbuf = torch.zeros(rows * cols // 2 + 16, dtype=torch.uint8, device="cuda")
    mbuf = torch.zeros(rows * (cols // block) + 8, dtype=torch.int16, device="cuda")
    codes = cbuf[4:4 + rows * cols // 2].view(rows, cols // 2)
    meta = mbuf[1:1 + rows * (cols // block)].view(rows, cols // block)
    assert codes.data_ptr() % 16 == 4 and meta.data_ptr() % 4 == 2
    F.fb4_quantize(luts, o, x, codes=codes, meta=meta)
    y = F.fb4_dequantize(luts, codes, meta, block=block)
    torch.cuda.synchronize()
    cr, mr = O.quantize(DEFAULT_FORMATBOOK, xb, block=block)
    assert np.array_equal(host_u8(codes), cr) and np.array_equal(host_u16(meta), mr)
    assert np.array_equal(synth.bf16_bits(y), O.dequantize(DEFAULT_FORMATBOOK, cr, mr, block=block))
    assert int(cbuf[:4].sum()) == 0 and int(cbuf[4 + rows * cols // 2:].sum()) == 0 and int(mbuf[0]) == 0
    # 2000 SeDA groups
    sub = synth.seda_sub_formatbooks(DEFAULT_FORMATBOOK, n_groups=2000, seed=51)
    tg = ((np.arange(rows) * 37) % 2000).astype(np.int32)
    c, m = F.fb4_quantize_seda(luts, o, x, torch.from_numpy(tg).cuda(), torch.from_numpy(sub).cuda())
    torch.cuda.synchronize()
    cr, mr = O.quantize(DEFAULT_FORMATBOOK, xb, block=block, token_group=tg, sub_formatbooks=sub)
    assert np.array_equal(host_u8(c), cr) and np.array_equal(host_u16(m), mr)


# ------------------------------------------------ both planes in one call
def _both_planes_separately(F, luts, o, x, sal_d, tg_d=None, sub_d=None):
    if tg_d is None:
        c1, m1 = F.fb4_quantize(luts, o, x)
    else:
        c1, m1 = F.fb4_quantize_seda(luts, o, x, tg_d, sub_d)
    c2, m2 = F.fb4_decompose(luts, o, x, c1, m1, sal_d, token_group=tg_d, sub_formatbooks=sub_d)
    return c1, m1, c2, m2


@pytest.mark.parametrize("block", [32, 16])
def test_quantize_decompose_in_one_pass(F, luts, block):
    fbk = DEFAULT_FORMATBOOK
    # the decomposition workload (cfg3 shape): the fused kernel against the oracle on the salient rows
    x = synth.vdit_activation(device="cuda")
    xb = synth.bf16_bits(x)
    sal = synth.salient_rows_from_attention(16384, frac=0.05, heads=24, seed=3, device="cuda")
    sal_d = torch.from_numpy(sal).cuda()
    o = F.opts(block=block)
    c1, m1, c2, m2 = F.fb4_quantize_decompose(luts, o, x, sal_d)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([sal, np.arange(0, 16384, 61)]))
    c1r, m1r = O.quantize(fbk, xb[rows], block=block)
    assert np.array_equal(host_u8(c1)[rows], c1r) and np.array_equal(host_u16(m1)[rows], m1r)
    c2r, m2r = O.decompose(fbk, xb[sal], host_u8(c1)[sal], host_u16(m1)[sal], np.arange(sal.size, dtype=np.int32),
                           block=block)
    assert np.array_equal(host_u8(c2), c2r) and np.array_equal(host_u16(m2), m2r)
    s1, t1, s2, t2 = _both_planes_separately(F, luts, o, x, sal_d)
    assert torch.equal(c1, s1) and torch.equal(m1, t1) and torch.equal(c2, s2) and torch.equal(m2, t2)
    # the exhaustive selector in one pass, against the oracle (first 2048 rows of the same tensor)
    xs, xsb = x[:2048], xb[:2048]
    sal_s = sal[sal < 2048]
    o = F.opts(block=block, selector=F.SEL_SSE)
    c1, m1, c2, m2 = F.fb4_quantize_decompose(luts, o, xs, torch.from_numpy(sal_s).cuda())
    torch.cuda.synchronize()
    c1r, m1r = O.quantize(fbk, xsb, block=block, selector=O.SEL_SSE)
    compare_quant(fbk, xsb, host_u8(c1), host_u16(m1), c1r, m1r, 0, 8, block=block, what="one pass, exhaustive")
    c2r, m2r = O.decompose(fbk, xsb[sal_s], host_u8(c1)[sal_s], host_u16(m1)[sal_s],
                           np.arange(sal_s.size, dtype=np.int32), block=block, selector=O.SEL_SSE)
    compare_quant(fbk, xsb[sal_s], host_u8(c2), host_u16(m2), c2r, m2r, 0, 8, block=block,
                  what="one pass, exhaustive, plane 2")
    # variants: two-stage, SeDA, row stride, list entries outside the tensor, no salient row at all
    xm, comp = synth.mixture_activation(rows=300, cols=32 * 21 + 8, seed=55, device="cuda", n_components=5)
    xs = xm[:, :32 * 21]
    sub_d = torch.from_numpy(synth.seda_sub_formatbooks(fbk, n_groups=5, seed=55)).cuda()
    tg = comp.copy()
    tg[::9] = -1
    tg_d = torch.from_numpy(tg).cuda()
    for flags in (0, F.FLAG_TWO_STAGE):
        for seda in (False, True):
            for sal in (np.arange(0, 300, 7), np.array([-5, -1, 0, 3, 299, 300, 4000]), np.zeros(0)):
                o = F.opts(block=block, flags=flags)
                sal_d = torch.from_numpy(sal.astype(np.int32)).cuda()
                a = (tg_d, sub_d) if seda else (None, None)
                c2 = torch.full((sal.size, 32 * 21 // 2), 0x5A, dtype=torch.uint8, device="cuda")
                c1, m1, c2, m2 = F.fb4_quantize_decompose(luts, o, xs, sal_d, token_group=a[0], sub_formatbooks=a[1],
                                                          codes2=c2)
                s2 = torch.full((sal.size, 32 * 21 // 2), 0x5A, dtype=torch.uint8, device="cuda")
                if seda:
                    s1, t1 = F.fb4_quantize_seda(luts, o, xs, tg_d, sub_d)
                else:
                    s1, t1 = F.fb4_quantize(luts, o, xs)
                _, t2 = F.fb4_decompose(luts, o, xs, s1, t1, sal_d, token_group=a[0], sub_formatbooks=a[1], codes2=s2)
                torch.cuda.synchronize()
                ok = torch.from_numpy((sal >= 0) & (sal < 300)).cuda()
                assert torch.equal(c1, s1) and torch.equal(m1, t1) and torch.equal(c2, s2)
                assert torch.equal(m2[ok], t2[ok])
    # degenerate values: every row salient, residuals with Inf / NaN / tiny magnitudes
    xe = synth.edge_case_tensor(cols=256)
    x = dev_bits(xe)
    sal = np.arange(xe.shape[0], dtype=np.int32)
    for flags in (0, F.FLAG_TWO_STAGE):
        o = F.opts(block=block, flags=flags)
        c1, m1, c2, m2 = F.fb4_quantize_decompose(luts, o, x, torch.from_numpy(sal).cuda())
        torch.cuda.synchronize()
        c1r, m1r = O.quantize(fbk, xe, block=block, flags=flags)
        c2r, m2r = O.decompose(fbk, xe, c1r, m1r, sal, block=block, flags=flags)
        compare_quant(fbk, xe, host_u8(c1), host_u16(m1), c1r, m1r, 1, 8, flags=flags, block=block, what="fused edge 1")
        assert np.array_equal(host_u8(c2), c2r) and np.array_equal(host_u16(m2), m2r)
    # the exhaustive selector in one pass, and requests the one-pass kernel does not serve (16 groups, too many
    # rows), which run the two kernels
    x = synth.gaussian_outlier(rows=64, cols=512, seed=56, device="cuda")
    sal_d = torch.arange(0, 64, 5, dtype=torch.int32, device="cuda")
    for o in (F.opts(block=block, selector=F.SEL_SSE), F.opts(block=block, num_groups=16)):
        got = F.fb4_quantize_decompose(luts, o, x, sal_d)
        want = _both_planes_separately(F, luts, o, x, sal_d)
        torch.cuda.synchronize()
        assert all(torch.equal(g, w) for g, w in zip(got, want))
    x = synth.gaussian_outlier(rows=65600, cols=32, seed=57, device="cuda")
    sal_d = torch.arange(0, 65600, 41, dtype=torch.int32, device="cuda")
    got = F.fb4_quantize_decompose(luts, F.opts(block=block), x, sal_d)
    want = _both_planes_separately(F, luts, F.opts(block=block), x, sal_d)
    torch.cuda.synchronize()
    assert all(torch.equal(g, w) for g, w in zip(got, want))
    # ... and the decode of that many rows adds the second plane in a pass of its own
    y = F.fb4_dequantize(luts, got[0], got[1], block=block, codes2=got[2], meta2=got[3], salient_rows=sal_d)
    torch.cuda.synchronize()
    sal = sal_d.cpu().numpy()
    yr = O.dequantize(DEFAULT_FORMATBOOK, host_u8(got[0]), host_u16(got[1]), block=block, codes2=host_u8(got[2]),
                      meta2=host_u16(got[3]), salient_rows=sal)
    assert np.array_equal(synth.bf16_bits(y), yr)


# ------------------------------------------------ sub-formatbook construction
def test_seda_profile_builds_sub_formatbooks(F, luts):
    fbk = DEFAULT_FORMATBOOK
    x, comp = synth.mixture_activation(device="cuda")         # cfg4: 16384 x 3072, 64 groups
    rng = np.random.default_rng(58)
    anchors = np.where(rng.random(16384) < 0.02, comp, -1).astype(np.int32)   # about 2 % of the tokens
    anchors[:5] = [64, 1000, -7, 0, 63]                       # values outside the groups are no anchors
    for block in (32, 16):
        c, m = F.fb4_quantize(luts, F.opts(block=block), x)
        counts = torch.full((64, 32), 12345, dtype=torch.int32, device="cuda")      # cleared by the call
        counts, sub = F.fb4_seda_profile(luts, m, torch.from_numpy(anchors).cuda(), 64, counts=counts)
        torch.cuda.synchronize()
        cr, sr = O.seda_profile(fbk, host_u16(m), anchors, 64)
        assert np.array_equal(counts.cpu().numpy().view(np.uint32), cr)
        assert np.array_equal(host_u8(sub), sr)
        # and the tables drive the restricted pass
        c2, m2 = F.fb4_quantize_seda(luts, F.opts(block=block), x, torch.from_numpy(comp).cuda(), sub)
        torch.cuda.synchronize()
        rows = np.arange(0, 16384, 16)
        c2r, m2r = O.quantize(fbk, synth.bf16_bits(x)[rows], block=block, token_group=comp[rows], sub_formatbooks=sr)
        assert np.array_equal(host_u8(c2)[rows], c2r) and np.array_equal(host_u16(m2)[rows], m2r)
    # a small formatbook: buckets without a dialect are marked 255; no anchors at all: first dialect per bucket
    l3 = F.fb4_build_luts(fbk[[0, 3, 31]])
    xs = synth.gaussian_outlier(rows=8, cols=256, seed=59, device="cuda")
    c, m = F.fb4_quantize(l3, F.opts(), xs)
    for anc in (np.zeros(8, dtype=np.int32), np.full(8, -1, dtype=np.int32)):
        counts, sub = F.fb4_seda_profile(l3, m, torch.from_numpy(anc).cuda(), 2)
        torch.cuda.synchronize()
        cr, sr = O.seda_profile(fbk[[0, 3, 31]], host_u16(m), anc, 2)
        assert np.array_equal(counts.cpu().numpy().view(np.uint32), cr) and np.array_equal(host_u8(sub), sr)
    l3.free()


# ------------------------------------------------------------ MXFP8 operands
@pytest.mark.parametrize("block", [32, 16])
def test_mxfp8_repack(F, luts, block):
    fbk = DEFAULT_FORMATBOOK
    for rows, cols, stride, seed in ((1024, 3072, 3072, 52), (2, 32, 32, 54), (37, 32 * 19, 32 * 19 + 8, 53)):
        x = synth.vdit_activation(rows=rows, cols=cols, seed=seed, device="cuda")
        if block == 16:
            # neighbouring blocks far apart in magnitude: exercises the shifted, rounded elements
            gen = torch.Generator(device="cpu").manual_seed(seed)
            gap = torch.randint(0, 16, (rows, cols // 16), generator=gen).cuda()
            x = (x.float() * torch.exp2(-gap.float()).repeat_interleave(16, dim=1)).to(torch.bfloat16)
        o = F.opts(block=block)
        c, m = F.fb4_quantize(luts, o, x)
        out = torch.full((rows, stride), 0x55, dtype=torch.uint8, device="cuda")
        el, sc = F.fb4_repack_mxfp8(luts, c, m, block=block, elems=out[:, :cols])
        torch.cuda.synchronize()
        elr, scr = O.repack_mxfp8(fbk, host_u8(c), host_u16(m), block=block)
        assert np.array_equal(host_u8(sc), scr)
        assert np.array_equal(host_u8(out)[:, :cols], elr)
        assert bool((out[:, cols:] == 0x55).all())
        if block == 32:
            # exact: E4M3 value times the E8M0 scale is the decoded tensor
            v = out[:, :cols].contiguous().view(torch.float8_e4m3fn).float()
            y = F.fb4_dequantize(luts, c, m, out_dtype=F.DTYPE_F32)
            scale = torch.exp2(sc.float() - 127).repeat_interleave(32, dim=1)
            assert torch.equal(v * scale, y)
    # the second plane of salient rows is repacked the same way
    sal = torch.arange(0, rows, 1, dtype=torch.int32, device="cuda")
    c2, m2 = F.fb4_decompose(luts, o, x, c, m, sal)
    el2, sc2 = F.fb4_repack_mxfp8(luts, c2, m2, block=block)
    torch.cuda.synchronize()
    elr, scr = O.repack_mxfp8(fbk, host_u8(c2), host_u16(m2), block=block)
    assert np.array_equal(host_u8(el2), elr) and np.array_equal(host_u8(sc2), scr)


# ------------------------------------------------------------ random sweep
def test_random_shapes_options_and_magnitudes(F, luts):
    """Seeded sweep over shapes (ragged tiles, row strides), block sizes, selectors, group counts, flags, SeDA
    lists and salient sets, on data whose rows span 40 binades and contain exact zeros; every entry point
    against the oracle."""
    fbk = DEFAULT_FORMATBOOK
    rng = np.random.default_rng(60)
    for case in range(48):
        block = int(rng.choice([32, 16]))
        rows = int(rng.integers(1, 70))
        nblk = int(rng.integers(1, 41))
        cols = block * nblk
        stride = cols + 8 * int(rng.integers(0, 4))
        sel = int(rng.choice([F.SEL_LUT, F.SEL_LUT, F.SEL_SSE]))
        g = int(rng.choice([8, 16, 32] if block == 32 else [8, 16]))
        flags = int(rng.choice([0, F.FLAG_TWO_STAGE]))
        what = "case %d: block %d %dx%d stride %d sel %d g %d flags %d" % (case, block, rows, cols, stride, sel, g, flags)
        v = rng.standard_t(3, size=(rows, stride)).astype(np.float32)
        v *= np.exp2(rng.integers(-20, 21, size=(rows, 1))).astype(np.float32)
        v[rng.random((rows, stride)) < 0.05] = 0.0
        full = torch.from_numpy(v).to(torch.bfloat16).cuda()
        x = full[:, :cols]
        xb = np.ascontiguousarray(synth.bf16_bits(full)[:, :cols])
        o = F.opts(block=block, selector=sel, num_groups=g, flags=flags)
        use_seda = bool(rng.random() < 0.5)
        tg = sub = tg_d = sub_d = None
        if use_seda:
            ng = int(rng.integers(1, 6))
            sub = synth.seda_sub_formatbooks(fbk, n_groups=ng, seed=100 + case)
            tg = rng.integers(-1, ng, size=rows).astype(np.int32)
            tg_d, sub_d = torch.from_numpy(tg).cuda(), torch.from_numpy(sub).cuda()
        sal = np.nonzero(rng.random(rows) < 0.4)[0].astype(np.int32)
        sal_d = torch.from_numpy(sal).cuda()
        c1, m1, c2, m2 = F.fb4_quantize_decompose(luts, o, x, sal_d, token_group=tg_d, sub_formatbooks=sub_d)
        s1, t1, s2, t2 = _both_planes_separately(F, luts, o, x, sal_d, tg_d, sub_d)
        y = F.fb4_dequantize(luts, c1, m1, block=block, codes2=c2, meta2=m2, salient_rows=sal_d)
        yf = F.fb4_dequantize(luts, c1, m1, block=block, out_dtype=F.DTYPE_F32)
        torch.cuda.synchronize()
        assert torch.equal(c1, s1) and torch.equal(m1, t1) and torch.equal(c2, s2) and torch.equal(m2, t2), what
        c1r, m1r = O.quantize(fbk, xb, block=block, selector=sel, num_groups=g, flags=flags, token_group=tg,
                              sub_formatbooks=sub)
        compare_quant(fbk, xb, host_u8(c1), host_u16(m1), c1r, m1r, sel, g, flags=flags, token_group=tg, sub=sub,
                      block=block, what=what)
        c2r, m2r = O.decompose(fbk, xb, host_u8(c1), host_u16(m1), sal, block=block, selector=sel, num_groups=g,
                               flags=flags, token_group=tg, sub_formatbooks=sub)
        if sal.size:
            compare_quant(fbk, xb[sal], host_u8(c2), host_u16(m2), c2r, m2r, sel, g, flags=flags,
                          token_group=None if tg is None else tg[sal], sub=sub, block=block, what=what + " plane 2")
        yr = O.dequantize(fbk, host_u8(c1), host_u16(m1), block=block, codes2=host_u8(c2), meta2=host_u16(m2),
                          salient_rows=sal)
        assert np.array_equal(synth.bf16_bits(y), yr), what
        yfr = O.dequantize(fbk, host_u8(c1), host_u16(m1), block=block, out_dtype=O.OUT_F32)
        assert np.array_equal(yf.cpu().numpy().view(np.uint32), yfr.view(np.uint32)), what
        if cols % 32 == 0:
            el, sc = F.fb4_repack_mxfp8(luts, c1, m1, block=block)
            torch.cuda.synchronize()
            elr, scr = O.repack_mxfp8(fbk, host_u8(c1), host_u16(m1), block=block)
            assert np.array_equal(host_u8(el), elr) and np.array_equal(host_u8(sc), scr), what


def test_entry_points_replay_correctly_from_a_hip_graph(F, luts):
    """Every entry point only enqueues kernels (no allocation, no memset node), so a captured sequence must
    give the eager results on every replay, also after the inputs changed in place."""
    rows, cols = 512, 3072
    x = torch.empty((rows, cols), dtype=torch.bfloat16, device="cuda")
    sal = torch.arange(3, rows, 17, dtype=torch.int32, device="cuda")
    anchors = torch.where(torch.arange(rows, device="cuda") % 5 == 0, torch.arange(rows, device="cuda") % 4, -1).int()
    o = F.opts()
    c1 = torch.empty((rows, cols // 2), dtype=torch.uint8, device="cuda")
    m1 = torch.empty((rows, cols // 32), dtype=torch.int16, device="cuda")
    c2 = torch.empty((sal.numel(), cols // 2), dtype=torch.uint8, device="cuda")
    m2 = torch.empty((sal.numel(), cols // 32), dtype=torch.int16, device="cuda")
    y = torch.empty((rows, cols), dtype=torch.bfloat16, device="cuda")
    el = torch.empty((rows, cols), dtype=torch.uint8, device="cuda")
    sc = torch.empty((rows, cols // 32), dtype=torch.uint8, device="cuda")
    counts = torch.empty((4, 32), dtype=torch.int32, device="cuda")
    sub = torch.empty((4, 8), dtype=torch.uint8, device="cuda")
    cs = torch.empty_like(c1)
    ms = torch.empty_like(m1)
    tg = (torch.arange(rows, device="cuda") % 4).int()

    def sequence():
        F.fb4_quantize_decompose(luts, o, x, sal, codes1=c1, meta1=m1, codes2=c2, meta2=m2)
        F.fb4_dequantize(luts, c1, m1, codes2=c2, meta2=m2, salient_rows=sal, out=y)
        F.fb4_repack_mxfp8(luts, c1, m1, elems=el, scales=sc)
        F.fb4_seda_profile(luts, m1, anchors, 4, counts=counts, sub_formatbooks=sub)
        F.fb4_quantize_seda(luts, o, x, tg, sub, codes=cs, meta=ms)
        F.fb4_decompose(luts, o, x, c1, m1, sal, codes2=c2b, meta2=m2b)
        F.fb4_quantize(luts, o_sse, x, codes=c3, meta=m3)
        F.fb4_layernorm_quantize(luts, o, x, gamma, beta, 1e-6, codes=c4, meta=m4)
        F.fb4_gelu_quantize(luts, o, x, 1, codes=c5, meta=m5)
        # attention-guided selection on the first 384 channels of x as Q and the next 384 as K: 2 frames x 3 heads x
        # 256 tokens x 128 channels
        F.fb4_attention_scores(qv, kv, 0, scores=att)
        F.fb4_select_salient_tokens(att.view(2, 3, 256), 16, 16, rows_out=anch)
        F.fb4_seda_assign(qv.view(2, 3, 256, 128), kv.view(2, 3, 256, 128), anch, 2, 16, 16, window=5, threshold=4.0,
                          token_group=tgo, anchor_group=ago)
        # step 2 on the same bits read as temporal projections [256 positions][3 heads][2 frames][128], and the 3D
        # variant's main anchors from the scores read as [3 heads][2 * 256 tokens]
        F.fb4_attention_scores(qv.view(768, 2, 128), kv.view(768, 2, 128), 1, scores=att_t)
        F.fb4_seda_main_anchor(att_t.view(256, 3, 2), qv.view(256, 3, 2, 128), kv.view(256, 3, 2, 128), anch, 16, 16,
                               prune_threshold=0.0, main_anchor=main_a, kept=kept_a)
        F.fb4_seda_main_anchor_3d(att.view(3, 512), 2, 16, 16, anchors=anch3)

    qk = torch.empty((2, 2 * 3 * 256 * 128), dtype=torch.bfloat16, device="cuda")
    qv, kv = qk[0].view(6, 256, 128), qk[1].view(6, 256, 128)
    att = torch.empty((6, 256), dtype=torch.float32, device="cuda")
    anch = torch.empty((2, 16), dtype=torch.int32, device="cuda")
    tgo = torch.empty(512, dtype=torch.int32, device="cuda")
    att_t = torch.empty((768, 2), dtype=torch.float32, device="cuda")
    main_a = torch.empty(16, dtype=torch.int32, device="cuda")
    kept_a = torch.empty((2, 16), dtype=torch.int32, device="cuda")
    anch3 = torch.empty(16, dtype=torch.int32, device="cuda")
    ago = torch.empty(512, dtype=torch.int32, device="cuda")
    c2b, m2b, c3, m3 = torch.empty_like(c2), torch.empty_like(m2), torch.empty_like(c1), torch.empty_like(m1)
    c4, m4, c5, m5 = torch.empty_like(c1), torch.empty_like(m1), torch.empty_like(c1), torch.empty_like(m1)
    gamma, beta = (torch.from_numpy(a).cuda() for a in synth.layernorm_affine(cols, seed=70))
    o_sse = F.opts(selector=F.SEL_SSE)
    outs = (c1, m1, c2, m2, y, el, sc, counts, sub, cs, ms, c2b, m2b, c3, m3, c4, m4, c5, m5, att, anch, tgo, ago, att_t, main_a,
            kept_a, anch3)
    x.copy_(synth.vdit_activation(rows=rows, cols=cols, seed=70, device="cuda"))
    qk.copy_(synth.vdit_activation(rows=2, cols=qk.shape[1], seed=170, device="cuda"))
    sequence()                                                # warm-up outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            sequence()
    torch.cuda.synchronize()
    for rep, seed in enumerate((71, 72, 73)):
        x.copy_(synth.vdit_activation(rows=rows, cols=cols, seed=seed, device="cuda"))
        qk.copy_(synth.vdit_activation(rows=2, cols=qk.shape[1], seed=seed + 100, device="cuda"))
        for t in outs:
            t.fill_(7 if t.dtype not in (torch.bfloat16, torch.float32) else 0.5)
        sequence()
        torch.cuda.synchronize()
        want = [t.clone() for t in outs]
        for t in outs:
            t.fill_(9 if t.dtype not in (torch.bfloat16, torch.float32) else 0.25)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k, (a, b) in enumerate(zip(outs, want)):
            assert torch.equal(a, b), "replay %d: output %d differs from the eager run" % (rep, k)
    # and the eager results themselves are the oracle's (last input)
    xb = synth.bf16_bits(x)
    c1r, m1r = O.quantize(DEFAULT_FORMATBOOK, xb)
    assert np.array_equal(host_u8(c1), c1r) and np.array_equal(host_u16(m1), m1r)


def test_luts_handle_is_reusable_across_streams(F, luts):
    x = synth.gaussian_outlier(rows=256, cols=1024, seed=45, device="cuda")
    o = F.opts()
    ref = F.fb4_quantize(luts, o, x)
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    outs = []
    for s in (s1, s2, s1, s2):
        with torch.cuda.stream(s):
            outs.append(F.fb4_quantize(luts, o, x))
    torch.cuda.synchronize()
    for c, m in outs:
        assert torch.equal(c, ref[0]) and torch.equal(m, ref[1])


def test_offsets_beyond_4_gib(F, luts):
    """A 1,500,001 x 3072 tensor (9.2 GB of input, 2.3 GB of codes): every byte offset past 2^32 and the ragged
    last tile, on sampled rows, through both quantize kernels, the second plane, decode and repack."""
    rows, cols = 1_500_001, 3072
    free, _ = torch.cuda.mem_get_info()
    if free < 40 * 2**30:
        pytest.skip("needs 40 GiB of free device memory")
    x = torch.empty((rows, cols), dtype=torch.bfloat16, device="cuda")
    g = torch.Generator(device="cuda")
    g.manual_seed(4242)
    for r0 in range(0, rows, 65536):
        r1 = min(rows, r0 + 65536)
        v = torch.randn((r1 - r0, cols), device="cuda", generator=g)
        v *= torch.exp2(torch.randint(-6, 7, (r1 - r0, cols // 32), device="cuda", generator=g)
                        .float()).repeat_interleave(32, dim=1)
        x[r0:r1] = v.to(torch.bfloat16)
    del v
    rng = np.random.default_rng(4242)
    sample = np.unique(np.concatenate([rng.integers(0, rows, 40), [0, 1, 699_050, 699_051, rows - 2, rows - 1]]))
    idx = torch.from_numpy(sample).cuda()
    xs = synth.bf16_bits(x[idx])
    sal = np.unique(np.concatenate([sample[::3], [rows - 1]])).astype(np.int32)
    sal_d = torch.from_numpy(sal).cuda()
    in_sal = np.isin(sample, sal)
    p_of = torch.from_numpy(np.searchsorted(sal, sample[in_sal])).cuda()
    for name, sel, gg in (SELECTORS[0], SELECTORS[2]):
        o = F.opts(selector=sel, num_groups=gg)
        c1, m1, c2, m2 = F.fb4_quantize_decompose(luts, o, x, sal_d)
        y = F.fb4_dequantize(luts, c1, m1, codes2=c2, meta2=m2, salient_rows=sal_d)
        torch.cuda.synchronize()
        c1s, m1s = host_u8(c1[idx]), host_u16(m1[idx])
        cr, mr = O.quantize(DEFAULT_FORMATBOOK, xs, selector=sel, num_groups=gg)
        compare_quant(DEFAULT_FORMATBOOK, xs, c1s, m1s, cr, mr, sel, gg, what="large " + name)
        c2r, m2r = O.decompose(DEFAULT_FORMATBOOK, xs[in_sal], c1s[in_sal], m1s[in_sal],
                               np.arange(int(in_sal.sum()), dtype=np.int32), selector=sel, num_groups=gg)
        c2s, m2s = host_u8(c2[p_of]), host_u16(m2[p_of])
        compare_quant(DEFAULT_FORMATBOOK, xs[in_sal], c2s, m2s, c2r, m2r, sel, gg, what="large plane 2 " + name)
        # decode of the sampled rows: both planes where the row is salient
        yr = O.dequantize(DEFAULT_FORMATBOOK, c1s, m1s)
        yr[in_sal] = O.dequantize(DEFAULT_FORMATBOOK, c1s[in_sal], m1s[in_sal], codes2=c2s, meta2=m2s,
                                  salient_rows=np.arange(int(in_sal.sum()), dtype=np.int32))
        assert np.array_equal(synth.bf16_bits(y[idx]), yr), "large decode " + name
        del y, c2, m2
        if sel == 1:
            el, sc = F.fb4_repack_mxfp8(luts, c1, m1)
            torch.cuda.synchronize()
            elr, scr = O.repack_mxfp8(DEFAULT_FORMATBOOK, c1s, m1s)
            assert np.array_equal(host_u8(el[idx]), elr) and np.array_equal(host_u8(sc[idx]), scr), "large repack"
            del el, sc
        del c1, m1
        torch.cuda.empty_cache()


# ------------------------------------------------- LayerNorm fused in front of the quantizer (App. E.2)
def _bf16_steps(a, b):
    """Distance of two bf16 bit patterns in representable values (sign-magnitude order, -0 = +0)."""
    oa = np.where(a & 0x8000, -(a & 0x7FFF).astype(np.int64), (a & 0x7FFF).astype(np.int64))
    ob = np.where(b & 0x8000, -(b & 0x7FFF).astype(np.int64), (b & 0x7FFF).astype(np.int64))
    return np.abs(oa - ob)


def check_layernorm_producer(y_gpu, xb, gamma, beta, eps, what="", min_exact=None):
    """The producer's bf16 result against the definition (the float64 oracle).  Bar: the same NaNs; everything else
    within one bf16 step, or -- where gamma * t and beta cancel, or the mean dwarfs the deviations -- within
    2^-19 (|gamma| (|t| + |mean| rstd + 1) + |beta|), the bound of the fp32 producer's error.  Returns the fraction
    of elements that are bit-identical."""
    y_ref, mean, rstd = O.layernorm(xb, gamma, beta, eps)
    nan_ref = (y_ref & 0x7FFF) > 0x7F80
    assert np.array_equal(y_gpu[nan_ref], y_ref[nan_ref]), what + ": NaN pattern"
    assert not ((y_gpu & 0x7FFF) > 0x7F80)[~nan_ref].any(), what + ": NaN where the definition is finite"
    steps = _bf16_steps(y_gpu, y_ref)
    far = (steps > 1) & ~nan_ref
    if far.any():
        x64 = synth_b2f(xb)
        g = np.ones(xb.shape[1]) if gamma is None else gamma.astype(np.float64)
        b = np.zeros(xb.shape[1]) if beta is None else beta.astype(np.float64)
        with np.errstate(all="ignore"):
            t = (x64 - mean[:, None]) * rstd[:, None]
            allow = 2.0 ** -19 * (np.abs(g) * (np.abs(t) + np.abs(mean * rstd)[:, None] + 1.0) + np.abs(b))
            err = np.abs(synth_b2f(y_gpu) - synth_b2f(y_ref))
        assert (err[far] <= allow[far]).all(), "%s: %d elements beyond one bf16 step and beyond the fp32 bound" % (what, far.sum())
    exact = float((y_gpu == y_ref)[~nan_ref].mean()) if (~nan_ref).any() else 1.0
    if min_exact is not None:
        assert exact >= min_exact, "%s: only %.5f of the elements are the correctly rounded ones" % (what, exact)
    return exact


def synth_b2f(bits):
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    with np.errstate(invalid="ignore"):
        return u.view(np.float32).astype(np.float64)


def _ln_case(F, luts, xb, gamma, beta, eps, flags=0, what="", x_dev=None, tg=None, sub=None, min_exact=None, block=32, ng=8):
    """One call with the checking output: (i) the producer's bf16 tensor against the float64 definition,
    (ii) codes and metadata bit for bit against the oracle's quantizer run on the GPU's own bf16 tensor."""
    x = dev_bits(xb) if x_dev is None else x_dev
    g = None if gamma is None else torch.from_numpy(gamma).cuda()
    b = None if beta is None else torch.from_numpy(beta).cuda()
    o = F.opts(block=block, selector=1, num_groups=ng, flags=flags)
    y_d = torch.full(x.shape, 7.0, dtype=torch.bfloat16, device="cuda")
    tg_d = None if tg is None else torch.from_numpy(tg).cuda()
    sub_d = None if sub is None else torch.from_numpy(sub).cuda()
    c, m = F.fb4_layernorm_quantize(luts, o, x, g, b, eps, token_group=tg_d, sub_formatbooks=sub_d, y_out=y_d)
    c0, m0 = F.fb4_layernorm_quantize(luts, o, x, g, b, eps, token_group=tg_d, sub_formatbooks=sub_d)   # as in production
    torch.cuda.synchronize()
    assert torch.equal(c, c0) and torch.equal(m, m0)
    y_gpu = synth.bf16_bits(y_d)
    cr, mr = O.quantize(DEFAULT_FORMATBOOK, y_gpu, block=block, selector=1, num_groups=ng, flags=flags, token_group=tg,
                        sub_formatbooks=sub)
    compare_quant(DEFAULT_FORMATBOOK, y_gpu, host_u8(c), host_u16(m), cr, mr, 1, ng, flags=flags, token_group=tg, sub=sub,
                  what="layernorm " + what, block=block)
    exact = check_layernorm_producer(y_gpu, xb, gamma, beta, eps, what="layernorm " + what, min_exact=min_exact)
    return c, m, y_gpu, exact


# rows x cols -> chunks per lane / rows per bundle the launcher picks: 3/2, 3/5 (ragged last bundle, bundles that
# do not fill the wavefront), 6/1, 1/64 cut to the row count, 2/1, 4/1, 5/1 with idle lanes, 1/2, 2/3
LN_SHAPES = [(1024, 3072), (1000, 1152), (37, 12288), (5, 32), (129, 4096), (50, 8192), (33, 9600), (131, 1024),
             (77, 1344), (1, 3072), (513, 64)]


@pytest.mark.parametrize("rows,cols", LN_SHAPES)
def test_layernorm_quantize_shapes(F, luts, rows, cols):
    x = synth.vdit_activation(rows=rows, cols=cols, seed=rows + cols, device="cuda")
    gamma, beta = synth.layernorm_affine(cols, seed=cols)
    _ln_case(F, luts, synth.bf16_bits(x), gamma, beta, 1e-6, what="%dx%d" % (rows, cols), x_dev=x, min_exact=0.999)


def test_layernorm_quantize_full_size_two_stage_and_no_affine(F, luts):
    x = synth.vdit_activation(device="cuda")                  # 16384 x 3072, the benchmark workload
    xb = synth.bf16_bits(x)
    gamma, beta = synth.layernorm_affine(3072)
    exact = _ln_case(F, luts, xb, gamma, beta, 1e-6, what="cfg2", x_dev=x, min_exact=0.999)[3]
    print("layernorm producer on the 16384x3072 tensor: %.6f of the bf16 values are the correctly rounded ones" % exact)
    _ln_case(F, luts, xb, gamma, beta, 1e-5, flags=F.FLAG_TWO_STAGE, what="cfg2 two-stage", x_dev=x, min_exact=0.999)
    _ln_case(F, luts, xb, None, None, 1e-6, what="cfg2 no affine", x_dev=x, min_exact=0.999)
    _ln_case(F, luts, xb, gamma, None, 0.0, what="cfg2 scale only, eps 0", x_dev=x, min_exact=0.999)


@pytest.mark.parametrize("block,g", [(32, 16), (16, 8), (16, 16)])
def test_fused_producers_other_block_sizes_and_group_counts(F, luts, block, g):
    """Sec. 4.1 evaluates block sizes 16 and 32; the online rule with 8 or 16 groups: both producers, with and without
    SeDA lists and the two-stage flag."""
    for rows, cols, flags, n_groups in [(700, 3072, 0, 0), (333, 1152, 1, 0), (64, 12288, 0, 5), (2048, 4096, 1, 64), (129, 64, 0, 0)]:
        x, comp = synth.mixture_activation(rows=rows, cols=cols, seed=rows + block + g, n_components=max(n_groups, 2), device="cuda")
        xb = synth.bf16_bits(x)
        tg = sub = tg_d = sub_d = None
        if n_groups:
            tg = comp.copy()
            tg[::9] = -1
            sub = synth.seda_sub_formatbooks(DEFAULT_FORMATBOOK, n_groups, rows)
            tg_d, sub_d = torch.from_numpy(tg).cuda(), torch.from_numpy(sub).cuda()
        gamma, beta = synth.layernorm_affine(cols, seed=cols)
        _ln_case(F, luts, xb, gamma, beta, 1e-6, flags=flags, what="block %d g %d %dx%d" % (block, g, rows, cols), x_dev=x, tg=tg,
                 sub=sub, min_exact=0.999, block=block, ng=g)
        o = F.opts(block=block, selector=1, num_groups=g, flags=flags)
        for approximate in (0, 1):
            c, m = F.fb4_gelu_quantize(luts, o, x, approximate, token_group=tg_d, sub_formatbooks=sub_d)
            torch.cuda.synchronize()
            y = O.gelu(xb, approximate)
            cr, mr = O.quantize(DEFAULT_FORMATBOOK, y, block=block, selector=1, num_groups=g, flags=flags, token_group=tg,
                                sub_formatbooks=sub)
            compare_quant(DEFAULT_FORMATBOOK, y, host_u8(c), host_u16(m), cr, mr, 1, g, flags=flags, token_group=tg, sub=sub,
                          what="gelu block %d g %d %dx%d" % (block, g, rows, cols), block=block)
    # degenerate values through both producers
    xe = synth.edge_case_tensor(cols=256)
    _ln_case(F, luts, xe, None, None, 1e-6, what="edge rows block %d g %d" % (block, g), block=block, ng=g)
    c, m = F.fb4_gelu_quantize(luts, F.opts(block=block, selector=1, num_groups=g), dev_bits(xe), 0)
    torch.cuda.synchronize()
    cr, mr = O.quantize(DEFAULT_FORMATBOOK, O.gelu(xe, 0), block=block, selector=1, num_groups=g)
    assert np.array_equal(host_u8(c), cr) and np.array_equal(host_u16(m), mr)
    # metadata of block-16 output must be 4-byte aligned
    if block == 16:
        x = synth.vdit_activation(rows=8, cols=256, seed=1, device="cuda")
        mbuf = torch.zeros(8 * 16 + 1, dtype=torch.int16, device="cuda")
        for call in (lambda **kw: F.fb4_layernorm_quantize(luts, F.opts(block=16, num_groups=g), x, **kw),
                     lambda **kw: F.fb4_gelu_quantize(luts, F.opts(block=16, num_groups=g), x, 0, **kw)):
            with pytest.raises(F.Fb4Error) as e:
                call(meta=mbuf[1:].view(8, 16))
            assert e.value.code == F.ERR_UNSUPPORTED


def test_layernorm_producer_constant_rows_and_large_means(F, luts):
    # a constant row: every x - mean is exactly 0, so y is exactly beta (rounded to bf16), whatever eps > 0
    gamma, beta = synth.layernorm_affine(3072, seed=12)
    vals = np.array([1.5, -1000.0, 3.0e-5, 0.0, 2.0 ** 100, -2.0 ** -100, 7.0], dtype=np.float32)
    xb = np.repeat(synth.bf16_bits(torch.from_numpy(vals).bfloat16())[:, None], 3072, axis=1)
    _, _, y_gpu, _ = _ln_case(F, luts, xb, gamma, beta, 1e-6, what="constant rows")
    want = synth.bf16_bits(torch.from_numpy(beta).bfloat16())
    assert (y_gpu == want[None, :]).all()
    # rows whose mean dwarfs their spread, and rows far from 1 in scale: still within the bar, nearly all exact
    rng = np.random.default_rng(13)
    for mu, sigma, floor in [(100.0, 1.0, 0.99), (-3.0, 20.0, 0.999), (1.0e4, 3.0, 0.9), (0.0, 1.0e-12, 0.999), (0.0, 1.0e12, 0.999),
                             (5.0e-20, 1.0e-20, 0.99), (1.0e25, 1.0e25, 0.99), (0.0, 1.0e-30, 0.99), (0.0, 1.0e35, 0.99)]:
        xf = (mu + sigma * rng.standard_normal((64, 1152))).astype(np.float32)
        xb = synth.bf16_bits(torch.from_numpy(xf).bfloat16())
        g, b = synth.layernorm_affine(1152, seed=14)
        for eps in (1e-6, 0.0):
            _ln_case(F, luts, xb, g, b, eps, what="mean %g std %g eps %g" % (mu, sigma, eps), min_exact=floor)


def test_layernorm_quantize_degenerate_rows_and_strides(F, luts):
    xe = synth.edge_case_tensor(cols=256)                      # zero rows, subnormals, Inf, NaN, constants, 1e30
    gamma, beta = synth.layernorm_affine(256, seed=9)
    for eps in (1e-6, 0.0):                                    # eps 0: a constant row divides by zero -> NaN row
        _ln_case(F, luts, xe, gamma, beta, eps, what="edge rows eps %g" % eps)
        _ln_case(F, luts, xe, None, None, eps, what="edge rows, no affine, eps %g" % eps)
    # scale / shift with zeros, huge values and an Inf: products overflow, Inf * 0 and Inf - Inf make single NaNs
    g2 = gamma.copy(); b2 = beta.copy()
    g2[3] = 0.0; g2[40] = 3e38; g2[41] = -3e38; b2[40] = 3e38; b2[41] = 3e38; g2[100] = np.inf; b2[100] = -np.inf
    g2[130] = 1e-30; b2[130] = 0.0; g2[131] = 1e-38; b2[131] = 1e-40
    x = synth.vdit_activation(rows=64, cols=256, seed=5, device="cuda")
    _ln_case(F, luts, synth.bf16_bits(x), g2, b2, 1e-6, what="extreme scale and shift", x_dev=x)
    # a row stride, and outputs that are only 16 / 2 byte aligned
    wide = synth.vdit_activation(rows=70, cols=3072 + 64, seed=6, device="cuda")
    xs = wide[:, 32:32 + 3072]
    gamma, beta = synth.layernorm_affine(3072, seed=2)
    o = F.opts(selector=1, num_groups=8)
    cbuf = torch.zeros(70 * 1536 + 16, dtype=torch.uint8, device="cuda")
    mbuf = torch.zeros(70 * 96 + 1, dtype=torch.int16, device="cuda")
    c = cbuf[16:].view(70, 1536); m = mbuf[1:].view(70, 96)
    y_d = torch.empty((70, 3072), dtype=torch.bfloat16, device="cuda")
    F.fb4_layernorm_quantize(luts, o, xs, torch.from_numpy(gamma).cuda(), torch.from_numpy(beta).cuda(), 1e-6, codes=c, meta=m,
                             y_out=y_d)
    torch.cuda.synchronize()
    xb = synth.bf16_bits(xs.contiguous())
    y_gpu = synth.bf16_bits(y_d)
    check_layernorm_producer(y_gpu, xb, gamma, beta, 1e-6, what="row stride", min_exact=0.999)
    cr, mr = O.quantize(DEFAULT_FORMATBOOK, y_gpu)
    assert np.array_equal(host_u8(c), cr) and np.array_equal(host_u16(m), mr)
    assert not cbuf[:16].any() and mbuf[0] == 0


def test_layernorm_quantize_is_the_unfused_pair_and_rejects_what_it_does_not_serve(F, luts):
    # the same codes as the plain entry point run on the oracle's normalized tensor
    x = synth.gaussian_outlier(rows=256, cols=3072, seed=8, device="cuda")
    gamma, beta = synth.layernorm_affine(3072, seed=8)
    c, m, y_gpu, _ = _ln_case(F, luts, synth.bf16_bits(x), gamma, beta, 1e-6, what="unfused", x_dev=x, min_exact=0.999)
    c2, m2 = F.fb4_quantize(luts, F.opts(), dev_bits(y_gpu))
    torch.cuda.synchronize()
    assert torch.equal(c, c2) and torch.equal(m, m2)
    for o, code in ((F.opts(num_groups=32), F.ERR_UNSUPPORTED), (F.opts(selector=0), F.ERR_UNSUPPORTED)):
        with pytest.raises(F.Fb4Error) as e:
            F.fb4_layernorm_quantize(luts, o, x)
        assert e.value.code == code
    with pytest.raises(F.Fb4Error) as e:
        F.fb4_layernorm_quantize(luts, F.opts(), x, eps=-1.0)
    assert e.value.code == F.ERR_INVALID_ARG
    with pytest.raises(F.Fb4Error) as e:
        F.fb4_layernorm_quantize(luts, F.opts(), x, eps=float("nan"))
    assert e.value.code == F.ERR_INVALID_ARG
    big = torch.zeros((2, 12288 + 32), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(F.Fb4Error) as e:
        F.fb4_layernorm_quantize(luts, F.opts(), big)
    assert e.value.code == F.ERR_UNSUPPORTED
    F.fb4_layernorm_quantize(luts, F.opts(), x[:0])           # no rows: a successful no-op


# ------------------------------------------------- GeLU fused in front of the quantizer (App. E.2)
def _gelu_case(F, luts, xb, approximate, flags=0, what="", x_dev=None, rows=None):
    """rows: compare these rows only (the oracle runs on them alone)."""
    x = dev_bits(xb) if x_dev is None else x_dev
    o = F.opts(selector=1, num_groups=8, flags=flags)
    c, m = F.fb4_gelu_quantize(luts, o, x, approximate)
    torch.cuda.synchronize()
    cg, mg = host_u8(c), host_u16(m)
    if rows is not None:
        xb, cg, mg = xb[rows], cg[rows], mg[rows]
    y = O.gelu(xb, approximate)
    cr, mr = O.quantize(DEFAULT_FORMATBOOK, y, selector=1, num_groups=8, flags=flags)
    compare_quant(DEFAULT_FORMATBOOK, y, cg, mg, cr, mr, 1, 8, flags=flags, what="gelu " + what)
    return c, m


@pytest.mark.parametrize("approximate", [0, 1])
def test_gelu_quantize_shapes_and_full_size(F, luts, approximate):
    for rows, cols in [(1024, 3072), (333, 1184), (1, 32), (7, 64), (65, 12288), (129, 4096)]:
        x = synth.vdit_activation(rows=rows, cols=cols, seed=rows + cols, device="cuda")
        _gelu_case(F, luts, synth.bf16_bits(x), approximate, what="%dx%d" % (rows, cols), x_dev=x)
    x = synth.vdit_activation(device="cuda")                  # 16384 x 3072, the benchmark workload
    xb = synth.bf16_bits(x)
    _gelu_case(F, luts, xb, approximate, what="cfg2", x_dev=x)
    _gelu_case(F, luts, xb, approximate, flags=F.FLAG_TWO_STAGE, what="cfg2 two-stage", x_dev=x)


def test_gelu_quantize_cfg5_sampled_rows(F, luts):
    R5, C5 = synth.CONFIG_SHAPES["cfg5"]                       # 65536 x 12288: the input of mlp.fc2
    x = synth.vdit_activation(rows=R5, cols=C5, seed=5, device="cuda", outlier_frac=0.01)
    rows = np.unique(np.concatenate([np.arange(0, 64), np.arange(R5 - 64, R5),
                                     np.random.default_rng(5).integers(0, R5, 384)]))
    xb = np.zeros((R5, C5), dtype=np.uint16)
    xb[rows] = synth.bf16_bits(x[torch.from_numpy(rows).cuda()])
    _gelu_case(F, luts, xb, 1, what="cfg5", x_dev=x, rows=rows)
    del x


def test_gelu_quantize_degenerate_values_strides_and_errors(F, luts):
    xe = synth.edge_case_tensor(cols=256).copy()               # zeros, subnormals, +-Inf, NaNs of both signs, 1e30
    xe[2, 9] = 0xFFFF; xe[2, 200] = 0xFF81; xe[12, 3] = 0xC180; xe[12, 4] = 0xC181; xe[12, 5] = 0x4180; xe[12, 6] = 0x7F7F
    for approximate in (0, 1):
        _gelu_case(F, luts, xe, approximate, what="edge rows")
        _gelu_case(F, luts, xe, approximate, flags=F.FLAG_TWO_STAGE, what="edge rows two-stage")
    # every bf16 pattern once
    allb = np.arange(65536, dtype=np.uint16).reshape(32, 2048)
    _gelu_case(F, luts, allb, 0, what="all patterns")
    _gelu_case(F, luts, allb, 1, what="all patterns, tanh form")
    # a row stride, outputs that are only 16 / 2 byte aligned
    wide = synth.vdit_activation(rows=70, cols=3072 + 64, seed=6, device="cuda")
    xs = wide[:, 32:32 + 3072]
    cbuf = torch.zeros(70 * 1536 + 16, dtype=torch.uint8, device="cuda")
    mbuf = torch.zeros(70 * 96 + 1, dtype=torch.int16, device="cuda")
    c = cbuf[16:].view(70, 1536); m = mbuf[1:].view(70, 96)
    F.fb4_gelu_quantize(luts, F.opts(), xs, 1, codes=c, meta=m)
    torch.cuda.synchronize()
    y = O.gelu(synth.bf16_bits(xs.contiguous()), 1)
    cr, mr = O.quantize(DEFAULT_FORMATBOOK, y)
    assert np.array_equal(host_u8(c), cr) and np.array_equal(host_u16(m), mr)
    assert not cbuf[:16].any() and mbuf[0] == 0
    # what it does not serve
    x = synth.gaussian_outlier(rows=64, cols=1024, seed=8, device="cuda")
    for o, code in ((F.opts(num_groups=32), F.ERR_UNSUPPORTED), (F.opts(selector=0), F.ERR_UNSUPPORTED)):
        with pytest.raises(F.Fb4Error) as e:
            F.fb4_gelu_quantize(luts, o, x)
        assert e.value.code == code
    with pytest.raises(F.Fb4Error) as e:
        F.fb4_gelu_quantize(luts, F.opts(), x, approximate=2)
    assert e.value.code == F.ERR_INVALID_ARG
    F.fb4_gelu_quantize(luts, F.opts(), x[:0])                 # no rows: a successful no-op


# ------------------------------------------------- SeDA candidate lists behind the fused producers (Sec. 3.4 + App. E.2)
def _odd_seda_tables(n_groups, seed):
    """Sub-formatbooks with some invalid DIDs and one group without any valid DID (inputs the oracle refuses:
    such a case is compared with fb4_quantize_seda on the oracle's producer output)."""
    sub = synth.seda_sub_formatbooks(DEFAULT_FORMATBOOK, n_groups, seed).copy()
    sub[1, 2] = 200; sub[1, 5] = 32
    sub[n_groups - 1, :] = 255
    return sub


@pytest.mark.parametrize("producer", ["layernorm", "gelu"])
def test_fused_producers_with_seda_candidate_lists(F, luts, producer):
    for rows, cols, n_groups, flags in [(2048, 3072, 64, 0), (515, 1152, 255, 0), (300, 4096, 7, 1), (64, 12288, 3, 0)]:
        x, comp = synth.mixture_activation(rows=rows, cols=cols, seed=rows, n_components=n_groups, device="cuda")
        xb = synth.bf16_bits(x)
        tg = comp.copy()
        tg[::13] = -1                                              # no group: full formatbook
        sub = synth.seda_sub_formatbooks(DEFAULT_FORMATBOOK, n_groups, rows)
        o = F.opts(selector=1, num_groups=8, flags=flags)
        tg_d, sub_d = torch.from_numpy(tg).cuda(), torch.from_numpy(sub).cuda()
        if producer == "layernorm":
            gamma, beta = synth.layernorm_affine(cols, seed=cols)
            c, m, y, _ = _ln_case(F, luts, xb, gamma, beta, 1e-6, flags=flags, what="seda %dx%d" % (rows, cols), x_dev=x,
                                  tg=tg, sub=sub, min_exact=0.999)
        else:
            c, m = F.fb4_gelu_quantize(luts, o, x, 1, token_group=tg_d, sub_formatbooks=sub_d)
            y = O.gelu(xb, 1)
        torch.cuda.synchronize()
        cr, mr = O.quantize(DEFAULT_FORMATBOOK, y, selector=1, num_groups=8, flags=flags, token_group=tg, sub_formatbooks=sub)
        compare_quant(DEFAULT_FORMATBOOK, y, host_u8(c), host_u16(m), cr, mr, 1, 8, flags=flags, token_group=tg, sub=sub,
                      what="%s seda %dx%d" % (producer, rows, cols))
        # the lists do constrain: rows in a valid group only use its DIDs
        dids = host_u16(m) & 0xFF
        for r in (0, 1, 2, 7):
            g = tg[r]
            if g >= 0:
                assert np.isin(dids[r], sub[g]).all()
    # degenerate values under the lists, and the argument checks
    xe = synth.edge_case_tensor(cols=256)
    tg = (np.arange(xe.shape[0]) % 5).astype(np.int32) - 1
    sub = synth.seda_sub_formatbooks(DEFAULT_FORMATBOOK, 4, 3)
    tg_d, sub_d = torch.from_numpy(tg).cuda(), torch.from_numpy(sub).cuda()
    if producer == "layernorm":
        c, m, y, _ = _ln_case(F, luts, xe, None, None, 1e-6, what="edge rows under lists", tg=tg, sub=sub)
    else:
        c, m = F.fb4_gelu_quantize(luts, F.opts(), dev_bits(xe), 0, token_group=tg_d, sub_formatbooks=sub_d)
        y = O.gelu(xe, 0)
    torch.cuda.synchronize()
    cr, mr = O.quantize(DEFAULT_FORMATBOOK, y, token_group=tg, sub_formatbooks=sub)
    assert np.array_equal(host_u8(c), cr) and np.array_equal(host_u16(m), mr)
    call = F.fb4_layernorm_quantize if producer == "layernorm" else F.fb4_gelu_quantize
    # lists with invalid DIDs, a group without a valid DID and rows outside every group behave as in
    # fb4_quantize_seda (the oracle refuses such tables): same codes as that call on the oracle's producer output
    x, comp = synth.mixture_activation(rows=200, cols=1024, seed=77, n_components=6, device="cuda")
    tg = comp.copy(); tg[::7] = -5; tg[3::11] = 9
    sub = _odd_seda_tables(6, 77)
    tg2_d, sub2_d = torch.from_numpy(tg).cuda(), torch.from_numpy(sub).cuda()
    if producer == "layernorm":
        y_d = torch.empty_like(x)
        c, m = call(luts, F.opts(), x, token_group=tg2_d, sub_formatbooks=sub2_d, y_out=y_d)
        torch.cuda.synchronize()
        y = synth.bf16_bits(y_d)
        check_layernorm_producer(y, synth.bf16_bits(x), None, None, 1e-6, what="odd lists", min_exact=0.999)
    else:
        c, m = call(luts, F.opts(), x, token_group=tg2_d, sub_formatbooks=sub2_d)
        y = O.gelu(synth.bf16_bits(x), 0)
    c2, m2 = F.fb4_quantize_seda(luts, F.opts(), dev_bits(y), tg2_d, sub2_d)
    torch.cuda.synchronize()
    assert torch.equal(c, c2) and torch.equal(m, m2)
    big = torch.zeros((256, 8), dtype=torch.uint8, device="cuda")
    with pytest.raises(F.Fb4Error) as e:
        call(luts, F.opts(), dev_bits(xe), token_group=tg_d, sub_formatbooks=big)
    assert e.value.code == F.ERR_UNSUPPORTED                       # more groups than the fused kernels hold
    with pytest.raises(F.Fb4Error) as e:
        call(luts, F.opts(), dev_bits(xe), token_group=tg_d, sub_formatbooks=None)
    assert e.value.code == F.ERR_INVALID_ARG


# ------------------------------------------------- attention-guided salient tokens (Sec. 3.3, App. F)
@pytest.mark.parametrize("mode", [0, 1])
def test_attention_scores_against_the_oracle(F, mode):
    """The one floating-point contraction of the library (bf16 products, fp32 accumulation on the matrix cores):
    compared with the float64 oracle to 2e-5 relative (the terms of a score are all non-negative: no cancellation
    in the sum over keys; a single dot product loses at most sqrt(dim) * 2^-24 of its operands' magnitude)."""
    # (groups of up to 64 tokens -- temporal attention -- run the small shape of the kernel, longer ones the large)
    for groups, tokens, dim in [(3, 100, 64), (2, 1024, 128), (5, 33, 72), (1, 1, 8), (2, 257, 256), (4, 128, 40),
                                (2, 300, 96), (1, 2049, 16), (300, 16, 72), (50, 64, 128), (7, 65, 64), (3, 513, 200),
                                # rows of 128 channels and a multiple of 128 tokens take the kernel that loads key blocks
                                # straight into LDS: one block per key half, an odd number of blocks, a last workgroup
                                # with 128 of its 256 queries, several workgroups per group; (2, 200, 128) does not
                                (3, 128, 128), (2, 384, 128), (1, 640, 128), (2, 2048, 128), (2, 200, 128)]:
        q, k = synth.attention_qk(groups, tokens, dim, seed=tokens + dim, device="cuda")
        got = F.fb4_attention_scores(q, k, mode).cpu().numpy().astype(np.float64)
        torch.cuda.synchronize()
        ref = O.attention_scores(synth.bf16_bits(q), synth.bf16_bits(k), "relu" if mode else "abs")
        # scale of the terms: mean |s| (for relu the sum can be much smaller than the terms it leaves out)
        scale = O.attention_scores(synth.bf16_bits(q), synth.bf16_bits(k), "abs")
        assert np.abs(got - ref).max() <= 2e-5 * scale.max(), (groups, tokens, dim)
        assert (np.abs(got - ref) <= 2e-5 * scale + 1e-30).all(), (groups, tokens, dim)
    # exactly representable case: 0 / 1 inputs give integer dot products, exact in fp32
    rng = np.random.default_rng(91)
    qb = (rng.random((2, 200, 64)) < 0.3).astype(np.float32) * np.where(rng.random((2, 200, 64)) < 0.5, -1, 1)
    kb = (rng.random((2, 200, 64)) < 0.3).astype(np.float32)
    q, k = torch.from_numpy(qb).cuda().bfloat16(), torch.from_numpy(kb).cuda().bfloat16()
    got = F.fb4_attention_scores(q, k, mode).cpu().numpy()
    ref = O.attention_scores(synth.bf16_bits(q), synth.bf16_bits(k), "relu" if mode else "abs")
    assert np.array_equal(got, ref.astype(np.float32))          # sums of small integers / 200: one rounding each
    qb = (rng.random((2, 384, 128)) < 0.3).astype(np.float32) * np.where(rng.random((2, 384, 128)) < 0.5, -1, 1)
    kb = (rng.random((2, 384, 128)) < 0.3).astype(np.float32)
    q, k = torch.from_numpy(qb).cuda().bfloat16(), torch.from_numpy(kb).cuda().bfloat16()
    got = F.fb4_attention_scores(q, k, mode).cpu().numpy()
    ref = O.attention_scores(synth.bf16_bits(q), synth.bf16_bits(k), "relu" if mode else "abs")
    assert np.array_equal(got, ref.astype(np.float32))          # the same through the other kernel


def test_mfma_rate_probe_runs_and_counts_its_operations(F):
    out, flop = F.fb4_probe_mfma_rate(8, 3, True)
    torch.cuda.synchronize()
    assert flop == 8 * 4 * 3 * 32 * 2 * 32 * 32 * 16 and out.shape == (8 * 256,) and bool(torch.isfinite(out).all())
    out0, _ = F.fb4_probe_mfma_rate(8, 3, False)
    # one bit pattern (1.0) everywhere: every accumulator is 3 * 8 * 16 products of 1, sixteen per lane and chain
    assert bool((out0 == 3 * 8 * 16 * 64).all())
    lib = F.binding.lib()
    assert lib.fb4_probe_mfma_rate(0, 1, 1, out.data_ptr(), None, None) == F.ERR_INVALID_ARG
    assert lib.fb4_probe_mfma_rate(8, 1, 1, None, None, None) == F.ERR_INVALID_ARG


def test_salient_token_selection_and_the_whole_chain(F, luts):
    # selection alone, on the oracle's scores: bit-exact (ties, NaNs, ragged tiles)
    rng = np.random.default_rng(92)
    for frames, heads, gh, gw, th, tw in [(3, 5, 7, 10, 4, 4), (16, 24, 32, 32, 4, 4), (1, 1, 1, 1, 4, 4), (2, 3, 64, 64, 8, 8),
                                          (2, 2, 9, 33, 2, 5)]:
        sc = rng.random((frames, heads, gh * gw)).astype(np.float32)
        sc[:, :, ::7] = 0.5                                        # ties
        if gh * gw > 20:
            sc[0, 0, 3] = np.nan; sc[-1, :, 11] = np.nan
        got = F.fb4_select_salient_tokens(torch.from_numpy(sc).cuda(), gh, gw, th, tw).cpu().numpy()
        assert np.array_equal(got, O.select_salient_tokens(sc, gh, gw, th, tw))
    # the chain: scores on the GPU, selection on the GPU, the rows into the one-pass decomposition.  The chosen token
    # of a tile must be (one of) the oracle's best: its float64 mean score within 1e-4 of the tile's largest.
    frames, heads, gh, gw, dim = 4, 6, 16, 16, 64
    tokens = gh * gw
    q, k = synth.attention_qk(frames * heads, tokens, dim, seed=5, device="cuda")
    scores = F.fb4_attention_scores(q, k, 0)
    rows = F.fb4_select_salient_tokens(scores.view(frames, heads, tokens), gh, gw)
    torch.cuda.synchronize()
    ref = O.attention_scores(synth.bf16_bits(q), synth.bf16_bits(k), "abs").reshape(frames, heads, tokens).mean(axis=1)
    r = rows.cpu().numpy()
    assert r.shape == (frames, 16) and (np.diff(r.reshape(-1)) > 0).all()
    for f in range(frames):
        tiles = set()
        for row in r[f]:
            t = int(row) - f * tokens
            y, x = divmod(t, gw)
            tiles.add((y // 4, x // 4))
            best = max(ref[f, yy * gw + xx] for yy in range(y // 4 * 4, y // 4 * 4 + 4) for xx in range(x // 4 * 4, x // 4 * 4 + 4))
            assert ref[f, t] >= best * (1 - 1e-4)
        assert len(tiles) == 16
    x = synth.vdit_activation(rows=frames * tokens, cols=1024, seed=9, device="cuda")
    c1, m1, c2, m2 = F.fb4_quantize_decompose(luts, F.opts(), x, rows.view(-1))
    torch.cuda.synchronize()
    xb = synth.bf16_bits(x)
    c1r, m1r = O.quantize(DEFAULT_FORMATBOOK, xb)
    c2r, m2r = O.decompose(DEFAULT_FORMATBOOK, xb, c1r, m1r, r.reshape(-1))
    assert np.array_equal(host_u8(c2), c2r) and np.array_equal(host_u16(m2), m2r)
    # argument checks
    with pytest.raises(F.Fb4Error) as e:
        F.fb4_attention_scores(q[:, :, :60].contiguous(), k[:, :, :60].contiguous(), 0)      # dim not a multiple of 8
    assert e.value.code == F.ERR_UNSUPPORTED
    with pytest.raises(F.Fb4Error) as e:
        F.fb4_attention_scores(q, k, 2)
    assert e.value.code == F.ERR_INVALID_ARG
    with pytest.raises(F.Fb4Error) as e:
        F.fb4_select_salient_tokens(torch.zeros((1, 1, 128 * 128), device="cuda"), 128, 128)   # more than 8192 tokens
    assert e.value.code == F.ERR_UNSUPPORTED


def _assign_case(F, q_d, k_d, qb, kb, anchors, frames, gh, gw, th, tw, window, window_t, thr, joint):
    """fb4_seda_assign against the oracle: scores to 2e-5, groups bit for bit (no score near the threshold)."""
    tg, ag, sc = F.fb4_seda_assign(q_d, k_d, torch.from_numpy(np.ascontiguousarray(anchors, dtype=np.int32)).cuda(), frames, gh, gw,
                                   tile_h=th, tile_w=tw, window=window, window_t=window_t, threshold=thr, joint=joint,
                                   want_scores=True)
    torch.cuda.synchronize()
    tgr, agr, scr = O.seda_assign(qb, kb, anchors, frames, gh, gw, tile_h=th, tile_w=tw, window=window, window_t=window_t,
                                  threshold=thr, joint=joint)
    got = sc.cpu().numpy().astype(np.float64)
    assert got.shape == scr.shape and np.array_equal(np.isnan(got), np.isnan(scr))
    inside = ~np.isnan(scr)
    if inside.any():
        assert np.abs(got[inside] - scr[inside]).max() <= 2e-5 * np.abs(scr[inside]).max() + 1e-6
        assert not (inside & (np.abs(scr - thr) <= 1e-4 * max(1.0, abs(thr)))).any()     # (seeded input: stays so)
    assert np.array_equal(ag.cpu().numpy(), agr)
    assert np.array_equal(tg.cpu().numpy(), tgr)
    return tg, ag, tgr, agr


def test_seda_assignment_and_the_chain_to_restricted_quantization(F, luts):
    """Sec. 3.4 on the GPU from Q and K: anchors (one per frame and tile) -> correlated tokens -> dialect profile of the
    anchors -> sub-formatbooks -> quantization restricted to them.  The threshold comparison is made on fp32 scores:
    a token whose float64 score lies within 1e-4 of the threshold may fall on either side and is left out of the
    comparison (none is expected on this input); everything else is bit-exact."""
    for frames, heads, gh, gw, dim, th, tw, window, thr in [(3, 4, 12, 16, 64, 4, 4, 5, 6.0), (2, 2, 7, 9, 40, 4, 4, 3, 2.0),
                                                            (1, 1, 4, 4, 8, 2, 2, 8, 0.5), (4, 3, 9, 10, 24, 2, 5, 4, 3.0)]:
        tokens = gh * gw
        q, k = synth.attention_qk(frames * heads, tokens, dim, seed=gh + dim, device="cuda")
        q4, k4 = q.view(frames, heads, tokens, dim), k.view(frames, heads, tokens, dim)
        qb, kb = synth.bf16_bits(q).reshape(frames, heads, tokens, dim), synth.bf16_bits(k).reshape(frames, heads, tokens, dim)
        ref_scores = O.attention_scores(qb.reshape(-1, tokens, dim), kb.reshape(-1, tokens, dim), "abs")
        sc32 = ref_scores.astype(np.float32).reshape(frames, heads, tokens)
        anchors = O.select_salient_tokens(sc32, gh, gw, th, tw)
        _, _, tgr, agr = _assign_case(F, q4, k4, qb, kb, anchors.ravel(), frames, gh, gw, th, tw, window, 1, thr, False)
        assert (tgr >= 0).sum() > anchors.size                      # some correlated tokens beyond the anchors
        # the group of an anchor is its tile, in every frame
        tiles_w = (gw + tw - 1) // tw
        for row in anchors.ravel():
            y, x = divmod(int(row) % tokens, gw)
            assert agr[row] == (y // th) * tiles_w + x // tw
        # dropped entries (a pruned frame's -1, a row past the clip) and a shuffled list
        rng = np.random.default_rng(frames)
        a2 = anchors.ravel().copy()
        a2[::3] = -1
        a2 = np.concatenate([a2, [frames * tokens, -7]])
        rng.shuffle(a2)
        _assign_case(F, q4, k4, qb, kb, a2, frames, gh, gw, th, tw, window, 1, thr, False)
    # the chain on the first shape: 3 frames x 192 tokens, 12 tiles = 12 groups
    frames, heads, gh, gw, dim = 3, 4, 12, 16, 64
    tokens = gh * gw
    q, k = synth.attention_qk(frames * heads, tokens, dim, seed=gh + dim, device="cuda")
    scores = F.fb4_attention_scores(q, k, 0)
    anchors_d = F.fb4_select_salient_tokens(scores.view(frames, heads, tokens), gh, gw)
    tg, ag = F.fb4_seda_assign(q.view(frames, heads, tokens, dim), k.view(frames, heads, tokens, dim), anchors_d, frames, gh, gw,
                               window=5, threshold=6.0)
    x = synth.vdit_activation(rows=frames * tokens, cols=1024, seed=4, device="cuda")
    c, m = F.fb4_quantize(luts, F.opts(), x)
    n_groups = anchors_d.shape[1]
    counts, sub = F.fb4_seda_profile(luts, m, ag, n_groups)
    cs, ms = F.fb4_quantize_seda(luts, F.opts(), x, tg, sub)
    torch.cuda.synchronize()
    tg_h, ag_h = tg.cpu().numpy(), ag.cpu().numpy()
    assert sorted(set(ag_h[ag_h >= 0].tolist())) == list(range(n_groups))
    assert all((ag_h == g).sum() == frames for g in range(n_groups))      # one anchor per frame in every group
    xb = synth.bf16_bits(x)
    cr, mr = O.quantize(DEFAULT_FORMATBOOK, xb)
    counts_r, sub_r = O.seda_profile(DEFAULT_FORMATBOOK, mr, ag_h, n_groups)
    assert np.array_equal(counts.cpu().numpy().astype(np.uint32), counts_r) and np.array_equal(sub.cpu().numpy(), sub_r)
    assert (counts_r.sum(axis=1) == frames * 32).all()              # the anchors of a tile are pooled over the frames
    valid = (sub_r < 32).all(axis=1)                                # (every range bucket has a dialect in the default table)
    assert valid.all()
    csr, msr = O.quantize(DEFAULT_FORMATBOOK, xb, token_group=tg_h, sub_formatbooks=sub_r)
    assert np.array_equal(host_u8(cs), csr) and np.array_equal(host_u16(ms), msr)
    # argument checks
    q4, k4 = q.view(frames, heads, tokens, dim), k.view(frames, heads, tokens, dim)
    with pytest.raises(F.Fb4Error) as e:
        F.fb4_seda_assign(q4, k4, anchors_d, frames, gh, gw, window=9, threshold=6.0)
    assert e.value.code == F.ERR_UNSUPPORTED
    with pytest.raises(F.Fb4Error) as e:
        F.fb4_seda_assign(q4, k4, anchors_d, frames, gh, gw, window=5, window_t=3, threshold=6.0)     # factorized: one frame
    assert e.value.code == F.ERR_INVALID_ARG


def test_seda_main_anchor_pruning_and_the_factorized_chain(F, luts):
    """Sec. 3.4 steps 1-3 for factorized attention: per-frame candidates from the spatial attention, the main anchor of
    every tile from the temporal attention's mean scores, frames pruned by the raw temporal score from the main anchor,
    then the marking step on what is left.  Main anchors and kept lists bit for bit (no score near the threshold)."""
    for frames, heads, gh, gw, dim, th, tw, thr in [(6, 3, 8, 8, 32, 4, 4, 0.0), (16, 4, 12, 16, 64, 4, 4, 2.0), (3, 2, 5, 7, 16, 2, 3, -1.0),
                                                    (40, 1, 4, 4, 8, 4, 4, 1.0)]:
        tokens = gh * gw
        # spatial attention: group = (frame, head); temporal attention: group = (position, head), tokens = frames
        q, k = synth.attention_qk(frames * heads, tokens, dim, seed=frames + dim, device="cuda")
        qt, kt = synth.attention_qk(tokens * heads, frames, dim, seed=frames + dim + 1, device="cuda")
        s_sp = F.fb4_attention_scores(q, k, 0)
        s_t = F.fb4_attention_scores(qt, kt, 1)                     # ReLU for temporal attention (Sec. 3.3)
        cand_d = F.fb4_select_salient_tokens(s_sp.view(frames, heads, tokens), gh, gw, th, tw)
        main, kept, ps = F.fb4_seda_main_anchor(s_t.view(tokens, heads, frames), qt.view(tokens, heads, frames, dim),
                                                kt.view(tokens, heads, frames, dim), cand_d, gh, gw, th, tw, thr, want_scores=True)
        torch.cuda.synchronize()
        cand = cand_d.cpu().numpy()
        ts = s_t.cpu().numpy().reshape(tokens, heads, frames)
        qtb = synth.bf16_bits(qt).reshape(tokens, heads, frames, dim)
        ktb = synth.bf16_bits(kt).reshape(tokens, heads, frames, dim)
        main_r, kept_r, ps_r = O.seda_main_anchor(ts, qtb, ktb, cand, gh, gw, th, tw, thr)
        got = ps.cpu().numpy().astype(np.float64)
        assert np.array_equal(np.isnan(got), np.isnan(ps_r))
        inside = ~np.isnan(ps_r)
        assert np.abs(got[inside] - ps_r[inside]).max() <= 2e-5 * np.abs(ps_r[inside]).max() + 1e-6
        assert not (inside & (np.abs(ps_r - thr) <= 1e-4 * max(1.0, abs(thr)))).any()
        assert np.array_equal(main.cpu().numpy(), main_r)
        assert np.array_equal(kept.cpu().numpy(), kept_r)
        n_kept = int((kept_r >= 0).sum())
        assert (main_r >= 0).all() and frames * 0 < n_kept <= cand.size
        if thr > 0:
            assert n_kept < cand.size                               # the threshold does prune on these inputs
        # step 3 on the kept candidates
        qb = synth.bf16_bits(q).reshape(frames, heads, tokens, dim)
        kb = synth.bf16_bits(k).reshape(frames, heads, tokens, dim)
        _assign_case(F, q.view(frames, heads, tokens, dim), k.view(frames, heads, tokens, dim), qb, kb, kept_r.ravel(), frames, gh, gw,
                     th, tw, 5, 1, 4.0, False)
    # hand-made cases through the kernel: several candidates of one tile in a frame (the first listed counts), entries
    # outside their frame, a tile without candidates, NaN scores, ties
    frames, heads, gh, gw, dim = 3, 2, 4, 4, 8
    tokens = 16
    rng = np.random.default_rng(7)
    ts = rng.random((tokens, heads, frames)).astype(np.float32)
    ts[5, :, 0] = np.nan
    ts[0, :, 1] = ts[0, :, 0]
    cand = np.array([[5, 0, 2, 40], [16 + 0, 16 + 1, -3, 16 + 10], [32 + 7, 32 + 6, 15, 32 + 15]], dtype=np.int32)
    qt, kt = synth.attention_qk(tokens * heads, frames, dim, seed=3, device="cuda")
    main, kept, ps = F.fb4_seda_main_anchor(torch.from_numpy(ts).cuda(), qt.view(tokens, heads, frames, dim),
                                            kt.view(tokens, heads, frames, dim), torch.from_numpy(cand).cuda(), gh, gw, 2, 2, 0.5,
                                            want_scores=True)
    torch.cuda.synchronize()
    main_r, kept_r, ps_r = O.seda_main_anchor(ts, synth.bf16_bits(qt).reshape(tokens, heads, frames, dim),
                                              synth.bf16_bits(kt).reshape(tokens, heads, frames, dim), cand, gh, gw, 2, 2, 0.5)
    assert np.array_equal(main.cpu().numpy(), main_r) and np.array_equal(kept.cpu().numpy(), kept_r)
    assert np.array_equal(np.isnan(ps.cpu().numpy()), np.isnan(ps_r))
    assert main_r[2] == -1                                          # no candidate in tile (1,0)
    with pytest.raises(F.Fb4Error) as e:
        F.fb4_seda_main_anchor(torch.from_numpy(ts).cuda(), qt.view(tokens, heads, frames, dim), kt.view(tokens, heads, frames, dim),
                               torch.from_numpy(cand).cuda(), gh, gw, 2, 2, float("nan"))
    assert e.value.code == F.ERR_INVALID_ARG


def test_seda_3d_attention_main_anchor_and_cuboid_window(F, luts):
    """Sec. 3.4, 3D attention: clip-wide scores -> one main anchor per spatial tile over all frames -> correlated tokens
    inside a cuboid window, then profile and restricted quantization."""
    for frames, heads, gh, gw, dim, th, tw, window, window_t, thr in [(4, 3, 8, 8, 32, 4, 4, 5, 3, 4.0), (5, 2, 6, 10, 16, 2, 5, 3, 5, 1.0),
                                                                      (2, 1, 4, 4, 8, 4, 4, 8, 1, 0.5), (7, 2, 9, 7, 40, 4, 4, 4, 64, 3.0)]:
        tokens = gh * gw
        q, k = synth.attention_qk(heads, frames * tokens, dim, seed=frames * 10 + dim, device="cuda")
        scores = F.fb4_attention_scores(q, k, 0)
        torch.cuda.synchronize()
        sc = scores.cpu().numpy()
        sc[:, ::11] = sc[0, 0]                                      # ties
        sc[0, 5] = np.nan
        anchors = F.fb4_seda_main_anchor_3d(torch.from_numpy(sc).cuda(), frames, gh, gw, th, tw)
        torch.cuda.synchronize()
        anchors_r = O.seda_main_anchor_3d(sc, frames, gh, gw, th, tw)
        assert np.array_equal(anchors.cpu().numpy(), anchors_r)
        qb, kb = synth.bf16_bits(q), synth.bf16_bits(k)
        tg, ag, tgr, agr = _assign_case(F, q, k, qb, kb, anchors_r, frames, gh, gw, th, tw, window, window_t, thr, True)
        assert (agr >= 0).sum() == anchors_r.size and (tgr >= 0).sum() > anchors_r.size
    # the chain on the last shape
    x = synth.vdit_activation(rows=frames * tokens, cols=512, seed=6, device="cuda")
    c, m = F.fb4_quantize(luts, F.opts(), x)
    n_groups = anchors_r.size
    counts, sub = F.fb4_seda_profile(luts, m, ag, n_groups)
    cs, ms = F.fb4_quantize_seda(luts, F.opts(), x, tg, sub)
    torch.cuda.synchronize()
    xb = synth.bf16_bits(x)
    cr, mr = O.quantize(DEFAULT_FORMATBOOK, xb)
    counts_r, sub_r = O.seda_profile(DEFAULT_FORMATBOOK, mr, agr, n_groups)
    assert np.array_equal(counts.cpu().numpy().astype(np.uint32), counts_r) and np.array_equal(sub.cpu().numpy(), sub_r)
    csr, msr = O.quantize(DEFAULT_FORMATBOOK, xb, token_group=tgr, sub_formatbooks=sub_r)
    assert np.array_equal(host_u8(cs), csr) and np.array_equal(host_u16(ms), msr)
