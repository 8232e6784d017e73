"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, validates its arguments before touching the GPU, and builds
lookup tables that agree with the oracle's brute-force rounding (Sec. 3.2)."""

import ctypes
import os
import re

import numpy as np
import pytest

import paper_2603_02883_amd as F
from paper_2603_02883_amd import binding as B
from fb4_inputs import DEFAULT_FORMATBOOK, E2M1_X2_FORMATBOOK
from oracle import fb4_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    text = open(os.path.join(ROOT, "include", "fb4.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fb4_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    syms = header_symbols()
    assert {"fb4_build_luts", "fb4_quantize", "fb4_quantize_seda", "fb4_decompose", "fb4_dequantize"} <= set(syms)
    lib = B.lib()
    for s in syms:
        assert hasattr(lib, s), s
    assert sorted(B.EXPORTS) == syms
    assert F.version() >= 100 and F.workspace_bytes() == 0
    for code in (0, -1, -2, -3, -4, -99):
        assert isinstance(F.strerror(code), str) and F.strerror(code)


def test_binding_has_no_cpu_fallback():
    src = open(os.path.join(ROOT, "paper_2603_02883_amd", "binding.py")).read()
    assert "oracle" not in src.replace("no CPU fallback", "")
    csrc = os.path.join(ROOT, "paper_2603_02883_amd", "csrc")
    for f in os.listdir(csrc):
        assert "oracle" not in open(os.path.join(csrc, f)).read()
    assert "paper_2603_02883_amd" not in open(os.path.join(ROOT, "oracle", "fb4_oracle.py")).read()
    assert "fb4.h" not in open(os.path.join(ROOT, "oracle", "fb4_oracle.c")).read()


# ------------------------------------------------------------ lookup tables
def _blob_views(blob):
    v = {}
    v["qerr8"] = blob[0:1024].reshape(32, 32)
    v["qval"] = blob[1024:3072].reshape(32, 64)
    v["qerr16"] = blob[3072:5120].view(np.uint16).reshape(32, 32)
    v["mag16"] = blob[5120:7168].view(np.uint16).reshape(32, 32)
    v["gain16"] = blob[7168:9216].view(np.uint16).reshape(32, 32)
    v["decode"] = blob[9216:9728].view(np.uint16).reshape(32, 8)
    v["top"] = blob[9728:9760]
    v["n"] = int(blob[9760:9764].view(np.int32)[0])
    v["qvalT"] = blob[9792:10816].reshape(32, 32)
    v["range_excl"] = blob[10816:11072].reshape(8, 32)
    return v


def _f2b(a):
    u = np.asarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return (((u + 0x7FFF + ((u >> 16) & 1)) >> 16) & 0xFFFF).astype(np.uint16)


def test_qvalue_table_equals_oracle_rounding_on_bin_edges_and_midpoints():
    """Sec. 3.2: a 0.5-wide bin maps to one exact index.  The oracle knows no
    bins; it is asked for the left edge (a tie whenever the edge is a decision
    boundary), the midpoint and the last bf16 value of every bin."""
    blob = F.fb4_build_luts_host(DEFAULT_FORMATBOOK)
    v = _blob_views(blob)
    assert v["n"] == 32
    for d in range(32):
        one = DEFAULT_FORMATBOOK[d:d + 1]
        x = np.zeros((32, 32), dtype=np.float32)
        x[:, 0] = 8.0                                   # fixes e = 3
        b = np.arange(32, dtype=np.float32)
        x[:, 1] = b / 2
        x[:, 2] = b / 2 + 0.25
        x[:, 3] = -(b / 2 + 0.25)
        xb = _f2b(x)
        # largest bf16 value below the next bin edge
        nxt = _f2b((b + 1) / 2)
        xb[:, 4] = nxt - 1
        codes, meta = O.quantize(one, xb, selector=O.SEL_SSE)
        assert ((meta >> 8) == 130).all()
        lo, hi = codes & 0xF, codes >> 4
        nib = np.stack([lo, hi], axis=-1).reshape(32, -1)
        for col in (1, 2, 4):
            assert np.array_equal(nib[:, col], v["qval"][d, :32])
        assert np.array_equal(nib[:, 3], v["qval"][d, 32:])            # sign folded into the table
        mag = DEFAULT_FORMATBOOK[d][v["qval"][d, :32] & 7].astype(int)
        assert np.array_equal(v["mag16"][:, d], mag)
        mid4 = 2 * np.arange(32) + 1
        assert np.array_equal(v["qerr8"][:, d], np.abs(mid4 - 4 * mag))  # |midpoint - magnitude| in quarters
        assert (v["qerr8"][:, d] % 2 == 1).all()
        assert np.array_equal(v["qerr16"][:, d], 32 * v["qerr8"][:, d].astype(int))
        assert np.array_equal(v["gain16"][:, d], mag * (np.arange(32) - mag))
        assert v["top"][d] == DEFAULT_FORMATBOOK[d, 7]
        assert np.array_equal(v["qvalT"][:, d], v["qval"][d, :32])
        dec = (v["decode"][d].astype(np.uint32) << 16).view(np.float32)
        assert np.array_equal(dec, DEFAULT_FORMATBOOK[d].astype(np.float32))


def test_qerror_sum_equals_oracle_score(fbk=DEFAULT_FORMATBOOK):
    """Summing the table over the bins of the group maxima reproduces the
    oracle's score for every dialect (quarter units)."""
    blob = F.fb4_build_luts_host(fbk)
    v = _blob_views(blob)
    rng = np.random.default_rng(3)
    for g in (8, 32):
        for _ in range(30):
            x = _f2b(rng.standard_t(3, size=32).astype(np.float32) * 5)
            cand, scores, did, e = O.block_scores(fbk, x, selector=O.SEL_LUT, num_groups=g)
            xv = (x.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
            xhat = np.abs(xv) * 2.0 ** (3 - e)
            gmax = xhat.reshape(g, -1).max(axis=1)
            bins = np.minimum(31, np.floor(2 * gmax)).astype(int)
            table = v["qerr8"][bins, :].astype(int).sum(axis=0)
            assert np.array_equal(table, (scores * 4).astype(int))


def test_range_exclusion_rows():
    v = _blob_views(F.fb4_build_luts_host(DEFAULT_FORMATBOOK))
    tops = DEFAULT_FORMATBOOK[:, 7].astype(int)
    for r in range(8):
        assert np.array_equal(v["range_excl"][r] == 0, tops == 8 + r)
    v = _blob_views(F.fb4_build_luts_host(DEFAULT_FORMATBOOK[[0, 3, 9]]))      # ranges 8, 9, 11 only
    assert (v["range_excl"][[2, 4, 5, 6, 7]] == 0).all()                        # absent range: no filter
    assert v["range_excl"][0].tolist() == [0] + [255] * 31
    assert v["range_excl"][3].tolist() == [255, 255, 0] + [255] * 29


def test_unused_dialects_can_never_win():
    blob = F.fb4_build_luts_host(E2M1_X2_FORMATBOOK)
    v = _blob_views(blob)
    assert v["n"] == 1
    assert (v["qerr8"][:, 1:] == 31).all() and (v["gain16"][:, 1:] == 0).all() and (v["mag16"][:, 1:] == 0).all()
    assert (v["qerr8"][:, 0] <= 31).all()


# ------------------------------------------------------------- error paths
def _call_quantize(luts, o, x, rows, cols, stride, codes, meta):
    return B.lib().fb4_quantize(luts, ctypes.byref(o) if o is not None else None, x, rows, cols, stride,
                                codes, meta, None)


def test_argument_validation_happens_before_any_gpu_work():
    lib = B.lib()
    fake = ctypes.create_string_buffer(16384)               # stands in for a handle; never dereferenced
    h = ctypes.cast(fake, ctypes.c_void_p)
    buf = ctypes.create_string_buffer(4096 + 64)
    base = ctypes.addressof(buf)
    al = (base + 63) // 64 * 64
    P = ctypes.c_void_p
    good = F.opts()
    # null handle / null opts / bad options
    assert _call_quantize(None, good, P(al), 1, 32, 32, P(al), P(al)) == F.ERR_INVALID_ARG
    assert _call_quantize(h, None, P(al), 1, 32, 32, P(al), P(al)) == F.ERR_INVALID_ARG
    assert _call_quantize(h, F.opts(selector=7), P(al), 1, 32, 32, P(al), P(al)) == F.ERR_INVALID_ARG
    assert _call_quantize(h, F.opts(num_groups=5), P(al), 1, 32, 32, P(al), P(al)) == F.ERR_INVALID_ARG
    assert _call_quantize(h, F.opts(block=24), P(al), 1, 32, 32, P(al), P(al)) == F.ERR_INVALID_ARG
    assert _call_quantize(h, F.opts(flags=8), P(al), 1, 32, 32, P(al), P(al)) == F.ERR_INVALID_ARG
    assert _call_quantize(h, F.opts(block=16, num_groups=32), P(al), 1, 32, 32, P(al), P(al)) == F.ERR_INVALID_ARG
    assert _call_quantize(h, F.opts(block=16), P(al), 1, 40, 40, P(al), P(al)) == F.ERR_UNSUPPORTED  # cols % 16
    # shapes
    assert _call_quantize(h, good, P(al), -1, 32, 32, P(al), P(al)) == F.ERR_INVALID_ARG
    assert _call_quantize(h, good, P(al), 1, 64, 32, P(al), P(al)) == F.ERR_INVALID_ARG      # stride < cols
    assert _call_quantize(h, good, P(al), 1, 40, 40, P(al), P(al)) == F.ERR_UNSUPPORTED      # cols % block
    assert _call_quantize(h, good, P(al), 0, 32, 32, None, None) == F.OK                     # empty: no-op
    assert _call_quantize(h, good, P(al), 4, 0, 0, None, None) == F.OK
    # null tensors, alignment
    assert _call_quantize(h, good, None, 1, 32, 32, P(al), P(al)) == F.ERR_INVALID_ARG
    assert _call_quantize(h, good, P(al), 1, 32, 32, None, P(al)) == F.ERR_INVALID_ARG
    assert _call_quantize(h, good, P(al + 2), 1, 32, 32, P(al), P(al)) == F.ERR_UNSUPPORTED
    assert _call_quantize(h, good, P(al), 2, 32, 36, P(al), P(al)) == F.ERR_UNSUPPORTED      # stride % 8
    assert _call_quantize(h, good, P(al), 1, 32, 32, P(al), P(al + 1)) == F.ERR_UNSUPPORTED
    # seda
    q = lib.fb4_quantize_seda
    assert q(h, ctypes.byref(good), P(al), 1, 32, 32, None, P(al), 4, P(al), P(al), None) == F.ERR_INVALID_ARG
    assert q(h, ctypes.byref(good), P(al), 1, 32, 32, P(al), P(al), 0, P(al), P(al), None) == F.ERR_INVALID_ARG
    # decompose
    d = lib.fb4_decompose
    assert d(h, ctypes.byref(good), P(al), 4, 32, 32, P(al), P(al), P(al), -1, None, None, 0, P(al), P(al),
             None) == F.ERR_INVALID_ARG
    assert d(h, ctypes.byref(good), P(al), 4, 32, 32, P(al), P(al), P(al), 9, None, None, 0, P(al), P(al),
             None) == F.ERR_INVALID_ARG                                                    # n_sal > rows
    assert d(h, ctypes.byref(good), P(al), 4, 32, 32, None, P(al), P(al), 1, None, None, 0, P(al), P(al),
             None) == F.ERR_INVALID_ARG
    assert d(h, ctypes.byref(good), P(al), 4, 32, 32, P(al), P(al), P(al), 1, P(al), None, 0, P(al), P(al),
             None) == F.ERR_INVALID_ARG                                                    # half a SeDA spec
    assert d(h, ctypes.byref(good), P(al), 4, 32, 32, P(al), P(al), P(al), 0, None, None, 0, None, None,
             None) == F.OK                                                                 # nothing salient
    # dequantize
    dq = lib.fb4_dequantize
    assert dq(None, P(al), P(al), 1, 32, 32, None, None, None, 0, P(al), 0, 32, None) == F.ERR_INVALID_ARG
    assert dq(h, P(al), P(al), 1, 32, 32, None, None, None, 0, P(al), 5, 32, None) == F.ERR_INVALID_ARG
    assert dq(h, P(al), P(al), 1, 32, 32, None, None, None, 2, P(al), 0, 32, None) == F.ERR_INVALID_ARG
    assert dq(h, P(al), P(al), 1, 40, 16, None, None, None, 0, P(al), 0, 40, None) == F.ERR_UNSUPPORTED
    assert dq(h, P(al), P(al), 1, 32, 32, None, None, None, 0, P(al + 16), 1, 32, None) == F.ERR_UNSUPPORTED
    assert dq(h, P(al), P(al), 0, 32, 32, None, None, None, 0, None, 0, 32, None) == F.OK


def test_build_luts_rejects_bad_formatbooks_on_the_host():
    bad = DEFAULT_FORMATBOOK.copy()
    bad[4, 0] = 1
    with pytest.raises(F.Fb4Error) as e:
        F.fb4_build_luts_host(bad)
    assert e.value.code == F.ERR_INVALID_ARG
    with pytest.raises(F.Fb4Error):
        F.fb4_build_luts(bad)                                # rejected before any HIP call
    with pytest.raises(F.Fb4Error):
        F.fb4_build_luts_host(np.zeros((33, 8), np.uint8))
    size = ctypes.c_size_t(0)
    fb = np.ascontiguousarray(DEFAULT_FORMATBOOK)
    rc = B.lib().fb4_build_luts_host(fb.ctypes.data_as(ctypes.c_void_p), 32, None, 0, ctypes.byref(size))
    assert rc == F.OK and size.value == B.BLOB_BYTES
    small = np.zeros(16, np.uint8)
    rc = B.lib().fb4_build_luts_host(fb.ctypes.data_as(ctypes.c_void_p), 32, small.ctypes.data_as(ctypes.c_void_p),
                                     16, ctypes.byref(size))
    assert rc == F.ERR_INVALID_ARG


def test_header_is_plain_c(tmp_path):
    """include/fb4.h must compile as C (no C++ or HIP types in the boundary) and as C++."""
    import subprocess
    src = tmp_path / "use_fb4.c"
    src.write_text('#include "fb4.h"\n'
                   "int use(const fb4_luts* l, const fb4_opts* o, const void* x, unsigned char* c, unsigned short* m) {\n"
                   "    return fb4_quantize(l, o, x, 1, 32, 32, c, m, (void*)0) + fb4_version();\n"
                   "}\n")
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-I", inc, str(src)], check=True)
    cpp = tmp_path / "use_fb4.cpp"
    cpp.write_text(src.read_text())
    subprocess.run(["g++", "-std=c++11", "-Wall", "-Werror", "-fsyntax-only", "-I", inc, str(cpp)], check=True)


def test_gelu_table_equals_the_oracle_on_every_pattern_it_covers():
    """The host-built table of fb4_gelu_quantize against the oracle's GeLU: every positive bf16 pattern, every
    negative one down to -16, and everything below -16 (which shares the entry of -16) is -0 in the oracle too."""
    from oracle import fb4_oracle as O
    allb = np.arange(65536, dtype=np.uint16)
    for approximate in (0, 1):
        t = F.fb4_gelu_table_host(approximate)
        assert t.size == 0xC181
        ref = O.gelu(allb, approximate)
        assert np.array_equal(t, ref[:0xC181])
        beyond = allb[(allb > 0xC180) & (allb <= 0xFF80)]            # -16 > x >= -Inf
        assert (ref[beyond] == 0x8000).all() and t[0xC180] == 0x8000
        assert (ref[allb > 0xFF80] == 0x7FC0).all()                   # negative NaNs: patched in the kernel
        # the runs the kernel fills in from the bit pattern instead of reading them: x / 2 for 2^-125 <= |x| <
        # 2^-9.25, x from 2.875 upwards, the quiet NaN for positive NaNs
        k = np.arange(0xC181)
        half = ((k & 0x7FFF) >= 0x0100) & ((k & 0x7FFF) < 0x3B00)
        assert np.array_equal(t[half], (k[half] - 0x80).astype(np.uint16))
        ident = (k >= 0x4038) & (k <= 0x7F80)
        assert np.array_equal(t[ident], k[ident].astype(np.uint16)) and (t[0x7F81:0x8000] == 0x7FC0).all()
    with pytest.raises(F.Fb4Error):
        F.fb4_gelu_table_host(2)


def test_argument_validation_of_the_attention_guided_entry_points():
    """Every check below returns before any GPU work: no device is needed (pointers are host buffers that are
    never dereferenced)."""
    lib = B.lib()
    buf = ctypes.create_string_buffer(4096 + 64)
    al = (ctypes.addressof(buf) + 63) // 64 * 64
    P = ctypes.c_void_p
    a = lib.fb4_attention_scores
    assert a(P(al), P(al), 0, 16, 64, 0, P(al), None) == F.OK                       # no groups: no-op
    assert a(P(al), P(al), 2, 0, 64, 0, P(al), None) == F.OK                        # no tokens: no-op
    assert a(P(al), P(al), -1, 16, 64, 0, P(al), None) == F.ERR_INVALID_ARG
    assert a(P(al), P(al), 2, 16, 64, 2, P(al), None) == F.ERR_INVALID_ARG          # mode
    assert a(None, P(al), 2, 16, 64, 0, P(al), None) == F.ERR_INVALID_ARG
    assert a(P(al), P(al), 2, 16, 64, 0, None, None) == F.ERR_INVALID_ARG
    assert a(P(al), P(al), 2, 16, 0, 0, P(al), None) == F.ERR_INVALID_ARG           # no channels
    assert a(P(al), P(al), 2, 16, 60, 0, P(al), None) == F.ERR_UNSUPPORTED          # channels % 8
    assert a(P(al), P(al), 2, 16, 264, 0, P(al), None) == F.ERR_UNSUPPORTED         # channels > 256
    assert a(P(al + 8), P(al), 2, 16, 64, 0, P(al), None) == F.ERR_UNSUPPORTED      # alignment
    s = lib.fb4_select_salient_tokens
    assert s(P(al), 0, 2, 8, 8, 4, 4, P(al), None) == F.OK                          # no frames
    assert s(P(al), 2, 0, 8, 8, 4, 4, P(al), None) == F.ERR_INVALID_ARG             # no heads
    assert s(P(al), 2, 2, 8, 8, 0, 4, P(al), None) == F.ERR_INVALID_ARG             # tile height 0
    assert s(None, 2, 2, 8, 8, 4, 4, P(al), None) == F.ERR_INVALID_ARG
    assert s(P(al), 2, 2, 128, 128, 4, 4, P(al), None) == F.ERR_UNSUPPORTED         # more than 8192 tokens
    g = lib.fb4_seda_assign
    ok_args = dict(q=P(al), k=P(al), joint=0, frames=2, heads=2, gh=8, gw=8, dim=64, anchors=P(al), n=4, th=4, tw=4, window=5,
                   wt=1, thr=5.0, tg=P(al), ag=P(al), sc=None)

    def assign(**kw):
        v = dict(ok_args, **kw)
        return g(v["q"], v["k"], v["joint"], v["frames"], v["heads"], v["gh"], v["gw"], v["dim"], v["anchors"], v["n"], v["th"],
                 v["tw"], v["window"], v["wt"], v["thr"], v["tg"], v["ag"], v["sc"], None)
    assert assign(frames=0) == F.OK
    assert assign(joint=2) == F.ERR_INVALID_ARG
    assert assign(wt=3) == F.ERR_INVALID_ARG                                        # no scores across frames without joint
    assert assign(thr=float("nan")) == F.ERR_INVALID_ARG
    assert assign(window=0) == F.ERR_INVALID_ARG
    assert assign(tg=None) == F.ERR_INVALID_ARG
    assert assign(anchors=None) == F.ERR_INVALID_ARG
    assert assign(window=9) == F.ERR_UNSUPPORTED
    assert assign(joint=1, wt=65) == F.ERR_UNSUPPORTED
    assert assign(dim=60) == F.ERR_UNSUPPORTED
    assert assign(q=P(al + 2)) == F.ERR_UNSUPPORTED
    m = lib.fb4_seda_main_anchor

    def main(ts=P(al), qt=P(al), kt=P(al), frames=3, heads=2, gh=8, gw=8, dim=64, cand=P(al), n=4, th=4, tw=4, thr=3.0,
             out=P(al), kept=P(al), sc=None):
        return m(ts, qt, kt, frames, heads, gh, gw, dim, cand, n, th, tw, thr, out, kept, sc, None)
    assert main(heads=0) == F.ERR_INVALID_ARG
    assert main(thr=float("nan")) == F.ERR_INVALID_ARG
    assert main(out=None) == F.ERR_INVALID_ARG
    assert main(kept=None) == F.ERR_INVALID_ARG
    assert main(cand=None) == F.ERR_INVALID_ARG
    assert main(frames=1025) == F.ERR_UNSUPPORTED
    assert main(dim=12) == F.ERR_UNSUPPORTED
    assert main(qt=P(al + 4)) == F.ERR_UNSUPPORTED
    d3 = lib.fb4_seda_main_anchor_3d
    assert d3(P(al), 0, 2, 8, 8, 4, 4, P(al), None) == F.ERR_INVALID_ARG            # no frames
    assert d3(None, 2, 2, 8, 8, 4, 4, P(al), None) == F.ERR_INVALID_ARG
    assert d3(P(al), 2, 2, 8, 8, 4, 4, None, None) == F.ERR_INVALID_ARG
    assert d3(P(al + 2), 2, 2, 8, 8, 4, 4, P(al), None) == F.ERR_UNSUPPORTED
    pr = lib.fb4_probe_mfma_rate
    assert pr(0, 1, 1, P(al), None, None) == F.ERR_INVALID_ARG
    assert pr(70000, 1, 1, P(al), None, None) == F.ERR_INVALID_ARG
    assert pr(8, -1, 1, P(al), None, None) == F.ERR_INVALID_ARG
    assert pr(8, 1, 1, None, None, None) == F.ERR_INVALID_ARG


def test_argument_validation_of_the_fused_producers():
    lib = B.lib()
    fake = ctypes.create_string_buffer(16384)               # stands in for a handle; never dereferenced
    h = ctypes.cast(fake, ctypes.c_void_p)
    buf = ctypes.create_string_buffer(4096 + 64)
    al = (ctypes.addressof(buf) + 63) // 64 * 64
    P = ctypes.c_void_p
    good = F.opts()
    ln = lib.fb4_layernorm_quantize

    def layernorm(handle=h, o=good, x=P(al), rows=2, cols=64, stride=64, gamma=P(al), beta=P(al), eps=1e-6, tg=None, sub=None,
                  ng=0, codes=P(al), meta=P(al), y=None):
        return ln(handle, ctypes.byref(o) if o is not None else None, x, rows, cols, stride, gamma, beta, eps, tg, sub, ng,
                  codes, meta, y, None)
    assert layernorm(handle=None) == F.ERR_INVALID_ARG
    assert layernorm(o=None) == F.ERR_INVALID_ARG
    assert layernorm(rows=0, codes=None, meta=None) == F.OK
    assert layernorm(eps=-1.0) == F.ERR_INVALID_ARG
    assert layernorm(eps=float("nan")) == F.ERR_INVALID_ARG
    assert layernorm(x=None) == F.ERR_INVALID_ARG
    assert layernorm(tg=P(al)) == F.ERR_INVALID_ARG                                 # half a SeDA spec
    assert layernorm(o=F.opts(selector=0)) == F.ERR_UNSUPPORTED                     # the online selector only
    assert layernorm(o=F.opts(num_groups=32)) == F.ERR_UNSUPPORTED
    assert layernorm(cols=40, stride=40) == F.ERR_UNSUPPORTED                       # whole 32-element chunks
    assert layernorm(cols=12320, stride=12320) == F.ERR_UNSUPPORTED                 # rows longer than 12288
    assert layernorm(gamma=P(al + 2)) == F.ERR_UNSUPPORTED
    ge = lib.fb4_gelu_quantize

    def gelu(handle=h, o=good, x=P(al), rows=2, cols=64, stride=64, approx=1, tg=None, sub=None, ng=0, codes=P(al), meta=P(al)):
        return ge(handle, ctypes.byref(o) if o is not None else None, x, rows, cols, stride, approx, tg, sub, ng, codes, meta, None)
    assert gelu(handle=None) == F.ERR_INVALID_ARG
    assert gelu(approx=2) == F.ERR_INVALID_ARG
    assert gelu(rows=0, codes=None, meta=None) == F.OK
    assert gelu(o=F.opts(selector=0)) == F.ERR_UNSUPPORTED
    assert gelu(o=F.opts(num_groups=32)) == F.ERR_UNSUPPORTED
    assert gelu(cols=48, stride=48) == F.ERR_UNSUPPORTED
    assert gelu(sub=P(al), ng=3) == F.ERR_INVALID_ARG                               # half a SeDA spec
