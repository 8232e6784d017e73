"""Thin ctypes binding of libfb4.so: the same entry points as include/fb4.h.

Argument marshalling only -- every step of the quantizer runs in the library's
HIP kernels.  PyTorch tensors are used for device memory and for the current
stream; nothing here computes on them.  There is no CPU fallback: if the
library is not there it is compiled once (hipcc), and if that fails importing
this module raises.
"""

import ctypes
import os

import numpy as np
import torch

from . import build as _build

OK = 0
ERR_INVALID_ARG = -1
ERR_UNSUPPORTED = -2
ERR_ALLOC = -3
ERR_HIP = -4

SEL_SSE = 0
SEL_LUT = 1
FLAG_TWO_STAGE = 1
DTYPE_BF16 = 0
DTYPE_F32 = 1

BLOB_BYTES = 11072


class Fb4Error(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s: %s (%d)" % (where, strerror(code), code))


class fb4_opts(ctypes.Structure):
    _fields_ = [("block", ctypes.c_int32), ("selector", ctypes.c_int32),
                ("num_groups", ctypes.c_int32), ("flags", ctypes.c_uint32)]


def _load():
    if not os.path.exists(_build.LIB):
        # nothing built yet (fresh checkout): compile once; an existing library is loaded as it is
        try:
            _build.build(force=True)
        except Exception as e:   # no compiler, compile error: fail loudly, there is no CPU fallback
            raise ImportError("libfb4.so is not built and could not be compiled (%s); run "
                              "`python paper_2603_02883_amd/build.py`; there is no CPU fallback" % e)
    lib = ctypes.CDLL(_build.LIB)
    p, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    lib.fb4_version.restype = i32
    lib.fb4_strerror.restype = ctypes.c_char_p
    lib.fb4_strerror.argtypes = [i32]
    lib.fb4_workspace_bytes.restype = ctypes.c_size_t
    lib.fb4_build_luts.argtypes = [p, i32, ctypes.POINTER(p)]
    lib.fb4_build_luts_host.argtypes = [p, i32, p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t)]
    lib.fb4_free_luts.argtypes = [p]
    lib.fb4_free_luts.restype = None
    lib.fb4_quantize.argtypes = [p, ctypes.POINTER(fb4_opts), p, i64, i64, i64, p, p, p]
    lib.fb4_quantize_seda.argtypes = [p, ctypes.POINTER(fb4_opts), p, i64, i64, i64, p, p, i32, p, p, p]
    lib.fb4_decompose.argtypes = [p, ctypes.POINTER(fb4_opts), p, i64, i64, i64, p, p, p, i64, p, p, i32,
                                  p, p, p]
    lib.fb4_dequantize.argtypes = [p, p, p, i64, i64, i32, p, p, p, i64, p, i32, i64, p]
    lib.fb4_quantize_decompose.argtypes = [p, ctypes.POINTER(fb4_opts), p, i64, i64, i64, p, p, i32, p, i64, p, p, p, p, p]
    lib.fb4_seda_profile.argtypes = [p, p, i64, i64, p, i32, p, p, p]
    lib.fb4_repack_mxfp8.argtypes = [p, p, p, i64, i64, i32, p, i64, p, p]
    lib.fb4_attention_scores.argtypes = [p, p, i64, i64, i64, i32, p, p]
    lib.fb4_select_salient_tokens.argtypes = [p, i64, i32, i32, i32, i32, i32, p, p]
    lib.fb4_seda_assign.argtypes = [p, p, i32, i64, i32, i32, i32, i64, p, i64, i32, i32, i32, i32, ctypes.c_float, p, p,
                                    p, p]
    lib.fb4_seda_main_anchor.argtypes = [p, p, p, i64, i32, i32, i32, i64, p, i32, i32, i32, ctypes.c_float, p, p, p, p]
    lib.fb4_seda_main_anchor_3d.argtypes = [p, i64, i32, i32, i32, i32, i32, p, p]
    lib.fb4_probe_mfma_rate.argtypes = [i64, i64, i32, p, ctypes.POINTER(ctypes.c_double), p]
    lib.fb4_gelu_table_host.argtypes = [i32, p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t)]
    lib.fb4_gelu_quantize.argtypes = [p, ctypes.POINTER(fb4_opts), p, i64, i64, i64, i32, p, p, i32, p, p, p]
    lib.fb4_layernorm_quantize.argtypes = [p, ctypes.POINTER(fb4_opts), p, i64, i64, i64, p, p, ctypes.c_float, p, p, i32,
                                           p, p, p, p]
    return lib


_lib = _load()

EXPORTS = ["fb4_version", "fb4_strerror", "fb4_workspace_bytes", "fb4_build_luts", "fb4_build_luts_host",
           "fb4_free_luts", "fb4_quantize", "fb4_quantize_seda", "fb4_decompose", "fb4_dequantize",
           "fb4_quantize_decompose", "fb4_seda_profile",
           "fb4_repack_mxfp8", "fb4_layernorm_quantize", "fb4_gelu_quantize",
           "fb4_gelu_table_host", "fb4_attention_scores", "fb4_select_salient_tokens",
           "fb4_seda_assign", "fb4_seda_main_anchor", "fb4_seda_main_anchor_3d", "fb4_probe_mfma_rate"]


def lib():
    """The loaded ctypes library (for tests that call the C ABI directly)."""
    return _lib


def version():
    return int(_lib.fb4_version())


def strerror(code):
    return _lib.fb4_strerror(int(code)).decode()


def workspace_bytes():
    return int(_lib.fb4_workspace_bytes())


def _dp(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check(rc, where):
    if rc != OK:
        raise Fb4Error(rc, where)


def opts(block=32, selector=SEL_LUT, num_groups=8, flags=0):
    return fb4_opts(block, selector, num_groups, flags)


class Luts:
    """Owner of an fb4_luts handle."""

    def __init__(self, handle, n_dialects):
        self.handle = handle
        self.n_dialects = n_dialects

    def free(self):
        if self.handle:
            _lib.fb4_free_luts(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def fb4_build_luts_host(formatbook):
    """Lookup-table blob as a uint8 numpy array (no GPU needed)."""
    fbk = np.ascontiguousarray(formatbook, dtype=np.uint8)
    blob = np.zeros(BLOB_BYTES, dtype=np.uint8)
    size = ctypes.c_size_t(0)
    rc = _lib.fb4_build_luts_host(fbk.ctypes.data_as(ctypes.c_void_p), fbk.shape[0] if fbk.ndim == 2 else 0,
                                  blob.ctypes.data_as(ctypes.c_void_p), blob.size, ctypes.byref(size))
    _check(rc, "fb4_build_luts_host")
    assert size.value == BLOB_BYTES
    return blob


def fb4_build_luts(formatbook):
    fbk = np.ascontiguousarray(formatbook, dtype=np.uint8)
    h = ctypes.c_void_p(None)
    rc = _lib.fb4_build_luts(fbk.ctypes.data_as(ctypes.c_void_p), fbk.shape[0] if fbk.ndim == 2 else 0,
                             ctypes.byref(h))
    _check(rc, "fb4_build_luts")
    return Luts(h, fbk.shape[0])


def fb4_free_luts(luts):
    luts.free()


def fb4_quantize(luts, o, x, codes=None, meta=None, stream=None):
    """x: bf16 cuda tensor [rows][cols] (row stride allowed).  Returns (codes, meta)."""
    rows, cols = x.shape
    if codes is None:
        codes = torch.empty((rows, cols // 2), dtype=torch.uint8, device=x.device)
    if meta is None:
        meta = torch.empty((rows, cols // o.block), dtype=torch.int16, device=x.device)
    rc = _lib.fb4_quantize(luts.handle, ctypes.byref(o), _dp(x), rows, cols, x.stride(0) if rows > 1 else cols,
                           _dp(codes), _dp(meta), _stream(stream))
    _check(rc, "fb4_quantize")
    return codes, meta


def fb4_layernorm_quantize(luts, o, x, gamma=None, beta=None, eps=1e-6, codes=None, meta=None, stream=None,
                           token_group=None, sub_formatbooks=None, y_out=None):
    """LayerNorm over the channels of each row (gamma, beta: float32 cuda [cols] or None), then quantize, in one
    pass; token_group / sub_formatbooks as in fb4_quantize_seda (optional); y_out: bf16 cuda [rows][cols] that
    receives the producer's result (checks only).  Returns (codes, meta)."""
    rows, cols = x.shape
    if codes is None:
        codes = torch.empty((rows, cols // 2), dtype=torch.uint8, device=x.device)
    if meta is None:
        meta = torch.empty((rows, cols // o.block), dtype=torch.int16, device=x.device)
    rc = _lib.fb4_layernorm_quantize(luts.handle, ctypes.byref(o), _dp(x), rows, cols,
                                     x.stride(0) if rows > 1 else cols, _dp(gamma), _dp(beta), float(eps),
                                     _dp(token_group), _dp(sub_formatbooks),
                                     0 if sub_formatbooks is None else sub_formatbooks.shape[0],
                                     _dp(codes), _dp(meta), _dp(y_out), _stream(stream))
    _check(rc, "fb4_layernorm_quantize")
    return codes, meta


def fb4_attention_scores(q, k, mode=0, scores=None, stream=None):
    """q, k: bf16 cuda [groups][tokens][dim].  mode 0: mean |Q.K^T| over the keys, 1: mean max(Q.K^T, 0).
    Returns float32 [groups][tokens]."""
    groups, tokens, dim = q.shape
    if scores is None:
        scores = torch.empty((groups, tokens), dtype=torch.float32, device=q.device)
    _check(_lib.fb4_attention_scores(_dp(q), _dp(k), groups, tokens, dim, int(mode), _dp(scores), _stream(stream)),
           "fb4_attention_scores")
    return scores


def fb4_select_salient_tokens(scores, grid_h, grid_w, tile_h=4, tile_w=4, rows_out=None, stream=None):
    """scores: float32 cuda [frames][heads][grid_h * grid_w].  Returns int32 [frames][tiles]: one row per tile,
    ascending within a frame, as rows of the [frames * tokens] tensor."""
    frames, heads, tokens = scores.shape
    assert tokens == grid_h * grid_w
    tiles = ((grid_h + tile_h - 1) // tile_h) * ((grid_w + tile_w - 1) // tile_w)
    if rows_out is None:
        rows_out = torch.empty((frames, tiles), dtype=torch.int32, device=scores.device)
    _check(_lib.fb4_select_salient_tokens(_dp(scores), frames, heads, grid_h, grid_w, tile_h, tile_w, _dp(rows_out),
                                          _stream(stream)), "fb4_select_salient_tokens")
    return rows_out


def fb4_seda_assign(q, k, anchors, frames, grid_h, grid_w, tile_h=4, tile_w=4, window=5, window_t=1, threshold=5.0,
                    joint=False, want_scores=False, stream=None, token_group=None, anchor_group=None):
    """q, k: bf16 cuda [frames][heads][tokens][dim] (joint=False) or [heads][frames * tokens][dim] (joint=True);
    anchors: int32 cuda, any shape, rows of the [frames * tokens] activation.  Returns (token_group, anchor_group)
    int32 [frames * tokens] (and the compared scores, float32 [n_anchors][window_t * window^2], if asked)."""
    heads, dim = (q.shape[0], q.shape[2]) if joint else (q.shape[1], q.shape[3])
    tokens = grid_h * grid_w
    n = anchors.numel()
    tg = torch.empty(frames * tokens, dtype=torch.int32, device=q.device) if token_group is None else token_group
    ag = torch.empty(frames * tokens, dtype=torch.int32, device=q.device) if anchor_group is None else anchor_group
    sc = torch.empty((n, window_t * window * window), dtype=torch.float32, device=q.device) if want_scores else None
    _check(_lib.fb4_seda_assign(_dp(q), _dp(k), 1 if joint else 0, frames, heads, grid_h, grid_w, dim, _dp(anchors), n,
                                tile_h, tile_w, window, window_t, float(threshold), _dp(tg), _dp(ag), _dp(sc),
                                _stream(stream)), "fb4_seda_assign")
    return (tg, ag, sc) if want_scores else (tg, ag)


def fb4_seda_main_anchor(temporal_scores, qt, kt, candidates, grid_h, grid_w, tile_h=4, tile_w=4, prune_threshold=3.0,
                         want_scores=False, stream=None, main_anchor=None, kept=None):
    """temporal_scores: float32 cuda [tokens][heads][frames]; qt, kt: bf16 cuda [tokens][heads][frames][dim];
    candidates: int32 cuda [frames][n].  Returns (main_anchor int32 [tiles], kept int32 [frames][n]) and the compared
    scores float32 [frames][tiles] if asked."""
    tokens, heads, frames, dim = qt.shape
    assert tokens == grid_h * grid_w and candidates.shape[0] == frames
    tiles = ((grid_h + tile_h - 1) // tile_h) * ((grid_w + tile_w - 1) // tile_w)
    main = torch.empty(tiles, dtype=torch.int32, device=qt.device) if main_anchor is None else main_anchor
    if kept is None:
        kept = torch.empty_like(candidates)
    ps = torch.empty((frames, tiles), dtype=torch.float32, device=qt.device) if want_scores else None
    _check(_lib.fb4_seda_main_anchor(_dp(temporal_scores), _dp(qt), _dp(kt), frames, heads, grid_h, grid_w, dim,
                                     _dp(candidates), candidates.shape[1], tile_h, tile_w, float(prune_threshold),
                                     _dp(main), _dp(kept), _dp(ps), _stream(stream)), "fb4_seda_main_anchor")
    return (main, kept, ps) if want_scores else (main, kept)


def fb4_seda_main_anchor_3d(scores, frames, grid_h, grid_w, tile_h=4, tile_w=4, stream=None, anchors=None):
    """scores: float32 cuda [heads][frames * tokens].  Returns int32 [tiles]: the main anchor of every spatial tile."""
    heads = scores.shape[0]
    tiles = ((grid_h + tile_h - 1) // tile_h) * ((grid_w + tile_w - 1) // tile_w)
    if anchors is None:
        anchors = torch.empty(tiles, dtype=torch.int32, device=scores.device)
    _check(_lib.fb4_seda_main_anchor_3d(_dp(scores), frames, heads, grid_h, grid_w, tile_h, tile_w, _dp(anchors),
                                        _stream(stream)), "fb4_seda_main_anchor_3d")
    return anchors


def fb4_probe_mfma_rate(workgroups, iterations, random_operands=True, out=None, stream=None):
    """Diagnostic launch of a register-only bf16 MFMA loop; returns (out, operations performed)."""
    if out is None:
        out = torch.empty(workgroups * 256, dtype=torch.float32, device="cuda")
    flop = ctypes.c_double(0.0)
    _check(_lib.fb4_probe_mfma_rate(int(workgroups), int(iterations), int(bool(random_operands)), _dp(out), ctypes.byref(flop),
                                    _stream(stream)), "fb4_probe_mfma_rate")
    return out, flop.value


def fb4_gelu_table_host(approximate=0):
    """The library's GeLU table as a uint16 numpy array (no GPU needed): entry k = GeLU of bit pattern k."""
    n = ctypes.c_size_t(0)
    _lib.fb4_gelu_table_host(int(approximate), None, 0, ctypes.byref(n))
    t = np.zeros(n.value, dtype=np.uint16)
    _check(_lib.fb4_gelu_table_host(int(approximate), t.ctypes.data_as(ctypes.c_void_p), t.size, ctypes.byref(n)),
           "fb4_gelu_table_host")
    return t


def fb4_gelu_quantize(luts, o, x, approximate=0, codes=None, meta=None, stream=None, token_group=None,
                      sub_formatbooks=None):
    """GeLU of every element (approximate: 0 = x Phi(x), 1 = the tanh form), then quantize, in one pass;
    token_group / sub_formatbooks as in fb4_quantize_seda (optional).  Returns (codes, meta)."""
    rows, cols = x.shape
    if codes is None:
        codes = torch.empty((rows, cols // 2), dtype=torch.uint8, device=x.device)
    if meta is None:
        meta = torch.empty((rows, cols // o.block), dtype=torch.int16, device=x.device)
    rc = _lib.fb4_gelu_quantize(luts.handle, ctypes.byref(o), _dp(x), rows, cols, x.stride(0) if rows > 1 else cols,
                                int(approximate), _dp(token_group), _dp(sub_formatbooks),
                                0 if sub_formatbooks is None else sub_formatbooks.shape[0],
                                _dp(codes), _dp(meta), _stream(stream))
    _check(rc, "fb4_gelu_quantize")
    return codes, meta


def fb4_quantize_seda(luts, o, x, token_group, sub_formatbooks, codes=None, meta=None, stream=None):
    """token_group: int32 cuda [rows]; sub_formatbooks: uint8 cuda [n_groups][8]."""
    rows, cols = x.shape
    if codes is None:
        codes = torch.empty((rows, cols // 2), dtype=torch.uint8, device=x.device)
    if meta is None:
        meta = torch.empty((rows, cols // o.block), dtype=torch.int16, device=x.device)
    rc = _lib.fb4_quantize_seda(luts.handle, ctypes.byref(o), _dp(x), rows, cols,
                                x.stride(0) if rows > 1 else cols, _dp(token_group), _dp(sub_formatbooks),
                                sub_formatbooks.shape[0], _dp(codes), _dp(meta), _stream(stream))
    _check(rc, "fb4_quantize_seda")
    return codes, meta


def fb4_decompose(luts, o, x, codes1, meta1, salient_rows, token_group=None, sub_formatbooks=None,
                  codes2=None, meta2=None, stream=None):
    """salient_rows: int32 cuda [n_sal], ascending.  Returns the compact second plane (codes2, meta2)."""
    rows, cols = x.shape
    n_sal = salient_rows.numel()
    if codes2 is None:
        codes2 = torch.empty((n_sal, cols // 2), dtype=torch.uint8, device=x.device)
    if meta2 is None:
        meta2 = torch.empty((n_sal, cols // o.block), dtype=torch.int16, device=x.device)
    rc = _lib.fb4_decompose(luts.handle, ctypes.byref(o), _dp(x), rows, cols, x.stride(0) if rows > 1 else cols,
                            _dp(codes1), _dp(meta1), _dp(salient_rows), n_sal, _dp(token_group),
                            _dp(sub_formatbooks), 0 if sub_formatbooks is None else sub_formatbooks.shape[0],
                            _dp(codes2), _dp(meta2), _stream(stream))
    _check(rc, "fb4_decompose")
    return codes2, meta2


def fb4_quantize_decompose(luts, o, x, salient_rows, token_group=None, sub_formatbooks=None,
                           codes1=None, meta1=None, codes2=None, meta2=None, stream=None):
    """Both planes in one call.  Returns (codes1, meta1, codes2, meta2)."""
    rows, cols = x.shape
    n_sal = salient_rows.numel()
    if codes1 is None:
        codes1 = torch.empty((rows, cols // 2), dtype=torch.uint8, device=x.device)
    if meta1 is None:
        meta1 = torch.empty((rows, cols // o.block), dtype=torch.int16, device=x.device)
    if codes2 is None:
        codes2 = torch.empty((n_sal, cols // 2), dtype=torch.uint8, device=x.device)
    if meta2 is None:
        meta2 = torch.empty((n_sal, cols // o.block), dtype=torch.int16, device=x.device)
    rc = _lib.fb4_quantize_decompose(luts.handle, ctypes.byref(o), _dp(x), rows, cols,
                                     x.stride(0) if rows > 1 else cols, _dp(token_group), _dp(sub_formatbooks),
                                     0 if sub_formatbooks is None else sub_formatbooks.shape[0],
                                     _dp(salient_rows), n_sal, _dp(codes1), _dp(meta1), _dp(codes2), _dp(meta2),
                                     _stream(stream))
    _check(rc, "fb4_quantize_decompose")
    return codes1, meta1, codes2, meta2


def fb4_dequantize(luts, codes1, meta1, block=32, codes2=None, meta2=None, salient_rows=None,
                   out=None, out_dtype=DTYPE_BF16, stream=None):
    rows, half = codes1.shape
    cols = half * 2
    if out is None:
        out = torch.empty((rows, cols), dtype=torch.bfloat16 if out_dtype == DTYPE_BF16 else torch.float32,
                          device=codes1.device)
    n_sal = 0 if salient_rows is None else salient_rows.numel()
    rc = _lib.fb4_dequantize(luts.handle, _dp(codes1), _dp(meta1), rows, cols, block, _dp(codes2), _dp(meta2),
                             _dp(salient_rows), n_sal, _dp(out), out_dtype, out.stride(0) if rows > 1 else cols,
                             _stream(stream))
    _check(rc, "fb4_dequantize")
    return out


def fb4_repack_mxfp8(luts, codes, meta, block=32, elems=None, scales=None, stream=None):
    """One code plane as MXFP8 operands: (E4M3 bytes uint8 [rows][cols], E8M0 scale bytes uint8 [rows][cols/32])."""
    rows, half = codes.shape
    cols = half * 2
    if elems is None:
        elems = torch.empty((rows, cols), dtype=torch.uint8, device=codes.device)
    if scales is None:
        scales = torch.empty((rows, cols // 32), dtype=torch.uint8, device=codes.device)
    rc = _lib.fb4_repack_mxfp8(luts.handle, _dp(codes), _dp(meta), rows, cols, block, _dp(elems),
                               elems.stride(0) if rows > 1 else cols, _dp(scales), _stream(stream))
    _check(rc, "fb4_repack_mxfp8")
    return elems, scales


def fb4_seda_profile(luts, meta, anchor_group, n_groups, counts=None, sub_formatbooks=None, stream=None):
    """Sub-formatbooks from the dialects selected on anchor tokens.  Returns (counts int32 [n_groups][32],
    sub_formatbooks uint8 [n_groups][8])."""
    rows, nb = meta.shape
    if counts is None:
        counts = torch.empty((n_groups, 32), dtype=torch.int32, device=meta.device)
    if sub_formatbooks is None:
        sub_formatbooks = torch.empty((n_groups, 8), dtype=torch.uint8, device=meta.device)
    rc = _lib.fb4_seda_profile(luts.handle, _dp(meta), rows, nb, _dp(anchor_group), n_groups, _dp(counts),
                               _dp(sub_formatbooks), _stream(stream))
    _check(rc, "fb4_seda_profile")
    return counts, sub_formatbooks
