"""ctypes front end of the plain-C CPU oracle (fb4_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's CPU-baseline leg.  It never touches the GPU library and the GPU
library never touches it.  Arrays are numpy; bf16 tensors travel as uint16 bit
patterns.
"""

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fb4_oracle.c")
_LIB = os.path.join(_HERE, "libfb4_oracle.so")

SEL_SSE = 0
SEL_LUT = 1
FLAG_TWO_STAGE = 1
OUT_BF16 = 0
OUT_F32 = 1


def build(force=False):
    """Compile fb4_oracle.c with gcc (no fast-math, no contraction)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, i32, p = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        lib.fb4o_validate_formatbook.argtypes = [p, i32]
        lib.fb4o_max_threads.argtypes = []
        lib.fb4o_quantize.argtypes = [p, i32, i32, i32, i32, i32, p, i64, i64, i64, p, p, i32, p, p, i32]
        lib.fb4o_block_scores.argtypes = [p, i32, i32, i32, i32, i32, p, p, p, p, p, p]
        lib.fb4o_decompose.argtypes = [p, i32, i32, i32, i32, i32, p, i64, i64, i64, p, p, p, i64,
                                       p, p, i32, p, p, i32]
        lib.fb4o_dequantize.argtypes = [p, i32, i32, p, p, i64, i64, p, p, p, i64, p, i32, i64, i32]
        lib.fb4o_repack_mxfp8.argtypes = [p, i32, i32, p, p, i64, i64, p, p]
        lib.fb4o_layernorm.argtypes = [p, i64, i64, i64, p, p, ctypes.c_float, p, p, p]
        lib.fb4o_gelu.argtypes = [p, i64, i32, p]
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def max_threads():
    return int(_load().fb4o_max_threads())


def validate_formatbook(fbk):
    fbk = _c(fbk, np.uint8)
    if fbk.ndim != 2 or fbk.shape[1] != 8:
        return False
    return _load().fb4o_validate_formatbook(_ptr(fbk), fbk.shape[0]) == 0


def quantize(fbk, x_bits, block=32, selector=SEL_LUT, num_groups=8, flags=0,
             token_group=None, sub_formatbooks=None, nthreads=0):
    """x_bits: uint16 [rows][cols] (any row stride).  Returns codes uint8
    [rows][cols/2], meta uint16 [rows][cols/block]."""
    fbk = _c(fbk, np.uint8)
    assert x_bits.dtype == np.uint16 and x_bits.ndim == 2 and x_bits.strides[1] == 2
    rows, cols = x_bits.shape
    stride = x_bits.strides[0] // 2 if rows > 1 else cols
    tg = _c(token_group, np.int32)
    sub = _c(sub_formatbooks, np.uint8)
    codes = np.zeros((rows, cols // 2), dtype=np.uint8)
    meta = np.zeros((rows, cols // block if block else 0), dtype=np.uint16)
    rc = _load().fb4o_quantize(_ptr(fbk), fbk.shape[0], block, selector, num_groups, flags,
                               _ptr(x_bits), rows, cols, stride, _ptr(tg), _ptr(sub),
                               0 if sub is None else sub.shape[0], _ptr(codes), _ptr(meta), nthreads)
    if rc != 0:
        raise ValueError("fb4o_quantize: invalid argument")
    return codes, meta


def block_scores(fbk, x_block_bits, selector=SEL_SSE, num_groups=8, flags=0, sub8=None):
    """Scores of one block.  Returns (cand DIDs, scores, selected DID, exponent)."""
    fbk = _c(fbk, np.uint8)
    xb = _c(x_block_bits, np.uint16)
    block = xb.size
    scores = np.zeros(32, dtype=np.float64)
    cand = np.zeros(32, dtype=np.int32)
    did = ctypes.c_int(0)
    e = ctypes.c_int(0)
    s8 = _c(sub8, np.uint8)
    n = _load().fb4o_block_scores(_ptr(fbk), fbk.shape[0], block, selector, num_groups, flags,
                                  _ptr(xb), _ptr(s8), _ptr(scores), _ptr(cand),
                                  ctypes.addressof(did), ctypes.addressof(e))
    if n < 0:
        raise ValueError("fb4o_block_scores: invalid argument")
    return cand[:n].copy(), scores[:n].copy(), did.value, e.value


def decompose(fbk, x_bits, codes1, meta1, salient_rows, block=32, selector=SEL_LUT, num_groups=8,
              flags=0, token_group=None, sub_formatbooks=None, nthreads=0):
    fbk = _c(fbk, np.uint8)
    assert x_bits.dtype == np.uint16 and x_bits.ndim == 2 and x_bits.strides[1] == 2
    rows, cols = x_bits.shape
    stride = x_bits.strides[0] // 2 if rows > 1 else cols
    codes1 = _c(codes1, np.uint8)
    meta1 = _c(meta1, np.uint16)
    sal = _c(salient_rows, np.int32)
    tg = _c(token_group, np.int32)
    sub = _c(sub_formatbooks, np.uint8)
    n_sal = sal.size
    codes2 = np.zeros((n_sal, cols // 2), dtype=np.uint8)
    meta2 = np.zeros((n_sal, cols // block), dtype=np.uint16)
    rc = _load().fb4o_decompose(_ptr(fbk), fbk.shape[0], block, selector, num_groups, flags,
                                _ptr(x_bits), rows, cols, stride, _ptr(codes1), _ptr(meta1),
                                _ptr(sal), n_sal, _ptr(tg), _ptr(sub),
                                0 if sub is None else sub.shape[0], _ptr(codes2), _ptr(meta2),
                                nthreads)
    if rc != 0:
        raise ValueError("fb4o_decompose: invalid argument")
    return codes2, meta2


def dequantize(fbk, codes1, meta1, block=32, codes2=None, meta2=None, salient_rows=None,
               out_dtype=OUT_BF16, nthreads=0):
    """Returns uint16 bit patterns (OUT_BF16) or float32 (OUT_F32), [rows][cols]."""
    fbk = _c(fbk, np.uint8)
    codes1 = _c(codes1, np.uint8)
    meta1 = _c(meta1, np.uint16)
    rows, half = codes1.shape
    cols = half * 2
    codes2 = _c(codes2, np.uint8)
    meta2 = _c(meta2, np.uint16)
    sal = _c(salient_rows, np.int32)
    n_sal = 0 if sal is None else sal.size
    out = np.zeros((rows, cols), dtype=np.uint16 if out_dtype == OUT_BF16 else np.float32)
    rc = _load().fb4o_dequantize(_ptr(fbk), fbk.shape[0], block, _ptr(codes1), _ptr(meta1), rows,
                                 cols, _ptr(codes2), _ptr(meta2), _ptr(sal), n_sal, _ptr(out),
                                 out_dtype, cols, nthreads)
    if rc != 0:
        raise ValueError("fb4o_dequantize: invalid argument")
    return out


def repack_mxfp8(fbk, codes, meta, block=32):
    """One code plane as MXFP8 operands: (E4M3 bytes [rows][cols], E8M0 scale bytes [rows][cols/32])."""
    fbk = _c(fbk, np.uint8)
    codes = _c(codes, np.uint8)
    meta = _c(meta, np.uint16)
    rows, half = codes.shape
    cols = half * 2
    elems = np.zeros((rows, cols), dtype=np.uint8)
    scales = np.zeros((rows, cols // 32), dtype=np.uint8)
    rc = _load().fb4o_repack_mxfp8(_ptr(fbk), fbk.shape[0], block, _ptr(codes), _ptr(meta), rows, cols,
                                   _ptr(elems), _ptr(scales))
    if rc != 0:
        raise ValueError("fb4o_repack_mxfp8: invalid argument")
    return elems, scales


def layernorm(x_bits, gamma=None, beta=None, eps=1e-6):
    """The LayerNorm producer in front of the quantizer (App. E.2), arithmetic as fixed in fb4_oracle.c.
    x_bits: uint16 [rows][cols]; gamma / beta: float32 [cols] or None.  Returns (y bf16 bit patterns
    [rows][cols], a float32 [rows] = 1/std, b float32 [rows] = -mean/std)."""
    assert x_bits.dtype == np.uint16 and x_bits.ndim == 2 and x_bits.strides[1] == 2
    rows, cols = x_bits.shape
    stride = x_bits.strides[0] // 2 if rows > 1 else cols
    g = _c(gamma, np.float32)
    b = _c(beta, np.float32)
    y = np.zeros((rows, cols), dtype=np.uint16)
    a_out = np.zeros(rows, dtype=np.float32)
    b_out = np.zeros(rows, dtype=np.float32)
    rc = _load().fb4o_layernorm(_ptr(x_bits), rows, cols, stride, _ptr(g), _ptr(b), float(eps), _ptr(y),
                                _ptr(a_out), _ptr(b_out))
    if rc != 0:
        raise ValueError("fb4o_layernorm: invalid argument")
    return y, a_out, b_out


def gelu(x_bits, approximate=0):
    """GeLU in front of the quantizer (App. E.2): elementwise on bf16 bit patterns, the value in double rounded
    once.  approximate: 0 = x Phi(x), 1 = the tanh form.  Returns uint16 of the same shape."""
    xb = np.ascontiguousarray(x_bits, dtype=np.uint16)
    y = np.zeros(xb.shape, dtype=np.uint16)
    rc = _load().fb4o_gelu(_ptr(xb), xb.size, int(approximate), _ptr(y))
    if rc != 0:
        raise ValueError("fb4o_gelu: invalid argument")
    return y


def _bf16_to_f64(bits):
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    with np.errstate(invalid="ignore"):
        return u.view(np.float32).astype(np.float64)


def attention_scores(q_bits, k_bits, mode="abs"):
    """Sec. 3.3, salient-token scoring: the mean pre-softmax attention score of every query token over the keys of
    its attention group, score[g][q] = (1/T) sum_k f(Q[g][q] . K[g][k]) with f = |.| ("abs": spatial / 3D attention)
    or max(., 0) ("relu": temporal attention).  q_bits, k_bits: uint16 [G][T][d] bf16 patterns (a group is one
    head of one frame, or of one spatial position for temporal attention).  float64 [G][T].  The product is
    numpy's float64 matmul."""
    assert mode in ("abs", "relu")
    q = _bf16_to_f64(q_bits)
    k = _bf16_to_f64(k_bits)
    assert q.ndim == 3 and q.shape == k.shape
    out = np.zeros(q.shape[:2], dtype=np.float64)
    for g in range(q.shape[0]):
        s = q[g] @ k[g].T
        s = np.abs(s) if mode == "abs" else np.maximum(s, 0.0)
        out[g] = s.sum(axis=1) / q.shape[1]
    return out


def select_salient_tokens(scores, grid_h, grid_w, tile_h=4, tile_w=4):
    """Sec. 3.3 / App. F: one salient token per tile.  scores: [frames][heads][grid_h * grid_w] (float32 or
    float64), tokens row-major on the frame's grid.  Per frame the head scores are averaged (summed head by head in
    float64), then the best token of every tile_h x tile_w tile is taken (ties: the lowest token index; a NaN
    never wins; ragged tiles at the right / bottom edge are allowed).  Returns the chosen tokens as rows of
    the [frames * tokens] tensor, frame by frame and ascending within a frame: int32 [frames][tiles]."""
    scores = np.asarray(scores)
    frames, heads, tokens = scores.shape
    assert tokens == grid_h * grid_w
    th, tw = (grid_h + tile_h - 1) // tile_h, (grid_w + tile_w - 1) // tile_w
    out = np.zeros((frames, th * tw), dtype=np.int32)
    for f in range(frames):
        mean = np.zeros(tokens, dtype=np.float64)
        for h in range(heads):
            mean += scores[f, h].astype(np.float64)
        mean /= heads
        picks = []
        for ty in range(th):
            for tx in range(tw):
                best, best_v = -1, -np.inf
                for y in range(ty * tile_h, min(grid_h, (ty + 1) * tile_h)):
                    for x in range(tx * tile_w, min(grid_w, (tx + 1) * tile_w)):
                        v = mean[y * grid_w + x]
                        if np.isnan(v):
                            v = -np.inf
                        if best < 0 or v > best_v:
                            best, best_v = y * grid_w + x, v
                picks.append(best)
        out[f] = np.sort(np.asarray(picks, dtype=np.int64)) + f * tokens
    return out


def seda_assign(q_bits, k_bits, anchors, grid_h, grid_w, window=5, threshold=5.0):
    """Sec. 3.4, "Attention-Guided Semantic Relatedness Extraction", the per-frame part: every tile's anchor token
    (one per frame and tile: `anchors`, int32 [frames][tiles], rows of the [frames * tokens] tensor, ascending per
    frame as select_salient_tokens returns them -- tile g of a frame is the g-th tile in row-major tile order, found
    again from the anchor's position) marks as correlated the tokens of a window x window square around it (clipped
    to the frame) whose raw pre-softmax attention score FROM the anchor, Q[anchor] . K[token] averaged over the heads,
    exceeds `threshold`.  A token marked by several anchors belongs to the one with the highest group number (the
    "subsequent" anchor); an anchor always belongs to its own group.  Group number = position of the anchor in its
    frame's list.  q_bits, k_bits: uint16 [frames][heads][tokens][dim].  Returns (token_group int32 [frames * tokens],
    -1 = none; anchor_group int32 [frames * tokens], the group on anchor rows and -1 elsewhere; score float64
    [frames][tiles][window * window], NaN outside the frame).  Plain loops; the dot products are numpy float64."""
    q = _bf16_to_f64(q_bits)
    k = _bf16_to_f64(k_bits)
    frames, heads, tokens, dim = q.shape
    assert tokens == grid_h * grid_w
    anchors = np.asarray(anchors, dtype=np.int64)
    tiles = anchors.shape[1]
    token_group = np.full(frames * tokens, -1, dtype=np.int32)
    anchor_group = np.full(frames * tokens, -1, dtype=np.int32)
    score = np.full((frames, tiles, window * window), np.nan)
    half = window // 2
    for f in range(frames):
        for g in range(tiles):
            a = int(anchors[f, g]) - f * tokens
            ay, ax = divmod(a, grid_w)
            for wy in range(window):
                for wx in range(window):
                    y, x = ay + wy - half, ax + wx - half
                    if not (0 <= y < grid_h and 0 <= x < grid_w):
                        continue
                    t = y * grid_w + x
                    sc = 0.0
                    for h in range(heads):
                        sc += float(q[f, h, a] @ k[f, h, t])
                    sc /= heads
                    score[f, g, wy * window + wx] = sc
                    if sc > threshold:
                        token_group[f * tokens + t] = max(token_group[f * tokens + t], g)
        for g in range(tiles):                      # an anchor belongs to its own group
            token_group[int(anchors[f, g])] = g
            anchor_group[int(anchors[f, g])] = g
    return token_group, anchor_group, score


def seda_profile(fbk, meta, anchor_group, n_groups):
    """Sec. 3.4, "Constructing an 8-Dialect Sub-Formatbook": bin-count profile of the dialects selected on the
    anchor tokens of each group, then per dynamic-range bucket (largest magnitude 8..15) the most frequently
    selected dialect of that bucket.  meta: uint16 [rows][blocks per row] of an already quantized tensor;
    anchor_group: int32 [rows], g in 0..n_groups-1 marks an anchor token of group g (anything else: not an
    anchor).  Ties go to the lowest DID; a bucket none of whose dialects was selected gets its lowest DID; a
    bucket the formatbook has no dialect for gets 255.  Returns (counts uint32 [n_groups][32], sub uint8
    [n_groups][8]).  Plain numpy loops."""
    fbk = np.asarray(fbk, dtype=np.uint8)
    meta = np.asarray(meta, dtype=np.uint16)
    anchor_group = np.asarray(anchor_group, dtype=np.int32)
    counts = np.zeros((n_groups, 32), dtype=np.uint32)
    for r in range(meta.shape[0]):
        g = int(anchor_group[r])
        if 0 <= g < n_groups:
            for did in (meta[r] & 0xFF).tolist():
                if did < 32:
                    counts[g, did] += 1
    sub = np.full((n_groups, 8), 255, dtype=np.uint8)
    for g in range(n_groups):
        for k in range(8):
            best, best_count = 255, -1
            for d in range(fbk.shape[0]):
                if int(fbk[d, 7]) == 8 + k and int(counts[g, d]) > best_count:
                    best, best_count = d, int(counts[g, d])
            sub[g, k] = best
    return counts, sub
