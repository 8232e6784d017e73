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
        lib.fb4o_layernorm.argtypes = [p, i64, i64, i64, p, p, ctypes.c_double, p, p, p]
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
    """The LayerNorm producer in front of the quantizer (App. E.2): the textbook two-pass definition in float64,
    rounded once to bf16.  x_bits: uint16 [rows][cols]; gamma / beta: float32 [cols] or None; eps is taken as the
    float32 value a caller of the library would pass.  Returns (y bf16 bit patterns [rows][cols], mean float64
    [rows], rstd float64 [rows] = 1 / sqrt(var + eps))."""
    assert x_bits.dtype == np.uint16 and x_bits.ndim == 2 and x_bits.strides[1] == 2
    rows, cols = x_bits.shape
    stride = x_bits.strides[0] // 2 if rows > 1 else cols
    g = _c(gamma, np.float32)
    b = _c(beta, np.float32)
    y = np.zeros((rows, cols), dtype=np.uint16)
    mean = np.zeros(rows, dtype=np.float64)
    rstd = np.zeros(rows, dtype=np.float64)
    rc = _load().fb4o_layernorm(_ptr(x_bits), rows, cols, stride, _ptr(g), _ptr(b), float(np.float32(eps)), _ptr(y),
                                _ptr(mean), _ptr(rstd))
    if rc != 0:
        raise ValueError("fb4o_layernorm: invalid argument")
    return y, mean, rstd


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


def _tile_of(token, grid_w, tile_h, tile_w):
    """Row-major number of the tile_h x tile_w tile that holds a token of a row-major grid of width grid_w."""
    y, x = divmod(int(token), grid_w)
    tiles_w = (grid_w + tile_w - 1) // tile_w
    return (y // tile_h) * tiles_w + x // tile_w


def seda_assign(q_bits, k_bits, anchors, frames, grid_h, grid_w, tile_h=4, tile_w=4, window=5, window_t=1,
                threshold=5.0, joint=False):
    """Sec. 3.4, "Attention-Guided Semantic Relatedness Extraction", the marking step (step 3 for factorized
    attention, the cuboid step for 3D attention).  `anchors`: int32 [n], rows of the [frames * tokens] activation
    (tokens = grid_h * grid_w, row-major per frame); an entry outside the tensor (say -1: a pruned frame's candidate)
    does nothing.  The GROUP of an anchor is the row-major number of the tile_h x tile_w spatial tile it lies in, so
    that the per-frame candidates of one tile share a group -- one sub-formatbook -- across the frames.  Every
    anchor marks as correlated the tokens of a window x window square (x window_t frames: a cuboid) centred on it
    and clipped to the clip, whose RAW pre-softmax attention score from the anchor, Q[anchor] . K[token] averaged
    over the heads, exceeds `threshold`.  A token marked by anchors of several groups belongs to the highest group
    number (App. D: overlapping windows go to the subsequent anchor = the later tile); an anchor always belongs to
    its own group.
    joint = False (factorized attention): q_bits, k_bits uint16 [frames][heads][tokens][dim], the projections of the
    spatial attention; scores exist inside a frame only, so window_t must be 1.
    joint = True (3D attention): uint16 [heads][frames * tokens][dim].
    Returns (token_group int32 [frames * tokens], -1 = none; anchor_group int32 [frames * tokens], the group on anchor
    rows and -1 elsewhere; score float64 [n][window_t * window * window], NaN outside the clip or for a dropped
    entry).  Plain loops; the dot products are numpy float64."""
    q = _bf16_to_f64(q_bits)
    k = _bf16_to_f64(k_bits)
    tokens = grid_h * grid_w
    if joint:
        heads, total, dim = q.shape
        assert total == frames * tokens
        at = lambda arr, f, h, t: arr[h, f * tokens + t]
    else:
        assert q.shape[0] == frames and q.shape[2] == tokens and window_t == 1
        heads = q.shape[1]
        at = lambda arr, f, h, t: arr[f, h, t]
    anchors = np.asarray(anchors, dtype=np.int64).ravel()
    n = anchors.size
    token_group = np.full(frames * tokens, -1, dtype=np.int32)
    anchor_group = np.full(frames * tokens, -1, dtype=np.int32)
    score = np.full((n, window_t * window * window), np.nan)
    half, half_t = window // 2, window_t // 2
    for i in range(n):
        row = int(anchors[i])
        if not 0 <= row < frames * tokens:
            continue
        fa, a = divmod(row, tokens)
        g = _tile_of(a, grid_w, tile_h, tile_w)
        ay, ax = divmod(a, grid_w)
        for wt in range(window_t):
            for wy in range(window):
                for wx in range(window):
                    f, y, x = fa + wt - half_t, ay + wy - half, ax + wx - half
                    if not (0 <= f < frames and 0 <= y < grid_h and 0 <= x < grid_w):
                        continue
                    t = y * grid_w + x
                    sc = 0.0
                    for h in range(heads):
                        sc += float(at(q, fa, h, a) @ at(k, f, h, t))
                    sc /= heads
                    score[i, (wt * window + wy) * window + wx] = sc
                    if sc > threshold:
                        token_group[f * tokens + t] = max(token_group[f * tokens + t], g)
    for i in range(n):                      # an anchor belongs to its own group
        row = int(anchors[i])
        if 0 <= row < frames * tokens:
            g = _tile_of(row % tokens, grid_w, tile_h, tile_w)
            token_group[row] = g
            anchor_group[row] = g
    return token_group, anchor_group, score


def seda_main_anchor(temporal_scores, qt_bits, kt_bits, candidates, grid_h, grid_w, tile_h=4, tile_w=4,
                     prune_threshold=3.0):
    """Sec. 3.4, factorized attention, step 2: per spatial tile, the main anchor among the tile's per-frame
    candidates and the pruning of weakly correlated frames.
    candidates: int32 [frames][n], per frame the anchor candidates of step 1 as rows of the [frames * tokens]
    activation (what select_salient_tokens returns); a candidate's tile is found from its position; an entry
    outside its own frame is no candidate.
    temporal_scores: [positions][heads][frames], the mean temporal attention score of every token (what
    attention_scores gives for the temporal attention: group = spatial position and head, tokens = frames).
    qt_bits, kt_bits: uint16 [positions][heads][frames][dim], the temporal attention's projections.
    Main anchor of a tile = the candidate whose own temporal mean score, averaged over the heads (summed head by
    head in float64), is highest; ties go to the earliest frame, a NaN never wins.  A frame's candidate is pruned
    when the raw temporal attention score FROM the main anchor TO that frame -- Qt[p*][h][f*] . Kt[p*][h][f] at the
    main anchor's position p*, averaged over the heads -- does not exceed prune_threshold; the main anchor's own
    frame always stays.
    Returns (main int32 [tiles] rows, -1 for a tile without candidates; kept int32 [frames][n] = candidates with
    the pruned and the invalid entries set to -1; prune_score float64 [frames][tiles], NaN where there is no
    candidate)."""
    ts = np.asarray(temporal_scores)
    qt = _bf16_to_f64(qt_bits)
    kt = _bf16_to_f64(kt_bits)
    positions, heads, frames = ts.shape
    tokens = grid_h * grid_w
    assert positions == tokens and qt.shape[:3] == (positions, heads, frames)
    cand = np.asarray(candidates, dtype=np.int64)
    assert cand.shape[0] == frames
    th, tw = (grid_h + tile_h - 1) // tile_h, (grid_w + tile_w - 1) // tile_w
    tiles = th * tw
    main = np.full(tiles, -1, dtype=np.int32)
    kept = np.full(cand.shape, -1, dtype=np.int32)
    prune_score = np.full((frames, tiles), np.nan)
    for tile in range(tiles):
        # the tile's candidate in every frame (the first listed one if a frame lists several)
        slot = [-1] * frames
        for f in range(frames):
            for j in range(cand.shape[1]):
                row = int(cand[f, j])
                if f * tokens <= row < (f + 1) * tokens and _tile_of(row - f * tokens, grid_w, tile_h, tile_w) == tile:
                    slot[f] = j
                    break
        best_f, best_v = -1, -np.inf
        for f in range(frames):
            if slot[f] < 0:
                continue
            p = int(cand[f, slot[f]]) - f * tokens
            v = 0.0
            for h in range(heads):
                v += float(ts[p, h, f])
            v /= heads
            if np.isnan(v):
                v = -np.inf
            if best_f < 0 or v > best_v:
                best_f, best_v = f, v
        if best_f < 0:
            continue
        main[tile] = int(cand[best_f, slot[best_f]])
        p = main[tile] - best_f * tokens
        for f in range(frames):
            if slot[f] < 0:
                continue
            sc = 0.0
            for h in range(heads):
                sc += float(qt[p, h, best_f] @ kt[p, h, f])
            sc /= heads
            prune_score[f, tile] = sc
            if f == best_f or sc > prune_threshold:
                kept[f, slot[f]] = int(cand[f, slot[f]])
    return main, kept, prune_score


def seda_main_anchor_3d(scores, frames, grid_h, grid_w, tile_h=4, tile_w=4):
    """Sec. 3.4, 3D attention: the main anchor of every spatial tile is the token with the highest mean attention
    score among the tile's tile_h x tile_w x frames tokens.  scores: [heads][frames * tokens], the mean attention
    score of every token of the clip (attention_scores with one group per head); averaged over the heads (summed
    head by head in float64); ties go to the lowest row, a NaN never wins.  Returns int32 [tiles] rows of the
    [frames * tokens] activation, in tile order."""
    scores = np.asarray(scores)
    heads, total = scores.shape
    tokens = grid_h * grid_w
    assert total == frames * tokens
    mean = np.zeros(total, dtype=np.float64)
    for h in range(heads):
        mean += scores[h].astype(np.float64)
    mean /= heads
    th, tw = (grid_h + tile_h - 1) // tile_h, (grid_w + tile_w - 1) // tile_w
    out = np.zeros(th * tw, dtype=np.int32)
    for ty in range(th):
        for tx in range(tw):
            best, best_v = -1, -np.inf
            for f in range(frames):
                for y in range(ty * tile_h, min(grid_h, (ty + 1) * tile_h)):
                    for x in range(tx * tile_w, min(grid_w, (tx + 1) * tile_w)):
                        row = f * tokens + y * grid_w + x
                        v = mean[row]
                        if np.isnan(v):
                            v = -np.inf
                        if best < 0 or v > best_v:
                            best, best_v = row, v
            out[ty * tw + tx] = best
    return out


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
