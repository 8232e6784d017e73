/*
 * fb4.h -- C ABI of the MI355X (gfx950) FB4 online quantizer.
 *
 * FB4 is the 4-bit block format of the SemanticDialect paper (Sec. 3.1): a
 * block of 32 (or 16) consecutive elements shares a power-of-two scale and one
 * "dialect" -- a set of eight integer magnitudes out of 0..15 -- chosen per
 * block from a 32-entry formatbook; an element is a sign bit plus a 3-bit
 * index into the dialect.
 *
 * Conventions shared by every entry point
 *   - Returns FB4_OK (0) or a negative FB4_ERR_* code; nothing aborts or
 *     throws across this boundary.  fb4_strerror() names a code.
 *   - Pointers marked "device" are GPU global-memory pointers owned by the
 *     caller; pointers marked "host" are ordinary CPU pointers.  The library
 *     allocates no tensor memory and never synchronizes: kernels are enqueued
 *     on the caller's HIP stream (`stream` is a hipStream_t passed as void*,
 *     NULL = the default stream) and the call returns immediately.
 *   - Tensors are row-major.  x is bf16 (raw 16-bit patterns) with an explicit
 *     row stride in elements; rows must start 16-byte aligned (base pointer
 *     16-byte aligned and row_stride a multiple of 8), cols must be a multiple
 *     of the block size; otherwise FB4_ERR_UNSUPPORTED.
 *   - codes: uint8 [rows][cols/2], contiguous.  Element 2j is the low nibble
 *     and element 2j+1 the high nibble of byte j; nibble = sign<<3 | index.
 *   - meta: uint16 [rows][cols/block], contiguous.  Low byte = dialect ID
 *     (DID), high byte = shared exponent e + 127, e = floor(log2(max|x|))
 *     clamped to [-123, 127] (all-zero block: -123).  The paper budgets 5+5
 *     metadata bits (Sec. 3.1); the wider exponent byte covers the bf16 range.
 *   - A code decodes to (-1)^sign * M[DID][index] * 2^(e-3) (Sec. 3.1: the
 *     normalized block lies in [0,16) with its maximum in [8,16)).
 *   - Degenerate inputs: a NaN element is ignored by the block maximum and by
 *     dialect selection and is emitted as index 0 with its sign; +/-Inf is read
 *     as the finite magnitude 2^128 (so it saturates and e = 127); the sign bit
 *     of the input is copied to the code even when the magnitude rounds to 0.
 *   - rows == 0 or cols == 0 is a successful no-op.
 *   - A call made while another device than the handle's is current returns
 *     FB4_ERR_INVALID_ARG.  The entry points without a handle
 *     (fb4_attention_scores, fb4_select_salient_tokens, fb4_seda_assign,
 *     fb4_seda_main_anchor, fb4_seda_main_anchor_3d, fb4_probe_mfma_rate) run on
 *     the current device.
 *   - The producer-fused entry points (fb4_layernorm_quantize,
 *     fb4_gelu_quantize) read x as plain IEEE bf16 and hand the quantizer the
 *     producer's bf16 result, to which the rules above then apply.
 */
#ifndef FB4_H
#define FB4_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FB4_OK 0
#define FB4_ERR_INVALID_ARG (-1) /* null pointer, bad size, bad option, bad formatbook */
#define FB4_ERR_UNSUPPORTED (-2) /* valid request this build cannot serve (alignment, ragged cols) */
#define FB4_ERR_ALLOC (-3)       /* host or device allocation of the LUT handle failed */
#define FB4_ERR_HIP (-4)         /* a HIP runtime call or kernel launch failed */

/* Dialect selectors (Sec. 3.2). */
#define FB4_SEL_SSE 0 /* exhaustive: squared error of every candidate over every element,
                         the "MSE-based" selection used for weights and the Exact-MSE ablation */
#define FB4_SEL_LUT 1 /* the paper's online rule: Qerror midpoint absolute error summed over
                         the group-wise maxima of num_groups contiguous groups */

/* Option flags. */
#define FB4_FLAG_TWO_STAGE 1u /* Sec. 3.2 "Two-stage Dialect Selection": first keep only the
                                 candidates whose largest magnitude equals the integer part of
                                 the normalized block maximum (8..15); if none has it, keep all */

#define FB4_DTYPE_BF16 0
#define FB4_DTYPE_F32 1

typedef struct fb4_luts fb4_luts; /* opaque, immutable after creation */

typedef struct fb4_opts {
    int32_t block;      /* 32 or 16 elements per block (Sec. 4.1 evaluates both)       */
    int32_t selector;   /* FB4_SEL_SSE or FB4_SEL_LUT                                  */
    int32_t num_groups; /* FB4_SEL_LUT only: 8, 16 or 32 groups per block, at most
                           `block` (paper: 8)                                           */
    uint32_t flags;     /* FB4_FLAG_*                                                */
} fb4_opts;

/* Library version, major*10000 + minor*100 + patch. */
int fb4_version(void);

/* Static, never-NULL description of a return code. */
const char* fb4_strerror(int code);

/* Bytes of caller-provided device workspace any call needs: always 0. */
size_t fb4_workspace_bytes(void);

/*
 * Sec. 3.2, "LUT-Based Quantization Error Approximation": build the per-dialect
 * lookup tables from a formatbook and upload them to the current HIP device.
 *   formatbook  host, uint8 [n_dialects][8], each row ascending and distinct,
 *               row[0] == 0, row[7] in 8..15 (FB4_ERR_INVALID_ARG otherwise)
 *   n_dialects  1..32
 *   out         host; receives a handle owned by the library until
 *               fb4_free_luts().  The handle is immutable and may be used from
 *               several streams and threads at once, on the device it was
 *               built on.
 * Tables: Qvalue (bin of width 0.5 over [0,16) -> exact 3-bit index of the
 * nearest magnitude, ties upward), Qerror (bin -> |bin midpoint - nearest
 * magnitude|, kept in quarter units so it is an odd integer 1..31), the
 * nearest-magnitude rows used by the exhaustive selector, and the decode table.
 */
int fb4_build_luts(const uint8_t* formatbook, int n_dialects, fb4_luts** out);

/*
 * Same tables, host only (no GPU needed): writes the blob that
 * fb4_build_luts() would upload into `blob` (host, `capacity` bytes) and its
 * size into *size (host, may be the only non-NULL output to query the size).
 * Blob layout, all little-endian, offsets in bytes:
 *      0  qerror8  uint8  [32 bins][32 dialects]   Qerror in quarter units
 *   1024  qvalue64 uint8  [32 dialects][64]        (sign<<5 | bin) -> sign<<3 | index
 *   3072  qerror16 uint16 [32 bins][32 dialects]   Qerror*32 (quarter units, pre-shifted)
 *   5120  mag16    uint16 [32 bins][32 dialects]   nearest magnitude m
 *   7168  gain16   uint16 [32 bins][32 dialects]   m * (bin - m)
 *   9216  decode   uint16 [32 dialects][8]         bf16 bit pattern of the magnitude
 *   9728  top      uint8  [32]                     largest magnitude of the dialect
 *   9760  n_dialects int32, then padding to 9792
 *   9792  qvalueT  uint8  [32 bins][32 dialects]   bin -> 3-bit index, bin-major copy of Qvalue
 *  10816  range_excl uint8 [8 ranges][32 dialects]  two-stage filter: 0xFF = largest magnitude != 8 + range
 * Total 11072 bytes.
 * Entries of dialects >= n_dialects are filled so that they never win.
 */
int fb4_build_luts_host(const uint8_t* formatbook, int n_dialects, void* blob, size_t capacity,
                        size_t* size);

/* Releases a handle (NULL is allowed).  The caller must have drained every
 * stream that still uses it. */
void fb4_free_luts(fb4_luts* luts);

/*
 * Sec. 3.1 + 3.2: quantize a [rows][cols] bf16 tensor with the full formatbook.
 * Per block: shared exponent from the largest magnitude, dialect selection by
 * opts->selector over all dialects (lowest DID wins ties), then every element
 * through Qvalue.  Also serves weight matrices (blocks along the contiguous
 * dimension).
 *   luts        handle from fb4_build_luts
 *   opts        host
 *   x           device, bf16 [rows][row_stride]
 *   codes,meta  device, outputs as described above
 */
int fb4_quantize(const fb4_luts* luts, const fb4_opts* opts, const void* x, int64_t rows,
                 int64_t cols, int64_t row_stride, uint8_t* codes, uint16_t* meta, void* stream);

/*
 * Sec. 3.4 (SeDA): as fb4_quantize, but a row whose token_group[r] = g >= 0
 * selects only among the eight DIDs sub_formatbooks[g][0..7]; the stored DID
 * is still the global one, so decoding is unchanged.
 *   token_group      device, int32 [rows]; -1 (or any value outside
 *                    0..n_groups-1) = full formatbook for that row
 *   sub_formatbooks  device, uint8 [n_groups][8]; entries >= n_dialects are
 *                    skipped; a group with no valid entry falls back to the
 *                    full formatbook
 *   n_groups         >= 1
 */
int fb4_quantize_seda(const fb4_luts* luts, const fb4_opts* opts, const void* x, int64_t rows,
                      int64_t cols, int64_t row_stride, const int32_t* token_group,
                      const uint8_t* sub_formatbooks, int n_groups, uint8_t* codes, uint16_t* meta,
                      void* stream);

/*
 * Sec. 3.3 (activation decomposition): for the salient rows only, form the
 * residual x - dequant(codes1, meta1) exactly, round it once to bf16 and
 * quantize it with the same routine into a compact second plane.
 *   x, rows, cols, row_stride   the original tensor (device)
 *   codes1, meta1               its first plane (device), as written by fb4_quantize*
 *   salient_rows                device, int32 [n_sal], ascending and unique row
 *                               indices; an index outside 0..rows-1 leaves its
 *                               output row untouched
 *   codes2                      device, uint8 [n_sal][cols/2]   (row p <-> salient_rows[p])
 *   meta2                       device, uint16 [n_sal][cols/block]
 *   token_group, sub_formatbooks, n_groups
 *                               optional SeDA restriction of the residual's
 *                               candidates (App. D); pass NULL, NULL, 0 for none
 */
int fb4_decompose(const fb4_luts* luts, const fb4_opts* opts, const void* x, int64_t rows,
                  int64_t cols, int64_t row_stride, const uint8_t* codes1, const uint16_t* meta1,
                  const int32_t* salient_rows, int64_t n_sal, const int32_t* token_group,
                  const uint8_t* sub_formatbooks, int n_groups, uint8_t* codes2, uint16_t* meta2,
                  void* stream);

/*
 * Sec. 3.1-3.4 in one pass: fb4_quantize (or fb4_quantize_seda when
 * token_group is given) followed by fb4_decompose of the salient rows with the
 * same options and SeDA lists, with identical results.  When the request fits
 * the streaming kernel (FB4_SEL_LUT with 8 groups or FB4_SEL_SSE, rows <=
 * 65536, cols a multiple of 32, 16-byte aligned code planes) x is read once and
 * the residual is formed from registers; otherwise the two kernels run one after
 * the other on `stream`.
 *   token_group, sub_formatbooks, n_groups   NULL, NULL, 0 for the full formatbook
 *   salient_rows, n_sal                      as in fb4_decompose; n_sal may be 0
 *   codes1, meta1                            first plane, every row
 *   codes2, meta2                            compact second plane, [n_sal] rows
 */
int fb4_quantize_decompose(const fb4_luts* luts, const fb4_opts* opts, const void* x, int64_t rows,
                           int64_t cols, int64_t row_stride, const int32_t* token_group,
                           const uint8_t* sub_formatbooks, int n_groups, const int32_t* salient_rows,
                           int64_t n_sal, uint8_t* codes1, uint16_t* meta1, uint8_t* codes2,
                           uint16_t* meta2, void* stream);

/*
 * Decode (Sec. 3.1; the 4-bit -> 16-bit decode of App. E.2).  Every row is
 * decoded from plane 1; a salient row additionally gets its second plane:
 * out = round_to_dtype(fp32(y1) + fp32(y2)) (Sec. 3.3, Q(Act) + Q(Delta)).
 *   codes2, meta2, salient_rows may all be NULL with n_sal = 0
 *   out             device, [rows][out_row_stride] of out_dtype
 *                   (FB4_DTYPE_BF16: 16-byte aligned rows; FB4_DTYPE_F32: 32-byte)
 * A DID >= n_dialects in the metadata decodes as all-zero magnitudes.
 */
int fb4_dequantize(const fb4_luts* luts, const uint8_t* codes1, const uint16_t* meta1,
                   int64_t rows, int64_t cols, int block, const uint8_t* codes2,
                   const uint16_t* meta2, const int32_t* salient_rows, int64_t n_sal, void* out,
                   int out_dtype, int64_t out_row_stride, void* stream);

/*
 * Sec. 3.4, "Constructing an 8-Dialect Sub-Formatbook": bin-count profile of
 * the dialects selected on the anchor tokens of each group, then per
 * dynamic-range bucket k (largest magnitude 8 + k) the most frequently selected
 * dialect of that bucket.  The result is a valid `sub_formatbooks` argument of
 * fb4_quantize_seda / fb4_decompose.
 *   meta             device, uint16 [rows][blocks_per_row], metadata of an
 *                    already quantized tensor (any block size)
 *   anchor_group     device, int32 [rows]: g in 0..n_groups-1 marks an anchor
 *                    token of group g; any other value: not an anchor
 *   counts           device, uint32 [n_groups][32], output (cleared by the
 *                    call): selections per group and DID, counted in blocks
 *   sub_formatbooks  device, uint8 [n_groups][8], output.  Ties go to the lowest
 *                    DID; a bucket none of whose dialects was selected gets its
 *                    lowest DID; a bucket the formatbook has no dialect for
 *                    gets 255, which the quantizing calls skip.
 * Which tokens are anchors is the caller's business (the paper derives them
 * from attention maps).
 */
int fb4_seda_profile(const fb4_luts* luts, const uint16_t* meta, int64_t rows, int64_t blocks_per_row,
                     const int32_t* anchor_group, int n_groups, uint32_t* counts,
                     uint8_t* sub_formatbooks, void* stream);

/*
 * Sec. 4.5 and App. E.2 (MXFP8 compatibility: the magnitudes 0..15 are exact
 * in FP8 E4M3 and the block scale is a power of two): re-encode one code plane
 * as MXFP8 operands for a block-scaled FP8 matrix unit, without going through
 * 16-bit values.  A salient row's second plane is repacked by a second call on
 * (codes2, meta2).
 *   codes, meta   device, one plane as written by fb4_quantize* / fb4_decompose
 *   cols          a multiple of 32 (FB4_ERR_UNSUPPORTED otherwise)
 *   elems         device, uint8 [rows][elem_row_stride]: OCP FP8 E4M3 (bias 7,
 *                 no infinities), sign bit copied from the code; rows 8-byte
 *                 aligned
 *   scales        device, uint8 [rows][cols/32], contiguous: E8M0, value 2^(s-127)
 * Block size 32: s = exponent byte - 3 and every element is its integer
 * magnitude, so elems * scale equals fb4_dequantize exactly.  Block size 16:
 * the two blocks of an MX block share the larger exponent; the elements of the
 * other block are magnitude * 2^-k (k = exponent difference) rounded to
 * nearest even in E4M3, which is exact for k <= 9 and zero for k >= 14.
 * A DID >= n_dialects gives zero magnitudes.
 */
int fb4_repack_mxfp8(const fb4_luts* luts, const uint8_t* codes, const uint16_t* meta, int64_t rows,
                     int64_t cols, int block, uint8_t* elems, int64_t elem_row_stride,
                     uint8_t* scales, void* stream);

/*
 * App. E.2 (the quantizer is fused into the operation that produces the
 * activation; LayerNorm is one of the two the paper names): LayerNorm over the
 * cols channels of every row, then fb4_quantize of the result, in one pass --
 * x is read once and the normalized tensor is never written.
 *   y[r][c] = (x[r][c] - mean_r) / sqrt(var_r + eps) * gamma[c] + beta[c]
 * with the biased variance, rounded once to bf16, is what gets quantized.  The
 * producer runs in fp32: mean_r from the sum of the row; var_r as the mean
 * square minus the squared mean where that difference keeps its bits (|mean_r|
 * below the standard deviation), else from the sum of the squared deviations
 * from mean_r in a walk of its own; then fma((x - mean_r) * rstd_r, gamma,
 * beta); a NaN result is the quiet NaN 0x7FC0.  Its bf16 result agrees with
 * the definition evaluated in double to within one bf16 step (almost always
 * exactly), or -- where gamma * t and beta cancel, or the mean dwarfs the
 * deviations -- to within 2^-19 (|gamma| (|t| + |mean_r| rstd_r + 1) + |beta|),
 * t = (x - mean_r) rstd_r; a constant row gives exactly beta, and the codes
 * are exactly fb4_quantize of that bf16 tensor.  Rows outside the
 * range of fp32 sums (an Inf or NaN, squares beyond 2^100, var + eps below
 * 2^-100) are evaluated in double instead.  x is read as plain IEEE bf16 (a
 * row with an Inf or NaN normalizes to NaN throughout).
 *   opts        FB4_SEL_LUT with 8 or 16 groups, block 32 or 16 (Sec. 4.1),
 *               FB4_FLAG_TWO_STAGE allowed; the exhaustive selector and 32 groups
 *               FB4_ERR_UNSUPPORTED
 *   cols        a multiple of 32, at most 12288 (FB4_ERR_UNSUPPORTED otherwise)
 *   gamma,beta  device, float [cols]; NULL = all ones / all zeros
 *   eps         >= 0 (FB4_ERR_INVALID_ARG otherwise)
 *   token_group, sub_formatbooks, n_groups
 *               Sec. 3.4, as in fb4_quantize_seda (the paper applies SeDA to
 *               mlp.fc1, whose input this is); all NULL / 0 = full formatbook;
 *               at most 255 groups (FB4_ERR_UNSUPPORTED beyond)
 *   codes       device, 16-byte aligned; meta 4-byte aligned with block 16
 *               (FB4_ERR_UNSUPPORTED otherwise)
 *   y_out       NULL in production.  For checking the producer: device, bf16
 *               [rows][cols], contiguous, 16-byte aligned; a second launch of
 *               the producer alone writes the normalized tensor there
 */
int fb4_layernorm_quantize(const fb4_luts* luts, const fb4_opts* opts, const void* x, int64_t rows,
                           int64_t cols, int64_t row_stride, const float* gamma, const float* beta,
                           float eps, const int32_t* token_group, const uint8_t* sub_formatbooks,
                           int n_groups, uint8_t* codes, uint16_t* meta, void* y_out, void* stream);

/*
 * App. E.2, the other producer the paper names: GeLU of every element, then
 * fb4_quantize of the result, in one pass -- x is read once and GeLU(x) is
 * never written.  What gets quantized is GeLU(x) evaluated in double and
 * rounded once to bf16 (nearest even); the library tabulates that for all
 * 65536 bf16 patterns when the handle is built.  GeLU(+Inf) = +Inf,
 * GeLU(-Inf) = -0 (the limit), GeLU(NaN) = the quiet NaN 0x7FC0, signed zeros
 * are kept.
 *   approximate  0: x * Phi(x) = 0.5 x erfc(-x / sqrt 2)
 *                1: the tanh form 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3)))
 *                anything else FB4_ERR_INVALID_ARG
 *   opts         FB4_SEL_LUT with 8 or 16 groups, block 32 or 16 (Sec. 4.1),
 *                FB4_FLAG_TWO_STAGE allowed; the exhaustive selector and 32 groups
 *                FB4_ERR_UNSUPPORTED; cols a multiple of 32
 *   token_group, sub_formatbooks, n_groups
 *                Sec. 3.4, as in fb4_quantize_seda (the paper applies SeDA to
 *                mlp.fc2, whose input this is); all NULL / 0 = full formatbook;
 *                at most 255 groups (FB4_ERR_UNSUPPORTED beyond)
 *   codes        device, 16-byte aligned; meta 4-byte aligned with block 16
 *                (FB4_ERR_UNSUPPORTED otherwise)
 */
int fb4_gelu_quantize(const fb4_luts* luts, const fb4_opts* opts, const void* x, int64_t rows,
                      int64_t cols, int64_t row_stride, int approximate, const int32_t* token_group,
                      const uint8_t* sub_formatbooks, int n_groups, uint8_t* codes, uint16_t* meta,
                      void* stream);

/*
 * The table fb4_gelu_quantize looks GeLU up in, for inspection without a GPU:
 * entry k is GeLU of the bf16 value with bit pattern k, for k = 0 .. 0xC180
 * (the positive patterns, then the negative ones down to -16.0; every value
 * below -16 shares the entry of -16, which is -0).
 *   table     host, uint16 [capacity]; capacity >= 49537 entries
 *             (FB4_ERR_INVALID_ARG otherwise)
 *   entries   host, optional: receives 49537
 */
int fb4_gelu_table_host(int approximate, uint16_t* table, size_t capacity, size_t* entries);

/*
 * Sec. 3.3 and App. F (attention-guided salient tokens): how strongly every
 * query token attends on average, pre-softmax:
 *   scores[g][i] = (1/tokens) * sum_j f(Q[g][i] . K[g][j]),
 *   f = |.| (mode 0: spatial / 3D attention) or max(., 0) (mode 1: temporal).
 * A group g is one attention problem: one head of one frame (spatial), of one
 * spatial position (temporal), or of the whole clip (3D).  Runs on the matrix
 * cores: bf16 products, fp32 accumulation and sums (results agree with a
 * float64 evaluation to about 1e-5 relative, not bit for bit).
 *   q, k     device, bf16 [groups][tokens][dim], contiguous, 16-byte aligned
 *   dim      a multiple of 8, at most 256 (FB4_ERR_UNSUPPORTED otherwise)
 *   scores   device, float [groups][tokens]
 */
int fb4_attention_scores(const void* q, const void* k, int64_t groups, int64_t tokens, int64_t dim,
                         int mode, float* scores, void* stream);

/*
 * Sec. 3.3 and App. F: one salient token per tile.  Per frame, the scores of
 * the heads are averaged (in double, head by head) and every tile_h x tile_w
 * tile of the grid_h x grid_w token grid (row-major tokens; ragged tiles at the
 * right / bottom edge allowed) contributes its best token: the lowest token
 * index on ties, a NaN never wins.
 *   scores    device, float [frames][heads][grid_h * grid_w]
 *   rows_out  device, int32 [frames][tiles], tiles = ceil(grid_h / tile_h) *
 *             ceil(grid_w / tile_w): the chosen tokens as rows frame * tokens +
 *             token of the [frames * tokens] activation, ascending -- the
 *             salient_rows argument of fb4_decompose / fb4_quantize_decompose
 *   grid_h * grid_w at most 8192 (FB4_ERR_UNSUPPORTED beyond)
 */
int fb4_select_salient_tokens(const float* scores, int64_t frames, int heads, int grid_h, int grid_w,
                              int tile_h, int tile_w, int32_t* rows_out, void* stream);

/*
 * Sec. 3.4 ("Attention-Guided Semantic Relatedness Extraction"), the marking
 * step (step 3 for factorized attention; the cuboid step for 3D attention):
 * every anchor token marks as correlated the tokens of a window x window
 * square -- times window_t frames: a cuboid -- centred on it and clipped to the
 * clip, whose raw pre-softmax attention score from the anchor, Q[anchor] .
 * K[token] averaged over the heads (fp32), exceeds `threshold`.
 * The GROUP of an anchor is the row-major number of the tile_h x tile_w spatial
 * tile it lies in, (y / tile_h) * ceil(grid_w / tile_w) + x / tile_w, so the
 * per-frame candidates of one tile share a group -- one sub-formatbook --
 * across the frames (step 1 yields one candidate per frame for a tile).  A token marked by
 * anchors of several groups belongs to the highest group number (App. D:
 * overlapping windows go to the subsequent anchor = the later tile); an anchor
 * belongs to its own group.
 *   q, k           device, bf16, 16-byte aligned, dim a multiple of 8
 *                  (FB4_ERR_UNSUPPORTED otherwise); tokens = grid_h * grid_w
 *                  joint = 0 (factorized attention): [frames][heads][tokens][dim],
 *                  the spatial attention's projections; window_t must be 1
 *                  joint = 1 (3D attention): [heads][frames * tokens][dim]
 *   anchors        device, int32 [n_anchors], rows of the [frames * tokens]
 *                  activation in any order (fb4_select_salient_tokens,
 *                  fb4_seda_main_anchor's `kept`, fb4_seda_main_anchor_3d); an
 *                  entry outside 0 .. frames * tokens - 1 (a pruned frame's -1)
 *                  does nothing
 *   window         1..8, window_t 1..64 (FB4_ERR_UNSUPPORTED beyond); the box
 *                  starts window / 2 tokens to the left and above and
 *                  window_t / 2 frames before the anchor
 *   token_group    device, int32 [frames * tokens]: group or -1 -- the
 *                  token_group argument of fb4_quantize_seda
 *   anchor_group   device, int32 [frames * tokens]: the group on anchor rows,
 *                  -1 elsewhere -- the anchor_group argument of
 *                  fb4_seda_profile (whose n_groups is the number of tiles)
 *   window_scores  device, float [n_anchors][window_t * window * window] or
 *                  NULL: the scores that were compared, frame offset major (NaN
 *                  outside the clip)
 */
int fb4_seda_assign(const void* q, const void* k, int joint, int64_t frames, int heads, int grid_h, int grid_w,
                    int64_t dim, const int32_t* anchors, int64_t n_anchors, int tile_h, int tile_w, int window,
                    int window_t, float threshold, int32_t* token_group, int32_t* anchor_group, float* window_scores,
                    void* stream);

/*
 * Sec. 3.4, factorized attention, step 2 (and App. H, "Temporal Axis
 * Integration"): per spatial tile, the main anchor among the tile's per-frame
 * candidates, and the pruning of the frames that are weakly correlated with it.
 * A candidate's tile is found from its position.  Main anchor = the candidate
 * whose own temporal mean attention score, averaged over the heads (in double,
 * head by head), is highest; the earliest frame on ties, a NaN never wins.
 * Frame f keeps its candidate if it is the main anchor's frame f*, or if the raw
 * temporal attention score from the main anchor to frame f at the main
 * anchor's position p*, Qt[p*][h][f*] . Kt[p*][h][f] averaged over the heads
 * (fp32), exceeds prune_threshold.
 *   temporal_scores  device, float [tokens][heads][frames]: what
 *                    fb4_attention_scores returns for the temporal attention
 *                    (group = spatial position and head, tokens = frames)
 *   qt, kt           device, bf16 [tokens][heads][frames][dim], the temporal
 *                    attention's projections; dim a multiple of 8
 *   candidates       device, int32 [frames][n_per_frame]: per frame the anchor
 *                    candidates of step 1 as rows of the [frames * tokens]
 *                    activation (fb4_select_salient_tokens); an entry outside
 *                    its own frame is no candidate; of several candidates of
 *                    one tile in one frame the first listed counts
 *   main_anchor      device, int32 [tiles]: the main anchor's row, -1 for a tile
 *                    without candidates
 *   kept             device, int32 [frames][n_per_frame]: `candidates` with the
 *                    pruned and the invalid entries set to -1 -- the `anchors`
 *                    argument of fb4_seda_assign
 *   prune_scores     device, float [frames][tiles] or NULL: the scores that
 *                    were compared (NaN where a frame has no candidate)
 *   frames at most 1024 (FB4_ERR_UNSUPPORTED beyond)
 */
int fb4_seda_main_anchor(const float* temporal_scores, const void* qt, const void* kt, int64_t frames, int heads,
                         int grid_h, int grid_w, int64_t dim, const int32_t* candidates, int n_per_frame, int tile_h,
                         int tile_w, float prune_threshold, int32_t* main_anchor, int32_t* kept, float* prune_scores,
                         void* stream);

/*
 * Sec. 3.4, 3D attention: the main anchor of every spatial tile is the token
 * with the highest mean attention score among the tile's tile_h x tile_w x
 * frames tokens; the scores of the heads are averaged in double, head by head;
 * the lowest row on ties, a NaN never wins.
 *   scores    device, float [heads][frames * tokens]: fb4_attention_scores with
 *             one group per head over the whole clip
 *   anchors   device, int32 [tiles], tiles = ceil(grid_h / tile_h) *
 *             ceil(grid_w / tile_w): rows of the [frames * tokens] activation,
 *             in tile order -- the `anchors` argument of fb4_seda_assign with
 *             joint = 1
 */
int fb4_seda_main_anchor_3d(const float* scores, int64_t frames, int heads, int grid_h, int grid_w, int tile_h,
                            int tile_w, int32_t* anchors, void* stream);

/*
 * Diagnostic, not part of the paper's method: launches a kernel that does
 * nothing but v_mfma_f32_32x32x16_bf16 on operands held in registers (four
 * independent accumulator chains per wavefront, four wavefronts per workgroup,
 * 32 MFMAs per iteration and wavefront), so that a caller who times it learns
 * the dense bf16 matrix rate this device sustains -- which depends on the
 * operand data, because the power management lowers the clock under load.
 * bench.py reports it beside the rate of fb4_attention_scores.
 *   workgroups        1..65536 (256 threads each; two per compute unit fill
 *                     the matrix cores)
 *   iterations        loop count per wavefront
 *   random_operands   0: one bit pattern in every operand element; otherwise
 *                     random signs and mantissas, magnitudes in [0.5, 2)
 *   out               device, float [workgroups * 256]: written so that the
 *                     loop is not optimized away; the values mean nothing
 *   flop              host, or NULL: receives the operations the launch performs
 */
int fb4_probe_mfma_rate(int64_t workgroups, int64_t iterations, int random_operands, float* out, double* flop, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FB4_H */
