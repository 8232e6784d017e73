/*
 * fb4_oracle.c -- plain CPU oracle for the FB4 online quantizer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines, in the slowest and plainest
 * way, what the GPU library must compute.  It shares no code, table or
 * constant with the library and must never be called from the product path;
 * only tests, the smoke check and the benchmark's CPU-baseline leg use it.
 *
 * Everything follows the paper's Sec. 3.1 (block normalization, the 4-bit
 * sign+index element, the formatbook), Sec. 3.2 (dialect selection and
 * quantization), Sec. 3.3 (activation decomposition) and Sec. 3.4 (SeDA
 * sub-formatbooks).  Floating point is done in double.  There are no lookup
 * tables here: rounding into a dialect is a scan over its eight magnitudes,
 * selection is a scan over the candidate dialects.  The only concurrency is
 * an OpenMP loop over rows, which are independent.
 *
 * Readings taken where the paper is silent (the same list is in the design
 * notes of the repository):
 *   - a NaN element is ignored by the block maximum and by every error sum
 *     and is emitted as index 0 with its sign bit;
 *   - +/-Inf is read from its bit pattern as the finite magnitude 2^128;
 *   - the shared exponent e = floor(log2(max|x|)) is clamped to [-123, 127]
 *     (an all-zero block gets -123) and stored as the byte e+127, so that
 *     every dequantized value is a normal bf16;
 *   - rounding ties go to the larger magnitude (Sec. 3.2: a truncating
 *     0.5-wide bin whose left edge is a decision boundary maps upward);
 *   - selection ties go to the lowest dialect ID;
 *   - groups for the group-wise maxima are contiguous runs of block/g
 *     elements;
 *   - the sign bit of the input is copied to the code unconditionally;
 *   - element 2j sits in the low nibble and 2j+1 in the high nibble of code
 *     byte j; metadata is DID | (e+127) << 8;
 *   - the residual of the decomposition is computed exactly and rounded once
 *     to bf16 (round to nearest even); a non-finite input is its own residual;
 *   - a reconstructed salient value is bf16(fp32(y1) + fp32(y2));
 *   - MXFP8 operands: block size 32 maps one to one; with block size 16 the
 *     two blocks of an MX block share the larger exponent and the other
 *     block's magnitudes are shifted down and rounded to nearest even in E4M3;
 *   - a producer in front of the quantizer (App. E.2 names GeLU and
 *     LayerNorm) hands the quantizer bf16 values: the producer's definition
 *     evaluated in double and rounded once to bf16 (LayerNorm: the textbook
 *     two-pass definition with the biased variance; GeLU(-Inf) = -0, the
 *     limit, and GeLU(NaN) = the quiet NaN 0x7FC0).
 *
 * Every routine here is pinned by tests/test_oracle_pins.py against hand-worked
 * fixtures, closed forms, exact rational brute force or torch's own number
 * formats.  Parity unpinned: the VALUES of the default 32-dialect formatbook
 * (input data of every routine; the paper gives them only in a figure that is
 * not available), and how often the online rule and the exhaustive rule pick
 * the same dialect (the paper only says quality is comparable).
 */
#define _GNU_SOURCE
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define FB4O_SEL_SSE 0 /* exhaustive squared error over all elements   */
#define FB4O_SEL_LUT 1 /* paper's online rule: midpoint abs error over  */
                       /* group-wise maxima                             */
#define FB4O_FLAG_TWO_STAGE 1

#define FB4O_OUT_BF16 0
#define FB4O_OUT_F32 1

#define FB4O_MAX_BLOCK 32
#define FB4O_MAX_DIALECTS 32

/* ------------------------------------------------------------------ */
/* bf16 <-> double                                                    */

typedef struct {
    int is_nan;
    int sign;
    double mag; /* |x| as a finite double (Inf read as 2^128) */
} fb4o_elem;

static fb4o_elem decode_bf16(uint16_t bits)
{
    fb4o_elem r;
    int ef = (bits >> 7) & 0xFF;
    int mant = bits & 0x7F;
    r.sign = bits >> 15;
    r.is_nan = 0;
    if (ef == 255) {
        if (mant != 0) {
            r.is_nan = 1;
            r.mag = 0.0;
        } else {
            r.mag = ldexp(1.0, 128);
        }
    } else if (ef == 0) {
        r.mag = ldexp((double)mant, -133);
    } else {
        r.mag = ldexp((double)(128 + mant), ef - 127 - 7);
    }
    return r;
}

/* Exact IEEE value of a bf16 bit pattern (Inf stays Inf), for residuals. */
static double bf16_value(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* float -> bf16 bits, round to nearest even (no NaN input reaches this). */
static uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* ------------------------------------------------------------------ */
/* Sec. 3.1: shared exponent and normalization                        */

/* floor(log2(a)) clamped to [-123, 127]; -123 for a == 0. */
static int block_exponent(double a)
{
    int ex;
    if (a == 0.0) return -123;
    frexp(a, &ex); /* a = f * 2^ex, f in [0.5, 1)  =>  floor(log2 a) = ex-1 */
    ex -= 1;
    if (ex < -123) ex = -123;
    if (ex > 127) ex = 127;
    return ex;
}

/* Normalized magnitude: |x| * 2^(3-e), in [0,16) with the block maximum in
 * [8,16) whenever e was not clamped. */
static double normalize(double mag, int e) { return ldexp(mag, 3 - e); }

/* Sec. 3.2: nearest representable magnitude of a dialect, ties upward,
 * saturating at the largest one.  Returns the 3-bit index. */
static int nearest_index(const uint8_t* dialect, double xhat)
{
    int best = 0;
    double bestd = fabs(xhat - (double)dialect[0]);
    for (int k = 1; k < 8; ++k) {
        double d = fabs(xhat - (double)dialect[k]);
        if (d <= bestd) { /* magnitudes ascend, so <= keeps the larger on a tie */
            bestd = d;
            best = k;
        }
    }
    return best;
}

/* ------------------------------------------------------------------ */
/* formatbook checks                                                  */

int fb4o_validate_formatbook(const uint8_t* fbk, int n)
{
    if (!fbk || n < 1 || n > FB4O_MAX_DIALECTS) return -1;
    for (int d = 0; d < n; ++d) {
        const uint8_t* m = fbk + 8 * d;
        if (m[0] != 0) return -1;
        for (int k = 1; k < 8; ++k)
            if (m[k] <= m[k - 1]) return -1;
        if (m[7] > 15 || m[7] < 8) return -1;
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* scores                                                             */

/* Exhaustive squared error (Sec. 3.2 first paragraph; the "Exact MSE" row of
 * the selector ablation).  Error is measured on normalized values; the block
 * scale is common to all dialects so the argmin is that of the unscaled
 * error.  An element with xhat < 0.5 rounds to 0 in every dialect (every
 * non-zero magnitude is >= 1), adds the same xhat^2 to every candidate and is
 * left out, which keeps every partial sum exactly representable in double
 * (each remaining term is a multiple of 2^-16 below 2^8). */
static double score_sse(const uint8_t* dialect, const double* xhat, const int* is_nan, int block)
{
    double s = 0.0;
    for (int i = 0; i < block; ++i) {
        if (is_nan[i] || xhat[i] < 0.5) continue;
        double m = (double)dialect[nearest_index(dialect, xhat[i])];
        s += (xhat[i] - m) * (xhat[i] - m);
    }
    return s;
}

/* The paper's online rule (Sec. 3.2, "Group-wise Maximum Extraction" and
 * "LUT-Based Quantization Error Approximation"): split the block into g
 * contiguous groups, take each group's largest normalized magnitude, replace
 * it by the midpoint of its 0.5-wide bin and add up the absolute distance from
 * that midpoint to the dialect's nearest magnitude. */
static double score_lut(const uint8_t* dialect, const double* xhat, const int* is_nan, int block,
                        int num_groups)
{
    int per = block / num_groups;
    double s = 0.0;
    for (int j = 0; j < num_groups; ++j) {
        double u = 0.0;
        for (int i = j * per; i < (j + 1) * per; ++i)
            if (!is_nan[i] && xhat[i] > u) u = xhat[i];
        double bin = floor(2.0 * u);
        if (bin > 31.0) bin = 31.0;
        double mid = 0.5 * bin + 0.25;
        double m = (double)dialect[nearest_index(dialect, mid)];
        s += fabs(mid - m);
    }
    return s;
}

/* ------------------------------------------------------------------ */
/* one block                                                          */

typedef struct {
    int did;
    int e;                       /* clamped shared exponent */
    int idx[FB4O_MAX_BLOCK];     /* 3-bit indices           */
    int sign[FB4O_MAX_BLOCK];
    double scores[FB4O_MAX_DIALECTS]; /* score per candidate, in candidate order */
    int cand[FB4O_MAX_DIALECTS];
    int n_cand;
} fb4o_block_result;

/* cand_in: ascending DIDs to consider (all dialects, or a SeDA sub-formatbook). */
static void quantize_block(const uint8_t* fbk, int selector, int num_groups, int flags,
                           const uint16_t* x, int block, const int* cand_in, int n_cand_in,
                           fb4o_block_result* out)
{
    double xhat[FB4O_MAX_BLOCK];
    int is_nan[FB4O_MAX_BLOCK];
    fb4o_elem el[FB4O_MAX_BLOCK];
    double a = 0.0;
    for (int i = 0; i < block; ++i) {
        el[i] = decode_bf16(x[i]);
        is_nan[i] = el[i].is_nan;
        out->sign[i] = el[i].sign;
        if (!el[i].is_nan && el[i].mag > a) a = el[i].mag;
    }
    int e = block_exponent(a);
    double xmax = 0.0;
    for (int i = 0; i < block; ++i) {
        xhat[i] = el[i].is_nan ? 0.0 : normalize(el[i].mag, e);
        if (xhat[i] > xmax) xmax = xhat[i];
    }

    /* candidate set; two-stage selection (Sec. 3.2, "Two-stage Dialect
     * Selection") first keeps only the dialects whose dynamic range -- their
     * largest magnitude -- equals the integer part of the block maximum
     * (8..15).  If no candidate has that range the first stage is skipped. */
    int n_cand = 0;
    if (flags & FB4O_FLAG_TWO_STAGE) {
        int r = (int)floor(xmax);
        if (r < 8) r = 8;
        if (r > 15) r = 15;
        for (int c = 0; c < n_cand_in; ++c)
            if (fbk[8 * cand_in[c] + 7] == r) out->cand[n_cand++] = cand_in[c];
    }
    if (n_cand == 0)
        for (int c = 0; c < n_cand_in; ++c) out->cand[n_cand++] = cand_in[c];
    out->n_cand = n_cand;

    int best = -1;
    double bests = 0.0;
    for (int c = 0; c < n_cand; ++c) {
        const uint8_t* dialect = fbk + 8 * out->cand[c];
        double s = (selector == FB4O_SEL_SSE) ? score_sse(dialect, xhat, is_nan, block)
                                              : score_lut(dialect, xhat, is_nan, block, num_groups);
        out->scores[c] = s;
        if (best < 0 || s < bests || (s == bests && out->cand[c] < best)) {
            best = out->cand[c];
            bests = s;
        }
    }
    out->did = best;
    out->e = e;
    for (int i = 0; i < block; ++i)
        out->idx[i] = is_nan[i] ? 0 : nearest_index(fbk + 8 * best, xhat[i]);
}

static void pack_block(const fb4o_block_result* r, int block, uint8_t* codes, uint16_t* meta)
{
    for (int j = 0; j < block / 2; ++j) {
        int lo = (r->sign[2 * j] << 3) | r->idx[2 * j];
        int hi = (r->sign[2 * j + 1] << 3) | r->idx[2 * j + 1];
        codes[j] = (uint8_t)(lo | (hi << 4));
    }
    *meta = (uint16_t)(r->did | ((r->e + 127) << 8));
}

/* value of one code: (-1)^sign * M[did][idx] * 2^(e-3) */
static double code_value(const uint8_t* fbk, uint16_t meta, int nibble)
{
    int did = meta & 0xFF;
    int e = (meta >> 8) - 127;
    double v = ldexp((double)fbk[8 * did + (nibble & 7)], e - 3);
    return (nibble & 8) ? -v : v;
}

static int nibble_at(const uint8_t* codes, int64_t i)
{
    return (i & 1) ? (codes[i >> 1] >> 4) : (codes[i >> 1] & 0xF);
}

static int check_common(const uint8_t* fbk, int n_dialects, int block, int selector, int num_groups,
                        int64_t rows, int64_t cols)
{
    if (fb4o_validate_formatbook(fbk, n_dialects)) return -1;
    if (block != 16 && block != 32) return -1;
    if (selector != FB4O_SEL_SSE && selector != FB4O_SEL_LUT) return -1;
    if (selector == FB4O_SEL_LUT && (num_groups < 1 || block % num_groups)) return -1;
    if (rows < 0 || cols < 0 || cols % block) return -1;
    return 0;
}

static int row_candidates(int n_dialects, const int32_t* token_group, const uint8_t* sub_fbk,
                          int n_groups, int64_t row, int* cand)
{
    if (token_group && token_group[row] >= 0) {
        /* Sec. 3.4: the token's group shares one 8-dialect sub-formatbook */
        const uint8_t* s = sub_fbk + 8 * (int64_t)token_group[row];
        (void)n_groups;
        for (int k = 0; k < 8; ++k) cand[k] = s[k];
        return 8;
    }
    for (int d = 0; d < n_dialects; ++d) cand[d] = d;
    return n_dialects;
}

static int check_seda(int n_dialects, const int32_t* token_group, const uint8_t* sub_fbk,
                      int n_groups, int64_t rows)
{
    if (!token_group) return 0;
    if (!sub_fbk || n_groups < 1) return -1;
    for (int g = 0; g < n_groups; ++g)
        for (int k = 0; k < 8; ++k) {
            if (sub_fbk[8 * g + k] >= n_dialects) return -1;
            if (k && sub_fbk[8 * g + k] <= sub_fbk[8 * g + k - 1]) return -1;
        }
    for (int64_t r = 0; r < rows; ++r)
        if (token_group[r] < -1 || token_group[r] >= n_groups) return -1;
    return 0;
}

/* ------------------------------------------------------------------ */
/* public entry points                                                */

int fb4o_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Quantize a [rows][cols] bf16 tensor (bit patterns, row stride in elements)
 * into codes [rows][cols/2] and meta [rows][cols/block].  token_group may be
 * NULL (full formatbook everywhere) or hold, per row, a SeDA group index or
 * -1.  Returns 0, or -1 on an invalid argument. */
int fb4o_quantize(const uint8_t* fbk, int n_dialects, int block, int selector, int num_groups,
                  int flags, const uint16_t* x, int64_t rows, int64_t cols, int64_t row_stride,
                  const int32_t* token_group, const uint8_t* sub_fbk, int n_groups, uint8_t* codes,
                  uint16_t* meta, int nthreads)
{
    if (check_common(fbk, n_dialects, block, selector, num_groups, rows, cols)) return -1;
    if (check_seda(n_dialects, token_group, sub_fbk, n_groups, rows)) return -1;
    if (row_stride < cols) return -1;
    int64_t nb = cols / block;
#ifdef _OPENMP
    if (nthreads < 1) nthreads = omp_get_max_threads();
#pragma omp parallel for schedule(static) num_threads(nthreads)
#endif
    for (int64_t r = 0; r < rows; ++r) {
        int cand[FB4O_MAX_DIALECTS];
        int n_cand = row_candidates(n_dialects, token_group, sub_fbk, n_groups, r, cand);
        for (int64_t b = 0; b < nb; ++b) {
            fb4o_block_result res;
            quantize_block(fbk, selector, num_groups, flags, x + r * row_stride + b * block, block,
                           cand, n_cand, &res);
            pack_block(&res, block, codes + r * (cols / 2) + b * (block / 2), meta + r * nb + b);
        }
    }
    (void)nthreads;
    return 0;
}

/* Scores of one block for every candidate dialect (diagnostics and pins).
 * scores[c] belongs to cand_out[c]; returns the number of candidates scored,
 * or -1.  did_out / e_out receive the selection and the clamped exponent. */
int fb4o_block_scores(const uint8_t* fbk, int n_dialects, int block, int selector, int num_groups,
                      int flags, const uint16_t* x, const uint8_t* sub8, double* scores,
                      int* cand_out, int* did_out, int* e_out)
{
    if (check_common(fbk, n_dialects, block, selector, num_groups, 1, block)) return -1;
    int cand[FB4O_MAX_DIALECTS];
    int n_cand;
    if (sub8) {
        for (int k = 0; k < 8; ++k) cand[k] = sub8[k];
        n_cand = 8;
    } else {
        for (int d = 0; d < n_dialects; ++d) cand[d] = d;
        n_cand = n_dialects;
    }
    fb4o_block_result res;
    quantize_block(fbk, selector, num_groups, flags, x, block, cand, n_cand, &res);
    for (int c = 0; c < res.n_cand; ++c) {
        scores[c] = res.scores[c];
        cand_out[c] = res.cand[c];
    }
    *did_out = res.did;
    *e_out = res.e;
    return res.n_cand;
}

/* Sec. 3.3: second plane for the salient rows.  For row salient_rows[p] the
 * residual x - dequant(plane 1) is formed exactly, rounded once to bf16 and
 * quantized by the same routine into codes2[p], meta2[p].  token_group (may be
 * NULL) restricts the residual's candidates the same way as the first plane
 * (App. D, decomposition combined with SeDA). */
int fb4o_decompose(const uint8_t* fbk, int n_dialects, int block, int selector, int num_groups,
                   int flags, const uint16_t* x, int64_t rows, int64_t cols, int64_t row_stride,
                   const uint8_t* codes1, const uint16_t* meta1, const int32_t* salient_rows,
                   int64_t n_sal, const int32_t* token_group, const uint8_t* sub_fbk, int n_groups,
                   uint8_t* codes2, uint16_t* meta2, int nthreads)
{
    if (check_common(fbk, n_dialects, block, selector, num_groups, rows, cols)) return -1;
    if (check_seda(n_dialects, token_group, sub_fbk, n_groups, rows)) return -1;
    if (row_stride < cols || n_sal < 0) return -1;
    for (int64_t p = 0; p < n_sal; ++p) {
        if (salient_rows[p] < 0 || salient_rows[p] >= rows) return -1;
        if (p && salient_rows[p] <= salient_rows[p - 1]) return -1;
    }
    int64_t nb = cols / block;
#ifdef _OPENMP
    if (nthreads < 1) nthreads = omp_get_max_threads();
#pragma omp parallel for schedule(static) num_threads(nthreads)
#endif
    for (int64_t p = 0; p < n_sal; ++p) {
        int64_t r = salient_rows[p];
        int cand[FB4O_MAX_DIALECTS];
        int n_cand = row_candidates(n_dialects, token_group, sub_fbk, n_groups, r, cand);
        for (int64_t b = 0; b < nb; ++b) {
            uint16_t delta[FB4O_MAX_BLOCK];
            const uint16_t* xb = x + r * row_stride + b * block;
            const uint8_t* cb = codes1 + r * (cols / 2) + b * (block / 2);
            uint16_t m1 = meta1[r * nb + b];
            for (int i = 0; i < block; ++i) {
                int ef = (xb[i] >> 7) & 0xFF;
                if (ef == 255) { /* Inf or NaN: its own residual */
                    delta[i] = xb[i];
                    continue;
                }
                double y = code_value(fbk, m1, nibble_at(cb, i));
                double d = bf16_value(xb[i]) - y; /* exact: at most 13 significant bits */
                delta[i] = f32_to_bf16_rne((float)d);
            }
            fb4o_block_result res;
            quantize_block(fbk, selector, num_groups, flags, delta, block, cand, n_cand, &res);
            pack_block(&res, block, codes2 + p * (cols / 2) + b * (block / 2), meta2 + p * nb + b);
        }
    }
    (void)nthreads;
    return 0;
}

/* Decode: y = (-1)^sign * M[did][idx] * 2^(e-3); for salient rows the two
 * planes are added in fp32 (Sec. 3.3: Q(Act) + Q(Delta)).  out is bf16 bit
 * patterns or float, row stride in elements. */
int fb4o_dequantize(const uint8_t* fbk, int n_dialects, int block, const uint8_t* codes1,
                    const uint16_t* meta1, int64_t rows, int64_t cols, const uint8_t* codes2,
                    const uint16_t* meta2, const int32_t* salient_rows, int64_t n_sal, void* out,
                    int out_dtype, int64_t out_row_stride, int nthreads)
{
    if (fb4o_validate_formatbook(fbk, n_dialects)) return -1;
    if ((block != 16 && block != 32) || rows < 0 || cols < 0 || cols % block) return -1;
    if (out_dtype != FB4O_OUT_BF16 && out_dtype != FB4O_OUT_F32) return -1;
    if (out_row_stride < cols || n_sal < 0) return -1;
    if (n_sal > 0 && (!codes2 || !meta2 || !salient_rows)) return -1;
    int64_t nb = cols / block;
    for (int64_t i = 0; i < rows * nb; ++i)
        if ((meta1[i] & 0xFF) >= n_dialects) return -1;
    for (int64_t i = 0; i < n_sal * nb; ++i)
        if ((meta2[i] & 0xFF) >= n_dialects) return -1;
    int64_t* pos = (int64_t*)malloc(sizeof(int64_t) * (size_t)(rows > 0 ? rows : 1));
    if (!pos) return -1;
    for (int64_t r = 0; r < rows; ++r) pos[r] = -1;
    for (int64_t p = 0; p < n_sal; ++p) {
        if (salient_rows[p] < 0 || salient_rows[p] >= rows ||
            (p && salient_rows[p] <= salient_rows[p - 1])) {
            free(pos);
            return -1;
        }
        pos[salient_rows[p]] = p;
    }
#ifdef _OPENMP
    if (nthreads < 1) nthreads = omp_get_max_threads();
#pragma omp parallel for schedule(static) num_threads(nthreads)
#endif
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t c = 0; c < cols; ++c) {
            int64_t b = c / block;
            float y = (float)code_value(fbk, meta1[r * nb + b], nibble_at(codes1 + r * (cols / 2), c));
            if (pos[r] >= 0) {
                int64_t p = pos[r];
                float y2 =
                    (float)code_value(fbk, meta2[p * nb + b], nibble_at(codes2 + p * (cols / 2), c));
                y = y + y2; /* one fp32 addition */
            }
            if (out_dtype == FB4O_OUT_F32)
                ((float*)out)[r * out_row_stride + c] = y;
            else
                ((uint16_t*)out)[r * out_row_stride + c] = f32_to_bf16_rne(y);
        }
    }
    free(pos);
    (void)nthreads;
    return 0;
}

/* ------------------------------------------------------------------ */
/* MXFP8 operands                                                      */
/* ------------------------------------------------------------------ */

/* OCP FP8 E4M3 encoding (bias 7, 3 mantissa bits, subnormals down to 2^-9,
 * no infinities) of a finite 0 <= v < 448, round to nearest, ties to even. */
static uint8_t e4m3_of(double v)
{
    if (v == 0.0) return 0;
    int ex;
    (void)frexp(v, &ex); /* v = f * 2^ex, f in [0.5, 1) */
    int e = ex - 1;      /* floor(log2 v) */
    if (e < -6) e = -6;  /* subnormals share the spacing of the smallest normal binade */
    double n = nearbyint(ldexp(v, 3 - e)); /* v in units of the spacing 2^(e-3); default rounding = ties to even */
    if (n < 8.0) return (uint8_t)n;        /* subnormal (only reachable with e == -6) */
    /* n in 8..16: exponent field and three mantissa bits; n == 16 (rounded up to the next power of two)
     * carries into the exponent field by itself */
    return (uint8_t)(((e + 7) << 3) + ((int)n - 8));
}

/* Sec. 4.5 / App. E.2: the integer magnitudes 0..15 are exact in FP8 E4M3 and
 * the block scale is a power of two, so a code plane is an MXFP8 operand: per
 * 32 elements one E8M0 scale byte s (scale 2^(s-127)) and 32 E4M3 bytes.
 * Block size 32: s = (e+127) - 3 and element = +/- magnitude, exact.  Block
 * size 16: the two blocks of an MX block share the larger exponent; the
 * elements of the other one are magnitude * 2^(e_small - e_large), rounded to
 * E4M3 (exact while the exponents differ by at most 9).
 * elems [rows][cols] bytes, scales [rows][cols/32]; cols % 32 == 0. */
int fb4o_repack_mxfp8(const uint8_t* fbk, int n_dialects, int block, const uint8_t* codes,
                      const uint16_t* meta, int64_t rows, int64_t cols, uint8_t* elems, uint8_t* scales)
{
    if (fb4o_validate_formatbook(fbk, n_dialects)) return -1;
    if ((block != 16 && block != 32) || rows < 0 || cols < 0 || cols % 32) return -1;
    int64_t nb = cols / block;
    for (int64_t i = 0; i < rows * nb; ++i)
        if ((meta[i] & 0xFF) >= n_dialects) return -1;
    int per = 32 / block; /* FB4 blocks per MX block */
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t q = 0; q < cols / 32; ++q) {
            int emax = 0;
            for (int k = 0; k < per; ++k) {
                int eb = meta[r * nb + q * per + k] >> 8;
                if (eb > emax) emax = eb;
            }
            scales[r * (cols / 32) + q] = (uint8_t)(emax - 3);
            for (int i = 0; i < 32; ++i) {
                int64_t c = q * 32 + i;
                uint16_t m = meta[r * nb + c / block];
                int nib = nibble_at(codes + r * (cols / 2), c);
                double mag = (double)fbk[(m & 0xFF) * 8 + (nib & 7)];
                double v = ldexp(mag, (int)(m >> 8) - emax);
                elems[r * cols + c] = (uint8_t)(e4m3_of(v) | ((nib & 8) << 4));
            }
        }
    }
    return 0;
}


/* ------------------------------------------------------------------ */
/* double -> bf16 bits, one rounding to nearest even (NaN -> the quiet NaN
 * 0x7FC0, overflow -> Inf, subnormals in steps of 2^-133). */
static uint16_t f64_to_bf16_rne(double v)
{
    if (isnan(v)) return 0x7FC0;
    uint16_t sign = signbit(v) ? 0x8000 : 0;
    double a = fabs(v);
    if (a == 0.0) return sign;
    if (isinf(a)) return (uint16_t)(sign | 0x7F80);
    int ex;
    (void)frexp(a, &ex); /* a = f * 2^ex, f in [0.5, 1) */
    int e = ex - 1;      /* floor(log2 a) */
    if (e < -126) {      /* subnormal range: steps of 2^-133 */
        double q = rint(ldexp(a, 133));
        return (uint16_t)(sign | (uint16_t)q); /* q == 128 is the smallest normal */
    }
    double q = rint(ldexp(a, 7 - e)); /* 128 .. 256 */
    if (q >= 256.0) {
        q = 128.0;
        e += 1;
    }
    if (e + 127 >= 255) return (uint16_t)(sign | 0x7F80);
    return (uint16_t)(sign | ((e + 127) << 7) | ((int)q - 128));
}

/* App. E.2: the quantizer runs fused behind the operation that produces the
 * activation; LayerNorm is one of the two the paper names.  The paper does not
 * define that operation, so this is the textbook one over the channels of a
 * token, written out from its definition in double:
 *   mean = (1/C) sum_c x_c
 *   var  = (1/C) sum_c (x_c - mean)^2            (biased; two passes)
 *   y_c  = (x_c - mean) / sqrt(var + eps) * gamma_c + beta_c
 * and the quantizer's input is y_c rounded ONCE to bf16 (nearest even; a NaN
 * becomes the quiet NaN 0x7FC0).  x is read as plain IEEE bf16: a row that
 * holds an Inf or a NaN is NaN throughout.
 * gamma / beta: [cols] or NULL (1 / 0).  y: [rows][cols] bf16 bit patterns;
 * mean_out, rstd_out: [rows] doubles or NULL (rstd = 1 / sqrt(var + eps)). */
int fb4o_layernorm(const uint16_t* x, int64_t rows, int64_t cols, int64_t row_stride, const float* gamma,
                   const float* beta, double eps, uint16_t* y, double* mean_out, double* rstd_out)
{
    if (!x || !y || rows < 0 || cols <= 0 || row_stride < cols) return -1;
    for (int64_t r = 0; r < rows; ++r) {
        const uint16_t* xr = x + r * row_stride;
        double sum = 0.0;
        for (int64_t c = 0; c < cols; ++c) sum += bf16_value(xr[c]);
        double mean = sum / (double)cols;
        double sq = 0.0;
        for (int64_t c = 0; c < cols; ++c) {
            double d = bf16_value(xr[c]) - mean;
            sq += d * d;
        }
        double var = sq / (double)cols;
        double rstd = 1.0 / sqrt(var + eps);
        if (mean_out) mean_out[r] = mean;
        if (rstd_out) rstd_out[r] = rstd;
        for (int64_t c = 0; c < cols; ++c) {
            double g = gamma ? (double)gamma[c] : 1.0;
            double b = beta ? (double)beta[c] : 0.0;
            double v = (bf16_value(xr[c]) - mean) * rstd * g + b;
            y[r * cols + c] = f64_to_bf16_rne(v);
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* App. E.2: the other producer the paper names is GeLU.  Elementwise on bf16:
 * the value in double, rounded once to bf16 (nearest even).
 *   approximate == 0:  x * Phi(x) = 0.5 * x * erfc(-x / sqrt(2))
 *   approximate == 1:  the tanh form 0.5 * x * (1 + tanh(u)),
 *                      u = sqrt(2/pi) * (x + 0.044715 x^3), written as
 *                      x / (1 + exp(-2u)) so that nothing cancels for x << 0
 * GeLU(+Inf) = +Inf, GeLU(-Inf) = -0 (the limit), GeLU(NaN) = 0x7FC0. */
int fb4o_gelu(const uint16_t* x, int64_t n, int approximate, uint16_t* y)
{
    if ((!x || !y) && n > 0) return -1;
    if (n < 0 || (approximate != 0 && approximate != 1)) return -1;
    for (int64_t i = 0; i < n; ++i) {
        double v = bf16_value(x[i]);
        double r;
        if (isnan(v)) {
            y[i] = 0x7FC0;
            continue;
        }
        if (isinf(v)) {
            y[i] = v > 0 ? 0x7F80 : 0x8000;
            continue;
        }
        if (approximate == 0) {
            r = 0.5 * v * erfc(-v / sqrt(2.0));
        } else {
            double u = sqrt(2.0 / M_PI) * (v + 0.044715 * v * v * v);
            r = v / (1.0 + exp(-2.0 * u));
        }
        y[i] = f64_to_bf16_rne(r);
        if (v == 0.0) y[i] = x[i]; /* +-0 stays +-0 */
    }
    return 0;
}
