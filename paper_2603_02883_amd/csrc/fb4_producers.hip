// C ABI of the FB4 quantizer library, the producer-fused entry points (App. E.2): the quantizer behind a
// LayerNorm and behind a GeLU.  Declarations and contracts are in include/fb4.h.
#include <cstring>

#include "fb4_common.hpp"
#include "fb4_gelu.hpp"
#include "fb4_layernorm.hpp"

namespace fb4 {

// The two GeLU tables, evaluated once per process (about 100,000 calls of erfc / exp).
const uint16_t* gelu_tables()
{
    static const uint16_t* tables = []() -> const uint16_t* {
        uint16_t* t = static_cast<uint16_t*>(std::malloc(2 * kGeluTableBytes));
        if (!t) return nullptr;
        build_gelu_table(false, t);
        build_gelu_table(true, t + kGeluTableBytes / 2);
        return t;
    }();
    return tables;
}

size_t gelu_tables_bytes() { return 2 * kGeluTableBytes; }

}  // namespace fb4

namespace {

using namespace fb4;

// The optional SeDA arguments of the producer-fused calls: all absent, or all there and small enough.
int check_fused_seda(const int32_t* token_group, const uint8_t* sub, int n_groups, int64_t rows)
{
    if (!token_group && !sub) return n_groups == 0 ? FB4_OK : FB4_ERR_INVALID_ARG;
    if (n_groups < 1) return FB4_ERR_INVALID_ARG;
    if (rows > 0 && (!token_group || !sub)) return FB4_ERR_INVALID_ARG;
    if (!aligned(token_group, 4) || (uint32_t)n_groups > kMaxFusedProducerGroups) return FB4_ERR_UNSUPPORTED;
    return FB4_OK;
}

}  // namespace

extern "C" {

int fb4_layernorm_quantize(const fb4_luts* luts, const fb4_opts* opts, const void* x, int64_t rows, int64_t cols,
                           int64_t row_stride, const float* gamma, const float* beta, float eps,
                           const int32_t* token_group, const uint8_t* sub_formatbooks, int n_groups, uint8_t* codes,
                           uint16_t* meta, void* y_out, void* stream)
{
    int rc = check_tensor(luts, opts, x, rows, cols, row_stride, codes, meta);
    if (rc != FB4_OK) return rc;
    if (!(eps >= 0.0f) || eps > 3.0e38f) return FB4_ERR_INVALID_ARG;
    if ((rc = check_fused_seda(token_group, sub_formatbooks, n_groups, rows)) != FB4_OK) return rc;
    if (opts->selector != FB4_SEL_LUT || opts->num_groups == 32) return FB4_ERR_UNSUPPORTED;
    if (cols % 32) return FB4_ERR_UNSUPPORTED;
    if (rows == 0 || cols == 0) return FB4_OK;
    const int64_t nb = cols / 32;
    if (nb > 64 * kLnMaxChunksPerLane || !aligned(codes, 16) || (gamma && !aligned(gamma, 4)) || (beta && !aligned(beta, 4)) ||
        (y_out && !aligned(y_out, 16)) || (opts->block == 16 && !aligned(meta, 4)))
        return FB4_ERR_UNSUPPORTED;
    if ((uint64_t)rows * (uint64_t)nb >= 0x7F000000ull) return FB4_ERR_UNSUPPORTED;
    if ((rc = check_device(luts)) != FB4_OK) return rc;
    // Chunks per lane B and rows per bundle: the fullest wavefront among B <= 4, the fewest chunks among equals;
    // rows longer than 8192 need 5 or 6.
    int B = 0;
    uint32_t rw = 0;
    double best = 0.0;
    for (int b = 1; b <= 4; ++b) {
        if (nb > 64 * b) continue;
        const uint32_t r = (uint32_t)(64 * b / nb);
        const double fill = (double)(r * nb) / (64.0 * b) - (b == 4 ? 0.05 : 0.0);
        if (fill > best + 1e-9) { best = fill; B = b; rw = r; }
    }
    if (B == 0) { B = (int)((nb + 63) / 64); rw = 1; }
    if (rw > (uint32_t)rows) rw = (uint32_t)rows;
    const uint32_t n_bundles = (uint32_t)((rows + rw - 1) / rw);
    const int kLnWaves = ln_threads(B, opts->num_groups) / 64;
    long long g = ((long long)n_bundles + kLnWaves - 1) / kLnWaves;
    if (g > luts->n_cu) g = luts->n_cu;
    const unsigned groups = (unsigned)g;
    LayerNormParams p = {};
    p.rows = (uint32_t)rows;
    p.cols = (uint32_t)cols;
    p.n_blocks = (uint32_t)(rows * nb);
    p.eps = eps;
    p.codes = codes;
    p.meta = meta;
    p.token_group = token_group;
    p.sub = sub_formatbooks;
    p.n_groups = (uint32_t)n_groups;
    p.n_dialects = (uint32_t)luts->n_dialects;
    p.y_out = static_cast<uint16_t*>(y_out);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool ts = (opts->flags & FB4_FLAG_TWO_STAGE) != 0;
    const bool seda = token_group != nullptr;
#define FB4_LN_ARGS luts->dev_blob, static_cast<const uint16_t*>(x), n_bundles, rw, (uint32_t)nb, groups, (long long)row_stride, gamma, beta, p
#define FB4_LN_LAUNCH(b, blk, g, t, sd, wy) hipLaunchKernelGGL((layernorm_quantize_kernel<b, blk, g, t, sd, wy>), dim3(groups), dim3(ln_threads(b, g)), 0, s, FB4_LN_ARGS)
#define FB4_LN_SHAPE(b, blk, g)                                \
    if (seda) {                                                \
        if (ts) FB4_LN_LAUNCH(b, blk, g, true, true, false);   \
        else FB4_LN_LAUNCH(b, blk, g, false, true, false);     \
    } else {                                                   \
        if (ts) FB4_LN_LAUNCH(b, blk, g, true, false, false);  \
        else FB4_LN_LAUNCH(b, blk, g, false, false, false);    \
    }
#define FB4_LN_CASE(b)                                                  \
    case b:                                                             \
        if (y_out) FB4_LN_LAUNCH(b, 32, 8, false, false, true);         \
        if (opts->block == 32) {                                        \
            if (opts->num_groups == 8) { FB4_LN_SHAPE(b, 32, 8) }       \
            else { FB4_LN_SHAPE(b, 32, 16) }                            \
        } else {                                                        \
            if (opts->num_groups == 8) { FB4_LN_SHAPE(b, 16, 8) }       \
            else { FB4_LN_SHAPE(b, 16, 16) }                            \
        }                                                               \
        break;
    switch (B) {
        FB4_LN_CASE(1) FB4_LN_CASE(2) FB4_LN_CASE(3) FB4_LN_CASE(4) FB4_LN_CASE(5) FB4_LN_CASE(6)
        default: return FB4_ERR_UNSUPPORTED;
    }
#undef FB4_LN_SHAPE
#undef FB4_LN_CASE
#undef FB4_LN_LAUNCH
#undef FB4_LN_ARGS
    return hipGetLastError() == hipSuccess ? FB4_OK : FB4_ERR_HIP;
}

int fb4_gelu_quantize(const fb4_luts* luts, const fb4_opts* opts, const void* x, int64_t rows, int64_t cols,
                      int64_t row_stride, int approximate, const int32_t* token_group, const uint8_t* sub_formatbooks,
                      int n_groups, uint8_t* codes, uint16_t* meta, void* stream)
{
    int rc = check_tensor(luts, opts, x, rows, cols, row_stride, codes, meta);
    if (rc != FB4_OK) return rc;
    if (approximate != 0 && approximate != 1) return FB4_ERR_INVALID_ARG;
    if ((rc = check_fused_seda(token_group, sub_formatbooks, n_groups, rows)) != FB4_OK) return rc;
    if (opts->selector != FB4_SEL_LUT || opts->num_groups == 32) return FB4_ERR_UNSUPPORTED;
    if (cols % 32) return FB4_ERR_UNSUPPORTED;
    if (rows == 0 || cols == 0) return FB4_OK;
    if (!aligned(codes, 16) || (opts->block == 16 && !aligned(meta, 4))) return FB4_ERR_UNSUPPORTED;
    const uint64_t nb = (uint64_t)cols / 32;
    const uint64_t n_blocks = (uint64_t)rows * nb;
    if (n_blocks >= 0x7F000000ull) return FB4_ERR_UNSUPPORTED;
    if ((rc = check_device(luts)) != FB4_OK) return rc;
    const uint32_t n_tiles = (uint32_t)((n_blocks + 63) / 64);
    uint32_t l = 0;
    while ((1ull << l) < nb) ++l;
    const uint32_t div_shift = 31 + l;
    const uint32_t div_mul = (uint32_t)(((1ull << div_shift) + nb - 1) / nb);
    long long g = ((long long)n_tiles + kGeluThreads / 64 - 1) / (kGeluThreads / 64);
    if (g > luts->n_cu) g = luts->n_cu;
    const unsigned groups = (unsigned)g;
    GeluParams p = {codes, meta, token_group, sub_formatbooks, (uint32_t)n_groups, (uint32_t)luts->n_dialects};
    const bool seda = token_group != nullptr, ts = (opts->flags & FB4_FLAG_TWO_STAGE) != 0;
    const uint16_t* table = reinterpret_cast<const uint16_t*>(luts->dev_blob + kBlobBytes + (approximate ? kGeluTableBytes : 0));
    hipStream_t s = static_cast<hipStream_t>(stream);
#define FB4_GELU_ARGS luts->dev_blob, static_cast<const uint16_t*>(x), table, (uint32_t)n_blocks, n_tiles, div_mul, div_shift, (uint32_t)nb, groups, (long long)row_stride, p
#define FB4_GELU_SHAPE(blk, g)                                                                                                        \
    if (seda) {                                                                                                                       \
        if (ts) hipLaunchKernelGGL((gelu_quantize_kernel<blk, g, true, true>), dim3(groups), dim3(kGeluThreads), 0, s, FB4_GELU_ARGS);  \
        else hipLaunchKernelGGL((gelu_quantize_kernel<blk, g, false, true>), dim3(groups), dim3(kGeluThreads), 0, s, FB4_GELU_ARGS);    \
    } else {                                                                                                                          \
        if (ts) hipLaunchKernelGGL((gelu_quantize_kernel<blk, g, true, false>), dim3(groups), dim3(kGeluThreads), 0, s, FB4_GELU_ARGS); \
        else hipLaunchKernelGGL((gelu_quantize_kernel<blk, g, false, false>), dim3(groups), dim3(kGeluThreads), 0, s, FB4_GELU_ARGS);   \
    }
    if (opts->block == 32) {
        if (opts->num_groups == 8) { FB4_GELU_SHAPE(32, 8) } else { FB4_GELU_SHAPE(32, 16) }
    } else {
        if (opts->num_groups == 8) { FB4_GELU_SHAPE(16, 8) } else { FB4_GELU_SHAPE(16, 16) }
    }
#undef FB4_GELU_SHAPE
#undef FB4_GELU_ARGS
    return hipGetLastError() == hipSuccess ? FB4_OK : FB4_ERR_HIP;
}

int fb4_gelu_table_host(int approximate, uint16_t* table, size_t capacity, size_t* entries)
{
    if (entries) *entries = kGeluEntries;
    if (approximate != 0 && approximate != 1) return FB4_ERR_INVALID_ARG;
    if (!table || capacity < kGeluEntries) return FB4_ERR_INVALID_ARG;
    const uint16_t* t = gelu_tables();
    if (!t) return FB4_ERR_ALLOC;
    std::memcpy(table, t + (approximate ? kGeluTableBytes / 2 : 0), kGeluEntries * 2);
    return FB4_OK;
}

}  // extern "C"
