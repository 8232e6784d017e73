// C ABI of the FB4 quantizer library, first part: lookup-table handle management, the quantizing, decoding,
// repacking and profiling entry points (the producer-fused ones are in fb4_producers.hip, the attention-guided
// ones in fb4_attention.hip).  Declarations and the contract of
// every entry point are in include/fb4.h.
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <new>

#include "fb4_common.hpp"
#include "fb4_dequant_fast.hpp"
#include "fb4_fast.hpp"
#include "fb4_kernels.hpp"
#include "fb4_profile.hpp"
#include "fb4_repack.hpp"

namespace fb4 {
const uint16_t* gelu_tables();   // fb4_producers.hip
size_t gelu_tables_bytes();
}

namespace {

using namespace fb4;

int grid_for(const fb4_luts* l, long long n_tiles)
{
    long long groups = (n_tiles + kWavesPerGroup - 1) / kWavesPerGroup;
    long long cap = (long long)l->n_cu * 8;
    if (groups > cap) groups = cap;
    if (groups < 1) groups = 1;
    return (int)groups;
}

template <int SEL, int G, int MODE, int LPB>
void launch_ts(bool two_stage, int grid, hipStream_t s, const QuantParams& p)
{
    // (the leading arguments repeat fields of p: see the kernel)
    if (two_stage)
        hipLaunchKernelGGL((quantize_kernel<SEL, G, MODE, true, LPB>), dim3(grid), dim3(kThreads), 0, s, p.blob, p.x,
                           p.salient, p.n_tiles, p.tiles_per_row, grid, p.row_stride, p.cols, p);
    else
        hipLaunchKernelGGL((quantize_kernel<SEL, G, MODE, false, LPB>), dim3(grid), dim3(kThreads), 0, s, p.blob, p.x,
                           p.salient, p.n_tiles, p.tiles_per_row, grid, p.row_stride, p.cols, p);
}

template <int MODE>
int launch_quant(const fb4_opts* o, int grid, hipStream_t s, const QuantParams& p)
{
    const bool ts = (o->flags & FB4_FLAG_TWO_STAGE) != 0;
    if (o->block == 32) {
        if (o->selector == FB4_SEL_SSE) {
            launch_ts<kSelSse, 8, MODE, 4>(ts, grid, s, p);
        } else if (o->num_groups == 8) {
            launch_ts<kSelLut, 8, MODE, 4>(ts, grid, s, p);
        } else if (o->num_groups == 16) {
            launch_ts<kSelLut, 16, MODE, 4>(ts, grid, s, p);
        } else {
            launch_ts<kSelLut, 32, MODE, 4>(ts, grid, s, p);
        }
    } else {   // block 16: two lanes per block
        if (o->selector == FB4_SEL_SSE) {
            launch_ts<kSelSse, 8, MODE, 2>(ts, grid, s, p);
        } else if (o->num_groups == 8) {
            launch_ts<kSelLut, 8, MODE, 2>(ts, grid, s, p);
        } else {
            launch_ts<kSelLut, 16, MODE, 2>(ts, grid, s, p);
        }
    }
    return hipGetLastError() == hipSuccess ? FB4_OK : FB4_ERR_HIP;
}

// Persistent workgroups, one per compute unit: measured 24.4 us against 26.0 us with two on the 16384x3072
// workload with 8 wavefronts each (SeDA: 25.7 against 27.2; 4, 12 or 16 wavefronts are slower too), and the
// kernels are free to use up to 256 vector registers per lane.  The exhaustive selector without candidate
// restrictions runs 12 wavefronts (37.7 against 39.1 us).
// kSedaToo = false: the variants with SeDA lists are not instantiated (`seda` must be false).
template <int kBlock, int G, bool kFlat, int kMode, int kThreads = kFastThreads, bool kSedaToo = true>
void launch_fast_variant(bool ts, bool seda, int n_cu, hipStream_t s, const FastParams& f)
{
    constexpr int kWaves = kThreads / 64;
    long long g = ((long long)f.n_tiles + kWaves - 1) / kWaves;
    if (g > n_cu) g = n_cu;
    const unsigned groups = (unsigned)g;
    // (the leading arguments repeat fields of f: see the kernel)
#define FB4_FAST_ARGS f.blob, f.x, f.n_blocks, f.n_tiles, f.div_mul, f.div_shift, f.nb, groups, f.row_stride, f.salient, f
    if (seda) {
        if constexpr (kSedaToo) {
            if (ts) hipLaunchKernelGGL((quantize_lut_kernel<kBlock, G, kFlat, true, true, kMode, kThreads>), dim3(groups), dim3(kThreads), 0, s, FB4_FAST_ARGS);
            else hipLaunchKernelGGL((quantize_lut_kernel<kBlock, G, kFlat, false, true, kMode, kThreads>), dim3(groups), dim3(kThreads), 0, s, FB4_FAST_ARGS);
        }
    } else {
        if (ts) hipLaunchKernelGGL((quantize_lut_kernel<kBlock, G, kFlat, true, false, kMode, kThreads>), dim3(groups), dim3(kThreads), 0, s, FB4_FAST_ARGS);
        else hipLaunchKernelGGL((quantize_lut_kernel<kBlock, G, kFlat, false, false, kMode, kThreads>), dim3(groups), dim3(kThreads), 0, s, FB4_FAST_ARGS);
    }
#undef FB4_FAST_ARGS
}

// Second-plane outputs of the fused quantize + decompose call.
struct FusedPlane {
    const int32_t* salient;
    int64_t n_sal;
    uint8_t* codes2;
    uint16_t* meta2;
};

// The streaming kernel serves both selectors (the online one with any supported block size and group count),
// with or without the two-stage filter and SeDA lists, when rows are whole 32-element chunks and the outputs
// are aligned for its wide stores; with `fused` it also writes the second plane of the salient rows (online
// selector: 8 groups; row and list counts that fit its LDS).  Returns false if the request is not one it
// serves.
bool launch_fast(const fb4_luts* luts, const fb4_opts* opts, const QuantParams& p, int64_t cols,
                 const int32_t* token_group, const uint8_t* sub, int n_groups, const FusedPlane* fused,
                 hipStream_t s, int* rc)
{
    if ((cols % 32) || !aligned(p.codes, 16)) return false;
    const bool sse = opts->selector == FB4_SEL_SSE;
    if (opts->block == 16 && !aligned(p.meta, 4)) return false;
    const uint64_t nb = (uint64_t)cols / 32;
    const uint64_t n_blocks = (uint64_t)p.rows * nb;
    if (n_blocks >= 0x7FFFFF00ull) return false;
    if (token_group && (uint32_t)n_groups > kMaxFastGroups) return false;
    if (fused && ((!sse && opts->num_groups != 8) || p.rows > (long long)kMaxFusedRows || !aligned(fused->codes2, 16)))
        return false;
    FastParams f = {};
    f.x = p.x;
    f.row_stride = p.row_stride;
    f.nb = (uint32_t)nb;
    f.n_blocks = (uint32_t)n_blocks;
    f.n_tiles = (uint32_t)((n_blocks + 63) / 64);
    uint32_t l = 0;
    while ((1ull << l) < nb) ++l;
    f.div_shift = 31 + l;
    f.div_mul = (uint32_t)(((1ull << f.div_shift) + nb - 1) / nb);
    f.codes = p.codes;
    f.meta = p.meta;
    f.blob = luts->dev_blob;
    f.token_group = token_group;
    f.sub = sub;
    f.n_groups = (uint32_t)n_groups;
    f.n_dialects = (uint32_t)luts->n_dialects;
    if (fused) {
        f.salient = fused->salient;
        f.n_sal = (uint32_t)fused->n_sal;
        f.rows = (uint32_t)p.rows;
        f.codes2 = fused->codes2;
        f.meta2 = fused->meta2;
    }
    const int ng = luts->n_cu;   // workgroups at most: one per compute unit
    const bool flat = p.row_stride == cols;
    const bool ts = (opts->flags & FB4_FLAG_TWO_STAGE) != 0;
    const bool seda = token_group != nullptr;
    if (sse) {
        // the exhaustive selector: group count 0 in the kernel's template
        if (fused) {
            if (opts->block == 32) launch_fast_variant<32, 0, false, 1>(ts, seda, ng, s, f);
            else launch_fast_variant<16, 0, false, 1>(ts, seda, ng, s, f);
        } else {
            // (matrix-core form) 12 wavefronts per workgroup; 8 with the SeDA rows, which leave LDS for no more
            // histograms, and with the two-stage filter, which would spill at the 168 registers of 12
            if (seda || ts) {
                if (opts->block == 32) launch_fast_variant<32, 0, false, 0>(ts, seda, ng, s, f);
                else launch_fast_variant<16, 0, false, 0>(ts, seda, ng, s, f);
            } else {
                if (opts->block == 32) launch_fast_variant<32, 0, false, 0, 768, false>(false, false, ng, s, f);
                else launch_fast_variant<16, 0, false, 0, 768, false>(false, false, ng, s, f);
            }
        }
    } else if (fused) {
        if (opts->block == 32) {
            if (flat) launch_fast_variant<32, 8, true, 1>(ts, seda, ng, s, f);
            else launch_fast_variant<32, 8, false, 1>(ts, seda, ng, s, f);
        } else {
            launch_fast_variant<16, 8, false, 1>(ts, seda, ng, s, f);
        }
    } else if (opts->block == 32) {
        if (opts->num_groups == 8) {
            if (flat) launch_fast_variant<32, 8, true, 0>(ts, seda, ng, s, f);
            else launch_fast_variant<32, 8, false, 0>(ts, seda, ng, s, f);
        } else if (opts->num_groups == 16) {
            launch_fast_variant<32, 16, false, 0>(ts, seda, ng, s, f);
        } else {
            launch_fast_variant<32, 32, false, 0>(ts, seda, ng, s, f);
        }
    } else {
        if (opts->num_groups == 8) launch_fast_variant<16, 8, false, 0>(ts, seda, ng, s, f);
        else launch_fast_variant<16, 16, false, 0>(ts, seda, ng, s, f);
    }
    *rc = hipGetLastError() == hipSuccess ? FB4_OK : FB4_ERR_HIP;
    return true;
}

// The second plane of listed rows from x and a first plane in memory (fb4_decompose) in the streaming kernel:
// the default online selector (8 groups) and the exhaustive one, when rows are whole 32-element chunks and
// the planes are aligned for its wide loads and stores.  p.codes / p.meta are the second plane.
bool launch_fast_second_plane(const fb4_luts* luts, const fb4_opts* opts, const QuantParams& p, int64_t cols,
                              int64_t n_sal, hipStream_t s, int* rc)
{
    const bool sse = opts->selector == FB4_SEL_SSE;
    if ((cols % 32) || !aligned(p.codes, 16) || !aligned(p.codes1, 16) || (!sse && opts->num_groups != 8)) return false;
    if (opts->block == 16 && (!aligned(p.meta, 4) || !aligned(p.meta1, 4))) return false;
    const uint64_t nb = (uint64_t)cols / 32;
    const uint64_t n_blocks = (uint64_t)n_sal * nb;
    if (n_blocks >= 0x7FFFFF00ull || p.rows > 0x7FFFFFFFll) return false;
    if (p.token_group && (uint32_t)p.n_groups > kMaxFastGroups) return false;
    FastParams f = {};
    f.x = p.x;
    f.row_stride = p.row_stride;
    f.nb = (uint32_t)nb;
    f.n_blocks = (uint32_t)n_blocks;
    f.n_tiles = (uint32_t)((n_blocks + 63) / 64);
    uint32_t l = 0;
    while ((1ull << l) < nb) ++l;
    f.div_shift = 31 + l;
    f.div_mul = (uint32_t)(((1ull << f.div_shift) + nb - 1) / nb);
    f.codes = p.codes;
    f.meta = p.meta;
    f.blob = luts->dev_blob;
    f.token_group = p.token_group;
    f.sub = p.sub;
    f.n_groups = (uint32_t)p.n_groups;
    f.n_dialects = (uint32_t)luts->n_dialects;
    f.salient = p.salient;
    f.n_sal = (uint32_t)n_sal;
    f.rows = (uint32_t)p.rows;
    f.codes1 = p.codes1;
    f.meta1 = p.meta1;
    const bool ts = (opts->flags & FB4_FLAG_TWO_STAGE) != 0;
    const bool seda = p.token_group != nullptr;
    if (sse) {
        if (opts->block == 32) launch_fast_variant<32, 0, false, 2>(ts, seda, luts->n_cu, s, f);
        else launch_fast_variant<16, 0, false, 2>(ts, seda, luts->n_cu, s, f);
    } else {
        if (opts->block == 32) launch_fast_variant<32, 8, false, 2>(ts, seda, luts->n_cu, s, f);
        else launch_fast_variant<16, 8, false, 2>(ts, seda, luts->n_cu, s, f);
    }
    *rc = hipGetLastError() == hipSuccess ? FB4_OK : FB4_ERR_HIP;
    return true;
}

// Tiling of `out_rows` rows of `cols` columns; false if it does not fit 32-bit tile indices.
bool tiling(int64_t out_rows, int64_t cols, int block, int* nb, int* tpr, int* n_tiles)
{
    int64_t b = cols / block;
    int64_t t = (cols + kTileElems - 1) / kTileElems;
    // the kernels step a 32-bit tile index by the grid size: leave room for that last step
    if (b > 0x7FFFFFFF || t * out_rows > 0x7FF00000LL) return false;
    *nb = (int)b;
    *tpr = (int)t;
    *n_tiles = (int)(t * out_rows);
    return true;
}

}  // namespace

extern "C" {

int fb4_version(void) { return 100; }

const char* fb4_strerror(int code)
{
    switch (code) {
    case FB4_OK: return "ok";
    case FB4_ERR_INVALID_ARG: return "invalid argument";
    case FB4_ERR_UNSUPPORTED: return "unsupported shape, alignment or option";
    case FB4_ERR_ALLOC: return "allocation failed";
    case FB4_ERR_HIP: return "HIP runtime error";
    default: return "unknown error code";
    }
}

size_t fb4_workspace_bytes(void) { return 0; }

int fb4_build_luts_host(const uint8_t* formatbook, int n_dialects, void* blob, size_t capacity, size_t* size)
{
    if (!formatbook_ok(formatbook, n_dialects)) return FB4_ERR_INVALID_ARG;
    if (size) *size = kBlobBytes;
    if (!blob) return size ? FB4_OK : FB4_ERR_INVALID_ARG;
    if (capacity < kBlobBytes) return FB4_ERR_INVALID_ARG;
    build_blob(formatbook, n_dialects, static_cast<uint8_t*>(blob));
    return FB4_OK;
}

int fb4_build_luts(const uint8_t* formatbook, int n_dialects, fb4_luts** out)
{
    if (!out) return FB4_ERR_INVALID_ARG;
    *out = nullptr;
    if (!formatbook_ok(formatbook, n_dialects)) return FB4_ERR_INVALID_ARG;
    fb4_luts* l = new (std::nothrow) fb4_luts;
    if (!l) return FB4_ERR_ALLOC;
    build_blob(formatbook, n_dialects, l->host_blob);
    l->n_dialects = n_dialects;
    l->dev_blob = nullptr;
    hipDeviceProp_t prop;
    if (hipGetDevice(&l->device) != hipSuccess || hipGetDeviceProperties(&prop, l->device) != hipSuccess) {
        delete l;
        return FB4_ERR_HIP;
    }
    l->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    // one allocation: the table blob, then the two GeLU tables (exact form, tanh form) of fb4_gelu_quantize
    if (hipMalloc(reinterpret_cast<void**>(&l->dev_blob), kBlobBytes + gelu_tables_bytes()) != hipSuccess) {
        (void)hipGetLastError();
        delete l;
        return FB4_ERR_ALLOC;
    }
    const uint16_t* gelu = gelu_tables();
    if (!gelu) {
        (void)hipFree(l->dev_blob);
        delete l;
        return FB4_ERR_ALLOC;
    }
    if (hipMemcpy(l->dev_blob, l->host_blob, kBlobBytes, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(l->dev_blob + kBlobBytes, gelu, gelu_tables_bytes(), hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFree(l->dev_blob);
        delete l;
        return FB4_ERR_HIP;
    }
    *out = l;
    return FB4_OK;
}

void fb4_free_luts(fb4_luts* luts)
{
    if (!luts) return;
    if (luts->dev_blob) (void)hipFree(luts->dev_blob);
    delete luts;
}

int fb4_quantize(const fb4_luts* luts, const fb4_opts* opts, const void* x, int64_t rows, int64_t cols,
                 int64_t row_stride, uint8_t* codes, uint16_t* meta, void* stream)
{
    int rc = check_tensor(luts, opts, x, rows, cols, row_stride, codes, meta);
    if (rc != FB4_OK || rows == 0 || cols == 0) return rc;
    if ((rc = check_device(luts)) != FB4_OK) return rc;
    QuantParams p = {};
    if (!tiling(rows, cols, opts->block, &p.nb, &p.tiles_per_row, &p.n_tiles)) return FB4_ERR_UNSUPPORTED;
    p.x = static_cast<const uint16_t*>(x);
    p.row_stride = row_stride;
    p.rows = rows;
    p.cols = cols;
    p.codes = codes;
    p.meta = meta;
    p.blob = luts->dev_blob;
    p.n_dialects = luts->n_dialects;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (launch_fast(luts, opts, p, cols, nullptr, nullptr, 0, nullptr, s, &rc)) return rc;
    return launch_quant<kPlain>(opts, grid_for(luts, p.n_tiles), s, p);
}

int fb4_quantize_seda(const fb4_luts* luts, const fb4_opts* opts, const void* x, int64_t rows, int64_t cols,
                      int64_t row_stride, const int32_t* token_group, const uint8_t* sub_formatbooks,
                      int n_groups, uint8_t* codes, uint16_t* meta, void* stream)
{
    int rc = check_tensor(luts, opts, x, rows, cols, row_stride, codes, meta);
    if (rc != FB4_OK) return rc;
    if (n_groups < 1) return FB4_ERR_INVALID_ARG;
    if (rows == 0 || cols == 0) return FB4_OK;
    if (!token_group || !sub_formatbooks) return FB4_ERR_INVALID_ARG;
    if (!aligned(token_group, 4)) return FB4_ERR_UNSUPPORTED;
    if ((rc = check_device(luts)) != FB4_OK) return rc;
    QuantParams p = {};
    if (!tiling(rows, cols, opts->block, &p.nb, &p.tiles_per_row, &p.n_tiles)) return FB4_ERR_UNSUPPORTED;
    p.x = static_cast<const uint16_t*>(x);
    p.row_stride = row_stride;
    p.rows = rows;
    p.cols = cols;
    p.codes = codes;
    p.meta = meta;
    p.token_group = token_group;
    p.sub = sub_formatbooks;
    p.n_groups = n_groups;
    p.blob = luts->dev_blob;
    p.n_dialects = luts->n_dialects;
    if (launch_fast(luts, opts, p, cols, token_group, sub_formatbooks, n_groups, nullptr,
                    static_cast<hipStream_t>(stream), &rc))
        return rc;
    return launch_quant<kSeda>(opts, grid_for(luts, p.n_tiles), static_cast<hipStream_t>(stream), p);
}

int fb4_decompose(const fb4_luts* luts, const fb4_opts* opts, const void* x, int64_t rows, int64_t cols,
                  int64_t row_stride, const uint8_t* codes1, const uint16_t* meta1, const int32_t* salient_rows,
                  int64_t n_sal, const int32_t* token_group, const uint8_t* sub_formatbooks, int n_groups,
                  uint8_t* codes2, uint16_t* meta2, void* stream)
{
    if (n_sal < 0) return FB4_ERR_INVALID_ARG;
    int rc = check_tensor(luts, opts, x, rows, cols, row_stride, n_sal ? (const void*)codes2 : (const void*)x,
                          n_sal ? (const void*)meta2 : (const void*)x);
    if (rc != FB4_OK) return rc;
    const bool seda = token_group || sub_formatbooks || n_groups;
    if (seda && (!token_group || !sub_formatbooks || n_groups < 1)) return FB4_ERR_INVALID_ARG;
    if (rows == 0 || cols == 0 || n_sal == 0) return FB4_OK;
    if (!codes1 || !meta1 || !salient_rows) return FB4_ERR_INVALID_ARG;
    if (!aligned(codes1, 4) || !aligned(meta1, 2) || !aligned(salient_rows, 4)) return FB4_ERR_UNSUPPORTED;
    if (n_sal > rows) return FB4_ERR_INVALID_ARG;   // ascending and unique implies n_sal <= rows
    if ((rc = check_device(luts)) != FB4_OK) return rc;
    QuantParams p = {};
    if (!tiling(n_sal, cols, opts->block, &p.nb, &p.tiles_per_row, &p.n_tiles)) return FB4_ERR_UNSUPPORTED;
    p.x = static_cast<const uint16_t*>(x);
    p.row_stride = row_stride;
    p.rows = rows;
    p.cols = cols;
    p.codes = codes2;
    p.meta = meta2;
    p.token_group = token_group;
    p.sub = sub_formatbooks;
    p.n_groups = n_groups;
    p.codes1 = codes1;
    p.meta1 = meta1;
    p.salient = salient_rows;
    p.blob = luts->dev_blob;
    p.n_dialects = luts->n_dialects;
    if (launch_fast_second_plane(luts, opts, p, cols, n_sal, static_cast<hipStream_t>(stream), &rc)) return rc;
    return launch_quant<kDecomp>(opts, grid_for(luts, p.n_tiles), static_cast<hipStream_t>(stream), p);
}

int fb4_quantize_decompose(const fb4_luts* luts, const fb4_opts* opts, const void* x, int64_t rows, int64_t cols,
                           int64_t row_stride, const int32_t* token_group, const uint8_t* sub_formatbooks,
                           int n_groups, const int32_t* salient_rows, int64_t n_sal, uint8_t* codes1,
                           uint16_t* meta1, uint8_t* codes2, uint16_t* meta2, void* stream)
{
    if (n_sal < 0) return FB4_ERR_INVALID_ARG;
    int rc = check_tensor(luts, opts, x, rows, cols, row_stride, codes1, meta1);
    if (rc != FB4_OK) return rc;
    const bool seda = token_group || sub_formatbooks || n_groups;
    if (seda && (!token_group || !sub_formatbooks || n_groups < 1)) return FB4_ERR_INVALID_ARG;
    if (n_sal > rows) return FB4_ERR_INVALID_ARG;
    if (rows == 0 || cols == 0) return FB4_OK;
    if (n_sal > 0 && (!salient_rows || !codes2 || !meta2)) return FB4_ERR_INVALID_ARG;
    if (seda && !aligned(token_group, 4)) return FB4_ERR_UNSUPPORTED;
    if (n_sal > 0 && (!aligned(salient_rows, 4) || !aligned(codes2, 4) || !aligned(meta2, 2))) return FB4_ERR_UNSUPPORTED;
    if ((rc = check_device(luts)) != FB4_OK) return rc;
    if (n_sal > 0) {
        // one pass: the second plane is formed from the registers that hold the tile
        QuantParams p = {};
        if (!tiling(rows, cols, opts->block, &p.nb, &p.tiles_per_row, &p.n_tiles)) return FB4_ERR_UNSUPPORTED;
        p.x = static_cast<const uint16_t*>(x);
        p.row_stride = row_stride;
        p.rows = rows;
        p.cols = cols;
        p.codes = codes1;
        p.meta = meta1;
        const FusedPlane fp = {salient_rows, n_sal, codes2, meta2};
        if (launch_fast(luts, opts, p, cols, token_group, sub_formatbooks, n_groups, &fp,
                        static_cast<hipStream_t>(stream), &rc))
            return rc;
    }
    // otherwise the two steps one after the other on the same stream
    rc = seda ? fb4_quantize_seda(luts, opts, x, rows, cols, row_stride, token_group, sub_formatbooks, n_groups,
                                  codes1, meta1, stream)
              : fb4_quantize(luts, opts, x, rows, cols, row_stride, codes1, meta1, stream);
    if (rc != FB4_OK || n_sal == 0) return rc;
    return fb4_decompose(luts, opts, x, rows, cols, row_stride, codes1, meta1, salient_rows, n_sal, token_group,
                         sub_formatbooks, n_groups, codes2, meta2, stream);
}

int fb4_dequantize(const fb4_luts* luts, const uint8_t* codes1, const uint16_t* meta1, int64_t rows, int64_t cols,
                   int block, const uint8_t* codes2, const uint16_t* meta2, const int32_t* salient_rows,
                   int64_t n_sal, void* out, int out_dtype, int64_t out_row_stride, void* stream)
{
    if (!luts) return FB4_ERR_INVALID_ARG;
    if (block != 32 && block != 16) return FB4_ERR_INVALID_ARG;
    if (out_dtype != FB4_DTYPE_BF16 && out_dtype != FB4_DTYPE_F32) return FB4_ERR_INVALID_ARG;
    if (rows < 0 || cols < 0 || n_sal < 0 || out_row_stride < cols) return FB4_ERR_INVALID_ARG;
    if (cols % block) return FB4_ERR_UNSUPPORTED;
    if (n_sal > 0 && (!codes2 || !meta2 || !salient_rows)) return FB4_ERR_INVALID_ARG;
    if (n_sal > rows) return FB4_ERR_INVALID_ARG;
    if (rows == 0 || cols == 0) return FB4_OK;
    if (!codes1 || !meta1 || !out) return FB4_ERR_INVALID_ARG;
    const size_t oal = out_dtype == FB4_DTYPE_BF16 ? 16 : 32;
    if (!aligned(out, oal) || (out_row_stride % 8) || !aligned(codes1, 4) || !aligned(meta1, 2))
        return FB4_ERR_UNSUPPORTED;
    if (n_sal > 0 && (!aligned(codes2, 4) || !aligned(meta2, 2) || !aligned(salient_rows, 4)))
        return FB4_ERR_UNSUPPORTED;

    if (int rc = check_device(luts)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    DequantParams p = {};
    if (!tiling(rows, cols, block, &p.nb, &p.tiles_per_row, &p.n_tiles)) return FB4_ERR_UNSUPPORTED;
    p.codes1 = codes1;
    p.meta1 = meta1;
    p.rows = rows;
    p.cols = cols;
    p.out = out;
    p.out_row_stride = out_row_stride;
    p.block_shift = block == 32 ? 5 : 4;
    p.blob = luts->dev_blob;
    int grid = grid_for(luts, p.n_tiles);
    const uint64_t nb32 = (uint64_t)cols / 32;          // 32-element chunks per row
    const uint64_t n_blocks = (uint64_t)rows * nb32;
    if ((cols % 32) == 0 && aligned(codes1, 16) && aligned(out, 16) && n_blocks < 0x3FFFFF00ull) {
        // plane 1 of every row: one lane per code word, pair table in LDS
        DeqFastParams f = {};
        f.codes = codes1;
        f.meta = meta1;
        f.meta_shift = block == 32 ? 2 : 1;
        f.out = out;
        f.out_row_stride = out_row_stride;
        f.nb = (uint32_t)nb32;
        f.n_blocks = (uint32_t)n_blocks;
        f.n_tiles = (uint32_t)((n_blocks + 63) / 64);
        uint32_t l = 0;
        while ((1ull << l) < nb32) ++l;
        f.div_shift = 31 + l;
        f.div_mul = (uint32_t)(((1ull << f.div_shift) + nb32 - 1) / nb32);
        f.blob = luts->dev_blob;
        long long groups = ((long long)f.n_tiles + kDeqWaves - 1) / kDeqWaves;
        const long long cap = (long long)luts->n_cu * 3;   // three workgroups (and their tables) per CU
        if (groups > cap) groups = cap;
        const bool flat = out_row_stride == cols;
        const dim3 dg((unsigned)groups), db(kDeqThreads);
        // (the leading arguments repeat fields of f: see the kernel)
#define FB4_DEQ_ARGS f.blob, f.codes, f.meta, f.n_blocks, f.meta_shift, dg.x, f
        if (n_sal > 0 && rows <= (int64_t)kMaxFusedRows) {
            // salient rows get both planes in the same pass
            f.codes2 = codes2;
            f.meta2 = meta2;
            f.salient = salient_rows;
            f.n_sal = (uint32_t)n_sal;
            f.rows = (uint32_t)rows;
            if (out_dtype == FB4_DTYPE_F32) {
                if (flat) hipLaunchKernelGGL((dequantize_fast_kernel<true, true, true>), dg, db, 0, s, FB4_DEQ_ARGS);
                else hipLaunchKernelGGL((dequantize_fast_kernel<false, true, true>), dg, db, 0, s, FB4_DEQ_ARGS);
            } else {
                if (flat) hipLaunchKernelGGL((dequantize_fast_kernel<true, false, true>), dg, db, 0, s, FB4_DEQ_ARGS);
                else hipLaunchKernelGGL((dequantize_fast_kernel<false, false, true>), dg, db, 0, s, FB4_DEQ_ARGS);
            }
            return hipGetLastError() == hipSuccess ? FB4_OK : FB4_ERR_HIP;
        }
        if (out_dtype == FB4_DTYPE_F32) {
            if (flat) hipLaunchKernelGGL((dequantize_fast_kernel<true, true>), dg, db, 0, s, FB4_DEQ_ARGS);
            else hipLaunchKernelGGL((dequantize_fast_kernel<false, true>), dg, db, 0, s, FB4_DEQ_ARGS);
        } else {
            if (flat) hipLaunchKernelGGL((dequantize_fast_kernel<true, false>), dg, db, 0, s, FB4_DEQ_ARGS);
            else hipLaunchKernelGGL((dequantize_fast_kernel<false, false>), dg, db, 0, s, FB4_DEQ_ARGS);
        }
#undef FB4_DEQ_ARGS
    } else if (out_dtype == FB4_DTYPE_F32) {
        hipLaunchKernelGGL((dequantize_kernel<false, true>), dim3(grid), dim3(kThreads), 0, s, p);
    } else {
        hipLaunchKernelGGL((dequantize_kernel<false, false>), dim3(grid), dim3(kThreads), 0, s, p);
    }
    if (hipGetLastError() != hipSuccess) return FB4_ERR_HIP;
    if (n_sal > 0) {
        // second pass, ordered after the first on the same stream: salient rows = plane 1 + plane 2
        DequantParams p2 = p;
        if (!tiling(n_sal, cols, block, &p2.nb, &p2.tiles_per_row, &p2.n_tiles)) return FB4_ERR_UNSUPPORTED;
        p2.codes2 = codes2;
        p2.meta2 = meta2;
        p2.salient = salient_rows;
        grid = grid_for(luts, p2.n_tiles);
        if (out_dtype == FB4_DTYPE_F32)
            hipLaunchKernelGGL((dequantize_kernel<true, true>), dim3(grid), dim3(kThreads), 0, s, p2);
        else
            hipLaunchKernelGGL((dequantize_kernel<true, false>), dim3(grid), dim3(kThreads), 0, s, p2);
        if (hipGetLastError() != hipSuccess) return FB4_ERR_HIP;
    }
    return FB4_OK;
}

int fb4_repack_mxfp8(const fb4_luts* luts, const uint8_t* codes, const uint16_t* meta, int64_t rows, int64_t cols,
                     int block, uint8_t* elems, int64_t elem_row_stride, uint8_t* scales, void* stream)
{
    if (!luts) return FB4_ERR_INVALID_ARG;
    if (block != 32 && block != 16) return FB4_ERR_INVALID_ARG;
    if (rows < 0 || cols < 0 || elem_row_stride < cols) return FB4_ERR_INVALID_ARG;
    if (cols % 32) return FB4_ERR_UNSUPPORTED;
    if (rows == 0 || cols == 0) return FB4_OK;
    if (!codes || !meta || !elems || !scales) return FB4_ERR_INVALID_ARG;
    if (!aligned(codes, 4) || !aligned(meta, 2) || !aligned(elems, 8) || (elem_row_stride % 8))
        return FB4_ERR_UNSUPPORTED;
    const uint64_t nb32 = (uint64_t)cols / 32;
    const uint64_t n_chunks = (uint64_t)rows * nb32;
    if (n_chunks >= 0x3FFFFF00ull) return FB4_ERR_UNSUPPORTED;
    if (int rc = check_device(luts)) return rc;
    RepackParams f = {};
    f.codes = codes;
    f.meta = meta;
    f.elems = elems;
    f.elem_row_stride = elem_row_stride;
    f.scales = scales;
    f.nb32 = (uint32_t)nb32;
    f.n_chunks = (uint32_t)n_chunks;
    uint32_t l = 0;
    while ((1ull << l) < nb32) ++l;
    f.div_shift = 31 + l;
    f.div_mul = (uint32_t)(((1ull << f.div_shift) + nb32 - 1) / nb32);
    f.blob = luts->dev_blob;
    long long groups = ((long long)n_chunks * 4 + kRepackThreads - 1) / kRepackThreads;
    const long long cap = (long long)luts->n_cu * 3;
    if (groups > cap) groups = cap;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool flat = elem_row_stride == cols;
    if (block == 16) {
        if (flat) hipLaunchKernelGGL((repack_mxfp8_kernel<true, true>), dim3((unsigned)groups), dim3(kRepackThreads), 0, s, f.blob, f.codes, f.meta, f.n_chunks, (uint32_t)groups, f);
        else hipLaunchKernelGGL((repack_mxfp8_kernel<false, true>), dim3((unsigned)groups), dim3(kRepackThreads), 0, s, f.blob, f.codes, f.meta, f.n_chunks, (uint32_t)groups, f);
    } else {
        if (flat) hipLaunchKernelGGL((repack_mxfp8_kernel<true, false>), dim3((unsigned)groups), dim3(kRepackThreads), 0, s, f.blob, f.codes, f.meta, f.n_chunks, (uint32_t)groups, f);
        else hipLaunchKernelGGL((repack_mxfp8_kernel<false, false>), dim3((unsigned)groups), dim3(kRepackThreads), 0, s, f.blob, f.codes, f.meta, f.n_chunks, (uint32_t)groups, f);
    }
    return hipGetLastError() == hipSuccess ? FB4_OK : FB4_ERR_HIP;
}

int fb4_seda_profile(const fb4_luts* luts, const uint16_t* meta, int64_t rows, int64_t blocks_per_row,
                     const int32_t* anchor_group, int n_groups, uint32_t* counts, uint8_t* sub_formatbooks,
                     void* stream)
{
    if (!luts || rows < 0 || blocks_per_row < 0 || n_groups < 1 || n_groups > (1 << 24)) return FB4_ERR_INVALID_ARG;
    if (!counts || !sub_formatbooks) return FB4_ERR_INVALID_ARG;
    if (rows > 0 && blocks_per_row > 0 && (!meta || !anchor_group)) return FB4_ERR_INVALID_ARG;
    if (!aligned(counts, 4) || (meta && !aligned(meta, 2)) || (anchor_group && !aligned(anchor_group, 4)))
        return FB4_ERR_UNSUPPORTED;
    if (int rc = check_device(luts)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint32_t n = (uint32_t)n_groups * 32u;
    // cleared by a kernel (not a memset node), so the call can be captured into a HIP graph
    hipLaunchKernelGGL(profile_clear_kernel, dim3((n + kProfileThreads - 1) / kProfileThreads), dim3(kProfileThreads),
                       0, s, counts, n);
    if (rows > 0 && blocks_per_row > 0) {
        long long groups = (rows + kProfileThreads / 64 - 1) / (kProfileThreads / 64);
        const long long cap = (long long)luts->n_cu * 8;
        if (groups > cap) groups = cap;
        hipLaunchKernelGGL(profile_count_kernel, dim3((unsigned)groups), dim3(kProfileThreads), 0, s, meta,
                           (long long)rows, (long long)blocks_per_row, anchor_group, n_groups, counts);
    }
    hipLaunchKernelGGL(profile_select_kernel, dim3(((unsigned)n_groups * 8u + kProfileThreads - 1) / kProfileThreads),
                       dim3(kProfileThreads), 0, s, counts, n_groups, luts->dev_blob, sub_formatbooks);
    return hipGetLastError() == hipSuccess ? FB4_OK : FB4_ERR_HIP;
}

}  // extern "C"
