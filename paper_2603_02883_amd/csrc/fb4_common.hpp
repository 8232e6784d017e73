// Shared by the translation units of the C ABI: the lookup-table handle and the argument checks that several
// entry points repeat.  Declarations and the contract of every entry point are in include/fb4.h.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdlib>

#include "../../include/fb4.h"
#include "fb4_tables.hpp"

struct fb4_luts {
    uint8_t host_blob[fb4::kBlobBytes];
    uint8_t* dev_blob;   // the table blob, then the two GeLU tables
    int n_dialects;
    int device;
    int n_cu;
};

namespace fb4 {

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// The tables live on the device the handle was built on: launching from another current device would hand
// the kernels a foreign pointer.
inline int check_device(const fb4_luts* l)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return FB4_ERR_HIP;
    }
    return dev == l->device ? FB4_OK : FB4_ERR_INVALID_ARG;
}

inline int check_opts(const fb4_opts* o)
{
    if (!o) return FB4_ERR_INVALID_ARG;
    if (o->selector != FB4_SEL_SSE && o->selector != FB4_SEL_LUT) return FB4_ERR_INVALID_ARG;
    if (o->flags & ~FB4_FLAG_TWO_STAGE) return FB4_ERR_INVALID_ARG;
    if (o->block != 32 && o->block != 16) return FB4_ERR_INVALID_ARG;
    if (o->selector == FB4_SEL_LUT &&
        ((o->num_groups != 8 && o->num_groups != 16 && o->num_groups != 32) || o->num_groups > o->block))
        return FB4_ERR_INVALID_ARG;
    return FB4_OK;
}

// Shared validation of the tensor arguments of the quantizing calls.
inline int check_tensor(const fb4_luts* l, const fb4_opts* o, const void* x, int64_t rows, int64_t cols,
                        int64_t row_stride, const void* codes, const void* meta)
{
    if (!l) return FB4_ERR_INVALID_ARG;
    int rc = check_opts(o);
    if (rc != FB4_OK) return rc;
    if (rows < 0 || cols < 0 || row_stride < cols) return FB4_ERR_INVALID_ARG;
    if (cols % o->block) return FB4_ERR_UNSUPPORTED;
    if (rows == 0 || cols == 0) return FB4_OK;
    if (!x || !codes || !meta) return FB4_ERR_INVALID_ARG;
    if (!aligned(x, 16) || (row_stride % 8) || !aligned(codes, 4) || !aligned(meta, 2)) return FB4_ERR_UNSUPPORTED;
    return FB4_OK;
}

}  // namespace fb4
