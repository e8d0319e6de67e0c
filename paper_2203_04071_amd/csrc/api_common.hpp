// Shared by the translation units of the C ABI: error reporting, device allocations, the table handle.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/adapt_mi355.h"
#include "elementwise.hpp"

namespace adapt_api {

extern thread_local char g_err[512];        // defined in api_core.hip

inline int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(expr)                                                                                  \
    do {                                                                                               \
        hipError_t e_ = (expr);                                                                        \
        if (e_ != hipSuccess)                                                                          \
            return fail(e_ == hipErrorOutOfMemory ? ADAPT_ERR_OUT_OF_MEMORY : ADAPT_ERR_HIP, "%s: %s", \
                        #expr, hipGetErrorString(e_));                                                 \
    } while (0)

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline unsigned ew_grid(size_t work_items) {
    size_t g = (work_items + adapt::EW_THREADS - 1) / adapt::EW_THREADS;
    if (g < 1) g = 1;
    if (g > 256 * 16) g = 256 * 16;   // grid-stride loops: 16 blocks per compute unit is plenty
    return (unsigned)g;
}

// Debugging aid: with ADAPT_POISON_ALLOC set in the environment every device allocation of the library is filled with
// 0xA5 bytes before use, so that code which relies on fresh memory being zero shows up in the tests.
inline bool poison_on() {
    static const bool v = getenv("ADAPT_POISON_ALLOC") != nullptr;
    return v;
}
inline hipError_t dbg_poison(void *p, size_t bytes, hipStream_t s) {
    if (!poison_on() || !p || bytes < 4) return hipSuccess;
    adapt::fill_u32_kernel<<<4096, 256, 0, s>>>(static_cast<uint32_t *>(p), 0xA5A5A5A5u, bytes / 4);
    return hipGetLastError();
}
inline hipError_t dbg_malloc_async(void **p, size_t bytes, hipStream_t s) {
    hipError_t e = hipMallocAsync(p, bytes, s);
    if (e == hipSuccess) e = dbg_poison(*p, bytes, s);
    return e;
}
inline hipError_t dbg_malloc(void **p, size_t bytes) {
    hipError_t e = hipMalloc(p, bytes);
    if (e == hipSuccess && poison_on()) {
        e = dbg_poison(*p, bytes, nullptr);
        if (e == hipSuccess) e = hipDeviceSynchronize();
    }
    return e;
}

// Scratch memory of one call.  Plain entry points take it from the stream-ordered allocator and give it back in stream
// order; a packed-weights handle keeps one grow-only buffer, so that its calls allocate nothing once they have run at
// their largest size (they can then be recorded into a HIP graph).
struct Workspace {
    void *ptr = nullptr;
    size_t bytes = 0;
};

inline int ws_get(Workspace *cache, size_t bytes, hipStream_t s, void **out) {
    if (!cache) {
        HIP_TRY(dbg_malloc_async(out, bytes, s));
        return ADAPT_OK;
    }
    if (cache->bytes < bytes) {
        if (cache->ptr) HIP_TRY(hipFree(cache->ptr));       // waits for the device: no earlier call still uses it
        cache->ptr = nullptr;
        cache->bytes = 0;
        HIP_TRY(dbg_malloc(&cache->ptr, bytes));
        cache->bytes = bytes;
    }
    *out = cache->ptr;
    return ADAPT_OK;
}

inline int ws_put(Workspace *cache, void *p, hipStream_t s, int rc) {
    if (cache || !p) return rc;
    hipError_t fe = hipFreeAsync(p, s);
    if (rc == ADAPT_OK && fe != hipSuccess) rc = fail(ADAPT_ERR_HIP, "hipFreeAsync: %s", hipGetErrorString(fe));
    return rc;
}

// compute units of the current device (asked once per device; 256 when there is no device to ask)
inline int device_cus() {
    static std::atomic<int> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int cu = cached[dev].load(std::memory_order_relaxed);
    if (cu > 0) return cu;
    if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu <= 0) return 256;
    cached[dev].store(cu, std::memory_order_relaxed);
    return cu;
}

inline adapt::FastDiv fast_div(uint32_t d) {
    int l = 0;
    while ((1ull << l) < d) ++l;
    adapt::FastDiv f;
    f.k = 31 + l;
    f.M = (uint32_t)((1ull << f.k) / d + 1);
    f.d = d;
    return f;
}

}  // namespace adapt_api

struct adapt_lut {
    int bits;
    int storage;            // 0: one signed 16-bit image; 1: low (unsigned) + high (signed) images
    int32_t min_entry, max_entry;
    int device;
    int rs;                 // entries per image row = 2^b + 2
    int img_bytes;          // per image, multiple of 16
    uint16_t *img_dev[2];   // [0] = only / low half, [1] = high half
    uint16_t *lut16_dev[2]; // same halves, plain [a & mask][w & mask] order (source of the derived line tables)
};
