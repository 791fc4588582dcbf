// Shared host-side plumbing of libpserve: error reporting, object layouts, launch helpers.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>
#include <mutex>
#include <new>
#include <vector>
#include <algorithm>

#include "../../include/pserve.h"

namespace pserve {

void set_error(const char* fmt, ...);

#define PS_CHECK_HIP(expr)                                                              \
    do {                                                                                \
        hipError_t _e = (expr);                                                         \
        if (_e != hipSuccess) {                                                         \
            pserve::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(_e),    \
                              __FILE__, __LINE__);                                      \
            return PSERVE_EHIP;                                                         \
        }                                                                               \
    } while (0)

#define PS_REQUIRE(cond, ...)                                                           \
    do {                                                                                \
        if (!(cond)) {                                                                  \
            pserve::set_error(__VA_ARGS__);                                             \
            return PSERVE_EINVAL;                                                       \
        }                                                                               \
    } while (0)

#define PS_TRY(expr)                                                                    \
    do {                                                                                \
        int _s = (expr);                                                                \
        if (_s != PSERVE_OK) return _s;                                                 \
    } while (0)

// Raise a kernel's dynamic LDS limit once per process; safe when two host threads make their first launch together.
#define PS_SET_LDS_ONCE(fn, bytes)                                                      \
    do {                                                                                \
        static std::once_flag _once;                                                    \
        static hipError_t _err = hipSuccess;                                            \
        std::call_once(_once, [&] {                                                     \
            _err = hipFuncSetAttribute((const void*)(fn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)(bytes)); \
        });                                                                             \
        PS_CHECK_HIP(_err);                                                             \
    } while (0)

inline int check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("launch of %s failed: %s", what, hipGetErrorString(e));
        return PSERVE_EHIP;
    }
    return PSERVE_OK;
}

// Runs the body of an entry point; no exception may unwind across the C boundary (the bodies use the standard
// containers, whose allocations can throw).
template <class F>
inline int guarded(const char* who, F&& body) {
    try {
        return body();
    } catch (const std::bad_alloc&) {
        set_error("%s: out of host memory", who);
        return PSERVE_ENOMEM;
    } catch (...) {
        set_error("%s: unexpected exception", who);
        return PSERVE_EINVAL;
    }
}

inline size_t dtype_size(int dtype) { return dtype == PSERVE_BF16 ? 2 : 4; }
inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Owns a set of device allocations; frees them in the destructor.
struct DevicePool {
    std::vector<void*> ptrs;
    ~DevicePool() {
        for (void* p : ptrs) (void)hipFree(p);
    }
    int alloc(void** out, size_t bytes) {
        if (bytes == 0) bytes = 256;
        hipError_t e = hipMalloc(out, bytes);
        if (e != hipSuccess) {
            set_error("hipMalloc(%zu) failed: %s", bytes, hipGetErrorString(e));
            *out = nullptr;
            return PSERVE_ENOMEM;
        }
        ptrs.push_back(*out);
        return PSERVE_OK;
    }
    template <class T>
    int alloc_t(T** out, size_t count) { return alloc((void**)out, count * sizeof(T)); }
};

}  // namespace pserve

// ---- object layouts -------------------------------------------------------------------
struct pserve_plan_s {
    int32_t n = 0, R = 0, P = 0, ph = 0, pw = 0, ring = 0;
    int64_t T = 0;
    int32_t S = 0;                              // tokens per patch
    int32_t max_tokens_per_image = 0;
    int32_t text_len = 0, text_patches = 0;     // joint plans: text tokens / text patches per request
    std::vector<int32_t> h_tab[PSERVE_TAB_COUNT];
    int32_t* d_tab[PSERVE_TAB_COUNT] = {};
    int64_t tab_count[PSERVE_TAB_COUNT] = {};
    int32_t* d_sorted_hw = nullptr;             // [n][2] (H, W) of sorted slot s
    std::vector<int32_t> h_sorted_hw;
    float* mse_partial = nullptr;               // [P][16] scratch of pserve_patch_mse
    pserve::DevicePool pool;
};
