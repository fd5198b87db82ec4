// Shared host-side helpers of librfx: error reporting and HIP call checking.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "rfx.h"

namespace rfx {

// Records a message for rfx_last_error() and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// RAII device buffer used for per-call scratch.
struct DevBuf {
    void* p = nullptr;
    DevBuf() = default;
    DevBuf(const DevBuf&) = delete;
    DevBuf& operator=(const DevBuf&) = delete;
    ~DevBuf() { release(); }
    hipError_t alloc(size_t bytes) {
        release();
        return hipMalloc(&p, bytes ? bytes : 1);
    }
    void release() {
        if (p) (void)hipFree(p);
        p = nullptr;
    }
    template <class T>
    T* as() const {
        return static_cast<T*>(p);
    }
};

// Optional per-kernel timing (rfx_timing_enable): brackets one kernel launch with HIP events on
// the launch stream; rfx_timing_get waits for the events and accumulates the elapsed times.
struct TimedLaunch {
    TimedLaunch(const char* name, hipStream_t st);
    TimedLaunch(const TimedLaunch&) = delete;
    TimedLaunch& operator=(const TimedLaunch&) = delete;
    ~TimedLaunch();
    const char* name_;
    hipStream_t st_;
    hipEvent_t start_ = nullptr;
};

// Whether the row pass over the samples grouped by leaf is expected to list the non-zero pairs faster than the pair
// tests on bit planes (prox_rows.hip).
int sparse_rows_cheaper(const uint32_t* leaf, int64_t N, int32_t B, int32_t leaf_bound, hipStream_t st, bool* rows_cheaper);

}  // namespace rfx

#define RFX_HIP(call)                                                                                    \
    do {                                                                                                 \
        hipError_t e_ = (call);                                                                          \
        if (e_ != hipSuccess)                                                                            \
            return rfx::fail(e_ == hipErrorOutOfMemory ? RFX_ERR_OOM : RFX_ERR_HIP, "%s failed: %s", #call, \
                             hipGetErrorString(e_));                                                     \
    } while (0)

#define RFX_LAUNCH_CHECK(name)                                                                  \
    do {                                                                                        \
        hipError_t e_ = hipGetLastError();                                                      \
        if (e_ != hipSuccess)                                                                   \
            return rfx::fail(RFX_ERR_HIP, "launch of %s failed: %s", name, hipGetErrorString(e_)); \
    } while (0)
