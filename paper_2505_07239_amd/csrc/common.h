// Shared host-side declarations of the comet_ring library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <new>

#include "comet_ring.h"

typedef unsigned long long u64;
typedef unsigned int u32;

struct comet_ctx {
    int device;
    int num_cu;
    hipStream_t stream;
    int gemm_grid;   // 0 = automatic
    int gemm_chunk;  // 0 = default
    int gemm_tile;   // 0 = automatic
    int skinny_mode;   // 0 = automatic, 1 = never take the vector-ALU path
    int skinny_slices; // 0 = automatic
    int components_mode; // 0 = automatic, 1 = always the multi-workgroup component search
    int group_mode;      // comet_share_group: 0 = automatic, 1 = one launch whenever possible, 2 = never
    hipEvent_t* ev;  // timing event pairs, or null
    int ev_cap, ev_used;
    int ev_stride;   // time every ev_stride-th share call (0 or 1: every call)
    long ev_seen;    // share calls since timing began
    void* static_ws; // this device's copy of the library's static scratch array (device address)
    char err[512];
};

// Device address and size of the static scratch array on `device` (which must be current).
// Defined beside the array, in ring_gemm.hip; looked up once per device.
int comet_static_scratch(int device, void** ptr, size_t* bytes);

static inline int comet_fail(comet_ctx* ctx, int code, const char* fmt, ...) {
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return code;
}

// Is the share kernel about to be launched a timed one?  (counts the launch)
static inline bool comet_time_this_launch(comet_ctx* ctx) {
    if (!ctx->ev) return false;
    const long seen = ctx->ev_seen++;
    if (ctx->ev_stride > 1 && seen % ctx->ev_stride != 0) return false;
    return ctx->ev_used + 2 <= ctx->ev_cap;
}

static inline bool comet_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Makes the context's device current for the duration of a call.
struct comet_device_guard {
    int prev;
    bool ok;
    explicit comet_device_guard(const comet_ctx* ctx) : prev(-1), ok(true) {
        if (hipGetDevice(&prev) != hipSuccess) { ok = false; return; }
        if (prev != ctx->device && hipSetDevice(ctx->device) != hipSuccess) ok = false;
    }
    ~comet_device_guard() {
        int cur = -1;
        if (prev >= 0 && hipGetDevice(&cur) == hipSuccess && cur != prev) (void)hipSetDevice(prev);
    }
};

#define COMET_CHECK_CTX(ctx)                                             \
    do {                                                                 \
        if (!(ctx)) return COMET_EINVAL;                                 \
    } while (0)

#define COMET_LAUNCH_CHECK(ctx, what)                                                            \
    do {                                                                                         \
        hipError_t e_ = hipGetLastError();                                                       \
        if (e_ != hipSuccess)                                                                    \
            return comet_fail((ctx), COMET_EDEVICE, "%s: launch failed: %s", (what),             \
                              hipGetErrorString(e_));                                            \
    } while (0)

// Limits shared by the host checks and the kernels' 32-bit index arithmetic.
static const int64_t COMET_DIM_MAX = (1ll << 24) - 1;
static const int64_t COMET_ROWS_MAX = (1ll << 22) - 128;   // rows of the activation side of a share call
