// Context management of the comet_ring library.
#include "common.h"

size_t comet_compact_workspace_bytes(int64_t n_tok, int64_t nb);
size_t comet_gemm_workspace_bytes(int64_t m, int64_t kc_cap, int64_t n_cap);

extern "C" {

const char* comet_version(void) { return "comet_ring 0.1 (gfx950)"; }

int comet_create(comet_ctx** out, int device_id) {
    if (!out) return COMET_EINVAL;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device_id < 0 || device_id >= count) {
        (void)hipGetLastError();
        return COMET_EDEVICE;
    }
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device_id) != hipSuccess) return COMET_EDEVICE;
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) return COMET_EDEVICE;
    // the device's copy of the static scratch array: looked up here, once, with the device current
    void* static_ws = nullptr;
    {
        int prev = -1;
        if (hipGetDevice(&prev) != hipSuccess) return COMET_EDEVICE;
        if (prev != device_id && hipSetDevice(device_id) != hipSuccess) return COMET_EDEVICE;
        size_t bytes = 0;
        const int rc = comet_static_scratch(device_id, &static_ws, &bytes);
        if (prev != device_id) (void)hipSetDevice(prev);
        if (rc != COMET_OK) return rc;
    }
    comet_ctx* ctx = new (std::nothrow) comet_ctx;
    if (!ctx) return COMET_EINVAL;
    ctx->device = device_id;
    ctx->static_ws = static_ws;
    ctx->num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    ctx->stream = nullptr;
    ctx->gemm_grid = 0;
    ctx->gemm_chunk = 0;
    ctx->gemm_tile = 0;
    ctx->skinny_mode = 0;
    ctx->skinny_slices = 0;
    ctx->ev_stride = 0;
    ctx->group_mode = 0;
    ctx->components_mode = 0;
    ctx->ev = nullptr;
    ctx->ev_cap = ctx->ev_used = 0;
    ctx->ev_seen = 0;
    ctx->err[0] = '\0';
    *out = ctx;
    return COMET_OK;
}

static void drop_events(comet_ctx* ctx) {
    if (!ctx->ev) return;
    for (int i = 0; i < ctx->ev_cap; ++i) (void)hipEventDestroy(ctx->ev[i]);
    delete[] ctx->ev;
    ctx->ev = nullptr;
    ctx->ev_cap = ctx->ev_used = 0;
    ctx->ev_seen = 0;
}

int comet_destroy(comet_ctx* ctx) {
    COMET_CHECK_CTX(ctx);
    {
        comet_device_guard guard(ctx);
        drop_events(ctx);
    }
    delete ctx;
    return COMET_OK;
}

int comet_set_stream(comet_ctx* ctx, void* hip_stream) {
    COMET_CHECK_CTX(ctx);
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    return COMET_OK;
}

int comet_set_tuning(comet_ctx* ctx, int key, int value) {
    COMET_CHECK_CTX(ctx);
    if (key < COMET_TUNE_GEMM_GRID || key > COMET_TUNE_GROUP || value < 0 || value > (1 << 16))
        return comet_fail(ctx, COMET_EINVAL, "comet_set_tuning: unknown key or bad value");
    if (key == COMET_TUNE_GEMM_GRID) ctx->gemm_grid = value;
    else if (key == COMET_TUNE_GEMM_CHUNK) ctx->gemm_chunk = value;
    else if (key == COMET_TUNE_GEMM_TILE) ctx->gemm_tile = value;
    else if (key == COMET_TUNE_SKINNY) ctx->skinny_mode = value;
    else if (key == COMET_TUNE_SKINNY_SLICES) ctx->skinny_slices = value;
    else if (key == COMET_TUNE_TIMING_STRIDE) ctx->ev_stride = value;
    else if (key == COMET_TUNE_GROUP) ctx->group_mode = value;
    else ctx->components_mode = value;
    return COMET_OK;
}

int comet_timing_begin(comet_ctx* ctx, int max_launches) {
    COMET_CHECK_CTX(ctx);
    if (max_launches < 1 || max_launches > (1 << 20))
        return comet_fail(ctx, COMET_EINVAL, "comet_timing_begin: bad max_launches");
    comet_device_guard guard(ctx);
    if (!guard.ok) return comet_fail(ctx, COMET_EDEVICE, "comet_timing_begin: cannot select device");
    drop_events(ctx);
    ctx->ev = new (std::nothrow) hipEvent_t[2 * (size_t)max_launches];
    if (!ctx->ev) return comet_fail(ctx, COMET_EINVAL, "comet_timing_begin: out of host memory");
    for (int i = 0; i < 2 * max_launches; ++i) {
        if (hipEventCreate(&ctx->ev[i]) != hipSuccess) {
            ctx->ev_cap = i;
            drop_events(ctx);
            return comet_fail(ctx, COMET_EDEVICE, "comet_timing_begin: hipEventCreate failed");
        }
    }
    ctx->ev_cap = 2 * max_launches;
    ctx->ev_used = 0;
    ctx->ev_seen = 0;
    return COMET_OK;
}

int comet_timing_end(comet_ctx* ctx, double* total_ms, int* launches) {
    COMET_CHECK_CTX(ctx);
    if (!total_ms || !launches) return comet_fail(ctx, COMET_EINVAL, "comet_timing_end: null pointer");
    comet_device_guard guard(ctx);
    if (!guard.ok) return comet_fail(ctx, COMET_EDEVICE, "comet_timing_end: cannot select device");
    double sum = 0.0;
    int n = 0;
    if (ctx->ev && ctx->ev_used >= 2) {
        if (hipEventSynchronize(ctx->ev[ctx->ev_used - 1]) != hipSuccess) {
            drop_events(ctx);
            return comet_fail(ctx, COMET_EDEVICE, "comet_timing_end: hipEventSynchronize failed");
        }
        for (int i = 0; i + 1 < ctx->ev_used; i += 2) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, ctx->ev[i], ctx->ev[i + 1]) == hipSuccess) { sum += ms; ++n; }
        }
    }
    drop_events(ctx);
    *total_ms = sum;
    *launches = n;
    return COMET_OK;
}

size_t comet_workspace_bytes(int op, int64_t m, int64_t k, int64_t n, int bs) {
    (void)bs;
    switch (op) {
        case COMET_OP_COMPACT: return comet_compact_workspace_bytes(m, n);
        case COMET_OP_SOMM:
        case COMET_OP_SIMM: return comet_gemm_workspace_bytes(m, k, n);
        default: return 0;
    }
}

const char* comet_last_error(const comet_ctx* ctx) { return ctx ? ctx->err : "null context"; }

}  // extern "C"
