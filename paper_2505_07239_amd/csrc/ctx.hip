// Context management of the comet_ring library.
#include "common.h"

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
    comet_ctx* ctx = new (std::nothrow) comet_ctx;
    if (!ctx) return COMET_EINVAL;
    ctx->device = device_id;
    ctx->num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    ctx->stream = nullptr;
    ctx->gemm_grid = 0;
    ctx->err[0] = '\0';
    *out = ctx;
    return COMET_OK;
}

int comet_destroy(comet_ctx* ctx) {
    COMET_CHECK_CTX(ctx);
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
    if (key != COMET_TUNE_GEMM_GRID || value < 0 || value > (1 << 16))
        return comet_fail(ctx, COMET_EINVAL, "comet_set_tuning: unknown key or bad value");
    ctx->gemm_grid = value;
    return COMET_OK;
}

const char* comet_last_error(const comet_ctx* ctx) { return ctx ? ctx->err : "null context"; }

}  // extern "C"
