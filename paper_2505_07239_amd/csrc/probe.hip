// Roofline probes: register-resident issue loops that measure what the chip
// sustains for the two candidate ways of doing ring arithmetic.  Measurement
// aids only; no protocol step uses them.
#include "common.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int PROBE_MFMA_PER_ITER = 8;

__device__ __forceinline__ u64 probe_mix(u64 z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Eight independent accumulators, one v_mfma_i32_32x32x32_i8 each per iteration, every one
// with its own operand pair.  RANDOM = false: small constants (most operand bits are zero);
// RANDOM = true: uniformly random bytes, which is what the digits of secret shares look like.
// The instruction stream is the same; the second draws far more power, and the chip lowers
// its clock accordingly, so the two rates bracket what a real kernel can reach.
template <bool RANDOM>
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, int* __restrict__ out) {
    v4i a[PROBE_MFMA_PER_ITER], b[PROBE_MFMA_PER_ITER];
    v16i acc[PROBE_MFMA_PER_ITER];
#pragma unroll
    for (int j = 0; j < PROBE_MFMA_PER_ITER; ++j) {
        if (RANDOM) {
            const u64 s = ((u64)blockIdx.x * 256 + threadIdx.x) * 64 + j * 8;
            const u64 r0 = probe_mix(s), r1 = probe_mix(s + 1), r2 = probe_mix(s + 2), r3 = probe_mix(s + 3);
            a[j] = v4i{(int)r0, (int)(r0 >> 32), (int)r1, (int)(r1 >> 32)};
            b[j] = v4i{(int)r2, (int)(r2 >> 32), (int)r3, (int)(r3 >> 32)};
        } else {
            a[j] = v4i{(int)threadIdx.x, 1, 2, 3 + j};
            b[j] = v4i{4, 5, (int)blockIdx.x, 7 + j};
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = j;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < PROBE_MFMA_PER_ITER; ++j)
            acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[j], b[j], acc[j], 0, 0, 0);
    }
    int r = 0;
#pragma unroll
    for (int j = 0; j < PROBE_MFMA_PER_ITER; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) r ^= acc[j][e];
    out[blockIdx.x * 256 + threadIdx.x] = r;
}

constexpr int PROBE_MAC_PER_ITER = 16;

// Sixteen independent 64-bit multiply-add chains per lane.
__global__ __launch_bounds__(256) void probe_mac64_kernel(int iters, u64* __restrict__ out) {
    u64 acc[PROBE_MAC_PER_ITER];
    u64 x = 0x9E3779B97F4A7C15ull * (threadIdx.x + 1), y = 0xBF58476D1CE4E5B9ull + blockIdx.x;
#pragma unroll
    for (int j = 0; j < PROBE_MAC_PER_ITER; ++j) acc[j] = j;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < PROBE_MAC_PER_ITER; ++j) acc[j] = acc[j] * x + y;
        x += 2;   // keeps the multiplier loop-variant without adding work per MAC
    }
    u64 r = 0;
#pragma unroll
    for (int j = 0; j < PROBE_MAC_PER_ITER; ++j) r ^= acc[j];
    out[blockIdx.x * 256 + threadIdx.x] = r;
}

}  // namespace

extern "C" {

int comet_probe_mfma_i8(comet_ctx* ctx, int blocks, int iters, int random_operands, int32_t* out,
                        double* macs) {
    COMET_CHECK_CTX(ctx);
    if (!out || blocks < 1 || iters < 0 || blocks > (1 << 20))
        return comet_fail(ctx, COMET_EINVAL, "comet_probe_mfma_i8: bad argument");
    comet_device_guard guard(ctx);
    if (!guard.ok) return comet_fail(ctx, COMET_EDEVICE, "comet_probe_mfma_i8: cannot select device");
    if (random_operands)
        hipLaunchKernelGGL(probe_mfma_kernel<true>, dim3(blocks), dim3(256), 0, ctx->stream, iters, out);
    else
        hipLaunchKernelGGL(probe_mfma_kernel<false>, dim3(blocks), dim3(256), 0, ctx->stream, iters, out);
    COMET_LAUNCH_CHECK(ctx, "comet_probe_mfma_i8");
    if (macs) *macs = (double)blocks * 4.0 * iters * PROBE_MFMA_PER_ITER * 32.0 * 32.0 * 32.0;
    return COMET_OK;
}

int comet_probe_valu_mac64(comet_ctx* ctx, int blocks, int iters, uint64_t* out, double* macs) {
    COMET_CHECK_CTX(ctx);
    if (!out || blocks < 1 || iters < 0 || blocks > (1 << 20))
        return comet_fail(ctx, COMET_EINVAL, "comet_probe_valu_mac64: bad argument");
    comet_device_guard guard(ctx);
    if (!guard.ok) return comet_fail(ctx, COMET_EDEVICE, "comet_probe_valu_mac64: cannot select device");
    hipLaunchKernelGGL(probe_mac64_kernel, dim3(blocks), dim3(256), 0, ctx->stream, iters, (u64*)out);
    COMET_LAUNCH_CHECK(ctx, "comet_probe_valu_mac64");
    if (macs) *macs = (double)blocks * 256.0 * iters * PROBE_MAC_PER_ITER;
    return COMET_OK;
}

}  // extern "C"
