// Weight-side operands of the share calls as digit planes (the format PlaneLoader of
// ring_gemm_kernel.h reads with LDS-DMA): the opening of the masked weights, F = [G]_0 + [G]_1
// (paper Sec. 2.1; Protocols 2 and 3 open only the indexed sub-matrices), written directly in
// that format, and the same packing for a single operand (the triple share B_i, which is
// offline material, Sec. 3.2).
//
// Format of a k x n matrix W: 16-byte units; unit (s, t, g, c) holds digit t of the sixteen words
// W[32 s + 16 g + 0..15][c].  Units are ordered (step s, chunk c / 64, digit t, k-half g, c % 64),
// so the sixteen (t, g) runs that one contraction step of a 64-column tile needs are 16 KB of
// consecutive memory.  Rows at or beyond k read as zero and the last chunk is padded to 64
// columns (never read), so the buffer has ceil(k / 32) * 32 * ceil(n / 64) * 64 * 8 bytes.
// HBM-bound: 8 bytes written per word read, like the plain opening.
#include "digits.h"

namespace {

using namespace comet_gemm;

constexpr int WT = 128;
typedef u64 u64x2 __attribute__((ext_vector_type(2)));

// One thread packs sixteen contraction rows of one column: its sixteen loads per operand are
// coalesced across the wavefront (adjacent columns), and so are its eight 16-byte stores.
__global__ __launch_bounds__(WT) void wpack_kernel(const u64* __restrict__ a, const u64* __restrict__ b,
                                                   u64x2* __restrict__ out, long k, long n, long groups) {
    const long c = (long)blockIdx.x * WT + threadIdx.x;
    const long nch = (n + 63) >> 6;
    if (c >= n) return;
    for (long q = blockIdx.y; q < groups; q += gridDim.y) {
        const long r0 = q * 16;
        u64 w[16];
        if (r0 + 16 <= k) {
#pragma unroll
            for (int i = 0; i < 16; ++i) w[i] = __builtin_nontemporal_load(a + (r0 + i) * n + c);
            if (b) {
#pragma unroll
                for (int i = 0; i < 16; ++i) w[i] += __builtin_nontemporal_load(b + (r0 + i) * n + c);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                w[i] = 0;
                if (r0 + i < k) w[i] = a[(r0 + i) * n + c] + (b ? b[(r0 + i) * n + c] : 0ull);
            }
        }
        u64 plane[2][8];
#pragma unroll
        for (int o = 0; o < 2; ++o) {
            u64 v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = to_digits(w[8 * o + i]);
            digits_to_planes(v, plane[o]);
        }
        const long s = q >> 1, g = q & 1;
        u64x2* dst = out + ((s * nch + (c >> 6)) * 16 + g) * 64 + (c & 63);
#pragma unroll
        for (int t = 0; t < 8; ++t)
            __builtin_nontemporal_store(u64x2{plane[0][t], plane[1][t]}, dst + t * 128);
    }
}

// The same planes from operands stored one ROW per column of W (n x k: the neuron-major layout of
// the SOMM weights, in which the sixteen contraction rows of a unit are 128 consecutive bytes).
// Loads want the lanes along k, the stores along the columns, so a workgroup passes a tile of 64
// columns x 64 contraction rows through LDS: coalesced 16-byte loads of both shares, their sum
// into the tile, then every thread takes the sixteen words of one (column, k-half) from there.
constexpr int TT = 256;
constexpr int TPITCH = 33;                       // 16-byte vectors per tile row (32 + 1 of padding)
__global__ __launch_bounds__(TT) void wpack_t_kernel(const u64* __restrict__ a, const u64* __restrict__ b,
                                                     u64x2* __restrict__ out, long k, long n) {
    __shared__ u64x2 tile[64 * TPITCH];
    const long c0 = (long)blockIdx.y * 64, k0 = (long)blockIdx.x * 64;
    const long nch = (n + 63) >> 6;
    const bool vec = (k & 1) == 0;               // rows start on 16-byte boundaries
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int v = i * TT + threadIdx.x;      // vector of the tile: column v / 32, words 2 (v % 32) ..
        const int c = v >> 5, kv = v & 31;
        const long col = c0 + c, kk = k0 + 2 * kv;
        u64x2 w = {0, 0};
        if (col < n) {
            const u64* pa = a + col * k + kk;
            const u64* pb = b ? b + col * k + kk : nullptr;
            if (vec && kk + 2 <= k) {
                w = __builtin_nontemporal_load(reinterpret_cast<const u64x2*>(pa));
                if (pb) w += __builtin_nontemporal_load(reinterpret_cast<const u64x2*>(pb));
            } else {
                if (kk < k) w.x = pa[0] + (pb ? pb[0] : 0ull);
                if (kk + 1 < k) w.y = pa[1] + (pb ? pb[1] : 0ull);
            }
        }
        tile[c * TPITCH + kv] = w;
    }
    __syncthreads();
    const int c = threadIdx.x & 63, q = threadIdx.x >> 6;      // column of the chunk, sixteen-row group of the tile
    const long col = c0 + c;
    const long r0 = k0 + 16 * q;
    if (col >= n || r0 >= ((k + 31) >> 5) * 32) return;
    u64 w[16];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const u64x2 t = tile[c * TPITCH + 8 * q + i];
        w[2 * i] = t.x; w[2 * i + 1] = t.y;
    }
    u64 plane[2][8];
#pragma unroll
    for (int o = 0; o < 2; ++o) {
        u64 v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = to_digits(w[8 * o + i]);
        digits_to_planes(v, plane[o]);
    }
    const long s = r0 >> 5, g = (r0 >> 4) & 1;
    u64x2* dst = out + ((s * nch + (col >> 6)) * 16 + g) * 64 + (col & 63);
#pragma unroll
    for (int t = 0; t < 8; ++t)
        __builtin_nontemporal_store(u64x2{plane[0][t], plane[1][t]}, dst + t * 128);
}

}  // namespace

extern "C" {

size_t comet_weight_planes_bytes(int64_t k, int64_t n) {
    if (k < 0 || n < 0 || k > COMET_DIM_MAX || n > COMET_DIM_MAX) return 0;
    return (size_t)((k + 31) / 32) * 32 * (size_t)((n + 63) / 64) * 64 * 8;
}

static int open_planes(comet_ctx* ctx, const char* what, const uint64_t* g_0, const uint64_t* g_1, int64_t k,
                       int64_t n, void* planes, bool neuron_major) {
    COMET_CHECK_CTX(ctx);
    if (k < 0 || n < 0) return comet_fail(ctx, COMET_EINVAL, "%s: bad size", what);
    if (k > COMET_DIM_MAX || n > COMET_DIM_MAX || k * n >= (1ll << 31))
        return comet_fail(ctx, COMET_ECAP, "%s: dimension beyond 2^24 or 2^31 words and more", what);
    if (k == 0 || n == 0) return COMET_OK;
    if (!g_0 || !planes) return comet_fail(ctx, COMET_EINVAL, "%s: null pointer", what);
    if (!comet_aligned16(g_0) || (g_1 && !comet_aligned16(g_1)) || !comet_aligned16(planes))
        return comet_fail(ctx, COMET_EALIGN, "%s: pointers must be 16-byte aligned", what);
    comet_device_guard guard(ctx);
    if (!guard.ok) return comet_fail(ctx, COMET_EDEVICE, "%s: cannot select device", what);
    if (neuron_major) {
        // one workgroup per (chunk of 64 columns, 64 contraction rows); the tiles along k of a chunk are
        // dispatched together: they read adjacent pieces of the same 64 operand rows (4 % faster than
        // the tiles of one contraction step together)
        const dim3 grid((unsigned)((k + 63) / 64), (unsigned)((n + 63) / 64));
        hipLaunchKernelGGL(wpack_t_kernel, grid, dim3(TT), 0, ctx->stream, (const u64*)g_0, (const u64*)g_1,
                           (u64x2*)planes, (long)k, (long)n);
        COMET_LAUNCH_CHECK(ctx, what);
        return COMET_OK;
    }
    const long groups = 2 * ((k + 31) / 32);
    const unsigned gx = (unsigned)((n + WT - 1) / WT);
    // one workgroup per (chunk of columns, group of sixteen rows), in dispatch order
    long gy = groups;
    if (gy > 65535) gy = 65535;
    if (gy < 1) gy = 1;
    hipLaunchKernelGGL(wpack_kernel, dim3(gx, (unsigned)gy), dim3(WT), 0, ctx->stream, (const u64*)g_0,
                       (const u64*)g_1, (u64x2*)planes, (long)k, (long)n, groups);
    COMET_LAUNCH_CHECK(ctx, what);
    return COMET_OK;
}

int comet_open_weight_planes(comet_ctx* ctx, const uint64_t* g_0, const uint64_t* g_1, int64_t k, int64_t n,
                             void* planes) {
    return open_planes(ctx, "comet_open_weight_planes", g_0, g_1, k, n, planes, false);
}

int comet_open_weight_planes_neuron_major(comet_ctx* ctx, const uint64_t* g_0, const uint64_t* g_1, int64_t k,
                                          int64_t n, void* planes) {
    return open_planes(ctx, "comet_open_weight_planes_neuron_major", g_0, g_1, k, n, planes, true);
}

}  // extern "C"
