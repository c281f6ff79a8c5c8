// Streaming kernels of the masking / opening step (paper Sec. 2.1, Sec. 5.1):
//   [D]_i = [X]_i - [A]_i   and   E = [D]_0 + [D]_1   over uint64 words,
// plain and block-indexed.  All are bound by HBM bandwidth: 24 bytes move per
// element (two 8-byte reads, one 8-byte write), so the work per lane is one
// 16-byte load from each input and one 16-byte store, several in flight.
#include "common.h"

namespace {

constexpr int EW_THREADS = 256;
constexpr int EW_UNROLL = 4;

typedef u64 u64x2 __attribute__((ext_vector_type(2)));

template <bool SUB>
__device__ __forceinline__ u64x2 combine(u64x2 a, u64x2 b) {
    return SUB ? (a - b) : (a + b);
}

// One block walks chunks of EW_THREADS * EW_UNROLL 16-byte vectors; all loads
// of a chunk are issued before the first store so that each lane keeps
// 2 * EW_UNROLL requests in flight.
// The output may be one of the inputs (same address): every element is read and then written by
// the same lane, so the pointers carry no no-alias promise.
template <bool SUB>
__global__ __launch_bounds__(EW_THREADS) void ew_kernel(const u64* a, const u64* b, u64* o,
                                                        size_t n_elems) {
    const size_t nvec = n_elems >> 1;
    const u64x2* av = reinterpret_cast<const u64x2*>(a);
    const u64x2* bv = reinterpret_cast<const u64x2*>(b);
    u64x2* ov = reinterpret_cast<u64x2*>(o);
    const size_t chunk = (size_t)EW_THREADS * EW_UNROLL;
    for (size_t base = (size_t)blockIdx.x * chunk; base < nvec; base += (size_t)gridDim.x * chunk) {
        u64x2 ra[EW_UNROLL], rb[EW_UNROLL];
#pragma unroll
        for (int j = 0; j < EW_UNROLL; ++j) {
            const size_t i = base + (size_t)j * EW_THREADS + threadIdx.x;
            if (i < nvec) {
                ra[j] = __builtin_nontemporal_load(av + i);
                rb[j] = __builtin_nontemporal_load(bv + i);
            }
        }
#pragma unroll
        for (int j = 0; j < EW_UNROLL; ++j) {
            const size_t i = base + (size_t)j * EW_THREADS + threadIdx.x;
            if (i < nvec) __builtin_nontemporal_store(combine<SUB>(ra[j], rb[j]), ov + i);
        }
    }
    if ((n_elems & 1) && blockIdx.x == 0 && threadIdx.x == 0) {
        const size_t i = n_elems - 1;
        o[i] = SUB ? (a[i] - b[i]) : (a[i] + b[i]);
    }
}

// Indexed masking along columns: one grid column per matrix row, one lane per
// pair of adjacent kept columns (a pair never straddles a block when bs is
// even; the scalar variant covers odd bs or odd widths).
constexpr int GC_THREADS = 128;   // a workgroup covers eight 32-word blocks of a row (measured: 256 threads 3 % slower, 512 8 %)
template <int VEC>
__global__ __launch_bounds__(GC_THREADS) void gather_cols_kernel(
    const u64* __restrict__ w, const u64* __restrict__ b, u64* __restrict__ g, int cols, int ld,
    int bs, const int* __restrict__ blk_idx, const int* __restrict__ n_blk_dev, int n_blk_cap, int gy) {
    const int n_blk = n_blk_dev ? min(*n_blk_dev, n_blk_cap) : n_blk_cap;
    const int width = n_blk * bs;
    // workgroups are numbered row by row (the pieces of a row are dispatched together)
    const size_t r = blockIdx.x / (unsigned)gy;
    const int piece = (int)(blockIdx.x % (unsigned)gy);
    for (int c = (piece * GC_THREADS + threadIdx.x) * VEC; c < width; c += gy * GC_THREADS * VEC) {
        const int blk = c / bs;
        const long start = (long)blk_idx[blk] * bs;
        if (start < 0 || start + bs > cols) continue;      // id outside the matrix: skip, never fault
        const size_t src = r * (size_t)cols + (size_t)start + (c - blk * bs);
        const size_t dst = r * (size_t)ld + c;
        if (VEC == 2) {
            const u64x2 x = __builtin_nontemporal_load(reinterpret_cast<const u64x2*>(w + src));
            const u64x2 y = __builtin_nontemporal_load(reinterpret_cast<const u64x2*>(b + src));
            __builtin_nontemporal_store(x - y, reinterpret_cast<u64x2*>(g + dst));
        } else {
            g[dst] = w[src] - b[src];
        }
    }
}

// Indexed masking along rows: the workgroups of a kept matrix row follow each other.
constexpr int GR_THREADS = 128;
template <int VEC>
__global__ __launch_bounds__(GR_THREADS) void gather_rows_kernel(
    const u64* __restrict__ w, const u64* __restrict__ b, u64* __restrict__ g, int rows, int cols,
    int bs, const int* __restrict__ blk_idx, const int* __restrict__ n_blk_dev, int n_blk_cap, int gy) {
    const int n_blk = n_blk_dev ? min(*n_blk_dev, n_blk_cap) : n_blk_cap;
    // workgroups are numbered row by row (the pieces of a row are dispatched together)
    const int r = (int)(blockIdx.x / (unsigned)gy);
    const int piece = (int)(blockIdx.x % (unsigned)gy);
    if (r >= n_blk * bs) return;
    const int blk = r / bs;
    const long start = (long)blk_idx[blk] * bs;
    if (start < 0 || start + bs > rows) return;             // id outside the matrix: skip, never fault
    const size_t src = ((size_t)start + (r - blk * bs)) * (size_t)cols;
    const size_t dst = (size_t)r * cols;
    for (int c = (piece * GR_THREADS + threadIdx.x) * VEC; c < cols; c += gy * GR_THREADS * VEC) {
        if (VEC == 2) {
            const u64x2 x = __builtin_nontemporal_load(reinterpret_cast<const u64x2*>(w + src + c));
            const u64x2 y = __builtin_nontemporal_load(reinterpret_cast<const u64x2*>(b + src + c));
            __builtin_nontemporal_store(x - y, reinterpret_cast<u64x2*>(g + dst + c));
        } else {
            g[dst + c] = w[src + c] - b[src + c];
        }
    }
}

template <bool SUB>
int launch_ew(comet_ctx* ctx, const char* what, const u64* a, const u64* b, u64* o, size_t n) {
    COMET_CHECK_CTX(ctx);
    if (n == 0) return COMET_OK;      // nothing to do; empty buffers may be null
    if (!a || !b || !o) return comet_fail(ctx, COMET_EINVAL, "%s: null pointer", what);
    if (!comet_aligned16(a) || !comet_aligned16(b) || !comet_aligned16(o))
        return comet_fail(ctx, COMET_EALIGN, "%s: pointers must be 16-byte aligned", what);
    if (n > ((size_t)1 << 40)) return comet_fail(ctx, COMET_ECAP, "%s: n_elems too large", what);
    comet_device_guard guard(ctx);
    if (!guard.ok) return comet_fail(ctx, COMET_EDEVICE, "%s: cannot select device", what);
    const size_t chunk = (size_t)EW_THREADS * EW_UNROLL;
    const size_t need = ((n >> 1) + chunk - 1) / chunk;
    // one chunk per workgroup, in dispatch order: the chip then walks the three buffers front to
    // back (a chip-sized grid looping over strided chunks measured 5 % slower); the loop in the
    // kernel only matters beyond 2^30 chunks
    const size_t cap = (size_t)1 << 30;
    const unsigned grid = (unsigned)(need < 1 ? 1 : (need < cap ? need : cap));
    hipLaunchKernelGGL((ew_kernel<SUB>), dim3(grid), dim3(EW_THREADS), 0, ctx->stream, a, b, o, n);
    COMET_LAUNCH_CHECK(ctx, what);
    return COMET_OK;
}

}  // namespace

extern "C" {

int comet_mask_share(comet_ctx* ctx, const uint64_t* x_i, const uint64_t* a_i, uint64_t* d_i,
                     size_t n_elems) {
    return launch_ew<true>(ctx, "comet_mask_share", (const u64*)x_i, (const u64*)a_i, (u64*)d_i,
                           n_elems);
}

int comet_open(comet_ctx* ctx, const uint64_t* d_0, const uint64_t* d_1, uint64_t* e,
               size_t n_elems) {
    return launch_ew<false>(ctx, "comet_open", (const u64*)d_0, (const u64*)d_1, (u64*)e, n_elems);
}

int comet_probe_copy(comet_ctx* ctx, const uint64_t* src, uint64_t* dst, size_t n_elems) {
    COMET_CHECK_CTX(ctx);
    if (!src || !dst) return comet_fail(ctx, COMET_EINVAL, "comet_probe_copy: null pointer");
    comet_device_guard guard(ctx);
    if (!guard.ok) return comet_fail(ctx, COMET_EDEVICE, "comet_probe_copy: cannot select device");
    if (hipMemcpyAsync(dst, src, n_elems * sizeof(u64), hipMemcpyDeviceToDevice, ctx->stream) !=
        hipSuccess)
        return comet_fail(ctx, COMET_EDEVICE, "comet_probe_copy: hipMemcpyAsync failed");
    return COMET_OK;
}

int comet_mask_share_gather(comet_ctx* ctx, const uint64_t* w_i, const uint64_t* b_i,
                            uint64_t* g_i, int64_t rows, int64_t cols, int axis, int bs,
                            const int32_t* blk_idx, const int32_t* n_blk_dev, int n_blk_cap) {
    const char* what = "comet_mask_share_gather";
    COMET_CHECK_CTX(ctx);
    if (!w_i || !b_i || !g_i || !blk_idx) return comet_fail(ctx, COMET_EINVAL, "%s: null pointer", what);
    if (rows < 0 || cols < 0 || bs < 1 || n_blk_cap < 0 ||
        (axis != COMET_AXIS_COLS && axis != COMET_AXIS_ROWS))
        return comet_fail(ctx, COMET_EINVAL, "%s: bad size or axis", what);
    if (rows > COMET_DIM_MAX || cols > COMET_DIM_MAX || (int64_t)n_blk_cap * bs > COMET_DIM_MAX)
        return comet_fail(ctx, COMET_ECAP, "%s: dimension beyond 2^24", what);
    const int64_t extent = axis == COMET_AXIS_COLS ? cols : rows;
    if ((int64_t)n_blk_cap * bs > extent)
        return comet_fail(ctx, COMET_EINVAL, "%s: n_blk_cap * bs exceeds the indexed axis", what);
    if (!comet_aligned16(w_i) || !comet_aligned16(b_i) || !comet_aligned16(g_i))
        return comet_fail(ctx, COMET_EALIGN, "%s: pointers must be 16-byte aligned", what);
    const int ld = n_blk_cap * bs;
    if (rows == 0 || cols == 0 || ld == 0) return COMET_OK;
    comet_device_guard guard(ctx);
    if (!guard.ok) return comet_fail(ctx, COMET_EDEVICE, "%s: cannot select device", what);
    if (axis == COMET_AXIS_COLS) {
        const bool vec = (bs % 2 == 0) && (cols % 2 == 0);
        const int per = GC_THREADS * (vec ? 2 : 1);
        long gy = (ld + per - 1) / per;
        // pieces per row, capped so that rows x pieces stays a valid one-dimensional grid
        const long gy_max = (1l << 31) / (rows > 0 ? rows : 1) - 1;
        if (gy > gy_max) gy = gy_max < 1 ? 1 : gy_max;
        const dim3 grid((unsigned)(rows * gy));
        if (vec)
            hipLaunchKernelGGL((gather_cols_kernel<2>), grid, dim3(GC_THREADS), 0, ctx->stream,
                               (const u64*)w_i, (const u64*)b_i, (u64*)g_i, (int)cols, ld, bs,
                               blk_idx, n_blk_dev, n_blk_cap, (int)gy);
        else
            hipLaunchKernelGGL((gather_cols_kernel<1>), grid, dim3(GC_THREADS), 0, ctx->stream,
                               (const u64*)w_i, (const u64*)b_i, (u64*)g_i, (int)cols, ld, bs,
                               blk_idx, n_blk_dev, n_blk_cap, (int)gy);
    } else {
        const bool vec = (cols % 2 == 0);
        const int per = GR_THREADS * (vec ? 2 : 1) * 2;
        long gy = (cols + per - 1) / per;
        const long gy_max = (1l << 31) / ld - 1;           // rows x pieces stays a valid one-dimensional grid
        if (gy > gy_max) gy = gy_max < 1 ? 1 : gy_max;
        const dim3 grid((unsigned)((long)ld * gy));
        if (vec)
            hipLaunchKernelGGL((gather_rows_kernel<2>), grid, dim3(GR_THREADS), 0, ctx->stream,
                               (const u64*)w_i, (const u64*)b_i, (u64*)g_i, (int)rows, (int)cols, bs,
                               blk_idx, n_blk_dev, n_blk_cap, (int)gy);
        else
            hipLaunchKernelGGL((gather_rows_kernel<1>), grid, dim3(GR_THREADS), 0, ctx->stream,
                               (const u64*)w_i, (const u64*)b_i, (u64*)g_i, (int)rows, (int)cols, bs,
                               blk_idx, n_blk_dev, n_blk_cap, (int)gy);
    }
    COMET_LAUNCH_CHECK(ctx, what);
    return COMET_OK;
}

}  // extern "C"
