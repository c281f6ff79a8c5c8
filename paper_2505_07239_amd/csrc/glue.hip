// Local steps around the sparse matrix products, all bound by HBM bandwidth:
//   * the two online steps of the oblivious shuffle (paper Sec. 4.2, Protocol 1):
//       y_i = tau_i(x_i) + a_i          and          z_i = rho_i(y_other) - b_i,
//     a permutation along one axis of a matrix fused with the mask add / subtract;
//   * the merge of a compact result back to the full width ("reshaped to origin size",
//     Protocol 2's Merge for whole column blocks);
//   * the share-local rescaling of a fixed-point product (each party shifts its own share).
// A permutation p acts as p(x)_j = x[p[j]]: the paper's example pi = [2, 1, 3] gives
// [x_2, x_1, x_3].
#include "common.h"

namespace {

constexpr int GT = 256;
constexpr int PT = 1024;              // threads of the column-permutation workgroup
constexpr int ROW_WORDS = 16384;      // longest row staged in LDS (128 KB)

typedef u64 u64x2 __attribute__((ext_vector_type(2)));

// Permutation of whole rows: dst(j, :) = src(perm[j], :) +/- mask(j, :).  One workgroup per
// (output row, chunk of columns); rows are contiguous, so every access is a full-width vector.
template <int VEC, bool SUB>
__global__ __launch_bounds__(GT) void permute_rows_kernel(const u64* __restrict__ src,
                                                          const int* __restrict__ perm,
                                                          const u64* __restrict__ mask,
                                                          u64* __restrict__ dst, int rows, int cols, int gy) {
    // workgroups are numbered row by row (the pieces of a row are dispatched together)
    const int j = (int)(blockIdx.x / (unsigned)gy);
    const int piece = (int)(blockIdx.x % (unsigned)gy);
    int from = perm[j];
    from = (from < 0 || from >= rows) ? 0 : from;             // a bad entry never leaves the operand
    const u64* s = src + (size_t)from * cols;
    const u64* mk = mask + (size_t)j * cols;
    u64* d = dst + (size_t)j * cols;
    const int nvec = cols / VEC;
    for (int c = piece * GT + threadIdx.x; c < nvec; c += gy * GT) {
        if (VEC == 2) {
            const u64x2 v = __builtin_nontemporal_load(reinterpret_cast<const u64x2*>(s) + c);
            const u64x2 q = __builtin_nontemporal_load(reinterpret_cast<const u64x2*>(mk) + c);
            __builtin_nontemporal_store(SUB ? v - q : v + q, reinterpret_cast<u64x2*>(d) + c);
        } else {
            d[c] = SUB ? s[c] - mk[c] : s[c] + mk[c];
        }
    }
}

// Permutation inside rows: dst(r, j) = src(r, perm[j]) +/- mask(r, j).  A workgroup stages a
// whole source row in LDS with coalesced loads and gathers from there, so that HBM sees each
// word once, in order; rows are dealt round-robin to the workgroups.  A row fills most of a
// compute unit's LDS, so one workgroup is resident per unit: to keep loads in flight during the
// gather, the next row is fetched into registers before the current one is gathered.
constexpr int ROW_VECS = ROW_WORDS / 2 / PT;                  // 16-byte vectors of a row per thread
template <bool SUB>
__global__ __launch_bounds__(PT) void permute_cols_lds_kernel(const u64* __restrict__ src,
                                                              const int* __restrict__ perm,
                                                              const u64* __restrict__ mask,
                                                              u64* __restrict__ dst, int rows, int cols) {
    __shared__ __align__(16) u64 row[ROW_WORDS];
    const bool vec = (cols & 1) == 0;
    const int nvec = cols / 2;
    u64x2 nxt[ROW_VECS];
    auto fetch = [&](int r) {
        const u64x2* s = reinterpret_cast<const u64x2*>(src + (size_t)r * cols);
#pragma unroll
        for (int i = 0; i < ROW_VECS; ++i) {
            const int c = i * PT + threadIdx.x;
            if (c < nvec) nxt[i] = __builtin_nontemporal_load(s + c);
        }
    };
    if (vec && (int)blockIdx.x < rows) fetch(blockIdx.x);
    for (int r = blockIdx.x; r < rows; r += gridDim.x) {
        if (vec) {
#pragma unroll
            for (int i = 0; i < ROW_VECS; ++i) {
                const int c = i * PT + threadIdx.x;
                if (c < nvec) reinterpret_cast<u64x2*>(row)[c] = nxt[i];
            }
        } else {
            const u64* s = src + (size_t)r * cols;
            for (int c = threadIdx.x; c < cols; c += PT) row[c] = s[c];
        }
        __syncthreads();
        if (vec && r + (int)gridDim.x < rows) fetch(r + gridDim.x);
        const u64* mk = mask + (size_t)r * cols;
        u64* d = dst + (size_t)r * cols;
        if (vec) {
            for (int c = threadIdx.x; c < nvec; c += PT) {
                int f0 = perm[2 * c], f1 = perm[2 * c + 1];
                f0 = (f0 < 0 || f0 >= cols) ? 0 : f0;
                f1 = (f1 < 0 || f1 >= cols) ? 0 : f1;
                const u64x2 v = {row[f0], row[f1]};
                const u64x2 q = __builtin_nontemporal_load(reinterpret_cast<const u64x2*>(mk) + c);
                __builtin_nontemporal_store(SUB ? v - q : v + q, reinterpret_cast<u64x2*>(d) + c);
            }
        } else {
            for (int c = threadIdx.x; c < cols; c += PT) {
                int from = perm[c];
                from = (from < 0 || from >= cols) ? 0 : from;
                const u64 v = row[from];
                const u64 q = mk[c];
                d[c] = SUB ? v - q : v + q;
            }
        }
        __syncthreads();
    }
}

// rows longer than the LDS stage: gather straight from global memory
template <bool SUB>
__global__ __launch_bounds__(GT) void permute_cols_direct_kernel(const u64* __restrict__ src,
                                                                 const int* __restrict__ perm,
                                                                 const u64* __restrict__ mask,
                                                                 u64* __restrict__ dst, int rows, int cols) {
    const int r = blockIdx.x;
    const u64* s = src + (size_t)r * cols;
    const u64* mk = mask + (size_t)r * cols;
    u64* d = dst + (size_t)r * cols;
    for (int c = blockIdx.y * GT + threadIdx.x; c < cols; c += gridDim.y * GT) {
        int from = perm[c];
        from = (from < 0 || from >= cols) ? 0 : from;
        const u64 v = s[from], q = mk[c];
        d[c] = SUB ? v - q : v + q;
    }
}

// (the streaming kernels below give every workgroup one contiguous chunk of GT * SU 16-byte
// vectors, in dispatch order: the chip walks the buffers front to back)
constexpr int SU = 4;
__global__ __launch_bounds__(GT) void fill_zero_kernel(u64* __restrict__ p, size_t n) {
    const size_t nvec = n >> 1;
    u64x2* pv = reinterpret_cast<u64x2*>(p);
    const size_t chunk = (size_t)GT * SU;
    for (size_t base = (size_t)blockIdx.x * chunk; base < nvec; base += (size_t)gridDim.x * chunk) {
#pragma unroll
        for (int j = 0; j < SU; ++j) {
            const size_t i = base + (size_t)j * GT + threadIdx.x;
            if (i < nvec) __builtin_nontemporal_store(u64x2{0, 0}, pv + i);
        }
    }
    if ((n & 1) && blockIdx.x == 0 && threadIdx.x == 0) p[n - 1] = 0;
}

// full(r, blk_idx[t] * bs + j) = compact(r, t * bs + j); grid.x = row, grid.y = column chunks
// (numbering the workgroups row by row, which helps the gathers, measured 3 % slower here)
template <int VEC>
__global__ __launch_bounds__(GT) void scatter_cols_kernel(const u64* __restrict__ compact, int ld, int bs,
                                                          const int* __restrict__ blk_idx,
                                                          const int* __restrict__ n_blk_dev, int n_blk_cap,
                                                          u64* __restrict__ full, int n_full) {
    int nblk = n_blk_cap;
    if (n_blk_dev) {
        const int d = *n_blk_dev;
        nblk = d < 0 ? 0 : (d < nblk ? d : nblk);
    }
    const int n_eff = nblk * bs;
    const u64* s = compact + (size_t)blockIdx.x * ld;
    u64* d = full + (size_t)blockIdx.x * n_full;
    for (int c = (blockIdx.y * GT + threadIdx.x) * VEC; c < n_eff; c += gridDim.y * GT * VEC) {
        const int t = c / bs;
        const long st = (long)blk_idx[t] * bs;
        if (st < 0 || st + bs > n_full) continue;             // an id that does not fit is dropped
        const long o = st + (c - t * bs);
        if (VEC == 2) *reinterpret_cast<u64x2*>(d + o) = *reinterpret_cast<const u64x2*>(s + c);
        else d[o] = s[c];
    }
}

// party 0: floor(z / 2^f) on the signed word;  party 1: -floor(-z / 2^f)
__global__ __launch_bounds__(GT) void truncate_kernel(int party, const u64* __restrict__ z,
                                                      u64* __restrict__ out, size_t n, int f) {
    auto one = [&](u64 v) -> u64 {
        return party == 0 ? (u64)((long long)v >> f) : (u64)0 - (u64)((long long)((u64)0 - v) >> f);
    };
    const size_t nvec = n >> 1;
    const size_t chunk = (size_t)GT * SU;
    for (size_t base = (size_t)blockIdx.x * chunk; base < nvec; base += (size_t)gridDim.x * chunk) {
        u64x2 v[SU];
#pragma unroll
        for (int j = 0; j < SU; ++j) {
            const size_t i = base + (size_t)j * GT + threadIdx.x;
            if (i < nvec) v[j] = __builtin_nontemporal_load(reinterpret_cast<const u64x2*>(z) + i);
        }
#pragma unroll
        for (int j = 0; j < SU; ++j) {
            const size_t i = base + (size_t)j * GT + threadIdx.x;
            if (i < nvec) __builtin_nontemporal_store(u64x2{one(v[j].x), one(v[j].y)}, reinterpret_cast<u64x2*>(out) + i);
        }
    }
    if ((n & 1) && blockIdx.x == 0 && threadIdx.x == 0) out[n - 1] = one(z[n - 1]);
}

// workgroups for n_elems words: one chunk each (the kernels loop beyond 2^30 chunks)
inline unsigned stream_grid(size_t n_elems) {
    const size_t chunk = (size_t)GT * SU * 2;
    size_t g = (n_elems + chunk - 1) / chunk;
    if (g > ((size_t)1 << 30)) g = (size_t)1 << 30;
    return (unsigned)(g < 1 ? 1 : g);
}

}  // namespace

extern "C" {

int comet_permute_mask(comet_ctx* ctx, const uint64_t* src, const int32_t* perm, const uint64_t* mask,
                       uint64_t* dst, int64_t rows, int64_t cols, int axis, int sign) {
    const char* what = "comet_permute_mask";
    COMET_CHECK_CTX(ctx);
    if (rows < 0 || cols < 0 || rows > COMET_DIM_MAX || cols > COMET_DIM_MAX)
        return comet_fail(ctx, COMET_EINVAL, "%s: bad size", what);
    if ((axis != COMET_AXIS_COLS && axis != COMET_AXIS_ROWS) || (sign != 1 && sign != -1))
        return comet_fail(ctx, COMET_EINVAL, "%s: axis must be COMET_AXIS_COLS or _ROWS, sign +1 or -1", what);
    if (rows == 0 || cols == 0) return COMET_OK;
    if (!src || !perm || !mask || !dst) return comet_fail(ctx, COMET_EINVAL, "%s: null pointer", what);
    if (src == dst) return comet_fail(ctx, COMET_EINVAL, "%s: dst must not alias src", what);
    if (!comet_aligned16(src) || !comet_aligned16(mask) || !comet_aligned16(dst))
        return comet_fail(ctx, COMET_EALIGN, "%s: operands must be 16-byte aligned", what);
    comet_device_guard guard(ctx);
    if (!guard.ok) return comet_fail(ctx, COMET_EDEVICE, "%s: cannot select device", what);
    const u64* s = (const u64*)src;
    const u64* mk = (const u64*)mask;
    u64* d = (u64*)dst;
    if (axis == COMET_AXIS_ROWS) {
        const bool vec = (cols & 1) == 0;
        unsigned gy = (unsigned)(((vec ? cols / 2 : cols) + GT * 4 - 1) / (GT * 4));
        if (gy < 1) gy = 1;
        if (gy > 64) gy = 64;
        const dim3 grid((unsigned)(rows * gy));               // rows < 2^24, gy <= 64
        if (vec && sign > 0) hipLaunchKernelGGL((permute_rows_kernel<2, false>), grid, dim3(GT), 0, ctx->stream, s, perm, mk, d, (int)rows, (int)cols, (int)gy);
        else if (vec) hipLaunchKernelGGL((permute_rows_kernel<2, true>), grid, dim3(GT), 0, ctx->stream, s, perm, mk, d, (int)rows, (int)cols, (int)gy);
        else if (sign > 0) hipLaunchKernelGGL((permute_rows_kernel<1, false>), grid, dim3(GT), 0, ctx->stream, s, perm, mk, d, (int)rows, (int)cols, (int)gy);
        else hipLaunchKernelGGL((permute_rows_kernel<1, true>), grid, dim3(GT), 0, ctx->stream, s, perm, mk, d, (int)rows, (int)cols, (int)gy);
    } else if (cols <= ROW_WORDS) {
        unsigned g = (unsigned)(rows < ctx->num_cu ? rows : ctx->num_cu);
        if (sign > 0) hipLaunchKernelGGL(permute_cols_lds_kernel<false>, dim3(g), dim3(PT), 0, ctx->stream, s, perm, mk, d, (int)rows, (int)cols);
        else hipLaunchKernelGGL(permute_cols_lds_kernel<true>, dim3(g), dim3(PT), 0, ctx->stream, s, perm, mk, d, (int)rows, (int)cols);
    } else {
        unsigned gy = (unsigned)((cols + GT * 4 - 1) / (GT * 4));
        if (gy > 256) gy = 256;
        const dim3 grid((unsigned)rows, gy);
        if (sign > 0) hipLaunchKernelGGL(permute_cols_direct_kernel<false>, grid, dim3(GT), 0, ctx->stream, s, perm, mk, d, (int)rows, (int)cols);
        else hipLaunchKernelGGL(permute_cols_direct_kernel<true>, grid, dim3(GT), 0, ctx->stream, s, perm, mk, d, (int)rows, (int)cols);
    }
    COMET_LAUNCH_CHECK(ctx, what);
    return COMET_OK;
}

int comet_scatter_cols(comet_ctx* ctx, const uint64_t* compact, int64_t m, int bs, const int32_t* blk_idx,
                       const int32_t* n_blk_dev, int n_blk_cap, uint64_t* full, int64_t n_full) {
    const char* what = "comet_scatter_cols";
    COMET_CHECK_CTX(ctx);
    if (m < 0 || bs < 1 || n_blk_cap < 0 || n_full < 0 || m > COMET_DIM_MAX || n_full > COMET_DIM_MAX ||
        (int64_t)n_blk_cap * bs > COMET_DIM_MAX)
        return comet_fail(ctx, COMET_EINVAL, "%s: bad size", what);
    if (m == 0 || n_full == 0) return COMET_OK;
    if (!full || (n_blk_cap > 0 && (!compact || !blk_idx)))
        return comet_fail(ctx, COMET_EINVAL, "%s: null pointer", what);
    if (!comet_aligned16(full) || (compact && !comet_aligned16(compact)))
        return comet_fail(ctx, COMET_EALIGN, "%s: operands must be 16-byte aligned", what);
    comet_device_guard guard(ctx);
    if (!guard.ok) return comet_fail(ctx, COMET_EDEVICE, "%s: cannot select device", what);
    const size_t total = (size_t)m * (size_t)n_full;
    hipLaunchKernelGGL(fill_zero_kernel, dim3(stream_grid(total)), dim3(GT), 0, ctx->stream,
                       (u64*)full, total);
    COMET_LAUNCH_CHECK(ctx, what);
    if (n_blk_cap == 0) return COMET_OK;
    const int ld = n_blk_cap * bs;
    const bool vec = (bs & 1) == 0 && (n_full & 1) == 0;      // ld is then even too
    unsigned gy = (unsigned)((ld / (vec ? 2 : 1) + GT * 2 - 1) / (GT * 2));
    if (gy < 1) gy = 1;
    if (gy > 64) gy = 64;
    const dim3 grid((unsigned)m, gy);
    if (vec) hipLaunchKernelGGL(scatter_cols_kernel<2>, grid, dim3(GT), 0, ctx->stream, (const u64*)compact, ld, bs, blk_idx, n_blk_dev, n_blk_cap, (u64*)full, (int)n_full);
    else hipLaunchKernelGGL(scatter_cols_kernel<1>, grid, dim3(GT), 0, ctx->stream, (const u64*)compact, ld, bs, blk_idx, n_blk_dev, n_blk_cap, (u64*)full, (int)n_full);
    COMET_LAUNCH_CHECK(ctx, what);
    return COMET_OK;
}

int comet_truncate_share(comet_ctx* ctx, int party, const uint64_t* z, uint64_t* out, size_t n_elems,
                         int frac_bits) {
    const char* what = "comet_truncate_share";
    COMET_CHECK_CTX(ctx);
    if ((party != 0 && party != 1) || frac_bits < 0 || frac_bits > 62)
        return comet_fail(ctx, COMET_EINVAL, "%s: party must be 0 or 1, 0 <= frac_bits <= 62", what);
    if (n_elems == 0) return COMET_OK;
    if (!z || !out) return comet_fail(ctx, COMET_EINVAL, "%s: null pointer", what);
    if (!comet_aligned16(z) || !comet_aligned16(out))
        return comet_fail(ctx, COMET_EALIGN, "%s: operands must be 16-byte aligned", what);
    comet_device_guard guard(ctx);
    if (!guard.ok) return comet_fail(ctx, COMET_EDEVICE, "%s: cannot select device", what);
    hipLaunchKernelGGL(truncate_kernel, dim3(stream_grid(n_elems)), dim3(GT), 0, ctx->stream,
                       party, (const u64*)z, (u64*)out, n_elems, frac_bits);
    COMET_LAUNCH_CHECK(ctx, what);
    return COMET_OK;
}

}  // extern "C"
