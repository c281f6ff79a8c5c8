// Plaintext sparsity distribution -> ordered list of active neuron blocks.
//
// The predictor's mask is plaintext on each server (paper Sec. 4.2), so the
// local first step of Protocols 2 and 3 -- find the columns that are kept -- is
// an ordered stream compaction.  The per-token masks of a batch are OR-ed first
// because one matmul serves the whole batch.
//
// Two paths:
//   small (nb <= 4096): one 256-thread workgroup does everything in one launch;
//     this is every real FFN mask (a few hundred blocks) and is latency-bound.
//   large: three wait-free launches.  (1) each lane ORs 16 adjacent flags over
//     the tokens into a 16-bit word and each workgroup stores its popcount
//     (with many tokens and few columns the tokens are split over workgroups,
//     which meet through atomic ORs, and a small extra pass counts);
//     (2) one workgroup scans the workgroup counts; (3) each workgroup scans its
//     own words with wavefront prefix sums and writes the indices through LDS.
//     The mask bytes are read exactly once; passes 2 and 3 touch only the
//     bit-packed words (1/8 of a byte per flag) and the outputs.
#include "common.h"

namespace {

constexpr int CT = 256;             // threads per workgroup
constexpr int FL = 16;              // flags per lane
constexpr int ITEMS = 4;            // 16-flag groups per lane in the large path
constexpr int CHUNK = CT * FL * ITEMS;   // flags per workgroup in the large path

typedef u32 u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ u32 nz_bits4(u32 w, int shift) {
    // one bit per non-zero byte of w, placed at bit positions shift .. shift+3, without a compare
    // per byte: the top bit of (byte & 0x7f) + 0x7f, or-ed with the byte itself, is set exactly for
    // a non-zero byte (no carry leaves a byte), and one multiplication moves the four top bits,
    // which sit at bits 0, 8, 16, 24 after the shift, next to each other at bits 21 .. 24
    u32 t = (w & 0x7f7f7f7fu) + 0x7f7f7f7fu;
    t = ((t | w) & 0x80808080u) >> 7;
    return (((t * 0x00204081u) >> 21) & 0xfu) << shift;
}

// OR over tokens of flags [c0, c0+16) -> 16-bit word.  Flags at or beyond nb read as 0.
// rows_aligned: every token row starts on a 16-byte boundary (one 16-byte load per token);
// otherwise the sixteen flags of a token are sixteen independent byte loads (index clamped to
// the row, surplus masked afterwards), so that a token costs one memory round trip, not sixteen.
__device__ __forceinline__ u32 or_flags16(const uint8_t* __restrict__ mask, long n_tok, long nb,
                                          long c0, bool rows_aligned) {
    if (c0 >= nb) return 0;
    if (rows_aligned && c0 + FL <= nb) {
        u32x4 acc = {0, 0, 0, 0};
        for (long t = 0; t < n_tok; ++t)
            acc |= __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(mask + t * nb + c0));
        return nz_bits4(acc.x, 0) | nz_bits4(acc.y, 4) | nz_bits4(acc.z, 8) | nz_bits4(acc.w, 12);
    }
    const int lim = (int)((nb - c0) < FL ? (nb - c0) : FL);
    u32 any[FL];
#pragma unroll
    for (int j = 0; j < FL; ++j) any[j] = 0;
    const uint8_t* src = mask + c0;
    for (long t = 0; t < n_tok; ++t, src += nb) {
#pragma unroll
        for (int j = 0; j < FL; ++j) any[j] |= src[j < lim ? j : 0];
    }
    u32 bits = 0;
#pragma unroll
    for (int j = 0; j < FL; ++j) bits |= ((j < lim && any[j]) ? 1u : 0u) << j;
    return bits;
}

// Exclusive prefix sum of one value per lane over the 64-lane wavefront.
__device__ __forceinline__ int wave_excl_scan(int v, int lane, int* total) {
    int inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(inc, d, 64);
        if (lane >= d) inc += o;
    }
    *total = __shfl(inc, 63, 64);
    return inc - v;
}

// Exclusive prefix over the workgroup (CT threads).  sm: CT/64 + 1 ints.
__device__ __forceinline__ int block_excl_scan(int v, int* sm, int* block_total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int wtot;
    const int ex = wave_excl_scan(v, lane, &wtot);
    if (lane == 0) sm[wave] = wtot;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < CT / 64; ++w) {
        const int x = sm[w];
        if (w < wave) base += x;
        tot += x;
    }
    __syncthreads();
    *block_total = tot;
    return base + ex;
}

__device__ __forceinline__ void emit_bits(u32 bits, int first_block, int* __restrict__ out) {
    while (bits) {
        const int j = __builtin_ctz(bits);
        *out++ = first_block + j;
        bits &= bits - 1;
    }
}

__global__ __launch_bounds__(CT) void compact_small_kernel(const uint8_t* __restrict__ mask,
                                                           long n_tok, long nb, bool rows_aligned,
                                                           int* __restrict__ blk_idx,
                                                           int* __restrict__ n_blk_dev) {
    __shared__ int sm[CT / 64 + 1];
    const long c0 = (long)threadIdx.x * FL;
    const u32 bits = or_flags16(mask, n_tok, nb, c0, rows_aligned);
    int total;
    const int off = block_excl_scan(__builtin_popcount(bits), sm, &total);
    emit_bits(bits, (int)c0, blk_idx + off);
    if (threadIdx.x == 0) *n_blk_dev = total;
}

// pass 1: bit-pack and count.  gridDim.y > 1 splits the tokens over several
// workgroups per column chunk; their partial ORs meet in the (pre-cleared)
// words through 32-bit atomic ORs and the counting is left to pass 1b.
__global__ __launch_bounds__(CT) void compact_pack_kernel(const uint8_t* __restrict__ mask,
                                                          long n_tok, long nb, bool rows_aligned,
                                                          unsigned short* __restrict__ words,
                                                          int* __restrict__ counts) {
    __shared__ int sm[CT / 64 + 1];
    const long base = (long)blockIdx.x * CHUNK;
    const bool split = gridDim.y > 1;
    const long tok_per = (n_tok + gridDim.y - 1) / gridDim.y;
    const long t0 = (long)blockIdx.y * tok_per;
    const long t1 = t0 + tok_per < n_tok ? t0 + tok_per : n_tok;
    if (t0 >= t1) return;
    u32 bits[ITEMS];
    if (rows_aligned && base + CHUNK <= nb) {
        // whole chunk inside the mask: the 16-byte loads of a token row are all in flight at once
        u32x4 acc[ITEMS];
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) acc[j] = u32x4{0, 0, 0, 0};
        const uint8_t* src = mask + t0 * nb + base + (long)threadIdx.x * FL;
        for (long t = t0; t < t1; ++t, src += nb) {
#pragma unroll
            for (int j = 0; j < ITEMS; ++j)
                acc[j] |= __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + (long)j * CT * FL));
        }
#pragma unroll
        for (int j = 0; j < ITEMS; ++j)
            bits[j] = nz_bits4(acc[j].x, 0) | nz_bits4(acc[j].y, 4) | nz_bits4(acc[j].z, 8) | nz_bits4(acc[j].w, 12);
    } else {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j)
            bits[j] = or_flags16(mask + t0 * nb, t1 - t0, nb, base + ((long)j * CT + threadIdx.x) * FL,
                                 rows_aligned);
    }
    int cnt = 0;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        cnt += __builtin_popcount(bits[j]);
        const long w = (base / FL) + (long)j * CT + threadIdx.x;
        if (w * FL < nb) {
            if (split) {
                if (bits[j]) atomicOr(reinterpret_cast<u32*>(words) + (w >> 1), bits[j] << (16 * (int)(w & 1)));
            } else {
                words[w] = (unsigned short)bits[j];
            }
        }
    }
    if (split) return;
    int total;
    (void)block_excl_scan(cnt, sm, &total);
    if (threadIdx.x == 0) counts[blockIdx.x] = total;
}

// clears the words before a token-split pass 1 (a fill kernel rather than a memset
// so that the whole call can be captured in a HIP graph)
__global__ __launch_bounds__(CT) void compact_clear_kernel(u32* __restrict__ words32, long n) {
    for (long i = (long)blockIdx.x * CT + threadIdx.x; i < n; i += (long)gridDim.x * CT) words32[i] = 0u;
}

// pass 1b (token-split only): population count of each workgroup-sized chunk of words
__global__ __launch_bounds__(CT) void compact_count_kernel(const unsigned short* __restrict__ words,
                                                           long nb, int* __restrict__ counts) {
    __shared__ int sm[CT / 64 + 1];
    const long w0 = (long)blockIdx.x * (CHUNK / FL) + (long)threadIdx.x * ITEMS;
    int cnt = 0;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j)
        if ((w0 + j) * FL < nb) cnt += __builtin_popcount((u32)words[w0 + j]);
    int total;
    (void)block_excl_scan(cnt, sm, &total);
    if (threadIdx.x == 0) counts[blockIdx.x] = total;
}

// pass 2: exclusive scan of the workgroup counts, in place; writes the grand total.
// One workgroup; the counts pass through LDS in tiles so that global accesses are
// coalesced and each thread scans a contiguous run out of LDS.
constexpr int ST = 1024;
constexpr int SCAN_PER = 8;                       // counts per thread per tile
__global__ __launch_bounds__(ST) void compact_scan_kernel(int* __restrict__ counts, int n,
                                                          int* __restrict__ n_blk_dev) {
    __shared__ int tile[ST * SCAN_PER];
    __shared__ int sm[ST / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int carry = 0;
    for (int base = 0; base < n; base += ST * SCAN_PER) {
#pragma unroll
        for (int j = 0; j < SCAN_PER; ++j) {
            const int i = base + j * ST + threadIdx.x;
            tile[j * ST + threadIdx.x] = i < n ? counts[i] : 0;
        }
        __syncthreads();
        int v[SCAN_PER], sum = 0;
#pragma unroll
        for (int j = 0; j < SCAN_PER; ++j) { v[j] = tile[threadIdx.x * SCAN_PER + j]; sum += v[j]; }
        int wtot;
        const int ex = wave_excl_scan(sum, lane, &wtot);
        if (lane == 0) sm[wave] = wtot;
        __syncthreads();
        int wbase = 0, tot = 0;
#pragma unroll
        for (int w = 0; w < ST / 64; ++w) {
            const int x = sm[w];
            if (w < wave) wbase += x;
            tot += x;
        }
        int run = carry + wbase + ex;
#pragma unroll
        for (int j = 0; j < SCAN_PER; ++j) { tile[threadIdx.x * SCAN_PER + j] = run; run += v[j]; }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < SCAN_PER; ++j) {
            const int i = base + j * ST + threadIdx.x;
            if (i < n) counts[i] = tile[j * ST + threadIdx.x];
        }
        carry += tot;
        __syncthreads();
    }
    if (threadIdx.x == 0) *n_blk_dev = carry;
}

// pass 3: each lane owns 64 consecutive flags (four 16-bit words, one 8-byte load), one
// workgroup scan gives the positions.  When the workgroup's indices fit the LDS stage they are
// scattered there and copied out as one contiguous run with 16-byte stores: the run is placed
// in the stage at the same position inside a 16-byte quad as in the output, so that aligned quads of the
// stage are aligned quads of the output, and only the ragged ends are written one by one.
// A denser chunk writes its indices directly.
constexpr int STAGE_CAP = 4092;
__global__ __launch_bounds__(CT) void compact_emit_kernel(const unsigned short* __restrict__ words,
                                                          const int* __restrict__ offsets, long nb,
                                                          int* __restrict__ blk_idx) {
    __shared__ int sm[CT / 64 + 1];
    __shared__ __align__(16) int stage[STAGE_CAP + 4];
    const long w0 = (long)blockIdx.x * (CHUNK / FL) + (long)threadIdx.x * ITEMS;
    static_assert(ITEMS == 4, "one 8-byte load per lane");
    // the word array is padded to whole workgroup chunks, so the load is always in range
    const unsigned long long packed = *reinterpret_cast<const unsigned long long*>(words + w0);
    u32 bits[ITEMS];
    int cnt = 0;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        bits[j] = ((w0 + j) * FL < nb) ? (u32)((packed >> (16 * j)) & 0xffffu) : 0u;
        cnt += __builtin_popcount(bits[j]);
    }
    int total;
    int pos = block_excl_scan(cnt, sm, &total);
    const long off = offsets[blockIdx.x];
    int* out = blk_idx + off;
    if (total <= STAGE_CAP) {
        const int ph = (int)((reinterpret_cast<uintptr_t>(out) >> 2) & 3);   // position inside a 16-byte quad
        // the lane's 64 consecutive flags as two 32-bit halves: fewer, longer loops diverge less
        // between the lanes than one loop per 16-bit word
        const u32 lo = bits[0] | (bits[1] << 16), hi = bits[2] | (bits[3] << 16);
        emit_bits(lo, (int)(w0 * FL), stage + ph + pos);
        emit_bits(hi, (int)(w0 * FL) + 32, stage + ph + pos + __builtin_popcount(lo));
        __syncthreads();
        // stage[ph .. ph + total) -> out[0 .. total); quads q cover stage[4q .. 4q + 4)
        const int end = ph + total;
        const int q0 = ph ? 1 : 0, q1 = end >> 2;            // whole quads inside the run
        typedef int int4v __attribute__((ext_vector_type(4)));
        int4v* out4 = reinterpret_cast<int4v*>(out - ph);     // 16-byte aligned by construction
        const int4v* st4 = reinterpret_cast<const int4v*>(stage);
        for (int q = q0 + threadIdx.x; q < q1; q += CT) __builtin_nontemporal_store(st4[q], out4 + q);
        // ragged head (before the first whole quad) and tail (after the last)
        const int head_end = q0 * 4 < end ? q0 * 4 : end;
        if ((int)threadIdx.x >= ph && (int)threadIdx.x < head_end) out[threadIdx.x - ph] = stage[threadIdx.x];
        const int tail0 = q1 * 4 > head_end ? q1 * 4 : head_end;
        const int ti = tail0 + (int)threadIdx.x;
        if (ti < end) out[ti - ph] = stage[ti];
    } else {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            emit_bits(bits[j], (int)((w0 + j) * FL), out + pos);
            pos += __builtin_popcount(bits[j]);
        }
    }
}

inline size_t compact_ws_bytes(int64_t nb) {
    if (nb <= (int64_t)CT * FL) return 0;
    const int64_t groups = (nb + CHUNK - 1) / CHUNK;
    const size_t words = ((size_t)groups * CT * ITEMS * sizeof(unsigned short) + 255) & ~(size_t)255;
    return words + (size_t)groups * sizeof(int);
}

}  // namespace

size_t comet_compact_workspace_bytes(int64_t n_tok, int64_t nb) {
    if (n_tok < 1 || nb < 0 || nb >= (1ll << 31) - (1ll << 16)) return 0;
    return compact_ws_bytes(nb);
}

extern "C" int comet_compact_mask(comet_ctx* ctx, const uint8_t* mask, int64_t n_tok, int64_t nb,
                                  int32_t* blk_idx, int32_t* n_blk_dev, void* ws, size_t ws_bytes) {
    const char* what = "comet_compact_mask";
    COMET_CHECK_CTX(ctx);
    if (!mask || !blk_idx || !n_blk_dev) return comet_fail(ctx, COMET_EINVAL, "%s: null pointer", what);
    if (n_tok < 1 || nb < 0) return comet_fail(ctx, COMET_EINVAL, "%s: need n_tok >= 1, nb >= 0", what);
    if (nb >= (1ll << 31) - (1ll << 16) || n_tok > (1ll << 40) / (nb > 0 ? nb : 1))
        return comet_fail(ctx, COMET_ECAP, "%s: mask too large", what);
    if ((reinterpret_cast<uintptr_t>(blk_idx) & 3u) || (reinterpret_cast<uintptr_t>(n_blk_dev) & 3u))
        return comet_fail(ctx, COMET_EALIGN, "%s: int32 outputs must be 4-byte aligned", what);
    const size_t need = compact_ws_bytes(nb);
    if (need && (!ws || ws_bytes < need))
        return comet_fail(ctx, COMET_EWORKSPACE, "%s: workspace of %zu bytes required", what, need);
    if (need && (reinterpret_cast<uintptr_t>(ws) & 255u))
        return comet_fail(ctx, COMET_EALIGN, "%s: workspace must be 256-byte aligned", what);
    comet_device_guard guard(ctx);
    if (!guard.ok) return comet_fail(ctx, COMET_EDEVICE, "%s: cannot select device", what);
    // 16-byte loads need every token row to start on a 16-byte boundary
    const bool rows_aligned =
        (reinterpret_cast<uintptr_t>(mask) & 15u) == 0 && (n_tok == 1 || (nb & 15) == 0);
    if (!need) {
        hipLaunchKernelGGL(compact_small_kernel, dim3(1), dim3(CT), 0, ctx->stream, mask,
                           (long)n_tok, (long)nb, rows_aligned, blk_idx, n_blk_dev);
        COMET_LAUNCH_CHECK(ctx, what);
        return COMET_OK;
    }
    const int groups = (int)((nb + CHUNK - 1) / CHUNK);
    unsigned short* words = static_cast<unsigned short*>(ws);
    const size_t words_bytes = ((size_t)groups * CT * ITEMS * sizeof(unsigned short) + 255) & ~(size_t)255;
    int* counts = reinterpret_cast<int*>(static_cast<char*>(ws) + words_bytes);
    // enough workgroups to fill the chip: split the tokens when the column chunks alone are too few
    long gy = 1;
    if (n_tok > 1 && groups < 8 * ctx->num_cu) {
        gy = (8l * ctx->num_cu + groups - 1) / groups;
        if (gy > n_tok) gy = n_tok;
        if (gy > 65535) gy = 65535;
    }
    if (gy > 1) {
        const long n32 = (long)(words_bytes / 4);
        hipLaunchKernelGGL(compact_clear_kernel, dim3((unsigned)((n32 + CT - 1) / CT)), dim3(CT), 0,
                           ctx->stream, reinterpret_cast<u32*>(words), n32);
        COMET_LAUNCH_CHECK(ctx, what);
    }
    hipLaunchKernelGGL(compact_pack_kernel, dim3(groups, (unsigned)gy), dim3(CT), 0, ctx->stream, mask,
                       (long)n_tok, (long)nb, rows_aligned, words, counts);
    COMET_LAUNCH_CHECK(ctx, what);
    if (gy > 1) {
        hipLaunchKernelGGL(compact_count_kernel, dim3(groups), dim3(CT), 0, ctx->stream, words, (long)nb,
                           counts);
        COMET_LAUNCH_CHECK(ctx, what);
    }
    hipLaunchKernelGGL(compact_scan_kernel, dim3(1), dim3(ST), 0, ctx->stream, counts, groups,
                       n_blk_dev);
    COMET_LAUNCH_CHECK(ctx, what);
    hipLaunchKernelGGL(compact_emit_kernel, dim3(groups), dim3(CT), 0, ctx->stream, words, counts,
                       (long)nb, blk_idx);
    COMET_LAUNCH_CHECK(ctx, what);
    return COMET_OK;
}
