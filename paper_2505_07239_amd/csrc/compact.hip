// Plaintext sparsity distribution -> ordered list of active neuron blocks.
//
// The predictor's mask is plaintext on each server (paper Sec. 4.2), so the
// local first step of Protocols 2 and 3 -- find the columns that are kept -- is
// an ordered stream compaction.  The per-token masks of a batch are OR-ed first
// because one matmul serves the whole batch.
//
// Paths:
//   small (one token row, nb <= 4096): one 256-thread workgroup does everything in
//     one launch; this is the shared FFN mask (a few hundred blocks), latency-bound.
//   large: three wait-free launches.  (1) each lane ORs 16 adjacent flags over
//     the tokens into a 16-bit word and each workgroup stores its popcount;
//     (2) one workgroup scans the workgroup counts; (3) each workgroup scans its
//     own words with wavefront prefix sums and writes the indices through LDS.
//     The mask bytes are read exactly once; passes 2 and 3 touch only the
//     bit-packed words (1/8 of a byte per flag) and the outputs.
//   several token rows: the OR over the tokens is a column-wise reduction of a
//     byte matrix.  Up to 65536 columns the matrix is read as one flat stream of
//     16-byte vectors, whatever the row length and alignment: a lane turns a
//     vector into 16 bits and ORs them into a bitmap of the columns in LDS at the
//     position its flat offset gives (mod nb).  A small mask is finished by the
//     same workgroup; a big one is split over workgroups in contiguous spans, each
//     writes its bitmap, and a merge pass ORs the bitmaps (no atomics in global
//     memory, nothing to clear).  Wider masks of several tokens split the tokens
//     over workgroups per column chunk and merge the same way.
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
// workgroups per column chunk: workgroup (x, y) then writes its words into
// partial array y (stride part_stride 16-bit words), the merge pass ORs the
// partial arrays and the counting is left to pass 1b.
__global__ __launch_bounds__(CT) void compact_pack_kernel(const uint8_t* __restrict__ mask,
                                                          long n_tok, long nb, bool rows_aligned,
                                                          unsigned short* __restrict__ words,
                                                          long part_stride,
                                                          int* __restrict__ counts) {
    __shared__ int sm[CT / 64 + 1];
    const long base = (long)blockIdx.x * CHUNK;
    const bool split = gridDim.y > 1;
    const long tok_per = (n_tok + gridDim.y - 1) / gridDim.y;
    const long t0 = (long)blockIdx.y * tok_per;
    const long t1 = t0 + tok_per < n_tok ? t0 + tok_per : n_tok;
    if (split) words += (long)blockIdx.y * part_stride;
    u32 bits[ITEMS];
    if (t0 >= t1) {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) bits[j] = 0;          // an empty token range still writes its part
    } else if (rows_aligned && base + CHUNK <= nb) {
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
        if (w * FL < nb) words[w] = (unsigned short)bits[j];
    }
    if (split) return;
    int total;
    (void)block_excl_scan(cnt, sm, &total);
    if (threadIdx.x == 0) counts[blockIdx.x] = total;
}

// ---- masks of several tokens and at most FLAT_NB_MAX columns: flat pass ----
constexpr long FLAT_NB_MAX = 65536;
constexpr int FLAT_VEC = CT * ITEMS;              // 16-byte vectors per 256-thread workgroup and trip (16 KB)
constexpr int FLAT_WIDE = 4;                      // the wide workgroup has four times the threads
constexpr long FLAT_ONE_WG_BYTES = 128 * 1024;    // masks up to this size are finished by one workgroup

__device__ __forceinline__ u32 nz_bits16(u32x4 v) {
    return nz_bits4(v.x, 0) | nz_bits4(v.y, 4) | nz_bits4(v.z, 8) | nz_bits4(v.w, 12);
}

// ORs sixteen flag bits, the first of which belongs to column c, into the column bitmap bm (LDS);
// the bits may run over the end of a row (several times when nb < 16).
__device__ __forceinline__ void deposit16(u32* bm, u32 bits, int c, long nb) {
    while (bits) {
        const long room = nb - c;
        const u32 part = room >= 16 ? bits : (bits & ((1u << (int)room) - 1u));
        if (part) {
            const int wi = c >> 5, sh = c & 31;
            atomicOr(bm + wi, part << sh);
            if (sh > 16 && (part >> (32 - sh))) atomicOr(bm + wi + 1, part >> (32 - sh));
        }
        if (room >= 16) break;
        bits >>= (int)room;
        c = 0;
    }
}

// flags of vector v of the flat mask as bits, without the bytes that lie outside [0, total)
__device__ __forceinline__ u32 flat_bits(u32x4 x, long v, int lead, long total) {
    u32 bits = nz_bits16(x);
    const long q0 = 16 * v - lead;                               // flat offset of the first byte
    if (q0 < 0) bits &= 0xffffu << (int)(-q0);
    if (q0 + 16 > total) bits &= (total > q0) ? (0xffffu >> (int)(16 - (total - q0))) : 0u;
    return bits;
}

// ORs the flags of the 16-byte vectors [v0, v1) of the flat mask into the column bitmap bm (LDS,
// zeroed by the caller, one bit per column).  Vectors are counted from the 16-byte boundary at or
// below the mask (lead = bytes between the two), so every load is aligned; bytes outside
// [0, total) of the mask are ignored.  Byte q of the mask is column q mod nb.
// period: the number of vectors after which the columns repeat (nb / gcd(nb, 16)) when that is at
// most the vectors of one workgroup trip, else 0.  With a period the workgroup strides by a multiple of it, every lane
// keeps its columns, ORs the raw vectors in registers and turns them into bits once; without,
// every vector is turned into bits and deposited where its offset says.
template <int T>
__device__ __forceinline__ void flat_or(const uint8_t* __restrict__ mask, long total, long nb, int lead,
                                        int period, long v0, long v1, u32* bm) {
    const u32x4* src = reinterpret_cast<const u32x4*>(mask - lead);
    constexpr int VEC = T * ITEMS;                              // vectors per workgroup trip
    if (period > VEC) period = 0;                               // (a stride of zero would never end)
    const int stride = period ? VEC / period * period : VEC;
    const int step = (int)((16l * stride) % nb);               // column shift from one trip to the next
    // the vectors that hold bytes from outside the mask (-1: none)
    const long nv = (lead + total + 15) >> 4;
    const long edge_lo = lead ? 0 : -1, edge_hi = ((lead + total) & 15) ? nv - 1 : -1;
    long v[ITEMS];
    int col[ITEMS];
    u32x4 acc[ITEMS];
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const int slot = j * T + threadIdx.x;
        v[j] = slot < stride ? v0 + slot : v1;
        // column of the vector's first byte (the lead bytes of vector 0 sit "before column 0")
        col[j] = (int)((16 * (v0 + slot) - lead + nb * 16) % nb);
        acc[j] = u32x4{0, 0, 0, 0};
    }
    // the loads of the next trip are issued before the vectors of this one are worked on
    u32x4 x[ITEMS], xn[ITEMS];
#pragma unroll
    for (int j = 0; j < ITEMS; ++j)
        if (v[j] < v1) x[j] = __builtin_nontemporal_load(src + v[j]);
    for (long trip = v0; trip < v1; trip += stride) {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j)
            if (v[j] + stride < v1) xn[j] = __builtin_nontemporal_load(src + v[j] + stride);
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            if (v[j] < v1) {
                if (period && v[j] != edge_lo && v[j] != edge_hi) acc[j] |= x[j];
                else deposit16(bm, flat_bits(x[j], v[j], lead, total), col[j], nb);
            }
            v[j] += stride;
            if (!period) {
                col[j] += step;
                if (col[j] >= nb) col[j] -= (int)nb;
            }
            x[j] = xn[j];
        }
    }
    if (period) {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) deposit16(bm, nz_bits16(acc[j]), col[j], nb);
    }
}

// One workgroup: whole mask -> index list (nb <= 4096, so one 16-bit word per thread).
__global__ __launch_bounds__(CT) void compact_flat_one_kernel(const uint8_t* __restrict__ mask, long n_tok,
                                                              long nb, int lead, int period,
                                                              int* __restrict__ blk_idx,
                                                              int* __restrict__ n_blk_dev) {
    __shared__ int sm[CT / 64 + 1];
    __shared__ u32 bm[CT * FL / 32 + 1];
    if (threadIdx.x <= CT * FL / 32) bm[threadIdx.x] = 0;
    __syncthreads();
    const long total = n_tok * nb;
    flat_or<CT>(mask, total, nb, lead, period, 0, (lead + total + 15) >> 4, bm);
    __syncthreads();
    const u32 bits = (bm[threadIdx.x >> 1] >> (16 * (threadIdx.x & 1))) & 0xffffu;
    int count;
    const int off = block_excl_scan(__builtin_popcount(bits), sm, &count);
    emit_bits(bits, (int)threadIdx.x * FL, blk_idx + off);
    if (threadIdx.x == 0) *n_blk_dev = count;
}

// Workgroup y: vectors [y * span, (y + 1) * span) of the flat mask -> bitmap y (stride32 words).
template <int T>
__global__ __launch_bounds__(T) void compact_flat_kernel(const uint8_t* __restrict__ mask, long n_tok,
                                                          long nb, int lead, int period, long span,
                                                          u32* __restrict__ parts, long stride32) {
    __shared__ u32 bm[FLAT_NB_MAX / 32 + 1];
    const int nw32 = (int)((nb + 31) >> 5);
    for (int i = threadIdx.x; i <= nw32; i += T) bm[i] = 0;
    __syncthreads();
    const long total = n_tok * nb;
    const long nv = (lead + total + 15) >> 4;
    const long v0 = (long)blockIdx.x * span;
    const long v1 = v0 + span < nv ? v0 + span : nv;
    if (v0 < v1) flat_or<T>(mask, total, nb, lead, period, v0, v1, bm);
    __syncthreads();
    u32* dst = parts + (long)blockIdx.x * stride32;
    for (int i = threadIdx.x; i < nw32; i += T) dst[i] = bm[i];
}

// ORs n_parts bitmaps (stride32 apart) into out[0 .. nw32).  A workgroup owns mw = 2^mw_log2
// adjacent words (16 .. 1024) of every bitmap; its 1024 / mw groups of mw lanes share the
// bitmaps among themselves and meet through wavefront shuffles and LDS.  Many bitmaps: few
// words per workgroup, so that the loop over the bitmaps is short; few bitmaps: many words.
constexpr int MT = 1024;
__global__ __launch_bounds__(MT) void compact_merge_kernel(const u32* __restrict__ parts, long n_parts,
                                                           long stride32, long nw32, int mw_log2,
                                                           u32* __restrict__ out) {
    __shared__ u32 red[MT];
    const int mw = 1 << mw_log2;
    const int wl = threadIdx.x & (mw - 1), q = threadIdx.x >> mw_log2, nq = MT >> mw_log2;
    const long w = (long)blockIdx.x * mw + wl;
    u32 acc = 0;
    if (w < nw32) {
        const u32* src = parts + w;
#pragma unroll 8
        for (long y = q; y < n_parts; y += nq) acc |= src[y * stride32];
    }
    int rows = nq;                                             // partial results per word left in LDS
    if (mw < 64) {
        for (int d = mw; d < 64; d <<= 1) acc |= __shfl_xor(acc, d, 64);
        rows = MT / 64;
        if ((threadIdx.x & 63) < mw) red[(threadIdx.x >> 6) * mw + wl] = acc;
    } else {
        red[threadIdx.x] = acc;
    }
    __syncthreads();
    if ((int)threadIdx.x < mw && w < nw32) {
        for (int r = 1; r < rows; ++r) acc |= red[r * mw + wl];
        out[w] = acc;
    }
}

// index list of a mask of at most 4096 columns from its bit words (one word per thread), or from
// a few bitmaps of them that are ORed on the way (n_parts of them, stride16 words apart)
constexpr long SMALL_MERGE_MAX = 32;
__global__ __launch_bounds__(CT) void compact_small_words_kernel(const unsigned short* __restrict__ words,
                                                                 long n_parts, long stride16, long nb,
                                                                 int* __restrict__ blk_idx,
                                                                 int* __restrict__ n_blk_dev) {
    __shared__ int sm[CT / 64 + 1];
    u32 bits = 0;
    if ((long)threadIdx.x * FL < nb) {
#pragma unroll 8
        for (long y = 0; y < n_parts; ++y) bits |= (u32)words[y * stride16 + threadIdx.x];
    }
    int count;
    const int off = block_excl_scan(__builtin_popcount(bits), sm, &count);
    emit_bits(bits, (int)threadIdx.x * FL, blk_idx + off);
    if (threadIdx.x == 0) *n_blk_dev = count;
}

// pass 1b (after a merge): population count of each workgroup-sized chunk of words
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
constexpr int SCAN_PER = 16;                      // counts per thread per tile (64 KB of LDS)
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

// How a mask of n_tok x nb flags is processed, and the workspace that takes: a pure function of
// the two sizes, so that the size query and the call agree.
enum { PATH_SMALL, PATH_FLAT_ONE, PATH_FLAT, PATH_LARGE };
constexpr long SPLIT_WG = 2048;                   // workgroups aimed at when the tokens are split
struct CompactPlan {
    int path;
    long groups;              // column chunks of CHUNK flags
    long gy;                  // bitmaps to merge (1: none)
    long span;                // PATH_FLAT: 16-byte vectors per workgroup
    long stride32;            // 32-bit words from one bitmap to the next
    size_t words_bytes, counts_bytes, total;
};

inline CompactPlan compact_plan(int64_t n_tok, int64_t nb) {
    CompactPlan p = {};
    p.groups = (nb + CHUNK - 1) / CHUNK;
    p.gy = 1;
    p.words_bytes = ((size_t)p.groups * CT * ITEMS * sizeof(unsigned short) + 255) & ~(size_t)255;
    p.counts_bytes = ((size_t)p.groups * sizeof(int) + 255) & ~(size_t)255;
    p.stride32 = (long)(p.words_bytes / 4);
    const long bytes = n_tok * nb;
    if (n_tok >= 2 && nb >= 1 && nb <= FLAT_NB_MAX) {
        if (nb <= (long)CT * FL && bytes <= FLAT_ONE_WG_BYTES) {
            p.path = PATH_FLAT_ONE;
            return p;                                          // no workspace
        }
        p.path = PATH_FLAT;
        const long nv = (bytes + 15) / 16 + 1;                 // an unaligned mask touches one vector more
        long span_min = (4 * nb > 65536 ? 4 * nb : 65536) / 16;
        long span = (nv + 2047) / 2048;
        if (span < span_min) span = span_min;
        p.span = (span + FLAT_WIDE * FLAT_VEC - 1) / (FLAT_WIDE * FLAT_VEC) * (FLAT_WIDE * FLAT_VEC);
        p.gy = (nv + p.span - 1) / p.span;
    } else if (nb <= (long)CT * FL) {
        p.path = PATH_SMALL;
        return p;                                              // no workspace
    } else {
        p.path = PATH_LARGE;
        if (n_tok >= 2 && p.groups < SPLIT_WG) {
            p.gy = (SPLIT_WG + p.groups - 1) / p.groups;
            if (p.gy > n_tok) p.gy = n_tok;
            if (p.gy > 65535) p.gy = 65535;
        }
    }
    p.total = p.words_bytes + p.counts_bytes + (p.gy > 1 ? (size_t)p.gy * p.words_bytes : 0);
    return p;
}

}  // namespace

size_t comet_compact_workspace_bytes(int64_t n_tok, int64_t nb) {
    if (n_tok < 1 || nb < 0 || nb >= (1ll << 31) - (1ll << 16) || n_tok > (1ll << 40) / (nb > 0 ? nb : 1)) return 0;
    return compact_plan(n_tok, nb).total;
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
    const CompactPlan p = compact_plan(n_tok, nb);
    const size_t need = p.total;
    if (need && (!ws || ws_bytes < need))
        return comet_fail(ctx, COMET_EWORKSPACE, "%s: workspace of %zu bytes required", what, need);
    if (need && (reinterpret_cast<uintptr_t>(ws) & 255u))
        return comet_fail(ctx, COMET_EALIGN, "%s: workspace must be 256-byte aligned", what);
    comet_device_guard guard(ctx);
    if (!guard.ok) return comet_fail(ctx, COMET_EDEVICE, "%s: cannot select device", what);
    // 16-byte loads need every token row to start on a 16-byte boundary
    const bool rows_aligned =
        (reinterpret_cast<uintptr_t>(mask) & 15u) == 0 && (n_tok == 1 || (nb & 15) == 0);
    const int lead = (int)(reinterpret_cast<uintptr_t>(mask) & 15u);
    // vectors of the flat mask after which the columns repeat, if one workgroup trip can hold them
    long per = nb > 0 ? nb : 1;
    for (int d = 0; d < 4 && (per & 1) == 0; ++d) per >>= 1;
    const int period = per <= FLAT_WIDE * FLAT_VEC ? (int)per : 0;
    const bool wide = period > FLAT_VEC;                      // (the plan's spans are whole wide trips)
    if (p.path == PATH_SMALL) {
        hipLaunchKernelGGL(compact_small_kernel, dim3(1), dim3(CT), 0, ctx->stream, mask,
                           (long)n_tok, (long)nb, rows_aligned, blk_idx, n_blk_dev);
        COMET_LAUNCH_CHECK(ctx, what);
        return COMET_OK;
    }
    if (p.path == PATH_FLAT_ONE) {
        hipLaunchKernelGGL(compact_flat_one_kernel, dim3(1), dim3(CT), 0, ctx->stream, mask, (long)n_tok,
                           (long)nb, lead, wide ? 0 : period, blk_idx, n_blk_dev);
        COMET_LAUNCH_CHECK(ctx, what);
        return COMET_OK;
    }
    const int groups = (int)p.groups;
    unsigned short* words = static_cast<unsigned short*>(ws);
    int* counts = reinterpret_cast<int*>(static_cast<char*>(ws) + p.words_bytes);
    u32* parts = reinterpret_cast<u32*>(static_cast<char*>(ws) + p.words_bytes + p.counts_bytes);
    const long nw32 = (nb + 31) / 32;
    if (p.path == PATH_FLAT) {
        // (one bitmap only: it is the word array itself)
        u32* dst = p.gy > 1 ? parts : reinterpret_cast<u32*>(words);
        if (wide)
            hipLaunchKernelGGL(compact_flat_kernel<FLAT_WIDE * CT>, dim3((unsigned)p.gy), dim3(FLAT_WIDE * CT), 0,
                               ctx->stream, mask, (long)n_tok, (long)nb, lead, period, p.span, dst, p.stride32);
        else
            hipLaunchKernelGGL(compact_flat_kernel<CT>, dim3((unsigned)p.gy), dim3(CT), 0, ctx->stream, mask,
                               (long)n_tok, (long)nb, lead, period, p.span, dst, p.stride32);
        COMET_LAUNCH_CHECK(ctx, what);
    } else {
        hipLaunchKernelGGL(compact_pack_kernel, dim3(groups, (unsigned)p.gy), dim3(CT), 0, ctx->stream, mask,
                           (long)n_tok, (long)nb, rows_aligned,
                           p.gy > 1 ? reinterpret_cast<unsigned short*>(parts) : words, 2 * p.stride32, counts);
        COMET_LAUNCH_CHECK(ctx, what);
    }
    const bool small_merge = nb <= (long)CT * FL && p.gy > 1 && p.gy <= SMALL_MERGE_MAX;
    if (p.gy > 1 && !small_merge) {
        int mw_log2 = 4;                                       // 64 lane groups share the bitmaps ...
        while (mw_log2 < 10 && (MT >> (mw_log2 + 1)) >= p.gy) ++mw_log2;   // ... or as many as there are bitmaps
        const long mw = 1l << mw_log2;
        hipLaunchKernelGGL(compact_merge_kernel, dim3((unsigned)((nw32 + mw - 1) / mw)), dim3(MT), 0, ctx->stream,
                           parts, p.gy, p.stride32, nw32, mw_log2, reinterpret_cast<u32*>(words));
        COMET_LAUNCH_CHECK(ctx, what);
    }
    if (nb <= (long)CT * FL) {
        if (small_merge)                                       // the few bitmaps are merged on the way
            hipLaunchKernelGGL(compact_small_words_kernel, dim3(1), dim3(CT), 0, ctx->stream,
                               reinterpret_cast<const unsigned short*>(parts), p.gy, 2 * p.stride32, (long)nb,
                               blk_idx, n_blk_dev);
        else
            hipLaunchKernelGGL(compact_small_words_kernel, dim3(1), dim3(CT), 0, ctx->stream, words, 1l, 0l,
                               (long)nb, blk_idx, n_blk_dev);
        COMET_LAUNCH_CHECK(ctx, what);
        return COMET_OK;
    }
    if (p.gy > 1 || p.path == PATH_FLAT) {
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
