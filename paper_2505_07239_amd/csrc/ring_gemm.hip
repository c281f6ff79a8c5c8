// One party's output share of the Beaver-triple matrix product (paper Eq. 1 in
// matrix form, invoked on the indexed sub-matrices of Protocols 2 and 3):
//
//     [Z]_i = [C]_i + E [B]_i + [A]_i F + party * E F          (mod 2^64)
//
// Formulation used here
//   * E F + [A]_i F = (E + [A]_i) F, so each party needs exactly two products,
//     and they share one accumulator when the contraction axes are stacked:
//         [Z]_i = [C]_i + [ E | A' ] . [ B_i ; F ],   A' = A_i + party * E.
//   * A 64-bit ring product is carried out on the int8 matrix cores.  Every
//     operand word x is rewritten as eight SIGNED base-256 digits,
//         x = sum_t d_t 2^(8t)  (mod 2^64),  d_t in [-128, 127],
//     which costs two 64-bit ALU operations: the bytes of
//     (x + 0x0080808080808080) ^ 0x0080808080808080 are exactly those digits
//     (adding 128 to a byte and flipping its top bit subtracts 128 again, with
//     the borrow already propagated by the addition; the top digit may be
//     read signed because 2^64 = 0).  Then
//         x y = sum_{t+u <= 7} d_t e_u 2^(8(t+u))      (mod 2^64),
//     36 digit products instead of 64, each an int8 x int8 -> int32 GEMM.
//     All digit pairs of equal weight s = t + u share one int32 accumulator:
//     eight accumulator planes per output element, recombined at the end as
//     sum_s sext64(S_s) << 8s.  |d e| <= 2^14 and a plane receives at most
//     8 * 32 products per contraction step, so a plane cannot overflow within
//     MAX_SEG = 256 steps; longer contractions are cut into segments.
//   * Addition mod 2^64 is associative and commutative, so partial sums may be
//     formed in any order and by any number of workgroups: segments of the
//     stacked contraction are dealt out evenly over a fixed, chip-sized grid
//     (a stream-K split) and every segment ends with 64-bit atomic adds onto
//     Z, which starts out as [C]_i.  The result is bit-exact whatever the split.
//
// Data flow
//   xpack kernel : E, A_i  -> digit planes of [E | A'] in the workspace, laid
//                  out so that a tile is a linear copy into LDS (small operand).
//   gemm kernel  : weight-side words are loaded once as uint64 (with the block
//                  gather folded into the addressing), split into digits and
//                  byte-transposed in registers, staged through LDS, and fed
//                  to v_mfma_i32_32x32x32_i8.  The weight matrices are the
//                  large operands; they are never re-written to memory.
#include "common.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef u32 u32x4 __attribute__((ext_vector_type(4)));

constexpr int KSTEP = 32;       // ring words contracted per matrix instruction
constexpr int MAX_SEG = 256;    // contraction steps an int32 plane can absorb
constexpr int GT = 256;         // threads per workgroup (4 wavefronts)
constexpr u64 DIGIT_BIAS = 0x0080808080808080ull;

constexpr int KIND_SOMM = 0;
constexpr int KIND_SIMM = 1;

struct GemmParams {
    int kind, party;
    int m;          // rows of X / Z
    int kc_cap;     // contraction length bound: SOMM k, SIMM n_blk_cap * bs
    int n_cap;      // output width bound: SOMM n_blk_cap * bs, SIMM n
    int bs, n_blk_cap;
    int full_extent; // length of the axis blk_idx refers to (neurons)
    const int* blk_idx;
    const int* n_blk_dev;
    // X side
    const u64* E;  long lde;
    const u64* A;  long lda;  int a_full;
    // W side
    const u64* B;  long ldb;  int b_full;
    const u64* F;  long ldf;
    const u64* C;
    u64* Z;        long ldz;
    // packed digit planes of [E | A']
    unsigned char* xp;
    int mpad;       // rows of xp, multiple of 128
    int ks_cap;     // contraction steps per half, ceil(kc_cap / 32)
};

__device__ __forceinline__ int n_blocks(const GemmParams& p) {
    int nb = p.n_blk_cap;
    if (p.n_blk_dev) {
        const int d = *p.n_blk_dev;
        nb = d < 0 ? 0 : (d < nb ? d : nb);
    }
    return nb;
}

// Start of block `blk` on the indexed axis, or -1 when the id does not fit the
// axis (such ids contribute zeros instead of faulting).
__device__ __forceinline__ long block_start(const GemmParams& p, int blk) {
    const long s = (long)p.blk_idx[blk] * p.bs;
    return (s < 0 || s + p.bs > p.full_extent) ? -1 : s;
}

__device__ __forceinline__ u64 to_digits(u64 x) { return (x + DIGIT_BIAS) ^ DIGIT_BIAS; }

// 4x4 byte transpose: in a0..a3 byte b of word j  ->  out word b, byte j
__device__ __forceinline__ void transpose4(u32 a0, u32 a1, u32 a2, u32 a3, u32& o0, u32& o1,
                                           u32& o2, u32& o3) {
    const u32 p01l = __builtin_amdgcn_perm(a1, a0, 0x05010400u);
    const u32 p01h = __builtin_amdgcn_perm(a1, a0, 0x07030602u);
    const u32 p23l = __builtin_amdgcn_perm(a3, a2, 0x05010400u);
    const u32 p23h = __builtin_amdgcn_perm(a3, a2, 0x07030602u);
    o0 = __builtin_amdgcn_perm(p23l, p01l, 0x05040100u);
    o1 = __builtin_amdgcn_perm(p23l, p01l, 0x07060302u);
    o2 = __builtin_amdgcn_perm(p23h, p01h, 0x05040100u);
    o3 = __builtin_amdgcn_perm(p23h, p01h, 0x07060302u);
}

// Eight consecutive-k words (already in digit form) -> for each digit t one
// 8-byte group holding digit t of k0..k7.
__device__ __forceinline__ void digits_to_planes(const u64 (&v)[8], u64 (&plane)[8]) {
    u32 lo[8], hi[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { lo[j] = (u32)v[j]; hi[j] = (u32)(v[j] >> 32); }
    u32 a[8], b[8];   // a: k0..3, b: k4..7, index = digit
    transpose4(lo[0], lo[1], lo[2], lo[3], a[0], a[1], a[2], a[3]);
    transpose4(hi[0], hi[1], hi[2], hi[3], a[4], a[5], a[6], a[7]);
    transpose4(lo[4], lo[5], lo[6], lo[7], b[0], b[1], b[2], b[3]);
    transpose4(hi[4], hi[5], hi[6], hi[7], b[4], b[5], b[6], b[7]);
#pragma unroll
    for (int t = 0; t < 8; ++t) plane[t] = (u64)a[t] | ((u64)b[t] << 32);
}

// Packed layout of [E | A'] (bytes): group (half h, step s, digit t, octet q)
// is a run of mpad rows x 8 bytes; the 8 bytes are digit t of words
// k = 32 s + 8 q + 0..7 of that row.  Groups are ordered (h, s, t, q).
__device__ __host__ __forceinline__ size_t xp_group(int h, int s, int t, int q, int ks_cap) {
    return ((((size_t)h * ks_cap + s) * 8 + t) * 4 + q);
}

// ---------------------------------------------------------------------------
// xpack: digit planes of the stacked activation-side operand, and Z := C
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(GT) void xpack_kernel(GemmParams p) {
    const int nblk = n_blocks(p);
    const int kc = p.kind == KIND_SOMM ? p.kc_cap : nblk * p.bs;
    const int row = blockIdx.y * 128 + threadIdx.x;    // < mpad by construction (128 threads)
    const int oct = blockIdx.x;                        // octet index over the half: 0 .. ks_cap*4
    const int h = blockIdx.z;                          // 0: E, 1: A'
    const int k0 = oct * 8;
    u64 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = 0;
    if (row < p.m && k0 < kc) {
        int blk = 0, off = 0;
        if (h == 1 && p.a_full) { blk = k0 / p.bs; off = k0 - blk * p.bs; }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int k = k0 + j;
            if (k < kc) {
                const u64 e = p.E[(size_t)row * p.lde + k];
                u64 x = e;
                if (h == 1) {
                    long col = k;
                    if (p.a_full) {
                        while (off >= p.bs) { off -= p.bs; ++blk; }
                        const long st = block_start(p, blk);
                        col = st < 0 ? -1 : st + off;
                        ++off;
                    }
                    const u64 a = col < 0 ? 0ull : p.A[(size_t)row * p.lda + col];
                    x = a + (p.party ? e : 0ull);
                }
                v[j] = to_digits(x);
            }
        }
    }
    u64 plane[8];
    digits_to_planes(v, plane);
    const int s = oct >> 2, q = oct & 3;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        u64* dst = reinterpret_cast<u64*>(p.xp) + xp_group(h, s, t, q, p.ks_cap) * p.mpad + row;
        *dst = plane[t];
    }
}

__global__ __launch_bounds__(GT) void init_z_kernel(GemmParams p) {
    const int nblk = n_blocks(p);
    const int n_eff = p.kind == KIND_SOMM ? nblk * p.bs : p.n_cap;
    const int r = blockIdx.y;
    for (int c = blockIdx.x * GT + threadIdx.x; c < n_eff; c += gridDim.x * GT)
        p.Z[(size_t)r * p.ldz + c] = p.C[(size_t)r * p.ldz + c];
}

// ---------------------------------------------------------------------------
// gemm
// ---------------------------------------------------------------------------
template <int WAVES_M, int WAVES_N, int WM, int WN>
struct Tile {
    static constexpr int BM = 32 * WM * WAVES_M;
    static constexpr int BN = 32 * WN * WAVES_N;
    static constexpr int XBYTES = BM * 256;          // 8 digits x 4 octets x BM rows x 8 bytes
    static constexpr int WBYTES = BN * 256;
    static constexpr int STAGE = XBYTES + WBYTES;
    static constexpr int SMEM = 2 * STAGE;
    static constexpr int XVEC = XBYTES / 16 / GT;    // 16-byte vectors per thread per stage
    static constexpr int WTASK = BN * 4 / GT;        // (column, octet) tasks per thread per stage
    static_assert(WAVES_M * WAVES_N * 64 == GT, "four wavefronts per workgroup");
    static_assert(XVEC >= 1 && WTASK >= 1, "tile too small for the loader");
};

// Weight-side and activation-side loads of one contraction step, staged in
// registers.  Every load is unconditional: out-of-range rows and columns are
// clamped to a valid address instead of being predicated off.  That is exact
// because (a) a weight column only feeds its own output column, and columns at
// or beyond the kept width are never written back, and (b) the packed
// activation planes hold zeros beyond the contraction length, so whatever the
// weight side reads there is multiplied by zero.
template <class T, int KIND>
struct Loader {
    const u64* wb[T::WTASK];   // B_i at (row 0, this task's column), gather applied (SOMM)
    const u64* wf[T::WTASK];   // F   at (row 0, this task's column)
    bool bzero[T::WTASK];      // SOMM: the column's block id does not fit B_i -> contributes zeros
    const unsigned char* xsrc; // this thread's first 16-byte unit of step (h = 0, s = 0)
    u32x4 xr[T::XVEC];
    u64 wr[T::WTASK][8];

    static constexpr int XROWS2 = T::BM / 2;                 // 16-byte units per group
    static constexpr int XGRP_PER_PASS = GT / XROWS2;        // groups covered by one pass of the block

    __device__ __forceinline__ void setup(const GemmParams& p, int tm, int tn, int n_eff) {
#pragma unroll
        for (int j = 0; j < T::WTASK; ++j) {
            const int id = threadIdx.x + GT * j;
            int col = tn * T::BN + id % T::BN;
            col = col < n_eff ? col : n_eff - 1;
            long bcol = col;
            bzero[j] = false;
            if (KIND == KIND_SOMM && p.b_full) {
                const int blk = col / p.bs;
                const long st = block_start(p, blk);
                bzero[j] = st < 0;
                bcol = st < 0 ? 0 : st + (col - blk * p.bs);
            }
            wb[j] = p.B + bcol;
            wf[j] = p.F + col;
        }
        const int grp = threadIdx.x / XROWS2, within = threadIdx.x % XROWS2;
        xsrc = p.xp + ((size_t)grp * p.mpad + (size_t)tm * T::BM) * 8 + within * 16;
    }

    __device__ __forceinline__ void load(const GemmParams& p, int ks, int KS, int kc) {
        const int h = ks >= KS ? 1 : 0;
        const int s = ks - h * KS;
        const unsigned char* xs = xsrc + (size_t)(h * p.ks_cap + s) * 32 * p.mpad * 8;
        const size_t xstride = (size_t)XGRP_PER_PASS * p.mpad * 8;
#pragma unroll
        for (int j = 0; j < T::XVEC; ++j)
            xr[j] = *reinterpret_cast<const u32x4*>(xs + j * xstride);

#pragma unroll
        for (int j = 0; j < T::WTASK; ++j) {
            // octet index is the same for all lanes of a wavefront
            const int oct = __builtin_amdgcn_readfirstlane((int)((threadIdx.x + GT * j) / T::BN));
            const int k0 = s * KSTEP + oct * 8;
            const u64* src = h ? wf[j] : wb[j];
            const long ld = h ? p.ldf : p.ldb;
            if (KIND == KIND_SIMM && !h && p.b_full) {
                // B_i rows are the kept neurons: compact row -> row of the full matrix
                if ((p.bs & 7) == 0) {
                    int kk = k0 <= kc - 8 ? k0 : kc - 8;          // kc is a positive multiple of 8 here
                    const int blk = kk / p.bs;
                    const long st = block_start(p, blk);
                    const long row0 = st < 0 ? 0 : st + (kk - blk * p.bs);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const u64 v = src[(row0 + e) * ld];
                        wr[j][e] = st < 0 ? 0ull : v;
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int kk = (k0 + e) < kc ? (k0 + e) : kc - 1;
                        const int blk = kk / p.bs;
                        const long st = block_start(p, blk);
                        const long row = st < 0 ? 0 : st + (kk - blk * p.bs);
                        const u64 v = src[row * ld];
                        wr[j][e] = st < 0 ? 0ull : v;
                    }
                }
            } else if (k0 + 8 <= kc) {
#pragma unroll
                for (int e = 0; e < 8; ++e) wr[j][e] = src[(long)(k0 + e) * ld];
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int kk = (k0 + e) < kc ? (k0 + e) : kc - 1;
                    wr[j][e] = src[(long)kk * ld];
                }
            }
            if (KIND == KIND_SOMM && !h && bzero[j]) {
#pragma unroll
                for (int e = 0; e < 8; ++e) wr[j][e] = 0;
            }
        }
    }

    // digits, byte transpose, and store of the staged registers into an LDS stage
    __device__ __forceinline__ void store(unsigned char* stage) {
#pragma unroll
        for (int j = 0; j < T::XVEC; ++j)
            *reinterpret_cast<u32x4*>(stage + (threadIdx.x + GT * j) * 16) = xr[j];
        unsigned char* ws = stage + T::XBYTES;
#pragma unroll
        for (int j = 0; j < T::WTASK; ++j) {
            u64 v[8], plane[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = to_digits(wr[j][e]);
            digits_to_planes(v, plane);
            const int id = threadIdx.x + GT * j;
            const int c = id % T::BN, oct = id / T::BN;
#pragma unroll
            for (int t = 0; t < 8; ++t)
                *reinterpret_cast<u64*>(ws + ((size_t)(t * 4 + oct) * T::BN + c) * 8) = plane[t];
        }
    }
};

__device__ __forceinline__ v4i lds_frag(const unsigned char* base, int stride_bytes) {
    const u64 x0 = *reinterpret_cast<const u64*>(base);
    const u64 x1 = *reinterpret_cast<const u64*>(base + stride_bytes);
    return v4i{(int)(u32)x0, (int)(u32)(x0 >> 32), (int)(u32)x1, (int)(u32)(x1 >> 32)};
}

template <int WAVES_M, int WAVES_N, int WM, int WN, int KIND>
__global__ __launch_bounds__(GT) void ring_gemm_kernel(GemmParams p) {
    using T = Tile<WAVES_M, WAVES_N, WM, WN>;
    extern __shared__ __align__(16) unsigned char smem[];

    const int nblk = n_blocks(p);
    const int n_eff = KIND == KIND_SOMM ? nblk * p.bs : p.n_cap;
    const int kc = KIND == KIND_SOMM ? p.kc_cap : nblk * p.bs;
    const int KS = (kc + KSTEP - 1) / KSTEP;
    const int KT = 2 * KS;
    const int tiles_m = (p.m + T::BM - 1) / T::BM;
    const int tiles_n = (n_eff + T::BN - 1) / T::BN;
    const long units = (long)tiles_m * tiles_n * KT;
    if (units == 0) return;

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD one
    // contiguous range of work so that tiles sharing weight columns meet in
    // the same L2.
    const int G = gridDim.x;
    int b = blockIdx.x;
    if ((G & 7) == 0) b = (b & 7) * (G >> 3) + (b >> 3);
    long u = units * b / G;
    const long u_end = units * (b + 1) / G;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave % WAVES_M, wn = wave / WAVES_M;
    const int g = lane >> 5, r = lane & 31;
    // this lane's fragment offsets inside a stage (digit 0)
    const int a_off = ((2 * g) * T::BM + wm * WM * 32 + r) * 8;
    const int b_off = T::XBYTES + ((2 * g) * T::BN + wn * WN * 32 + r) * 8;

    Loader<T, KIND> ld;

    while (u < u_end) {
        const int tile = (int)(u / KT);
        const int ks0 = (int)(u - (long)tile * KT);
        long len = KT - ks0;
        if (len > u_end - u) len = u_end - u;
        if (len > MAX_SEG) len = MAX_SEG;
        const int ks1 = ks0 + (int)len;
        const int tm = tile % tiles_m, tn = tile / tiles_m;

        ld.setup(p, tm, tn, n_eff);
        v16i acc[WM][WN][8];
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int j = 0; j < WN; ++j)
#pragma unroll
                for (int s = 0; s < 8; ++s)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[i][j][s][e] = 0;

        ld.load(p, ks0, KS, kc);
        ld.store(smem);
        __syncthreads();
        int cur = 0;
        for (int ks = ks0; ks < ks1; ++ks) {
            const bool more = ks + 1 < ks1;
            if (more) ld.load(p, ks + 1, KS, kc);

            const unsigned char* st = smem + cur * T::STAGE;
            v4i bf[WN][8];
#pragma unroll
            for (int j = 0; j < WN; ++j)
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    bf[j][t] = lds_frag(st + b_off + (t * 4 * T::BN + j * 32) * 8, T::BN * 8);
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                v4i a[WM];
#pragma unroll
                for (int i = 0; i < WM; ++i)
                    a[i] = lds_frag(st + a_off + (t * 4 * T::BM + i * 32) * 8, T::BM * 8);
#pragma unroll
                for (int uu = 0; uu < 8 - t; ++uu)
#pragma unroll
                    for (int i = 0; i < WM; ++i)
#pragma unroll
                        for (int j = 0; j < WN; ++j)
                            acc[i][j][t + uu] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                                a[i], bf[j][uu], acc[i][j][t + uu], 0, 0, 0);
                // the next stage is written while the matrix cores work through the queue
                if (t == 2 && more) ld.store(smem + (cur ^ 1) * T::STAGE);
            }
            __syncthreads();
            cur ^= 1;
        }

        // recombine the eight planes and add the partial sum onto Z
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int j = 0; j < WN; ++j) {
                const int col = tn * T::BN + (wn * WN + j) * 32 + r;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = tm * T::BM + (wm * WM + i) * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
                    u64 z = 0;
#pragma unroll
                    for (int s = 0; s < 8; ++s) z += (u64)(long long)acc[i][j][s][e] << (8 * s);
                    if (row < p.m && col < n_eff) atomicAdd(p.Z + (size_t)row * p.ldz + col, z);
                }
            }
        u += len;
    }
}

template <int WAVES_M, int WAVES_N, int WM, int WN>
int launch_gemm(comet_ctx* ctx, const char* what, const GemmParams& p, long units_cap) {
    using T = Tile<WAVES_M, WAVES_N, WM, WN>;
    auto kern = p.kind == KIND_SOMM ? ring_gemm_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SOMM>
                                    : ring_gemm_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SIMM>;
    static bool lds_reserved[2][64] = {};
    const int dev_slot = ctx->device & 63;
    if (!lds_reserved[p.kind][dev_slot]) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, T::SMEM) != hipSuccess)
            return comet_fail(ctx, COMET_EDEVICE, "%s: cannot reserve %d bytes of LDS", what, T::SMEM);
        lds_reserved[p.kind][dev_slot] = true;
    }
    // a chip-sized grid, shrunk when there is too little work to share out
    long grid = (ctx->num_cu / 8) * 8;
    if (grid < 8) grid = 8;
    const long want = (units_cap + 3) / 4;
    if (want < grid) grid = want < 8 ? (want < 1 ? 1 : want) : (want / 8) * 8;
    if (ctx->gemm_grid > 0) grid = ctx->gemm_grid;
    const bool timed = ctx->ev && ctx->ev_used + 2 <= ctx->ev_cap;
    if (timed) (void)hipEventRecord(ctx->ev[ctx->ev_used], ctx->stream);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(GT), T::SMEM, ctx->stream, p);
    if (timed) {
        (void)hipEventRecord(ctx->ev[ctx->ev_used + 1], ctx->stream);
        ctx->ev_used += 2;
    }
    COMET_LAUNCH_CHECK(ctx, what);
    return COMET_OK;
}

inline int round_up(int64_t v, int64_t to) { return (int)(((v + to - 1) / to) * to); }

size_t gemm_ws_bytes(int64_t m, int64_t kc_cap) {
    if (m < 1 || kc_cap < 0 || m > COMET_DIM_MAX || kc_cap > COMET_DIM_MAX) return 0;
    const size_t mpad = (size_t)round_up(m, 128);
    const size_t ks_cap = (size_t)((kc_cap + KSTEP - 1) / KSTEP);
    const size_t bytes = mpad * 2 * ks_cap * 256;
    return bytes ? bytes : 256;
}

int run_share(comet_ctx* ctx, const char* what, GemmParams p, void* ws, size_t ws_bytes) {
    const size_t need = gemm_ws_bytes(p.m, p.kc_cap);
    if (!ws || ws_bytes < need)
        return comet_fail(ctx, COMET_EWORKSPACE, "%s: workspace of %zu bytes required", what, need);
    if (reinterpret_cast<uintptr_t>(ws) & 255u)
        return comet_fail(ctx, COMET_EALIGN, "%s: workspace must be 256-byte aligned", what);
    comet_device_guard guard(ctx);
    if (!guard.ok) return comet_fail(ctx, COMET_EDEVICE, "%s: cannot select device", what);

    p.xp = static_cast<unsigned char*>(ws);
    p.mpad = round_up(p.m, 128);
    p.ks_cap = (p.kc_cap + KSTEP - 1) / KSTEP;

    if (p.n_cap == 0) return COMET_OK;
    // Z := C on the kept region
    {
        unsigned gx = (unsigned)((p.n_cap + GT - 1) / GT);
        if (gx > 64) gx = 64;
        for (int r0 = 0; r0 < p.m; r0 += 65535) {
            GemmParams q = p;
            q.Z = p.Z + (size_t)r0 * p.ldz;
            q.C = p.C + (size_t)r0 * p.ldz;
            const unsigned gy = (unsigned)((p.m - r0) < 65535 ? (p.m - r0) : 65535);
            hipLaunchKernelGGL(init_z_kernel, dim3(gx, gy), dim3(GT), 0, ctx->stream, q);
            COMET_LAUNCH_CHECK(ctx, what);
        }
    }
    if (p.ks_cap == 0) return COMET_OK;
    hipLaunchKernelGGL(xpack_kernel, dim3((unsigned)(p.ks_cap * 4), (unsigned)(p.mpad / 128), 2),
                       dim3(128), 0, ctx->stream, p);
    COMET_LAUNCH_CHECK(ctx, what);

    const long kt = 2l * p.ks_cap;
    if (p.m <= 32) {
        const long units = (long)((p.m + 31) / 32) * ((p.n_cap + 255) / 256) * kt;
        return launch_gemm<1, 4, 1, 2>(ctx, what, p, units);
    }
    if (p.m <= 64) {
        const long units = (long)((p.m + 63) / 64) * ((p.n_cap + 63) / 64) * kt;
        return launch_gemm<2, 2, 1, 1>(ctx, what, p, units);
    }
    const long units = (long)((p.m + 127) / 128) * ((p.n_cap + 63) / 64) * kt;
    return launch_gemm<2, 2, 2, 1>(ctx, what, p, units);
}

int check_common(comet_ctx* ctx, const char* what, int party, int64_t m, int bs, int n_blk_cap,
                 int flags, const void* const* ptrs, int n_ptrs, const int32_t* blk_idx) {
    if (party != 0 && party != 1) return comet_fail(ctx, COMET_EINVAL, "%s: party must be 0 or 1", what);
    if (m < 1 || bs < 1 || n_blk_cap < 0) return comet_fail(ctx, COMET_EINVAL, "%s: bad size", what);
    if (flags & ~(COMET_FULL_A | COMET_FULL_B)) return comet_fail(ctx, COMET_EINVAL, "%s: unknown flag", what);
    for (int i = 0; i < n_ptrs; ++i) {
        if (!ptrs[i]) return comet_fail(ctx, COMET_EINVAL, "%s: null pointer (operand %d)", what, i);
        if (!comet_aligned16(ptrs[i]))
            return comet_fail(ctx, COMET_EALIGN, "%s: operand %d is not 16-byte aligned", what, i);
    }
    if (!blk_idx && (flags & (COMET_FULL_A | COMET_FULL_B)))
        return comet_fail(ctx, COMET_EINVAL, "%s: blk_idx required for full-size operands", what);
    if (m > COMET_DIM_MAX / 2 || (int64_t)n_blk_cap * bs > COMET_DIM_MAX)
        return comet_fail(ctx, COMET_ECAP, "%s: dimension beyond 2^24 (m beyond 2^23)", what);
    return COMET_OK;
}

}  // namespace

size_t comet_gemm_workspace_bytes(int64_t m, int64_t kc_cap) { return gemm_ws_bytes(m, kc_cap); }

extern "C" {

int comet_somm_share(comet_ctx* ctx, int party, int64_t m, int64_t k, int64_t n_full, int bs,
                     const int32_t* blk_idx, const int32_t* n_blk_dev, int n_blk_cap, int flags,
                     const uint64_t* E, const uint64_t* F, const uint64_t* A_i,
                     const uint64_t* B_i, const uint64_t* C_i, uint64_t* Z_i, void* ws,
                     size_t ws_bytes) {
    const char* what = "comet_somm_share";
    COMET_CHECK_CTX(ctx);
    const void* ptrs[] = {E, F, A_i, B_i, C_i, Z_i};
    int rc = check_common(ctx, what, party, m, bs, n_blk_cap, flags, ptrs, 6, blk_idx);
    if (rc) return rc;
    if (k < 1 || n_full < 0) return comet_fail(ctx, COMET_EINVAL, "%s: bad size", what);
    if (flags & COMET_FULL_A) return comet_fail(ctx, COMET_EINVAL, "%s: A_i is never indexed in SOMM", what);
    if (k > COMET_DIM_MAX || n_full > COMET_DIM_MAX) return comet_fail(ctx, COMET_ECAP, "%s: dimension beyond 2^24", what);
    const int64_t ld = (int64_t)n_blk_cap * bs;
    if ((flags & COMET_FULL_B) && ld > n_full)
        return comet_fail(ctx, COMET_EINVAL, "%s: n_blk_cap * bs exceeds n_full", what);
    GemmParams p = {};
    p.kind = KIND_SOMM; p.party = party; p.m = (int)m; p.kc_cap = (int)k; p.n_cap = (int)ld;
    p.bs = bs; p.n_blk_cap = n_blk_cap; p.blk_idx = blk_idx; p.n_blk_dev = n_blk_dev;
    p.full_extent = (int)n_full;
    p.E = (const u64*)E; p.lde = k;
    p.A = (const u64*)A_i; p.lda = k; p.a_full = 0;
    p.B = (const u64*)B_i; p.b_full = (flags & COMET_FULL_B) ? 1 : 0; p.ldb = p.b_full ? n_full : ld;
    p.F = (const u64*)F; p.ldf = ld;
    p.C = (const u64*)C_i; p.Z = (u64*)Z_i; p.ldz = ld;
    return run_share(ctx, what, p, ws, ws_bytes);
}

int comet_simm_share(comet_ctx* ctx, int party, int64_t m, int64_t k_full, int64_t n, int bs,
                     const int32_t* blk_idx, const int32_t* n_blk_dev, int n_blk_cap, int flags,
                     const uint64_t* E, const uint64_t* F, const uint64_t* A_i,
                     const uint64_t* B_i, const uint64_t* C_i, uint64_t* Z_i, void* ws,
                     size_t ws_bytes) {
    const char* what = "comet_simm_share";
    COMET_CHECK_CTX(ctx);
    const void* ptrs[] = {E, F, A_i, B_i, C_i, Z_i};
    int rc = check_common(ctx, what, party, m, bs, n_blk_cap, flags, ptrs, 6, blk_idx);
    if (rc) return rc;
    if (n < 1 || k_full < 0) return comet_fail(ctx, COMET_EINVAL, "%s: bad size", what);
    if (n > COMET_DIM_MAX || k_full > COMET_DIM_MAX) return comet_fail(ctx, COMET_ECAP, "%s: dimension beyond 2^24", what);
    const int64_t ld = (int64_t)n_blk_cap * bs;
    if ((flags & (COMET_FULL_A | COMET_FULL_B)) && ld > k_full)
        return comet_fail(ctx, COMET_EINVAL, "%s: n_blk_cap * bs exceeds k_full", what);
    GemmParams p = {};
    p.kind = KIND_SIMM; p.party = party; p.m = (int)m; p.kc_cap = (int)ld; p.n_cap = (int)n;
    p.bs = bs; p.n_blk_cap = n_blk_cap; p.blk_idx = blk_idx; p.n_blk_dev = n_blk_dev;
    p.full_extent = (int)k_full;
    p.E = (const u64*)E; p.lde = ld;
    p.A = (const u64*)A_i; p.a_full = (flags & COMET_FULL_A) ? 1 : 0; p.lda = p.a_full ? k_full : ld;
    p.B = (const u64*)B_i; p.b_full = (flags & COMET_FULL_B) ? 1 : 0; p.ldb = n;
    p.F = (const u64*)F; p.ldf = n;
    p.C = (const u64*)C_i; p.Z = (u64*)Z_i; p.ldz = n;
    return run_share(ctx, what, p, ws, ws_bytes);
}

}  // extern "C"
