// One party's output share (paper Eq. 1 on the indexed sub-matrices of Protocols 2 and 3)
// when the activation side has only a few rows, as in token-by-token decoding:
//
//     [Z]_i = [C]_i + [ E | A' ] . [ B_i ; F ],   A' = A_i + party * E      (mod 2^64)
//
// With m <= 8 rows every weight word is used m times and the product is bound by reading the
// two weight operands once from memory, not by arithmetic: the matrix cores would spend most of
// their 32-row tiles on padding, and the digit split they need costs more vector work per
// weight word than the m multiply-adds themselves.  So this path multiplies directly in the
// vector ALU.  A ring multiply-add  z += x w  is three 32 x 32 -> 64 bit multiply-adds
// (v_mad_u64_u32, full rate on this chip): the low halves go into one 64-bit accumulator with
// their carry, the two cross products into a second one of which only the low 32 bits matter,
// and the result is  acc + (cross << 32); the high x high product lies beyond 2^64.
//   * a wavefront owns 64 * VEC adjacent output columns and a run of the stacked contraction;
//     per contraction index it issues one coalesced load of the weight row segment and takes
//     the m activation words from scalar registers (they are the same for every lane);
//   * the activation words are first rewritten k-major (prep kernel), so that the words of one
//     contraction index are one aligned scalar load; the same kernel sets Z := C;
//   * the four wavefronts of a workgroup take consecutive runs, add their partial sums in LDS
//     and issue one 64-bit atomic add per output element; addition mod 2^64 is associative and
//     commutative, so the result is bit-exact for any split.
// The block gather of Protocols 2 and 3 is folded into the addressing: a column offset per lane
// (SOMM with a full-size B_i) or a row offset per contraction index (SIMM).
#include "gemm_params.h"

namespace {

constexpr int ST = 256;        // threads per workgroup
constexpr int SW = ST / 64;    // wavefronts per workgroup
constexpr int UNROLL = 8;      // weight rows in flight per wavefront
constexpr int RG = 8;          // rows reduced through LDS at a time

typedef u64 u64x2 __attribute__((ext_vector_type(2)));

// xs[(h * kc_cap + k) * MR + r]: h = 0: E[r][k], h = 1: A'[r][k]; rows r >= m hold zero.
// blockIdx.y == 1: Z := C on the kept region.
__global__ __launch_bounds__(ST) void skinny_prep_kernel(GemmParams p, u64* xs, int MR) {
    const int nblk = n_blocks(p);
    const int m_eff = n_rows(p);
    const long stride = (long)gridDim.x * ST;
    const long t0 = (long)blockIdx.x * ST + threadIdx.x;
    if (blockIdx.y == 1) {
        // with result blocks (Protocol 2 in general form): C on the blocks, zero between them
        const int n_eff = p.kind == KIND_SOMM ? nblk * p.bs : p.n_cap;
        const long total = (long)m_eff * n_eff;
        for (long i = t0; i < total; i += stride) {
            const long r = i / n_eff, c = i - r * n_eff;
            u64 v = p.C[r * p.ldz + c];
            if (p.row_comp && p.row_comp[r] != p.blk_comp[c / p.bs]) v = 0;
            p.Z[r * p.ldz + c] = v;
        }
        return;
    }
    const int kc = p.kind == KIND_SOMM ? p.kc_cap : nblk * p.bs;
    const long total = 2l * MR * kc;
    for (long i = t0; i < total; i += stride) {
        const int k = (int)(i % kc);
        const int r = (int)((i / kc) % MR);
        const int h = (int)(i / ((long)kc * MR));
        u64 x = 0;
        // entries the token does not use take no part (Protocol 3 with per-token row sets)
        if (r < m_eff && (!p.tmask || token_uses(p, r, k / p.bs))) {
            const u64 e = p.E[(size_t)r * p.lde + k];
            x = e;
            if (h == 1) {
                long col = k;
                if (p.a_full) {
                    const int blk = k / p.bs;
                    const long st = block_start(p, blk);
                    col = (st < 0 ? 0 : st) + (k - blk * p.bs);
                }
                x = p.A[(size_t)r * p.lda + col] + (p.party ? e : 0ull);
            }
        }
        xs[((size_t)h * p.kc_cap + k) * MR + r] = x;
    }
}

template <int VEC>
struct WVec;
template <>
struct WVec<1> {
    u64 v[1];
    __device__ __forceinline__ void load(const u64* q) { v[0] = __builtin_nontemporal_load(q); }
    __device__ __forceinline__ void zero() { v[0] = 0; }
    __device__ __forceinline__ void add(const WVec& o) { v[0] += o.v[0]; }
};
template <>
struct WVec<2> {
    u64 v[2];
    __device__ __forceinline__ void load(const u64* q) {
        const u64x2 t = __builtin_nontemporal_load(reinterpret_cast<const u64x2*>(q));   // read once
        v[0] = t.x; v[1] = t.y;
    }
    __device__ __forceinline__ void zero() { v[0] = v[1] = 0; }
    __device__ __forceinline__ void add(const WVec& o) { v[0] += o.v[0]; v[1] += o.v[1]; }
};

__device__ __forceinline__ void mac(u64& acc, u64& cross, u64 x, u64 w) {
    const u32 xl = (u32)x, xh = (u32)(x >> 32), wl = (u32)w, wh = (u32)(w >> 32);
    acc += (u64)xl * wl;
    cross += (u64)xh * wl;
    cross += (u64)xl * wh;
}

// Weight row of stacked contraction index kk (wave-uniform): rows [0, kc) are B_i (gathered by
// block when B_i is the full-size operand of a SIMM call), rows [kc, 2 kc) are F.
template <int KIND>
__device__ __forceinline__ const u64* weight_row(const GemmParams& p, int kk, int kc, const u64* wB,
                                                 const u64* wF) {
    if (kk >= kc) return wF + (size_t)(kk - kc) * p.ldf;
    long row = kk;
    if (KIND == KIND_SIMM && p.b_full) {
        const int blk = p.bs_shift >= 0 ? (kk >> p.bs_shift) : kk / p.bs;
        const long st = block_start(p, blk);
        row = (st < 0 ? 0 : st) + (kk - blk * p.bs);
    }
    return wB + (size_t)row * p.ldb;
}

// UNOPENED: the rows of F are given as the two masked shares whose sum F is (p.F and p.F2, same
// layout): both are streamed and added on the fly, F itself is never written to memory.
template <int MR, int VEC, int KIND, bool UNOPENED>
__global__ __launch_bounds__(ST) void ring_skinny_kernel(GemmParams p, const u64* __restrict__ xs,
                                                         int slices) {
    constexpr int RGM = MR < RG ? MR : RG;                     // rows reduced through LDS at a time
    __shared__ __align__(16) u64 red[SW][RGM][64 * VEC];
    const int nblk = n_blocks(p);
    const int n_eff = KIND == KIND_SOMM ? nblk * p.bs : p.n_cap;
    const int kc = KIND == KIND_SOMM ? p.kc_cap : nblk * p.bs;
    const int m_eff = n_rows(p);
    const int tile0 = blockIdx.x * 64 * VEC;
    if (tile0 >= n_eff || kc <= 0) return;                    // uniform over the workgroup
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    int col = tile0 + lane * VEC;
    if (col >= n_eff) col = n_eff - VEC;                      // loads stay in range; never written back
    long colB = col;
    if (KIND == KIND_SOMM && p.b_full) {
        const int blk = col / p.bs;
        const long st = block_start(p, blk);
        colB = (st < 0 ? 0 : st) + (col - blk * p.bs);
    }
    const u64* wB = p.B + colB;
    const u64* wF = p.F + col;
    const u64* wF2 = UNOPENED ? p.F2 + col : nullptr;

    // this wavefront's run [k0, k1) of the stacked contraction [0, 2 kc), taken in interleaved
    // order: position j is row j / 2 of B_i (j even) or of F (j odd), so that every run reads
    // both operands alike (with the opening folded in an F row is two loads, a B_i row one)
    auto stacked = [&](int j) { return (j >> 1) + ((j & 1) ? kc : 0); };
    const int kt = 2 * kc;
    const int per_wg = (kt + slices - 1) / slices;
    const int per_wave = (per_wg + SW - 1) / SW;
    const int wg0 = blockIdx.y * per_wg;
    int wg1 = wg0 + per_wg;
    wg1 = wg1 < kt ? wg1 : kt;
    int k0 = wg0 + wave * per_wave;
    int k1 = k0 + per_wave;
    k1 = k1 < wg1 ? k1 : wg1;

    u64 acc[MR][VEC], cross[MR][VEC];
#pragma unroll
    for (int r = 0; r < MR; ++r)
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[r][v] = cross[r][v] = 0;

    int kk = k0;
    for (; kk + UNROLL <= k1; kk += UNROLL) {
        WVec<VEC> w[UNROLL], w2[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int q = stacked(kk + u);
            const u64* src = weight_row<KIND>(p, q, kc, wB, wF);
            w[u].load(src);
            if (UNOPENED) {
                if (q >= kc) w2[u].load(wF2 + (src - wF));       // the same row of the other share
                else w2[u].zero();
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            if (UNOPENED) w[u].add(w2[u]);
            const int q = stacked(kk + u);
            const u64* x = xs + ((size_t)(q >= kc ? p.kc_cap + (q - kc) : q)) * MR;
#pragma unroll
            for (int r = 0; r < MR; ++r)
#pragma unroll
                for (int v = 0; v < VEC; ++v) mac(acc[r][v], cross[r][v], x[r], w[u].v[v]);
        }
    }
    for (; kk < k1; ++kk) {
        WVec<VEC> w;
        const int q = stacked(kk);
        const u64* src = weight_row<KIND>(p, q, kc, wB, wF);
        w.load(src);
        if (UNOPENED && q >= kc) {
            WVec<VEC> w2;
            w2.load(wF2 + (src - wF));
            w.add(w2);
        }
        const u64* x = xs + ((size_t)(q >= kc ? p.kc_cap + (q - kc) : q)) * MR;
#pragma unroll
        for (int r = 0; r < MR; ++r)
#pragma unroll
            for (int v = 0; v < VEC; ++v) mac(acc[r][v], cross[r][v], x[r], w.v[v]);
    }

    // partial sums of the four wavefronts -> LDS -> one atomic add per output element
#pragma unroll
    for (int r0 = 0; r0 < MR; r0 += RGM) {
        if (r0) __syncthreads();
#pragma unroll
        for (int r = 0; r < RGM; ++r)
#pragma unroll
            for (int v = 0; v < VEC; ++v)
                red[wave][r][lane * VEC + v] = acc[r0 + r][v] + (cross[r0 + r][v] << 32);
        __syncthreads();
        for (int i = threadIdx.x; i < RGM * 64 * VEC; i += ST) {
            const int r = i / (64 * VEC), c = i - r * (64 * VEC);
            u64 s = 0;
#pragma unroll
            for (int wv = 0; wv < SW; ++wv) s += red[wv][r][c];
            const int row = r0 + r, oc = tile0 + c;
            bool live = row < m_eff && oc < n_eff;
            if (live && p.row_comp) live = p.row_comp[row] == p.blk_comp[oc / p.bs];   // on a result block
            if (live) atomicAdd(p.Z + (size_t)row * p.ldz + oc, s);
        }
    }
}

template <int MR, int VEC>
void (*pick_kernel(int kind, bool unopened))(GemmParams, const u64*, int) {
    if (unopened)
        return kind == KIND_SOMM ? ring_skinny_kernel<MR, VEC, KIND_SOMM, true> : ring_skinny_kernel<MR, VEC, KIND_SIMM, true>;
    return kind == KIND_SOMM ? ring_skinny_kernel<MR, VEC, KIND_SOMM, false> : ring_skinny_kernel<MR, VEC, KIND_SIMM, false>;
}

}  // namespace

int comet_launch_skinny(comet_ctx* ctx, const char* what, const GemmParams& p) {
    if (p.m < 1 || p.m > COMET_SKINNY_MAX_ROWS)
        return comet_fail(ctx, COMET_EINVAL, "%s: row count outside the vector-ALU path", what);
    // rows the kernel carries: every weight word is multiplied into all of them, and at eight
    // rows the vector ALU is as busy as the memory system, so fewer rows get a narrower variant
    const int MR = p.m <= 2 ? 2 : p.m <= 4 ? 4 : p.m <= 6 ? 6 : COMET_SKINNY_MAX_ROWS;
    u64* xs = reinterpret_cast<u64*>(p.xp);
    // k-major activation words and Z := C (the workspace of the matrix-core path, 2048 bytes per
    // contraction index, always covers the 2 * MR * 8 bytes per index used here)
    {
        long work = 2l * MR * p.kc_cap;
        const long zwork = (long)p.m * p.n_cap;
        if (zwork > work) work = zwork;
        long gx = (work + ST - 1) / ST;
        if (gx > 2048) gx = 2048;
        if (gx < 1) gx = 1;
        hipLaunchKernelGGL(skinny_prep_kernel, dim3((unsigned)gx, 2), dim3(ST), 0, ctx->stream, p, xs, MR);
        COMET_LAUNCH_CHECK(ctx, what);
    }
    if (p.kc_cap == 0) return COMET_OK;
    // two columns per lane need 16-byte aligned row segments on both weight operands and
    // column pairs that never straddle a gathered block
    const bool vec2 = (p.ldb & 1) == 0 && (p.ldf & 1) == 0 && (p.n_cap & 1) == 0 && (p.bs & 1) == 0;
    const int cols = vec2 ? 128 : 64;
    const long tiles = (p.n_cap + cols - 1) / cols;
    // about sixteen workgroups per compute unit, each wavefront with at least one full batch of
    // rows in flight
    long slices = (16l * ctx->num_cu + tiles - 1) / tiles;
    const long max_slices = (2l * p.kc_cap) / (SW * UNROLL);
    if (slices > max_slices) slices = max_slices;
    if (ctx->skinny_slices > 0) slices = ctx->skinny_slices;
    if (slices > 65535) slices = 65535;
    if (slices < 1) slices = 1;
    void (*kern)(GemmParams, const u64*, int);
    const bool un = p.F2 != nullptr;
    if (MR == 2) kern = vec2 ? pick_kernel<2, 2>(p.kind, un) : pick_kernel<2, 1>(p.kind, un);
    else if (MR == 4) kern = vec2 ? pick_kernel<4, 2>(p.kind, un) : pick_kernel<4, 1>(p.kind, un);
    else if (MR == 6) kern = vec2 ? pick_kernel<6, 2>(p.kind, un) : pick_kernel<6, 1>(p.kind, un);
    else kern = vec2 ? pick_kernel<COMET_SKINNY_MAX_ROWS, 2>(p.kind, un) : pick_kernel<COMET_SKINNY_MAX_ROWS, 1>(p.kind, un);
    const bool timed = comet_time_this_launch(ctx);
    if (timed) {
        // the event pair rides on the dispatch itself: no marker packets around the kernel
        hipExtLaunchKernelGGL(kern, dim3((unsigned)tiles, (unsigned)slices), dim3(ST), 0, ctx->stream,
                              ctx->ev[ctx->ev_used], ctx->ev[ctx->ev_used + 1], 0, p, (const u64*)xs, (int)slices);
        ctx->ev_used += 2;
    } else {
        hipLaunchKernelGGL(kern, dim3((unsigned)tiles, (unsigned)slices), dim3(ST), 0, ctx->stream, p,
                           (const u64*)xs, (int)slices);
    }
    COMET_LAUNCH_CHECK(ctx, what);
    return COMET_OK;
}
