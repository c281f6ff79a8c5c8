// One party's output share (paper Eq. 1 on the indexed sub-matrices of Protocols 2 and 3)
//
//     [Z]_i = [C]_i + [ E | A' ] . [ B_i ; F ],   A' = A_i + party * E      (mod 2^64)
//
// for at most 32 activation rows (a decoding batch) when the weight side arrives as digit planes.
// Such a product is bound by reading B_i and F once: every weight fragment feeds exactly one
// matrix instruction per digit pair, so staging it in LDS for other wavefronts buys nothing.
// Here every wavefront works on its own, without a barrier anywhere in the kernel:
//   * it owns 32 output columns and a run of the stacked contraction; per contraction step of 32
//     it loads its eight weight fragments (one per digit) and the eight activation fragments
//     straight from memory into registers -- both plane formats are stored in matrix-instruction
//     operand order, a fragment is one 16-byte load per lane -- NST - 1 steps ahead of their use,
//     and issues the 36 digit-pair instructions (v_mfma_i32_32x32x32_i8) into eight int32 planes;
//   * the four wavefronts of a workgroup take four adjacent column tiles at the same contraction
//     steps, so the workgroup reads 32 KB of consecutive weight planes per step and its
//     activation fragments (the same for all four, a few MB in all) come from the cache;
//   * the (column group, step) units are dealt out evenly over the workgroups; a run ends at a
//     column group's last step or after 256 steps (a plane cannot overflow before that), its
//     planes are recombined and added onto Z, which started out as C, with 64-bit atomics:
//     addition mod 2^64 is associative and commutative, so the result is bit-exact for any split.
// The block gather of Protocols 2 and 3 is folded into the addressing: a column offset per lane
// (SOMM with a full-size B_i) or a row offset per 16 contraction indices (SIMM).
#include <hip/hip_ext.h>

#include "ring_gemm_kernel.h"

namespace {

using namespace comet_gemm;

constexpr int FT = 256;          // threads per workgroup
constexpr int FW = FT / 64;      // independent wavefronts
constexpr int FCOLS = 32 * FW;   // output columns per workgroup
constexpr int FSEG = 256;        // longest run of steps between two recombinations

template <int KIND, bool GATHER, int NST>
__global__ __launch_bounds__(FT) void ring_fewrow_kernel(GemmParams p) {
    // SIMM with a full-size B_i: first row of every (step, k-half) of a run in B_i's own row
    // numbering, looked up once per run (a load from the index list inside the pipelined loop would
    // have to wait for every weight load issued before it).  One table per wavefront.
    __shared__ int row_tab[(KIND == KIND_SIMM && GATHER) ? FW : 1][(KIND == KIND_SIMM && GATHER) ? 2 * FSEG : 1];
    const int nblk = n_blocks(p);
    const int n_eff = KIND == KIND_SOMM ? nblk * p.bs : p.n_cap;
    const int kc = KIND == KIND_SOMM ? p.kc_cap : nblk * p.bs;
    const int m_eff = n_rows(p);
    if (n_eff <= 0 || kc <= 0 || m_eff <= 0) return;           // uniform over the workgroup
    const int KS = (kc + KSTEP - 1) / KSTEP, KT = 2 * KS;
    const int groups = (n_eff + FCOLS - 1) / FCOLS;
    const long units = (long)groups * KT;
    const int G = gridDim.x;
    const int b = xcd_contiguous(blockIdx.x, G);
    long u = units * b / G;
    const long u_end = units * (b + 1) / G;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int r = lane & 31, g = lane >> 5;
    const size_t prow_b = (size_t)((p.ldb + 63) >> 6) * 16384u, prow_f = (size_t)((p.ldf + 63) >> 6) * 16384u;
    const char* const Bp = reinterpret_cast<const char*>(p.B);
    const char* const Fp = reinterpret_cast<const char*>(p.F);
    // Addresses are a wave-uniform base (scalar registers) plus a 32-bit offset per lane that does
    // not change inside a run.  Activation fragment of (half h, step s, digit t): unit
    // xp_group(h, s, t, g) * mpad + r, i.e. uniform group (h, s, t, 0) plus the lane's (g, r).
    const char* const Xp = reinterpret_cast<const char*>(p.xp);
    const unsigned x_off = (unsigned)((g * p.mpad + r) * 16);
    const size_t x_digit = (size_t)2 * p.mpad * 16;            // bytes from one digit to the next

    while (u < u_end) {
        const int cg = (int)(u / KT);
        const int q0 = (int)(u - (long)cg * KT);
        int len = KT - q0;
        if (len > u_end - u) len = (int)(u_end - u);
        if (len > FSEG) len = FSEG;
        u += len;
        const int qe = q0 + len;
        if (cg * FCOLS + wave * 32 >= n_eff) continue;          // a column tile beyond the last column
        const int out_col = cg * FCOLS + wave * 32 + r;
        const int col = out_col < n_eff ? out_col : n_eff - 1;
        long bcol = col;
        if (KIND == KIND_SOMM && GATHER) {
            const int blk = col / p.bs;
            const long st = block_start(p, blk);
            bcol = (st < 0 ? 0 : st) + (col - blk * p.bs);
        }
        // the lane's byte offset inside a contraction step of each weight operand (columns stay
        // below 2^24: host check), with the k-half it feeds
        const unsigned off_b = (unsigned)(bcol >> 6) * 16384u + (unsigned)(bcol & 63) * 16u + (unsigned)g * 1024u;
        const unsigned off_f = (unsigned)(col >> 6) * 16384u + (unsigned)(col & 63) * 16u + (unsigned)g * 1024u;

        if constexpr (KIND == KIND_SIMM && GATHER) {
            for (int i = lane; i < 2 * len; i += 64) {
                const int q = q0 + (i >> 1);
                int row = 0;
                if (q < KS) {
                    // bs is a multiple of 16 (host check), so the sixteen rows lie inside one block;
                    // beyond the contraction the activation digits are zero and any valid rows do
                    int kb = q * KSTEP + 16 * (i & 1);
                    kb = kb <= kc - 16 ? kb : kc - 16;
                    const int blk = p.bs_shift >= 0 ? (kb >> p.bs_shift) : kb / p.bs;
                    const long st = block_start(p, blk);
                    row = (int)(st < 0 ? 0 : st) + (kb - blk * p.bs);
                }
                row_tab[wave][i] = row;
            }
        }

        v4i w[NST][8], xa[NST][8];
        v16i acc[8];
#pragma unroll
        for (int s = 0; s < 8; ++s)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[s][e] = 0;

        auto issue = [&](int q, v4i (&xf)[8], v4i (&wf)[8]) {
            const int h = q >= KS ? 1 : 0;
            const int s = q - h * KS;
            const char* xs = Xp + xp_group(h, s, 0, 0, p.ks_cap) * p.mpad * 16;
#pragma unroll
            for (int t = 0; t < 8; ++t) xf[t] = *reinterpret_cast<const v4i*>(xs + t * x_digit + x_off);
            if (KIND == KIND_SIMM && GATHER && h == 0) {
                // the lane's sixteen rows start at its own row of B_i
                const int row = row_tab[wave][2 * (q - q0) + g];
                const char* wb = Bp + (size_t)(row >> 5) * prow_b + (size_t)((row >> 4) & 1) * 1024u +
                                 (off_b - (unsigned)g * 1024u);
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    wf[t] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(wb + t * 2048));
            } else {
                // rows 32 s + 16 g + 0..15: step s of the operand, the k-half is in the lane's offset
                const char* ws = (h ? Fp : Bp) + (size_t)s * (h ? prow_f : prow_b);
                const unsigned off = h ? off_f : off_b;
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    wf[t] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(ws + t * 2048 + off));
            }
        };
        auto step = [&](const v4i (&af)[8], const v4i (&wf)[8]) {
#pragma unroll
            for (int t = 0; t < 8; ++t)
#pragma unroll
                for (int uu = 0; uu + t < 8; ++uu)
                    acc[t + uu] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[t], wf[uu], acc[t + uu], 0, 0, 0);
        };

#pragma unroll
        for (int i = 0; i < NST - 1; ++i)
            if (q0 + i < qe) issue(q0 + i, xa[i], w[i]);
        for (int q = q0; q < qe; q += NST) {
#pragma unroll
            for (int i = 0; i < NST; ++i) {
                if (q + i < qe) {
                    if (q + i + NST - 1 < qe)
                        issue(q + i + NST - 1, xa[(i + NST - 1) % NST], w[(i + NST - 1) % NST]);
                    step(xa[i], w[i]);
                }
            }
        }

        // recombine the eight planes, sum_s sext64(S_s) << 8 s, and add the partial sum onto Z
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int row = 8 * (e >> 2) + 4 * g + (e & 3);
            long long lo = (long long)acc[0][e];
            lo += (long long)acc[1][e] * (1 << 8);
            lo += (long long)acc[2][e] * (1 << 16);
            lo += (long long)acc[3][e] * (1 << 24);
            const u32 hi = (u32)acc[4][e] + ((u32)acc[5][e] << 8) + ((u32)acc[6][e] << 16) + ((u32)acc[7][e] << 24);
            const u64 z = (u64)lo + ((u64)hi << 32);
            if (row < m_eff && out_col < n_eff) atomicAdd(p.Z + (size_t)row * p.ldz + out_col, z);
        }
    }
}

constexpr int FEWROW_STAGES = 3;

template <int KIND, bool GATHER>
int launch_fewrow(comet_ctx* ctx, const char* what, const GemmParams& p) {
    auto kern = ring_fewrow_kernel<KIND, GATHER, FEWROW_STAGES>;
    // one workgroup per compute unit: the accumulator planes and the fragments in flight take a
    // wavefront's whole register budget, so that is what the chip holds at once
    int grid = ctx->gemm_grid > 0 ? ctx->gemm_grid : ctx->num_cu;
    const long units = (long)((p.n_cap + FCOLS - 1) / FCOLS) * 2 * p.ks_cap;
    if (grid > units) grid = (int)(units > 0 ? units : 1);
    if (comet_time_this_launch(ctx)) {
        // the event pair rides on the dispatch itself: no marker packets around the kernel
        hipExtLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(FT), 0, ctx->stream, ctx->ev[ctx->ev_used],
                              ctx->ev[ctx->ev_used + 1], 0, p);
        ctx->ev_used += 2;
    } else {
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(FT), 0, ctx->stream, p);
    }
    COMET_LAUNCH_CHECK(ctx, what);
    return COMET_OK;
}

}  // namespace

int comet_launch_fewrow(comet_ctx* ctx, const char* what, const GemmParams& p) {
    if (p.m < 1 || p.m > COMET_FEWROW_MAX_ROWS || !p.w_planes || p.w_tr || p.row_comp || p.tmask)
        return comet_fail(ctx, COMET_EINVAL, "%s: operands outside the few-row matrix-core path", what);
    if (p.kind == KIND_SOMM) return p.b_full ? launch_fewrow<KIND_SOMM, true>(ctx, what, p) : launch_fewrow<KIND_SOMM, false>(ctx, what, p);
    return p.b_full ? launch_fewrow<KIND_SIMM, true>(ctx, what, p) : launch_fewrow<KIND_SIMM, false>(ctx, what, p);
}
