// The int8 matrix-core kernel behind the share calls (see ring_gemm.hip for the formulation):
// tile shapes, the loader that stages both operands, one contraction step, the stream-K kernel
// and its launcher.  The kernel variants are instantiated in translation units of their own
// (ring_gemm_tile_*.hip), so that they compile side by side.
#pragma once

#include "common.h"
#include "digits.h"
#include "gemm_params.h"

#include <type_traits>
#include <utility>

namespace comet_gemm {


typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef u32 u32x4 __attribute__((ext_vector_type(4)));

constexpr int KSTEP = 32;       // ring words contracted per matrix instruction
constexpr int MAX_SEG = 256;    // contraction steps an int32 plane can absorb
constexpr int GT = 256;         // threads per workgroup (4 wavefronts)

// how the weight-side rows of B_i are addressed (SIMM with a full-size B_i only)
constexpr int GATHER_NONE = 0;   // rows are the compact contraction index
constexpr int GATHER_POW2 = 1;   // block gather, bs a power of two >= 8
constexpr int GATHER_ANY = 2;    // block gather, any bs
// SOMM with neuron-major weights: B_i and F hold one row of k contiguous words per output column
constexpr int WEIGHTS_TR = 3;
// B_i and F arrive as digit planes (see PlaneLoader); with W_PLANES_GATHER the rows of a
// full-size B_i are gathered by block (SIMM, bs a multiple of 16)
constexpr int W_PLANES = 4;
constexpr int W_PLANES_GATHER = 5;
constexpr bool is_planes(int gmode) { return gmode == W_PLANES || gmode == W_PLANES_GATHER; }

// Packed layout of [E | A'] in 16-byte units: group (half h, step s, digit t,
// k-half g) is a run of mpad units, one per row; the 16 bytes of a unit are
// digit t of words k = 32 s + 16 g + 0..15 of that row, which is exactly what
// one lane feeds to v_mfma_i32_32x32x32_i8.  Groups are ordered (h, s, t, g).
__device__ __host__ __forceinline__ size_t xp_group(int h, int s, int t, int g, int ks_cap) {
    return ((((size_t)h * ks_cap + s) * 8 + t) * 2 + g);
}


// ---------------------------------------------------------------------------
// gemm
// ---------------------------------------------------------------------------
template <int WAVES_M, int WAVES_N, int WM, int WN>
struct Tile {
    static constexpr int BM = 32 * WM * WAVES_M;
    static constexpr int BN = 32 * WN * WAVES_N;
    static constexpr int XBYTES = BM * 256;          // 8 digits x 2 k-halves x BM rows x 16 bytes
    static constexpr int WBYTES = BN * 256;
    static constexpr int XSTAGES = 3;                // written by LDS-DMA two steps ahead
    static constexpr int WSTAGES = 2;                // written from registers one step ahead
    static constexpr int WBASE = XSTAGES * XBYTES;
    static constexpr int SMEM = XSTAGES * XBYTES + WSTAGES * WBYTES;
    // four wavefronts, one per SIMD (the plane variants also build with eight -- Tile<4, 2, 1, 1>,
    // two wavefronts per SIMD on the 128 x 64 tile -- which measured no faster and is not instantiated)
    static constexpr int THREADS = WAVES_M * WAVES_N * 64;
    static constexpr int XVEC = XBYTES / 16 / THREADS;    // 16-byte units per thread per stage
    static constexpr int WVEC = WBYTES / 16 / THREADS;    // same for a weight stage filled by LDS-DMA
    static constexpr int WTASK = BN * 4 / GT;        // (column, octet) tasks per thread per stage (word loader: 256 threads)
    // vector-memory loads a thread issues per step: the LDS-DMA units plus, per weight task,
    // eight 8-byte loads (or four 16-byte loads when the weights are neuron-major)
    // and one load of a block id with the power-of-two row gather; with weight planes only
    // LDS-DMA units
    static constexpr int vm_per_step(int gmode) {
        if (is_planes(gmode)) return XVEC + WVEC;
        return XVEC + (gmode == WEIGHTS_TR ? 4 : 8) * WTASK + (gmode == GATHER_POW2 ? WTASK : 0);
    }
    // weight planes are written by LDS-DMA two steps ahead, like the activation planes: three
    // stages, plus the step table of the segment
    static constexpr int wstages(int gmode) { return is_planes(gmode) ? 3 : WSTAGES; }
    static constexpr int smem(int gmode) {
        return XSTAGES * XBYTES + wstages(gmode) * WBYTES + (is_planes(gmode) ? MAX_SEG * 16 : 0);
    }
    // two workgroups share a compute unit when one needs at most half of its registers and LDS
    static constexpr int wg_per_cu(int gmode) {
        return (WM * WN == 1 && THREADS == GT && smem(gmode) <= 80 * 1024) ? 2 : 1;
    }
    static_assert(THREADS == GT || THREADS == 2 * GT, "four or eight wavefronts per workgroup");
    static_assert(XVEC >= 1 && WTASK >= 1, "tile too small for the loader");
    static_assert(vm_per_step(GATHER_POW2) < 63, "outstanding-load counter has 6 bits");
    static_assert(SMEM <= 160 * 1024, "LDS of one CDNA4 compute unit");
};

// Workgroup barrier of the main loop.  Waits until at most N of this
// wavefront's vector-memory loads are still in flight (loads return in order,
// so everything older than the N youngest has landed, including LDS-DMA
// writes) and until all of its LDS accesses are done, then meets the other
// wavefronts.  Written out by hand because the generic barrier would also
// wait for the LDS-DMA loads that were only just issued for a later step.
template <int N>
__device__ __forceinline__ void wait_and_barrier() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

// Loads and staging of the operands, cut into small pieces.
//
// A contraction step issues 36 * WM * WN matrix instructions.  Everything else
// a step has to do -- start the LDS-DMA of the activation planes two steps
// ahead, request the weight words of the step after next, turn the weight
// words of the next step (requested a step ago) into digit planes and store
// them to LDS -- is cut into pieces of a handful of instructions, and
// gemm_step() places a piece behind every second or third matrix instruction
// so that they execute in its shadow.
//
// Activation side: the packed digit planes go from global memory straight into
// LDS (global_load_lds_dwordx4: every lane supplies its own global address, the
// wavefront's 64 x 16 bytes land contiguously at a wave-uniform LDS address),
// so they occupy no registers and need no LDS store.
//
// Weight side: raw uint64 words into registers; one step later each word is
// split into digits and its register immediately reused for the next request.
// Every load is unconditional: out-of-range rows and columns are clamped to a
// valid address instead of being predicated off.  That is exact because
// (a) a weight column only feeds its own output column, and columns at or
// beyond the kept width are never written back, and (b) the packed activation
// planes hold zeros beyond the contraction length, so whatever the weight side
// reads there is multiplied by zero.
template <class T, int KIND, int GMODE, bool LISTED>
struct Loader {
    static constexpr int W = T::WTASK;
    // Where this task's weight words are.  Without a row gather: pointers to (row 0, the task's
    // column) of B_i (column gather applied for SOMM) and of F; neuron-major weights: to the
    // column's own row of k words.  With a row gather (SIMM, full-size B_i): the byte offset of
    // the column inside a row; the row is wave-uniform, so a load is "scalar row address +
    // 32-bit lane offset" and the compiler has no per-load 64-bit vector addresses to keep
    // (it would form all of a step's addresses ahead of time and run out of registers on the
    // 32 x 256 tile).
    static constexpr bool ROW_GATHER = GMODE == GATHER_POW2 || GMODE == GATHER_ANY;
    unsigned cb[W], cf[W];
    const char* wbase;         // row gather: B_i or F, whichever half the look-ahead step is in
    // GATHER_POW2: the eight rows of a task's octet are consecutive, so a task keeps a running
    // (wave-uniform) row address that moves on by one row pitch per load, and the lane's column
    // offset of the half it is in: a load is two scalar additions and the load itself
    const char* wcur[W];
    size_t wpitch;
    unsigned csel[W];
    const u64* wb[W];
    const u64* wf[W];
    const unsigned char* xsrc; // this thread's first 16-byte unit of step (h = 0, s = 0)
    u64 wn[W][8];              // weight words in flight (requested one step before they are split)
    u64 wa[W][8];              // digits of the weight words being staged for the next step
    u32 pl[W][16];             // transposed digits: [t] = words 0..3, [8 + t] = words 4..7
    // wave-uniform state of the look-ahead step, set by begin()
    int h2, s2;
    int ld2;                   // row pitch of the weight-side source in words
    const unsigned char* xs2;
    size_t xstride;            // bytes between the 16-byte units one thread moves per step
    int g0[W];                 // GATHER_POW2: first gathered row of this task's octet
    int gpend[W];              // GATHER_POW2: block id requested for the step after this one
    const int* steps;          // listed contraction steps of this row tile, or null (all steps)

    static_assert(T::THREADS == GT, "the word loader is written for four wavefronts");
    static constexpr int XGRP_PER_PASS = GT / T::BM;         // groups covered by one pass of the block
    static_assert(GT % T::BM == 0, "tile rows must divide the block");

    // Piece list of one step, in execution order: the DMA issues, then task by task the eight
    // split-and-reload pieces, the four transposes and the eight LDS stores (task-major, so the
    // digits and transposed planes of a task are dead before the next task starts).
    static constexpr int P_DMA = 0;
    static constexpr int P_TASK = P_DMA + T::XVEC;
    static constexpr int PER_TASK = 8 + 4 + 8;
    static constexpr int P_END = P_TASK + PER_TASK * W;
    static constexpr int VM_PER_STEP = T::vm_per_step(GMODE);

    __device__ __forceinline__ void setup(const GemmParams& p, int tm, int tn, int n_eff) {
#pragma unroll
        for (int j = 0; j < W; ++j) {
            const int id = threadIdx.x + GT * j;
            int col = tn * T::BN + id % T::BN;
            col = col < n_eff ? col : n_eff - 1;
            long bcol = col;
            if (KIND == KIND_SOMM && p.b_full) {
                const int blk = col / p.bs;
                const long st = block_start(p, blk);
                bcol = (st < 0 ? 0 : st) + (col - blk * p.bs);
            }
            if (GMODE == WEIGHTS_TR) {
                // the column's own row of k words; the contraction index is then the word offset
                wb[j] = p.B + bcol * p.ldb;
                wf[j] = p.F + (long)col * p.ldf;
            } else if (ROW_GATHER) {
                cb[j] = (unsigned)bcol * 8u;      // columns stay below 2^24 (host check)
                cf[j] = (unsigned)col * 8u;
            } else {
                wb[j] = p.B + bcol;
                wf[j] = p.F + col;
            }
        }
        steps = nullptr;
        const int grp = threadIdx.x / T::BM, within = threadIdx.x % T::BM;
        xsrc = p.xp + ((size_t)grp * p.mpad + (size_t)tm * T::BM + within) * 16;
        xstride = (size_t)XGRP_PER_PASS * p.mpad * 16;
    }

    // block id that holds compact row octet (step ks, task j); GATHER_POW2 only
    // A position ks in [0, 2 KS) of the stacked contraction of this tile -> half h and step s.
    // Without a step list the positions are the steps themselves; with one (per-token row sets)
    // a half has KS listed steps and position q stands for step steps[q].
    __device__ __forceinline__ void resolve(int ks, int KS, int& h, int& s) const {
        h = ks >= KS ? 1 : 0;
        s = ks - h * KS;
        if constexpr (LISTED) s = steps[s];
    }

    __device__ __forceinline__ int gather_id(const GemmParams& p, int ks, int KS, int kc, int j) {
        int h, s;
        resolve(ks, KS, h, s);
        const int oct = __builtin_amdgcn_readfirstlane((int)((threadIdx.x + GT * j) / T::BN));
        const int k0 = s * KSTEP + oct * 8;
        const int kb = k0 <= kc - 8 ? k0 : kc - 8;
        // The index is the same for all lanes, but it is made a vector value on purpose (a zero
        // the compiler cannot see through): the id then arrives through the vector-memory queue,
        // in order with the weight words, instead of through a scalar load, whose counter is
        // shared with the LDS reads -- every fragment read of the step would wait for it.
        int lane_zero = 0;
        asm volatile("" : "+v"(lane_zero));
        return p.blk_idx[((kb >> p.bs_shift) & (h - 1)) + lane_zero];
    }

    // first step of a segment: nothing has been requested ahead yet
    __device__ __forceinline__ void prime(const GemmParams& p, int ks, int KS, int kc) {
        if (GMODE == GATHER_POW2) {
#pragma unroll
            for (int j = 0; j < W; ++j) gpend[j] = gather_id(p, ks, KS, kc, j);
        }
    }

    // Fix the step the following dma / load pieces work on.  Steps are visited in
    // order (ks, then ks + 1 capped at ks_limit), which lets the block id of the
    // next step be requested here, a whole step before it is needed (see gather_id()
    // for why that request is a vector load).
    __device__ __forceinline__ void begin(const GemmParams& p, int ks, int KS, int kc, int ks_limit) {
        resolve(ks, KS, h2, s2);
        h2 = __builtin_amdgcn_readfirstlane(h2);
        s2 = __builtin_amdgcn_readfirstlane(s2);
        ld2 = GMODE == WEIGHTS_TR ? 1 : (int)(h2 ? p.ldf : p.ldb);
        if (ROW_GATHER) {
            // both halves as one expression without control flow (h2 is 0 or 1): a branch inside a
            // step makes the compiler lose track of which loads are still in flight, and it then
            // waits for all of the previous step's at the first use
            // (a select between two pointers keeps their address space; going through integers
            // would turn the loads into flat loads, which also count against the LDS counter)
            wbase = reinterpret_cast<const char*>(h2 ? p.F : p.B);
        }
        xs2 = xsrc + (size_t)(h2 * p.ks_cap + s2) * 16 * p.mpad * 16;
        if (GMODE == GATHER_POW2) {
            const int ksn = ks + 1 < ks_limit ? ks + 1 : ks_limit;
#pragma unroll
            for (int j = 0; j < W; ++j) {
                // consumed here, ahead of the fragment reads (the scheduling fence that follows
                // them keeps this arithmetic from sinking to its first use)
                const int id = __builtin_amdgcn_readfirstlane(gpend[j]);
                const long st = (long)id * p.bs;
                const int oct = __builtin_amdgcn_readfirstlane((int)((threadIdx.x + GT * j) / T::BN));
                const int k0 = s2 * KSTEP + oct * 8;
                const int kb = k0 <= kc - 8 ? k0 : kc - 8;
                const long ok = ((st < 0) | (st + p.bs > p.full_extent)) ? 0l : -1l;
                g0[j] = (int)(st & ok) + (kb & (p.bs - 1));
                // first row of the octet: gathered in the B_i half, compact (kb) in the F half;
                // kc is a multiple of 8 here, so an octet lies inside the contraction as a whole
                // or not at all, and kb keeps the latter in range (its activation digits are zero)
                const int r0 = g0[j] + ((kb - g0[j]) & -h2);
                wpitch = (size_t)ld2 * 8u;
                wcur[j] = wbase + (size_t)r0 * wpitch;
                csel[j] = cb[j] + ((cf[j] - cb[j]) & (0u - (unsigned)h2));
                gpend[j] = gather_id(p, ksn, KS, kc, j);
            }
        }
    }

    // one 16-byte unit per lane of the activation planes -> LDS stage (asynchronous)
    template <int J>
    __device__ __forceinline__ void dma_piece(const GemmParams& p, unsigned char* xstage) {
        const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
        const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) void*)xstage;
        // Issued as plain text so that the compiler's own wait-count bookkeeping does not treat
        // every later LDS read as dependent on this transfer; the waits that order it are the
        // explicit ones in wait_and_barrier().  M0 carries the wave's LDS address.
        const unsigned lds = __builtin_amdgcn_readfirstlane(lds0 + (wave * 64 + GT * J) * 16);
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                     :
                     : "s"(lds), "v"(xs2 + J * xstride)
                     : "memory", "m0");
    }

    // Word E of task J: split the word that is in the register into digits
    // (it was requested a step ago), then request the word of the step fixed by
    // begin() into the same register.  The choice between the two halves of the
    // stacked contraction and the row gather are selects on wave-uniform values.
    template <int J, int E, bool SPLIT>
    __device__ __forceinline__ void load_piece(const GemmParams& p, int kc) {
        // The compiler's wait for this word (requested a step ago) does not know about the LDS-DMA
        // transfers issued since, which sit between the two in the in-order load queue, so it also
        // waits for those.  Measured, that costs nothing: the kernel is bound by power, and a
        // hand-written, exact wait (which needs the request in inline assembly, outside the
        // compiler's view of the register) gave the same time per step.
        if (SPLIT) wa[J][E] = to_digits(wn[J][E]);
        // octet index is the same for all lanes of a wavefront
        const int oct = __builtin_amdgcn_readfirstlane((int)((threadIdx.x + GT * J) / T::BN));
        const int k0 = s2 * KSTEP + oct * 8;
        if constexpr (GMODE == WEIGHTS_TR) {
            const u64* src = h2 ? wf[J] : wb[J];
            // Words E - 1 and E of the octet are neighbours in memory: one 16-byte load behind the
            // split of the second (k is even and the rows are 16-byte aligned, host check).  Past
            // the end of the contraction any valid pair will do: its activation digits are zero.
            if constexpr ((E & 1) == 1) {
                typedef u64 u64x2 __attribute__((ext_vector_type(2)));
                const int kp = (k0 + E) < kc ? (k0 + E - 1) : kc - 2;
                const u64x2 v = *reinterpret_cast<const u64x2*>(src + kp);
                wn[J][E - 1] = v.x;
                wn[J][E] = v.y;
            }
            return;
        }
        if constexpr (GMODE == GATHER_POW2) {
            const char* rowp = wcur[J];
            wcur[J] += wpitch;
            wn[J][E] = *reinterpret_cast<const u64*>(rowp + csel[J]);
            return;
        }
        const int kk = (k0 + E) < kc ? (k0 + E) : kc - 1;
        int row = kk;
        if (GMODE == GATHER_POW2) {
            // B_i rows are the kept neurons; bs is a power of two >= 8, so an octet of compact
            // rows lies inside one block (g0 is its first row, set by begin()); F rows are compact
            const int rg = g0[J] + E;
            row = rg + ((kk - rg) & -h2);
        } else if (GMODE == GATHER_ANY) {
            const int blk = kk / p.bs;
            const long st = block_start(p, blk);
            row = h2 ? kk : (int)(st < 0 ? 0 : st) + (kk - blk * p.bs);
        }
        if constexpr (ROW_GATHER) {
            // wave-uniform start of the row, then this lane's column
            const char* rowp = wbase + (size_t)row * (size_t)ld2 * 8u;
            const unsigned c = cb[J] + ((cf[J] - cb[J]) & (0u - (unsigned)h2));
            wn[J][E] = *reinterpret_cast<const u64*>(rowp + c);
        } else {
            // every operand holds fewer than 2^31 words (host check), so the word offset fits 32 bits
            const u64* src = h2 ? wf[J] : wb[J];
            const unsigned off = (unsigned)row * (unsigned)ld2;
            wn[J][E] = src[off];
        }
    }

    // quarter Q of the byte transpose of task J: Q = 0: low digits of words 0..3,
    // 1: high digits of words 0..3, 2: low digits of words 4..7, 3: high digits of words 4..7
    template <int J, int Q>
    __device__ __forceinline__ void transpose_piece() {
        constexpr int e0 = (Q >> 1) * 4, d0 = (Q & 1) * 4, o = (Q >> 1) * 8 + d0;
        u32 x[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] = (Q & 1) ? (u32)(wa[J][e0 + i] >> 32) : (u32)wa[J][e0 + i];
        transpose4(x[0], x[1], x[2], x[3], pl[J][o], pl[J][o + 1], pl[J][o + 2], pl[J][o + 3]);
    }

    // digit plane Tt of task J -> LDS.  Weight stage layout: 16-byte fragments ordered
    // (digit, k-half, column); an octet is one 8-byte half of a fragment, so a matrix-instruction
    // operand is a single 16-byte LDS read.
    template <int J, int Tt>
    __device__ __forceinline__ void write_piece(unsigned char* wstage) {
        const int id = threadIdx.x + GT * J;
        const int c = id % T::BN, oct = id / T::BN;
        const u64 v = (u64)pl[J][Tt] | ((u64)pl[J][8 + Tt] << 32);
        *reinterpret_cast<u64*>(wstage + ((size_t)(Tt * 2 + (oct >> 1)) * T::BN + c) * 16 + (oct & 1) * 8) = v;
    }

    // SPLIT = false: first visit of a segment, nothing to split or store yet, loads only
    template <int P, bool SPLIT>
    __device__ __forceinline__ void piece(const GemmParams& p, int kc, unsigned char* xstage,
                                          unsigned char* wstage) {
        if constexpr (P < P_TASK) {
            dma_piece<P - P_DMA>(p, xstage);
        } else if constexpr (P < P_END) {
            constexpr int J = (P - P_TASK) / PER_TASK, R = (P - P_TASK) % PER_TASK;
            if constexpr (R < 8) load_piece<J, R, SPLIT>(p, kc);
            else if constexpr (R < 12) { if (SPLIT) transpose_piece<J, R - 8>(); }
            else { if (SPLIT) write_piece<J, R - 12>(wstage); }
        }
    }

    template <int P0, bool SPLIT, int... Ps>
    __device__ __forceinline__ void pieces(std::integer_sequence<int, Ps...>, const GemmParams& p,
                                           int kc, unsigned char* xstage, unsigned char* wstage) {
        (piece<P0 + Ps, SPLIT>(p, kc, xstage, wstage), ...);
    }

};


// Loader for weight-side operands that arrive as digit planes (W_PLANES, W_PLANES_GATHER).
//
// B_i and F are stored in the unit format of the packed activation planes, transposed: a
// 16-byte unit holds digit t of the sixteen contraction words k = 32 s + 16 g + 0..15 of ONE
// column, and units are ordered (step s, chunk of 64 columns, digit t, k-half g, column inside
// the chunk): the sixteen runs (t, g) of a step and a column chunk are 16 KB of consecutive
// memory.  A weight stage of a tile is sixteen runs of BN units, each run of 64 columns one
// wavefront-wide LDS-DMA transfer:
// the step needs no vector arithmetic, no registers and no LDS store for either operand, only
// the matrix instructions and their fragment reads.  The planes of F come out of the opening
// kernel, those of B_i (triple material) are packed offline.
//
// Everything a step's transfers depend on -- which half of the stacked contraction it is in,
// where its activation planes start, which rows of the weight operand it contracts (after the
// block gather of a full-size B_i, or through the step list of Protocol 3's row sets) -- is put
// into a small LDS table once per segment (build_table) and read one step ahead, so that a
// step contains no global index loads and no address arithmetic beyond a few scalar operations.
template <class T, int KIND, int GMODE, bool LISTED>
struct PlaneLoader {
    static constexpr int XV = T::XVEC, WV = T::WVEC;
    static constexpr int P_END = XV + WV;
    static constexpr int VM_PER_STEP = XV + WV;
    static constexpr int XGRP_PER_PASS = T::THREADS / T::BM;
    static_assert(T::THREADS % T::BM == 0, "tile rows must divide the block");
    static_assert(T::BN % 64 == 0, "a wavefront's transfer stays inside one run of units");

    unsigned pcb[WV], pcf[WV], pcsel[WV];   // lane's byte offset of its column inside a run: B_i, F, selected
    const unsigned char* xsrc;              // this thread's first 16-byte unit of step (h = 0, s = 0)
    size_t xstride;
    const unsigned char* xs2;               // same for the look-ahead step
    const char* pbase;                      // planes of the half the look-ahead step is in
    size_t prow;                            // bytes per contraction step of the whole operand (its column chunks x 16 KB)
    int n0a, n0b;                           // first row of the two k-halves in the operand's own row numbering
    v4i pend;                               // table entry of the step after the look-ahead step
    const int* tab;                         // LDS: per position of the segment {x group, n0a, n0b, half}
    const int* steps;                       // listed contraction steps of this row tile, or null

    __device__ __forceinline__ void setup(const GemmParams& p, int tm, int tn, int n_eff) {
#pragma unroll
        for (int j = 0; j < WV; ++j) {
            const int u = threadIdx.x + T::THREADS * j;            // unit of the stage: run u / BN, column u % BN
            int col = tn * T::BN + u % T::BN;
            col = col < n_eff ? col : n_eff - 1;
            long bcol = col;
            if (KIND == KIND_SOMM && p.b_full) {
                const int blk = col / p.bs;
                const long st = block_start(p, blk);
                bcol = (st < 0 ? 0 : st) + (col - blk * p.bs);
            }
            // chunk of 64 columns, then the column inside it (columns stay below 2^24: host check)
            pcb[j] = ((unsigned)bcol >> 6) * 16384u + ((unsigned)bcol & 63u) * 16u;
            pcf[j] = ((unsigned)col >> 6) * 16384u + ((unsigned)col & 63u) * 16u;
        }
        steps = nullptr;
        const int grp = threadIdx.x / T::BM, within = threadIdx.x % T::BM;
        xsrc = p.xp + ((size_t)grp * p.mpad + (size_t)tm * T::BM + within) * 16;
        xstride = (size_t)XGRP_PER_PASS * p.mpad * 16;
    }

    // Table of the segment that starts at position ks0 of the stacked contraction and has L
    // steps (all threads; the caller synchronises).  Rows past the end of the contraction keep
    // a valid address: their activation digits are zero.
    __device__ __forceinline__ void build_table(const GemmParams& p, int* table, int ks0, int L, int KS, int kc) {
        for (int q = threadIdx.x; q < L; q += T::THREADS) {
            const int ks = ks0 + q;
            const int h = ks >= KS ? 1 : 0;
            int s = ks - h * KS;
            if constexpr (LISTED) s = steps[s];
            int n0[2];
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const int k0 = s * KSTEP + 16 * g;
                n0[g] = k0;
                if (GMODE == W_PLANES_GATHER && h == 0) {
                    // bs is a multiple of 16 (host check), so a half lies inside one block
                    const int kb = k0 <= kc - 16 ? k0 : kc - 16;
                    const int blk = kb / p.bs;
                    const long st = block_start(p, blk);
                    n0[g] = (int)(st < 0 ? 0 : st) + (kb - blk * p.bs);
                }
            }
            v4i e = {h * p.ks_cap + s, n0[0], n0[1], h};
            *reinterpret_cast<v4i*>(table + 4 * q) = e;
        }
        tab = table;
    }

    __device__ __forceinline__ void prime() { pend = *reinterpret_cast<const v4i*>(tab); }

    // Fix the step (position q of the segment) the following transfers work on.  Positions are
    // visited in order (q, then q + 1 capped at qlimit), which lets the entry of the next one be
    // read here, a whole step before it is needed.
    __device__ __forceinline__ void begin(const GemmParams& p, int q, int, int, int qlimit) {
        const int xg = __builtin_amdgcn_readfirstlane(pend.x);
        n0a = __builtin_amdgcn_readfirstlane(pend.y);
        n0b = __builtin_amdgcn_readfirstlane(pend.z);
        const int h2 = __builtin_amdgcn_readfirstlane(pend.w);
        const int qn = q + 1 < qlimit ? q + 1 : qlimit;
        pend = *reinterpret_cast<const v4i*>(tab + 4 * qn);
        xs2 = xsrc + (size_t)xg * 16 * p.mpad * 16;
        pbase = reinterpret_cast<const char*>(h2 ? p.F : p.B);
        prow = (size_t)(((h2 ? p.ldf : p.ldb) + 63) >> 6) * 16384u;
#pragma unroll
        for (int j = 0; j < WV; ++j) pcsel[j] = pcb[j] + ((pcf[j] - pcb[j]) & (0u - (unsigned)h2));
    }

    template <int J>
    __device__ __forceinline__ void xdma_piece(unsigned char* xstage) {
        const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
        const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) void*)xstage;
        const unsigned lds = __builtin_amdgcn_readfirstlane(lds0 + (wave * 64 + T::THREADS * J) * 16);
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                     :
                     : "s"(lds), "v"(xs2 + J * xstride)
                     : "memory", "m0");
    }

    // run (digit t, k-half g) of the weight stage: scalar start of the run in the operand, the
    // lane's column offset, one transfer per wavefront
    template <int J>
    __device__ __forceinline__ void wdma_piece(unsigned char* wstage) {
        const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
        const int run = __builtin_amdgcn_readfirstlane((int)((threadIdx.x + T::THREADS * J) / T::BN));   // t * 2 + g
        const int r0 = (run & 1) ? n0b : n0a;
        const char* sb = pbase + (size_t)(r0 >> 5) * prow + (size_t)((run & ~1) | ((r0 >> 4) & 1)) * 1024u;
        const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) void*)wstage;
        const unsigned lds = __builtin_amdgcn_readfirstlane(lds0 + (wave * 64 + T::THREADS * J) * 16);
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :
                     : "s"(lds), "v"(pcsel[J]), "s"(sb)
                     : "memory", "m0");
    }

    template <int P, bool SPLIT>
    __device__ __forceinline__ void piece(const GemmParams&, int, unsigned char* xstage, unsigned char* wstage) {
        if constexpr (P < XV) xdma_piece<P>(xstage);
        else if constexpr (P < P_END) wdma_piece<P - XV>(wstage);
    }

    template <int P0, bool SPLIT, int... Ps>
    __device__ __forceinline__ void pieces(std::integer_sequence<int, Ps...>, const GemmParams& p,
                                           int kc, unsigned char* xstage, unsigned char* wstage) {
        (piece<P0 + Ps, SPLIT>(p, kc, xstage, wstage), ...);
    }
};

__device__ __forceinline__ v4i lds_frag(const unsigned char* p) {
    return *reinterpret_cast<const v4i*>(p);
}

// Position of matrix instruction M inside a step: activation digit t, weight digit uu, wave
// sub-tiles (ii, j); the accumulator plane is t + uu <= 7.  The 36 digit pairs are walked with
// the digit of the side that has MORE fragments per digit in the outer loop, so that this side's
// fragments are live for one group of instructions only and the other side's are held for the
// step: activation digit outermost for WM >= WN, weight digit outermost for WN > WM (measured on
// the 32 x 256 tile with a row gather: 262 against 330 us on a 938 MB weight side).
template <int WM, int WN>
struct SlotMap {
    static constexpr bool W_OUTER = WN > WM;
    static constexpr int per_outer(int o) { return (8 - o) * WM * WN; }
    static constexpr int outer_of(int m) {
        int o = 0;
        while (m >= per_outer(o)) { m -= per_outer(o); ++o; }
        return o;
    }
    static constexpr int in_outer(int m) {
        int o = 0;
        while (m >= per_outer(o)) { m -= per_outer(o); ++o; }
        return m;
    }
    static constexpr int inner_of(int m) { return in_outer(m) / (WM * WN); }
    static constexpr int t_of(int m) { return W_OUTER ? inner_of(m) : outer_of(m); }
    static constexpr int u_of(int m) { return W_OUTER ? outer_of(m) : inner_of(m); }
    static constexpr int i_of(int m) { return (in_outer(m) / WN) % WM; }
    static constexpr int j_of(int m) { return in_outer(m) % WN; }
};

// Fragment reads of a step: read R < 8 WM is activation fragment a[R / WM][R % WM], the others
// are weight fragments bf[j][uu] with (uu, j) = ((R - 8 WM) / WN, (R - 8 WM) % WN).  slot(R) is
// the matrix instruction after which read R is issued, READ_LEAD instructions ahead of the
// first one that uses it; -1 for the reads issued before the first instruction.
template <int WM, int WN>
struct ReadMap {
    using SM = SlotMap<WM, WN>;
    static constexpr int NR = 8 * (WM + WN);
    static constexpr int NM = 36 * WM * WN;
    static constexpr int READ_LEAD = 8;
    static constexpr bool is_a(int r) { return r < 8 * WM; }
    static constexpr int need(int r) {
        for (int m = 0; m < NM; ++m) {
            if (is_a(r)) {
                if (SM::t_of(m) == r / WM && SM::i_of(m) == r % WM) return m;
            } else {
                if (SM::u_of(m) == (r - 8 * WM) / WN && SM::j_of(m) == (r - 8 * WM) % WN) return m;
            }
        }
        return NM;
    }
    static constexpr int slot(int r) { return need(r) - READ_LEAD < 0 ? -1 : need(r) - READ_LEAD; }
};

// One contraction step of a workgroup: 36 * WM * WN matrix instructions on the
// fragments of activation stage xs and weight stage ws, each followed by its
// share of the look-ahead pieces (see Loader).  The scheduling fences keep the
// compiler from regrouping them.  ks_next2 is clamped by the caller: past the
// end of a segment the look-ahead work is redundant but harmless.
template <class T, class L, int WM, int WN, int... Ms>
__device__ __forceinline__ void gemm_step_impl(std::integer_sequence<int, Ms...>, const GemmParams& p,
                                               L& ld, v16i (&acc)[WM][WN][8],
                                               const unsigned char* xs, const unsigned char* ws,
                                               unsigned char* ws_next, unsigned char* xs_next2,
                                               int a_off, int b_off, int ks_next2, int ks_limit, int KS, int kc) {
    using SM = SlotMap<WM, WN>;
    constexpr int NM = 36 * WM * WN;
    v4i bf[WN][8];
    v4i a[8][WM];
    ld.begin(p, ks_next2, KS, kc, ks_limit);
    // Fragment reads are issued in the order the matrix instructions consume them, each
    // READ_LEAD instructions ahead of its first use: the first instruction of a step then waits
    // for a handful of reads instead of the whole step's, and a fragment of a late digit plane
    // does not hold its registers through the early ones.
    using RM = ReadMap<WM, WN>;
    auto read_frag = [&](auto rc) {
        constexpr int R = decltype(rc)::value;
        if constexpr (RM::is_a(R)) {
            constexpr int t = R / WM, ii = R % WM;
            a[t][ii] = lds_frag(xs + a_off + (t * 2 * T::BM + ii * 32) * 16);
        } else {
            constexpr int uu = (R - 8 * WM) / WN, j = (R - 8 * WM) % WN;
            bf[j][uu] = lds_frag(ws + b_off + (uu * 2 * T::BN + j * 32) * 16);
        }
    };
    auto reads_at = [&](auto slot) {
        constexpr int S = decltype(slot)::value;
        [&]<int... Rs>(std::integer_sequence<int, Rs...>) {
            ([&] { if constexpr (RM::slot(Rs) == S) read_frag(std::integral_constant<int, Rs>{}); }(), ...);
        }(std::make_integer_sequence<int, RM::NR>{});
    };
    reads_at(std::integral_constant<int, -1>{});
    __builtin_amdgcn_sched_barrier(0);
    (
        [&] {
            constexpr int M = Ms;
            constexpr int t = SM::t_of(M), uu = SM::u_of(M), ii = SM::i_of(M), j = SM::j_of(M);
            acc[ii][j][t + uu] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[t][ii], bf[j][uu],
                                                                        acc[ii][j][t + uu], 0, 0, 0);
            reads_at(std::integral_constant<int, M>{});
            constexpr int p0 = (int)((long)M * L::P_END / NM), p1 = (int)((long)(M + 1) * L::P_END / NM);
            ld.template pieces<p0, true>(std::make_integer_sequence<int, p1 - p0>{}, p, kc, xs_next2, ws_next);
            __builtin_amdgcn_sched_barrier(0);
        }(),
        ...);
    // The activation planes of the next step were requested one step ago; only the loads
    // issued during this step may still be in flight past this point.
    wait_and_barrier<L::VM_PER_STEP>();
}

template <class T, class L, int WM, int WN>
__device__ __forceinline__ void gemm_step(const GemmParams& p, L& ld,
                                          v16i (&acc)[WM][WN][8], const unsigned char* xs,
                                          const unsigned char* ws, unsigned char* ws_next,
                                          unsigned char* xs_next2, int a_off, int b_off,
                                          int ks_next2, int ks_limit, int KS, int kc) {
    gemm_step_impl<T, L, WM, WN>(std::make_integer_sequence<int, 36 * WM * WN>{}, p, ld, acc,
                                 xs, ws, ws_next, xs_next2, a_off, b_off, ks_next2, ks_limit, KS, kc);
}

// ---------------------------------------------------------------------------
// step with the barrier in its middle (weight planes)
// ---------------------------------------------------------------------------
// With both operands arriving by LDS-DMA a step has nothing left to hide in the shadow of its
// matrix instructions, and what then costs time is the step boundary: a barrier, and behind it a
// full LDS round trip before the first matrix instruction has its fragments.  So here
//   * the digit pairs are walked with the activation digit DESCENDING (7, 6, .., 0; weight digit
//     ascending inside), which makes every fragment that the first instructions of a step need
//     dead in the last instructions of the step before;
//   * fragment reads run READ_LEAD instructions ahead straight across the step boundary: the last
//     instructions of step i already read, from the stage of step i + 1, what the first ones of
//     step i + 1 consume;
//   * the barrier sits in the MIDDLE of the step.  Barrier b_i publishes the stage of step i + 1
//     (requested after b_(i-1), a whole step earlier), so reads of that stage may start right
//     after it, and it retires the stage of step i - 1 (every wavefront's reads of it are older
//     than its b_i), which the transfers for step i + 2, issued behind b_i, then overwrite.
// No instruction after a barrier waits for a read that was issued after that barrier.
template <int WM, int WN>
struct SlotMapDesc {
    static constexpr int per_group(int g) { return (g + 1) * WM * WN; }      // group g holds digit t = 7 - g
    static constexpr int group_of(int m) {
        int g = 0;
        while (m >= per_group(g)) { m -= per_group(g); ++g; }
        return g;
    }
    static constexpr int in_group(int m) {
        int g = 0;
        while (m >= per_group(g)) { m -= per_group(g); ++g; }
        return m;
    }
    static constexpr int t_of(int m) { return 7 - group_of(m); }
    static constexpr int u_of(int m) { return in_group(m) / (WM * WN); }
    static constexpr int i_of(int m) { return (in_group(m) / WN) % WM; }
    static constexpr int j_of(int m) { return in_group(m) % WN; }
};

template <int WM, int WN>
struct ReadMapMid {
    using SM = SlotMapDesc<WM, WN>;
    static constexpr int NR = 8 * (WM + WN);
    static constexpr int NM = 36 * WM * WN;
    static constexpr int READ_LEAD = 8;
    static constexpr int MID = NM / 2;
    static_assert(READ_LEAD < NM - MID, "reads of the next stage start behind the barrier");
    static constexpr bool is_a(int r) { return r < 8 * WM; }
    static constexpr int need(int r) {
        for (int m = 0; m < NM; ++m) {
            if (is_a(r)) {
                if (SM::t_of(m) == r / WM && SM::i_of(m) == r % WM) return m;
            } else {
                if (SM::u_of(m) == (r - 8 * WM) / WN && SM::j_of(m) == (r - 8 * WM) % WN) return m;
            }
        }
        return NM;
    }
    // instruction of the SAME step after which read R is issued, or, when negative, NM + slot is
    // the instruction of the step BEFORE after which it is issued
    static constexpr int slot(int r) { return need(r) - READ_LEAD; }
};

template <class T, int WM, int WN, int R>
__device__ __forceinline__ void read_frag_mid(v4i (&a)[8][WM], v4i (&bf)[WN][8], const unsigned char* xs,
                                              const unsigned char* ws, int a_off, int b_off) {
    using RM = ReadMapMid<WM, WN>;
    if constexpr (RM::is_a(R)) {
        constexpr int t = R / WM, ii = R % WM;
        a[t][ii] = lds_frag(xs + a_off + (t * 2 * T::BM + ii * 32) * 16);
    } else {
        constexpr int uu = (R - 8 * WM) / WN, j = (R - 8 * WM) % WN;
        bf[j][uu] = lds_frag(ws + b_off + (uu * 2 * T::BN + j * 32) * 16);
    }
}

// the reads a step's first instructions need, issued before the first step of a segment
template <class T, int WM, int WN>
__device__ __forceinline__ void prefetch_first_frags(v4i (&a)[8][WM], v4i (&bf)[WN][8], const unsigned char* xs,
                                                     const unsigned char* ws, int a_off, int b_off) {
    using RM = ReadMapMid<WM, WN>;
    [&]<int... Rs>(std::integer_sequence<int, Rs...>) {
        ([&] { if constexpr (RM::slot(Rs) < 0) read_frag_mid<T, WM, WN, Rs>(a, bf, xs, ws, a_off, b_off); }(), ...);
    }(std::make_integer_sequence<int, RM::NR>{});
}

template <class T, class L, int WM, int WN, int... Ms>
__device__ __forceinline__ void gemm_step_mid_impl(std::integer_sequence<int, Ms...>, const GemmParams& p, L& ld,
                                                   v16i (&acc)[WM][WN][8], v4i (&a)[8][WM], v4i (&bf)[WN][8],
                                                   const unsigned char* xs, const unsigned char* ws,
                                                   const unsigned char* xs_next, const unsigned char* ws_next,
                                                   unsigned char* xs_fill, unsigned char* ws_fill, int a_off,
                                                   int b_off, int q_fill, int q_limit, int KS, int kc) {
    using SM = SlotMapDesc<WM, WN>;
    using RM = ReadMapMid<WM, WN>;
    constexpr int NM = RM::NM, MID = RM::MID;
    (
        [&] {
            constexpr int M = Ms;
            if constexpr (M == MID) {
                // b_i: this wavefront's transfers for the next step have landed and its reads of the
                // previous step's stage are done; behind the barrier that holds for all wavefronts
                wait_and_barrier<0>();
                ld.begin(p, q_fill, KS, kc, q_limit);
            }
            constexpr int t = SM::t_of(M), uu = SM::u_of(M), ii = SM::i_of(M), j = SM::j_of(M);
            acc[ii][j][t + uu] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[t][ii], bf[j][uu],
                                                                        acc[ii][j][t + uu], 0, 0, 0);
            // reads for this step (its own stage) and, near the end, for the first instructions of
            // the next step (the next stage, published by this step's barrier)
            [&]<int... Rs>(std::integer_sequence<int, Rs...>) {
                ([&] {
                    if constexpr (RM::slot(Rs) == M) read_frag_mid<T, WM, WN, Rs>(a, bf, xs, ws, a_off, b_off);
                    if constexpr (RM::slot(Rs) + NM == M)
                        read_frag_mid<T, WM, WN, Rs>(a, bf, xs_next, ws_next, a_off, b_off);
                }(), ...);
            }(std::make_integer_sequence<int, RM::NR>{});
            if constexpr (M >= MID) {
                constexpr int p0 = (int)((long)(M - MID) * L::P_END / (NM - MID)),
                              p1 = (int)((long)(M - MID + 1) * L::P_END / (NM - MID));
                ld.template pieces<p0, true>(std::make_integer_sequence<int, p1 - p0>{}, p, kc, xs_fill, ws_fill);
            }
            __builtin_amdgcn_sched_barrier(0);
        }(),
        ...);
}

template <class T, class L, int WM, int WN>
__device__ __forceinline__ void gemm_step_mid(const GemmParams& p, L& ld, v16i (&acc)[WM][WN][8],
                                              v4i (&a)[8][WM], v4i (&bf)[WN][8], const unsigned char* xs,
                                              const unsigned char* ws, const unsigned char* xs_next,
                                              const unsigned char* ws_next, unsigned char* xs_fill,
                                              unsigned char* ws_fill, int a_off, int b_off, int q_fill,
                                              int q_limit, int KS, int kc) {
    gemm_step_mid_impl<T, L, WM, WN>(std::make_integer_sequence<int, 36 * WM * WN>{}, p, ld, acc, a, bf, xs, ws,
                                     xs_next, ws_next, xs_fill, ws_fill, a_off, b_off, q_fill, q_limit, KS, kc);
}

// What a launch computes, from the device-resident counts.
struct Geometry {
    int n_eff, kc, KS, KT, m_eff, tiles_m, tiles_n, tiles;
    long units;     // work units: (tile, contraction step) pairs
};

template <class T, int KIND, bool LISTED>
__device__ __forceinline__ Geometry gemm_geometry(const GemmParams& p) {
    Geometry q;
    const int nblk = n_blocks(p);
    q.n_eff = KIND == KIND_SOMM ? nblk * p.bs : p.n_cap;
    q.kc = KIND == KIND_SOMM ? p.kc_cap : nblk * p.bs;
    q.KS = (q.kc + KSTEP - 1) / KSTEP;
    q.KT = 2 * q.KS;
    q.m_eff = n_rows(p);
    q.tiles_m = (q.m_eff + T::BM - 1) / T::BM;
    q.tiles_n = (q.n_eff + T::BN - 1) / T::BN;
    // with result blocks only the listed tiles are computed
    q.tiles = p.row_comp ? p.tile_list[0] : q.tiles_m * q.tiles_n;
    // with per-token row sets only the listed steps of each row tile are computed
    q.units = LISTED ? (long)q.tiles_n * 2 * p.step_off[q.tiles_m] : (long)q.tiles * q.KT;
    return q;
}

// The work units [u, u_end) of one product: segment by segment (a run of contraction steps of one
// output tile), the main loop and the write-out of the partial sum.  G: workgroups of the launch.
template <int WAVES_M, int WAVES_N, int WM, int WN, int KIND, int GMODE, bool LISTED>
__device__ __forceinline__ void gemm_sweep(const GemmParams& p, const Geometry& q, long u, const long u_end,
                                           const int G, const bool own, unsigned char* xs0, unsigned char* xs1,
                                           unsigned char* xs2, unsigned char* wsm, int* steptab,
                                           const int team_tm = -1) {
    using T = Tile<WAVES_M, WAVES_N, WM, WN>;
    constexpr bool PLANES = is_planes(GMODE);
    using LD = std::conditional_t<PLANES, PlaneLoader<T, KIND, GMODE, LISTED>, Loader<T, KIND, GMODE, LISTED>>;
    constexpr bool listed = LISTED;
    const int n_eff = q.n_eff, kc = q.kc, KS = q.KS, KT = q.KT, m_eff = q.m_eff;
    // team_tm >= 0: this workgroup computes row tile team_tm only and the units are (column tile,
    // contraction step) pairs; the workgroups of a team walk the same units side by side
    const int tiles_m = q.tiles_m, tiles_n = q.tiles_n, tiles = team_tm >= 0 ? q.tiles_n : q.tiles;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave % WAVES_M, wn = wave / WAVES_M;
    const int g = lane >> 5, r = lane & 31;
    // this lane's fragment offsets inside a stage (digit 0)
    const int a_off = (g * T::BM + wm * WM * 32 + r) * 16;
    const int b_off = (g * T::BN + wn * WN * 32 + r) * 16;

    LD ld;
    const long u_begin = u;

    // Work units are ordered chunk-major: all tiles for contraction steps
    // [0, CH), then all tiles for [CH, 2 CH), ...  Workgroups that run side by
    // side therefore sweep the same slice of the contraction at the same time
    // (the activation planes of that slice stay hot in L2) and each XCD ends up
    // with whole slices, so a weight word is fetched from HBM by one XCD only.
    int CH = p.chunk;
    // every workgroup owns whole tiles: units tile by tile, all of a tile's contraction in a row
    if (own) CH = KT;
    if (p.row_comp) {
        // the number of listed tiles is only known here: as many slices as workgroups per tile
        int slices = (int)((G + tiles / 2) / tiles);
        if (slices < 1) slices = 1;
        CH = (KT + slices - 1) / slices;
        if (CH > MAX_SEG) CH = MAX_SEG;
        if (CH < 1) CH = 1;
    }
    const long full_chunk_units = (long)tiles * CH;
    const int n_chunks = (KT + CH - 1) / CH;
    while (u < u_end) {
        int tm, tn, ks0, KSt = KS;
        long len;
        const int* listed_steps = nullptr;
        if (listed) {
            // units are ordered row tile by row tile, inside a row tile column tile by column
            // tile, inside a tile along its listed steps (E B_i half, then A' F half)
            int lo = 0, hi = tiles_m;
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if ((long)tiles_n * 2 * p.step_off[mid] <= u) lo = mid; else hi = mid;
            }
            tm = lo;
            KSt = p.step_cnt[tm];
            const long rem = u - (long)tiles_n * 2 * p.step_off[tm];
            tn = (int)(rem / (2 * KSt));
            ks0 = (int)(rem - (long)tn * 2 * KSt);
            len = 2 * KSt - ks0;
            if (len > MAX_SEG) len = MAX_SEG;
            listed_steps = p.step_list + (size_t)tm * p.ks_cap;
        } else {
            int c = (int)(u / full_chunk_units);
            if (c > n_chunks - 1) c = n_chunks - 1;
            const long rem = u - (long)c * full_chunk_units;
            const int clen = (c == n_chunks - 1) ? KT - c * CH : CH;
            const int tile_pos = (int)(rem / clen);
            ks0 = c * CH + (int)(rem - (long)tile_pos * clen);
            const int tile = p.row_comp ? p.tile_list[1 + tile_pos] : tile_pos;
            len = c * CH + clen - ks0;
            if (len > MAX_SEG) len = MAX_SEG;      // (an owned tile's contraction may be longer than a segment)
            tm = tile % tiles_m;
            tn = tile / tiles_m;
            if (team_tm >= 0) { tm = team_tm; tn = tile; }
        }
        if (len > u_end - u) len = u_end - u;
        const int L = (int)len;
        if (!listed && p.k_rotate) {
            // Units tile by tile, a tile cut into parts by the workgroup ranges: the parts take their
            // contraction steps in reverse order of their positions (the part [c, d) of a tile gets
            // the steps [KT - d, KT - c); any order gives the same sum).  A workgroup that starts
            // in the middle of a tile thus begins at step 0 like one that starts on a tile, and
            // all workgroups sweep the contraction in two phases only, KT - share apart: the
            // activation planes of a phase are shared through L2 instead of being fetched per tile.
            const long tile_u0 = u - ks0;
            const long c_lo = u_begin - tile_u0, c_hi = u_end - tile_u0;
            ks0 += KT - (c_lo > 0 ? (int)c_lo : 0) - (c_hi < KT ? (int)c_hi : KT);
        }

        ld.setup(p, tm, tn, n_eff);
        ld.steps = listed_steps;
        v16i acc[WM][WN][8];
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int j = 0; j < WN; ++j)
#pragma unroll
                for (int s = 0; s < 8; ++s)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[i][j][s][e] = 0;

        // prologue: step ks0 staged, step ks0+1 in flight
        const int ks_last = ks0 + L - 1;
        if constexpr (PLANES) {
            // the segment's step table first (the stages and the table of the previous segment
            // are no longer read: every wavefront has passed that segment's last barrier)
            ld.build_table(p, steptab, ks0, L, KSt, kc);
            __syncthreads();
            ld.prime();
            ld.begin(p, 0, KSt, kc, L - 1);
            ld.template pieces<0, true>(std::make_integer_sequence<int, LD::P_END>{}, p, kc, xs0, wsm);
            ld.begin(p, 1 < L - 1 ? 1 : L - 1, KSt, kc, L - 1);
            ld.template pieces<0, true>(std::make_integer_sequence<int, LD::P_END>{}, p, kc, xs1, wsm + T::WBYTES);
            wait_and_barrier<0>();
            // Positions of the segment instead of contraction steps; stage i % 3 of both operands.
            // Step i reads stage i % 3, prefetches from stage (i + 1) % 3 and, behind its barrier,
            // requests position i + 2 into stage (i + 2) % 3.
            v4i fa[8][WM], fb[WN][8];
            prefetch_first_frags<T, WM, WN>(fa, fb, xs0, wsm, a_off, b_off);
            for (int i = 0; i < L; i += 3) {
                const int q2 = i + 2;
                gemm_step_mid<T, LD, WM, WN>(p, ld, acc, fa, fb, xs0, wsm, xs1, wsm + T::WBYTES, xs2,
                                             wsm + 2 * T::WBYTES, a_off, b_off, q2 < L - 1 ? q2 : L - 1, L - 1,
                                             KSt, kc);
                if (i + 1 < L)
                    gemm_step_mid<T, LD, WM, WN>(p, ld, acc, fa, fb, xs1, wsm + T::WBYTES, xs2,
                                                 wsm + 2 * T::WBYTES, xs0, wsm, a_off, b_off,
                                                 q2 + 1 < L - 1 ? q2 + 1 : L - 1, L - 1, KSt, kc);
                if (i + 2 < L)
                    gemm_step_mid<T, LD, WM, WN>(p, ld, acc, fa, fb, xs2, wsm + 2 * T::WBYTES, xs0, wsm, xs1,
                                                 wsm + T::WBYTES, a_off, b_off, q2 + 2 < L - 1 ? q2 + 2 : L - 1,
                                                 L - 1, KSt, kc);
            }
        } else {
            ld.prime(p, ks0, KSt, kc);
            ld.begin(p, ks0, KSt, kc, ks_last);
            ld.template pieces<LD::P_DMA, false>(std::make_integer_sequence<int, LD::P_END - LD::P_DMA>{}, p, kc, xs0, wsm);
            ld.begin(p, ks0 + 1 < ks_last ? ks0 + 1 : ks_last, KSt, kc, ks_last);
            ld.template pieces<LD::P_DMA, true>(std::make_integer_sequence<int, LD::P_END - LD::P_DMA>{}, p, kc, xs1, wsm);
            wait_and_barrier<0>();

            for (int i = 0; i < L; i += 3) {
                const int k2 = ks0 + i + 2;
                gemm_step<T, LD, WM, WN>(p, ld, acc, xs0, wsm + (i & 1) * T::WBYTES,
                                         wsm + ((i + 1) & 1) * T::WBYTES, xs2, a_off, b_off,
                                         k2 < ks_last ? k2 : ks_last, ks_last, KSt, kc);
                if (i + 1 < L)
                    gemm_step<T, LD, WM, WN>(p, ld, acc, xs1, wsm + ((i + 1) & 1) * T::WBYTES,
                                             wsm + (i & 1) * T::WBYTES, xs0, a_off, b_off,
                                             k2 + 1 < ks_last ? k2 + 1 : ks_last, ks_last, KSt, kc);
                if (i + 2 < L)
                    gemm_step<T, LD, WM, WN>(p, ld, acc, xs2, wsm + (i & 1) * T::WBYTES,
                                             wsm + ((i + 1) & 1) * T::WBYTES, xs1, a_off, b_off,
                                             k2 + 2 < ks_last ? k2 + 2 : ks_last, ks_last, KSt, kc);
            }
        }
        // the look-ahead transfers of the last steps are redundant; let them land before the
        // stages are reused
        wait_and_barrier<0>();

        // recombine the eight planes and add the partial sum onto Z
        auto recombine = [&](int i, int j, int e) -> u64 {
            // sum_s sext64(S_s) << 8s: the four low planes as 32 x 32 -> 64 bit signed
            // multiply-adds, the four high planes only reach the upper word
            long long lo = (long long)acc[i][j][0][e];
            lo += (long long)acc[i][j][1][e] * (1 << 8);
            lo += (long long)acc[i][j][2][e] * (1 << 16);
            lo += (long long)acc[i][j][3][e] * (1 << 24);
            const u32 hi = (u32)acc[i][j][4][e] + ((u32)acc[i][j][5][e] << 8) +
                           ((u32)acc[i][j][6][e] << 16) + ((u32)acc[i][j][7][e] << 24);
            return (u64)lo + ((u64)hi << 32);
        };
        // The only writer of a tile (own) stores Z = C + sum (Z += sum for a later segment of a long
        // contraction: this lane's own earlier store, complete since the barrier above); the loads of
        // a sub-tile go out together, ahead of the arithmetic.  Slices of a shared tile meet in Z,
        // which started out as C, through atomic adds.
        const u64* src = ks0 == 0 ? p.C : p.Z;
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int j = 0; j < WN; ++j) {
                const int col = tn * T::BN + (wn * WN + j) * 32 + r;
                const int ccomp = (p.row_comp && col < n_eff) ? p.blk_comp[col / p.bs] : 0;
                u64 prev[16];
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = tm * T::BM + (wm * WM + i) * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
                    prev[e] = 0;
                    if (own && row < m_eff && col < n_eff) prev[e] = src[(size_t)row * p.ldz + col];
                }
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = tm * T::BM + (wm * WM + i) * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
                    const u64 z = recombine(i, j, e);
                    bool live = row < m_eff && col < n_eff;
                    if (live && p.row_comp) live = p.row_comp[row] == ccomp;   // on a result block
                    if (live) {
                        if (own) p.Z[(size_t)row * p.ldz + col] = prev[e] + z;
                        else atomicAdd(p.Z + (size_t)row * p.ldz + col, z);
                    }
                }
            }
        u += len;
    }
}

// LDS of the kernels: three activation stages filled by LDS-DMA two steps ahead, as separate
// arrays so that the compiler can tell a stage being filled from the one
// being read; two weight stages written from registers one step ahead (three, filled by
// LDS-DMA, for weight planes, with the step table of a segment).
#define COMET_GEMM_LDS(T, GMODE)                                                        \
    __shared__ __align__(16) unsigned char xs0[T::XBYTES];                              \
    __shared__ __align__(16) unsigned char xs1[T::XBYTES];                              \
    __shared__ __align__(16) unsigned char xs2[T::XBYTES];                              \
    __shared__ __align__(16) unsigned char wsm[T::wstages(GMODE) * T::WBYTES];          \
    __shared__ __align__(16) int steptab[is_planes(GMODE) ? MAX_SEG * 4 : 4]

// Workgroups are dealt round-robin to the 8 XCDs; give each XCD one contiguous range of work.
__device__ __forceinline__ int xcd_contiguous(int b, int G) {
    return (G & 7) == 0 ? (b & 7) * (G >> 3) + (b >> 3) : b;
}

// OWN: the variant for launches planned so that every workgroup gets whole output tiles (see
// owns_tiles()); it still checks that on the device, where the counts are, and falls back to the
// shared-tile path.  The other variant never owns: it carries none of that code.
template <int WAVES_M, int WAVES_N, int WM, int WN, int KIND, int GMODE, bool LISTED, bool OWN = false>
__global__ __launch_bounds__((Tile<WAVES_M, WAVES_N, WM, WN>::THREADS), (Tile<WAVES_M, WAVES_N, WM, WN>::wg_per_cu(GMODE))) void ring_gemm_kernel(GemmParams p) {
    using T = Tile<WAVES_M, WAVES_N, WM, WN>;
    COMET_GEMM_LDS(T, GMODE);
    if (p.tile_sel && *p.tile_sel != p.tile_sel_want) return;   // the other tile shape was chosen
    const Geometry q = gemm_geometry<T, KIND, LISTED>(p);
    if (q.units == 0) return;
    const int G = gridDim.x;
    const int b = xcd_contiguous(blockIdx.x, G);
    bool own = false;
    if constexpr (OWN) own = owns_tiles(p, q.m_eff, q.n_eff, q.kc);
    gemm_sweep<WAVES_M, WAVES_N, WM, WN, KIND, GMODE, LISTED>(p, q, q.units * b / G, q.units * (b + 1) / G, G, own,
                                                             xs0, xs1, xs2, wsm, steptab);
}

// Several products of one shape and one index list (so: one geometry) in one launch: the work
// units of the members follow each other, tile by tile inside a member, and the workgroups share
// out the whole sequence.  A workgroup's range may run across members.
constexpr int GROUP_MAX = COMET_SHARE_GROUP_MAX;
struct GemmGroup {
    int n;
    GemmParams p[GROUP_MAX];
};

template <int WAVES_M, int WAVES_N, int WM, int WN, int KIND, int GMODE, bool OWN>
__global__ __launch_bounds__((Tile<WAVES_M, WAVES_N, WM, WN>::THREADS), (Tile<WAVES_M, WAVES_N, WM, WN>::wg_per_cu(GMODE))) void ring_gemm_group_kernel(GemmGroup grp) {
    using T = Tile<WAVES_M, WAVES_N, WM, WN>;
    COMET_GEMM_LDS(T, GMODE);
    const Geometry q = gemm_geometry<T, KIND, false>(grp.p[0]);
    if (q.units == 0) return;
    const int G = gridDim.x;
    const int b = xcd_contiguous(blockIdx.x, G);
    // Teams: when the row tiles divide the grid, tiles_m consecutive workgroups (same XCD) form a
    // team that walks one sequence of (column tile, contraction step) units, each member for its
    // own row tile: the weight planes of a unit are fetched once for all row tiles, in lockstep.
    const bool team = grp.p[0].team && q.tiles_m > 1 && G % q.tiles_m == 0;
    const long units = team ? q.units / q.tiles_m : q.units;        // of one member
    const int parts = team ? G / q.tiles_m : G, part = team ? b / q.tiles_m : b;
    const long total = units * grp.n;
    long u = total * part / parts;
    const long u_end = total * (part + 1) / parts;
    bool own = false;
    if constexpr (OWN) own = owns_tiles(grp.p[0], q.m_eff, q.n_eff, q.kc);
#pragma nounroll
    for (int j = (int)(u / units); u < u_end; ++j) {
        const long base = (long)j * units;
        const long hi = u_end - base < units ? u_end - base : units;
        gemm_sweep<WAVES_M, WAVES_N, WM, WN, KIND, GMODE, false>(grp.p[j], q, u - base, hi, G, own, xs0, xs1, xs2,
                                                                 wsm, steptab, team ? b % q.tiles_m : -1);
        u = base + units;
    }
}

// The kernel variant for a call: the kind of product, how the weight side is addressed, and
// (LISTED) whether a step list is walked.  Instantiated explicitly, one translation unit per
// (tile shape, LISTED), so that the variants compile side by side.
using GemmKernel = void (*)(GemmParams);

// the OWN variants (128 x 64 tile, no step lists): translation units of their own
template <int WAVES_M, int WAVES_N, int WM, int WN>
GemmKernel gemm_own_planes_kernel_for(const GemmParams& p) {
    if (p.kind == KIND_SIMM) {
        if (p.b_full) return ring_gemm_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SIMM, W_PLANES_GATHER, false, true>;
        return ring_gemm_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SIMM, W_PLANES, false, true>;
    }
    return ring_gemm_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SOMM, W_PLANES, false, true>;
}
extern template GemmKernel gemm_own_planes_kernel_for<2, 2, 2, 1>(const GemmParams&);

template <int WAVES_M, int WAVES_N, int WM, int WN>
GemmKernel gemm_own_kernel_for(const GemmParams& p) {
    if (p.kind == KIND_SIMM) {
        if (!p.b_full) return ring_gemm_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SIMM, GATHER_NONE, false, true>;
        if (p.bs_shift >= 3) return ring_gemm_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SIMM, GATHER_POW2, false, true>;
        return ring_gemm_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SIMM, GATHER_ANY, false, true>;
    }
    if (p.w_tr) return ring_gemm_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SOMM, WEIGHTS_TR, false, true>;
    return ring_gemm_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SOMM, GATHER_NONE, false, true>;
}
extern template GemmKernel gemm_own_kernel_for<2, 2, 2, 1>(const GemmParams&);

template <int WAVES_M, int WAVES_N, int WM, int WN, bool LISTED>
GemmKernel gemm_kernel_for(const GemmParams& p) {
    if (p.kind == KIND_SIMM) {
        if (!p.b_full) return ring_gemm_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SIMM, GATHER_NONE, LISTED>;
        if (p.bs_shift >= 3) return ring_gemm_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SIMM, GATHER_POW2, LISTED>;
        return ring_gemm_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SIMM, GATHER_ANY, LISTED>;
    }
    if constexpr (LISTED) {
        return nullptr;      // step lists belong to Protocol 3
    } else {
        if (p.w_tr) return ring_gemm_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SOMM, WEIGHTS_TR, false>;
        return ring_gemm_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SOMM, GATHER_NONE, false>;
    }
}

// The variants that read weight planes: their own translation units (ring_gemm_planes_*.hip).
template <int WAVES_M, int WAVES_N, int WM, int WN, bool LISTED>
GemmKernel gemm_planes_kernel_for(const GemmParams& p) {
    if (p.kind == KIND_SIMM) {
        if (p.b_full) return ring_gemm_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SIMM, W_PLANES_GATHER, LISTED>;
        return ring_gemm_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SIMM, W_PLANES, LISTED>;
    }
    if constexpr (LISTED) {
        return nullptr;
    } else {
        return ring_gemm_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SOMM, W_PLANES, false>;
    }
}

extern template GemmKernel gemm_planes_kernel_for<2, 2, 2, 1, false>(const GemmParams&);
extern template GemmKernel gemm_planes_kernel_for<2, 2, 1, 1, false>(const GemmParams&);
extern template GemmKernel gemm_planes_kernel_for<2, 2, 1, 1, true>(const GemmParams&);
extern template GemmKernel gemm_planes_kernel_for<1, 4, 1, 1, false>(const GemmParams&);
extern template GemmKernel gemm_planes_kernel_for<1, 4, 1, 1, true>(const GemmParams&);

extern template GemmKernel gemm_kernel_for<2, 2, 2, 1, false>(const GemmParams&);
extern template GemmKernel gemm_kernel_for<2, 2, 1, 1, false>(const GemmParams&);
extern template GemmKernel gemm_kernel_for<2, 2, 1, 1, true>(const GemmParams&);
extern template GemmKernel gemm_kernel_for<1, 4, 1, 2, false>(const GemmParams&);
extern template GemmKernel gemm_kernel_for<1, 4, 1, 2, true>(const GemmParams&);

// Launch plan of the matrix-core kernel for an output tile BM x BN: the grid, the slice length and
// whether the launch may turn out to own its tiles.  Fixed before the packing kernel is launched,
// which has to know whether the share kernel will initialise Z itself.
inline void plan_gemm(const comet_ctx* ctx, GemmParams& p, int BM, int BN, int wg_per_cu) {
    const long tiles = (long)((p.m + BM - 1) / BM) * ((p.n_cap + BN - 1) / BN);
    const long kt = 2l * p.ks_cap;
    const long units_cap = tiles * kt;
    // a chip-sized grid, shrunk when there is too little work to share out
    long grid = (ctx->num_cu / 8) * 8 * wg_per_cu;
    if (grid < 8) grid = 8;
    const long want = (units_cap + 1) / 2;      // at least two contraction steps per workgroup
    if (want < grid) grid = want < 8 ? (want < 1 ? 1 : want) : (want / 8) * 8;
    if (ctx->gemm_grid > 0) grid = ctx->gemm_grid;
    // Slice length: as many slices as there are workgroups per tile, so that a workgroup's
    // share of the units is one slice of one tile and all workgroups sweep their slice in
    // lockstep (the activation planes of a slice are then shared through L2).
    if (ctx->gemm_chunk > 0) {
        p.chunk = ctx->gemm_chunk;
    } else {
        long slices = (grid + tiles / 2) / tiles;
        if (slices < 1) slices = 1;
        p.chunk = (int)((kt + slices - 1) / slices);
    }
    if (p.chunk > MAX_SEG) p.chunk = MAX_SEG;
    if (p.chunk < 1) p.chunk = 1;
    p.grid = (int)grid;
    p.tile_bm = BM;
    p.tile_bn = BN;
    // Owned tiles: plain product, default slicing, the 128 x 64 tile, and a tile count (at full
    // capacity; the kernel checks the device-resident counts) that the grid divides
    p.own_try = (!p.row_comp && !p.tmask && ctx->gemm_chunk == 0 && BM == 128 && tiles % grid == 0) ? 1 : 0;
}

template <int WAVES_M, int WAVES_N, int WM, int WN>
int launch_gemm(comet_ctx* ctx, const char* what, GemmParams p) {
    using T = Tile<WAVES_M, WAVES_N, WM, WN>;
    GemmKernel kern = nullptr;
    constexpr bool PLANES_ONLY = WAVES_N == 4 && WN == 1;     // the 32 x 128 tile exists for weight planes only
    constexpr bool WORDS_ONLY = WAVES_N == 4 && WN == 2;      // the 32 x 256 tile needs two weight stages
    constexpr bool HAS_OWN = WM * WN == 2 && WAVES_N == 2;    // the 128 x 64 tile
    if (p.own_try) {
        if constexpr (HAS_OWN)
            kern = p.w_planes ? gemm_own_planes_kernel_for<WAVES_M, WAVES_N, WM, WN>(p)
                              : gemm_own_kernel_for<WAVES_M, WAVES_N, WM, WN>(p);
    } else if (p.w_planes) {
        if constexpr (WORDS_ONLY) {
            kern = nullptr;
        } else if (p.step_list) {
            if constexpr (WM * WN == 2 && WAVES_N == 2) kern = nullptr;
            else kern = gemm_planes_kernel_for<WAVES_M, WAVES_N, WM, WN, true>(p);
        } else {
            kern = gemm_planes_kernel_for<WAVES_M, WAVES_N, WM, WN, false>(p);
        }
    } else if constexpr (PLANES_ONLY) {
        kern = nullptr;
    } else if (p.step_list) {
        // per-token row sets: only the tile shapes the dispatch picks for them have such variants
        if constexpr (WM * WN == 2 && WAVES_N == 2) kern = nullptr;
        else kern = gemm_kernel_for<WAVES_M, WAVES_N, WM, WN, true>(p);
    } else {
        kern = gemm_kernel_for<WAVES_M, WAVES_N, WM, WN, false>(p);
    }
    if (!kern) return comet_fail(ctx, COMET_EINVAL, "%s: no kernel variant for this call", what);
    if (p.tile_bm != T::BM || p.tile_bn != T::BN || p.grid < 1)
        return comet_fail(ctx, COMET_EINVAL, "%s: launch plan does not match the kernel", what);
    const long grid = p.grid;
    const bool timed = comet_time_this_launch(ctx);
    if (timed) {
        // the event pair rides on the dispatch itself (its start and end timestamps): no marker
        // packets before or after the kernel, so timing leaves the stream's schedule as it is
        hipExtLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(T::THREADS), 0, ctx->stream, ctx->ev[ctx->ev_used],
                              ctx->ev[ctx->ev_used + 1], 0, p);
        ctx->ev_used += 2;
    } else {
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(T::THREADS), 0, ctx->stream, p);
    }
    COMET_LAUNCH_CHECK(ctx, what);
    return COMET_OK;
}

// The grouped kernel exists for weight planes and the 128 x 64 tile (translation units
// ring_gemm_group_128x64*.hip).
using GemmGroupKernel = void (*)(GemmGroup);

template <int WAVES_M, int WAVES_N, int WM, int WN, bool OWN>
GemmGroupKernel gemm_group_kernel_for(const GemmParams& p) {
    if (p.kind == KIND_SIMM) {
        if (p.b_full) return ring_gemm_group_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SIMM, W_PLANES_GATHER, OWN>;
        return ring_gemm_group_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SIMM, W_PLANES, OWN>;
    }
    return ring_gemm_group_kernel<WAVES_M, WAVES_N, WM, WN, KIND_SOMM, W_PLANES, OWN>;
}
extern template GemmGroupKernel gemm_group_kernel_for<2, 2, 2, 1, false>(const GemmParams&);
extern template GemmGroupKernel gemm_group_kernel_for<2, 2, 2, 1, true>(const GemmParams&);

template <int WAVES_M, int WAVES_N, int WM, int WN>
int launch_gemm_group(comet_ctx* ctx, const char* what, const GemmGroup& grp) {
    using T = Tile<WAVES_M, WAVES_N, WM, WN>;
    const GemmParams& p = grp.p[0];
    if (grp.n < 1 || grp.n > GROUP_MAX || !p.w_planes || p.tile_bm != T::BM || p.tile_bn != T::BN || p.grid < 1)
        return comet_fail(ctx, COMET_EINVAL, "%s: launch plan does not match the grouped kernel", what);
    GemmGroupKernel kern = p.own_try ? gemm_group_kernel_for<WAVES_M, WAVES_N, WM, WN, true>(p)
                                     : gemm_group_kernel_for<WAVES_M, WAVES_N, WM, WN, false>(p);
    if (comet_time_this_launch(ctx)) {
        hipExtLaunchKernelGGL(kern, dim3((unsigned)p.grid), dim3(T::THREADS), 0, ctx->stream, ctx->ev[ctx->ev_used],
                              ctx->ev[ctx->ev_used + 1], 0, grp);
        ctx->ev_used += 2;
    } else {
        hipLaunchKernelGGL(kern, dim3((unsigned)p.grid), dim3(T::THREADS), 0, ctx->stream, grp);
    }
    COMET_LAUNCH_CHECK(ctx, what);
    return COMET_OK;
}

}  // namespace comet_gemm
