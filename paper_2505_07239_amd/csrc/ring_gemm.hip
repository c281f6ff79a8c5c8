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
//     MAX_SEG = 256 steps; the schedule below never accumulates more than that
//     before it flushes.
//   * Addition mod 2^64 is associative and commutative, so partial sums may be
//     formed in any order and by any number of workgroups: the (tile, slice of
//     the stacked contraction) work units are dealt out evenly over a fixed,
//     chip-sized grid (a stream-K split) and every run of units inside one
//     tile ends with 64-bit atomic adds onto Z, which starts out as [C]_i.
//     The result is bit-exact whatever the split.  When the grid divides the
//     number of tiles every workgroup owns whole tiles instead: it stores
//     Z = C + sum itself and no atomic add is issued (owns_tiles()).
//   * Several products of one shape (comet_share_group) run as one launch over
//     the concatenation of their work units.
//
// Data flow
//   xpack kernel : E, A_i  -> digit planes of [E | A'] in the workspace, laid
//                  out so that a tile is a linear copy into LDS (small operand).
//   gemm kernel  : weight-side WORDS are loaded once as uint64 (with the block
//                  gather folded into the addressing), split into digits and
//                  byte-transposed in registers, staged through LDS, and fed
//                  to v_mfma_i32_32x32x32_i8; they are never re-written to
//                  memory.  Weight-side PLANES (COMET_WEIGHT_PLANES: F opened in
//                  that format, B_i packed offline, see wplanes.hip) go to LDS
//                  by LDS-DMA like the activation planes: a step then holds
//                  nothing but matrix instructions and their fragment reads.
#include "ring_gemm_kernel.h"

#include <mutex>

// Scratch of comet_somm_share_static, the entry point for callers that cannot allocate: a
// file-scope device array, one copy per GPU for the life of the process.  In host code the
// name `scratch` is only a handle for hipGetSymbolAddress: the address a kernel may use is the
// one that call returns for the current device, kept in scratch_ptr[] and handed to the kernels
// as an argument like any caller-owned workspace.
constexpr size_t STATIC_SCRATCH_BYTES = COMET_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
static void* scratch_ptr[MAX_DEVICES];
static std::mutex scratch_mutex;

int comet_static_scratch(int device, void** ptr, size_t* bytes) {
    if (device < 0 || device >= MAX_DEVICES || !ptr || !bytes) return COMET_EINVAL;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[device]) {
        void* q = nullptr;
        if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) {
            (void)hipGetLastError();
            return COMET_EDEVICE;
        }
        scratch_ptr[device] = q;
    }
    *ptr = scratch_ptr[device];
    *bytes = STATIC_SCRATCH_BYTES;
    return COMET_OK;
}

namespace {

using namespace comet_gemm;

// ---------------------------------------------------------------------------
// xpack: digit planes of the stacked activation-side operand, and Z := C
// ---------------------------------------------------------------------------
// grid: x = chunks of four 16-word groups, y = chunks of 64 rows, z = 0 (E), 1 (A'), 2 (Z := C).
// A workgroup packs a 64-row x 64-word tile: four adjacent lanes read 512 contiguous bytes of
// one row, and the sixteen lanes that share a group write sixteen adjacent 16-byte units.
__device__ __forceinline__ void xpack_body(const GemmParams& p, const int part) {
    const int nblk = n_blocks(p);
    const int m_eff = n_rows(p);
    if (part == 2) {
        // Z := C on the kept region (the GEMM adds its partial sums onto it); with result blocks
        // (Protocol 2 in general form) Z := C on the blocks and zero between them
        const int n_eff = p.kind == KIND_SOMM ? nblk * p.bs : p.n_cap;
        // (the share kernel writes Z = C + sum itself when every workgroup owns whole tiles)
        if (owns_tiles(p, m_eff, n_eff, p.kind == KIND_SOMM ? p.kc_cap : nblk * p.bs)) return;
        const long stride = (long)gridDim.x * gridDim.y * GT;
        const long t0 = ((long)blockIdx.y * gridDim.x + blockIdx.x) * GT + threadIdx.x;
        if (((n_eff | p.ldz | p.bs) & 1) == 0 || (!p.row_comp && ((n_eff | p.ldz) & 1) == 0)) {
            // 16-byte accesses (the operands are 16-byte aligned, every row starts on a pair, and
            // a pair never straddles two blocks when that matters)
            typedef u64 u64x2 __attribute__((ext_vector_type(2)));
            const int half = n_eff >> 1;
            const long total = (long)m_eff * half;
            for (long i = t0; i < total; i += stride) {
                const long r = i / half, c = (i - r * half) * 2;
                u64x2 v = *reinterpret_cast<const u64x2*>(p.C + r * p.ldz + c);
                if (p.row_comp && p.row_comp[r] != p.blk_comp[c / p.bs]) v = u64x2{0, 0};
                *reinterpret_cast<u64x2*>(p.Z + r * p.ldz + c) = v;
            }
        } else {
            const long total = (long)m_eff * n_eff;
            for (long i = t0; i < total; i += stride) {
                const long r = i / n_eff, c = i - r * n_eff;
                u64 v = p.C[r * p.ldz + c];
                if (p.row_comp && p.row_comp[r] != p.blk_comp[c / p.bs]) v = 0;
                p.Z[r * p.ldz + c] = v;
            }
        }
        return;
    }
    const int kc = p.kind == KIND_SOMM ? p.kc_cap : nblk * p.bs;
    // Whole tile of 64 rows x 64 contraction words inside the operands: the loads want the lanes
    // along k (a row piece of 512 bytes per half wavefront), the stores want them along the rows (a
    // digit group is one run of rows), so the tile passes through LDS in between.
    {
        const int kw = blockIdx.x * 64;                        // first word of the workgroup's four groups
        // (an indexed A_i keeps the direct path: one block lookup per sixteen words there, one per pair here)
        const bool tiled = !p.tmask && (p.lde & 1) == 0 && (p.lda & 1) == 0 && !p.a_full &&
                           kw + 64 <= kc;                      // uniform over the workgroup
        if (tiled) {
            typedef u64 u64x2 __attribute__((ext_vector_type(2)));
            constexpr int PITCH = 33;                          // 16-byte vectors per tile row (32 + padding)
            __shared__ u64x2 tile[64 * PITCH];
            const int h = part;                                // 0: E, 1: A'
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int v = i * GT + threadIdx.x;            // vector of the tile: row v / 32, words 2 (v % 32) ..
                const int r = v >> 5, kv = v & 31;
                const int trow = blockIdx.y * 64 + r, kk = kw + 2 * kv;
                u64x2 w = {0, 0};
                if (trow < m_eff) {
                    u64x2 ev = {0, 0};
                    if (h == 0 || p.party)                      // party 0's A' is A_i itself
                        ev = *reinterpret_cast<const u64x2*>(p.E + (size_t)trow * p.lde + kk);
                    if (h == 0) {
                        w = ev;
                    } else {
                        w = *reinterpret_cast<const u64x2*>(p.A + (size_t)trow * p.lda + kk) + ev;
                    }
                }
                tile[r * PITCH + kv] = w;
            }
            __syncthreads();
            const int r = threadIdx.x & 63, q = threadIdx.x >> 6;
            const int trow = blockIdx.y * 64 + r;
            if (trow >= p.mpad) return;                        // (the few-row kernel packs 32 rows)
            u64 plane[2][8];
#pragma unroll
            for (int o = 0; o < 2; ++o) {
                u64 v[8];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const u64x2 t = tile[r * PITCH + 8 * q + 4 * o + j];
                    v[2 * j] = to_digits(t.x);
                    v[2 * j + 1] = to_digits(t.y);
                }
                digits_to_planes(v, plane[o]);
            }
            const int half16 = blockIdx.x * 4 + q;
            const int s = half16 >> 1, g = half16 & 1;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                u64x2* dst = reinterpret_cast<u64x2*>(p.xp) + xp_group(h, s, t, g, p.ks_cap) * p.mpad + trow;
                *dst = u64x2{plane[0][t], plane[1][t]};
            }
            return;
        }
    }
    const int row = blockIdx.y * 64 + (threadIdx.x >> 2);
    if (row >= p.mpad) return;                                 // (the few-row kernel packs 32 rows)
    const int half16 = blockIdx.x * 4 + (threadIdx.x & 3);     // 16-word group over the half
    if (half16 >= p.ks_cap * 2) return;
    const int h = part;                                        // 0: E, 1: A'
    const int k0 = half16 * 16;
    typedef u64 u64x2 __attribute__((ext_vector_type(2)));
    u64 w[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) w[j] = 0;
    // fast path: the sixteen words are inside the contraction, 16-byte aligned, and (when A_i is
    // indexed) inside one block -- eight 16-byte loads per operand
    const bool wide = row < m_eff && k0 + 16 <= kc && (p.lde & 1) == 0 && (p.lda & 1) == 0 &&
                      ((!p.a_full && !p.tmask) || (p.bs & 15) == 0);
    if (wide && p.tmask && !token_uses(p, row, k0 / p.bs)) {
        // the token does not use this block: its sixteen entries take no part (w stays zero)
    } else if (wide) {
        const u64* e = p.E + (size_t)row * p.lde + k0;
        u64x2 ev[8];
        if (h == 0 || p.party) {                       // party 0's A' is A_i itself
#pragma unroll
            for (int j = 0; j < 8; ++j) ev[j] = *reinterpret_cast<const u64x2*>(e + 2 * j);
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) ev[j] = u64x2{0, 0};
        }
        if (h == 0) {
#pragma unroll
            for (int j = 0; j < 8; ++j) { w[2 * j] = ev[j].x; w[2 * j + 1] = ev[j].y; }
        } else {
            long col = k0;
            if (p.a_full) {
                const int blk = k0 / p.bs;
                const long st = block_start(p, blk);
                col = (st < 0 ? 0 : st) + (k0 - blk * p.bs);
            }
            const u64* a = p.A + (size_t)row * p.lda + col;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const u64x2 av = *reinterpret_cast<const u64x2*>(a + 2 * j);
                w[2 * j] = av.x + (p.party ? ev[j].x : 0ull);
                w[2 * j + 1] = av.y + (p.party ? ev[j].y : 0ull);
            }
        }
    } else if (row < m_eff && k0 < kc) {
        for (int j = 0; j < 16; ++j) {
            const int k = k0 + j;
            if (k >= kc) break;
            const int blk = k / p.bs;
            if (p.tmask && !token_uses(p, row, blk)) continue;
            const u64 e = p.E[(size_t)row * p.lde + k];
            u64 x = e;
            if (h == 1) {
                long col = k;
                if (p.a_full) {
                    const long st = block_start(p, blk);
                    col = (st < 0 ? 0 : st) + (k - blk * p.bs);
                }
                x = p.A[(size_t)row * p.lda + col] + (p.party ? e : 0ull);
            }
            w[j] = x;
        }
    }
    u64 plane[2][8];
#pragma unroll
    for (int o = 0; o < 2; ++o) {
        u64 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = (row < m_eff && k0 + 8 * o + j < kc) ? to_digits(w[8 * o + j]) : 0ull;
        digits_to_planes(v, plane[o]);
    }
    const int s = half16 >> 1, g = half16 & 1;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        u64x2* dst = reinterpret_cast<u64x2*>(p.xp) + xp_group(h, s, t, g, p.ks_cap) * p.mpad + row;
        *dst = u64x2{plane[0][t], plane[1][t]};
    }
}

__global__ __launch_bounds__(GT) void xpack_kernel(GemmParams p) { xpack_body(p, blockIdx.z); }

// the members of a group (one shape): grid.z = 3 * member + part
__global__ __launch_bounds__(GT) void xpack_group_kernel(GemmGroup grp) {
    xpack_body(grp.p[blockIdx.z / 3], blockIdx.z % 3);
}

// ---------------------------------------------------------------------------
// result blocks (Protocol 2 in general form): which output tiles are computed
// ---------------------------------------------------------------------------
// Rows and columns are listed component by component, so a tile touches a result block exactly
// when the component ranges of its rows and of its columns overlap.  One workgroup writes the
// numbers of those tiles, in the order the GEMM enumerates tiles (tile = tn * tiles_m + tm),
// to list[1 ..] and their count to list[0]; the GEMM then deals out work over that list only.
// For tall operands two shapes are listed (128 x 64 and 64 x 64) and the choice between them is
// made here, on the device, from the area each would compute: both GEMM kernels are launched
// and the one that was not chosen returns at once, so the host never waits for the counts.
__global__ __launch_bounds__(GT) void tile_list_kernel(GemmParams p, int BM, int BN, int* list,
                                                        const int* other, int other_area, int* sel) {
    __shared__ int wave_tot[GT / 64];
    __shared__ int base;
    const int nblk = n_blocks(p);
    const int m_eff = n_rows(p), n_eff = nblk * p.bs;
    const int tiles_m = (m_eff + BM - 1) / BM, tiles_n = (n_eff + BN - 1) / BN;
    const int tiles = tiles_m * tiles_n;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) base = 0;
    __syncthreads();
    for (int t0 = 0; t0 < tiles; t0 += GT) {
        const int tile = t0 + threadIdx.x;
        bool on = false;
        if (tile < tiles) {
            const int tm = tile % tiles_m, tn = tile / tiles_m;
            const int r_hi = (tm + 1) * BM < m_eff ? (tm + 1) * BM - 1 : m_eff - 1;
            const int c_hi = (tn + 1) * BN < n_eff ? (tn + 1) * BN - 1 : n_eff - 1;
            const int rc0 = p.row_comp[tm * BM], rc1 = p.row_comp[r_hi];
            const int cc0 = p.blk_comp[tn * BN / p.bs], cc1 = p.blk_comp[c_hi / p.bs];
            on = !(rc1 < cc0 || cc1 < rc0);
        }
        const unsigned long long bal = __ballot(on);
        if (lane == 0) wave_tot[wave] = __builtin_popcountll(bal);
        __syncthreads();
        int pos = base + __builtin_popcountll(bal & ((1ull << lane) - 1));
        for (int w = 0; w < wave; ++w) pos += wave_tot[w];
        if (on) list[1 + pos] = tile;
        __syncthreads();
        if (threadIdx.x == 0) {
            int s = 0;
            for (int w = 0; w < GT / 64; ++w) s += wave_tot[w];
            base += s;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        list[0] = base;
        // second of two shapes: this one runs when it computes at most 80 % of the other's area
        // (smaller tiles follow the block structure more closely but reuse operands less)
        if (sel) *sel = (5l * base * BM * BN < 4l * other[0] * other_area) ? 1 : 0;
    }
}

// ---------------------------------------------------------------------------
// per-token row sets (Protocol 3 in general form): which contraction steps a row tile computes
// ---------------------------------------------------------------------------
// Protocol 3 multiplies column j of X only on its row set R_j.  At tile granularity: a row tile
// needs contraction step s (32 consecutive kept neurons) only if one of its tokens uses one of
// the blocks the step touches; for all other steps the tile's activation digits are zero.  One
// workgroup per row tile lists its steps in ascending order (grid.x = row tiles); a second,
// one-workgroup kernel turns the counts into offsets.  The GEMM then deals out work over the
// listed steps only.
__global__ __launch_bounds__(GT) void step_list_kernel(GemmParams p, int BM) {
    __shared__ int wave_tot[GT / 64];
    __shared__ int base;
    const int nblk = n_blocks(p);
    const int m_eff = n_rows(p);
    const int kc = nblk * p.bs;
    const int KS = (kc + KSTEP - 1) / KSTEP;
    const int tm = blockIdx.x;
    const int r0 = tm * BM, r1 = (tm + 1) * BM < m_eff ? (tm + 1) * BM : m_eff;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int* list = p.step_list + (size_t)tm * p.ks_cap;
    if (threadIdx.x == 0) base = 0;
    __syncthreads();
    for (int s0 = 0; s0 < KS; s0 += GT) {
        const int st = s0 + threadIdx.x;
        bool on = false;
        if (st < KS && r0 < r1) {
            const int t0 = st * KSTEP / p.bs;
            int t1 = (st * KSTEP + KSTEP - 1) / p.bs;
            t1 = t1 < nblk - 1 ? t1 : nblk - 1;
            for (int t = t0; t <= t1 && !on; ++t)
                for (int r = r0; r < r1 && !on; ++r) on = token_uses(p, r, t);
        }
        const unsigned long long bal = __ballot(on);
        if (lane == 0) wave_tot[wave] = __builtin_popcountll(bal);
        __syncthreads();
        int pos = base + __builtin_popcountll(bal & ((1ull << lane) - 1));
        for (int w = 0; w < wave; ++w) pos += wave_tot[w];
        if (on) list[pos] = st;
        __syncthreads();
        if (threadIdx.x == 0) {
            int sum = 0;
            for (int w = 0; w < GT / 64; ++w) sum += wave_tot[w];
            base += sum;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) p.step_cnt[tm] = base;
}

// step_off[t] = step_cnt[0] + ... + step_cnt[t - 1] for t = 0 .. tiles (one workgroup)
__global__ __launch_bounds__(GT) void step_offsets_kernel(GemmParams p, int BM) {
    __shared__ int wave_tot[GT / 64];
    __shared__ int base;
    const int m_eff = n_rows(p);
    const int tiles = (m_eff + BM - 1) / BM;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) base = 0;
    __syncthreads();
    for (int t0 = 0; t0 < tiles; t0 += GT) {
        const int t = t0 + threadIdx.x;
        const int v = t < tiles ? p.step_cnt[t] : 0;
        int inc = v;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int o = __shfl_up(inc, d, 64);
            if (lane >= d) inc += o;
        }
        if (lane == 63) wave_tot[wave] = inc;
        __syncthreads();
        int pre = base + inc - v;
        for (int w = 0; w < wave; ++w) pre += wave_tot[w];
        if (t < tiles) p.step_off[t] = pre;
        __syncthreads();
        if (threadIdx.x == 0) {
            int sum = 0;
            for (int w = 0; w < GT / 64; ++w) sum += wave_tot[w];
            base += sum;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) p.step_off[tiles] = base;
}
inline int round_up(int64_t v, int64_t to) { return (int)(((v + to - 1) / to) * to); }

// digit planes of [E | A'] (the few-row path keeps its k-major copy there instead)
size_t planes_bytes(int64_t m, int64_t kc_cap) {
    const size_t mpad = (size_t)round_up(m, 128);
    const size_t ks_cap = (size_t)((kc_cap + KSTEP - 1) / KSTEP);
    const size_t bytes = mpad * 2 * ks_cap * 256;
    return bytes ? bytes : 256;
}

// step lists of Protocol 3 with per-token row sets: per row tile of the smallest tile height (32)
// a count, an offset and up to ks_cap listed steps
size_t step_ws_bytes(int64_t m, int64_t kc_cap) {
    const size_t tiles = (size_t)((m + 31) / 32);
    const size_t ks_cap = (size_t)((kc_cap + KSTEP - 1) / KSTEP);
    return ((tiles * (ks_cap + 2) + 1) * sizeof(int) + 255) & ~(size_t)255;
}

// followed by the list of output tiles that touch a result block (general form of Protocol 2):
// a selector, then twice (two tile shapes) one count plus one entry per tile of the smallest
// tile shape, 64 x 64
size_t gemm_ws_bytes(int64_t m, int64_t kc_cap, int64_t n_cap) {
    if (m < 1 || kc_cap < 0 || n_cap < 0 || m > COMET_ROWS_MAX || kc_cap > COMET_DIM_MAX || n_cap > COMET_DIM_MAX)
        return 0;
    const size_t tiles = (size_t)((m + 63) / 64) * (size_t)((n_cap + 63) / 64);
    return planes_bytes(m, kc_cap) + (((2 * (tiles + 1) + 1) * sizeof(int) + 255) & ~(size_t)255) +
           step_ws_bytes(m, kc_cap);
}

// the parts of the workspace and the derived sizes
void place_in_workspace(GemmParams& p, void* ws) {
    p.xp = static_cast<unsigned char*>(ws);
    p.tile_list = reinterpret_cast<int*>(p.xp + planes_bytes(p.m, p.kc_cap));
    p.mpad = round_up(p.m, 128);
    p.ks_cap = (p.kc_cap + KSTEP - 1) / KSTEP;
    p.bs_shift = -1;
    for (int sh = 0; sh < 30; ++sh)
        if (p.bs == (1 << sh)) p.bs_shift = sh;
}

int run_share(comet_ctx* ctx, const char* what, GemmParams p, void* ws, size_t ws_bytes) {
    const size_t need = gemm_ws_bytes(p.m, p.kc_cap, p.n_cap);
    if (!ws || ws_bytes < need)
        return comet_fail(ctx, COMET_EWORKSPACE, "%s: workspace of %zu bytes required", what, need);
    if (reinterpret_cast<uintptr_t>(ws) & 255u)
        return comet_fail(ctx, COMET_EALIGN, "%s: workspace must be 256-byte aligned", what);
    comet_device_guard guard(ctx);
    if (!guard.ok) return comet_fail(ctx, COMET_EDEVICE, "%s: cannot select device", what);

    place_in_workspace(p, ws);

    if (p.n_cap == 0) return COMET_OK;
    if (p.F2 && (p.m > COMET_SKINNY_MAX_ROWS || ctx->skinny_mode == 1 || p.w_tr || p.w_planes || p.row_comp || p.tmask))
        return comet_fail(ctx, COMET_EINVAL, "%s: unopened weight shares are taken by the few-row kernel only "
                          "(m <= %d, row-major words)", what, COMET_SKINNY_MAX_ROWS);
    // (the few-row kernel reads the weights along the output columns: row-major words only)
    if (p.m <= COMET_SKINNY_MAX_ROWS && ctx->skinny_mode != 1 && !p.w_tr && !p.w_planes)
        return comet_launch_skinny(ctx, what, p);
    // Tile shape and launch plan first: the packing kernel has to know whether the share kernel
    // will own its tiles (and then initialise Z itself).
    using T128 = Tile<2, 2, 2, 1>;
    using T64 = Tile<2, 2, 1, 1>;
    using T32W = Tile<1, 4, 1, 2>;
    using T32P = Tile<1, 4, 1, 1>;
    const int gm = p.w_planes ? W_PLANES : GATHER_NONE;     // what decides the LDS footprint
    auto plan = [&](int bm) {
        if (bm == 128) plan_gemm(ctx, p, T128::BM, T128::BN, T128::wg_per_cu(gm));
        else if (bm == 64) plan_gemm(ctx, p, T64::BM, T64::BN, T64::wg_per_cu(gm));
        else if (p.w_planes) plan_gemm(ctx, p, T32P::BM, T32P::BN, T32P::wg_per_cu(gm));
        else plan_gemm(ctx, p, T32W::BM, T32W::BN, T32W::wg_per_cu(gm));
    };
    auto launch = [&](int bm) {
        plan(bm);
        if (bm == 128) return launch_gemm<2, 2, 2, 1>(ctx, what, p);
        if (bm == 64) return launch_gemm<2, 2, 1, 1>(ctx, what, p);
        return p.w_planes ? launch_gemm<1, 4, 1, 1>(ctx, what, p) : launch_gemm<1, 4, 1, 2>(ctx, what, p);
    };
    // rows per workgroup tile: 128, 64 or 32
    int bm = 128;
    const long big_tiles = (long)((p.m + 127) / 128) * ((p.n_cap + 63) / 64);
    if (ctx->gemm_tile == 2) bm = 64;
    else if (p.m <= 32) bm = 32;
    else if (p.m <= 64) bm = 64;
    // a small product (a handful of 128 x 64 tiles) is bound by the fixed cost per workgroup:
    // the 64 x 64 tile doubles the number of independent tiles
    else if (!p.row_comp && big_tiles * 8 <= ctx->num_cu) bm = 64;
    // a ragged last row tile: 64-row tiles when they pad the rows by clearly less (the smaller
    // tile is about 5 % slower per product)
    else if (!p.row_comp && (long)round_up(p.m, 64) * 110 < (long)round_up(p.m, 128) * 100) bm = 64;
    // per-token row sets: 64-row tiles follow the row sets more closely
    else if (p.tmask) bm = 64;
    plan(bm);
    // a decoding batch on weight planes: the kernel that streams the planes wavefront by wavefront
    const bool fewrow = p.w_planes && p.m <= COMET_FEWROW_MAX_ROWS && !p.w_tr && !p.row_comp && !p.tmask &&
                        ctx->skinny_mode != 1 && ctx->gemm_tile != 2;
    if (fewrow) {
        p.own_try = 0;                                         // Z := C comes from the packing kernel
        p.mpad = 32;                                           // one row tile: a digit group is 512 bytes
    }

    // digit planes of [E | A'] and Z := C, one launch
    {
        unsigned gx = (unsigned)((p.ks_cap * 2 + 3) / 4);
        if (gx < 1) gx = 1;
        // the Z := C slab shares the launch: give it enough workgroups for about four 16-byte
        // accesses per thread (the packing slabs return at once from the extra ones)
        const int slabs = (p.mpad + 63) / 64;
        const long zgx = ((long)p.m * p.n_cap / (2l * 4 * GT) + slabs - 1) / slabs;
        if (zgx > gx) gx = (unsigned)(zgx > 4096 ? 4096 : zgx);
        hipLaunchKernelGGL(xpack_kernel, dim3(gx, (unsigned)slabs, 3), dim3(GT), 0, ctx->stream, p);
        COMET_LAUNCH_CHECK(ctx, what);
    }
    if (p.ks_cap == 0) return COMET_OK;
    if (fewrow) return comet_launch_fewrow(ctx, what, p);
    if (p.row_comp) {
        // result blocks: list the tiles that are computed (see tile_list_kernel)
        int* sel = p.tile_list;
        int* list_a = sel + 1;
        int* list_b = list_a + 1 + (size_t)((p.m + 63) / 64) * (size_t)((p.n_cap + 63) / 64);
        p.tile_list = list_a;
        if (bm != 128) {
            hipLaunchKernelGGL(tile_list_kernel, dim3(1), dim3(GT), 0, ctx->stream, p, bm,
                               bm == 64 ? 64 : (p.w_planes ? 128 : 256), list_a, (const int*)nullptr, 0,
                               (int*)nullptr);
            COMET_LAUNCH_CHECK(ctx, what);
            return launch(bm);
        }
        hipLaunchKernelGGL(tile_list_kernel, dim3(1), dim3(GT), 0, ctx->stream, p, 128, 64, list_a,
                           (const int*)nullptr, 0, (int*)nullptr);
        COMET_LAUNCH_CHECK(ctx, what);
        hipLaunchKernelGGL(tile_list_kernel, dim3(1), dim3(GT), 0, ctx->stream, p, 64, 64, list_b,
                           (const int*)list_a, 128 * 64, sel);
        COMET_LAUNCH_CHECK(ctx, what);
        p.tile_sel = sel;
        p.tile_sel_want = 0;
        int rc = launch(128);
        if (rc) return rc;
        p.tile_list = list_b;
        p.tile_sel_want = 1;
        return launch(64);
    }
    if (p.tmask) {
        // list, per row tile, the contraction steps some token of the tile takes part in
        const size_t tiles64 = (size_t)((p.m + 63) / 64) * (size_t)((p.n_cap + 63) / 64);
        const size_t tl_bytes = ((2 * (tiles64 + 1) + 1) * sizeof(int) + 255) & ~(size_t)255;
        const size_t t32 = (size_t)((p.m + 31) / 32);
        int* base = reinterpret_cast<int*>(p.xp + planes_bytes(p.m, p.kc_cap) + tl_bytes);
        p.step_cnt = base;
        p.step_off = base + t32;
        p.step_list = base + 2 * t32 + 1;
        const unsigned tiles_m = (unsigned)((p.m + bm - 1) / bm);
        hipLaunchKernelGGL(step_list_kernel, dim3(tiles_m), dim3(GT), 0, ctx->stream, p, bm);
        COMET_LAUNCH_CHECK(ctx, what);
        hipLaunchKernelGGL(step_offsets_kernel, dim3(1), dim3(GT), 0, ctx->stream, p, bm);
        COMET_LAUNCH_CHECK(ctx, what);
    }
    return launch(bm);
}

// Several products of one shape, one index list and one operand format.  When they suit the
// grouped matrix-core kernel (weight planes, more than 64 rows, no few-row path) they run as one
// packing launch and one share launch over the union of their work units; otherwise one by one.
int run_share_group(comet_ctx* ctx, const char* what, GemmParams* ps, int n, void* ws, size_t ws_bytes) {
    const size_t each = gemm_ws_bytes(ps[0].m, ps[0].kc_cap, ps[0].n_cap);
    if (!ws || each == 0 || ws_bytes / (size_t)n < each)
        return comet_fail(ctx, COMET_EWORKSPACE, "%s: workspace of %zu bytes required", what, each * (size_t)n);
    if (reinterpret_cast<uintptr_t>(ws) & 255u)
        return comet_fail(ctx, COMET_EALIGN, "%s: workspace must be 256-byte aligned", what);
    unsigned char* base = static_cast<unsigned char*>(ws);
    const GemmParams& p0 = ps[0];
    // One launch for all members pays when a member alone is a short launch: between 8 and 128
    // contraction steps per workgroup.  Below that the single calls shrink their grid instead;
    // above it the fixed cost of a launch is amortised already and one long launch only runs
    // at a lower sustained clock than the same work in pieces.
    using T = Tile<2, 2, 2, 1>;
    long grid = (ctx->num_cu / 8) * 8 * T::wg_per_cu(W_PLANES);
    if (grid < 8) grid = 8;
    if (ctx->gemm_grid > 0) grid = ctx->gemm_grid;
    const long tiles = (long)((p0.m + T::BM - 1) / T::BM) * ((p0.n_cap + T::BN - 1) / T::BN);
    const long steps_each = tiles * 2 * ((p0.kc_cap + KSTEP - 1) / KSTEP) / grid;
    const bool grouped = n > 1 && p0.w_planes && p0.m > 64 && p0.n_cap > 0 && ctx->gemm_tile != 2 &&
                         (ctx->group_mode == 1 || ctx->group_mode == 3 ||
                          (ctx->group_mode == 0 && steps_each >= 8 && steps_each <= 128));
    if (!grouped) {
        for (int j = 0; j < n; ++j) {
            const int rc = run_share(ctx, what, ps[j], base + (size_t)j * each, each);
            if (rc) return rc;
        }
        return COMET_OK;
    }
    comet_device_guard guard(ctx);
    if (!guard.ok) return comet_fail(ctx, COMET_EDEVICE, "%s: cannot select device", what);

    GemmGroup grp = {};
    grp.n = n;
    for (int j = 0; j < n; ++j) {
        GemmParams& p = grp.p[j];
        p = ps[j];
        place_in_workspace(p, base + (size_t)j * each);
        // units tile by tile (all of a tile's contraction in a row): a workgroup's share of the
        // whole sequence then covers few tiles, and whole ones when the grid divides their number
        p.chunk = 2 * p.ks_cap > 0 ? 2 * p.ks_cap : 1;
        p.grid = (int)grid;
        p.tile_bm = T::BM;
        p.tile_bn = T::BN;
        p.group_n = n;
        p.own_try = (tiles * n % grid == 0) ? 1 : 0;
        p.k_rotate = 1;
        p.team = ctx->group_mode != 3;      // (3: one launch without teams, for comparison)
    }
    {
        const GemmParams& p = grp.p[0];
        unsigned gx = (unsigned)((p.ks_cap * 2 + 3) / 4);
        if (gx < 1) gx = 1;
        const long zgx = ((long)p.m * p.n_cap / (2l * 4 * GT) + p.mpad / 64 - 1) / (p.mpad / 64);
        if (zgx > gx) gx = (unsigned)(zgx > 4096 ? 4096 : zgx);
        hipLaunchKernelGGL(xpack_group_kernel, dim3(gx, (unsigned)(p.mpad / 64), 3u * (unsigned)n), dim3(GT), 0,
                           ctx->stream, grp);
        COMET_LAUNCH_CHECK(ctx, what);
    }
    return launch_gemm_group<2, 2, 2, 1>(ctx, what, grp);
}

int check_common(comet_ctx* ctx, const char* what, int party, int64_t m, int bs, int n_blk_cap,
                 int flags, const void* const* ptrs, int n_ptrs, const int32_t* blk_idx) {
    if (party != 0 && party != 1) return comet_fail(ctx, COMET_EINVAL, "%s: party must be 0 or 1", what);
    if (m < 1 || bs < 1 || n_blk_cap < 0) return comet_fail(ctx, COMET_EINVAL, "%s: bad size", what);
    if (flags & ~(COMET_FULL_A | COMET_FULL_B | COMET_WEIGHTS_NEURON_MAJOR | COMET_WEIGHT_PLANES))
        return comet_fail(ctx, COMET_EINVAL, "%s: unknown flag", what);
    if ((flags & COMET_WEIGHT_PLANES) && (flags & COMET_WEIGHTS_NEURON_MAJOR))
        return comet_fail(ctx, COMET_EINVAL, "%s: weight planes have a layout of their own", what);
    for (int i = 0; i < n_ptrs; ++i) {
        if (!ptrs[i]) return comet_fail(ctx, COMET_EINVAL, "%s: null pointer (operand %d)", what, i);
        if (!comet_aligned16(ptrs[i]))
            return comet_fail(ctx, COMET_EALIGN, "%s: operand %d is not 16-byte aligned", what, i);
    }
    if (!blk_idx && (flags & (COMET_FULL_A | COMET_FULL_B)))
        return comet_fail(ctx, COMET_EINVAL, "%s: blk_idx required for full-size operands", what);
    // rows: the packing kernel walks 64-row slabs of the padded row count on grid.y (< 65536)
    if (m > COMET_ROWS_MAX || (int64_t)n_blk_cap * bs > COMET_DIM_MAX)
        return comet_fail(ctx, COMET_ECAP, "%s: dimension beyond 2^24 (m beyond 2^22 - 128)", what);
    return COMET_OK;
}

int somm_params(comet_ctx* ctx, const char* what, GemmParams& p, int party, int64_t m, int64_t k,
                int64_t n_full, int bs, const int32_t* blk_idx, const int32_t* n_blk_dev, int n_blk_cap,
                int flags, const uint64_t* E, const uint64_t* F, const uint64_t* A_i,
                const uint64_t* B_i, const uint64_t* C_i, uint64_t* Z_i) {
    const void* ptrs[] = {E, F, A_i, B_i, C_i, Z_i};
    int rc = check_common(ctx, what, party, m, bs, n_blk_cap, flags, ptrs, 6, blk_idx);
    if (rc) return rc;
    if (k < 1 || n_full < 0) return comet_fail(ctx, COMET_EINVAL, "%s: bad size", what);
    if (flags & COMET_FULL_A) return comet_fail(ctx, COMET_EINVAL, "%s: A_i is never indexed in SOMM", what);
    if (k > COMET_DIM_MAX || n_full > COMET_DIM_MAX) return comet_fail(ctx, COMET_ECAP, "%s: dimension beyond 2^24", what);
    const int64_t ld = (int64_t)n_blk_cap * bs;
    if ((flags & COMET_FULL_B) && ld > n_full)
        return comet_fail(ctx, COMET_EINVAL, "%s: n_blk_cap * bs exceeds n_full", what);
    if (k * ((flags & COMET_FULL_B) ? n_full : ld) >= (1ll << 31) || k * ld >= (1ll << 31))
        return comet_fail(ctx, COMET_ECAP, "%s: a weight-side operand holds 2^31 words or more", what);
    p.kind = KIND_SOMM; p.party = party; p.m = (int)m; p.kc_cap = (int)k; p.n_cap = (int)ld;
    p.bs = bs; p.n_blk_cap = n_blk_cap; p.blk_idx = blk_idx; p.n_blk_dev = n_blk_dev;
    p.full_extent = (int)n_full;
    p.E = (const u64*)E; p.lde = k;
    p.A = (const u64*)A_i; p.lda = k; p.a_full = 0;
    p.B = (const u64*)B_i; p.b_full = (flags & COMET_FULL_B) ? 1 : 0; p.ldb = p.b_full ? n_full : ld;
    p.F = (const u64*)F; p.ldf = ld;
    if (flags & COMET_WEIGHTS_NEURON_MAJOR) {
        // B_i: n_full x k or ld x k, F: ld x k; the kernel reads pairs of contraction words
        if (k & 1) return comet_fail(ctx, COMET_EINVAL, "%s: neuron-major weights need an even k", what);
        p.w_tr = 1; p.ldb = k; p.ldf = k;
    }
    p.w_planes = (flags & COMET_WEIGHT_PLANES) ? 1 : 0;
    p.C = (const u64*)C_i; p.Z = (u64*)Z_i; p.ldz = ld;
    return COMET_OK;
}

int simm_params(comet_ctx* ctx, const char* what, GemmParams& p, int party, int64_t m, int64_t k_full,
                int64_t n, int bs, const int32_t* blk_idx, const int32_t* n_blk_dev, int n_blk_cap,
                int flags, const uint64_t* E, const uint64_t* F, const uint64_t* A_i,
                const uint64_t* B_i, const uint64_t* C_i, uint64_t* Z_i) {
    const void* ptrs[] = {E, F, A_i, B_i, C_i, Z_i};
    int rc = check_common(ctx, what, party, m, bs, n_blk_cap, flags, ptrs, 6, blk_idx);
    if (rc) return rc;
    if (n < 1 || k_full < 0) return comet_fail(ctx, COMET_EINVAL, "%s: bad size", what);
    if (flags & COMET_WEIGHTS_NEURON_MAJOR)
        return comet_fail(ctx, COMET_EINVAL, "%s: B_i and F of SIMM are neuron-major as they are (one row per neuron)", what);
    if (n > COMET_DIM_MAX || k_full > COMET_DIM_MAX) return comet_fail(ctx, COMET_ECAP, "%s: dimension beyond 2^24", what);
    const int64_t ld = (int64_t)n_blk_cap * bs;
    if ((flags & (COMET_FULL_A | COMET_FULL_B)) && ld > k_full)
        return comet_fail(ctx, COMET_EINVAL, "%s: n_blk_cap * bs exceeds k_full", what);
    if (((flags & COMET_FULL_B) ? k_full : ld) * n >= (1ll << 31))
        return comet_fail(ctx, COMET_ECAP, "%s: a weight-side operand holds 2^31 words or more", what);
    p.kind = KIND_SIMM; p.party = party; p.m = (int)m; p.kc_cap = (int)ld; p.n_cap = (int)n;
    p.bs = bs; p.n_blk_cap = n_blk_cap; p.blk_idx = blk_idx; p.n_blk_dev = n_blk_dev;
    p.full_extent = (int)k_full;
    p.E = (const u64*)E; p.lde = ld;
    p.A = (const u64*)A_i; p.a_full = (flags & COMET_FULL_A) ? 1 : 0; p.lda = p.a_full ? k_full : ld;
    p.B = (const u64*)B_i; p.b_full = (flags & COMET_FULL_B) ? 1 : 0; p.ldb = n;
    p.F = (const u64*)F; p.ldf = n;
    p.w_planes = (flags & COMET_WEIGHT_PLANES) ? 1 : 0;
    // planes of a full-size B_i are gathered in units of sixteen contraction rows
    if (p.w_planes && p.b_full && (bs % 16) != 0)
        return comet_fail(ctx, COMET_EINVAL, "%s: weight planes of a full-size B_i need bs to be a multiple of 16", what);
    p.C = (const u64*)C_i; p.Z = (u64*)Z_i; p.ldz = n;
    return COMET_OK;
}

}  // namespace

size_t comet_gemm_workspace_bytes(int64_t m, int64_t kc_cap, int64_t n_cap) {
    return gemm_ws_bytes(m, kc_cap, n_cap);
}

extern "C" {

int comet_somm_share(comet_ctx* ctx, int party, int64_t m, int64_t k, int64_t n_full, int bs,
                     const int32_t* blk_idx, const int32_t* n_blk_dev, int n_blk_cap, int flags,
                     const uint64_t* E, const uint64_t* F, const uint64_t* A_i,
                     const uint64_t* B_i, const uint64_t* C_i, uint64_t* Z_i, void* ws,
                     size_t ws_bytes) {
    const char* what = "comet_somm_share";
    COMET_CHECK_CTX(ctx);
    GemmParams p = {};
    const int rc = somm_params(ctx, what, p, party, m, k, n_full, bs, blk_idx, n_blk_dev, n_blk_cap, flags,
                               E, F, A_i, B_i, C_i, Z_i);
    if (rc) return rc;
    return run_share(ctx, what, p, ws, ws_bytes);
}

// second masked share of the weights for the *_unopened calls: same layout and checks as F
static int set_unopened(comet_ctx* ctx, const char* what, GemmParams& p, const uint64_t* G_1) {
    if (!G_1) return comet_fail(ctx, COMET_EINVAL, "%s: null pointer", what);
    if (!comet_aligned16(G_1)) return comet_fail(ctx, COMET_EALIGN, "%s: operands must be 16-byte aligned", what);
    p.F2 = (const u64*)G_1;
    return COMET_OK;
}

int comet_somm_share_unopened(comet_ctx* ctx, int party, int64_t m, int64_t k, int64_t n_full, int bs,
                              const int32_t* blk_idx, const int32_t* n_blk_dev, int n_blk_cap, int flags,
                              const uint64_t* E, const uint64_t* G_0, const uint64_t* G_1,
                              const uint64_t* A_i, const uint64_t* B_i, const uint64_t* C_i, uint64_t* Z_i,
                              void* ws, size_t ws_bytes) {
    const char* what = "comet_somm_share_unopened";
    COMET_CHECK_CTX(ctx);
    GemmParams p = {};
    int rc = somm_params(ctx, what, p, party, m, k, n_full, bs, blk_idx, n_blk_dev, n_blk_cap, flags,
                         E, G_0, A_i, B_i, C_i, Z_i);
    if (rc) return rc;
    if ((rc = set_unopened(ctx, what, p, G_1)) != COMET_OK) return rc;
    return run_share(ctx, what, p, ws, ws_bytes);
}

int comet_simm_share_unopened(comet_ctx* ctx, int party, int64_t m, int64_t k_full, int64_t n, int bs,
                              const int32_t* blk_idx, const int32_t* n_blk_dev, int n_blk_cap, int flags,
                              const uint64_t* E, const uint64_t* G_0, const uint64_t* G_1,
                              const uint64_t* A_i, const uint64_t* B_i, const uint64_t* C_i, uint64_t* Z_i,
                              void* ws, size_t ws_bytes) {
    const char* what = "comet_simm_share_unopened";
    COMET_CHECK_CTX(ctx);
    GemmParams p = {};
    int rc = simm_params(ctx, what, p, party, m, k_full, n, bs, blk_idx, n_blk_dev, n_blk_cap, flags,
                         E, G_0, A_i, B_i, C_i, Z_i);
    if (rc) return rc;
    if ((rc = set_unopened(ctx, what, p, G_1)) != COMET_OK) return rc;
    return run_share(ctx, what, p, ws, ws_bytes);
}

int comet_somm_share_static(comet_ctx* ctx, int party, int64_t m, int64_t k, int64_t n_full, int bs,
                            const int32_t* blk_idx, const int32_t* n_blk_dev, int n_blk_cap,
                            int flags, const uint64_t* E, const uint64_t* F, const uint64_t* A_i,
                            const uint64_t* B_i, const uint64_t* C_i, uint64_t* Z_i) {
    const char* what = "comet_somm_share_static";
    COMET_CHECK_CTX(ctx);
    GemmParams p = {};
    const int rc = somm_params(ctx, what, p, party, m, k, n_full, bs, blk_idx, n_blk_dev, n_blk_cap, flags,
                               E, F, A_i, B_i, C_i, Z_i);
    if (rc) return rc;
    const size_t need = gemm_ws_bytes(p.m, p.kc_cap, p.n_cap);
    if (need == 0 || need > STATIC_SCRATCH_BYTES)
        return comet_fail(ctx, COMET_ECAP,
                          "%s: needs %zu bytes of scratch, the static array holds %zu "
                          "(use comet_somm_share with a workspace)", what, need, STATIC_SCRATCH_BYTES);
    if (!ctx->static_ws)
        return comet_fail(ctx, COMET_EDEVICE, "%s: static scratch was not resolved on this device", what);
    // every part of the scratch a call reads it has written before, so nothing needs clearing
    return run_share(ctx, what, p, ctx->static_ws, STATIC_SCRATCH_BYTES);
}

int comet_somm_share_blocks(comet_ctx* ctx, int party, int64_t m_cap, int64_t k, int64_t n_full,
                            int bs, const int32_t* blk_idx, const int32_t* blk_comp,
                            const int32_t* n_blk_dev, int n_blk_cap, const int32_t* row_comp,
                            const int32_t* n_row_dev, int flags, const uint64_t* E,
                            const uint64_t* F, const uint64_t* A_i, const uint64_t* B_i,
                            const uint64_t* C_i, uint64_t* Z_i, void* ws, size_t ws_bytes) {
    const char* what = "comet_somm_share_blocks";
    COMET_CHECK_CTX(ctx);
    if (!blk_idx || !blk_comp || !row_comp)
        return comet_fail(ctx, COMET_EINVAL, "%s: blk_idx, blk_comp and row_comp are required", what);
    GemmParams p = {};
    const int rc = somm_params(ctx, what, p, party, m_cap, k, n_full, bs, blk_idx, n_blk_dev, n_blk_cap,
                               flags, E, F, A_i, B_i, C_i, Z_i);
    if (rc) return rc;
    p.row_comp = row_comp; p.blk_comp = blk_comp; p.n_row_dev = n_row_dev;
    return run_share(ctx, what, p, ws, ws_bytes);
}

int comet_simm_share(comet_ctx* ctx, int party, int64_t m, int64_t k_full, int64_t n, int bs,
                     const int32_t* blk_idx, const int32_t* n_blk_dev, int n_blk_cap, int flags,
                     const uint64_t* E, const uint64_t* F, const uint64_t* A_i,
                     const uint64_t* B_i, const uint64_t* C_i, uint64_t* Z_i, void* ws,
                     size_t ws_bytes) {
    const char* what = "comet_simm_share";
    COMET_CHECK_CTX(ctx);
    GemmParams p = {};
    const int rc = simm_params(ctx, what, p, party, m, k_full, n, bs, blk_idx, n_blk_dev, n_blk_cap, flags,
                               E, F, A_i, B_i, C_i, Z_i);
    if (rc) return rc;
    return run_share(ctx, what, p, ws, ws_bytes);
}

int comet_share_group(comet_ctx* ctx, int op, int n_members, const comet_share_operands* members,
                      int64_t m, int64_t k, int64_t n, int bs, const int32_t* blk_idx,
                      const int32_t* n_blk_dev, int n_blk_cap, int flags, void* ws, size_t ws_bytes) {
    const char* what = "comet_share_group";
    COMET_CHECK_CTX(ctx);
    if (op != COMET_OP_SOMM && op != COMET_OP_SIMM)
        return comet_fail(ctx, COMET_EINVAL, "%s: op must be COMET_OP_SOMM or COMET_OP_SIMM", what);
    if (!members || n_members < 1 || n_members > COMET_SHARE_GROUP_MAX)
        return comet_fail(ctx, COMET_EINVAL, "%s: 1 to %d members", what, (int)COMET_SHARE_GROUP_MAX);
    GemmParams ps[COMET_SHARE_GROUP_MAX] = {};
    for (int j = 0; j < n_members; ++j) {
        const comet_share_operands& o = members[j];
        const int rc = op == COMET_OP_SOMM
            ? somm_params(ctx, what, ps[j], o.party, m, k, n, bs, blk_idx, n_blk_dev, n_blk_cap, flags, o.E, o.F,
                          o.A_i, o.B_i, o.C_i, o.Z_i)
            : simm_params(ctx, what, ps[j], o.party, m, k, n, bs, blk_idx, n_blk_dev, n_blk_cap, flags, o.E, o.F,
                          o.A_i, o.B_i, o.C_i, o.Z_i);
        if (rc) return rc;
    }
    return run_share_group(ctx, what, ps, n_members, ws, ws_bytes);
}

int comet_simm_share_masked(comet_ctx* ctx, int party, int64_t m, int64_t k_full, int64_t n,
                            int bs, const int32_t* blk_idx, const int32_t* n_blk_dev,
                            int n_blk_cap, int flags, const uint8_t* token_mask, int64_t nb,
                            const uint64_t* E, const uint64_t* F, const uint64_t* A_i,
                            const uint64_t* B_i, const uint64_t* C_i, uint64_t* Z_i, void* ws,
                            size_t ws_bytes) {
    const char* what = "comet_simm_share_masked";
    COMET_CHECK_CTX(ctx);
    if (!token_mask || !blk_idx)
        return comet_fail(ctx, COMET_EINVAL, "%s: token_mask and blk_idx are required", what);
    if (nb < 1 || nb > COMET_DIM_MAX) return comet_fail(ctx, COMET_EINVAL, "%s: bad nb", what);
    GemmParams p = {};
    const int rc = simm_params(ctx, what, p, party, m, k_full, n, bs, blk_idx, n_blk_dev, n_blk_cap, flags,
                               E, F, A_i, B_i, C_i, Z_i);
    if (rc) return rc;
    p.tmask = token_mask; p.tmask_nb = nb;
    return run_share(ctx, what, p, ws, ws_bytes);
}

}  // extern "C"
