// Step 1 of Protocol 2 (paper Sec. 5.1): the optimal grouping of the requested outputs into
// result blocks is the set of connected components of the bipartite graph (rows of X | columns
// of Y, one edge per non-zero output).  The sparsity distribution is plaintext on each server,
// so this is a local, communication-free search.  Here the graph is at (token, neuron block)
// granularity: at most 1024 tokens and 4096 blocks, a few hundred edges per token.
//
// The paper names depth-first search; on the GPU the whole graph fits the LDS of one compute
// unit, so one workgroup finds the same components by label propagation:
//   * the mask is packed into one bit per edge (row-major bit words in LDS);
//   * every token starts with its own number as label; a round gives every block the smallest
//     label among its tokens (pushed along the edges with LDS atomics) and then every token
//     the smallest label among its blocks; labels
//     only ever decrease, so the rounds end, with every node of a component carrying the
//     component's smallest token;
//   * components are numbered by that token (ascending), and the tokens and blocks that take
//     part are sorted by (component, own number) with a bitonic sort in LDS.
// The result is unique (the partition) up to the order of listing, which is fixed as above.
//
// Graphs beyond the one-workgroup limits (element-granular masks at FFN width: hundreds of tokens
// by more than ten thousand neurons) take a second path of four launches without any waiting
// between workgroups:
//   * init: every token and every block is its own tree (parent = own number; tokens are
//     numbered below blocks);
//   * hook: the mask bytes are read once, by as many workgroups as there are; every edge unites
//     the trees of its token and its block with a compare-and-swap that hangs the larger root
//     under the smaller one (lock-free union-find: a failed swap means another edge got there
//     first, the roots are looked up again), so the root of a tree ends up as the smallest
//     token of its component;
//   * flatten: every node looks up its root once more and stores it;
//   * list: one workgroup numbers the roots in ascending order and sorts the tokens and the
//     blocks that take part by component with a stable one-bit-per-pass radix split in LDS.
// The parent pointers and the "takes part" flags live in the caller's four output arrays, so
// this path needs no workspace either.
#include "common.h"

namespace {

constexpr int CT = 256;
constexpr int MAX_TOK = 1024;       // tokens: the label fits 10 bits of a sort key
constexpr int MAX_NB = 4096;        // blocks: 12 bits of a sort key
constexpr int MAX_WORDS = 16384;    // bit words of the packed mask (64 KB of LDS)
constexpr int NONE = 0x7fffffff;

// ascending bitonic sort of keys[0 .. P), P a power of two
__device__ void sort_keys(int* keys, int P) {
    for (int k = 2; k <= P; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = threadIdx.x; i < P; i += CT) {
                const int l = i ^ j;
                if (l > i) {
                    const int a = keys[i], b = keys[l];
                    const bool asc = (i & k) == 0;
                    if ((a > b) == asc) { keys[i] = b; keys[l] = a; }
                }
            }
            __syncthreads();
        }
}

__global__ __launch_bounds__(CT) void components_kernel(const uint8_t* __restrict__ mask, int n_tok, int nb,
                                                        int* __restrict__ row_idx, int* __restrict__ row_comp,
                                                        int* __restrict__ n_row_dev, int* __restrict__ blk_idx,
                                                        int* __restrict__ blk_comp, int* __restrict__ n_blk_dev,
                                                        int* __restrict__ n_comp_dev) {
    __shared__ u32 bits[MAX_WORDS];
    __shared__ int lr[MAX_TOK];      // label of a token, NONE when it has no active block
    __shared__ int lb[MAX_NB];       // label of a block, NONE when no token uses it
    __shared__ int keys[MAX_NB];
    __shared__ int cnum[MAX_TOK];    // component number of the component whose smallest token is t
    __shared__ int changed;
    const int wpr = (nb + 31) >> 5;

    // edges -> bit words; the 32 flags of a word are requested together (independent loads),
    // as eight 4-byte words when every row starts on a 4-byte boundary
    const bool rows4 = (reinterpret_cast<uintptr_t>(mask) & 3u) == 0 && (nb & 3) == 0;
    for (int i = threadIdx.x; i < n_tok * wpr; i += CT) {
        const int t = i / wpr, w = i - t * wpr;
        const uint8_t* src = mask + (size_t)t * nb + w * 32;
        const int lim = nb - w * 32 < 32 ? nb - w * 32 : 32;          // flags of this word inside the row
        u32 v = 0;
        if (rows4) {
            u32 q[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) q[j] = *reinterpret_cast<const u32*>(src + (4 * j < lim ? 4 * j : 0));
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (4 * j >= lim) continue;
                v |= ((q[j] & 0x000000ffu) ? 1u : 0u) << (4 * j);
                v |= ((q[j] & 0x0000ff00u) ? 2u : 0u) << (4 * j);
                v |= ((q[j] & 0x00ff0000u) ? 4u : 0u) << (4 * j);
                v |= ((q[j] & 0xff000000u) ? 8u : 0u) << (4 * j);
            }
        } else {
            uint8_t q[32];
#pragma unroll
            for (int j = 0; j < 32; ++j) q[j] = src[j < lim ? j : 0];
#pragma unroll
            for (int j = 0; j < 32; ++j) v |= ((j < lim && q[j]) ? 1u : 0u) << j;
        }
        bits[i] = v;
    }
    __syncthreads();
    for (int t = threadIdx.x; t < n_tok; t += CT) {
        u32 any = 0;
        for (int w = 0; w < wpr; ++w) any |= bits[t * wpr + w];
        lr[t] = any ? t : NONE;
    }
    __syncthreads();

    // label propagation; a label is a token number and only decreases, so n_tok rounds suffice
    for (int round = 0; round <= n_tok; ++round) {
        if (threadIdx.x == 0) changed = 0;
        // blocks take the smallest label among their tokens: every token pushes its label along
        // its edges (work proportional to the number of edges, LDS atomics)
        for (int b = threadIdx.x; b < nb; b += CT) lb[b] = NONE;
        __syncthreads();
        for (int t = threadIdx.x; t < n_tok; t += CT) {
            const int mine = lr[t];
            for (int w = 0; w < wpr; ++w) {
                u32 v = bits[t * wpr + w];
                while (v) {
                    atomicMin(&lb[w * 32 + __builtin_ctz(v)], mine);
                    v &= v - 1;
                }
            }
        }
        __syncthreads();
        // tokens take the smallest label among their blocks
        for (int t = threadIdx.x; t < n_tok; t += CT) {
            int m = lr[t];
            for (int w = 0; w < wpr; ++w) {
                u32 v = bits[t * wpr + w];
                while (v) {
                    const int x = lb[w * 32 + __builtin_ctz(v)];
                    m = x < m ? x : m;
                    v &= v - 1;
                }
            }
            if (m < lr[t]) { lr[t] = m; changed = 1; }
        }
        __syncthreads();
        const int again = changed;
        __syncthreads();
        if (!again) break;
    }

    // number the components by their smallest token
    if (threadIdx.x == 0) {
        int c = 0;
        for (int t = 0; t < n_tok; ++t) cnum[t] = (lr[t] == t) ? c++ : -1;
        *n_comp_dev = c;
    }
    __syncthreads();

    // tokens that take part, by (component, token)
    int P = 1;
    while (P < n_tok) P <<= 1;
    for (int i = threadIdx.x; i < P; i += CT)
        keys[i] = (i < n_tok && lr[i] != NONE) ? (cnum[lr[i]] << 10) | i : NONE;
    __syncthreads();
    sort_keys(keys, P);
    for (int i = threadIdx.x; i < n_tok; i += CT) {
        const int key = keys[i];
        if (key != NONE) { row_idx[i] = key & 1023; row_comp[i] = key >> 10; }
        if (key != NONE && (i + 1 == n_tok || keys[i + 1] == NONE)) *n_row_dev = i + 1;
    }
    if (threadIdx.x == 0 && keys[0] == NONE) *n_row_dev = 0;
    __syncthreads();

    // blocks that are used, by (component, block)
    P = 1;
    while (P < nb) P <<= 1;
    for (int i = threadIdx.x; i < P; i += CT)
        keys[i] = (i < nb && lb[i] != NONE) ? (cnum[lb[i]] << 12) | i : NONE;
    __syncthreads();
    sort_keys(keys, P);
    for (int i = threadIdx.x; i < nb; i += CT) {
        const int key = keys[i];
        if (key != NONE) { blk_idx[i] = key & 4095; blk_comp[i] = key >> 12; }
        if (key != NONE && (i + 1 == nb || keys[i + 1] == NONE)) *n_blk_dev = i + 1;
    }
    if (threadIdx.x == 0 && keys[0] == NONE) *n_blk_dev = 0;
}

// ---------------------------------------------------------------------------
// multi-workgroup path
// ---------------------------------------------------------------------------
constexpr int BIG_MAX_TOK = 4096;     // component numbers and token numbers fit 12 bits
constexpr int BIG_MAX_NB = 16384;     // block numbers fit 14 bits
constexpr int LT = 1024;              // threads of the listing workgroup
constexpr unsigned short NONE16 = 0xffff;

// parent of node v: tokens 0 .. n_tok-1 in par_r, blocks n_tok .. in par_b
__device__ __forceinline__ int* parent_of(int v, int n_tok, int* par_r, int* par_b) {
    return v < n_tok ? par_r + v : par_b + (v - n_tok);
}

// Root of v with path halving.  Parent pointers only ever move towards the root, so a stale
// read is still an ancestor and the racy shortcut stores are harmless.
__device__ __forceinline__ int find_root(int v, int n_tok, int* par_r, int* par_b) {
    int p = __atomic_load_n(parent_of(v, n_tok, par_r, par_b), __ATOMIC_RELAXED);
    while (p != v) {
        const int gp = __atomic_load_n(parent_of(p, n_tok, par_r, par_b), __ATOMIC_RELAXED);
        if (gp != p) __atomic_store_n(parent_of(v, n_tok, par_r, par_b), gp, __ATOMIC_RELAXED);
        v = p;
        p = gp;
    }
    return v;
}

__device__ __forceinline__ void unite(int a, int b, int n_tok, int* par_r, int* par_b) {
    int ra = find_root(a, n_tok, par_r, par_b), rb = find_root(b, n_tok, par_r, par_b);
    while (ra != rb) {
        const int hi = ra > rb ? ra : rb, lo = ra > rb ? rb : ra;
        const int old = atomicCAS(parent_of(hi, n_tok, par_r, par_b), hi, lo);
        if (old == hi) return;                       // hi was still a root: hooked under lo
        ra = find_root(old, n_tok, par_r, par_b);    // somebody else moved hi: start from where it points now
        rb = find_root(lo, n_tok, par_r, par_b);
    }
}

__global__ __launch_bounds__(CT) void cc_init_kernel(int n_tok, int nb, int* par_r, int* flag_r, int* par_b,
                                                     int* flag_b) {
    const int i = blockIdx.x * CT + threadIdx.x;
    if (i < n_tok) { par_r[i] = i; flag_r[i] = 0; }
    if (i < nb) { par_b[i] = n_tok + i; flag_b[i] = 0; }
}

// one thread per run of 16 flags of one token
__global__ __launch_bounds__(CT) void cc_hook_kernel(const uint8_t* __restrict__ mask, int n_tok, int nb,
                                                     int* par_r, int* flag_r, int* par_b, int* flag_b) {
    const int groups = (nb + 15) >> 4;
    const long total = (long)n_tok * groups;
    const bool rows16 = (reinterpret_cast<uintptr_t>(mask) & 15u) == 0 && (nb & 15) == 0;
    for (long i = (long)blockIdx.x * CT + threadIdx.x; i < total; i += (long)gridDim.x * CT) {
        const int t = (int)(i / groups), c0 = (int)(i - (long)t * groups) * 16;
        const uint8_t* src = mask + (size_t)t * nb + c0;
        u32 bits = 0;
        if (rows16) {
            typedef u32 u32x4 __attribute__((ext_vector_type(4)));
            const u32x4 q = *reinterpret_cast<const u32x4*>(src);
            const u32 w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                bits |= ((w[j] & 0x000000ffu) ? 1u : 0u) << (4 * j);
                bits |= ((w[j] & 0x0000ff00u) ? 2u : 0u) << (4 * j);
                bits |= ((w[j] & 0x00ff0000u) ? 4u : 0u) << (4 * j);
                bits |= ((w[j] & 0xff000000u) ? 8u : 0u) << (4 * j);
            }
        } else {
            const int lim = nb - c0 < 16 ? nb - c0 : 16;
            for (int j = 0; j < lim; ++j) bits |= (src[j] ? 1u : 0u) << j;
        }
        if (!bits) continue;
        flag_r[t] = 1;
        while (bits) {
            const int c = c0 + __builtin_ctz(bits);
            bits &= bits - 1;
            flag_b[c] = 1;
            unite(t, n_tok + c, n_tok, par_r, par_b);
        }
    }
}

// Every node stores its root.  The walk up writes nothing here: a shortcut store from another
// node's walk could otherwise land after this node's final store and leave an ancestor that
// is not the root.  Whatever a walk reads is an ancestor (old parent or root), so it still
// ends at the root.
__global__ __launch_bounds__(CT) void cc_flatten_kernel(int n_tok, int nb, int* par_r, int* par_b) {
    const int v = blockIdx.x * CT + threadIdx.x;
    if (v >= n_tok + nb) return;
    int r = v;
    for (;;) {
        const int p = __atomic_load_n(parent_of(r, n_tok, par_r, par_b), __ATOMIC_RELAXED);
        if (p == r) break;
        r = p;
    }
    __atomic_store_n(parent_of(v, n_tok, par_r, par_b), r, __ATOMIC_RELAXED);
}

// Exclusive prefix sum over the LT threads of the listing workgroup.  sm: LT / 64 ints.
__device__ __forceinline__ int list_excl_scan(int v, int* sm, int* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(inc, d, 64);
        if (lane >= d) inc += o;
    }
    if (lane == 63) sm[wave] = inc;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < LT / 64; ++w) {
        const int x = sm[w];
        if (w < wave) base += x;
        tot += x;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

// Stable split of ids[0 .. n) (in src) by predicate: the ids whose predicate is false keep their
// order at the front of dst, the others follow in their order.  Every thread owns a contiguous
// run of PER ids.  Returns the number of ids at the front.
template <int PER, class Pred>
__device__ __forceinline__ int stable_split(const unsigned short* src, unsigned short* dst, int n, int* sm,
                                            Pred pred) {
    const int i0 = threadIdx.x * PER;
    int zeros = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j)
        if (i0 + j < n && !pred(src[i0 + j])) ++zeros;
    int total0;
    int z = list_excl_scan(zeros, sm, &total0);
    // ids with a true predicate: position = total0 + (ids before minus false ones before)
    int o = total0 + (i0 < n ? i0 : n) - z;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        if (i0 + j < n) {
            const unsigned short id = src[i0 + j];
            if (!pred(id)) dst[z++] = id; else dst[o++] = id;
        }
    }
    __syncthreads();
    return total0;
}

// ids 0 .. n with comp[id] != NONE16, ordered by (comp, id): compaction, then one stable split
// per bit of the component number, lowest bit first.  Result in `a` (b is scratch).
template <int PER>
__device__ int sort_by_component(unsigned short* a, unsigned short* b, const unsigned short* comp, int n,
                                 int n_comp, int* sm) {
    for (int i = threadIdx.x; i < n; i += LT) a[i] = (unsigned short)i;
    __syncthreads();
    const int valid = stable_split<PER>(a, b, n, sm, [&](unsigned short id) { return comp[id] == NONE16; });
    unsigned short *src = b, *dst = a;
    for (int bit = 0; bit < 12 && ((n_comp - 1) >> bit) > 0; ++bit) {
        stable_split<PER>(src, dst, valid, sm, [&](unsigned short id) { return (comp[id] >> bit) & 1; });
        unsigned short* t = src; src = dst; dst = t;
    }
    if (src != a) {
        for (int i = threadIdx.x; i < valid; i += LT) a[i] = src[i];
        __syncthreads();
    }
    return valid;
}

__global__ __launch_bounds__(LT) void cc_list_kernel(int n_tok, int nb, int* row_idx, int* row_comp,
                                                     int* n_row_dev, int* blk_idx, int* blk_comp,
                                                     int* n_blk_dev, int* n_comp_dev) {
    __shared__ unsigned short comp_r[BIG_MAX_TOK];   // first the root of token t, then its component number
    __shared__ unsigned short comp_b[BIG_MAX_NB];
    __shared__ unsigned short cnum[BIG_MAX_TOK];     // component number of the component rooted at token t
    __shared__ unsigned short ping[BIG_MAX_NB], pong[BIG_MAX_NB];
    __shared__ int sm[LT / 64];
    // everything this kernel reads from the output arrays is read here, before anything is written
    for (int t = threadIdx.x; t < n_tok; t += LT) comp_r[t] = row_idx[t] ? (unsigned short)row_comp[t] : NONE16;
    for (int c = threadIdx.x; c < nb; c += LT) comp_b[c] = blk_idx[c] ? (unsigned short)blk_comp[c] : NONE16;
    __syncthreads();
    // number the roots (a root is a token that takes part and is its own root) in ascending order
    constexpr int TPER = BIG_MAX_TOK / LT;
    int mine = 0;
    const int t0 = threadIdx.x * TPER;
#pragma unroll
    for (int j = 0; j < TPER; ++j)
        if (t0 + j < n_tok && comp_r[t0 + j] == t0 + j) ++mine;
    int n_comp;
    int at = list_excl_scan(mine, sm, &n_comp);
#pragma unroll
    for (int j = 0; j < TPER; ++j)
        if (t0 + j < n_tok && comp_r[t0 + j] == t0 + j) cnum[t0 + j] = (unsigned short)at++;
    __syncthreads();
    // roots -> component numbers (every root is a token below n_tok)
    for (int t = threadIdx.x; t < n_tok; t += LT) {
        const unsigned short r = comp_r[t];
        comp_r[t] = r == NONE16 ? NONE16 : cnum[r];
    }
    for (int c = threadIdx.x; c < nb; c += LT) {
        const unsigned short r = comp_b[c];
        comp_b[c] = r == NONE16 ? NONE16 : cnum[r];
    }
    __syncthreads();
    if (threadIdx.x == 0) *n_comp_dev = n_comp;
    const int n_row = sort_by_component<BIG_MAX_TOK / LT>(ping, pong, comp_r, n_tok, n_comp, sm);
    for (int i = threadIdx.x; i < n_row; i += LT) { row_idx[i] = ping[i]; row_comp[i] = comp_r[ping[i]]; }
    if (threadIdx.x == 0) *n_row_dev = n_row;
    __syncthreads();
    const int n_blk = sort_by_component<BIG_MAX_NB / LT>(ping, pong, comp_b, nb, n_comp, sm);
    for (int i = threadIdx.x; i < n_blk; i += LT) { blk_idx[i] = ping[i]; blk_comp[i] = comp_b[ping[i]]; }
    if (threadIdx.x == 0) *n_blk_dev = n_blk;
}

}  // namespace

extern "C" int comet_components(comet_ctx* ctx, const uint8_t* mask, int64_t n_tok, int64_t nb,
                                int32_t* row_idx, int32_t* row_comp, int32_t* n_row_dev,
                                int32_t* blk_idx, int32_t* blk_comp, int32_t* n_blk_dev,
                                int32_t* n_comp_dev) {
    const char* what = "comet_components";
    COMET_CHECK_CTX(ctx);
    if (!mask || !row_idx || !row_comp || !n_row_dev || !blk_idx || !blk_comp || !n_blk_dev || !n_comp_dev)
        return comet_fail(ctx, COMET_EINVAL, "%s: null pointer", what);
    if (n_tok < 1 || nb < 1) return comet_fail(ctx, COMET_EINVAL, "%s: need n_tok >= 1, nb >= 1", what);
    const bool small = n_tok <= MAX_TOK && nb <= MAX_NB && n_tok * ((nb + 31) / 32) <= MAX_WORDS;
    if (n_tok > BIG_MAX_TOK || nb > BIG_MAX_NB)
        return comet_fail(ctx, COMET_ECAP, "%s: at most 4096 tokens and 16384 blocks", what);
    const void* outs[] = {row_idx, row_comp, n_row_dev, blk_idx, blk_comp, n_blk_dev, n_comp_dev};
    for (const void* q : outs)
        if (reinterpret_cast<uintptr_t>(q) & 3u)
            return comet_fail(ctx, COMET_EALIGN, "%s: int32 outputs must be 4-byte aligned", what);
    comet_device_guard guard(ctx);
    if (!guard.ok) return comet_fail(ctx, COMET_EDEVICE, "%s: cannot select device", what);
    if (small && ctx->components_mode != 1) {
        hipLaunchKernelGGL(components_kernel, dim3(1), dim3(CT), 0, ctx->stream, mask, (int)n_tok, (int)nb,
                           row_idx, row_comp, n_row_dev, blk_idx, blk_comp, n_blk_dev, n_comp_dev);
        COMET_LAUNCH_CHECK(ctx, what);
        return COMET_OK;
    }
    // parent pointers in row_comp / blk_comp, "takes part" flags in row_idx / blk_idx
    const int nt = (int)n_tok, nbi = (int)nb;
    const int most = nt > nbi ? nt : nbi;
    hipLaunchKernelGGL(cc_init_kernel, dim3((most + CT - 1) / CT), dim3(CT), 0, ctx->stream, nt, nbi, row_comp,
                       row_idx, blk_comp, blk_idx);
    COMET_LAUNCH_CHECK(ctx, what);
    const long runs = (long)nt * ((nbi + 15) / 16);
    long grid = (runs + CT - 1) / CT;
    if (grid > 16l * ctx->num_cu) grid = 16l * ctx->num_cu;
    hipLaunchKernelGGL(cc_hook_kernel, dim3((unsigned)grid), dim3(CT), 0, ctx->stream, mask, nt, nbi, row_comp,
                       row_idx, blk_comp, blk_idx);
    COMET_LAUNCH_CHECK(ctx, what);
    hipLaunchKernelGGL(cc_flatten_kernel, dim3((nt + nbi + CT - 1) / CT), dim3(CT), 0, ctx->stream, nt, nbi,
                       row_comp, blk_comp);
    COMET_LAUNCH_CHECK(ctx, what);
    hipLaunchKernelGGL(cc_list_kernel, dim3(1), dim3(LT), 0, ctx->stream, nt, nbi, row_idx, row_comp, n_row_dev,
                       blk_idx, blk_comp, n_blk_dev, n_comp_dev);
    COMET_LAUNCH_CHECK(ctx, what);
    return COMET_OK;
}
