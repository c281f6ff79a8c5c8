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
    __shared__ int changed, n_comp;
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
        n_comp = c;
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
    if (n_tok > MAX_TOK || nb > MAX_NB || n_tok * ((nb + 31) / 32) > MAX_WORDS)
        return comet_fail(ctx, COMET_ECAP,
                          "%s: at most 1024 tokens, 4096 blocks and 16384 packed mask words", what);
    const void* outs[] = {row_idx, row_comp, n_row_dev, blk_idx, blk_comp, n_blk_dev, n_comp_dev};
    for (const void* q : outs)
        if (reinterpret_cast<uintptr_t>(q) & 3u)
            return comet_fail(ctx, COMET_EALIGN, "%s: int32 outputs must be 4-byte aligned", what);
    comet_device_guard guard(ctx);
    if (!guard.ok) return comet_fail(ctx, COMET_EDEVICE, "%s: cannot select device", what);
    hipLaunchKernelGGL(components_kernel, dim3(1), dim3(CT), 0, ctx->stream, mask, (int)n_tok, (int)nb,
                       row_idx, row_comp, n_row_dev, blk_idx, blk_comp, n_blk_dev, n_comp_dev);
    COMET_LAUNCH_CHECK(ctx, what);
    return COMET_OK;
}
