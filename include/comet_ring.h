/*
 * comet_ring.h -- C ABI of the MI355X (gfx950) library for one party's local
 * work in the sparse, secret-shared FFN matrix multiply over the ring Z_{2^64}.
 *
 * Notation follows the paper's Sec. 5: Z = X Y with X (m x k) the activations
 * and Y (k x n) the weights, additively shared between two parties
 * (Sec. 2.1).  "party" is 0-based: party 0 is the paper's P_1, party 1 is
 * P_2, the one whose share carries the extra E F term of Eq. 1.
 *
 * Conventions that hold for every call unless stated otherwise
 *   - every matrix / vector pointer is a DEVICE pointer owned by the caller,
 *     16-byte aligned, dense row-major, elements are uint64_t taken mod 2^64
 *     (int32 index lists and counts: 4-byte aligned; byte masks: any alignment);
 *   - the library never allocates or frees device memory and never frees or
 *     retains caller memory; scratch space comes in through (ws, ws_bytes),
 *     sized with comet_workspace_bytes(), must be 256-byte aligned (COMET_EALIGN
 *     otherwise) and may be reused between calls that do not overlap in time;
 *   - calls enqueue work on the context's stream and return without waiting;
 *     buffers must stay valid until that work has run;
 *   - the predicted sparsity distribution is a plaintext list of active
 *     blocks of `bs` consecutive neurons: blk_idx[0 .. n_blk) ascending block
 *     ids on the device, with the count n_blk itself on the device
 *     (n_blk_dev, one int32) so that compaction and the matmul chain without
 *     a host round trip.  n_blk_cap is a host-side upper bound on n_blk (the
 *     sparsity LEVEL is public in the paper's threat model, Sec. 3.2); it
 *     fixes the leading dimension of every compact operand,
 *     ld = n_blk_cap * bs.  n_blk_dev may be NULL, meaning n_blk = n_blk_cap.
 *     Columns / rows of compact operands at or beyond n_blk * bs are neither
 *     read nor written;
 *   - return value 0 on success, a negative COMET_E* code otherwise;
 *     comet_last_error() gives a text for the last failure on that context.
 *     Argument errors are detected on the host before anything is enqueued.
 *     No C++ types or exceptions cross this boundary.
 */
#ifndef COMET_RING_H
#define COMET_RING_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct comet_ctx comet_ctx;

enum {
    COMET_OK = 0,
    COMET_EINVAL = -1,     /* null pointer, negative or inconsistent size, bad enum      */
    COMET_EALIGN = -2,     /* an operand is not 16-byte, a workspace not 256-byte aligned */
    COMET_ECAP = -3,       /* size beyond what the kernels index (see each call)         */
    COMET_EDEVICE = -4,    /* no such device / wrong architecture / HIP runtime failure  */
    COMET_EWORKSPACE = -5  /* ws is NULL or smaller than comet_workspace_bytes() says    */
};

/* which axis of a full-size matrix the block list selects */
enum { COMET_AXIS_COLS = 0, COMET_AXIS_ROWS = 1 };

/* operations known to comet_workspace_bytes() */
enum { COMET_OP_COMPACT = 0, COMET_OP_SOMM = 1, COMET_OP_SIMM = 2 };

/* flags of the share calls.
 * COMET_FULL_A / COMET_FULL_B: the named triple share is passed at FULL size
 * and is indexed by blk_idx inside the kernel (otherwise it is already compact).
 * COMET_WEIGHTS_NEURON_MAJOR (SOMM calls): the weight-side operands B_i and F
 * are stored one ROW per neuron (n x k, the transpose of the k x n form), the
 * layout in which a kept neuron is one contiguous run of k words in both
 * projections of an FFN (the weights are permuted and stored once, offline,
 * Sec. 4.2, so their layout is free to choose).  The result is the same.
 * COMET_WEIGHT_PLANES: the weight-side operands B_i and F are passed as DIGIT
 * PLANES, the format comet_open_weight_planes() writes (the opened F directly
 * from the two masked shares, B_i packed once, offline, like the triple itself,
 * Sec. 3.2), at the same logical shapes as their word forms.  The share kernels
 * then move both operands into the matrix cores without any per-step
 * arithmetic; the result is the same, bit for bit.  Not with
 * COMET_WEIGHTS_NEURON_MAJOR; with COMET_FULL_B in a SIMM call bs must be a
 * multiple of 16 (COMET_EINVAL otherwise). */
enum { COMET_FULL_A = 1, COMET_FULL_B = 2, COMET_WEIGHTS_NEURON_MAJOR = 4, COMET_WEIGHT_PLANES = 8 };

/* ---- context ---------------------------------------------------------- */

/* Create a context bound to HIP device `device_id` (must be a gfx950 part).
 * Allocates host memory only.  The context starts on the NULL stream. */
int comet_create(comet_ctx** out, int device_id);
int comet_destroy(comet_ctx* ctx);
/* hip_stream: a hipStream_t (NULL = default stream).  Not owned. */
int comet_set_stream(comet_ctx* ctx, void* hip_stream);
const char* comet_last_error(const comet_ctx* ctx);
/* Library version string, static storage. */
const char* comet_version(void);

/* Bytes of scratch the operation needs for the given sizes.
 *   COMET_OP_COMPACT: m = n_tok, k unused, n = nb, bs unused
 *   COMET_OP_SOMM   : m, k, n = n_blk_cap * bs (compact width), bs
 *   COMET_OP_SIMM   : m, k = n_blk_cap * bs (compact contraction), n, bs
 * Returns 0 for sizes the operation would reject. */
size_t comet_workspace_bytes(int op, int64_t m, int64_t k, int64_t n, int bs);

/* ---- (1) mask and open shares: Sec. 2.1 multiplication, Sec. 5.1 -------- */

/* [D]_i = [X]_i - [A]_i, elementwise over n_elems words: the masked share a
 * party sends to the other one.  d_i may be the same buffer as x_i or a_i
 * (exactly the same address; partially overlapping buffers are not allowed). */
int comet_mask_share(comet_ctx* ctx, const uint64_t* x_i, const uint64_t* a_i,
                     uint64_t* d_i, size_t n_elems);

/* Indexed variant: masks only what the sparsity distribution keeps, which is
 * where the protocol's communication saving comes from (Protocol 2: IndexCols
 * before Pi_MatMul; Protocol 3: IndexCol / IndexRow before Pi_MatMul).
 * w_i, b_i: full rows x cols.
 *   axis = COMET_AXIS_COLS: g_i is rows x ld, g[r][c] = w[r][j] - b[r][j],
 *                           j = blk_idx[c / bs] * bs + c % bs, c < n_blk * bs
 *   axis = COMET_AXIS_ROWS: g_i is ld x cols, g[r][c] = w[j][c] - b[j][c],
 *                           j = blk_idx[r / bs] * bs + r % bs, r < n_blk * bs
 * Block ids should satisfy (blk_idx[t] + 1) * bs <= cols (resp. rows); a block
 * whose id does not fit is skipped (its outputs are left untouched). */
int comet_mask_share_gather(comet_ctx* ctx, const uint64_t* w_i, const uint64_t* b_i,
                            uint64_t* g_i, int64_t rows, int64_t cols, int axis, int bs,
                            const int32_t* blk_idx, const int32_t* n_blk_dev, int n_blk_cap);

/* E = [D]_0 + [D]_1: reconstruction of the masked value after the exchange
 * (both parties live in one process here, so the exchange is this add).
 * e may be the same buffer as d_0 or d_1 (same address, no partial overlap). */
int comet_open(comet_ctx* ctx, const uint64_t* d_0, const uint64_t* d_1, uint64_t* e,
               size_t n_elems);

/* The opening of a weight-side operand written as digit planes: planes :=
 * pack(g_0 + g_1) for a k x n row-major matrix of words (k = contraction rows,
 * n = columns), or pack(g_0) when g_1 is NULL (used once, offline, for a triple
 * share B_i).  Each word x is split into eight signed base-256 digits d_t
 * (x = sum d_t 2^(8t) mod 2^64, -128 <= d_t <= 127); a 16-byte unit holds digit t
 * of the sixteen rows 32 s + 16 g + 0..15 of one column c, and units are ordered
 * (s, c / 64, t, g, c % 64); rows at or beyond k read as zero, the last chunk of
 * 64 columns is padded (its padding is never read).  planes must hold
 * comet_weight_planes_bytes(k, n) = ceil(k / 32) * 32 * ceil(n / 64) * 64 * 8
 * bytes and must not overlap the inputs.  Pass the
 * result wherever a share call takes F or B_i, together with
 * COMET_WEIGHT_PLANES.  k, n < 2^24, k * n < 2^31. */
size_t comet_weight_planes_bytes(int64_t k, int64_t n);
int comet_open_weight_planes(comet_ctx* ctx, const uint64_t* g_0, const uint64_t* g_1, int64_t k,
                             int64_t n, void* planes);

/* comet_open_weight_planes for operands stored one ROW per column of the matrix
 * (g_0, g_1: n x k words, row c = column c of the k x n matrix the planes stand
 * for): the neuron-major layout of the SOMM weights (see
 * COMET_WEIGHTS_NEURON_MAJOR), in which the kept neurons are gathered as whole
 * rows (comet_mask_share_gather with COMET_AXIS_ROWS).  The planes are the same,
 * byte for byte, as those of the row-major call on the transposed operands. */
int comet_open_weight_planes_neuron_major(comet_ctx* ctx, const uint64_t* g_0, const uint64_t* g_1,
                                          int64_t k, int64_t n, void* planes);

/* ---- (2) sparsity distribution -> ordered index list -------------------- */

/* mask: n_tok x nb bytes, non-zero = block predicted active for that token
 * (any alignment).  The masks of all tokens are OR-ed (one matmul serves the
 * whole batch), then blk_idx[0 .. T) receives the ascending ids of the active
 * blocks and *n_blk_dev = T.  blk_idx must hold nb int32 (4-byte aligned);
 * entries at or beyond T are left untouched.  1 <= n_tok, 0 <= nb < 2^31 - 2^16,
 * n_tok * nb <= 2^40.  ws: comet_workspace_bytes(COMET_OP_COMPACT, n_tok, 0, nb, 0)
 * bytes of device memory, 256-byte aligned (none for a single row of at most
 * 4096 flags, nor for up to 128 KB of flags in rows of at most 4096); it depends
 * on both sizes (COMET_EWORKSPACE when too small).
 * This is the local, communication-free step that Protocol 2 starts with (its
 * graph search degenerates to this when every token keeps the same blocks) and
 * the "find all non-zero columns" step of Protocol 3. */
int comet_compact_mask(comet_ctx* ctx, const uint8_t* mask, int64_t n_tok, int64_t nb,
                       int32_t* blk_idx, int32_t* n_blk_dev, void* ws, size_t ws_bytes);

/* ---- (3) one party's output share: Eq. 1 in matrix form ----------------- */

/* SOMM (Protocol 2, preceding layer: FC1 / gate / up), restricted to the kept
 * output columns:
 *     [Z]_i = [C]_i + E [B]_i + [A]_i F + party * E F        (mod 2^64)
 *   E, A_i : m x k
 *   F      : k x ld   (compact: opened masked weights of the kept columns)
 *   B_i    : k x n_full when flags & COMET_FULL_B (kept columns are indexed in
 *            the kernel), else k x ld
 *   C_i,Z_i: m x ld   (compact; C = A B on the kept columns)
 * With flags & COMET_WEIGHTS_NEURON_MAJOR, F is ld x k and B_i is n_full x k
 * (COMET_FULL_B: kept rows are indexed in the kernel) or ld x k; k must then
 * be even (COMET_EINVAL otherwise).  Calls with m <= 8 take the matrix-core
 * kernel in this layout (the few-row kernel reads row-major weights).
 * ld = n_blk_cap * bs; column c of a compact operand is neuron
 * blk_idx[c / bs] * bs + c % bs.  Z_i must not alias any input.  A block id
 * that does not fit n_full is read as block 0 (the outputs it feeds are then
 * meaningless; no access ever leaves the operands).
 * Limits: 1 <= m, k, bs; m <= 2^22 - 128; k, ld, n_full < 2^24; F and B_i hold
 * fewer than 2^31 words each (COMET_ECAP beyond them). */
int comet_somm_share(comet_ctx* ctx, int party, int64_t m, int64_t k, int64_t n_full, int bs,
                     const int32_t* blk_idx, const int32_t* n_blk_dev, int n_blk_cap, int flags,
                     const uint64_t* E, const uint64_t* F, const uint64_t* A_i,
                     const uint64_t* B_i, const uint64_t* C_i, uint64_t* Z_i,
                     void* ws, size_t ws_bytes);

/* comet_somm_share for callers that cannot allocate device memory and have no
 * workspace to pass: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments and result as
 * comet_somm_share, without (ws, ws_bytes): the scratch is a static device array
 * of COMET_STATIC_SCRATCH_BYTES inside the library (each GPU the library runs
 * on holds its own copy until the process ends).  The call allocates nothing.
 * Sizes whose comet_workspace_bytes(COMET_OP_SOMM, ...) exceeds the array are
 * rejected with COMET_ECAP.  All calls on one GPU share that GPU's array, from
 * any context or stream: calls that overlap in time on one GPU race, the caller
 * must order them (one stream, or events). */
enum { COMET_STATIC_SCRATCH_BYTES = 32 * 1024 * 1024 };
int comet_somm_share_static(comet_ctx* ctx, int party, int64_t m, int64_t k, int64_t n_full, int bs,
                            const int32_t* blk_idx, const int32_t* n_blk_dev, int n_blk_cap,
                            int flags, const uint64_t* E, const uint64_t* F, const uint64_t* A_i,
                            const uint64_t* B_i, const uint64_t* C_i, uint64_t* Z_i);

/* SIMM (Protocol 3, subsequent layer: FC2 / down), contraction restricted to
 * the kept neurons (the sum of the per-neuron outer products of Protocol 3):
 *     [Z]_i = [C]_i + E [B]_i + [A]_i F + party * E F        (mod 2^64)
 *   E      : m x ld   (compact: opened masked activations of the kept neurons)
 *   A_i    : m x k_full when flags & COMET_FULL_A, else m x ld
 *   F      : ld x n   (compact: opened masked weight rows of the kept neurons)
 *   B_i    : k_full x n when flags & COMET_FULL_B, else ld x n
 *   C_i,Z_i: m x n    (C = A_sel B_sel)
 * ld = n_blk_cap * bs; only the first n_blk * bs columns of E / rows of F are
 * contracted.  Z_i must not alias any input.  A block id that does not fit
 * k_full is read as block 0 (see comet_somm_share).
 * Limits: 1 <= m, n, bs; m <= 2^22 - 128; n, ld, k_full < 2^24; F and B_i hold
 * fewer than 2^31 words each (COMET_ECAP beyond them). */
int comet_simm_share(comet_ctx* ctx, int party, int64_t m, int64_t k_full, int64_t n, int bs,
                     const int32_t* blk_idx, const int32_t* n_blk_dev, int n_blk_cap, int flags,
                     const uint64_t* E, const uint64_t* F, const uint64_t* A_i,
                     const uint64_t* B_i, const uint64_t* C_i, uint64_t* Z_i,
                     void* ws, size_t ws_bytes);

/* Decoding (m <= 8 rows): comet_somm_share / comet_simm_share with the opening of
 * the masked weights folded in (Sec. 2.1: F = [G]_0 + [G]_1).  Instead of the
 * opened F the call takes the two masked shares of the indexed weights -- what
 * comet_mask_share(_gather) wrote and what the other party sent -- in F's
 * layout (G_0, G_1: k x ld for SOMM, ld x n for SIMM) and adds them while it
 * streams them.  With a few rows the share is bound by reading the weight side
 * once; opening F first costs a read of both shares, a write of F and a read of
 * F where this call reads both shares once.  The result is the one of the
 * opened call, bit for bit.  Everything else as in comet_somm_share /
 * comet_simm_share, with these limits: m <= 8, row-major words (neither
 * COMET_WEIGHTS_NEURON_MAJOR nor COMET_WEIGHT_PLANES); COMET_EINVAL otherwise. */
int comet_somm_share_unopened(comet_ctx* ctx, int party, int64_t m, int64_t k, int64_t n_full, int bs,
                              const int32_t* blk_idx, const int32_t* n_blk_dev, int n_blk_cap,
                              int flags, const uint64_t* E, const uint64_t* G_0, const uint64_t* G_1,
                              const uint64_t* A_i, const uint64_t* B_i, const uint64_t* C_i,
                              uint64_t* Z_i, void* ws, size_t ws_bytes);
int comet_simm_share_unopened(comet_ctx* ctx, int party, int64_t m, int64_t k_full, int64_t n, int bs,
                              const int32_t* blk_idx, const int32_t* n_blk_dev, int n_blk_cap,
                              int flags, const uint64_t* E, const uint64_t* G_0, const uint64_t* G_1,
                              const uint64_t* A_i, const uint64_t* B_i, const uint64_t* C_i,
                              uint64_t* Z_i, void* ws, size_t ws_bytes);

/* Several share products of one shape in one call: the gate and up projections
 * of one layer (Protocol 2 twice, over the same index list), the share
 * products of several requests, or -- where one process plays both parties --
 * the two parties' shares of one product.  Member j of `members` (an array in
 * HOST memory, read before the call returns) names its party and its own six
 * operands; shape, block size, index list and flags are common to all and mean
 * what they mean for comet_somm_share (op = COMET_OP_SOMM: m, k, n = n_full) or
 * comet_simm_share (op = COMET_OP_SIMM: m, k = k_full, n).  The result is, bit
 * for bit, that of the n_members single calls.  With COMET_WEIGHT_PLANES and
 * m > 64, members that are short launches on their own (see COMET_TUNE_GROUP)
 * run as one operand-packing launch and one matrix-core launch over the union
 * of their work units: the fixed cost of a launch is paid once and the tail of
 * one product is filled by the next.  Otherwise they run one after the other.  No Z_i may alias another member's Z_i or any
 * input.  Workspace: n_members * comet_workspace_bytes(op, ...) bytes.
 * 1 <= n_members <= COMET_SHARE_GROUP_MAX; other limits as for the single
 * calls. */
enum { COMET_SHARE_GROUP_MAX = 8 };
typedef struct comet_share_operands {
    int32_t party;          /* 0 or 1 */
    int32_t reserved;       /* 0 */
    const uint64_t* E;
    const uint64_t* F;
    const uint64_t* A_i;
    const uint64_t* B_i;
    const uint64_t* C_i;
    uint64_t* Z_i;
} comet_share_operands;
int comet_share_group(comet_ctx* ctx, int op, int n_members, const comet_share_operands* members,
                      int64_t m, int64_t k, int64_t n, int bs, const int32_t* blk_idx,
                      const int32_t* n_blk_dev, int n_blk_cap, int flags, void* ws, size_t ws_bytes);

/* ---- (4) Protocols 2 and 3 in general form: per-token sparsity ---------- */

/* Protocol 2 step 1 at (token, neuron block) granularity: connected components
 * of the bipartite graph whose left nodes are the tokens (rows of X), right
 * nodes the neuron blocks (column blocks of Y) and edges the non-zero bytes of
 * mask (n_tok x nb).  Components are numbered by their smallest token.
 *   row_idx / row_comp [n_tok]: the tokens that have at least one active block,
 *       ordered by (component, token), and the component number of each;
 *   blk_idx / blk_comp [nb]: the blocks at least one token uses, ordered by
 *       (component, block), and their component numbers;
 *   *n_row_dev, *n_blk_dev, *n_comp_dev: the three counts (device).
 * Entries beyond the counts hold unspecified values afterwards (the arrays
 * double as scratch).  Small graphs (n_tok <= 1024, nb <= 4096, n_tok *
 * ceil(nb / 32) <= 16384) are searched by one workgroup in LDS; larger ones, up
 * to n_tok <= 4096 and nb <= 16384 (element-granular masks, bs = 1, at FFN
 * width), by a lock-free union-find over all workgroups; COMET_ECAP beyond.
 * All outputs int32, 4-byte aligned.  No workspace. */
int comet_components(comet_ctx* ctx, const uint8_t* mask, int64_t n_tok, int64_t nb,
                     int32_t* row_idx, int32_t* row_comp, int32_t* n_row_dev,
                     int32_t* blk_idx, int32_t* blk_comp, int32_t* n_blk_dev,
                     int32_t* n_comp_dev);

/* Protocol 2 with the result blocks of all components computed by one call.
 * Operands are in the order comet_components lists them: row r of E, A_i, C_i,
 * Z_i is token row_idx[r], column c of the compact operands is neuron
 * blk_idx[c / bs] * bs + c % bs.  Element (r, c) lies on a result block when
 * row_comp[r] == blk_comp[c / bs]; there
 *     [Z]_i = [C]_i + E [B]_i + [A]_i F + party * E F        (mod 2^64)
 * with the component's own triple stored at those rows and columns; everywhere
 * else on the first *n_row_dev rows and *n_blk_dev * bs columns Z_i is set to
 * zero (the merge into an empty matrix).  Tiles of the output that touch no
 * block are skipped.
 *   E, A_i : m_cap x k   (rows at or beyond *n_row_dev are ignored)
 *   F      : k x ld;  B_i: k x n_full when flags & COMET_FULL_B, else k x ld
 *            (transposed, as in comet_somm_share, with COMET_WEIGHTS_NEURON_MAJOR)
 *   C_i,Z_i: m_cap x ld, ld = n_blk_cap * bs
 * n_row_dev may be null (then all m_cap rows take part).  Limits as for
 * comet_somm_share. */
int comet_somm_share_blocks(comet_ctx* ctx, int party, int64_t m_cap, int64_t k, int64_t n_full,
                            int bs, const int32_t* blk_idx, const int32_t* blk_comp,
                            const int32_t* n_blk_dev, int n_blk_cap, const int32_t* row_comp,
                            const int32_t* n_row_dev, int flags, const uint64_t* E,
                            const uint64_t* F, const uint64_t* A_i, const uint64_t* B_i,
                            const uint64_t* C_i, uint64_t* Z_i, void* ws, size_t ws_bytes);

/* Protocol 3 with per-token row sets: as comet_simm_share, but entry (r, j) of
 * the activation-side operands takes part only when token r uses the block of
 * neuron j, i.e. token_mask[r * nb + blk_idx[j / bs]] != 0 (token_mask: m x nb
 * bytes, the sparsity distribution of X at block granularity; R_j of Protocol 3
 * is the set of such r).  Entries outside it are never read as values: they
 * are the ones the parties do not exchange.  C_i is the sum of the scattered
 * column triples' C shares. */
int comet_simm_share_masked(comet_ctx* ctx, int party, int64_t m, int64_t k_full, int64_t n,
                            int bs, const int32_t* blk_idx, const int32_t* n_blk_dev,
                            int n_blk_cap, int flags, const uint8_t* token_mask, int64_t nb,
                            const uint64_t* E, const uint64_t* F, const uint64_t* A_i,
                            const uint64_t* B_i, const uint64_t* C_i, uint64_t* Z_i,
                            void* ws, size_t ws_bytes);

/* ---- (5) local steps around the products ------------------------------- */

/* One local step of the oblivious shuffle's online stage (Protocol 1):
 *     dst = perm(src) + mask   (sign = +1:  y_i = tau_i(x_i) + a_i)
 *     dst = perm(src) - mask   (sign = -1:  z_i = rho_i(y_other) - b_i)
 * A permutation acts as perm(x)_j = x[perm[j]] (the paper's pi = [2,1,3] gives
 * [x_2, x_1, x_3]), along the columns (COMET_AXIS_COLS: dst(r, j) = src(r, perm[j]),
 * perm has cols entries) or the rows (COMET_AXIS_ROWS: dst(j, c) = src(perm[j], c),
 * rows entries) of a rows x cols matrix; mask is in the order of dst.  dst must
 * not alias src.  An entry of perm outside the axis is read as 0 (never a
 * fault; the output is then meaningless).  rows, cols < 2^24. */
int comet_permute_mask(comet_ctx* ctx, const uint64_t* src, const int32_t* perm,
                       const uint64_t* mask, uint64_t* dst, int64_t rows, int64_t cols, int axis,
                       int sign);

/* Merge of a compact result back to the full width ("reshaped to origin size";
 * Protocol 2's Merge for whole column blocks): full (m x n_full) is set to zero
 * and column block t of compact (m x n_blk_cap*bs) is written to neurons
 * blk_idx[t]*bs .. +bs, for t < *n_blk_dev (or n_blk_cap when null).  Applied to
 * each party's share separately it yields shares of the scattered secret.  A
 * block id that does not fit n_full is dropped. */
int comet_scatter_cols(comet_ctx* ctx, const uint64_t* compact, int64_t m, int bs,
                       const int32_t* blk_idx, const int32_t* n_blk_dev, int n_blk_cap,
                       uint64_t* full, int64_t n_full);

/* Share-local rescaling of a fixed-point product by 2^frac_bits:
 *   party 0: out = floor(z / 2^f) on the signed word;  party 1: out = -floor(-z / 2^f).
 * The reconstruction is within one unit of the exact quotient unless the shares
 * wrap around 2^64 (probability about |secret| / 2^63 over the sharing
 * randomness).  The paper does not state its rescaling rule; this is the usual
 * two-party one.  out may alias z. */
int comet_truncate_share(comet_ctx* ctx, int party, const uint64_t* z, uint64_t* out,
                         size_t n_elems, int frac_bits);

/* ---- measurement aids (roofline probes; not part of the protocol) ------- */

/* Launch-shape overrides for sweeps and for tests that must reach a particular
 * code path.  Results never depend on them.  value 0 restores the default.
 *   COMET_TUNE_GEMM_GRID: number of workgroups the share calls launch
 *                         (default: one per compute unit, fewer for tiny work)
 *   COMET_TUNE_GEMM_CHUNK: contraction steps (of 32 words) per scheduling slice,
 *                         clamped to 256
 *   COMET_TUNE_GEMM_TILE: 2 forces the 64 x 64 output tile (two workgroups per
 *                         compute unit) whatever m is
 *   COMET_TUNE_SKINNY:    calls with m <= 8 normally take a vector-ALU kernel
 *                         bound by reading the weights once; 1 sends them to the
 *                         matrix-core kernel like any other call
 *   COMET_TUNE_SKINNY_SLICES: pieces the stacked contraction is cut into by
 *                         the vector-ALU kernel (default: about eight
 *                         workgroups per compute unit)
 *   COMET_TUNE_COMPONENTS: 1 sends every comet_components call to the
 *                         multi-workgroup search (small graphs normally take a
 *                         one-workgroup kernel)
 *   COMET_TUNE_TIMING_STRIDE: while timing is on (comet_timing_begin), time
 *                         every value-th share call instead of every one; a
 *                         timed launch costs the stream about ten microseconds
 *                         of idle time around the kernel
 *   COMET_TUNE_GROUP:     comet_share_group normally runs its members as one
 *                         launch when a member alone is a short launch (8 to
 *                         128 contraction steps of 32 words per workgroup);
 *                         1 = whenever the operands allow it, 2 = never,
 *                         3 = as 1 but without teaming the workgroups of a
 *                         column of tiles (a measurement aid) */
enum { COMET_TUNE_GEMM_GRID = 0, COMET_TUNE_GEMM_CHUNK = 1, COMET_TUNE_GEMM_TILE = 2,
       COMET_TUNE_SKINNY = 3, COMET_TUNE_SKINNY_SLICES = 4, COMET_TUNE_COMPONENTS = 5,
       COMET_TUNE_TIMING_STRIDE = 6, COMET_TUNE_GROUP = 7 };
int comet_set_tuning(comet_ctx* ctx, int key, int value);

/* Device-side timing of the ring-GEMM kernel alone (the share calls also run a
 * small operand-packing kernel, which this excludes).  comet_timing_begin
 * creates up to max_launches HIP event pairs; while timing is on, every share
 * call (every n-th with COMET_TUNE_TIMING_STRIDE = n) attaches one pair to the
 * dispatch of its GEMM kernel on the context's stream: the pair reads the
 * kernel's own start and end (do not keep timing on while the stream is being
 * captured into a HIP graph).  comet_timing_end waits for the last recorded event, returns the summed
 * kernel time and the number of launches timed, and destroys the events. */
int comet_timing_begin(comet_ctx* ctx, int max_launches);
int comet_timing_end(comet_ctx* ctx, double* total_ms, int* launches);

/* Register-resident issue loop of the int8 matrix instruction the ring GEMM
 * uses: launches `blocks` x 256 threads, `iters` dependent-free MFMA groups
 * each.  random_operands = 0: small constant operands; 1: uniformly random
 * operand bytes (the digits of secret shares are uniformly random; the same
 * instruction stream then draws more power and the chip clocks down, so this
 * is the rate a real kernel can approach).  out (device, blocks*256 int32)
 * keeps the results alive.  Returns the number of int8 multiply-accumulates
 * issued through *macs (host). */
int comet_probe_mfma_i8(comet_ctx* ctx, int blocks, int iters, int random_operands, int32_t* out,
                        double* macs);
/* Same for the plain 64-bit vector multiply-add: *macs = ring MACs issued. */
int comet_probe_valu_mac64(comet_ctx* ctx, int blocks, int iters, uint64_t* out, double* macs);
/* Plain device copy of n_elems words (bandwidth yardstick, 16 B per element). */
int comet_probe_copy(comet_ctx* ctx, const uint64_t* src, uint64_t* dst, size_t n_elems);

#ifdef __cplusplus
}
#endif
#endif /* COMET_RING_H */
