/*
 * CPU oracle for the sparse secret-shared FFN matrix multiply over Z_{2^64}.
 *
 * TEST INFRASTRUCTURE ONLY.  Only the test-suite, the smoke check and the
 * benchmark's cpu_baseline leg may use this file.  It shares no code with the
 * HIP library and the HIP library never calls it.
 *
 * Everything is the plain definition written out: uint64_t arithmetic wraps
 * mod 2^64 by the C standard, matrices are dense row-major, products are
 * naive triple loops (the only liberty taken is the i-k-j loop nest and an
 * OpenMP pragma over output rows; neither changes a single result bit because
 * addition mod 2^64 is associative and commutative).
 *
 * Passages followed (paper section / equation / protocol):
 *   Sec. 2.1  additive sharing, reconstruction, Beaver multiplication (Eq. 1)
 *   Sec. 5.1  per-product masking E = X - a, F = Y - b, exchange, Eq. 1
 *   Protocol 2 (SOMM): IndexRows / IndexCols, then Pi_MatMul
 *   Protocol 3 (SIMM): IndexCol / IndexRows / IndexRow, then Pi_MatMul
 *   Appendix (optimality proof): cost model C1 = 2(|X|+|Y|), C2 = 3|X||Y|
 *
 * Parity pins live in tests/test_oracle_*.py; every function below is pinned
 * there against something other than itself (big-integer brute force, numpy's
 * integer matmul, the reconstruction identity, hand-worked Eq. 1 values,
 * float64 matmul for the fixed-point decode).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

typedef uint64_t u64;

/* ---- fixed point (ring Z_{2^64}, two's complement, frac_bits fractional bits) ---- */

/* encode(x) = round-half-away(x * 2^f) reduced mod 2^64 */
void co_encode(const double* x, u64* q, size_t n, int frac_bits) {
    const double scale = ldexp(1.0, frac_bits);
    for (size_t i = 0; i < n; ++i) q[i] = (u64)(int64_t)llround(x[i] * scale);
}

/* decode(v) = (signed interpretation of v) / 2^f */
void co_decode(const u64* q, double* x, size_t n, int frac_bits) {
    const double inv = ldexp(1.0, -frac_bits);
    for (size_t i = 0; i < n; ++i) x[i] = (double)(int64_t)q[i] * inv;
}

/* ---- Sec. 2.1: additive sharing ---- */

/* Sharing: [v]_0 = r (uniform randomness supplied by the caller), [v]_1 = v - r */
void co_share(const u64* v, const u64* r, u64* v0, u64* v1, size_t n) {
    for (size_t i = 0; i < n; ++i) { v0[i] = r[i]; v1[i] = v[i] - r[i]; }
}

/* Reconstruction: v = [v]_0 + [v]_1 */
void co_reconstruct(const u64* v0, const u64* v1, u64* v, size_t n) {
    for (size_t i = 0; i < n; ++i) v[i] = v0[i] + v1[i];
}

/* ---- plain ring product Z = X Y, X: m x k, Y: k x n ---- */
void co_ring_matmul(const u64* X, const u64* Y, u64* Z, int m, int k, int n) {
#pragma omp parallel for schedule(static)
    for (int i = 0; i < m; ++i) {
        u64* z = Z + (size_t)i * n;
        for (int j = 0; j < n; ++j) z[j] = 0;
        for (int l = 0; l < k; ++l) {
            const u64 x = X[(size_t)i * k + l];
            const u64* y = Y + (size_t)l * n;
            for (int j = 0; j < n; ++j) z[j] += x * y[j];
        }
    }
}

/* Same product, rows [r0, r1) of the output only (bounded samples for timing
 * and for spot checks at sizes where the full product takes minutes). */
void co_ring_matmul_rows(const u64* X, const u64* Y, u64* Z, int m, int k, int n, int r0, int r1) {
    (void)m;
#pragma omp parallel for schedule(static)
    for (int i = r0; i < r1; ++i) {
        u64* z = Z + (size_t)(i - r0) * n;
        for (int j = 0; j < n; ++j) z[j] = 0;
        for (int l = 0; l < k; ++l) {
            const u64 x = X[(size_t)i * k + l];
            const u64* y = Y + (size_t)l * n;
            for (int j = 0; j < n; ++j) z[j] += x * y[j];
        }
    }
}

/* ---- Sec. 5.1 / Eq. 1: local masking and opening ---- */

/* [D]_i = [X]_i - [A]_i  (elementwise; the value each party sends) */
void co_mask_share(const u64* x_i, const u64* a_i, u64* d_i, size_t n) {
    for (size_t i = 0; i < n; ++i) d_i[i] = x_i[i] - a_i[i];
}

/* E = [D]_0 + [D]_1  (what both parties hold after the exchange) */
void co_open(const u64* d0, const u64* d1, u64* e, size_t n) {
    for (size_t i = 0; i < n; ++i) e[i] = d0[i] + d1[i];
}

/* ---- plaintext sparsity distribution -> index list ---- */

/* OR the per-token block flags, then list active block ids in ascending order.
 * Returns the number of active blocks T; idx[0..T) is filled. */
int co_compact_mask(const uint8_t* mask, int n_tok, int nb, int32_t* idx) {
    int t = 0;
    for (int b = 0; b < nb; ++b) {
        int any = 0;
        for (int r = 0; r < n_tok; ++r) any |= (mask[(size_t)r * nb + b] != 0);
        if (any) idx[t++] = b;
    }
    return t;
}

/* IndexCols: out[r][c] = M[r][idx[c / bs] * bs + c % bs], out is rows x (T*bs) */
void co_index_cols(const u64* M, int rows, int cols, const int32_t* idx, int T, int bs, u64* out) {
    const int w = T * bs;
    for (int r = 0; r < rows; ++r)
        for (int c = 0; c < w; ++c)
            out[(size_t)r * w + c] = M[(size_t)r * cols + (size_t)idx[c / bs] * bs + c % bs];
}

/* IndexRows: out[r][c] = M[idx[r / bs] * bs + r % bs][c], out is (T*bs) x cols */
void co_index_rows(const u64* M, int rows, int cols, const int32_t* idx, int T, int bs, u64* out) {
    (void)rows;
    const int h = T * bs;
    for (int r = 0; r < h; ++r)
        memcpy(out + (size_t)r * cols, M + ((size_t)idx[r / bs] * bs + r % bs) * cols,
               (size_t)cols * sizeof(u64));
}

/* ---- Eq. 1 in matrix form: one party's output share ----
 * [Z]_i = [C]_i + E [B]_i + [A]_i F + (i-1) E F   with i in {1,2};
 * here party is 0-based, so party 1 is the paper's P_2 and adds E F.
 * E, A_i: m x k;  F, B_i: k x n;  C_i, Z_i: m x n.  Three separate products,
 * as the paper's cost model counts them.  tmp: scratch of m*n words. */
void co_beaver_share(int party, const u64* E, const u64* F, const u64* A_i, const u64* B_i,
                     const u64* C_i, u64* Z_i, u64* tmp, int m, int k, int n) {
    const size_t mn = (size_t)m * n;
    for (size_t t = 0; t < mn; ++t) Z_i[t] = C_i[t];
    co_ring_matmul(E, B_i, tmp, m, k, n);
    for (size_t t = 0; t < mn; ++t) Z_i[t] += tmp[t];
    co_ring_matmul(A_i, F, tmp, m, k, n);
    for (size_t t = 0; t < mn; ++t) Z_i[t] += tmp[t];
    if (party == 1) {
        co_ring_matmul(E, F, tmp, m, k, n);
        for (size_t t = 0; t < mn; ++t) Z_i[t] += tmp[t];
    }
}

/* Same share, output rows [r0, r1) only (Z_i, tmp: (r1-r0) x n; C_i full m x n). */
void co_beaver_share_rows(int party, const u64* E, const u64* F, const u64* A_i, const u64* B_i,
                          const u64* C_i, u64* Z_i, u64* tmp, int m, int k, int n, int r0, int r1) {
    const size_t cnt = (size_t)(r1 - r0) * n;
    for (size_t t = 0; t < cnt; ++t) Z_i[t] = C_i[(size_t)r0 * n + t];
    co_ring_matmul_rows(E, B_i, tmp, m, k, n, r0, r1);
    for (size_t t = 0; t < cnt; ++t) Z_i[t] += tmp[t];
    co_ring_matmul_rows(A_i, F, tmp, m, k, n, r0, r1);
    for (size_t t = 0; t < cnt; ++t) Z_i[t] += tmp[t];
    if (party == 1) {
        co_ring_matmul_rows(E, F, tmp, m, k, n, r0, r1);
        for (size_t t = 0; t < cnt; ++t) Z_i[t] += tmp[t];
    }
}

/* One output element of a party's share (spot checks at full benchmark size). */
u64 co_beaver_share_at(int party, const u64* E, const u64* F, const u64* A_i, const u64* B_i,
                       const u64* C_i, int m, int k, int n, int r, int c) {
    (void)m;
    u64 z = C_i[(size_t)r * n + c];
    for (int l = 0; l < k; ++l) z += E[(size_t)r * k + l] * B_i[(size_t)l * n + c];
    for (int l = 0; l < k; ++l) z += A_i[(size_t)r * k + l] * F[(size_t)l * n + c];
    if (party == 1)
        for (int l = 0; l < k; ++l) z += E[(size_t)r * k + l] * F[(size_t)l * n + c];
    return z;
}

/* ---- Protocol 2 (SOMM), all components in one pass ----
 * The components of the bipartite graph partition the participating rows of X
 * and columns of Y; rows and columns carry the number of their component
 * (row_comp[r], col_comp[c]; a negative number = takes part in none).  Output
 * element (r, c) belongs to the result block of a component exactly when both
 * numbers agree, and is then that component's Pi_MatMul share by Eq. 1 with
 * the component's own triple, stored in the same m x n layout (A_i row r is the
 * triple row of X row r, B_i column c that of Y column c, C_i(r, c) defined on
 * the blocks only).  Everything else is zero ("Merge" into an empty matrix).
 * E, A_i: m x k;  F, B_i: k x n;  C_i, Z_i: m x n. */
void co_beaver_share_blocks(int party, const u64* E, const u64* F, const u64* A_i, const u64* B_i,
                            const u64* C_i, const int32_t* row_comp, const int32_t* col_comp,
                            u64* Z_i, int m, int k, int n) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < m; ++r)
        for (int c = 0; c < n; ++c) {
            u64 z = 0;
            if (row_comp[r] >= 0 && row_comp[r] == col_comp[c]) {
                z = C_i[(size_t)r * n + c];
                for (int l = 0; l < k; ++l) z += E[(size_t)r * k + l] * B_i[(size_t)l * n + c];
                for (int l = 0; l < k; ++l) z += A_i[(size_t)r * k + l] * F[(size_t)l * n + c];
                if (party == 1)
                    for (int l = 0; l < k; ++l) z += E[(size_t)r * k + l] * F[(size_t)l * n + c];
            }
            Z_i[(size_t)r * n + c] = z;
        }
}

/* ---- Protocol 3 (SIMM), all columns in one pass ----
 * Column j of X contributes the outer product of its sub-vector on the row set
 * R_j = { r : S(r, j) != 0 } with row j of Y; Merge&Sum adds the result blocks
 * of a row.  With the column triples stored at their positions (A_i(r, j) for
 * r in R_j, B_i row j, and C_i = the sum over j of the scattered C shares) the
 * sum over the columns of Eq. 1 is
 *   Z_i(r, :) = C_i(r, :) + sum_{j : S(r,j) != 0} ( E(r,j) B_i(j,:) + A_i(r,j) F(j,:) + (i-1) E(r,j) F(j,:) ).
 * S: m x k bytes.  E, A_i: m x k (entries outside S never read);  F, B_i: k x n. */
void co_beaver_share_sparse_input(int party, const u64* E, const u64* F, const u64* A_i,
                                  const u64* B_i, const u64* C_i, const uint8_t* S, u64* Z_i,
                                  int m, int k, int n) {
#pragma omp parallel for schedule(static)
    for (int r = 0; r < m; ++r) {
        u64* z = Z_i + (size_t)r * n;
        for (int c = 0; c < n; ++c) z[c] = C_i[(size_t)r * n + c];
        for (int j = 0; j < k; ++j) {
            if (!S[(size_t)r * k + j]) continue;
            const u64 e = E[(size_t)r * k + j], a = A_i[(size_t)r * k + j];
            const u64* f = F + (size_t)j * n;
            const u64* b = B_i + (size_t)j * n;
            for (int c = 0; c < n; ++c) z[c] += e * b[c];
            for (int c = 0; c < n; ++c) z[c] += a * f[c];
            if (party == 1)
                for (int c = 0; c < n; ++c) z[c] += e * f[c];
        }
    }
}

/* ---- oblivious shuffle, the two local steps of the online stage (Protocol 1) ----
 * A permutation p acts on a vector as p(x) = [x_{p_1}, x_{p_2}, ...], i.e.
 * p(x)_j = x[p[j]] (0-based here).  On a matrix it acts along one axis:
 * axis 0 (columns): out(r, j) = in(r, p[j]);  axis 1 (rows): out(j, c) = in(p[j], c).
 * step 1:  y_i = tau_i(x_i) + a_i        (sign = +1)
 * step 2:  z_i = rho_i(y_other) - b_i    (sign = -1)
 * src, dst: rows x cols;  mask in the order of dst. */
void co_permute_mask(const u64* src, const int32_t* perm, const u64* mask, u64* dst, int rows,
                     int cols, int axis, int sign) {
    for (int r = 0; r < rows; ++r)
        for (int c = 0; c < cols; ++c) {
            const u64 v = axis == 0 ? src[(size_t)r * cols + perm[c]] : src[(size_t)perm[r] * cols + c];
            const u64 mk = mask[(size_t)r * cols + c];
            dst[(size_t)r * cols + c] = sign > 0 ? v + mk : v - mk;
        }
}

/* ---- Merge of Protocol 2 back to the full width ("reshaped to origin size") ----
 * full (m x n_full) := 0, then the kept column blocks of compact (m x n_blk*bs)
 * are written to their neurons: full(r, idx[t]*bs + j) = compact(r, t*bs + j). */
void co_scatter_cols(const u64* compact, const int32_t* idx, int n_blk, int bs, u64* full, int m,
                     int n_full) {
    const int ld = n_blk * bs;
    for (size_t i = 0; i < (size_t)m * n_full; ++i) full[i] = 0;
    for (int r = 0; r < m; ++r)
        for (int t = 0; t < n_blk; ++t)
            for (int j = 0; j < bs; ++j)
                full[(size_t)r * n_full + (size_t)idx[t] * bs + j] = compact[(size_t)r * ld + (size_t)t * bs + j];
}

/* ---- share-local rescaling after a fixed-point product ----
 * The product of two values with f fractional bits carries 2f; each party
 * divides its own share by 2^f without talking to the other:
 *   party 0:  z_0' =   floor( z_0 / 2^f )          (z_0 read as signed)
 *   party 1:  z_1' = - floor( (-z_1) / 2^f )
 * The reconstruction differs from the exact quotient by at most one unit in the
 * last place, except when the shares wrap (probability about |z| / 2^63 over
 * the sharing randomness).  The paper does not state its rescaling; this is the
 * usual two-party rule of the fixed-point framework it builds on. */
void co_truncate_share(int party, const u64* z, u64* out, size_t n, int f) {
    for (size_t i = 0; i < n; ++i) {
        if (party == 0) out[i] = (u64)((int64_t)z[i] >> f);
        else out[i] = (u64)0 - (u64)((int64_t)((u64)0 - z[i]) >> f);
    }
}
