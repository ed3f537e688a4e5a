/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of what the GCN hot path computes, written
 * from the paper's definitions ("Reducing Communication in Graph Neural Network Training",
 * sections "Graph Neural Networks", "Forward Propagation", "Backpropagation Derivations").
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may use it.  It shares no
 * code with the GPU library and the GPU library never calls it.
 *
 * Dense matrices are row-major arrays of REAL (float in the parity build, double in the build
 * used for finite-difference checks).  Every sum is accumulated in double and rounded once
 * when stored.  Loops are parallel over output rows only; each output element is summed
 * sequentially in index order, so results do not depend on the thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifndef REAL
#define REAL float
#endif

int orc_real_bytes(void) { return (int)sizeof(REAL); }

int orc_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Number of threads of the loops below from now on (timing the oracle on one core); no effect on results:
 * every output element is computed by one thread in a fixed order. */
void orc_set_threads(int count) {
#ifdef _OPENMP
    if (count >= 1) omp_set_num_threads(count);
#else
    (void)count;
#endif
}

/* ------------------------------------------------------------------------------------------
 * Graph: section "Graph Neural Networks".  The adjacency matrix gets self-connections, and for
 * an undirected graph is scaled to D^-1/2 (A + I) D^-1/2 with D the diagonal of the degrees of
 * the modified matrix.  nnz(A) counts the self loops (section "Notation").
 * ---------------------------------------------------------------------------------------- */

static int cmp_u64(const void* a, const void* b) {
    uint64_t x = *(const uint64_t*)a, y = *(const uint64_t*)b;
    return (x > y) - (x < y);
}

/* The set E' = {(u,v)} u {(v,u) if symmetrise} over input pairs with u != v, plus (i,i) for all
 * i if self_loops.  Each member is encoded major<<32 | minor where (major, minor) = (row, col)
 * if by_col == 0 and (col, row) otherwise.  keys has room for 2m+n entries; on return its first
 * `count` entries are the distinct members in ascending order.  Returns count, or -1 if a
 * vertex id is outside [0, n). */
int64_t orc_edge_set(int64_t n, int64_t m, const int32_t* src, const int32_t* dst, int symmetrise,
                     int self_loops, int by_col, uint64_t* keys) {
    int64_t c = 0;
    for (int64_t e = 0; e < m; ++e) {
        int64_t u = src[e], v = dst[e];
        if (u < 0 || v < 0 || u >= n || v >= n) return -1;
        if (u == v) continue; /* input loops are dropped; exactly one is inserted below */
        uint64_t r = (uint64_t)u, q = (uint64_t)v;
        keys[c++] = by_col ? (q << 32 | r) : (r << 32 | q);
        if (symmetrise) keys[c++] = by_col ? (r << 32 | q) : (q << 32 | r);
    }
    if (self_loops)
        for (int64_t i = 0; i < n; ++i) keys[c++] = ((uint64_t)i << 32) | (uint64_t)i;
    qsort(keys, (size_t)c, sizeof(uint64_t), cmp_u64);
    int64_t w = 0;
    for (int64_t i = 0; i < c; ++i)
        if (i == 0 || keys[i] != keys[i - 1]) keys[w++] = keys[i];
    return w;
}

/* Compressed rows from sorted distinct keys: ptr[i] = number of keys with major < i. */
void orc_compress(int64_t n, int64_t count, const uint64_t* keys, int64_t* ptr, int32_t* minor) {
    for (int64_t i = 0; i <= n; ++i) ptr[i] = 0;
    for (int64_t k = 0; k < count; ++k) {
        ptr[(keys[k] >> 32) + 1] += 1;
        minor[k] = (int32_t)(keys[k] & 0xffffffffu);
    }
    for (int64_t i = 0; i < n; ++i) ptr[i + 1] += ptr[i];
}

/* Modified vertex degree = number of stored entries in the row (self loop included). */
void orc_degrees(int64_t n, const int64_t* rowptr, int32_t* deg) {
    for (int64_t i = 0; i < n; ++i) deg[i] = (int32_t)(rowptr[i + 1] - rowptr[i]);
}

/* Entry (i,j) of D^-1/2 (A+I) D^-1/2 = 1/sqrt(d_i d_j): one exact product of two integers below
 * 2^31 in double, one correctly rounded square root, one division, one rounding to float.  The
 * expression is symmetric in (i,j), so the same call values the transposed structure when given
 * the degrees of the untransposed matrix. */
void orc_values_sym(int64_t n, const int64_t* ptr, const int32_t* minor, const int32_t* deg, float* val) {
    for (int64_t i = 0; i < n; ++i)
        for (int64_t k = ptr[i]; k < ptr[i + 1]; ++k)
        {
            /* D^-1/2 is taken as the pseudo-inverse: a vertex whose row has no entry (possible only without
             * self-connections, for a vertex with no outgoing edge) scales by 0, not by 1/0. */
            const double dd = (double)deg[i] * (double)deg[minor[k]];
            val[k] = dd > 0.0 ? (float)(1.0 / sqrt(dd)) : 0.0f;
        }
}

/* Row normalisation D^-1 (A+I) for directed graphs: entry (i,j) = 1/d_i with d the degrees of the
 * untransposed matrix.  `transposed` says that ptr/minor describe the transposed structure, whose
 * entry in compressed row j with minor index i is the untransposed (i,j). */
void orc_values_row(int64_t n, const int64_t* ptr, const int32_t* minor, const int32_t* deg, int transposed,
                    float* val) {
    for (int64_t r = 0; r < n; ++r)
        for (int64_t k = ptr[r]; k < ptr[r + 1]; ++k)
            val[k] = (float)(1.0 / (double)deg[transposed ? minor[k] : r]);
}

/* ------------------------------------------------------------------------------------------
 * Sparse-dense product, the "SpMM" of sections "Graph Neural Networks" and "A One-Dimensional
 * (1D) Algorithm":  Z[i,:] = sum_k val[k] X[col[k],:]  over the stored entries k of row i.
 * ---------------------------------------------------------------------------------------- */
void orc_spmm(int64_t n, const int64_t* rowptr, const int32_t* colidx, const float* val, int32_t f,
              const REAL* X, int64_t ldx, REAL* Z, int64_t ldz) {
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t i = 0; i < n; ++i) {
        for (int32_t j = 0; j < f; ++j) {
            double acc = 0.0;
            for (int64_t k = rowptr[i]; k < rowptr[i + 1]; ++k)
                acc += (double)val[k] * (double)X[(int64_t)colidx[k] * ldx + j];
            Z[i * ldz + j] = (REAL)acc;
        }
    }
}

/* The same sum for the listed rows only; Zsel is nsel x f, row r holding Z[rows[r],:]. */
void orc_spmm_rows(int64_t nsel, const int64_t* rows, const int64_t* rowptr, const int32_t* colidx,
                   const float* val, int32_t f, const REAL* X, int64_t ldx, REAL* Zsel) {
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t r = 0; r < nsel; ++r) {
        int64_t i = rows[r];
        for (int32_t j = 0; j < f; ++j) {
            double acc = 0.0;
            for (int64_t k = rowptr[i]; k < rowptr[i + 1]; ++k)
                acc += (double)val[k] * (double)X[(int64_t)colidx[k] * ldx + j];
            Zsel[r * (int64_t)f + j] = (REAL)acc;
        }
    }
}

/* Value-free form of the same product for the symmetric normalisation of section "Graph Neural
 * Networks": with s_i = (float)(1/sqrt(d_i)),  D^-1/2 (A+I) D^-1/2 X = D^-1/2 ((A+I) (D^-1/2 X)).
 * The three steps are kept apart as the definition states them: scale the rows of X (stored in
 * REAL), sum the gathered rows without values, scale the output rows (scale may be NULL = 1). */
void orc_inv_sqrt_deg(int64_t n, const int32_t* deg, float* s) {
    for (int64_t i = 0; i < n; ++i) s[i] = deg[i] > 0 ? (float)(1.0 / sqrt((double)deg[i])) : 0.0f;
}

void orc_scale_rows(int64_t n, int32_t f, const REAL* X, int64_t ldx, const float* scale, REAL* Y, int64_t ldy) {
    for (int64_t i = 0; i < n; ++i)
        for (int32_t j = 0; j < f; ++j) Y[i * ldy + j] = (REAL)((double)scale[i] * (double)X[i * ldx + j]);
}

void orc_spmm_pattern(int64_t n, const int64_t* rowptr, const int32_t* colidx, const float* row_scale, int32_t f,
                      const REAL* X, int64_t ldx, REAL* Z, int64_t ldz) {
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t i = 0; i < n; ++i) {
        for (int32_t j = 0; j < f; ++j) {
            double acc = 0.0;
            for (int64_t k = rowptr[i]; k < rowptr[i + 1]; ++k) acc += (double)X[(int64_t)colidx[k] * ldx + j];
            Z[i * ldz + j] = (REAL)(row_scale ? (double)row_scale[i] * acc : acc);
        }
    }
}

/* ------------------------------------------------------------------------------------------
 * Dense product C = op(A) op(B), textbook triple loop.  op(A) is M x K, op(B) is K x N.
 * ta/tb nonzero means the stored matrix is the transpose (stored A is K x M, stored B is N x K).
 * ---------------------------------------------------------------------------------------- */
void orc_gemm(int ta, int tb, int64_t M, int64_t N, int64_t K, const REAL* A, int64_t lda,
              const REAL* B, int64_t ldb, REAL* C, int64_t ldc) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double a = ta ? (double)A[k * lda + i] : (double)A[i * lda + k];
                double b = tb ? (double)B[j * ldb + k] : (double)B[k * ldb + j];
                acc += a * b;
            }
            C[i * ldc + j] = (REAL)acc;
        }
    }
}

/* sigma = ReLU ("Forward Propagation"): y = max(x, 0). */
void orc_relu(int64_t count, const REAL* x, REAL* y) {
    for (int64_t i = 0; i < count; ++i) y[i] = x[i] > (REAL)0 ? x[i] : (REAL)0;
}

/* Hadamard product with sigma'(Z) of Equations 1 and 2; sigma'(z) = 1 if z > 0 else 0. */
void orc_relu_mask(int64_t count, const REAL* g, const REAL* z, REAL* out) {
    for (int64_t i = 0; i < count; ++i) out[i] = z[i] > (REAL)0 ? g[i] : (REAL)0;
}

/* Row-wise log-softmax (the non-elementwise activation of the last layer, section "Block
 * Two-Dimensional (2D) Algorithms", "Equation H = sigma(Z)") followed by the mean negative
 * log-likelihood over the labelled vertices (label >= 0; the paper trains Reddit on a training
 * split and the other graphs on all vertices).  Also Equation 1 for this loss:
 *   G[i,j] = (softmax(Z[i,:])[j] - [j == y_i]) / m   for labelled i,   0 for unlabelled i,
 * with m the number of labelled vertices.  G may be NULL.  Returns the loss in double. */
double orc_softmax_nll(int64_t n, int32_t C, const REAL* Z, int64_t ldz, const int32_t* labels, REAL* G,
                       int64_t ldg) {
    int64_t m_lab = 0;
    for (int64_t i = 0; i < n; ++i) m_lab += labels[i] >= 0;
    double loss = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        const REAL* z = Z + i * ldz;
        if (labels[i] < 0) {
            if (G)
                for (int32_t j = 0; j < C; ++j) G[i * ldg + j] = (REAL)0;
            continue;
        }
        double m = (double)z[0];
        for (int32_t j = 1; j < C; ++j)
            if ((double)z[j] > m) m = (double)z[j];
        double s = 0.0;
        for (int32_t j = 0; j < C; ++j) s += exp((double)z[j] - m);
        double lse = m + log(s);
        loss -= ((double)z[labels[i]] - lse);
        if (G)
            for (int32_t j = 0; j < C; ++j) {
                double p = exp((double)z[j] - lse);
                G[i * ldg + j] = (REAL)((p - (j == labels[i] ? 1.0 : 0.0)) / (double)m_lab);
            }
    }
    return m_lab ? loss / (double)m_lab : 0.0;
}

/* Gradient step of Equation 3: W <- W - lr * Y. */
void orc_sgd(int64_t count, REAL* W, const REAL* Y, double lr) {
    for (int64_t i = 0; i < count; ++i) W[i] = (REAL)((double)W[i] - lr * (double)Y[i]);
}
