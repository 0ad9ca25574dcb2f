/*
 * CPU oracle for the per-GPU GCN hot path -- TEST INFRASTRUCTURE, not part of the product.
 *
 * Plain, slow, fp64 implementations of what the path computes, written from the paper's
 * definitions (Sec. 2.1, Eq. 2.1-2.7; Sec. 5.1, Eq. 5.1-5.4).  Only tests, the smoke check
 * and the benchmark's cpu_baseline leg may call this file.  It shares no code with the HIP
 * library and includes none of its headers.
 *
 * Conventions: all indices int64, all reals double, matrices row-major with an explicit
 * leading dimension.  Sparse matrices are coordinate lists (row[e], col[e], val[e]).
 * Loops are parallelised over DESTINATION rows only (each output element is written by
 * one thread, accumulation order inside an element is the serial order), so results do not
 * depend on the thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_API __attribute__((visibility("default")))

ORC_API int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

ORC_API void orc_set_num_threads(int t) {
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

static int cmp_u64(const void* a, const void* b) {
    uint64_t x = *(const uint64_t*)a, y = *(const uint64_t*)b;
    return (x > y) - (x < y);
}

/*
 * Sec. 2.1, adjacency preprocessing.  From an arbitrary edge list (either direction, may
 * hold duplicates and self-loops) form the set S = {(u,v),(v,u) : u != v}, then A~ = 1[S] + I
 * (exactly one self-loop per node), d_u = row sum of A~ (so d_u >= 1), and
 * A^_uv = A~_uv / sqrt(d_u d_v).
 *
 * Outputs (caller allocates 2*n_edges + n entries): row/col/val sorted by (row, col) in
 * ORIGINAL node ids; deg[n].  Returns nnz, or -1 on an out-of-range node id / bad size.
 */
ORC_API int64_t orc_adj_build(int64_t n, int64_t n_edges, const int64_t* src, const int64_t* dst,
                              int64_t* row, int64_t* col, double* val, int64_t* deg) {
    if (n < 0 || n_edges < 0) return -1;
    int64_t cap = 2 * n_edges + n;
    uint64_t* key = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)(cap > 0 ? cap : 1));
    if (!key) return -1;
    int64_t c = 0;
    for (int64_t e = 0; e < n_edges; ++e) {
        int64_t u = src[e], v = dst[e];
        if (u < 0 || v < 0 || u >= n || v >= n) { free(key); return -1; }
        if (u == v) continue;                          /* input loops dropped, I added below */
        key[c++] = (uint64_t)u * (uint64_t)n + (uint64_t)v;
        key[c++] = (uint64_t)v * (uint64_t)n + (uint64_t)u;
    }
    for (int64_t u = 0; u < n; ++u) key[c++] = (uint64_t)u * (uint64_t)n + (uint64_t)u;
    qsort(key, (size_t)c, sizeof(uint64_t), cmp_u64);
    int64_t nnz = 0;
    for (int64_t u = 0; u < n; ++u) deg[u] = 0;
    for (int64_t i = 0; i < c; ++i) {
        if (i > 0 && key[i] == key[i - 1]) continue;   /* duplicate */
        int64_t u = (int64_t)(key[i] / (uint64_t)n), v = (int64_t)(key[i] % (uint64_t)n);
        row[nnz] = u; col[nnz] = v; deg[u] += 1; ++nnz;
    }
    for (int64_t e = 0; e < nnz; ++e)
        val[e] = 1.0 / sqrt((double)deg[row[e]] * (double)deg[col[e]]);
    free(key);
    return nnz;
}

typedef struct { int64_t r, c; int64_t src; } perm_entry;
static int cmp_entry(const void* a, const void* b) {
    const perm_entry* x = (const perm_entry*)a; const perm_entry* y = (const perm_entry*)b;
    if (x->r != y->r) return (x->r > y->r) - (x->r < y->r);
    return (x->c > y->c) - (x->c < y->c);
}

/*
 * Sec. 5.1, Eq. 5.3: the stored matrix P_r A^ P_c^T as canonical CSR.  perm[old] = new
 * (NULL = identity).  Entry (u,v) moves to (perm_r[u], perm_c[v]); rows ascending, columns
 * strictly ascending inside a row.  The fp32 value is the fp64 value 1/sqrt(d_u d_v) rounded
 * once to nearest-even.  Returns 0, or -1 if a permutation is not a bijection on [0,n).
 */
ORC_API int orc_permuted_csr(int64_t n, int64_t nnz, const int64_t* row, const int64_t* col,
                             const int64_t* deg, const int64_t* perm_r, const int64_t* perm_c,
                             int64_t* rowptr, int32_t* out_col, float* out_val) {
    for (int pass = 0; pass < 2; ++pass) {
        const int64_t* p = pass ? perm_c : perm_r;
        if (!p) continue;
        char* seen = (char*)calloc((size_t)(n > 0 ? n : 1), 1);
        for (int64_t i = 0; i < n; ++i) {
            if (p[i] < 0 || p[i] >= n || seen[p[i]]) { free(seen); return -1; }
            seen[p[i]] = 1;
        }
        free(seen);
    }
    perm_entry* ent = (perm_entry*)malloc(sizeof(perm_entry) * (size_t)(nnz > 0 ? nnz : 1));
    for (int64_t e = 0; e < nnz; ++e) {
        ent[e].r = perm_r ? perm_r[row[e]] : row[e];
        ent[e].c = perm_c ? perm_c[col[e]] : col[e];
        ent[e].src = e;
    }
    qsort(ent, (size_t)nnz, sizeof(perm_entry), cmp_entry);
    for (int64_t i = 0; i <= n; ++i) rowptr[i] = 0;
    for (int64_t e = 0; e < nnz; ++e) {
        int64_t s = ent[e].src;
        rowptr[ent[e].r + 1] += 1;
        out_col[e] = (int32_t)ent[e].c;
        out_val[e] = (float)(1.0 / sqrt((double)deg[row[s]] * (double)deg[col[s]]));
    }
    for (int64_t i = 0; i < n; ++i) rowptr[i + 1] += rowptr[i];
    free(ent);
    return 0;
}

/* lower bound of `x` in the ascending array a[0..len) */
static int64_t lower_bound_i64(const int64_t* a, int64_t len, int64_t x) {
    int64_t lo = 0, hi = len;
    while (lo < hi) { int64_t mid = lo + (hi - lo) / 2; if (a[mid] < x) lo = mid + 1; else hi = mid; }
    return lo;
}

/*
 * Eq. 2.1, aggregation: Y[m x d] = A X, A given as a coordinate list whose `row` array is
 * ascending (entries of one row contiguous).  Y[row[e], :] += val[e] * X[col[e], :].
 */
ORC_API void orc_spmm_coo(int64_t m, int64_t nnz, const int64_t* row, const int64_t* col, const double* val,
                          const double* X, int64_t ldx, double* Y, int64_t ldy, int64_t d) {
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t i = 0; i < m; ++i) {
        double* y = Y + i * ldy;
        for (int64_t j = 0; j < d; ++j) y[j] = 0.0;
        int64_t e0 = lower_bound_i64(row, nnz, i), e1 = lower_bound_i64(row, nnz, i + 1);
        for (int64_t e = e0; e < e1; ++e) {
            const double* x = X + col[e] * ldx;
            double a = val[e];
            for (int64_t j = 0; j < d; ++j) y[j] += a * x[j];
        }
    }
}

/*
 * Eq. 2.7, transposed aggregation: Y[k x d] = A^T X for the same coordinate list (any
 * order).  Y[col[e], :] += val[e] * X[row[e], :].  Each thread owns a contiguous range of
 * destination rows and scans the whole list for entries that land in it.
 */
ORC_API void orc_spmm_t_coo(int64_t k, int64_t nnz, const int64_t* row, const int64_t* col, const double* val,
                            const double* X, int64_t ldx, double* Y, int64_t ldy, int64_t d) {
#pragma omp parallel
    {
        int t = 0, nt = 1;
#ifdef _OPENMP
        t = omp_get_thread_num(); nt = omp_get_num_threads();
#endif
        int64_t c0 = k * t / nt, c1 = k * (t + 1) / nt;
        for (int64_t i = c0; i < c1; ++i)
            for (int64_t j = 0; j < d; ++j) Y[i * ldy + j] = 0.0;
        for (int64_t e = 0; e < nnz; ++e) {
            int64_t c = col[e];
            if (c < c0 || c >= c1) continue;
            const double* x = X + row[e] * ldx;
            double* y = Y + c * ldy;
            double a = val[e];
            for (int64_t j = 0; j < d; ++j) y[j] += a * x[j];
        }
    }
}

/*
 * Sampled rows of Y = A X (or Y = A^T X) for a block given as CSR with fp32 values and an
 * fp32 dense operand -- the definition of single output rows, used where the full product
 * is too large for the host.  out[s, :] = row sample[s] of the product.
 */
ORC_API void orc_spmm_rows_csr(const int64_t* rowptr, const int32_t* col, const float* val,
                               const float* X, int64_t ldx, int64_t d,
                               const int64_t* sample, int64_t ns, double* out) {
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t s = 0; s < ns; ++s) {
        double* y = out + s * d;
        for (int64_t j = 0; j < d; ++j) y[j] = 0.0;
        int64_t i = sample[s];
        for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            const float* x = X + (int64_t)col[e] * ldx;
            double a = (double)val[e];
            for (int64_t j = 0; j < d; ++j) y[j] += a * (double)x[j];
        }
    }
}

/* X is fp64 here (it may itself be an fp64 oracle result); values stay the stored fp32 */
ORC_API void orc_spmm_t_rows_csr(int64_t m, int64_t k, const int64_t* rowptr, const int32_t* col, const float* val,
                                 const double* X, int64_t ldx, int64_t d,
                                 const int64_t* sample, int64_t ns, double* out) {
    int64_t* slot = (int64_t*)malloc(sizeof(int64_t) * (size_t)(k > 0 ? k : 1));
    for (int64_t c = 0; c < k; ++c) slot[c] = -1;
    for (int64_t s = 0; s < ns; ++s) slot[sample[s]] = s;   /* a repeated sample keeps the last slot */
    for (int64_t s = 0; s < ns * d; ++s) out[s] = 0.0;
    for (int64_t i = 0; i < m; ++i)
        for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            int64_t s = slot[col[e]];
            if (s < 0) continue;
            const double* x = X + i * ldx;
            double a = (double)val[e];
            for (int64_t j = 0; j < d; ++j) out[s * d + j] += a * x[j];
        }
    /* repeated samples: copy from the slot that accumulated */
    for (int64_t s = 0; s < ns; ++s) {
        int64_t t = slot[sample[s]];
        if (t != s) memcpy(out + s * d, out + t * d, sizeof(double) * (size_t)d);
    }
    free(slot);
}

/*
 * Eq. 2.2 / 2.5 / 2.6, dense products: C[M x N] = op(A) op(B), op = transpose when the flag
 * is set.  Textbook triple loop, fp64.
 */
ORC_API void orc_gemm(int ta, int tb, int64_t M, int64_t N, int64_t K,
                      const double* A, int64_t lda, const double* B, int64_t ldb, double* C, int64_t ldc) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int64_t p = 0; p < K; ++p) {
                double a = ta ? A[p * lda + i] : A[i * lda + p];
                double b = tb ? B[j * ldb + p] : B[p * ldb + j];
                acc += a * b;
            }
            C[i * ldc + j] = acc;
        }
}

/* Eq. 2.3 with sigma = ReLU */
ORC_API void orc_relu(int64_t count, const double* z, double* f) {
    for (int64_t i = 0; i < count; ++i) f[i] = z[i] > 0.0 ? z[i] : 0.0;
}

/* Eq. 2.4 with sigma = ReLU: dZ = dF * [Z > 0] (derivative at 0 taken as 0) */
ORC_API void orc_relu_bwd(int64_t count, const double* z, const double* df, double* dz) {
    for (int64_t i = 0; i < count; ++i) dz[i] = z[i] > 0.0 ? df[i] : 0.0;
}

/*
 * Node classification loss (Sec. 2.1): mean over all n nodes of the softmax cross-entropy of
 * row i of the logits against label y[i].  Returns the loss; dZ = (softmax - onehot) / n.
 */
ORC_API double orc_softmax_ce(int64_t n, int64_t c, const double* Z, int64_t ldz, const int64_t* y,
                              double* dZ, int64_t lddz) {
    double loss = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        const double* z = Z + i * ldz;
        double mx = z[0];
        for (int64_t j = 1; j < c; ++j) if (z[j] > mx) mx = z[j];
        double sum = 0.0;
        for (int64_t j = 0; j < c; ++j) sum += exp(z[j] - mx);
        loss += -(z[y[i]] - mx - log(sum));
        if (dZ)
            for (int64_t j = 0; j < c; ++j)
                dZ[i * lddz + j] = (exp(z[j] - mx) / sum - (j == y[i] ? 1.0 : 0.0)) / (double)n;
    }
    return n > 0 ? loss / (double)n : 0.0;
}
