/*
 * CPU oracle for the dynamic-GNN hot path.  TEST INFRASTRUCTURE ONLY: it exists to check the
 * GPU library and to be timed as a CPU baseline; the product never calls it.  It shares no
 * code, header, table or helper with the HIP sources.
 *
 * Everything here is the plain definition written out, in double precision for real numbers
 * and exact integers for structure:
 *   - snapshot reconstruction from a graph difference: Section "Graph-difference Based Input
 *     Transfer" (A^com = A_i minus the extra edges of A_i; A_{i+1} = A^com plus the extra
 *     edges of A_{i+1}), with each snapshot held as a set of (row, col) pairs;
 *   - normalised adjacency: Eqn (1), A~ = D^{-1/2} (A + I) D^{-1/2}, D[u,u] = 1 + deg_u;
 *   - GCN operation: Eqn (2), Y = sigma(A~ X W), evaluated as A~ (X W);
 *   - M-transform: Section "TM-GCN", Y = X x_1 M with the banded lower-triangular M printed
 *     there (M_tk = 1 / min(w, t) for max(1, t-w+1) <= k <= t, 1-based);
 *   - gradient propagation through those steps (Section "Gradient Checkpoint"): the adjoint of each
 *     step, A~^T G, X^T G, G W^T, G x_1 M^T, and the ReLU mask.
 *
 * Conventions: the stored matrix is A + I (every row holds its diagonal entry), rows are CSR
 * with ascending, duplicate-free columns, indices are 0-based int32.  With the diagonal stored,
 * 1 + deg_u is the row length.  Parity status: every function below is pinned by tests that
 * do not go through this file (dense brute force, numpy set algebra, closed forms).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef uint64_t key_t_;

static int cmp_key(const void *a, const void *b) {
    key_t_ x = *(const key_t_ *)a, y = *(const key_t_ *)b;
    return (x > y) - (x < y);
}

static key_t_ make_key(int32_t r, int32_t c) { return ((key_t_)(uint32_t)r << 32) | (uint32_t)c; }

/* sort and drop repeats; returns the number of distinct keys */
static int64_t sort_unique(key_t_ *k, int64_t m) {
    if (m == 0) return 0;
    int sorted = 1;
    for (int64_t i = 1; i < m; ++i) if (k[i - 1] >= k[i]) { sorted = 0; break; }
    if (!sorted) qsort(k, (size_t)m, sizeof(key_t_), cmp_key);
    int64_t o = 1;
    for (int64_t i = 1; i < m; ++i) if (k[i] != k[o - 1]) k[o++] = k[i];
    return o;
}

static int is_member(const key_t_ *sorted, int64_t m, key_t_ q) {
    int64_t lo = 0, hi = m;
    while (lo < hi) { int64_t mid = lo + (hi - lo) / 2; if (sorted[mid] < q) lo = mid + 1; else hi = mid; }
    return lo < m && sorted[lo] == q;
}

/* sorted distinct keys -> CSR.  Returns nnz, or -1 if cap is too small, -2 on a bad index. */
static int64_t keys_to_csr(int64_t n, const key_t_ *k, int64_t m, int32_t *rowptr, int32_t *colidx, int64_t cap) {
    if (m > cap) return -1;
    for (int64_t r = 0; r <= n; ++r) rowptr[r] = 0;
    for (int64_t i = 0; i < m; ++i) {
        int64_t r = (int64_t)(k[i] >> 32), c = (int64_t)(k[i] & 0xffffffffu);
        if (r >= n || c >= n) return -2;
        rowptr[r + 1] += 1;
        colidx[i] = (int32_t)c;
    }
    for (int64_t r = 0; r < n; ++r) rowptr[r + 1] += rowptr[r];
    return m;
}

/* Snapshot "from scratch": the edge set given as an arbitrary list of (row, col) pairs, in any
 * order, possibly with repeats -> canonical CSR.  (Standard sparse representation, Section
 * "Graph-difference Based Input Transfer", first snapshot of a block.) */
int64_t oracle_csr_from_edges(int64_t n, const int32_t *row, const int32_t *col, int64_t m,
                              int32_t *rowptr, int32_t *colidx, int64_t cap) {
    key_t_ *k = (key_t_ *)malloc(sizeof(key_t_) * (size_t)(m > 0 ? m : 1));
    if (!k) return -3;
    for (int64_t i = 0; i < m; ++i) k[i] = make_key(row[i], col[i]);
    int64_t u = sort_unique(k, m);
    int64_t rc = keys_to_csr(n, k, u, rowptr, colidx, cap);
    free(k);
    return rc;
}

/* Reconstruction of A_{i+1} from A_i and the graph difference, as set algebra on edge keys:
 *   common = E_i \ del ;  E_{i+1} = common U add.
 * Nothing is assumed of the difference lists beyond being lists of pairs (they are sorted and
 * de-duplicated here); edges of `del` that are absent and edges of `add` that are present are
 * harmless under set semantics.  Returns nnz of the result (or <0: -1 capacity, -2 index,
 * -3 memory). */
int64_t oracle_delta_apply(int64_t n, const int32_t *rowptr, const int32_t *colidx,
                           const int32_t *add_row, const int32_t *add_col, int64_t n_add,
                           const int32_t *del_row, const int32_t *del_col, int64_t n_del,
                           int32_t *rowptr_out, int32_t *colidx_out, int64_t cap) {
    int64_t nnz = rowptr[n];
    key_t_ *prev = (key_t_ *)malloc(sizeof(key_t_) * (size_t)(nnz + n_add + 1));
    key_t_ *add = (key_t_ *)malloc(sizeof(key_t_) * (size_t)(n_add + 1));
    key_t_ *del = (key_t_ *)malloc(sizeof(key_t_) * (size_t)(n_del + 1));
    if (!prev || !add || !del) { free(prev); free(add); free(del); return -3; }
    for (int64_t r = 0; r < n; ++r)
        for (int64_t e = rowptr[r]; e < rowptr[r + 1]; ++e) prev[e] = make_key((int32_t)r, colidx[e]);
    for (int64_t i = 0; i < n_add; ++i) add[i] = make_key(add_row[i], add_col[i]);
    for (int64_t i = 0; i < n_del; ++i) del[i] = make_key(del_row[i], del_col[i]);
    n_add = sort_unique(add, n_add);
    n_del = sort_unique(del, n_del);
    /* common edges: those of E_i not listed for deletion */
    int64_t m = 0;
    for (int64_t e = 0; e < nnz; ++e)
        if (!is_member(del, n_del, prev[e])) prev[m++] = prev[e];
    m = sort_unique(prev, m);           /* a no-op when the rows of A_i were already canonical */
    /* union with the added edges: textbook merge of two sorted duplicate-free lists */
    key_t_ *next = (key_t_ *)malloc(sizeof(key_t_) * (size_t)(m + n_add + 1));
    if (!next) { free(prev); free(add); free(del); return -3; }
    int64_t i = 0, j = 0, o = 0;
    while (i < m || j < n_add) {
        if (j >= n_add || (i < m && prev[i] < add[j])) next[o++] = prev[i++];
        else if (i >= m || add[j] < prev[i]) next[o++] = add[j++];
        else { next[o++] = prev[i]; ++i; ++j; }
    }
    free(prev);
    prev = next;
    m = o;
    int64_t rc = keys_to_csr(n, prev, m, rowptr_out, colidx_out, cap);
    free(prev); free(add); free(del);
    return rc;
}

/* ---- snapshots that carry a value per stored entry (Section "Graph-difference Based Input Transfer" ships
 * the values of the new snapshot next to the two index lists; Section "Smoothening the Input Graphs" is where
 * values other than 0/1 come from).  A snapshot is then a map (row, col) -> value, and a difference is
 *   deleted edges, added edges with their values, and surviving edges whose value changes. ---- */
typedef struct { key_t_ key; double val; } kv_t_;

static int cmp_kv(const void *a, const void *b) {
    key_t_ x = ((const kv_t_ *)a)->key, y = ((const kv_t_ *)b)->key;
    return (x > y) - (x < y);
}

static int64_t find_kv(const kv_t_ *sorted, int64_t m, key_t_ q) {
    int64_t lo = 0, hi = m;
    while (lo < hi) { int64_t mid = lo + (hi - lo) / 2; if (sorted[mid].key < q) lo = mid + 1; else hi = mid; }
    return (lo < m && sorted[lo].key == q) ? lo : -1;
}

/* next = (prev without the deleted edges, values replaced where the update list names the edge) plus the added
 * edges with their values.  An added edge that survives from prev takes the added value.  Returns nnz of the
 * result, or <0 as oracle_delta_apply. */
int64_t oracle_delta_apply_weighted(int64_t n, const int32_t *rowptr, const int32_t *colidx, const double *val,
                                    const int32_t *add_row, const int32_t *add_col, const double *add_val, int64_t n_add,
                                    const int32_t *del_row, const int32_t *del_col, int64_t n_del,
                                    const int32_t *upd_row, const int32_t *upd_col, const double *upd_val, int64_t n_upd,
                                    int32_t *rowptr_out, int32_t *colidx_out, double *val_out, int64_t cap) {
    int64_t nnz = rowptr[n];
    kv_t_ *all = (kv_t_ *)malloc(sizeof(kv_t_) * (size_t)(nnz + n_add + 1));
    kv_t_ *add = (kv_t_ *)malloc(sizeof(kv_t_) * (size_t)(n_add + 1));
    kv_t_ *upd = (kv_t_ *)malloc(sizeof(kv_t_) * (size_t)(n_upd + 1));
    key_t_ *del = (key_t_ *)malloc(sizeof(key_t_) * (size_t)(n_del + 1));
    if (!all || !add || !upd || !del) { free(all); free(add); free(upd); free(del); return -3; }
    for (int64_t i = 0; i < n_add; ++i) { add[i].key = make_key(add_row[i], add_col[i]); add[i].val = add_val[i]; }
    for (int64_t i = 0; i < n_upd; ++i) { upd[i].key = make_key(upd_row[i], upd_col[i]); upd[i].val = upd_val[i]; }
    for (int64_t i = 0; i < n_del; ++i) del[i] = make_key(del_row[i], del_col[i]);
    qsort(add, (size_t)n_add, sizeof(kv_t_), cmp_kv);
    qsort(upd, (size_t)n_upd, sizeof(kv_t_), cmp_kv);
    n_del = sort_unique(del, n_del);
    int64_t m = 0;
    for (int64_t r = 0; r < n; ++r)
        for (int64_t e = rowptr[r]; e < rowptr[r + 1]; ++e) {
            key_t_ k = make_key((int32_t)r, colidx[e]);
            if (is_member(del, n_del, k)) continue;
            if (find_kv(add, n_add, k) >= 0) continue;          /* comes back below with the added value */
            int64_t u = find_kv(upd, n_upd, k);
            all[m].key = k;
            all[m].val = u >= 0 ? upd[u].val : val[e];
            ++m;
        }
    for (int64_t i = 0; i < n_add; ++i)
        if (i == 0 || add[i].key != add[i - 1].key) all[m++] = add[i];
    qsort(all, (size_t)m, sizeof(kv_t_), cmp_kv);
    int64_t rc = m <= cap ? m : -1;
    if (rc >= 0) {
        for (int64_t r = 0; r <= n; ++r) rowptr_out[r] = 0;
        for (int64_t i = 0; i < m; ++i) {
            int64_t r = (int64_t)(all[i].key >> 32), c = (int64_t)(all[i].key & 0xffffffffu);
            if (r < 0 || r >= n || c < 0 || c >= n) { rc = -2; break; }
            rowptr_out[r + 1]++;
            colidx_out[i] = (int32_t)c;
            val_out[i] = all[i].val;
        }
        if (rc >= 0) for (int64_t r = 0; r < n; ++r) rowptr_out[r + 1] += rowptr_out[r];
    }
    free(all); free(add); free(upd); free(del);
    return rc;
}

/* Eqn (1): explicit value of every stored entry of A~: 1 / sqrt((1+deg_u) (1+deg_v)), where the
 * stored matrix is A + I so that 1 + deg_u is the length of row u. */
void oracle_gcn_values(int64_t n, const int32_t *rowptr, const int32_t *colidx, double *val) {
    for (int64_t u = 0; u < n; ++u) {
        double du = (double)(rowptr[u + 1] - rowptr[u]);
        for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e) {
            int64_t v = colidx[e];
            double dv = (double)(rowptr[v + 1] - rowptr[v]);
            val[e] = 1.0 / sqrt(du * dv);
        }
    }
}

/* H = X W, X is n x f_in, W is f_in x f_out, all row-major (Eqn (2), dense factor). */
void oracle_xw(int64_t n, int64_t f_in, int64_t f_out, const double *x, const double *w, double *h) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < f_out; ++j) {
            double s = 0.0;
            for (int64_t k = 0; k < f_in; ++k) s += x[i * f_in + k] * w[k * f_out + j];
            h[i * f_out + j] = s;
        }
}

/* Z = sigma?(A~ H) (Eqn (2), sparse factor).  If rows != NULL only those rows are computed and
 * written compactly: z[i] is row rows[i]. */
void oracle_spmm(int64_t n, const int32_t *rowptr, const int32_t *colidx, const double *val,
                 const double *h, int64_t f, int relu, const int64_t *rows, int64_t n_rows, double *z) {
    int64_t cnt = rows ? n_rows : n;
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t i = 0; i < cnt; ++i) {
        int64_t u = rows ? rows[i] : i;
        double *zu = z + i * f;
        for (int64_t j = 0; j < f; ++j) zu[j] = 0.0;
        for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e) {
            const double *hv = h + (int64_t)colidx[e] * f;
            for (int64_t j = 0; j < f; ++j) zu[j] += val[e] * hv[j];
        }
        if (relu) for (int64_t j = 0; j < f; ++j) if (zu[j] < 0.0) zu[j] = 0.0;
    }
}

/* The T x T matrix M of the M-transform (1-based t, k in the paper; 0-based storage here). */
void oracle_m_matrix(int64_t T, int64_t w, double *M) {
    for (int64_t t = 1; t <= T; ++t)
        for (int64_t k = 1; k <= T; ++k) {
            int64_t lo = t - w + 1 > 1 ? t - w + 1 : 1;
            double mn = (double)(w < t ? w : t);
            M[(t - 1) * T + (k - 1)] = (k >= lo && k <= t) ? 1.0 / mn : 0.0;
        }
}

/* Mode-1 tensor-times-matrix: Y_t = sum_k M[t][k] Z_k over all k; each frame has `frame` numbers. */
void oracle_mproduct(int64_t T, int64_t frame, const double *M, const double *z, double *y) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < frame; ++i)
        for (int64_t t = 0; t < T; ++t) {
            double s = 0.0;
            for (int64_t k = 0; k < T; ++k) s += M[t * T + k] * z[k * frame + i];
            y[t * frame + i] = s;
        }
}

/* ---- backward of the same path (Section "Gradient Checkpoint": after a block has been run forward
 * again, gradients are propagated through it in the reverse direction).  Each function is the adjoint of
 * one forward step above, written out from the definition of that step. ---- */

/* Adjoint of the aggregation of Eqn (2): out = A~^T G, i.e. every stored entry (u, v) of A + I sends
 * val(u, v) * G[u] to out[v].  Entries are visited in storage order, one thread per feature column. */
void oracle_spmm_t(int64_t n, const int32_t *rowptr, const int32_t *colidx, const double *val,
                   const double *g, int64_t f, double *out) {
    for (int64_t i = 0; i < n * f; ++i) out[i] = 0.0;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < f; ++j)
        for (int64_t u = 0; u < n; ++u)
            for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e)
                out[(int64_t)colidx[e] * f + j] += val[e] * g[u * f + j];
}

/* Gradient of the weight of H = X W (dense factor of Eqn (2)) for an upstream G = dL/dH: dW = X^T G. */
void oracle_weight_grad(int64_t n, int64_t f_in, int64_t f_out, const double *x, const double *g, double *dw) {
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < f_in; ++k)
        for (int64_t j = 0; j < f_out; ++j) {
            double s = 0.0;
            for (int64_t i = 0; i < n; ++i) s += x[i * f_in + k] * g[i * f_out + j];
            dw[k * f_out + j] = s;
        }
}

/* Adjoint of the M-transform (Section "TM-GCN"): out_k = sum_t M[t][k] G_t. */
void oracle_mproduct_t(int64_t T, int64_t frame, const double *M, const double *g, double *out) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < frame; ++i)
        for (int64_t k = 0; k < T; ++k) {
            double s = 0.0;
            for (int64_t t = 0; t < T; ++t) s += M[t * T + k] * g[t * frame + i];
            out[k * frame + i] = s;
        }
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int t) {
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}
