/*
 * dgnn.h -- C boundary of the MI355X (gfx950) dynamic-GNN hot path.
 *
 * The path, for one GPU's block of timesteps of a discrete-time dynamic graph G_1..G_T over N
 * vertices (Section "Discrete Time Dynamic Graphs"):
 *
 *   A_1 arrives whole; for t > 1 only the graph difference arrives and A_t is rebuilt on the
 *   GPU from A_{t-1}                                   dgnn_delta_h2d, dgnn_delta_rebuild
 *   H_t = X_t W                                        dgnn_feature_transform
 *   Z_t = sigma(A~_t H_t)                              dgnn_spmm
 *   Y   = Z x_1 M  (TM-GCN's temporal mixing)          dgnn_mproduct
 *
 * Conventions shared by every call
 *   - A snapshot is stored as CSR of A_t + I: int32 rowptr[n+1], int32 colidx[nnz], columns
 *     strictly ascending inside a row, the diagonal entry present in every row.  With the
 *     diagonal stored, the 1 + deg_u of Eqn (1) is the length of row u, and
 *     dinv[u] = (1 + deg_u)^(-1/2) is all that is needed for the values of A~ (the snapshots
 *     are unweighted, so no value array exists).
 *   - Dense matrices are row-major with leading dimension equal to the feature width; tensors
 *     over time are [T][n][f] contiguous.  Feature widths must be one of 16, 32, 64, 128.
 *   - Unless a parameter is marked HOST, every pointer is a DEVICE pointer, 16-byte aligned for
 *     feature matrices, owned by the caller, and must stay valid until the work enqueued on
 *     `stream` has run.  `stream` is a hipStream_t passed as void* (NULL = the default
 *     stream).  Calls only enqueue work and return; nothing is allocated, nothing is kept
 *     between calls, nothing is printed.
 *   - Return value: DGNN_OK (0) or a negative dgnn_status.  Argument errors are detected on
 *     the host before anything is enqueued.
 *   - All indices and counts that live in device arrays are int32; n and nnz (and the lengths of the
 *     difference lists) must not exceed 2^31 - 2^16 - 1, else DGNN_ERR_OVERFLOW.
 */
#ifndef DGNN_H
#define DGNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DGNN_OK = 0,
    DGNN_ERR_NULL = -1,      /* a required pointer is NULL                                   */
    DGNN_ERR_SHAPE = -2,     /* non-positive size, unsupported feature width / window / dtype */
    DGNN_ERR_CAPACITY = -3,  /* output buffer or workspace too small                          */
    DGNN_ERR_OVERFLOW = -4,  /* n or nnz beyond the int32 index range (see below)             */
    DGNN_ERR_ALIAS = -5,     /* output aliases an input where that is not allowed             */
    DGNN_ERR_HIP = -6,       /* the HIP runtime refused a launch or copy                      */
    DGNN_ERR_ALIGN = -7      /* a feature pointer is not 16-byte aligned                      */
} dgnn_status;

/* Storage type of feature matrices; accumulation is always fp32.  bf16 stores round to nearest even. */
typedef enum { DGNN_F32 = 0, DGNN_BF16 = 1 } dgnn_dtype;

/* Flags of dgnn_delta_rebuild and dgnn_delta_rebuild_weighted. */
#define DGNN_VALIDATE 1u         /* check the difference lists against A_prev on the device */
#define DGNN_UPDATES_SORTED 2u   /* weighted only: the value-update list is sorted by (row, col) without repeats */

/* Codes written to *d_status by dgnn_delta_rebuild (0 = nothing found; the smallest code found wins). */
#define DGNN_BAD_INDEX_RANGE 1   /* a row or column index outside [0, n)                         */
#define DGNN_BAD_DELTA_ORDER 2   /* a list is not strictly ascending by (row, col)               */
#define DGNN_BAD_DIAGONAL 3      /* a list names a diagonal entry                                */
#define DGNN_BAD_DEL_ABSENT 4    /* a deleted edge is not in A_prev                              */
#define DGNN_BAD_ADD_PRESENT 5   /* an added edge is already in A_prev                           */
#define DGNN_BAD_EMPTY_ROW 6     /* A_prev has a row without entries (the diagonal is missing)   */
/* ... and by dgnn_csr_validate: */
#define DGNN_BAD_ROWPTR 7        /* rowptr[0] != 0, rowptr not ascending, or rowptr[n] != nnz     */
#define DGNN_BAD_ROW_ORDER 8     /* the columns of a row are not strictly ascending              */
#define DGNN_BAD_NO_DIAGONAL 9   /* a row does not hold its diagonal entry (only if asked for)   */
/* ... and by dgnn_csr_combine (the largest code found wins): */
#define DGNN_BAD_CAPACITY 10     /* the result has more stored entries than colidx_c / val_c hold */

/* Flags of dgnn_spmm. */
#define DGNN_RELU 1u             /* apply sigma = ReLU to the aggregated rows (Eqn (2)) */
#define DGNN_H_PRESCALED 2u      /* h already holds dinv[v] * H[v] (see dgnn_feature_transform) */

/* Text for a dgnn_status value; never NULL; static storage. */
const char *dgnn_strerror(int code);

/*
 * dinv[u] = (rowptr[u+1] - rowptr[u])^(-1/2), u in [0, n): the diagonal of D^(-1/2) in Eqn (1)
 * for a snapshot that did not come out of dgnn_delta_rebuild (the first one of a block).
 */
int dgnn_csr_dinv(int64_t n, const int32_t *rowptr, float *dinv, void *stream);

/*
 * Graph-difference transfer (Section "Graph-difference Based Input Transfer"): instead of the
 * whole snapshot, only the indices of the edges that disappear and of the edges that appear
 * are shipped from the host.  Copies the four index lists from PINNED HOST memory (h_*) to
 * device staging buffers (d_*), n_add resp. n_del int32 each, asynchronously on `stream`.
 * Zero-length lists are allowed (their pointers may then be NULL).
 * Bytes moved: 8 * (n_add + n_del), against 4 * (nnz + n + 1) for a whole CSR snapshot.
 */
int dgnn_delta_h2d(const int32_t *h_add_row, const int32_t *h_add_col, int64_t n_add,
                   const int32_t *h_del_row, const int32_t *h_del_col, int64_t n_del,
                   int32_t *d_add_row, int32_t *d_add_col, int32_t *d_del_row, int32_t *d_del_col,
                   void *stream);

/* Workspace size of dgnn_delta_rebuild and dgnn_delta_rebuild_weighted in bytes (HOST out-parameter): 40 per range of
 * 8192 stored entries (never fewer than 16386 ranges), rounded up; it grows with nnz_prev only, so the size queried
 * for the largest snapshot of a block serves every step. */
int dgnn_delta_rebuild_workspace(int64_t n, int64_t nnz_prev, int64_t n_add, int64_t n_del, size_t *bytes);

/*
 * On-GPU reconstruction of a snapshot (same section): with A_prev on the device,
 *     common = A_prev minus the deleted edges,   A_next = common plus the added edges,
 * both as CSR of A + I in the canonical form above.  Also emits dinv_next (may be NULL).
 *
 *   n                       vertices
 *   rowptr_prev, colidx_prev, nnz_prev    A_{t-1}; nnz_prev == rowptr_prev[n] (known to the host)
 *   add_row/add_col, n_add  edges of A_t not in A_{t-1}, sorted by (row, col), no repeats
 *   del_row/del_col, n_del  edges of A_{t-1} not in A_t, sorted by (row, col), no repeats
 *                           (the two lists are disjoint from each other by construction and
 *                           never name the diagonal)
 *   rowptr_next [n+1], colidx_next [cap_next]   output; cap_next >= nnz_prev + n_add - n_del
 *   nnz_next                HOST out-parameter (may be NULL): nnz_prev + n_add - n_del
 *   ws, ws_bytes            scratch of at least dgnn_delta_rebuild_workspace() bytes
 *   flags                   0 or DGNN_VALIDATE
 *   d_status                device int32 (may be NULL).  Always reset to 0 by the call; under
 *                           DGNN_VALIDATE receives the smallest DGNN_BAD_* code found.
 *
 * Lists that break the preconditions give an unspecified A_next (never an out-of-bounds
 * access); use DGNN_VALIDATE to find out.  Outputs must not overlap inputs (DGNN_ERR_ALIAS
 * when the base pointers coincide).  The result is bit-for-bit unique.
 */
int dgnn_delta_rebuild(int64_t n,
                       const int32_t *rowptr_prev, const int32_t *colidx_prev, int64_t nnz_prev,
                       const int32_t *add_row, const int32_t *add_col, int64_t n_add,
                       const int32_t *del_row, const int32_t *del_col, int64_t n_del,
                       int32_t *rowptr_next, int32_t *colidx_next, int64_t cap_next, int64_t *nnz_next,
                       float *dinv_next,
                       void *ws, size_t ws_bytes, uint32_t flags, int32_t *d_status, void *stream);

/*
 * Dense factor of the GCN operation, Eqn (2): H = X W, or H = diag(row_scale) X W.
 *   x [n][f_in], w [f_in][f_out], h [n][f_out], all of storage type dt, fp32 accumulation on
 *   the matrix cores.  W is a per-call argument, so a model that keeps one weight per
 *   timestep (Section "EvolveGCN") passes W_t.  h must not alias x.
 *   row_scale [n] fp32, or NULL.  Passing the snapshot's dinv folds the right-hand D^(-1/2) of
 *   Eqn (1) into the rows of H while they are still in registers, so that the aggregation
 *   (dgnn_spmm with DGNN_H_PRESCALED) gathers rows of H only and no per-neighbour dinv.
 */
int dgnn_feature_transform(const void *x, int64_t n, int32_t f_in, const void *w, int32_t f_out,
                           const float *row_scale, void *h, dgnn_dtype dt, void *stream);

/* Workspace size of dgnn_spmm in bytes (HOST out-parameter); depends on n, nnz and f only. */
int dgnn_spmm_workspace(int64_t n, int64_t nnz, int32_t f, size_t *bytes);

/*
 * Sparse factor of the GCN operation, Eqn (1) and Eqn (2): Z = sigma?(A~ H),
 *     Z[u] = dinv[u] * sum over stored (u,v) of dinv[v] * H[v],
 * i.e. every stored entry of A + I weighs 1/sqrt((1+deg_u)(1+deg_v)).
 *   rowptr, colidx, nnz     the snapshot (CSR of A + I)
 *   dinv [n]                from dgnn_delta_rebuild or dgnn_csr_dinv; NULL means all ones
 *                           (plain A + I, no normalisation)
 *   h [n][f], z [n][f]      storage type dt; z must not alias h
 *   flags                   any of DGNN_RELU, DGNN_H_PRESCALED.  With DGNN_H_PRESCALED the rows of h
 *                           are taken to be dinv[v] * H[v] already and only dinv[u] is applied:
 *                           Z[u] = dinv[u] * sum over stored (u,v) of h[v]
 *   ws, ws_bytes            scratch of at least dgnn_spmm_workspace() bytes
 * nnz may be an upper bound of the number of stored entries (the capacity of colidx, say): the kernels take the
 * smaller of it and rowptr[n].  The result does not depend on scheduling: no floating-point atomics are used.
 */
int dgnn_spmm(int64_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, const float *dinv,
              const void *h, int32_t f, void *z, dgnn_dtype dt, uint32_t flags,
              void *ws, size_t ws_bytes, void *stream);

/*
 * dgnn_spmm for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments and same kernels as dgnn_spmm, but no workspace argument: the carry
 * records, (16 + 8 f) bytes per range of stored entries that one wavefront streams, live in a device array of fixed
 * size inside the library (dgnn_spmm_static_limit() bytes, 32 MiB, held by every GPU the library runs on until the
 * process ends).  Where dgnn_spmm's ranges (2048 entries, fewer on small snapshots) would need more records than
 * the array holds, this call makes its ranges longer, up to 8192 entries: rows that a range's end cuts are then
 * summed in other pieces, so the result equals dgnn_spmm's bit for bit when the ranges are the same and within the
 * rounding of the fp32 sums otherwise.  DGNN_ERR_CAPACITY if ranges of 8192 entries are still too many
 * (f = 32: beyond 1.0e9 stored entries; f = 128: beyond 2.6e8); nothing is enqueued then.  Neither this call nor anything it calls allocates or frees; the
 * first call on a device looks up the array's address on that device, once.  All calls on one GPU share the one array:
 * calls that overlap in time on the same GPU (two streams, two threads) race on it, and the caller must order them.
 */
int dgnn_spmm_static_limit(size_t *bytes);
int dgnn_spmm_static(int64_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, const float *dinv,
                     const void *h, int32_t f, void *z, dgnn_dtype dt, uint32_t flags, void *stream);

/*
 * M-transform (Section "TM-GCN"): Y = Z x_1 M for the banded lower-triangular M,
 *     Y_t = sum_{j=0}^{min(w,t)-1} m(t,j) Z_{t-j},   t = 1..T (1-based),
 *   z, y [T][n][f]          storage type dt; y may be the same pointer as z (in place), and
 *                           must not overlap it in any other way
 *   w                       window, 1 <= min(w, T) <= 32
 *   m_band                  DEVICE float [T][w] with m_band[(t-1)*w + j] = m(t,j), or NULL for
 *                           the paper's weights m(t,j) = 1/min(w,t); entries with j >= t are
 *                           ignored
 */
int dgnn_mproduct(const void *z, void *y, int64_t T, int64_t n, int32_t f, int32_t w,
                  const float *m_band, dgnn_dtype dt, void *stream);

/*
 * ---- Snapshots that carry a value per stored entry (Section "Graph-difference Based Input Transfer" ships the
 * values of the new snapshot along with the two index lists; the smoothed graphs of Section "Smoothening the
 * Input Graphs" are where values other than 0/1 come from).  val[e] belongs to the stored entry colidx[e].
 * Two ways to get the values of the next snapshot onto the device:
 *   - as the paper does: rebuild the structure with dgnn_delta_rebuild and copy the whole value array of the new
 *     snapshot (it is in the canonical entry order, which both sides know);
 *   - only what changed: dgnn_delta_rebuild_weighted below.
 */

/*
 * A_next = (A_prev minus the deleted edges) plus the added edges, as dgnn_delta_rebuild, with values: surviving
 * entries keep their value unless the update list names them, added entries bring theirs.
 *   val_prev [nnz_prev], val_next [cap_next]    fp32, must not be the same array
 *   add_val [n_add]                             values of the added edges (list order)
 *   upd_row/upd_col/upd_val, n_upd              surviving edges whose value changes, each named once; must name
 *                                               neither deleted nor added edges (entries that are not in A_next
 *                                               are skipped)
 *   flags                                       DGNN_VALIDATE and/or DGNN_UPDATES_SORTED.  Without the latter the
 *                                               update list may come in any order and is applied by a pass of its
 *                                               own after the merge.  With
 *                                               it the list is sorted by (row, col) like the other two and the one
 *                                               streaming merge consumes it as well; a list that is not sorted
 *                                               then gives unspecified values, never an out-of-bounds access, and
 *                                               DGNN_VALIDATE reports DGNN_BAD_DELTA_ORDER for it.
 * No dinv is produced: the values are the matrix.  Everything else as dgnn_delta_rebuild.
 */
int dgnn_delta_rebuild_weighted(int64_t n,
                                const int32_t *rowptr_prev, const int32_t *colidx_prev, const float *val_prev,
                                int64_t nnz_prev,
                                const int32_t *add_row, const int32_t *add_col, const float *add_val, int64_t n_add,
                                const int32_t *del_row, const int32_t *del_col, int64_t n_del,
                                const int32_t *upd_row, const int32_t *upd_col, const float *upd_val, int64_t n_upd,
                                int32_t *rowptr_next, int32_t *colidx_next, float *val_next, int64_t cap_next,
                                int64_t *nnz_next,
                                void *ws, size_t ws_bytes, uint32_t flags, int32_t *d_status, void *stream);

/*
 * Checks that (rowptr, colidx) is a snapshot in the form every call here takes (the canonical form of a snapshot,
 * Section "Graph-difference Based Input Transfer": sent whole once, rebuilt from differences afterwards): rowptr[0] = 0,
 * rowptr ascending, rowptr[n] = nnz, every column in [0, n), columns strictly ascending inside a row and, with
 * require_diagonal != 0, the diagonal entry present in every row (the stored matrix is A + I, Eqn (1)).
 *   d_status  device int32, required: 0 if nothing was found, else the smallest DGNN_BAD_* code found.
 * Enqueue-only.  Errors: NULL, SHAPE (n <= 0, nnz < 0), OVERFLOW.
 */
int dgnn_csr_validate(int64_t n, const int32_t *rowptr, const int32_t *colidx, int64_t nnz, int require_diagonal,
                      int32_t *d_status, void *stream);

/*
 * Z = sigma?(V H) for a snapshot with explicit values, Z[u] = sum over stored (u,v) of val(u,v) * H[v]
 * (Eqn (2) with the matrix given entry by entry instead of through Eqn (1)).
 *   dinv NULL:      exactly that; flags: DGNN_RELU or 0.
 *   dinv [n] given: the sym-normalised weighted matrix D^(-1/2) V D^(-1/2) without materialising its values,
 *                   Z[u] = dinv[u] * sum val(u,v) * h[v] with h[v] = dinv[v] * H[v] already (DGNN_H_PRESCALED is
 *                   then required: the row_scale of dgnn_feature_transform).  With dinv from
 *                   dgnn_csr_weighted_dinv this is Eqn (1) generalised to weighted snapshots: only the values that
 *                   change travel from the host (dgnn_delta_rebuild_weighted), the normalisation is recomputed here.
 * Everything else as dgnn_spmm (same workspace query).  The adjoint is the same call on the transposed snapshot.
 */
int dgnn_spmm_weighted(int64_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, const float *val,
                       const float *dinv, const void *h, int32_t f, void *z, dgnn_dtype dt, uint32_t flags,
                       void *ws, size_t ws_bytes, void *stream);

/*
 * dinv[u] = (sum of val over row u)^(-1/2): the weighted counterpart of (1 + deg_u)^(-1/2) of Eqn (1) (for values
 * that are all 1 it is the same number).  Reading: the paper normalises its smoothed, weighted snapshots but does
 * not print the formula; this is Eqn (1) with the degree taken as the weighted row sum, self loop included.
 * ws: device scratch (16-byte aligned) of at least dgnn_csr_weighted_dinv_workspace(nnz) bytes (pieces of rows
 * that are summed by several wavefronts); contents need not be preserved.  Every sum has a fixed
 * order, results repeat bit for bit.  val[0 .. min(nnz, rowptr[n])) is read (nnz may be an upper bound of the
 * number of stored entries); errors: NULL, SHAPE (n <= 0, nnz <= 0), OVERFLOW,
 * CAPACITY (workspace too small), ALIGN.  A row whose sum is not positive (no entries, or
 * weights that cancel) gets 0: such a vertex neither sends nor receives, instead of producing infinities.
 */
int dgnn_csr_weighted_dinv_workspace(int64_t nnz, size_t *bytes);
int dgnn_csr_weighted_dinv(int64_t n, int64_t nnz, const int32_t *rowptr, const float *val, float *dinv,
                           void *ws, size_t ws_bytes, void *stream);

/*
 * One step of the sliding-window sum that smooths the input graphs (Section "Smoothening the Input Graphs"):
 *     C = S + alpha * A_in + beta * A_out
 * with S a snapshot with values and A_in, A_out unweighted snapshots (every stored entry counts 1), all n x n in
 * CSR with rows sorted by column: S_t = S_{t-1} + A_t - A_{t-l} is alpha = 1, beta = -1 (A_out NULL while the
 * window still grows).  Entries of equal (row, column) are added as S, then alpha, then beta, in fp32; an entry whose
 * result is exactly 0 is not stored (counts are small integers, so this is exact for them).
 *   diag_value: 0 = diagonal entries are summed like all others.  Otherwise every stored diagonal entry of C takes
 *   this value: the snapshots here hold A + I, but the section smooths A and Eqn (1) then adds the self loop once,
 *   so edge-life smoothing passes 1 (the self loop keeps weight 1 however long the window is); the M-transform of
 *   the adjacency tensor divides the sum of the A_i by min(l, t) before I is added, which after the symmetric
 *   normalisation is the same matrix as the plain sum with the diagonal at min(l, t): what 0 leaves there.
 *   rowptr_s/colidx_s/val_s, nnz_s: S; val_s NULL = all ones (S_1 = A_1).  rowptr_in/colidx_in, nnz_in and
 *   rowptr_out_of/colidx_out_of, nnz_out_of: A_in and A_out, each may be NULL (nothing to add).
 *   rowptr_c [n+1], colidx_c / val_c [capacity]: the result, canonical order; must not be S's arrays.
 * The number of stored entries of C is not known beforehand (at most nnz_s + nnz_in + nnz_out_of) and the host never
 * waits for it: it is left in rowptr_c[n], on the device.  The calls that take C afterwards (this one as S,
 * dgnn_csr_weighted_dinv, dgnn_spmm_weighted) accept an upper bound as their nnz argument, e.g. `capacity`, and read
 * the actual count from rowptr[n] themselves; so does this call for S.  If C does not fit `capacity`, nothing but
 * rowptr_c[n] (the size needed) is written and *d_status becomes DGNN_BAD_CAPACITY.
 *   d_status: device int32, may be NULL; reset to 0 by the call, DGNN_BAD_CAPACITY if C did not fit.
 *   ws: device scratch of at least dgnn_csr_combine_workspace(nnz_s) bytes.
 * Enqueue-only like every other call (it can be recorded in a HIP graph): a count launch, a scan that leaves the
 * total on the device, and a write launch that reads it there.
 * All pointers are device pointers.  Errors: NULL, SHAPE, OVERFLOW (nnz_s + nnz_in + nnz_out_of beyond the index
 * range), CAPACITY (workspace), ALIAS, ALIGN (ws not 16-byte aligned), HIP.
 */
int dgnn_csr_combine_workspace(int64_t nnz_s, size_t *bytes);
int dgnn_csr_combine(int64_t n, const int32_t *rowptr_s, const int32_t *colidx_s, const float *val_s, int64_t nnz_s,
                     const int32_t *rowptr_in, const int32_t *colidx_in, int64_t nnz_in, float alpha,
                     const int32_t *rowptr_out_of, const int32_t *colidx_out_of, int64_t nnz_out_of, float beta,
                     float diag_value,
                     int32_t *rowptr_c, int32_t *colidx_c, float *val_c, int64_t capacity, int32_t *d_status,
                     void *ws, size_t ws_bytes, void *stream);
/*
 * ---- Gradient propagation through the same path (Section "Gradient Checkpoint": a block is run forward
 * again and gradients then travel through it in the reverse direction).  For one GCN layer
 *     H = X W,  P = A~ H,  Z = max(P, 0),  Y = Z x_1 M
 * with G_Y = dL/dY given, the adjoints of the forward steps, in the order they are applied:
 *     G_Z = G_Y x_1 M^T                              dgnn_mproduct_backward
 *     G_P = G_Z where Z > 0, else 0                  dgnn_relu_backward
 *     G_H = A~^T G_P                                 dgnn_spmm on the TRANSPOSED snapshot (see below)
 *     dW += X^T G_H,   dX = G_H W^T                  dgnn_weight_grad, dgnn_input_grad
 *
 * A~^T G = D^(-1/2) (A + I)^T D^(-1/2) G needs no kernel of its own: call dgnn_spmm with rowptr/colidx of
 * (A + I)^T and with dinv of A (NOT the one derived from the transposed row lengths).  For an undirected
 * snapshot the transpose is the snapshot itself.  For a directed one the transposed snapshots form a dynamic
 * graph of their own, rebuilt by dgnn_delta_rebuild from the difference lists sorted by (col, row) with rows
 * and columns swapped (dgnn_csr_transpose for the first snapshot, dgnn_coo_transpose for the lists).  Walking a block backwards needs A_{t-1} from A_t: that is dgnn_delta_rebuild with the
 * added and deleted lists exchanged.
 */

/*
 * The transposed snapshot, for the adjoint of the aggregation (Section "Gradient Checkpoint": gradients travel through a
 * block in the reverse direction, which needs A~^T): (rowptr_t, colidx_t) = CSR of the transpose of (rowptr, colidx), in
 * the same canonical form (columns ascending inside a row); val / val_t: the values travel with their entries, or both
 * NULL.  nnz must be exact here.  The pairs are sorted by (column, row) with the device library's radix sort; ws: device
 * scratch of at least dgnn_csr_transpose_workspace() bytes (two arrays of 8-byte keys and the sort's own scratch; the
 * query asks the sort, so it needs a device).  Input formatting, once per block: not meant for graph capture.
 * Errors: NULL, SHAPE, OVERFLOW, ALIGN, ALIAS (an output is its input), CAPACITY, HIP.
 */
int dgnn_csr_transpose_workspace(int64_t n, int64_t nnz, int with_values, size_t *bytes);
int dgnn_csr_transpose(int64_t n, int64_t nnz, const int32_t *rowptr, const int32_t *colidx, const float *val,
                       int32_t *rowptr_t, int32_t *colidx_t, float *val_t, void *ws, size_t ws_bytes, void *stream);

/*
 * A difference list for the transposed series: the m pairs (row[i], col[i]) with rows and columns exchanged and sorted
 * by (new row, new column), i.e. (row_t[i], col_t[i]) = the pairs (col, row) in ascending order.  The transposed
 * snapshots of a directed dynamic graph are rebuilt by dgnn_delta_rebuild from such lists.  n: vertices (indices lie
 * in [0, n)).  Outputs must not overlap inputs.  ws as above, dgnn_coo_transpose_workspace() bytes.  m = 0 is allowed.
 */
int dgnn_coo_transpose_workspace(int64_t n, int64_t m, size_t *bytes);
int dgnn_coo_transpose(int64_t n, int64_t m, const int32_t *row, const int32_t *col, int32_t *row_t, int32_t *col_t,
                       void *ws, size_t ws_bytes, void *stream);

/*
 * Adjoint of the M-transform (Section "TM-GCN"): G_Z = G_Y x_1 M^T,
 *     G_Z[k] = sum_{j=0}^{min(w, T-k+1)-1} m(k+j, j) G_Y[k+j],   k = 1..T (1-based),
 * with the same m, w, m_band, layouts, limits and aliasing rules as dgnn_mproduct (g_z may be g_y).
 */
int dgnn_mproduct_backward(const void *g_y, void *g_z, int64_t T, int64_t n, int32_t f, int32_t w,
                           const float *m_band, dgnn_dtype dt, void *stream);

/*
 * The M-transform of a series that is processed in blocks of timesteps (Section "Gradient Checkpoint": the
 * frames of the last w timesteps of a block are among what is handed to the next block).  The block holds the
 * frames of timesteps t0+1 .. t0+T (1-based) of the whole series; the weights are those of the whole series,
 * 1/min(w, t) with t counted from the start of the series.
 *   z_before [n_before][n][f]   the frames of timesteps t0-n_before+1 .. t0, oldest first;
 *                               n_before must be min(w-1, t0) (NULL when that is 0)
 *   m_band [T][w]               optional, the block's rows of the band
 * Everything else as dgnn_mproduct; y must not overlap z_before.  Blocks chained this way give exactly the
 * frames dgnn_mproduct gives on the whole series.
 */
int dgnn_mproduct_block(const void *z, void *y, int64_t T, int64_t n, int32_t f, int32_t w,
                        const float *m_band, int64_t t0, const void *z_before, int64_t n_before,
                        dgnn_dtype dt, void *stream);

/*
 * Its adjoint, block by block from the last block to the first: the gradient frames of a block depend on the
 * upstream gradient of up to w-1 timesteps AFTER the block.
 *   g_after [n_after][n][f]     upstream gradient frames of timesteps t0+T+1 .. t0+T+n_after, nearest first
 *                               (in time order); n_after = min(w-1, timesteps after the block)
 *   m_band [T + n_after][w]     optional, the rows of the band for the block and for the frames after it
 * Everything else as dgnn_mproduct_backward; g_z must not overlap g_after.
 */
int dgnn_mproduct_backward_block(const void *g_y, void *g_z, int64_t T, int64_t n, int32_t f, int32_t w,
                                 const float *m_band, int64_t t0, const void *g_after, int64_t n_after,
                                 dgnn_dtype dt, void *stream);

/*
 * Gradient through sigma = ReLU of Eqn (2): out[u][:] = row_scale[u] * (z[u][:] > 0 ? g[u][:] : 0).
 *   g, z, out [n][f]        storage type dt; z is the layer's OUTPUT (positive exactly where the
 *                           pre-activation was); out may be the same pointer as g
 *   row_scale [n] fp32 or NULL; passing dinv prepares the rows for dgnn_spmm with DGNN_H_PRESCALED
 */
int dgnn_relu_backward(const void *g, const void *z, const float *row_scale, void *out, int64_t n, int32_t f,
                       dgnn_dtype dt, void *stream);

/* Workspace size of dgnn_weight_grad in bytes (HOST out-parameter); depends on the widths only. */
int dgnn_weight_grad_workspace(int32_t f_in, int32_t f_out, size_t *bytes);

/*
 * Gradient of the weight of H = X W (dense factor of Eqn (2)): dw = X^T G, or dw += X^T G.
 *   x [n][f_in], g [n][f_out]   storage type dt (g = dL/dH); products accumulate in fp32 on the matrix cores
 *   dw [f_in][f_out]            fp32 whatever dt is; with accumulate != 0 the result is added to it (the sum
 *                               over the timesteps of a block that share one W)
 *   ws, ws_bytes                scratch of at least dgnn_weight_grad_workspace() bytes
 * The sum over rows has a fixed order: results repeat bit for bit.
 */
int dgnn_weight_grad(const void *x, const void *g, int64_t n, int32_t f_in, int32_t f_out, float *dw,
                     int32_t accumulate, dgnn_dtype dt, void *ws, size_t ws_bytes, void *stream);

/*
 * Gradient of the input of H = X W: dx = G W^T, or diag(row_scale) G W^T.
 *   g [n][f_out], w [f_in][f_out] (the forward layout, read transposed), dx [n][f_in]; otherwise as
 *   dgnn_feature_transform.
 */
int dgnn_input_grad(const void *g, int64_t n, int32_t f_out, const void *w, int32_t f_in,
                    const float *row_scale, void *dx, dgnn_dtype dt, void *stream);

/*
 * ---- The CD-GCN layer (Section "CD-GCN"): its GCN operation has a skip connection,
 *     Y0 = A~ X,   Y1 = Y0 W,   Y = sigma(Y0 o Y1)      (o = side by side: F + F' features),
 * and an LSTM aggregates over time, one state (h, c) per vertex.  Y0 is dgnn_spmm (without DGNN_RELU and without
 * DGNN_H_PRESCALED), Y1 and the two products of the gate pre-activations are dgnn_feature_transform; the two calls
 * below are the steps that are left.  Forward only.
 */

/* out [n][f0 + f1] = relu of the rows of y0 [n][f0] and y1 [n][f1] laid side by side; out must not be y0 or y1. */
int dgnn_concat_relu(const void *y0, int32_t f0, const void *y1, int32_t f1, void *out, int64_t n,
                     dgnn_dtype dt, void *stream);

/*
 * The same Y formed in one pass, without materialising Y1: out [n][f_in + f_out] = relu([x | x W]) with
 * x [n][f_in] = Y0 and w [f_in][f_out], the ReLU and the concatenation folded into the kernel that forms the product.
 * Supported where both tiles and W fit on chip together: fp32 with f_in in {16, 32, 64} and f_out in {32, 64};
 * bf16 with f_in, f_out in {32, 64} and f_in + f_out <= 128 (DGNN_ERR_SHAPE otherwise: use dgnn_feature_transform and
 * dgnn_concat_relu).  Same values as that composition (bf16: the product is rounded to bf16 once either way).
 * out must not be x.  Errors as dgnn_feature_transform.
 */
int dgnn_transform_concat_relu(const void *x, int64_t n, int32_t f_in, const void *w, int32_t f_out, void *out,
                               dgnn_dtype dt, void *stream);

/*
 * LSTM cell.  gates_x = X_t W_x and gates_h = h_{t-1} W_h, both [n][4 * hidden] with the gates in the order
 * (input, forget, cell, output); bias fp32 [4 * hidden] or NULL.  With a = gates_x + gates_h + bias:
 *     c_next = sig(a_f) * c_prev + sig(a_i) * tanh(a_g),     h_next = sig(a_o) * tanh(c_next).
 * c_prev, c_next, h_next [n][hidden]; c_next may be c_prev (in place); h_next must be a buffer of its own.
 * hidden must be a supported feature width.
 */
int dgnn_lstm_cell(const void *gates_x, const void *gates_h, const float *bias, const void *c_prev, void *c_next,
                   void *h_next, int64_t n, int32_t hidden, dgnn_dtype dt, void *stream);

/*
 * One whole LSTM step without materialising the gate pre-activations: a = [y | h_prev] [w_x ; w_h] + bias is formed
 * on the matrix cores and the cell of dgnn_lstm_cell is applied to the accumulators.
 *   y [n][f_y], h_prev [n][hidden], w_x [f_y][4 * hidden], w_h [hidden][4 * hidden], bias fp32 [4 * hidden] or NULL
 *   c [n][hidden]        cell state, updated IN PLACE;   h_next [n][hidden]   a buffer of its own
 * Supported: fp32 storage with hidden = 16 or 32, bf16 storage with hidden = 32 or 64, and f_y = hidden or
 * 2 * hidden (DGNN_ERR_SHAPE otherwise: use the two dense transforms and dgnn_lstm_cell).  fp32: same result as that
 * composition up to the order of the fp32 sums.  bf16: the pre-activations stay in fp32 here, where the composition
 * rounds the two products to bf16 before it adds them; c and h are rounded once, when they are stored.
 */
int dgnn_lstm_step(const void *y, int32_t f_y, const void *h_prev, const void *w_x, const void *w_h,
                   const float *bias, void *c, void *h_next, int64_t n, int32_t hidden, dgnn_dtype dt,
                   void *stream);

/*
 * ---- Gradient propagation through the CD-GCN layer (Section "CD-GCN"; trained as in Section "Gradient
 * Checkpoint": the forward values of a timestep are recomputed when its gradients are formed) ----
 *
 * LSTM cell: from the gradient with respect to the new state to the gradient with respect to the gate
 * pre-activations and the old cell state.  gates_x, gates_h [n, 4*hidden] and bias as in dgnn_lstm_cell (recomputed
 * by the caller), c_prev [n, hidden] the cell state the step started from.
 *   dL/dh_t = dh_a + dh_b (either may be NULL: the loss's own gradient and the one carried back from step t+1),
 *   dL/dc_t = dc_next (NULL = zero).  At least one of the three must be given.
 *   da [n, 4*hidden]: dL/d(pre-activations), gate order (input, forget, cell, output); dc_prev [n, hidden]: dL/dc_{t-1}
 *   (may be the same buffer as dc_next).  The other gradients are the dense transform's adjoints applied to da:
 *   dW_x = Y^T da and dW_h = h_{t-1}^T da (dgnn_weight_grad), dY = da W_x^T and dh_{t-1} = da W_h^T (dgnn_input_grad),
 *   db = column sums of da (dgnn_bias_grad).
 * Errors: NULL, SHAPE (hidden not a feature width), OVERFLOW, ALIGN, ALIAS.
 */
int dgnn_lstm_cell_backward(const void *gates_x, const void *gates_h, const float *bias, const void *c_prev,
                            const void *dh_a, const void *dh_b, const void *dc_next, void *da, void *dc_prev,
                            int64_t n, int32_t hidden, dgnn_dtype dt, void *stream);

/*
 * The same with the gate pre-activations recomputed on chip (the adjoint of dgnn_lstm_step): takes Y, h_{t-1}, W_x,
 * W_h and the bias instead of the two halves of the pre-activations, everything else as dgnn_lstm_cell_backward.
 * fp32 storage with hidden = 16 or 32, bf16 storage with hidden = 32; f_y = hidden or 2 * hidden (DGNN_ERR_SHAPE otherwise: use the two dense transforms and
 * dgnn_lstm_cell_backward).  bf16: the pre-activations and the cell's formulas in fp32, da and dc_prev rounded once.
 */
int dgnn_lstm_step_backward(const void *y, int32_t f_y, const void *h_prev, const void *w_x, const void *w_h,
                            const float *bias, const void *c_prev, const void *dh_a, const void *dh_b,
                            const void *dc_next, void *da, void *dc_prev, int64_t n, int32_t hidden, dgnn_dtype dt,
                            void *stream);

/*
 * Adjoint of dgnn_concat_relu: dy, y [n, f0 + f1] (y = the forward output); d0 [n, f0] and d1 [n, f1] receive the
 * two column blocks of dy where y > 0, zero elsewhere.  d0 may be NULL (the gradient with respect to Y0's own block
 * is needed only when a layer lies below).  Errors as dgnn_concat_relu.
 */
int dgnn_concat_relu_backward(const void *dy, const void *y, void *d0, int32_t f0, void *d1, int32_t f1, int64_t n,
                              dgnn_dtype dt, void *stream);

/*
 * db[c] (+)= sum over rows of g[r][c]: the gradient of a bias added to every row (fp32 sums of fp32 / bf16 rows, in
 * a fixed order: results repeat bit for bit).  g [n, f]; f a power of two times 4 (fp32) or 8 (bf16), at most 512.
 * ws: device scratch of at least dgnn_bias_grad_workspace(f) bytes.  accumulate != 0 adds to db.
 */
int dgnn_bias_grad_workspace(int32_t f, size_t *bytes);
int dgnn_bias_grad(const void *g, int64_t n, int32_t f, float *db, int accumulate, dgnn_dtype dt, void *ws,
                   size_t ws_bytes, void *stream);

/*
 * out = a + b for [n, f] tensors of one storage type (the sum is formed in fp32 and rounded once): a gradient that
 * reaches a tensor along two paths.  out may be a or b.  f a feature width.  Errors: NULL, SHAPE, OVERFLOW, ALIGN.
 */
int dgnn_add(const void *a, const void *b, void *out, int64_t n, int32_t f, dgnn_dtype dt, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DGNN_H */
