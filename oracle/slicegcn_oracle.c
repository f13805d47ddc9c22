/*
 * SliceGCN reference oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, fp64 CPU statement of what the slice-GCN hot path computes, written
 * from the paper's definitions.  It shares no code with the HIP library and must only be
 * called from the tests, the smoke check and the benchmark's CPU-baseline leg.
 *
 * Everything is the textbook definition written out: no blocking, no fusion, no
 * reordering.  Rows may be processed by different OpenMP threads, but every individual
 * sum runs sequentially in index order in fp64.
 *
 * Conventions: row-major matrices with explicit leading dimension (in elements);
 * CSR with int64 rowptr, int32 colidx (ascending, unique per row), fp64 vals.
 *
 * Pins (see tests/test_oracle_*.py): dense brute force on tiny graphs, closed-form graphs
 * (empty, complete, ring, star), the fixed-point invariant of the normalised adjacency,
 * the slice/concat identity, adjoint identities, finite differences, and library
 * cross-checks (tests/test_oracle_classifier.py for the dense layer and the loss; tests/test_oracle_order.py
 * for the row orders: hand examples, queue invariants, scipy's breadth-first order).  No function
 * here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_EINVAL (-1)
#define ORACLE_ERANGE (-2)
#define ORACLE_ENOMEM (-3)

#define ORACLE_SYMMETRIZE 1u
#define ORACLE_ADD_SELF_LOOPS 2u

/* ------------------------------------------------------------------------------------
 * Slice strategy: the paper's Algorithm 1 (slice strategy generation).
 * slice_size = ceil(in_d / p); slice i starts at i*slice_size and is
 * int(slice_size * scale) wide; a slice that would run past in_d is shifted left so
 * that it ends exactly at in_d.
 * ---------------------------------------------------------------------------------- */
int oracle_slice_strategy(int32_t in_d, int32_t p, double slice_size_scale,
                          int32_t *starts, int32_t *ends, int32_t *slice_size)
{
    if (in_d < 1 || p < 1 || p > in_d || !starts || !ends || !slice_size) return ORACLE_EINVAL;
    if (!(slice_size_scale > 0.0)) return ORACLE_EINVAL;
    int32_t s = (in_d + p - 1) / p;
    double scaled = (double)s * slice_size_scale;
    if (!(scaled >= 1.0) || scaled > (double)in_d) return ORACLE_EINVAL;
    int32_t width = (int32_t)scaled; /* truncation toward zero, as int() does */
    for (int32_t i = 0; i < p; ++i) {
        int64_t start = (int64_t)i * s;
        int64_t end = start + width;
        if (end > in_d) {
            start -= end - in_d;
            end = in_d;
        }
        if (start < 0) return ORACLE_EINVAL;
        starts[i] = (int32_t)start;
        ends[i] = (int32_t)end;
    }
    *slice_size = s;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------
 * Normalised adjacency in CSR.
 *
 * Pattern: A~ = A (or A | A^T when SYMMETRIZE) with duplicates collapsed (A is a 0/1
 * matrix), input self pairs dropped, and -- when ADD_SELF_LOOPS -- exactly one diagonal
 * entry per row.  d~_v = number of stored entries of row v (|N(v)| with v counted among
 * its own neighbours); entry (v,u) carries 1/c_vu = 1/(sqrt(d~_v) sqrt(d~_u)), the
 * normalisation constant of the paper's GCN layer equation.  A row with no entry (only
 * possible without self loops) uses degree 1 so the value stays finite.
 * ---------------------------------------------------------------------------------- */
static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

int oracle_build_norm_csr(const int64_t *src, const int64_t *dst, int64_t n_edges,
                          int64_t n_nodes, uint32_t flags,
                          int64_t *rowptr /* n_nodes+1 */, int32_t *deg /* n_nodes */,
                          double *dinv /* n_nodes */,
                          int32_t **colidx_out, double **vals_out)
{
    if (n_nodes < 1 || n_edges < 0 || (n_edges > 0 && (!src || !dst))) return ORACLE_EINVAL;
    if (!rowptr || !deg || !dinv || !colidx_out || !vals_out) return ORACLE_EINVAL;
    if (flags & ~(ORACLE_SYMMETRIZE | ORACLE_ADD_SELF_LOOPS)) return ORACLE_EINVAL;
    if (n_nodes > INT32_MAX) return ORACLE_ERANGE;
    const int sym = (flags & ORACLE_SYMMETRIZE) != 0;
    const int loops = (flags & ORACLE_ADD_SELF_LOOPS) != 0;

    for (int64_t e = 0; e < n_edges; ++e)
        if (src[e] < 0 || src[e] >= n_nodes || dst[e] < 0 || dst[e] >= n_nodes) return ORACLE_ERANGE;

    /* candidate count per row (duplicates still in) */
    int64_t *start = (int64_t *)calloc((size_t)n_nodes + 1, sizeof(int64_t));
    if (!start) return ORACLE_ENOMEM;
    for (int64_t e = 0; e < n_edges; ++e) {
        if (src[e] == dst[e]) continue;
        start[src[e] + 1]++;
        if (sym) start[dst[e] + 1]++;
    }
    if (loops)
        for (int64_t v = 0; v < n_nodes; ++v) start[v + 1]++;
    for (int64_t v = 0; v < n_nodes; ++v) start[v + 1] += start[v];
    const int64_t n_cand = start[n_nodes];

    int32_t *cand = (int32_t *)malloc((size_t)(n_cand > 0 ? n_cand : 1) * sizeof(int32_t));
    int64_t *fill = (int64_t *)malloc((size_t)n_nodes * sizeof(int64_t));
    if (!cand || !fill) { free(start); free(cand); free(fill); return ORACLE_ENOMEM; }
    memcpy(fill, start, (size_t)n_nodes * sizeof(int64_t));
    for (int64_t e = 0; e < n_edges; ++e) {
        int64_t u = src[e], v = dst[e];
        if (u == v) continue;
        cand[fill[u]++] = (int32_t)v;
        if (sym) cand[fill[v]++] = (int32_t)u;
    }
    if (loops)
        for (int64_t v = 0; v < n_nodes; ++v) cand[fill[v]++] = (int32_t)v;

    /* sort each row's candidates ascending and collapse repeats */
#pragma omp parallel for schedule(dynamic, 1024)
    for (int64_t v = 0; v < n_nodes; ++v) {
        int32_t *row = cand + start[v];
        int64_t len = start[v + 1] - start[v];
        qsort(row, (size_t)len, sizeof(int32_t), cmp_i32);
        int64_t m = 0;
        for (int64_t i = 0; i < len; ++i)
            if (i == 0 || row[i] != row[i - 1]) row[m++] = row[i];
        fill[v] = m; /* distinct entries of row v */
    }

    rowptr[0] = 0;
    for (int64_t v = 0; v < n_nodes; ++v) rowptr[v + 1] = rowptr[v] + fill[v];
    const int64_t nnz = rowptr[n_nodes];
    int32_t *colidx = (int32_t *)malloc((size_t)(nnz > 0 ? nnz : 1) * sizeof(int32_t));
    double *vals = (double *)malloc((size_t)(nnz > 0 ? nnz : 1) * sizeof(double));
    if (!colidx || !vals) { free(start); free(cand); free(fill); free(colidx); free(vals); return ORACLE_ENOMEM; }

    for (int64_t v = 0; v < n_nodes; ++v) {
        deg[v] = (int32_t)fill[v];
        int32_t dnorm = deg[v] > 0 ? deg[v] : 1;
        dinv[v] = 1.0 / sqrt((double)dnorm);
        memcpy(colidx + rowptr[v], cand + start[v], (size_t)fill[v] * sizeof(int32_t));
    }
    for (int64_t v = 0; v < n_nodes; ++v)
        for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) vals[e] = dinv[v] * dinv[colidx[e]];

    free(start); free(cand); free(fill);
    *colidx_out = colidx;
    *vals_out = vals;
    return ORACLE_OK;
}

void oracle_free(void *p) { free(p); }

/* ------------------------------------------------------------------------------------
 * Row processing order (the library's optional locality preprocessing; the paper fixes no
 * execution order, so this is defined here, uniquely, and the library must reproduce it):
 *   mode 1, by degree: rows by descending number of stored entries, ties by ascending id;
 *   mode 2, breadth first: at most `max_trees` times, take the not yet placed row that comes
 *     first in the degree order as a root and place the rows reachable from it in the order
 *     a first-in-first-out queue visits them, the neighbours of a row in ascending id; rows
 *     still unplaced after that follow in degree order.
 * order[p] = id of the row at position p.
 * ---------------------------------------------------------------------------------- */
typedef struct { int32_t deg; int32_t id; } deg_id;

static int cmp_deg_desc(const void *a, const void *b)
{
    const deg_id *x = (const deg_id *)a, *y = (const deg_id *)b;
    if (x->deg != y->deg) return x->deg > y->deg ? -1 : 1;
    return (x->id > y->id) - (x->id < y->id);
}

int oracle_row_order(int64_t n, const int64_t *rowptr, const int32_t *colidx, int mode, int32_t max_trees,
                     int32_t *order)
{
    if (n < 1 || !rowptr || !order || (mode != 1 && mode != 2)) return ORACLE_EINVAL;
    deg_id *by_deg = (deg_id *)malloc((size_t)n * sizeof(deg_id));
    if (!by_deg) return ORACLE_ENOMEM;
    for (int64_t v = 0; v < n; ++v) {
        by_deg[v].deg = (int32_t)(rowptr[v + 1] - rowptr[v]);
        by_deg[v].id = (int32_t)v;
    }
    qsort(by_deg, (size_t)n, sizeof(deg_id), cmp_deg_desc);
    if (mode == 1) {
        for (int64_t p = 0; p < n; ++p) order[p] = by_deg[p].id;
        free(by_deg);
        return ORACLE_OK;
    }
    unsigned char *placed = (unsigned char *)calloc((size_t)n, 1);
    if (!placed) { free(by_deg); return ORACLE_ENOMEM; }
    int64_t count = 0, cursor = 0;
    for (int32_t tree = 0; tree < max_trees && count < n; ++tree) {
        while (placed[by_deg[cursor].id]) ++cursor;
        int64_t head = count;                 /* the queue is order[head .. count) */
        order[count++] = by_deg[cursor].id;
        placed[by_deg[cursor].id] = 1;
        while (head < count) {
            const int32_t v = order[head++];
            for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {   /* columns ascend within a row */
                const int32_t u = colidx[e];
                if (!placed[u]) { placed[u] = 1; order[count++] = u; }
            }
        }
    }
    for (int64_t p = 0; p < n && count < n; ++p)
        if (!placed[by_deg[p].id]) order[count++] = by_deg[p].id;
    free(placed);
    free(by_deg);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------
 * Sparse aggregation: the inner sum of the SliceGCN layer equation,
 *     Z[v, j] = sum over stored (v,u) of vals_vu * X[u, j].
 * transpose != 0 applies the transposed matrix by scatter, a separate code path:
 *     Z[u, j] += vals_vu * X[v, j].
 * ---------------------------------------------------------------------------------- */
int oracle_spmm(int64_t n, const int64_t *rowptr, const int32_t *colidx, const double *vals,
                int transpose, const double *X, int64_t ldx, int32_t w, double *Z, int64_t ldz)
{
    if (n < 1 || !rowptr || !colidx || !vals || !X || !Z || w < 1 || ldx < w || ldz < w) return ORACLE_EINVAL;
    if (!transpose) {
#pragma omp parallel for schedule(dynamic, 256)
        for (int64_t v = 0; v < n; ++v) {
            for (int32_t j = 0; j < w; ++j) {
                double acc = 0.0;
                for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e)
                    acc += vals[e] * X[(int64_t)colidx[e] * ldx + j];
                Z[v * ldz + j] = acc;
            }
        }
    } else {
        for (int64_t v = 0; v < n; ++v)
            for (int32_t j = 0; j < w; ++j) Z[v * ldz + j] = 0.0;
        for (int64_t v = 0; v < n; ++v)
            for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
                int64_t u = colidx[e];
                for (int32_t j = 0; j < w; ++j) Z[u * ldz + j] += vals[e] * X[v * ldx + j];
            }
    }
    return ORACLE_OK;
}

/* Selected output rows of the non-transposed aggregation (for checks at sizes where the
 * whole product is too slow): Zrows[i, :] = row rows[i] of A^ X. */
int oracle_spmm_rows(int64_t n, const int64_t *rowptr, const int32_t *colidx, const double *vals,
                     const double *X, int64_t ldx, int32_t w,
                     const int64_t *rows, int64_t n_rows, double *Zrows, int64_t ldz)
{
    if (n < 1 || !rowptr || !colidx || !vals || !X || !Zrows || !rows || w < 1 || ldx < w || ldz < w) return ORACLE_EINVAL;
    for (int64_t i = 0; i < n_rows; ++i) {
        int64_t v = rows[i];
        if (v < 0 || v >= n) return ORACLE_ERANGE;
        for (int32_t j = 0; j < w; ++j) {
            double acc = 0.0;
            for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e)
                acc += vals[e] * X[(int64_t)colidx[e] * ldx + j];
            Zrows[i * ldz + j] = acc;
        }
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------
 * Plain dense helpers (triple loops).
 * ---------------------------------------------------------------------------------- */
/* C[n x q] = A[n x m] * B[m x q] */
static void matmul_nn(int64_t n, int32_t m, int32_t q, const double *A, int64_t lda,
                      const double *B, int64_t ldb, double *C, int64_t ldc)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int32_t j = 0; j < q; ++j) {
            double acc = 0.0;
            for (int32_t t = 0; t < m; ++t) acc += A[i * lda + t] * B[(int64_t)t * ldb + j];
            C[i * ldc + j] = acc;
        }
}

/* ------------------------------------------------------------------------------------
 * One SliceGCN layer, forward: the paper's layer equation as typeset,
 *     Z = A^ Hin;  P = b + Z W_agg;  Hout = act(P) + Hin W_self + b_self,
 * with the self term outside the activation.  act: 0 = identity, 1 = ReLU.
 * W_self and b_self may be NULL (term absent).  Z (n x w_in) and P (n x w_out) are
 * returned because the backward pass needs them.
 * ---------------------------------------------------------------------------------- */
int oracle_layer_fwd(int64_t n, const int64_t *rowptr, const int32_t *colidx, const double *vals,
                     int32_t w_in, int32_t w_out, int act,
                     const double *Hin, int64_t ldi,
                     const double *W_agg /* w_in x w_out */, const double *b /* w_out or NULL */,
                     const double *W_self /* w_in x w_out or NULL */, const double *b_self /* w_out or NULL */,
                     double *Z /* n x w_in, ld w_in */, double *P /* n x w_out, ld w_out */,
                     double *Hout, int64_t ldo)
{
    if (!Hin || !W_agg || !Z || !P || !Hout || w_in < 1 || w_out < 1 || ldi < w_in || ldo < w_out) return ORACLE_EINVAL;
    if (act != 0 && act != 1) return ORACLE_EINVAL;
    int rc = oracle_spmm(n, rowptr, colidx, vals, 0, Hin, ldi, w_in, Z, w_in);
    if (rc) return rc;
    matmul_nn(n, w_in, w_out, Z, w_in, W_agg, w_out, P, w_out);
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < n; ++v)
        for (int32_t j = 0; j < w_out; ++j) {
            if (b) P[v * w_out + j] += b[j];
            double p = P[v * w_out + j];
            double r = (act == 1) ? (p > 0.0 ? p : 0.0) : p;
            double s = 0.0;
            if (W_self)
                for (int32_t t = 0; t < w_in; ++t) s += Hin[v * ldi + t] * W_self[(int64_t)t * w_out + j];
            if (b_self) s += b_self[j];
            Hout[v * ldo + j] = r + s;
        }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------
 * One SliceGCN layer, backward: the derivative of oracle_layer_fwd by the chain rule.
 *   dP = dHout * mask          (mask[v,j] = 1 where the activation passed the value;
 *                               all ones for act = identity; ReLU'(0) = 0)
 *   db = column sums of dP;    db_self = column sums of dHout
 *   dW_agg = Z^T dP;           dW_self = Hin^T dHout
 *   dZ = dP W_agg^T;           dHin = A^^T dZ + dHout W_self^T
 * The mask is an explicit input (n x w_out bytes) so that a caller can state which
 * activation decisions the gradient is taken for.  Any output pointer may be NULL.
 * ---------------------------------------------------------------------------------- */
int oracle_layer_bwd(int64_t n, const int64_t *rowptr, const int32_t *colidx, const double *vals,
                     int32_t w_in, int32_t w_out,
                     const double *Hin, int64_t ldi, const double *Z /* ld w_in */,
                     const uint8_t *mask /* n x w_out */,
                     const double *W_agg, const double *W_self /* or NULL */,
                     const double *dHout, int64_t ldo,
                     double *dW_agg, double *db, double *dW_self, double *db_self,
                     double *dHin, int64_t ldgi)
{
    if (!Hin || !Z || !mask || !W_agg || !dHout || w_in < 1 || w_out < 1 || ldi < w_in || ldo < w_out) return ORACLE_EINVAL;
    double *dP = (double *)malloc((size_t)n * w_out * sizeof(double));
    if (!dP) return ORACLE_ENOMEM;
    for (int64_t v = 0; v < n; ++v)
        for (int32_t j = 0; j < w_out; ++j)
            dP[v * w_out + j] = mask[v * w_out + j] ? dHout[v * ldo + j] : 0.0;

    if (db)
        for (int32_t j = 0; j < w_out; ++j) {
            double acc = 0.0;
            for (int64_t v = 0; v < n; ++v) acc += dP[v * w_out + j];
            db[j] = acc;
        }
    if (db_self)
        for (int32_t j = 0; j < w_out; ++j) {
            double acc = 0.0;
            for (int64_t v = 0; v < n; ++v) acc += dHout[v * ldo + j];
            db_self[j] = acc;
        }
    if (dW_agg)
#pragma omp parallel for schedule(static)
        for (int32_t t = 0; t < w_in; ++t)
            for (int32_t j = 0; j < w_out; ++j) {
                double acc = 0.0;
                for (int64_t v = 0; v < n; ++v) acc += Z[v * w_in + t] * dP[v * w_out + j];
                dW_agg[(int64_t)t * w_out + j] = acc;
            }
    if (dW_self)
#pragma omp parallel for schedule(static)
        for (int32_t t = 0; t < w_in; ++t)
            for (int32_t j = 0; j < w_out; ++j) {
                double acc = 0.0;
                for (int64_t v = 0; v < n; ++v) acc += Hin[v * ldi + t] * dHout[v * ldo + j];
                dW_self[(int64_t)t * w_out + j] = acc;
            }
    if (dHin) {
        if (ldgi < w_in) { free(dP); return ORACLE_EINVAL; }
        double *dZ = (double *)malloc((size_t)n * w_in * sizeof(double));
        if (!dZ) { free(dP); return ORACLE_ENOMEM; }
#pragma omp parallel for schedule(static)
        for (int64_t v = 0; v < n; ++v)
            for (int32_t t = 0; t < w_in; ++t) {
                double acc = 0.0;
                for (int32_t j = 0; j < w_out; ++j) acc += dP[v * w_out + j] * W_agg[(int64_t)t * w_out + j];
                dZ[v * w_in + t] = acc;
            }
        int rc = oracle_spmm(n, rowptr, colidx, vals, 1, dZ, w_in, w_in, dHin, ldgi);
        free(dZ);
        if (rc) { free(dP); return rc; }
        if (W_self)
#pragma omp parallel for schedule(static)
            for (int64_t v = 0; v < n; ++v)
                for (int32_t t = 0; t < w_in; ++t) {
                    double acc = 0.0;
                    for (int32_t j = 0; j < w_out; ++j) acc += dHout[v * ldo + j] * W_self[(int64_t)t * w_out + j];
                    dHin[v * ldgi + t] += acc;
                }
    }
    free(dP);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------
 * Slice encoding + concatenation (the paper's slice-encoding and CONCAT equations):
 *     H[v, off_i + j] = H^i[v, j] + E[i, j],   off_i = sum of widths of slices before i.
 * E (k rows, leading dimension lde) may be NULL: plain concatenation.
 * Backward: dH^i is the column block of dH; dE[i, j] = sum over nodes of dH[v, off_i + j].
 * ---------------------------------------------------------------------------------- */
int oracle_encode_concat(int32_t k, const double *const *Hs, const int64_t *lds, const int32_t *widths,
                         const double *E, int64_t lde, int64_t n, double *H, int64_t ldh)
{
    if (k < 1 || !Hs || !lds || !widths || !H || n < 1) return ORACLE_EINVAL;
    int64_t off = 0;
    for (int32_t i = 0; i < k; ++i) {
        if (widths[i] < 1 || lds[i] < widths[i] || !Hs[i]) return ORACLE_EINVAL;
        if (off + widths[i] > ldh) return ORACLE_EINVAL;
        for (int64_t v = 0; v < n; ++v)
            for (int32_t j = 0; j < widths[i]; ++j)
                H[v * ldh + off + j] = Hs[i][v * lds[i] + j] + (E ? E[(int64_t)i * lde + j] : 0.0);
        off += widths[i];
    }
    return ORACLE_OK;
}

int oracle_encode_concat_bwd(int32_t k, const double *dH, int64_t ldh, int64_t n, const int32_t *widths,
                             double *const *dHs /* entries may be NULL */, const int64_t *lds,
                             double *dE /* may be NULL */, int64_t lde)
{
    if (k < 1 || !dH || !widths || n < 1) return ORACLE_EINVAL;
    int64_t off = 0;
    for (int32_t i = 0; i < k; ++i) {
        if (widths[i] < 1 || off + widths[i] > ldh) return ORACLE_EINVAL;
        if (dHs && dHs[i]) {
            if (!lds || lds[i] < widths[i]) return ORACLE_EINVAL;
            for (int64_t v = 0; v < n; ++v)
                for (int32_t j = 0; j < widths[i]; ++j) dHs[i][v * lds[i] + j] = dH[v * ldh + off + j];
        }
        if (dE)
            for (int32_t j = 0; j < widths[i]; ++j) {
                double acc = 0.0;
                for (int64_t v = 0; v < n; ++v) acc += dH[v * ldh + off + j];
                dE[(int64_t)i * lde + j] = acc;
            }
        off += widths[i];
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------
 * Dense layer Y = act(X W + b): the unit the paper's classifier MLP_CLS (classifier equation)
 * and its feature-fusion MLP_FF (feature-fusion equation) are stacked from.
 * X: n x w_in (ldx), W: w_in x w_out row-major, b: w_out or NULL, act: 0 identity / 1 ReLU.
 * P (n x w_out, ld w_out) receives the pre-activation X W + b, Y (ldy) the output.
 * ---------------------------------------------------------------------------------- */
int oracle_linear_fwd(int64_t n, int32_t w_in, int32_t w_out, int act, const double *X, int64_t ldx,
                      const double *W, const double *b, double *P, double *Y, int64_t ldy)
{
    if (!X || !W || !P || !Y || n < 1 || w_in < 1 || w_out < 1 || ldx < w_in || ldy < w_out) return ORACLE_EINVAL;
    if (act != 0 && act != 1) return ORACLE_EINVAL;
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < n; ++v)
        for (int32_t j = 0; j < w_out; ++j) {
            double acc = 0.0;
            for (int32_t t = 0; t < w_in; ++t) acc += X[v * ldx + t] * W[(int64_t)t * w_out + j];
            if (b) acc += b[j];
            P[v * w_out + j] = acc;
            Y[v * ldy + j] = (act == 1 && !(acc > 0.0)) ? 0.0 : acc;
        }
    return ORACLE_OK;
}

/* Backward of the dense layer (chain rule; ReLU'(0) = 0):
 *   dP = dY * mask;  db = column sums of dP;  dW = X^T dP;  dX = dP W^T.
 * mask: n x w_out bytes (1 where the activation passed the value; all ones for identity).
 * Any output pointer may be NULL. */
int oracle_linear_bwd(int64_t n, int32_t w_in, int32_t w_out, const double *X, int64_t ldx,
                      const double *W, const uint8_t *mask, const double *dY, int64_t lddy,
                      double *dX, int64_t lddx, double *dW, double *db)
{
    if (!X || !W || !mask || !dY || n < 1 || w_in < 1 || w_out < 1 || ldx < w_in || lddy < w_out) return ORACLE_EINVAL;
    if (dX && lddx < w_in) return ORACLE_EINVAL;
    if (db)
        for (int32_t j = 0; j < w_out; ++j) {
            double acc = 0.0;
            for (int64_t v = 0; v < n; ++v) acc += mask[v * w_out + j] ? dY[v * lddy + j] : 0.0;
            db[j] = acc;
        }
    if (dW) {
#pragma omp parallel for schedule(static)
        for (int32_t t = 0; t < w_in; ++t)
            for (int32_t j = 0; j < w_out; ++j) {
                double acc = 0.0;
                for (int64_t v = 0; v < n; ++v)
                    acc += X[v * ldx + t] * (mask[v * w_out + j] ? dY[v * lddy + j] : 0.0);
                dW[(int64_t)t * w_out + j] = acc;
            }
    }
    if (dX) {
#pragma omp parallel for schedule(static)
        for (int64_t v = 0; v < n; ++v)
            for (int32_t t = 0; t < w_in; ++t) {
                double acc = 0.0;
                for (int32_t j = 0; j < w_out; ++j)
                    acc += (mask[v * w_out + j] ? dY[v * lddy + j] : 0.0) * W[(int64_t)t * w_out + j];
                dX[v * lddx + t] = acc;
            }
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------
 * Mean softmax cross-entropy over all nodes (the paper's loss equation with every node
 * labelled):  loss = -(1/n) sum_v log softmax(logits[v, :])[label_v].
 * log softmax(x)[y] = x_y - log sum_j exp(x_j); the row maximum is subtracted before
 * exponentiating, which changes nothing mathematically and keeps exp() in range.
 * dlogits (n x c, ldd; may be NULL) receives the gradient (softmax - onehot) / n.
 * ---------------------------------------------------------------------------------- */
int oracle_softmax_ce(int64_t n, int32_t c, const double *logits, int64_t ld, const int32_t *labels,
                      double *loss, double *dlogits, int64_t ldd)
{
    if (!logits || !labels || !loss || n < 1 || c < 1 || ld < c || (dlogits && ldd < c)) return ORACLE_EINVAL;
    double total = 0.0;
    for (int64_t v = 0; v < n; ++v) {
        const double *x = logits + v * ld;
        const int32_t y = labels[v];
        if (y < 0 || y >= c) return ORACLE_ERANGE;
        double m = x[0];
        for (int32_t j = 1; j < c; ++j) if (x[j] > m) m = x[j];
        double sum = 0.0;
        for (int32_t j = 0; j < c; ++j) sum += exp(x[j] - m);
        total += (m + log(sum)) - x[y];
        if (dlogits)
            for (int32_t j = 0; j < c; ++j)
                dlogits[v * ldd + j] = (exp(x[j] - m) / sum - (j == y ? 1.0 : 0.0)) / (double)n;
    }
    *loss = total / (double)n;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------
 * Optimiser of the paper's experiments: Adam with a cosine-annealed learning rate.
 * One Adam step on `count` parameters (Kingma & Ba, with bias correction), step t >= 1:
 *   g' = g + weight_decay * p;  m = b1 m + (1 - b1) g';  v = b2 v + (1 - b2) g'^2;
 *   p -= lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps).
 * ---------------------------------------------------------------------------------- */
int oracle_adam_step(double *p, const double *g, double *m, double *v, int64_t count, double lr,
                     double beta1, double beta2, double eps, double weight_decay, int32_t t)
{
    if (!p || !g || !m || !v || count < 0 || t < 1) return ORACLE_EINVAL;
    const double c1 = 1.0 - pow(beta1, (double)t), c2 = 1.0 - pow(beta2, (double)t);
    for (int64_t i = 0; i < count; ++i) {
        const double gi = g[i] + weight_decay * p[i];
        m[i] = beta1 * m[i] + (1.0 - beta1) * gi;
        v[i] = beta2 * v[i] + (1.0 - beta2) * gi * gi;
        p[i] -= lr * (m[i] / c1) / (sqrt(v[i] / c2) + eps);
    }
    return ORACLE_OK;
}

/* Cosine annealing: lr(t) = lr_min + (lr_max - lr_min) (1 + cos(pi t / t_max)) / 2 for epoch t in [0, t_max]. */
double oracle_cosine_lr(double lr_max, double lr_min, int32_t t, int32_t t_max)
{
    const double pi = 3.14159265358979323846;
    return lr_min + 0.5 * (lr_max - lr_min) * (1.0 + cos(pi * (double)t / (double)t_max));
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Threads the row loops may use from now on (timing the oracle on one core); no arithmetic depends on it:
 * every output element is summed by one thread in a fixed order. */
void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    extern void omp_set_num_threads(int);
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
