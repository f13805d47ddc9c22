/*
 * slicegcn.h -- C ABI of the MI355X (gfx950) SliceGCN hot path.
 *
 * The library evaluates, for one feature slice at a time, the full-graph layer of the
 * SliceGCN model (arXiv 2408.11500): sparse aggregation with the symmetric-normalised
 * adjacency held as CSR over the whole graph, the dense slice transform with bias, ReLU and
 * self term, the backward pass of both, and slice encoding + concatenation of the slice
 * outputs.  Every step runs in hand-written HIP kernels; nothing falls back to the CPU.
 *
 * General conventions
 *  - Every function returns an int status: SLICEGCN_OK (0) or a negative SLICEGCN_E* code.
 *    No exception or abort crosses this boundary.  slicegcn_last_error() returns a
 *    thread-local text for the most recent failure in the calling thread.
 *  - Unless marked HOST, array pointers are DEVICE pointers on the current HIP device.
 *  - Matrices are fp32, row-major, with an explicit leading dimension counted in elements
 *    (ld >= width), so column slices and concatenation targets are plain views.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Device calls
 *    are asynchronous with respect to the host and ordered on that stream, except
 *    slicegcn_build_norm_csr, which synchronises the stream before returning.
 *  - Ownership: the caller owns every tensor, workspace and edge-list buffer.  The library
 *    owns only what a slicegcn_graph handle holds (the CSR arrays and the row schedule derived
 *    from them), from slicegcn_build_norm_csr until slicegcn_graph_destroy.  Apart from
 *    building a graph, no call allocates or frees device memory.
 *  - A handle is read-only after it has been built: any number of calls may use one handle at
 *    the same time from different streams or host threads, as long as each call has its own
 *    workspace and output buffers.  Workspaces (`ws`, `ws_bytes`) are scratch: 256-byte aligned,
 *    at least the size the matching *_workspace_bytes query returns, contents undefined before
 *    and after a call; `ws` may be NULL when that size is 0.  Two calls that share a workspace
 *    must be ordered on one stream.
 *  - Results are deterministic: kernels use no floating-point atomics, so two calls on the
 *    same inputs give bitwise equal outputs.
 */
#ifndef SLICEGCN_H
#define SLICEGCN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SLICEGCN_OK 0
#define SLICEGCN_EINVAL (-1)       /* NULL / misaligned / inconsistent argument            */
#define SLICEGCN_ERANGE (-2)       /* node id outside [0, n_nodes) or a count beyond int32  */
#define SLICEGCN_ENOMEM (-3)       /* device or host allocation failed                      */
#define SLICEGCN_EHIP (-4)         /* a HIP runtime call failed (text in last_error)        */
#define SLICEGCN_EUNSUPPORTED (-5) /* valid request this build does not implement           */
#define SLICEGCN_EWORKSPACE (-6)   /* workspace pointer NULL or smaller than required       */

/* flags of slicegcn_build_norm_csr */
#define SLICEGCN_SYMMETRIZE 1u     /* store A | A^T (undirected graph)                      */
#define SLICEGCN_ADD_SELF_LOOPS 2u /* add exactly one diagonal entry per row (A + I)        */
/* Locality preprocessing (optional; the paper fixes no execution order): the aggregation visits the rows
 * in the order below instead of by ascending id, so that rows visited together gather the same rows and
 * find them in cache.  Inputs and outputs of every call stay in the caller's numbering, the CSR arrays of
 * slicegcn_graph_view are unchanged, and results differ from the natural order by rounding at most (the
 * sum of a row is formed in the same order).  The chosen order is slicegcn_csr_view.order.
 *   REORDER_DEGREE: rows by descending number of stored entries, ties by ascending id.
 *   REORDER_BFS   : at most 16 times, the not yet placed row that comes first in the degree order becomes a
 *                   root, and the rows reachable from it (along stored entries of A^) are placed in the order a
 *                   first-in-first-out queue visits them, the neighbours of a row in ascending id; rows
 *                   still unplaced follow in degree order.  Graphs whose vertices were numbered without
 *                   regard to their communities gain from this; a random graph does not. */
#define SLICEGCN_REORDER_DEGREE 4u
#define SLICEGCN_REORDER_BFS 8u
/* schedule tuning (optional, results are unaffected): by default rows of up to 32 stored entries are
 * served by 8-lane groups when the whole graph stays in the last-level cache and rows of up to 64
 * otherwise; these two flags force one of the limits */
#define SLICEGCN_SCHED_SHORT_ITEMS 16u
#define SLICEGCN_SCHED_LONG_ITEMS 32u

/* activation of slicegcn_layer_desc.act */
#define SLICEGCN_ACT_NONE 0
#define SLICEGCN_ACT_RELU 1

typedef struct slicegcn_graph slicegcn_graph; /* opaque; owns the CSR arrays on the device */

/* Borrowed device pointers into a graph handle; valid until the handle is destroyed. */
typedef struct {
    int64_t n_nodes;
    int64_t nnz;
    const int32_t *rowptr; /* [n_nodes + 1]                                   */
    const int32_t *colidx; /* [nnz], strictly ascending within each row       */
    const int32_t *deg;    /* [n_nodes] stored entries per row (d~_v)         */
    const float *dinv;     /* [n_nodes] 1/sqrt(max(d~_v, 1))                  */
    const float *vals;     /* [nnz] dinv[row] * dinv[col]                     */
    int32_t symmetric;     /* 1 when the pattern was symmetrised              */
    const int32_t *order;  /* [n_nodes] row visited at each position, or NULL (ascending id) */
} slicegcn_csr_view;

/* flags of slicegcn_layer_desc.flags */
#define SLICEGCN_LAYER_Z_VALID 1u /* forward only: saved->Z already holds A^ Hin, skip the aggregation */
/* Order of the two products of the layer equation's aggregation term.  (A^ Hin) W_agg and A^ (Hin W_agg) are equal
 * in exact arithmetic (results differ by rounding only); the default aggregates first, as the layer is stated.
 * TRANSFORM_FIRST multiplies by W_agg first, so the aggregation gathers rows of w_out instead of w_in columns, in
 * the forward and in the backward pass; ORDER_AUTO picks it when w_out < w_in.  The transform-first order keeps
 * nothing but the activation mask for the backward pass (saved->Z is neither written nor read and may be NULL),
 * and its backward pass always runs one aggregation (of dP, w_out wide), where the default order runs one of
 * w_in columns only when dHin is wanted.  Pass the same flags to slicegcn_layer_fwd, slicegcn_layer_bwd and the
 * workspace queries of a layer. */
#define SLICEGCN_LAYER_TRANSFORM_FIRST 2u
#define SLICEGCN_LAYER_ORDER_AUTO 4u
/* Scaled layout of activations (aggregate-first order only).  1/c_vu factors as dinv[v] dinv[u], so an
 * activation kept as H' = D~^-1/2 H (row v times dinv[v]) is aggregated without reading the 4-byte value of every
 * stored entry (SLICEGCN_SPMM_PRESCALED).  IN_SCALED: Hin holds D~^-1/2 times the layer's input (the self term
 * and its weight gradient multiply the rows back by sqrt(d~_v)).  OUT_SCALED: Hout receives D~^-1/2 times the
 * layer's output, ready to be the next layer's IN_SCALED input.  Gradients (dHout, dHin) are always those of the
 * unscaled activations, and saved->Z is always the unscaled A^ Hin.  A stack of layers scales its constant input
 * once (slicegcn_scale_rows), sets IN_SCALED on every layer and OUT_SCALED on all but the last. */
#define SLICEGCN_LAYER_IN_SCALED 8u
#define SLICEGCN_LAYER_OUT_SCALED 16u

typedef struct {
    int32_t w_in;   /* width of the layer input  (columns of Hin, rows of W)    */
    int32_t w_out;  /* width of the layer output (columns of Hout, cols of W)   */
    int32_t act;    /* SLICEGCN_ACT_*                                           */
    uint32_t flags; /* SLICEGCN_LAYER_* or 0                                    */
} slicegcn_layer_desc;

/* Parameters of one layer of one slice.  W_* are row-major w_in x w_out, contiguous
 * (leading dimension w_out).  b, W_self, b_self may be NULL (term absent). */
typedef struct {
    const float *W_agg;
    const float *b;      /* [w_out] bias inside the activation                  */
    const float *W_self;
    const float *b_self; /* [w_out] bias of the self term, outside the activation */
} slicegcn_layer_params;

/* What the forward pass keeps for the backward pass (caller-owned buffers).
 * Z    : n x w_in aggregation result A^ Hin, leading dimension ldz (>= w_in, multiple of 4,
 *        16-byte aligned base).  It doubles as the staging buffer of the forward aggregation, so it is
 *        required in the default (aggregate-first) order; there is no "recompute in backward" mode.  Unused
 *        (may be NULL) in the transform-first order.
 * mask : n x mask_words uint32; bit (j % 32) of word (j / 32) of row v is 1 where the
 *        pre-activation P[v, j] > 0.  mask_words >= ceil(w_out / 32).  For ACT_NONE the
 *        mask is neither written nor read and may be NULL. */
typedef struct {
    float *Z;
    int64_t ldz;
    uint32_t *mask;
    int64_t mask_words;
} slicegcn_layer_saved;

/* Gradient outputs of one layer, same shapes as the parameters; NULL entries are skipped. */
typedef struct {
    float *dW_agg;
    float *db;
    float *dW_self;
    float *db_self;
} slicegcn_layer_grads;

/* ---------------------------------------------------------------------------------------
 * Slice strategy (HOST only).  Algorithm "Slice Strategy Generation" of the paper, equal to
 * its closed-form start/end equation when slice_size_scale = 1:
 *   slice_size = ceil(in_d / p); slice i = [i*slice_size, i*slice_size + int(slice_size*scale));
 *   a slice that would pass in_d is shifted left to end at in_d (so it may overlap).
 * starts/ends: HOST arrays of p entries (0-based, half-open).  slice_size: HOST scalar out.
 * EINVAL: NULL output, p < 1, p > in_d, scale <= 0 or int(slice_size*scale) outside [1, in_d].
 * ------------------------------------------------------------------------------------- */
int slicegcn_slice_strategy(int32_t in_d, int32_t p, double slice_size_scale,
                            int32_t *starts, int32_t *ends, int32_t *slice_size);

/* ---------------------------------------------------------------------------------------
 * Normalised adjacency.  From n_edges pairs (src[e], dst[e]) (DEVICE int64 arrays, any order,
 * repeats and self pairs allowed) builds A~ = A (| A^T) (+ I) as a 0/1 pattern -- the paper's
 * binary adjacency matrix with every node counted among its own neighbours -- and the
 * normalisation 1/c_vu = 1/(sqrt(d~_v) sqrt(d~_u)) of the paper's GCN layer equation, with
 * d~_v the number of stored entries of row v.  Input self pairs are dropped and repeats
 * collapsed, so the diagonal is exactly 1 entry when ADD_SELF_LOOPS is set.
 * On success *out holds a new handle (free it with slicegcn_graph_destroy).  Allocates device
 * memory (the handle's arrays plus temporaries of a few times the edge list, freed before it
 * returns) and synchronises `stream` several times: it runs once per graph, not per epoch.
 * Sorting, duplicate removal and prefix sums are rocPRIM device primitives; the kernels around
 * them are this library's.  rowptr/colidx/deg are exact integers; dinv/vals are fp32 and always
 * kept (there is no flag to drop vals: every aggregation path reads them).
 * EINVAL: NULL out, n_nodes < 1, n_edges < 0, NULL src/dst with n_edges > 0, unknown flag, both
 *         REORDER flags or both SCHED flags.
 * ERANGE: n_nodes > 2^31-1, more than 2^31-1 stored entries, or a node id outside [0, n_nodes).
 * ------------------------------------------------------------------------------------- */
int slicegcn_build_norm_csr(const int64_t *src, const int64_t *dst, int64_t n_edges,
                            int64_t n_nodes, uint32_t flags, void *stream, slicegcn_graph **out);
int slicegcn_graph_view(const slicegcn_graph *g, slicegcn_csr_view *view /* HOST struct out */);
int slicegcn_graph_destroy(slicegcn_graph *g); /* NULL is accepted */

/* ---------------------------------------------------------------------------------------
 * Direct feature slicing: Xs = X[:, start:end] (the paper's direct-slicing equation and its
 * "Feature Slicing" algorithm, without the device copy).  X: n x (>= end) with leading
 * dimension ldx; Xs: n x ldxs, ldxs >= end - start.  Columns [end-start, ldxs) of Xs are
 * written as zeros, so a padded slice can be read with vector loads.
 * EINVAL: NULL pointer, n < 1, start < 0, start >= end, end > ldx, ldxs < end - start.
 * ------------------------------------------------------------------------------------- */
int slicegcn_slice_feature(const float *X, int64_t n, int64_t ldx, int32_t start, int32_t end,
                           float *Xs, int64_t ldxs, void *stream);

/* ---------------------------------------------------------------------------------------
 * Slice aggregation, the inner sum of the SliceGCN layer equation:
 *   Y[v, 0:width] = sum over stored (v,u) of vals_vu * X[u, 0:width]       (op = 0)
 *   Y = A^^T X                                                              (op & SLICEGCN_SPMM_TRANSPOSE)
 * With SLICEGCN_SPMM_PRESCALED the caller passes X' = D~^-1/2 X (every row u already multiplied by dinv[u],
 * e.g. by slicegcn_scale_rows; worthwhile when X is constant or its producer can scale it for free) and the
 * call forms dinv[v] * sum of X'[u, :] instead: the same Y up to rounding, without reading the 4-byte value
 * of every stored entry (1/c_vu factors as dinv[v] dinv[u]).
 * X, Y: n_nodes x width with leading dimensions ldx, ldy.  X and Y must not overlap.
 * The fast path needs X 16-byte aligned with ldx a multiple of 4 and ldx >= width rounded up
 * to 4 (padding columns are read but never used); other layouts take a scalar path.  Only
 * columns [0, width) of Y are written.  A symmetrised graph serves transpose != 0 with the
 * same arrays; otherwise the handle holds the transposed pattern as well.
 * ws: rows cut into several work items (long rows, see the schedule notes of the library) keep
 * per-item partial sums there; slicegcn_spmm_workspace_bytes gives the size for this graph,
 * direction and width (0 for graphs without such rows).
 * EINVAL: NULL pointer, width < 1, ldx < width, ldy < width, misaligned ws;
 * EWORKSPACE: ws NULL or too small.
 * ------------------------------------------------------------------------------------- */
#define SLICEGCN_SPMM_TRANSPOSE 1
#define SLICEGCN_SPMM_PRESCALED 2
size_t slicegcn_spmm_workspace_bytes(const slicegcn_graph *g, int op, int32_t width);
int slicegcn_spmm_slice(const slicegcn_graph *g, int op, const float *X, int64_t ldx,
                        int32_t width, float *Y, int64_t ldy, void *ws, size_t ws_bytes, void *stream);

/* Xs[u, 0:width] = dinv[u] * X[u, 0:width] (n_nodes rows; columns [width, ldxs) of Xs are written as zeros):
 * the operand form SLICEGCN_SPMM_PRESCALED and SLICEGCN_LAYER_IN_SCALED expect.  Xs may be X itself (in place,
 * same leading dimension).  EINVAL: NULL pointer, width < 1, ld < width. */
int slicegcn_scale_rows(const slicegcn_graph *g, const float *X, int64_t ldx, int32_t width,
                        float *Xs, int64_t ldxs, void *stream);

/* ---------------------------------------------------------------------------------------
 * The same aggregation for callers that cannot allocate device memory and have no workspace to pass
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the partial
 * sums go to a fixed SLICEGCN_STATIC_WS_BYTES buffer inside the library (one per GPU, held until the
 * process ends) and the call allocates nothing.  Results are bitwise those of slicegcn_spmm_slice.
 * Every call on one GPU shares that buffer, which keeps the last call's contents (nothing in it has to
 * start at zero: every slot is written before it is read): calls that may overlap on one GPU, from
 * several streams or threads, race -- order them on one stream or use slicegcn_spmm_slice.
 * EINVAL as slicegcn_spmm_slice; EWORKSPACE: slicegcn_spmm_workspace_bytes(g, op, width) exceeds
 * SLICEGCN_STATIC_WS_BYTES (graphs with very many long rows); EUNSUPPORTED: device index >= 64.
 * ------------------------------------------------------------------------------------- */
#define SLICEGCN_STATIC_WS_BYTES (16u << 20)
int slicegcn_spmm_slice_static(const slicegcn_graph *g, int op, const float *X, int64_t ldx,
                               int32_t width, float *Y, int64_t ldy, void *stream);

/* ---------------------------------------------------------------------------------------
 * One layer of one slice, forward (the SliceGCN layer equation as typeset, self term outside
 * the activation):
 *   Z = A^ Hin;  P = b + Z W_agg;  Hout = act(P) + Hin W_self + b_self.
 * Hin: n x w_in (ldi); Hout: n x w_out (ldo, any value >= w_out: the last layer can store
 * straight into its column block of the concatenated representation).  saved->Z is always
 * written (it is the staging buffer of the aggregation); saved->mask is written for ACT_RELU.
 * Hin must satisfy the fast-path layout of slicegcn_spmm_slice or the scalar path is taken.
 * With SLICEGCN_LAYER_Z_VALID the caller vouches that saved->Z still holds A^ Hin from an earlier
 * call with the same graph and Hin (the first layer over raw, constant features is the same in
 * every epoch); the aggregation is then skipped.  The paper's own implementation recomputes it.
 * ws: at least slicegcn_layer_fwd_workspace_bytes(g, desc) bytes (the aggregation's workspace; in the
 * transform-first order also the staged Hin W_agg and its aggregation).
 * EINVAL: NULL Hin/Hout/W_agg/saved->Z, widths < 1, ld too small, ldz not a multiple of 4,
 *         mask NULL or mask_words too small with ACT_RELU, unknown act or flag, misaligned ws;
 * EWORKSPACE: ws NULL or too small.
 * ------------------------------------------------------------------------------------- */
size_t slicegcn_layer_fwd_workspace_bytes(const slicegcn_graph *g, const slicegcn_layer_desc *desc);
int slicegcn_layer_fwd(const slicegcn_graph *g, const slicegcn_layer_desc *desc,
                       const slicegcn_layer_params *params, const float *Hin, int64_t ldi,
                       float *Hout, int64_t ldo, slicegcn_layer_saved *saved,
                       void *ws, size_t ws_bytes, void *stream);

/* Bytes of workspace slicegcn_layer_bwd needs for this graph and layer (0 on bad input).
 * need_dHin = 0 when the input gradient is not wanted (first layer over raw features). */
size_t slicegcn_layer_bwd_workspace_bytes(const slicegcn_graph *g, const slicegcn_layer_desc *desc, int need_dHin);

/* ---------------------------------------------------------------------------------------
 * One layer of one slice, backward (chain rule of the forward above; ReLU'(0) = 0):
 *   dP = dHout * mask;  db = colsum dP;  db_self = colsum dHout;
 *   dW_agg = Z^T dP;    dW_self = Hin^T dHout;
 *   dHin = A^^T (dP W_agg^T) + dHout W_self^T         (skipped when dHin == NULL).
 * saved holds Z and mask exactly as slicegcn_layer_fwd wrote them (read only here).
 * Reductions over the nodes run in fp32 over short row blocks and are combined in fp64 in a
 * fixed order.  ws: at least slicegcn_layer_bwd_workspace_bytes bytes (partial weight gradients,
 * the staged dZ = dP W_agg^T and the aggregation's workspace).  In the transform-first order the pass reads
 * G = A^^T dP instead of Z: dW_agg = Hin^T G, dHin = G W_agg^T + dHout W_self^T.
 * EINVAL as for the forward; EWORKSPACE when ws is NULL or ws_bytes too small.
 * ------------------------------------------------------------------------------------- */
int slicegcn_layer_bwd(const slicegcn_graph *g, const slicegcn_layer_desc *desc,
                       const slicegcn_layer_params *params, const float *Hin, int64_t ldi,
                       const slicegcn_layer_saved *saved, const float *dHout, int64_t ldo,
                       float *dHin, int64_t ldgi, slicegcn_layer_grads *grads,
                       void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------
 * Slice encoding + concatenation (the paper's slice-encoding and CONCAT equations):
 *   H[v, off_i + j] = Hs[i][v, j] + E[i, j],  off_i = widths[0] + ... + widths[i-1].
 * Hs: HOST array of k DEVICE pointers (n x widths[i], leading dimension lds[i]);
 * lds, widths: HOST arrays.  E: DEVICE k x lde matrix, or NULL for plain concatenation.
 * If Hs[i] already is the column block H + off_i with lds[i] == ldh, the slice is encoded in
 * place (no copy).  EINVAL: NULL pointer, k < 1, n < 1, width < 1, ld too small,
 * sum of widths > ldh, lde < max width.
 * ------------------------------------------------------------------------------------- */
int slicegcn_concat(int32_t k, const float *const *Hs, const int64_t *lds, const int32_t *widths,
                    const float *E, int64_t lde, int64_t n, float *H, int64_t ldh, void *stream);

size_t slicegcn_concat_bwd_workspace_bytes(int64_t n, int32_t k, const int32_t *widths /* HOST */);

/* Backward of the above: dHs[i] = dH[:, off_i : off_i + widths[i]] (copied only when dHs is
 * non-NULL and dHs[i] is non-NULL -- callers normally use the column view of dH instead) and
 * dE[i, j] = sum over nodes of dH[v, off_i + j] (skipped when dE == NULL; needs ws). */
int slicegcn_concat_bwd(int32_t k, const float *dH, int64_t ldh, int64_t n, const int32_t *widths,
                        float *const *dHs, const int64_t *lds, float *dE, int64_t lde,
                        void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------
 * Dense layer Y = act(X W + b): the unit the paper's classifier MLP_CLS (its classifier equation:
 * the concatenated representation goes through an MLP) and its feature-fusion network MLP_FF
 * (feature-fusion equation) are stacked from.
 * X: n x w_in (ldx); W: w_in x w_out row-major, contiguous; b: [w_out] or NULL; Y: n x w_out (ldy).
 * For ACT_RELU the pattern [X W + b > 0] is written to mask (n x mask_words uint32, bit layout as
 * in slicegcn_layer_saved); for ACT_NONE mask is ignored and may be NULL.  X and Y must not overlap.
 * EINVAL: NULL X/W/Y, sizes < 1, ld too small, unknown act, mask missing for ACT_RELU.
 * ------------------------------------------------------------------------------------- */
int slicegcn_linear_fwd(const float *X, int64_t ldx, int64_t n, int32_t w_in, int32_t w_out,
                        const float *W, const float *b, int32_t act, float *Y, int64_t ldy,
                        uint32_t *mask, int64_t mask_words, void *stream);

/* Bytes of workspace slicegcn_linear_bwd needs when dW or db is wanted (0 on bad input). */
size_t slicegcn_linear_bwd_workspace_bytes(int64_t n, int32_t w_in, int32_t w_out);

/* Backward of the dense layer (chain rule; ReLU'(0) = 0), with dP = dY * mask:
 *   dX = dP W^T (n x w_in, lddx);  dW = X^T dP (w_in x w_out);  db = colsum dP.
 * NULL outputs are skipped (dX = NULL for a first layer over constant inputs).  mask is what
 * slicegcn_linear_fwd wrote (read only; ignored for ACT_NONE).  The node-axis reductions run in
 * fp32 over blocks of 1024 rows and are combined in fp64 in a fixed order.  ws: 256-byte aligned,
 * at least slicegcn_linear_bwd_workspace_bytes bytes when dW or db is non-NULL, else unused.
 * EINVAL as for the forward; EWORKSPACE when ws is NULL or too small. */
int slicegcn_linear_bwd(const float *X, int64_t ldx, int64_t n, int32_t w_in, int32_t w_out,
                        const float *W, int32_t act, const uint32_t *mask, int64_t mask_words,
                        const float *dY, int64_t lddy, float *dX, int64_t lddx, float *dW, float *db,
                        void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------
 * dst[:, 0:w] += src[:, 0:w] (n rows).  With feature fusion (the paper's feature-fusion equation:
 * one learned projection feeds every slice model) the gradient of the fused features is the sum
 * of the k slice models' input gradients; this adds one of them.  dst and src must not overlap.
 * EINVAL: NULL pointer, sizes < 1, ld < w.
 * ------------------------------------------------------------------------------------- */
int slicegcn_accumulate(float *dst, int64_t ldd, const float *src, int64_t lds, int64_t n, int32_t w,
                        void *stream);

/* ---------------------------------------------------------------------------------------
 * Mean softmax cross-entropy over all n nodes and its gradient (the paper's loss equation with
 * every node labelled):
 *   *loss = -(1/n) sum_v log softmax(logits[v, :])[labels[v]]           (DEVICE float scalar)
 *   dlogits[v, j] = (softmax(logits[v, :])[j] - [j == labels[v]]) / n   (skipped when NULL)
 * logits: n x n_classes (ld); labels: DEVICE int32 [n] in [0, n_classes); dlogits may alias
 * logits only if ldd == ld (each row is fully read before it is written).  Row losses are added
 * in fp64 in a fixed order.  ws: 256-byte aligned, slicegcn_softmax_ce_workspace_bytes(n) bytes.
 * Asynchronous like every other device call, so a label outside [0, n_classes) cannot come back
 * as a status: it makes *loss NaN (the gradient rows of such nodes are unspecified).
 * EINVAL: NULL pointer, sizes < 1, ld < n_classes; EWORKSPACE: ws NULL or too small.
 * ------------------------------------------------------------------------------------- */
size_t slicegcn_softmax_ce_workspace_bytes(int64_t n);
int slicegcn_softmax_ce(const float *logits, int64_t ld, int64_t n, int32_t n_classes,
                        const int32_t *labels, float *loss, float *dlogits, int64_t ldd,
                        void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------
 * Optimiser of the paper's experiments (its experimental settings: Adam with cosine-annealed
 * learning rate).  One bias-corrected Adam step, step >= 1, on `count` contiguous fp32 parameters:
 *   g' = grad + weight_decay * param;  m = beta1 m + (1 - beta1) g';  v = beta2 v + (1 - beta2) g'^2;
 *   param -= lr * (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps).
 * param, m, v are updated in place (m and v start as zeros); the four arrays must not overlap.
 * Keeping all parameters of a model in one buffer makes this one launch per step.
 * EINVAL: NULL pointer, count < 1, step < 1, beta outside [0, 1), eps < 0.
 * ------------------------------------------------------------------------------------- */
int slicegcn_adam_step(float *param, const float *grad, float *m, float *v, int64_t count, double lr,
                       double beta1, double beta2, double eps, double weight_decay, int32_t step, void *stream);

/* HOST: cosine annealing, lr(t) = lr_min + (lr_max - lr_min) (1 + cos(pi t / t_max)) / 2 for
 * epoch t in [0, t_max]; returns lr_max when t_max < 1. */
double slicegcn_cosine_lr(double lr_max, double lr_min, int32_t t, int32_t t_max);

/* ---------------------------------------------------------------------------------------
 * Measurement aid (no part of the method): per-kernel timing with HIP events recorded on the
 * stream each kernel is launched on.  Between slicegcn_profile_begin and slicegcn_profile_end
 * every kernel group the library launches is bracketed by an event pair.  _end synchronises
 * the device, adds the elapsed times up by (kind, width) and writes at most `capacity` entries
 * to the HOST array `entries`; *count receives the number of distinct (kind, width) pairs.
 * Process-wide state; not meant to be used from several threads at once.
 * ------------------------------------------------------------------------------------- */
#define SLICEGCN_PROF_SPMM 0        /* aggregation pass (main kernel + fix-up); width = operand width */
#define SLICEGCN_PROF_DENSE_FWD 1   /* forward weight products + epilogue; width = w_out              */
#define SLICEGCN_PROF_DENSE_BWD 2   /* backward dZ / self products; width = w_in                      */
#define SLICEGCN_PROF_GRAD_REDUCE 3 /* weight-gradient reductions; width = w_out                      */
#define SLICEGCN_PROF_CONCAT 4      /* slice encoding / concat / their backward; width = slice width  */
#define SLICEGCN_PROF_SPMM_ADD 5    /* aggregation pass fused with an addend (backward); operand width */
#define SLICEGCN_PROF_LINEAR_FWD 6  /* dense layer forward; width = w_out                             */
#define SLICEGCN_PROF_LINEAR_BWD 7  /* dense layer input gradient; width = w_in                       */
#define SLICEGCN_PROF_LINEAR_GRAD 8 /* dense layer weight/bias gradients; width = w_out               */
#define SLICEGCN_PROF_LOSS 9        /* softmax cross-entropy; width = classes                         */
#define SLICEGCN_PROF_ACCUM 10      /* gradient accumulation over slices; width = w                   */
typedef struct {
    int32_t kind;
    int32_t width;
    int64_t launches;
    double total_ms;
    double min_ms; /* shortest and longest single launch group of this (kind, width) */
    double max_ms;
    double median_ms;
} slicegcn_profile_entry;
/* Creates the events of `scopes` kernel groups ahead of time, so that a profiled region that launches at
 * most that many groups creates none itself (events are reused from one profiled region to the next). */
int slicegcn_profile_reserve(int32_t scopes);
int slicegcn_profile_begin(void);
int slicegcn_profile_end(slicegcn_profile_entry *entries, int32_t capacity, int32_t *count);

const char *slicegcn_strerror(int status);
const char *slicegcn_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SLICEGCN_H */
