// Internal declarations shared by the translation units of libslicegcn (not installed).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstring>

#include "slicegcn.h"

namespace slicegcn {

// ---- error plumbing ------------------------------------------------------------------
void set_error(const char *fmt, ...) __attribute__((format(printf, 1, 2)));

#define SG_REQUIRE(cond, code, ...)        \
    do {                                   \
        if (!(cond)) {                     \
            ::slicegcn::set_error(__VA_ARGS__); \
            return (code);                 \
        }                                  \
    } while (0)

#define SG_HIP(call)                                                                       \
    do {                                                                                   \
        hipError_t sg_e_ = (call);                                                         \
        if (sg_e_ != hipSuccess) {                                                         \
            ::slicegcn::set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(sg_e_), \
                                  __FILE__, __LINE__);                                     \
            return sg_e_ == hipErrorOutOfMemory ? SLICEGCN_ENOMEM : SLICEGCN_EHIP;         \
        }                                                                                  \
    } while (0)

#define SG_LAUNCH_CHECK() SG_HIP(hipGetLastError())

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }
inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }
__host__ __device__ inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---- aggregation schedule -------------------------------------------------------------
// Rows are split by their number of stored entries d:
//   d <= TINY_ROW            : handled whole, 64 consecutive rows per wavefront, in natural order;
//   TINY_ROW < d <= item_max : one lane-group item (the whole row);
//   d > item_max             : wavefront items of at most SEG_NNZ entries;
//   d > PART_ROW (schedules with 8 classes only): the row is first cut by column class
//       (8 contiguous column ranges holding equal shares of the stored entries; a row's entries of
//       one class are contiguous because columns ascend); a class piece of at most item_max
//       entries is a lane-group item, a longer one is cut into wavefront items.
// item_max is fixed per graph: ITEM_SHORT when the whole working set stays in the last-level cache
// (the kernels are then bound by instruction issue, and shorter lane-group items win), ITEM_LONG when
// the gathers go to memory (fewer, longer items keep more gathers in flight).
// Pieces of class c are executed by workgroups whose index is c modulo n_classes; with 8 classes
// and the round-robin placement of workgroups over the 8 XCDs, each XCD's L2 only ever sees its
// own class of columns of the gathered operand for the partitioned rows.  Whole-row items form
// two lists of their own (wavefront and lane-group items, in row order) that are dealt to the
// classes in fixed-size chunks, round-robin, and run behind the class's pieces.  A row with
// several items gets one partial-sum slot per item (in a workspace the caller of the aggregation
// provides) and is finished by a fix-up pass that adds the slots in order.
constexpr int TINY_ROW = 4;
constexpr int ITEM_SHORT = 32;
constexpr int ITEM_LONG = 64;
constexpr int PART_ROW = 256;
constexpr int SEG_NNZ = 2048;
constexpr int MAX_CLASSES = 8;
constexpr int WIDE_SLOT_COLS = 256; // floats per slot, single-class schedule (256 columns per pass)
constexpr int XCD_SLOT_COLS = 128;  // floats per slot, 8-class schedule (128 columns per pass)

struct Segment { // 16 bytes, read as one int4
    int32_t row;
    int32_t beg;
    int32_t end;
    int32_t dst; // >= 0: final (write the row); < 0: partial slot index -(dst+1)
};

struct FixRow { // a row whose items went to partial slots [slot_beg, slot_end)
    int32_t row;
    int32_t slot_beg;
    int32_t slot_end;
    int32_t pad;
};

struct Schedule {
    int32_t n_classes = 0;
    int32_t item_max = ITEM_LONG; // longest lane-group item (whole row or class piece)
    Segment *items = nullptr; // per class its wavefront pieces, then its lane-group pieces; then the whole-row lists
    FixRow *fix = nullptr;
    int32_t big_off[MAX_CLASSES] = {0}, big_cnt[MAX_CLASSES] = {0};     // wavefront pieces of class c
    int32_t small_off[MAX_CLASSES] = {0}, small_cnt[MAX_CLASSES] = {0}; // lane-group pieces of class c
    int32_t wbig_off = 0, wbig_cnt = 0;     // wavefront items of rows kept whole
    int32_t wsmall_off = 0, wsmall_cnt = 0; // lane-group items that are whole rows
    int64_t n_items = 0;
    int64_t n_fix = 0;
    int64_t n_slots = 0;
};

struct Csr {
    int32_t *rowptr = nullptr;
    int32_t *colidx = nullptr;
    float *vals = nullptr;
    Schedule wide; // one class: rows cut by length only
    Schedule xcd;  // eight column classes
};

} // namespace slicegcn

struct slicegcn_graph {
    int64_t n = 0;
    int64_t nnz = 0;
    int symmetric = 0;
    int device = 0;
    int32_t *deg = nullptr;
    float *dinv = nullptr;
    float *sqrtd = nullptr; // sqrt(max(d~_v, 1)) = 1 / dinv: undoes the row scaling of activations kept as D~^-1/2 H
    int32_t *order = nullptr; // order[p] = row at position p of the aggregation's schedule; NULL = natural order
    slicegcn::Csr fwd;  // A^
    slicegcn::Csr tr;   // A^^T (arrays alias fwd when the pattern is symmetric)
};

namespace slicegcn {

// spmm.hip: Y[:, 0:width] = M X (+ Add), M given by `m`.  Add may alias Y.  ws: 256-byte aligned, at least
// spmm_workspace_bytes(m, width) bytes (partial sums of rows cut into several items; may be NULL when that is 0).
int launch_spmm(const slicegcn_graph *g, const Csr &m, const float *X, int64_t ldx, int32_t width,
                float *Y, int64_t ldy, const float *Add, int64_t ldadd, void *ws, size_t ws_bytes, hipStream_t stream,
                bool prescaled = false); // prescaled: X rows carry dinv[u] already (the value stream is not read)
size_t spmm_workspace_bytes(const Csr &m, int32_t width);

// dense.hip: column sums of an n x w matrix: fp32 per block of rows into ws[blocks][w], then
// out[j] = sum over blocks of ws[b][first + j] in fp64 (ws_row = floats per ws row)
int launch_colsum_partial(const float *M, int64_t ld, int64_t n, int32_t w, float *ws, hipStream_t stream);
int launch_colsum_final(const float *ws_first, int64_t n, int32_t ws_row, int32_t count, float *out, hipStream_t stream);
size_t colsum_workspace_bytes(int64_t n, int32_t w);

// misc.hip: brackets the launches of its scope with an event pair while profiling is on
struct ProfScope {
    ProfScope(int kind, int width, hipStream_t stream);
    ~ProfScope();
    ProfScope(const ProfScope &) = delete;
    ProfScope &operator=(const ProfScope &) = delete;
    int slot_;
    hipStream_t stream_;
};

// build_csr.hip
int build_schedule(int64_t n, int64_t nnz, const Csr &m, const int32_t *colptr, const int32_t *order, int n_classes, uint32_t flags,
                   Schedule &out, hipStream_t stream);

// order.hip: order[p] = id of the row at position p (by degree, or breadth first); *out is a device array the caller frees
int build_row_order(int64_t n, const int32_t *rowptr, const int32_t *colidx, bool breadth_first, int32_t **out, hipStream_t stream);
void free_csr(Csr &m, bool owns_pattern);

} // namespace slicegcn
