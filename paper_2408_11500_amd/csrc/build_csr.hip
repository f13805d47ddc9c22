// Normalised-adjacency builder: edge pairs -> canonical CSR of A^ = D~^-1/2 (A + I) D~^-1/2
// (the normalisation 1/c_vu of the paper's GCN layer equation), plus the row schedule the
// aggregation kernels use.  Integer work only, apart from one rsqrt per node and one multiply
// per stored entry.  Sorting, scanning and duplicate removal use rocPRIM device primitives on
// 64-bit keys (row << 32 | col); everything else is a small kernel below.
#include "common.h"

#include <rocprim/rocprim.hpp>

#include <cstdarg>
#include <cstdlib>
#include <new>
#include <vector>

namespace slicegcn {

namespace {

struct DevBuf { // frees on scope exit; release() hands the pointer over
    void *p = nullptr;
    ~DevBuf() { if (p) (void)hipFree(p); }
    int alloc(size_t bytes) {
        hipError_t e = hipMalloc(&p, bytes ? bytes : 1);
        if (e != hipSuccess) {
            p = nullptr;
            set_error("hipMalloc of %zu bytes failed: %s", bytes, hipGetErrorString(e));
            return e == hipErrorOutOfMemory ? SLICEGCN_ENOMEM : SLICEGCN_EHIP;
        }
        return SLICEGCN_OK;
    }
    template <class T> T *as() const { return static_cast<T *>(p); }
    template <class T> T *release() { T *r = static_cast<T *>(p); p = nullptr; return r; }
};

constexpr int TPB = 256;
inline unsigned blocks_for(int64_t n) { return (unsigned)((n + TPB - 1) / TPB); }

// One key per directed candidate entry.  Self pairs and out-of-range pairs become the
// sentinel key (row n), which sorts behind every real row and is dropped later.
__global__ void make_keys_kernel(const int64_t *__restrict__ src, const int64_t *__restrict__ dst,
                                 int64_t n_edges, int64_t n, int sym, int loops,
                                 uint64_t *__restrict__ keys, int *__restrict__ n_bad)
{
    const int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    const uint64_t sentinel = (uint64_t)n << 32;
    if (i < n_edges) {
        const int64_t u = src[i], v = dst[i];
        uint64_t k1 = sentinel, k2 = sentinel;
        if (u < 0 || u >= n || v < 0 || v >= n) {
            atomicAdd(n_bad, 1);
        } else if (u != v) {
            k1 = ((uint64_t)u << 32) | (uint64_t)v;
            k2 = ((uint64_t)v << 32) | (uint64_t)u;
        }
        keys[i] = k1;
        if (sym) keys[n_edges + i] = k2;
    } else if (loops && i < n_edges + n) {
        const uint64_t v = (uint64_t)(i - n_edges);
        keys[(sym ? 2 : 1) * n_edges + (int64_t)v] = (v << 32) | v;
    }
}

// rowptr[r] = number of keys with row < r = lower bound of (r << 32) in the sorted keys.
__global__ void rowptr_kernel(const uint64_t *__restrict__ keys, int64_t nnz, int64_t n,
                              int32_t *__restrict__ rowptr)
{
    const int64_t r = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (r > n) return;
    const uint64_t target = (uint64_t)r << 32;
    int64_t lo = 0, hi = nnz;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (keys[mid] < target) lo = mid + 1; else hi = mid;
    }
    rowptr[r] = (int32_t)lo;
}

__global__ void degree_kernel(const int32_t *__restrict__ rowptr, int64_t n,
                              int32_t *__restrict__ deg, float *__restrict__ dinv, float *__restrict__ sqrtd)
{
    const int64_t v = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (v >= n) return;
    const int32_t d = rowptr[v + 1] - rowptr[v];
    deg[v] = d;
    dinv[v] = (float)(1.0 / sqrt((double)(d > 0 ? d : 1)));
    sqrtd[v] = (float)sqrt((double)(d > 0 ? d : 1));
}

__global__ void entries_kernel(const uint64_t *__restrict__ keys, int64_t nnz,
                               const float *__restrict__ dinv,
                               int32_t *__restrict__ colidx, float *__restrict__ vals)
{
    const int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (i >= nnz) return;
    const uint64_t k = keys[i];
    const uint32_t row = (uint32_t)(k >> 32), col = (uint32_t)(k & 0xffffffffu);
    colidx[i] = (int32_t)col;
    vals[i] = dinv[row] * dinv[col];
}

__global__ void swap_keys_kernel(const uint64_t *__restrict__ in, int64_t nnz, uint64_t *__restrict__ out)
{
    const int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (i >= nnz) return;
    const uint64_t k = in[i];
    out[i] = (k << 32) | (k >> 32);
}

// ---- schedule ---------------------------------------------------------------------------
// Column class c holds the columns [first[c], first[c+1]); the boundaries are the 1/n_classes
// quantiles of the stored entries per column, so that the classes carry equal numbers of entries
// whatever the vertex numbering (with hubs numbered first, equal column ranges would put almost
// half of the entries into the first class).
struct ClassBounds {
    int32_t first[MAX_CLASSES + 1];
};

// colptr: row pointer of the transposed pattern (entries per column, scanned)
__global__ void class_bounds_kernel(const int32_t *__restrict__ colptr, int64_t n, int n_classes, int32_t *__restrict__ first)
{
    const int c = threadIdx.x;
    if (c > MAX_CLASSES) return;
    if (c == 0) { first[0] = 0; return; }
    if (c >= n_classes) { first[c] = (int32_t)n; return; }
    const int64_t target = (int64_t)colptr[n] * c / n_classes;
    int64_t lo = 0, hi = n; // smallest column j with colptr[j] >= target
    while (lo < hi) {
        const int64_t mid = lo + ((hi - lo) >> 1);
        if (colptr[mid] < target) lo = mid + 1; else hi = mid;
    }
    first[c] = (int32_t)lo;
}

// Item tables: 2c = wavefront items of class c (pieces of rows cut by column class), 2c + 1 =
// lane-group items of class c, 2 * n_classes = wavefront items of rows kept whole, 2 * n_classes + 1
// = lane-group items that are whole rows.  counts layout: cnt[table * (n+1) + row].
constexpr int MAX_TABLES = 2 * MAX_CLASSES + 2;
struct RowCut {
    int32_t lo[MAX_CLASSES + 1];
};

// Per long row: the entries of column class c are [lower_bound(first[c]), lower_bound(first[c+1])).
__device__ inline RowCut cut_row(const int32_t *__restrict__ colidx, int32_t beg, int32_t end, int n_classes, const ClassBounds &cb)
{
    RowCut rc;
    rc.lo[0] = beg;
    for (int c = 1; c < n_classes; ++c) {
        const int32_t target = cb.first[c];
        int32_t lo = rc.lo[c - 1], hi = end;
        while (lo < hi) {
            const int32_t mid = lo + ((hi - lo) >> 1);
            if (colidx[mid] < target) lo = mid + 1; else hi = mid;
        }
        rc.lo[c] = lo;
    }
    for (int c = n_classes; c <= MAX_CLASSES; ++c) rc.lo[c] = end;
    return rc;
}

__device__ inline int pieces_of(int32_t len) { return (len + SEG_NNZ - 1) / SEG_NNZ; }

// The items of one row, in (class, piece) order.  F is called as f(table, beg, end).
template <class F>
__device__ inline int for_each_item(const int32_t *__restrict__ colidx, int32_t beg, int32_t end,
                                    int n_classes, const ClassBounds &cb, int32_t part_row, int32_t item_max, F f)
{
    const int32_t d = end - beg;
    int total = 0;
    if (d <= TINY_ROW) return 0;
    if (d <= item_max) {
        f(2 * n_classes + 1, beg, end);
        return 1;
    }
    if (n_classes == 1 || d <= part_row) {
        const int s = pieces_of(d);
        const int32_t piece = (d + s - 1) / s; // equal cuts, the last one takes the remainder
        for (int j = 0; j < s; ++j) f(2 * n_classes, beg + j * piece, min(end, beg + (j + 1) * piece));
        return s;
    }
    const RowCut rc = cut_row(colidx, beg, end, n_classes, cb);
    for (int c = 0; c < n_classes; ++c) {
        const int32_t b = rc.lo[c], e = rc.lo[c + 1], len = e - b;
        if (len <= 0) continue;
        if (len <= item_max) {
            f(2 * c + 1, b, e);
            ++total;
        } else {
            const int s = pieces_of(len);
            const int32_t piece = (len + s - 1) / s;
            for (int j = 0; j < s; ++j) f(2 * c, b + j * piece, min(e, b + (j + 1) * piece));
            total += s;
        }
    }
    return total;
}

// Thread p handles the row at position p of the schedule (order[p], or p itself in natural order); all
// per-row tables are indexed by position, so the scans below lay the items out in schedule order.
__global__ void sched_count_kernel(const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx, int64_t n,
                                   const int32_t *__restrict__ order,
                                   int n_classes, const ClassBounds cb, int32_t part_row, int32_t item_max, int32_t *__restrict__ cnt,
                                   int32_t *__restrict__ c_slot, int32_t *__restrict__ c_fix)
{
    const int64_t p = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (p > n) return;
    const int64_t stride = n + 1;
    int32_t per[MAX_TABLES];
    for (int t = 0; t < MAX_TABLES; ++t) per[t] = 0;
    int total = 0;
    if (p < n) {
        const int64_t r = order ? order[p] : p;
        total = for_each_item(colidx, rowptr[r], rowptr[r + 1], n_classes, cb, part_row, item_max,
                              [&](int t, int32_t, int32_t) { per[t] += 1; });
    }
    for (int t = 0; t < 2 * n_classes + 2; ++t) cnt[t * stride + p] = per[t];
    c_slot[p] = total > 1 ? total : 0;
    c_fix[p] = total > 1 ? 1 : 0;
}

__global__ void sched_fill_kernel(const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx, int64_t n,
                                  const int32_t *__restrict__ order,
                                  int n_classes, const ClassBounds cb, int32_t part_row, int32_t item_max, const int32_t *__restrict__ off,
                                  const int32_t *__restrict__ o_slot, const int32_t *__restrict__ o_fix,
                                  Segment *__restrict__ items, FixRow *__restrict__ fix)
{
    const int64_t p = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (p >= n) return;
    const int64_t r = order ? order[p] : p;
    const int64_t stride = n + 1;
    const int32_t beg = rowptr[r], end = rowptr[r + 1];
    if (end - beg <= TINY_ROW) return;
    // first pass: how many items (decides whether they write the row or partial slots)
    const int total = for_each_item(colidx, beg, end, n_classes, cb, part_row, item_max, [](int, int32_t, int32_t) {});
    int32_t used[MAX_TABLES];
    for (int t = 0; t < MAX_TABLES; ++t) used[t] = 0;
    int slot = o_slot[p]; // slots are handed out in (class, piece) order
    for_each_item(colidx, beg, end, n_classes, cb, part_row, item_max, [&](int t, int32_t b, int32_t e) {
        Segment sg;
        sg.row = (int32_t)r;
        sg.beg = b;
        sg.end = e;
        sg.dst = total == 1 ? (int32_t)r : -(slot + 1);
        items[off[t * stride + p] + used[t]] = sg;
        used[t] += 1;
        ++slot;
    });
    if (total > 1) {
        FixRow f;
        f.row = (int32_t)r;
        f.slot_beg = o_slot[p];
        f.slot_end = o_slot[p] + total;
        f.pad = 0;
        fix[o_fix[p]] = f;
    }
}

int scan_i32(const int32_t *in, int32_t *out, int64_t count, hipStream_t stream)
{
    size_t bytes = 0;
    SG_HIP(rocprim::exclusive_scan(nullptr, bytes, in, out, (int32_t)0, (size_t)count, rocprim::plus<int32_t>(), stream));
    DevBuf tmp;
    if (int rc = tmp.alloc(bytes)) return rc;
    SG_HIP(rocprim::exclusive_scan(tmp.p, bytes, in, out, (int32_t)0, (size_t)count, rocprim::plus<int32_t>(), stream));
    SG_HIP(hipStreamSynchronize(stream));
    return SLICEGCN_OK;
}

int sort_keys(const uint64_t *in, uint64_t *out, int64_t count, unsigned end_bit, hipStream_t stream)
{
    size_t bytes = 0;
    SG_HIP(rocprim::radix_sort_keys(nullptr, bytes, in, out, (size_t)count, 0u, end_bit, stream));
    DevBuf tmp;
    if (int rc = tmp.alloc(bytes)) return rc;
    SG_HIP(rocprim::radix_sort_keys(tmp.p, bytes, in, out, (size_t)count, 0u, end_bit, stream));
    SG_HIP(hipStreamSynchronize(stream));
    return SLICEGCN_OK;
}

// rowptr / colidx / vals of the pattern whose sorted distinct keys are given
int pattern_from_keys(const uint64_t *keys, int64_t nnz, int64_t n, const float *dinv, Csr &m, hipStream_t stream)
{
    DevBuf col, val;
    if (int rc = col.alloc((size_t)nnz * sizeof(int32_t))) return rc;
    if (int rc = val.alloc((size_t)nnz * sizeof(float))) return rc;
    if (nnz > 0) {
        entries_kernel<<<blocks_for(nnz), TPB, 0, stream>>>(keys, nnz, dinv, col.as<int32_t>(), val.as<float>());
        SG_LAUNCH_CHECK();
    }
    m.colidx = col.release<int32_t>();
    m.vals = val.release<float>();
    return SLICEGCN_OK;
}

} // namespace

static void free_schedule(Schedule &sc)
{
    (void)hipFree(sc.items);
    (void)hipFree(sc.fix);
    sc = Schedule();
}

void free_csr(Csr &m, bool owns_pattern)
{
    if (owns_pattern) {
        (void)hipFree(m.rowptr);
        (void)hipFree(m.colidx);
        (void)hipFree(m.vals);
    }
    free_schedule(m.wide);
    free_schedule(m.xcd);
    m = Csr();
}

int build_schedule(int64_t n, int64_t nnz, const Csr &m, const int32_t *colptr, const int32_t *order, int n_classes, uint32_t flags,
                   Schedule &out, hipStream_t stream)
{
    out = Schedule();
    out.n_classes = n_classes;
    // entries (8 bytes each) plus one 128-byte operand row per node against the 256 MB last-level cache
    const bool resident = nnz * 8 + n * 128 <= ((int64_t)256 << 20);
    int32_t item_max = resident ? ITEM_SHORT : ITEM_LONG;
    if (flags & SLICEGCN_SCHED_SHORT_ITEMS) item_max = ITEM_SHORT;
    if (flags & SLICEGCN_SCHED_LONG_ITEMS) item_max = ITEM_LONG;
    out.item_max = item_max;
    const int n_tables = 2 * n_classes + 2;
    const size_t stride = (size_t)(n + 1);
    const size_t n_cnt = (size_t)n_tables * stride;
    SG_REQUIRE(n_cnt <= (size_t)INT32_MAX, SLICEGCN_ERANGE, "build_norm_csr: schedule tables exceed int32 indexing");
    DevBuf cnt, off, aux;
    if (int rc = cnt.alloc(n_cnt * sizeof(int32_t))) return rc;
    if (int rc = off.alloc(n_cnt * sizeof(int32_t))) return rc;
    if (int rc = aux.alloc((4 * stride + 16) * sizeof(int32_t))) return rc; // slot counts, fix counts, their scans, class bounds
    int32_t *c = cnt.as<int32_t>(), *o = off.as<int32_t>(), *x = aux.as<int32_t>();
    ClassBounds cb;
    class_bounds_kernel<<<1, 64, 0, stream>>>(colptr, n, n_classes, x + 4 * stride);
    SG_LAUNCH_CHECK();
    SG_HIP(hipMemcpyAsync(cb.first, x + 4 * stride, sizeof(cb.first), hipMemcpyDeviceToHost, stream));
    SG_HIP(hipStreamSynchronize(stream));
    const int32_t part_row = PART_ROW;
    sched_count_kernel<<<blocks_for(n + 1), TPB, 0, stream>>>(m.rowptr, m.colidx, n, order, n_classes, cb, part_row, item_max, c, x, x + stride);
    SG_LAUNCH_CHECK();
    if (int rc = scan_i32(c, o, (int64_t)n_cnt, stream)) return rc;
    if (int rc = scan_i32(x, x + 2 * stride, n + 1, stream)) return rc;
    if (int rc = scan_i32(x + stride, x + 3 * stride, n + 1, stream)) return rc;
    // the scan runs over all tables back to back: table t starts at o[t * stride]
    std::vector<int32_t> starts(n_tables + 1);
    for (int t = 0; t < n_tables; ++t)
        SG_HIP(hipMemcpy(&starts[t], o + (size_t)t * stride, sizeof(int32_t), hipMemcpyDeviceToHost));
    int32_t last_off = 0, last_cnt = 0, n_slots = 0, n_fix = 0;
    SG_HIP(hipMemcpy(&last_off, o + n_cnt - 1, sizeof(int32_t), hipMemcpyDeviceToHost));
    SG_HIP(hipMemcpy(&last_cnt, c + n_cnt - 1, sizeof(int32_t), hipMemcpyDeviceToHost));
    SG_HIP(hipMemcpy(&n_slots, x + 2 * stride + n, sizeof(int32_t), hipMemcpyDeviceToHost));
    SG_HIP(hipMemcpy(&n_fix, x + 3 * stride + n, sizeof(int32_t), hipMemcpyDeviceToHost));
    starts[n_tables] = last_off + last_cnt;
    for (int cl = 0; cl < n_classes; ++cl) {
        out.big_off[cl] = starts[2 * cl];
        out.big_cnt[cl] = starts[2 * cl + 1] - starts[2 * cl];
        out.small_off[cl] = starts[2 * cl + 1];
        out.small_cnt[cl] = starts[2 * cl + 2] - starts[2 * cl + 1];
    }
    out.wbig_off = starts[2 * n_classes];
    out.wbig_cnt = starts[2 * n_classes + 1] - starts[2 * n_classes];
    out.wsmall_off = starts[2 * n_classes + 1];
    out.wsmall_cnt = starts[2 * n_classes + 2] - starts[2 * n_classes + 1];
    out.n_items = starts[n_tables];
    out.n_slots = n_slots;
    out.n_fix = n_fix;
    DevBuf items, fix;
    if (int rc = items.alloc((size_t)out.n_items * sizeof(Segment))) return rc;
    if (int rc = fix.alloc((size_t)out.n_fix * sizeof(FixRow))) return rc;
    sched_fill_kernel<<<blocks_for(n), TPB, 0, stream>>>(m.rowptr, m.colidx, n, order, n_classes, cb, part_row, item_max, o, x + 2 * stride,
                                                         x + 3 * stride, items.as<Segment>(), fix.as<FixRow>());
    SG_LAUNCH_CHECK();
    SG_HIP(hipStreamSynchronize(stream));
    out.items = items.release<Segment>();
    out.fix = fix.release<FixRow>();
    static const bool verbose = getenv("SLICEGCN_VERBOSE") != nullptr;
    if (verbose) {
        fprintf(stderr, "[slicegcn] schedule with %d class(es): whole rows %d wavefront + %d lane-group items, %lld rows with "
                        "several items, %lld partial-sum slots\n", n_classes, out.wbig_cnt, out.wsmall_cnt,
                (long long)out.n_fix, (long long)out.n_slots);
        for (int cl = 0; cl < n_classes && n_classes > 1; ++cl)
            fprintf(stderr, "[slicegcn]   class %d: columns [%d, %d), %d wavefront + %d lane-group pieces\n", cl,
                    cb.first[cl], cb.first[cl + 1], out.big_cnt[cl], out.small_cnt[cl]);
    }
    return SLICEGCN_OK;
}

// colptr: row pointer of the transposed pattern
static int build_schedules(int64_t n, int64_t nnz, Csr &m, const int32_t *colptr, const int32_t *order, uint32_t flags, hipStream_t stream)
{
    if (int rc = build_schedule(n, nnz, m, colptr, order, 1, flags, m.wide, stream)) return rc;
    return build_schedule(n, nnz, m, colptr, order, MAX_CLASSES, flags, m.xcd, stream);
}

} // namespace slicegcn

using namespace slicegcn;

extern "C" int slicegcn_build_norm_csr(const int64_t *src, const int64_t *dst, int64_t n_edges,
                                       int64_t n_nodes, uint32_t flags, void *stream_, slicegcn_graph **out)
{
    SG_REQUIRE(out != nullptr, SLICEGCN_EINVAL, "build_norm_csr: out is NULL");
    *out = nullptr;
    SG_REQUIRE(n_nodes >= 1, SLICEGCN_EINVAL, "build_norm_csr: n_nodes = %lld < 1", (long long)n_nodes);
    SG_REQUIRE(n_edges >= 0, SLICEGCN_EINVAL, "build_norm_csr: n_edges = %lld < 0", (long long)n_edges);
    SG_REQUIRE(n_edges == 0 || (src && dst), SLICEGCN_EINVAL, "build_norm_csr: NULL edge arrays");
    SG_REQUIRE((flags & ~(SLICEGCN_SYMMETRIZE | SLICEGCN_ADD_SELF_LOOPS | SLICEGCN_REORDER_DEGREE | SLICEGCN_REORDER_BFS |
                          SLICEGCN_SCHED_SHORT_ITEMS | SLICEGCN_SCHED_LONG_ITEMS)) == 0,
               SLICEGCN_EINVAL, "build_norm_csr: unknown flag bits 0x%x", flags);
    SG_REQUIRE(!((flags & SLICEGCN_REORDER_DEGREE) && (flags & SLICEGCN_REORDER_BFS)), SLICEGCN_EINVAL,
               "build_norm_csr: REORDER_DEGREE and REORDER_BFS exclude each other");
    SG_REQUIRE(!((flags & SLICEGCN_SCHED_SHORT_ITEMS) && (flags & SLICEGCN_SCHED_LONG_ITEMS)), SLICEGCN_EINVAL,
               "build_norm_csr: SCHED_SHORT_ITEMS and SCHED_LONG_ITEMS exclude each other");
    SG_REQUIRE(n_nodes <= INT32_MAX, SLICEGCN_ERANGE, "build_norm_csr: n_nodes exceeds int32");
    const int sym = (flags & SLICEGCN_SYMMETRIZE) != 0, loops = (flags & SLICEGCN_ADD_SELF_LOOPS) != 0;
    SG_REQUIRE(n_edges <= (int64_t)INT32_MAX, SLICEGCN_ERANGE, "build_norm_csr: n_edges exceeds int32");
    const int64_t n_keys = n_edges * (sym ? 2 : 1) + (loops ? n_nodes : 0);
    SG_REQUIRE(n_keys <= (int64_t)INT32_MAX, SLICEGCN_ERANGE,
               "build_norm_csr: %lld candidate entries exceed int32 indexing", (long long)n_keys);
    hipStream_t stream = as_stream(stream_);

    slicegcn_graph *g = new (std::nothrow) slicegcn_graph();
    SG_REQUIRE(g != nullptr, SLICEGCN_ENOMEM, "build_norm_csr: host allocation failed");
    struct Guard { // destroys the half-built handle on any early return
        slicegcn_graph *g;
        ~Guard() { if (g) slicegcn_graph_destroy(g); }
    } guard{g};
    g->n = n_nodes;
    g->symmetric = sym;
    SG_HIP(hipGetDevice(&g->device));

    DevBuf keys_a, keys_b, counters;
    if (int rc = keys_a.alloc((size_t)n_keys * sizeof(uint64_t))) return rc;
    if (int rc = keys_b.alloc((size_t)n_keys * sizeof(uint64_t))) return rc;
    if (int rc = counters.alloc(64)) return rc;
    SG_HIP(hipMemsetAsync(counters.p, 0, 64, stream));
    int *d_bad = counters.as<int>();
    size_t *d_count = reinterpret_cast<size_t *>(counters.as<char>() + 16);

    int64_t nnz = 0;
    if (n_keys > 0) {
        make_keys_kernel<<<blocks_for(n_edges + (loops ? n_nodes : 0)), TPB, 0, stream>>>(
            src, dst, n_edges, n_nodes, sym, loops, keys_a.as<uint64_t>(), d_bad);
        SG_LAUNCH_CHECK();
        int h_bad = 0;
        SG_HIP(hipMemcpyAsync(&h_bad, d_bad, sizeof(int), hipMemcpyDeviceToHost, stream));
        SG_HIP(hipStreamSynchronize(stream));
        SG_REQUIRE(h_bad == 0, SLICEGCN_ERANGE, "build_norm_csr: %d edge(s) name a node outside [0, %lld)", h_bad,
                   (long long)n_nodes);

        unsigned row_bits = 1;
        while (((uint64_t)n_nodes >> row_bits) != 0) ++row_bits; // bits needed for the value n_nodes (sentinel row)
        if (int rc = sort_keys(keys_a.as<uint64_t>(), keys_b.as<uint64_t>(), n_keys, 32 + row_bits, stream)) return rc;

        size_t bytes = 0;
        SG_HIP(rocprim::unique(nullptr, bytes, keys_b.as<uint64_t>(), keys_a.as<uint64_t>(), d_count, (size_t)n_keys,
                               rocprim::equal_to<uint64_t>(), stream));
        {
            DevBuf tmp;
            if (int rc = tmp.alloc(bytes)) return rc;
            SG_HIP(rocprim::unique(tmp.p, bytes, keys_b.as<uint64_t>(), keys_a.as<uint64_t>(), d_count, (size_t)n_keys,
                                   rocprim::equal_to<uint64_t>(), stream));
            SG_HIP(hipStreamSynchronize(stream));
        }
        size_t h_count = 0;
        SG_HIP(hipMemcpy(&h_count, d_count, sizeof(size_t), hipMemcpyDeviceToHost));
        nnz = (int64_t)h_count;
        if (nnz > 0) { // drop the sentinel (it is the largest key, so the last distinct one)
            uint64_t last = 0;
            SG_HIP(hipMemcpy(&last, keys_a.as<uint64_t>() + (nnz - 1), sizeof(uint64_t), hipMemcpyDeviceToHost));
            if ((last >> 32) == (uint64_t)n_nodes) --nnz;
        }
    }
    g->nnz = nnz;
    const uint64_t *uniq = keys_a.as<uint64_t>(); // sorted distinct keys [0, nnz)

    {
        DevBuf rowptr, deg, dinv, sqrtd;
        if (int rc = rowptr.alloc((size_t)(n_nodes + 1) * sizeof(int32_t))) return rc;
        if (int rc = deg.alloc((size_t)n_nodes * sizeof(int32_t))) return rc;
        if (int rc = dinv.alloc((size_t)n_nodes * sizeof(float))) return rc;
        if (int rc = sqrtd.alloc((size_t)n_nodes * sizeof(float))) return rc;
        rowptr_kernel<<<blocks_for(n_nodes + 1), TPB, 0, stream>>>(uniq, nnz, n_nodes, rowptr.as<int32_t>());
        SG_LAUNCH_CHECK();
        degree_kernel<<<blocks_for(n_nodes), TPB, 0, stream>>>(rowptr.as<int32_t>(), n_nodes, deg.as<int32_t>(),
                                                              dinv.as<float>(), sqrtd.as<float>());
        SG_LAUNCH_CHECK();
        g->fwd.rowptr = rowptr.release<int32_t>();
        g->deg = deg.release<int32_t>();
        g->dinv = dinv.release<float>();
        g->sqrtd = sqrtd.release<float>();
    }
    if (int rc = pattern_from_keys(uniq, nnz, n_nodes, g->dinv, g->fwd, stream)) return rc;

    if (flags & (SLICEGCN_REORDER_DEGREE | SLICEGCN_REORDER_BFS))
        if (int rc = build_row_order(n_nodes, g->fwd.rowptr, g->fwd.colidx, (flags & SLICEGCN_REORDER_BFS) != 0, &g->order, stream)) return rc;

    if (sym) {
        if (int rc = build_schedules(n_nodes, nnz, g->fwd, g->fwd.rowptr, g->order, flags, stream)) return rc;
        g->tr = g->fwd; // A^ is symmetric: the same arrays serve the transposed product
    } else {
        uint64_t *swapped = keys_b.as<uint64_t>();
        if (nnz > 0) {
            swap_keys_kernel<<<blocks_for(nnz), TPB, 0, stream>>>(uniq, nnz, swapped);
            SG_LAUNCH_CHECK();
        }
        DevBuf keys_c;
        if (int rc = keys_c.alloc((size_t)(nnz > 0 ? nnz : 1) * sizeof(uint64_t))) return rc;
        unsigned row_bits = 1;
        while (((uint64_t)n_nodes >> row_bits) != 0) ++row_bits;
        if (nnz > 0)
            if (int rc = sort_keys(swapped, keys_c.as<uint64_t>(), nnz, 32 + row_bits, stream)) return rc;
        DevBuf rowptr;
        if (int rc = rowptr.alloc((size_t)(n_nodes + 1) * sizeof(int32_t))) return rc;
        rowptr_kernel<<<blocks_for(n_nodes + 1), TPB, 0, stream>>>(keys_c.as<uint64_t>(), nnz, n_nodes, rowptr.as<int32_t>());
        SG_LAUNCH_CHECK();
        g->tr.rowptr = rowptr.release<int32_t>();
        if (int rc = pattern_from_keys(keys_c.as<uint64_t>(), nnz, n_nodes, g->dinv, g->tr, stream)) return rc;
        if (int rc = build_schedules(n_nodes, nnz, g->fwd, g->tr.rowptr, g->order, flags, stream)) return rc;
        if (int rc = build_schedules(n_nodes, nnz, g->tr, g->fwd.rowptr, g->order, flags, stream)) return rc;
        SG_HIP(hipStreamSynchronize(stream));
    }

    SG_HIP(hipStreamSynchronize(stream));
    guard.g = nullptr;
    *out = g;
    return SLICEGCN_OK;
}

extern "C" int slicegcn_graph_view(const slicegcn_graph *g, slicegcn_csr_view *view)
{
    SG_REQUIRE(g && view, SLICEGCN_EINVAL, "graph_view: NULL argument");
    view->n_nodes = g->n;
    view->nnz = g->nnz;
    view->rowptr = g->fwd.rowptr;
    view->colidx = g->fwd.colidx;
    view->deg = g->deg;
    view->dinv = g->dinv;
    view->vals = g->fwd.vals;
    view->symmetric = g->symmetric;
    view->order = g->order;
    return SLICEGCN_OK;
}

extern "C" int slicegcn_graph_destroy(slicegcn_graph *g)
{
    if (!g) return SLICEGCN_OK;
    if (!g->symmetric) free_csr(g->tr, true);
    free_csr(g->fwd, true);
    (void)hipFree(g->deg);
    (void)hipFree(g->dinv);
    (void)hipFree(g->sqrtd);
    (void)hipFree(g->order);
    delete g;
    return SLICEGCN_OK;
}
