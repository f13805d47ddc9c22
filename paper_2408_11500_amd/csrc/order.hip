// Optional row processing order of a graph handle (locality preprocessing; inputs and outputs of every
// call stay in the caller's numbering, only the order in which the aggregation kernels visit the rows
// changes, so that rows visited together share gathered rows in the L2s).
//   by degree    : rows by descending number of stored entries, ties by ascending id;
//   breadth first: up to BFS_MAX_TREES times the first not yet placed row of the degree order becomes a
//                  root and the rows reachable from it are placed in first-in-first-out order, the
//                  neighbours of a row in ascending id; what is left follows in degree order.
// The breadth-first order is computed level by level: every row of the current level offers its position
// to its unplaced neighbours (atomicMin on an integer key), a neighbour's key ends up as the position of
// its earliest parent, and the next level is the newly reached rows sorted by (parent position, id) --
// exactly the order in which a sequential queue would have appended them.  Integer work only; the
// atomics are integer minima and counters, so the result does not depend on timing.
#include "common.h"

#include <rocprim/rocprim.hpp>

namespace slicegcn {

namespace {

constexpr int TPB = 256;
constexpr int BFS_MAX_TREES = 16;
inline unsigned blocks_for(int64_t n) { return (unsigned)((n + TPB - 1) / TPB); }

struct Buf { // frees on scope exit
    void *p = nullptr;
    ~Buf() { if (p) (void)hipFree(p); }
    int alloc(size_t bytes)
    {
        hipError_t e = hipMalloc(&p, bytes ? bytes : 1);
        if (e != hipSuccess) {
            p = nullptr;
            set_error("hipMalloc of %zu bytes failed: %s", bytes, hipGetErrorString(e));
            return e == hipErrorOutOfMemory ? SLICEGCN_ENOMEM : SLICEGCN_EHIP;
        }
        return SLICEGCN_OK;
    }
    template <class T> T *as() const { return static_cast<T *>(p); }
};

// key = (INT32_MAX - degree) << 32 | id: ascending keys = descending degree, ties by ascending id
__global__ void degree_keys_kernel(const int32_t *__restrict__ rowptr, int64_t n, uint64_t *__restrict__ keys)
{
    const int64_t v = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (v >= n) return;
    const uint32_t d = (uint32_t)(rowptr[v + 1] - rowptr[v]);
    keys[v] = ((uint64_t)(0x7fffffffu - d) << 32) | (uint64_t)v;
}

__global__ void low_words_kernel(const uint64_t *__restrict__ keys, int64_t count, int32_t *__restrict__ out)
{
    const int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (i < count) out[i] = (int32_t)(keys[i] & 0xffffffffu);
}

__global__ void fill_i32_kernel(int32_t *__restrict__ a, int64_t count, int32_t value)
{
    const int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (i < count) a[i] = value;
}

// smallest index i >= from with pos[by_deg[i]] < 0 (n if none): atomicMin over the candidates
__global__ void first_unplaced_kernel(const int32_t *__restrict__ by_deg, const int32_t *__restrict__ pos, int64_t n,
                                      int64_t from, int32_t *__restrict__ result)
{
    const int64_t i = from + (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (i < n && pos[by_deg[i]] < 0) atomicMin(result, (int32_t)i);
}

__global__ void place_root_kernel(const int32_t *__restrict__ by_deg, const int32_t *__restrict__ cursor, int32_t at,
                                  int32_t *__restrict__ order, int32_t *__restrict__ pos)
{
    const int32_t v = by_deg[*cursor];
    order[at] = v;
    pos[v] = at;
}

// One wavefront per row of the current level order[beg, end): every unplaced neighbour u gets
// key[u] = min(key[u], position of this row); the first row to reach u appends it to the candidate list.
__global__ __launch_bounds__(256) void expand_kernel(const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
                                                     const int32_t *__restrict__ order, int32_t beg, int32_t end,
                                                     const int32_t *__restrict__ pos, int32_t *__restrict__ key,
                                                     int32_t *__restrict__ cand, int32_t *__restrict__ n_cand)
{
    const int64_t w = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (beg + w >= end) return;
    const int32_t p = beg + (int32_t)w;
    const int32_t v = order[p];
    for (int32_t e = rowptr[v] + lane; e < rowptr[v + 1]; e += 64) {
        const int32_t u = colidx[e];
        if (pos[u] >= 0) continue;
        const int32_t old = atomicMin(&key[u], p);
        if (old == INT32_MAX) cand[atomicAdd(n_cand, 1)] = u;
    }
}

__global__ void cand_keys_kernel(const int32_t *__restrict__ cand, int32_t count, const int32_t *__restrict__ key,
                                 uint64_t *__restrict__ keys)
{
    const int i = blockIdx.x * TPB + threadIdx.x;
    if (i >= count) return;
    const int32_t u = cand[i];
    keys[i] = ((uint64_t)(uint32_t)key[u] << 32) | (uint64_t)(uint32_t)u;
}

// order[at + i] = id of the i-th sorted key; pos of that row = at + i
__global__ void place_level_kernel(const uint64_t *__restrict__ sorted, int32_t count, int32_t at,
                                   int32_t *__restrict__ order, int32_t *__restrict__ pos)
{
    const int i = blockIdx.x * TPB + threadIdx.x;
    if (i >= count) return;
    const int32_t u = (int32_t)(sorted[i] & 0xffffffffu);
    order[at + i] = u;
    pos[u] = at + i;
}

// rows still unplaced, in degree order: flag, scan, scatter
__global__ void unplaced_flag_kernel(const int32_t *__restrict__ by_deg, const int32_t *__restrict__ pos, int64_t n,
                                     int32_t *__restrict__ flag)
{
    const int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (i < n) flag[i] = pos[by_deg[i]] < 0 ? 1 : 0;
}

__global__ void unplaced_scatter_kernel(const int32_t *__restrict__ by_deg, const int32_t *__restrict__ flag,
                                        const int32_t *__restrict__ offs, int64_t n, int32_t at, int32_t *__restrict__ order)
{
    const int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (i < n && flag[i]) order[at + offs[i]] = by_deg[i];
}

int sort_u64(const uint64_t *in, uint64_t *out, int64_t count, unsigned end_bit, hipStream_t stream)
{
    size_t bytes = 0;
    SG_HIP(rocprim::radix_sort_keys(nullptr, bytes, in, out, (size_t)count, 0u, end_bit, stream));
    Buf tmp;
    if (int rc = tmp.alloc(bytes)) return rc;
    SG_HIP(rocprim::radix_sort_keys(tmp.p, bytes, in, out, (size_t)count, 0u, end_bit, stream));
    SG_HIP(hipStreamSynchronize(stream)); // tmp is freed on return
    return SLICEGCN_OK;
}

} // namespace

// order[p] = id of the row at position p (device array of n entries, owned by the caller on success)
int build_row_order(int64_t n, const int32_t *rowptr, const int32_t *colidx, bool breadth_first, int32_t **out, hipStream_t stream)
{
    *out = nullptr;
    Buf keys_a, keys_b, by_deg, order;
    if (int rc = keys_a.alloc((size_t)n * sizeof(uint64_t))) return rc;
    if (int rc = keys_b.alloc((size_t)n * sizeof(uint64_t))) return rc;
    if (int rc = by_deg.alloc((size_t)n * sizeof(int32_t))) return rc;
    degree_keys_kernel<<<blocks_for(n), TPB, 0, stream>>>(rowptr, n, keys_a.as<uint64_t>());
    SG_LAUNCH_CHECK();
    if (int rc = sort_u64(keys_a.as<uint64_t>(), keys_b.as<uint64_t>(), n, 64, stream)) return rc;
    low_words_kernel<<<blocks_for(n), TPB, 0, stream>>>(keys_b.as<uint64_t>(), n, by_deg.as<int32_t>());
    SG_LAUNCH_CHECK();
    if (!breadth_first) {
        SG_HIP(hipStreamSynchronize(stream));
        *out = by_deg.as<int32_t>();
        by_deg.p = nullptr;
        return SLICEGCN_OK;
    }

    Buf pos, key, cand, counters;
    if (int rc = order.alloc((size_t)n * sizeof(int32_t))) return rc;
    if (int rc = pos.alloc((size_t)n * sizeof(int32_t))) return rc;
    if (int rc = key.alloc((size_t)n * sizeof(int32_t))) return rc;
    if (int rc = cand.alloc((size_t)n * sizeof(int32_t))) return rc;
    if (int rc = counters.alloc(2 * sizeof(int32_t))) return rc;
    int32_t *d_cursor = counters.as<int32_t>(), *d_ncand = counters.as<int32_t>() + 1;
    fill_i32_kernel<<<blocks_for(n), TPB, 0, stream>>>(pos.as<int32_t>(), n, -1);
    fill_i32_kernel<<<blocks_for(n), TPB, 0, stream>>>(key.as<int32_t>(), n, INT32_MAX);
    SG_LAUNCH_CHECK();
    unsigned pos_bits = 1;
    while (((uint64_t)n >> pos_bits) != 0) ++pos_bits;

    int64_t placed = 0, cursor = 0;
    for (int tree = 0; tree < BFS_MAX_TREES && placed < n; ++tree) {
        // root: the first unplaced row of the degree order at or after the cursor
        fill_i32_kernel<<<1, TPB, 0, stream>>>(d_cursor, 1, (int32_t)n);
        first_unplaced_kernel<<<blocks_for(n - cursor), TPB, 0, stream>>>(by_deg.as<int32_t>(), pos.as<int32_t>(), n, cursor, d_cursor);
        SG_LAUNCH_CHECK();
        int32_t h_cursor = 0;
        SG_HIP(hipMemcpyAsync(&h_cursor, d_cursor, sizeof(int32_t), hipMemcpyDeviceToHost, stream));
        SG_HIP(hipStreamSynchronize(stream));
        if (h_cursor >= n) break;
        cursor = h_cursor;
        place_root_kernel<<<1, 1, 0, stream>>>(by_deg.as<int32_t>(), d_cursor, (int32_t)placed, order.as<int32_t>(), pos.as<int32_t>());
        SG_LAUNCH_CHECK();
        int64_t beg = placed, end = placed + 1;
        placed = end;
        while (beg < end) { // one level per turn
            fill_i32_kernel<<<1, TPB, 0, stream>>>(d_ncand, 1, 0);
            const int64_t threads = (end - beg) * 64;
            expand_kernel<<<(unsigned)((threads + 255) / 256), 256, 0, stream>>>(rowptr, colidx, order.as<int32_t>(), (int32_t)beg,
                                                                                 (int32_t)end, pos.as<int32_t>(), key.as<int32_t>(),
                                                                                 cand.as<int32_t>(), d_ncand);
            SG_LAUNCH_CHECK();
            int32_t h_ncand = 0;
            SG_HIP(hipMemcpyAsync(&h_ncand, d_ncand, sizeof(int32_t), hipMemcpyDeviceToHost, stream));
            SG_HIP(hipStreamSynchronize(stream));
            if (h_ncand == 0) break;
            SG_REQUIRE(placed + h_ncand <= n, SLICEGCN_EHIP, "row order: more rows reached than exist");
            cand_keys_kernel<<<blocks_for(h_ncand), TPB, 0, stream>>>(cand.as<int32_t>(), h_ncand, key.as<int32_t>(), keys_a.as<uint64_t>());
            SG_LAUNCH_CHECK();
            if (int rc = sort_u64(keys_a.as<uint64_t>(), keys_b.as<uint64_t>(), h_ncand, 32 + pos_bits, stream)) return rc;
            place_level_kernel<<<blocks_for(h_ncand), TPB, 0, stream>>>(keys_b.as<uint64_t>(), h_ncand, (int32_t)placed,
                                                                        order.as<int32_t>(), pos.as<int32_t>());
            SG_LAUNCH_CHECK();
            beg = end;
            end = placed + h_ncand;
            placed = end;
        }
    }
    if (placed < n) { // the rest in degree order
        int32_t *flag = key.as<int32_t>(), *offs = cand.as<int32_t>(); // both free now
        unplaced_flag_kernel<<<blocks_for(n), TPB, 0, stream>>>(by_deg.as<int32_t>(), pos.as<int32_t>(), n, flag);
        SG_LAUNCH_CHECK();
        size_t bytes = 0;
        SG_HIP(rocprim::exclusive_scan(nullptr, bytes, flag, offs, (int32_t)0, (size_t)n, rocprim::plus<int32_t>(), stream));
        Buf tmp;
        if (int rc = tmp.alloc(bytes)) return rc;
        SG_HIP(rocprim::exclusive_scan(tmp.p, bytes, flag, offs, (int32_t)0, (size_t)n, rocprim::plus<int32_t>(), stream));
        unplaced_scatter_kernel<<<blocks_for(n), TPB, 0, stream>>>(by_deg.as<int32_t>(), flag, offs, n, (int32_t)placed, order.as<int32_t>());
        SG_LAUNCH_CHECK();
        SG_HIP(hipStreamSynchronize(stream));
    }
    SG_HIP(hipStreamSynchronize(stream));
    *out = order.as<int32_t>();
    order.p = nullptr;
    return SLICEGCN_OK;
}

} // namespace slicegcn
