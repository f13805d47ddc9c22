// Slice aggregation Y = A^ X (+ Add): the neighbour sum of the SliceGCN layer equation.
//
// Work split (fixed per graph when it is built, see the schedule notes in common.h):
//   * rows of at most TINY_ROW stored entries: 64 consecutive rows per wavefront (8-lane groups,
//     narrow slices).  Lane i loads the row pointers and entries of row i; the gather phase
//     then hands row (t * GROUPS + grp) to lane group grp in sub-round t through cross-lane reads,
//     so one wavefront keeps many independent row gathers in flight and the output stream stays
//     contiguous;
//   * lane-group items (whole rows of up to item_max entries, short class pieces of partitioned
//     rows): one item per lane group at a time, its (column, value) pairs read LPR at a time by the
//     group's lanes and handed out by cross-lane reads, the next item's pairs requested before the
//     current item's gathers;
//   * wavefront items (everything longer, cut at SEG_NNZ entries): the wavefront loads 64
//     (column, value) pairs per coalesced read, the 64/LPR lane groups take them in turn through
//     cross-lane reads with eight gathers in flight per lane, and the groups' sums are combined
//     with cross-lane shuffles;
//   * a row with several items stores per-item partial sums that a fix-up kernel adds in item order.
// Workgroup b serves class b mod n_classes.  With 8 classes this pins each column class of the
// gathered operand to one XCD's L2 (workgroups are placed round-robin over the XCDs), so the
// eight L2s hold disjoint sets of hot rows instead of eight copies of the same set.  If the
// placement were different the result would be the same, only slower.
// No floating-point atomics anywhere: the summation order is a function of the graph only.
//
// Lanes map to columns: with vector width V (4 floats when the operand layout allows 16-byte
// loads, else 1), lane `sub` of a group owns columns [V*sub, V*sub + V) of the current column
// pass; wider operands take several passes.
//
// The partial sums of rows with several items live in a workspace the caller passes in (its size comes
// from spmm_workspace_bytes), so a graph handle is read-only here and calls on different streams
// only have to use different workspaces.
#include "common.h"

#include <mutex>

namespace slicegcn {

namespace {

struct SpmmArgs {
    const int32_t *rowptr;
    const int32_t *colidx;
    const float *vals;
    const Segment *items;
    const FixRow *fix;
    const int32_t *order; // row at every position of the schedule (NULL: natural order), for the short rows
    const float *X;
    float *Y;
    const float *Add;
    const float *dinv;    // factored form only: X rows come pre-scaled by dinv[u], sums are scaled by dinv[row] on store
    float *scratch;
    int64_t ldx, ldy, ldadd;
    uint32_t ldx_bytes;   // S32 kernels: byte stride of X rows (n * ldx * 4 < 2^32, n and ldx * 4 < 2^24)
    int32_t n;
    int32_t n_classes;
    int32_t item_max;     // longest lane-group item of the schedule (ITEM_SHORT or ITEM_LONG)
    int32_t ipw;          // wavefront items per wavefront (one-launch kernel: 4; otherwise 1); a workgroup takes 4 * ipw
    int32_t big_blocks;   // workgroups per class in the wavefront-item section
    int32_t small_blocks; // workgroups per class in the lane-group-item section
    int32_t slot_cols;    // floats per partial-sum slot
    int32_t col0;         // first column of this pass
    int32_t col_end;      // one past the last column of this pass (<= width)
    int32_t vec_store;    // Y (and Add) allow 16-byte accesses
    int32_t big_off[MAX_CLASSES], big_cnt[MAX_CLASSES];     // wavefront pieces of class c
    int32_t small_off[MAX_CLASSES], small_cnt[MAX_CLASSES]; // lane-group pieces of class c
    int32_t wbig_off, wbig_cnt;     // wavefront items of rows kept whole (dealt to the classes four at a time)
    int32_t wsmall_off, wsmall_cnt; // lane-group whole rows (dealt one wavefront's share at a time)
};

template <int V> struct Acc;
template <> struct Acc<4> {
    float4 v;
    __device__ Acc() : v(make_float4(0.f, 0.f, 0.f, 0.f)) {}
    __device__ void fma(float a, const float4 &x) { v.x += a * x.x; v.y += a * x.y; v.z += a * x.z; v.w += a * x.w; }
    __device__ void plus(const float4 &x) { v.x += x.x; v.y += x.y; v.z += x.z; v.w += x.w; }
    __device__ void scale(float a) { v.x *= a; v.y *= a; v.z *= a; v.w *= a; }
    __device__ void add(const Acc &o) { v.x += o.v.x; v.y += o.v.y; v.z += o.v.z; v.w += o.v.w; }
    __device__ float get(int i) const { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }
};
template <> struct Acc<1> {
    float v;
    __device__ Acc() : v(0.f) {}
    __device__ void fma(float a, float x) { v += a * x; }
    __device__ void plus(float x) { v += x; }
    __device__ void scale(float a) { v *= a; }
    __device__ void add(const Acc &o) { v += o.v; }
    __device__ float get(int) const { return v; }
};

template <int V> struct Ld;
template <> struct Ld<4> {
    using T = float4;
    static __device__ T zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
    static __device__ T load(const float *p) { return *reinterpret_cast<const float4 *>(p); }
};
template <> struct Ld<1> {
    using T = float;
    static __device__ T zero() { return 0.f; }
    static __device__ T load(const float *p) { return *p; }
};

// Address of columns [col, col + V) of row c of the gathered operand.  S32: the whole operand lies
// within 4 GiB of its base and both factors fit 24 bits, so one 24-bit multiply-add gives an
// unsigned 32-bit byte offset from the (wavefront-uniform) base pointer.
template <int V, bool S32>
__device__ inline typename Ld<V>::T load_x(const SpmmArgs &a, int c, int col)
{
    if (S32) {
        const uint32_t off = __umul24((uint32_t)c, a.ldx_bytes) + (uint32_t)col * 4u;
        return Ld<V>::load(reinterpret_cast<const float *>(reinterpret_cast<const char *>(a.X) + off));
    }
    return Ld<V>::load(a.X + (int64_t)c * a.ldx + col);
}

// Factored form (FACT): the operand rows already carry dinv[u], so every stored entry weighs 1 (the value stream is
// not read, its cross-lane reads vanish and the multiply-adds fold to adds) and the row sum is scaled by dinv[row] on store.
template <bool FACT> __device__ inline float ld_val(const SpmmArgs &a, int idx) { return FACT ? 1.f : a.vals[idx]; }
template <bool FACT> __device__ inline float shfl_val(float v, int src) { return FACT ? 1.f : __shfl(v, src, 64); }

template <int V> __device__ inline Acc<V> shfl_xor_acc(const Acc<V> &a, int mask);
template <> __device__ inline Acc<4> shfl_xor_acc<4>(const Acc<4> &a, int mask)
{
    Acc<4> r;
    r.v.x = __shfl_xor(a.v.x, mask, 64);
    r.v.y = __shfl_xor(a.v.y, mask, 64);
    r.v.z = __shfl_xor(a.v.z, mask, 64);
    r.v.w = __shfl_xor(a.v.w, mask, 64);
    return r;
}
template <> __device__ inline Acc<1> shfl_xor_acc<1>(const Acc<1> &a, int mask)
{
    Acc<1> r;
    r.v = __shfl_xor(a.v, mask, 64);
    return r;
}

// Store the V columns a lane owns (clipped to col_end), adding `add_row` when present.
template <int V>
__device__ inline void store_cols(const Acc<V> &acc, float *y_row, const float *add_row, int col, int col_end, bool vec_ok)
{
    if (V == 4 && vec_ok && col + 4 <= col_end) {
        float4 o = make_float4(acc.get(0), acc.get(1), acc.get(2), acc.get(3));
        if (add_row) {
            const float4 a = *reinterpret_cast<const float4 *>(add_row + col);
            o.x += a.x; o.y += a.y; o.z += a.z; o.w += a.w;
        }
        *reinterpret_cast<float4 *>(y_row + col) = o;
    } else {
#pragma unroll
        for (int i = 0; i < V; ++i)
            if (col + i < col_end) y_row[col + i] = acc.get(i) + (add_row ? add_row[col + i] : 0.f);
    }
}

// Accumulate one chunk of a wavefront item: lane i holds the (column, value) pair of the chunk's
// entry i (lanes past the chunk hold a valid column).  Sub-step t hands entry t * G + grp to lane
// group grp through cross-lane reads, eight sub-steps (eight gathers per lane) at a time.  A
// full chunk (cnt >= 64) runs without any per-entry test.  Every lane of the wavefront must call
// this (lanes past the last column pass a valid `col` and drop their result).
template <int LPR, int V, bool S32, bool FACT>
__device__ inline void gather_chunk(Acc<V> &acc, const SpmmArgs &a, int c_l, float v_l, int cnt, int grp, int col)
{
    constexpr int G = 64 / LPR; // lane groups = entries per sub-step
    constexpr int U = 8;        // gathers in flight per lane
    using L = Ld<V>;
    if (cnt >= 64) {
        // not unrolled: with 16 or more lanes per row the unrolled loop holds the shuffled pairs of the whole chunk and
        // halves the wavefronts per SIMD (60 registers against 81-97), which costs 1.5 % at 301 columns
#pragma unroll 1
        for (int t = 0; t < LPR; t += U) {
            int c[U];
            float v[U];
            typename L::T x[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                c[u] = __shfl(c_l, (t + u) * G + grp, 64);
                v[u] = shfl_val<FACT>(v_l, (t + u) * G + grp);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) x[u] = load_x<V, S32>(a, c[u], col);
#pragma unroll
            for (int u = 0; u < U; ++u) acc.fma(v[u], x[u]);
        }
    } else {
        for (int t = 0; t * G < cnt; t += U) { // uniform trip count
            int c[U];
            float v[U];
            typename L::T x[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int src = ((t + u) * G + grp) & 63;
                c[u] = __shfl(c_l, src, 64);
                v[u] = shfl_val<FACT>(v_l, src);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) x[u] = load_x<V, S32>(a, c[u], col);
#pragma unroll
            for (int u = 0; u < U; ++u)
                if ((t + u) * G + grp < cnt) acc.fma(v[u], x[u]);
        }
    }
}

// Write an item's (or a row's) sum: to the output row, or to its partial-sum slot.
template <int V>
__device__ inline void store_result(Acc<V> acc, const SpmmArgs &a, int row, int dst, int col)
{
    if (dst >= 0) {
        if (a.dinv) acc.scale(a.dinv[row]); // factored form: the row's own factor (partial sums stay unscaled)
        store_cols<V>(acc, a.Y + (int64_t)row * a.ldy, a.Add ? a.Add + (int64_t)row * a.ldadd : nullptr, col, a.col_end,
                      a.vec_store != 0);
    } else {
        float *p = a.scratch + (int64_t)(-(dst + 1)) * a.slot_cols - a.col0; // slot row, pass-relative columns
        store_cols<V>(acc, p, nullptr, col, a.col_end, true);
    }
}

constexpr int NO_UNIT = INT32_MIN;

// One gather phase of the tiny-row path: sub-round t hands unit (t * GROUPS + grp) of the wavefront
// to lane group grp.  c_l / v_l hold, per lane, four (column, value) pairs of the unit that lane
// owns (column -1 = no entry).  Two sub-rounds (eight gathers per lane) are in flight at a time.
template <int LPR, int V, bool S32, bool FACT>
__device__ inline void batch_gather(Acc<V> (&acc)[8], const SpmmArgs &a, const int (&c_l)[4], const float (&v_l)[4],
                                    int grp, int colc)
{
    constexpr int G = 64 / LPR;
    using L = Ld<V>;
#pragma unroll
    for (int t0 = 0; t0 < 8; t0 += 2) {
        int cc[2][4];
        float vv[2][4];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                cc[u][i] = __shfl(c_l[i], (t0 + u) * G + grp, 64);
                vv[u][i] = shfl_val<FACT>(v_l[i], (t0 + u) * G + grp);
            }
        typename L::T x[2][4];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int c = cc[u][i] >= 0 ? cc[u][i] : 0; // an absent entry re-reads row 0 and is not accumulated
                x[u][i] = load_x<V, S32>(a, c, colc);
            }
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (cc[u][i] >= 0) acc[t0 + u].fma(vv[u][i], x[u][i]);
    }
}

// Rows of at most TINY_ROW (= 4) entries: 8 * GROUPS rows per wavefront.  Lane i owns row i
// (entries [beg_l, end_l), destination dst_l, NO_UNIT = nothing) and loads its entries; the gather
// phase hands them to the lane groups.  Every lane of the wavefront must call this.
template <int LPR, int V, bool S32, bool FACT>
__device__ inline void batch_units(const SpmmArgs &a, int beg_l, int end_l, int row_l, int dst_l, int lane)
{
    constexpr int G = 64 / LPR;
    const int grp = lane / LPR, sub = lane % LPR;
    const int col = a.col0 + sub * V;
    const bool col_ok = col < a.col_end;
    const int colc = col_ok ? col : a.col0;
    Acc<V> acc[8];
    int c_l[4];
    float v_l[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int idx = beg_l + i;
        const bool ok = idx < end_l;
        c_l[i] = ok ? a.colidx[idx] : -1;
        v_l[i] = ok ? ld_val<FACT>(a, idx) : 0.f;
    }
    batch_gather<LPR, V, S32, FACT>(acc, a, c_l, v_l, grp, colc);
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const int d = __shfl(dst_l, t * G + grp, 64);
        const int r = __shfl(row_l, t * G + grp, 64);
        if (d != NO_UNIT && col_ok) store_result<V>(acc[t], a, r, d, col);
    }
}

// Wavefront items: workgroup b serves class b mod n_classes, four items per workgroup: first the
// class's own pieces, then every n_classes-th group of four whole-row items.  An item's
// entries are read 64 (column, value) pairs at a time with one coalesced load each, lane i holding
// entry base + i, and the next 64 are requested before the current ones are consumed.  (Giving a
// wavefront several items and prefetching across them was measured and changes nothing: the
// kernel is bound by the traffic of the gathers, not by the latency of its index loads.)
template <int LPR, int V, bool S32, bool FACT>
__device__ __forceinline__ void wave_items_body(const SpmmArgs &a, int block)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int cls = block % a.n_classes, j = block / a.n_classes;
    const int piece_blocks = (a.big_cnt[cls] + 3) >> 2;
    int64_t item;
    if (j < piece_blocks) { // uniform per workgroup
        item = j * 4 + wave;
        if (item >= a.big_cnt[cls]) return;
        item += a.big_off[cls];
    } else {
        item = ((int64_t)(j - piece_blocks) * a.n_classes + cls) * 4 + wave;
        if (item >= a.wbig_cnt) return;
        item += a.wbig_off;
    }
    const int4 s = *reinterpret_cast<const int4 *>(a.items + item);
    const int grp = lane / LPR, sub = lane % LPR;
    const int col = a.col0 + sub * V;
    const bool active = col < a.col_end;
    const int colc = active ? col : a.col0;
    const int beg = s.y, end = s.z;
    Acc<V> acc;
    int idx = beg + lane;
    int c_l = a.colidx[idx < end ? idx : beg];
    float v_l = ld_val<FACT>(a, idx < end ? idx : beg);
    for (int base = beg; base < end; base += 64) {
        int c_n = 0;
        float v_n = 0.f;
        if (base + 64 < end) { // wavefront-uniform
            idx = base + 64 + lane;
            c_n = a.colidx[idx < end ? idx : beg];
            v_n = ld_val<FACT>(a, idx < end ? idx : beg);
        }
        gather_chunk<LPR, V, S32, FACT>(acc, a, c_l, v_l, end - base, grp, colc);
        c_l = c_n;
        v_l = v_n;
    }
#pragma unroll
    for (int m = LPR; m < 64; m <<= 1) acc.add(shfl_xor_acc<V>(acc, m));
    if (grp == 0 && active) store_result<V>(acc, a, s.x, s.w, col);
}

// The same for graphs that stay in cache (the one-launch kernel below): a workgroup takes 4 * ipw consecutive items,
// wavefront w the items w, w + 4, ... of them; the next item's descriptor is requested when an item starts and its first
// entries during the item's last chunk.  There a call lasts tens of microseconds and is made of chains of dependent loads
// (descriptor -> entries -> gathers), which this overlaps across items: 0.049 -> 0.043 ms per call at 2.5 M entries.  On
// graphs that stream from memory it changes nothing and its eight extra registers cost 2 %, so they keep one item per wavefront.
template <int LPR, int V, bool S32, bool FACT>
__device__ __forceinline__ void wave_items_run_body(const SpmmArgs &a, int block)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int cls = block % a.n_classes, j = block / a.n_classes;
    const int ipb = 4 * a.ipw; // items per workgroup
    const int piece_blocks = (a.big_cnt[cls] + ipb - 1) / ipb;
    int64_t first, left;
    if (j < piece_blocks) { // uniform per workgroup
        first = (int64_t)j * ipb;
        left = a.big_cnt[cls] - first;
        first += a.big_off[cls];
    } else {
        first = ((int64_t)(j - piece_blocks) * a.n_classes + cls) * ipb;
        left = a.wbig_cnt - first;
        first += a.wbig_off;
    }
    const int cnt = left < ipb ? (int)left : ipb;
    int t = wave; // this wavefront takes items wave, wave + 4, ... of the workgroup's run
    if (t >= cnt) return;
    const int grp = lane / LPR, sub = lane % LPR;
    const int col = a.col0 + sub * V;
    const bool active = col < a.col_end;
    const int colc = active ? col : a.col0;
    int4 s = *reinterpret_cast<const int4 *>(a.items + first + t);
    int idx = s.y + lane;
    int c_l = a.colidx[idx < s.z ? idx : s.y];
    float v_l = ld_val<FACT>(a, idx < s.z ? idx : s.y);
    for (;;) {
        const bool more = t + 4 < cnt; // wavefront-uniform
        // the next item's descriptor is requested now and its first entries during this item's last chunk, so
        // that a short item does not expose the whole chain descriptor -> entries -> gathers
        int4 sn = s;
        if (more) sn = *reinterpret_cast<const int4 *>(a.items + first + t + 4);
        const int beg = s.y, end = s.z;
        Acc<V> acc;
        for (int base = beg; base < end; base += 64) {
            int c_n = 0;
            float v_n = 0.f;
            if (base + 64 < end) { // wavefront-uniform
                idx = base + 64 + lane;
                c_n = a.colidx[idx < end ? idx : beg];
                v_n = ld_val<FACT>(a, idx < end ? idx : beg);
            } else if (more) {
                idx = sn.y + lane;
                c_n = a.colidx[idx < sn.z ? idx : sn.y];
                v_n = ld_val<FACT>(a, idx < sn.z ? idx : sn.y);
            }
            gather_chunk<LPR, V, S32, FACT>(acc, a, c_l, v_l, end - base, grp, colc);
            c_l = c_n;
            v_l = v_n;
        }
#pragma unroll
        for (int m = LPR; m < 64; m <<= 1) acc.add(shfl_xor_acc<V>(acc, m));
        if (grp == 0 && active) store_result<V>(acc, a, s.x, s.w, col);
        if (!more) break;
        s = sn;
        t += 4;
    }
}

// Lane-group items (whole rows and class pieces of 5..GI_MAX entries, GI_MAX = the schedule's item_max):
// workgroup b serves class b mod n_classes and takes a run of 32 * G consecutive items of its list (first the
// class's own pieces, then every n_classes-th run of the whole rows).  In round r its four wavefronts work on
// 4 * G consecutive items of the run, lane group grp of wavefront w on item r * 4 * G + w * G + grp (lane
// r * G + grp holds that item's descriptor).  The group
// reads the item's (column, value) pairs with one read per LPR entries (lane `sub` holds entries
// sub, sub + LPR, ...; the next round's pairs are requested before this round's gathers), and each
// gather takes its pair from the holding lane by a cross-lane read, eight gathers in flight.
template <int LPR, int V, bool S32, int GI_MAX, bool FACT>
__device__ __forceinline__ void group_items_body(const SpmmArgs &a, int block)
{
    constexpr int G = 64 / LPR;                 // items in flight per wavefront
    constexpr int UNITS = 8 * G;                // items per wavefront
    constexpr int K = LPR >= GI_MAX ? 1 : GI_MAX / LPR; // index registers per lane (K * LPR >= GI_MAX entries)
    constexpr int U = 8;
    using L = Ld<V>;
    constexpr int RUN = 4 * UNITS;              // items per workgroup: one run of consecutive items of its list
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int cls = block % a.n_classes, blk = block / a.n_classes;
    const int piece_blocks = (a.small_cnt[cls] + RUN - 1) / RUN;
    int64_t first, left;
    if (blk < piece_blocks) { // uniform per workgroup
        first = (int64_t)blk * RUN;
        left = a.small_cnt[cls] - first;
        first += a.small_off[cls];
    } else {
        first = ((int64_t)(blk - piece_blocks) * a.n_classes + cls) * RUN;
        left = a.wsmall_cnt - first;
        first += a.wsmall_off;
    }
    const int run = left < RUN ? (int)left : RUN;
    // Round r of the workgroup works on the 4 * G consecutive items [r * 4 * G, (r + 1) * 4 * G) of its run, wavefront w
    // on the G of them from w * G on: what is in flight together on a CU is a window of consecutive rows, so with a row
    // order that puts rows with common neighbours side by side their gathers meet in the caches while the rows are live.
    if (run <= wave * G) return; // uniform per wavefront
    const int rounds = (run - wave * G + 4 * G - 1) / (4 * G);
    int4 d = make_int4(0, 0, 0, NO_UNIT);
    {
        const int q = (lane / G) * (4 * G) + wave * G + lane % G; // lane r * G + g holds the descriptor of round r, group g
        if (lane < 8 * G && q < run) d = *reinterpret_cast<const int4 *>(a.items + first + q);
    }
    const int grp = lane / LPR, sub = lane % LPR, gbase = lane - sub;
    const int col = a.col0 + sub * V;
    const bool col_ok = col < a.col_end;
    const int colc = col_ok ? col : a.col0;
    int beg = __shfl(d.y, grp, 64), end = __shfl(d.z, grp, 64);
    int c_k[K];
    float v_k[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int e = beg + sub + LPR * k;
        const bool ok = e < end;
        c_k[k] = ok ? a.colidx[e] : 0;
        v_k[k] = ok ? ld_val<FACT>(a, e) : 0.f;
    }
    for (int r = 0; r < rounds; ++r) {
        const int row = __shfl(d.x, r * G + grp, 64), dst = __shfl(d.w, r * G + grp, 64);
        const int len = end - beg;
        const int nsrc = (r + 1 < rounds ? (r + 1) * G : 0) + grp;
        const int nbeg = __shfl(d.y, nsrc, 64), nend = r + 1 < rounds ? __shfl(d.z, nsrc, 64) : nbeg;
        int c_n[K];
        float v_n[K];
#pragma unroll
        for (int k = 0; k < K; ++k) { // the next round's pairs (none after the last round: nend == nbeg)
            const int e = nbeg + sub + LPR * k;
            const bool ok = e < nend;
            c_n[k] = ok ? a.colidx[e] : 0;
            v_n[k] = ok ? ld_val<FACT>(a, e) : 0.f;
        }
        Acc<V> acc;
#pragma unroll
        for (int j0 = 0; j0 < GI_MAX; j0 += U) {
            if (!__any(j0 < len)) break; // wavefront-uniform
            int c[U];
            float v[U];
            typename L::T x[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int jj = j0 + u;
                const int cc = __shfl(c_k[jj / LPR < K ? jj / LPR : 0], gbase + jj % LPR, 64);
                v[u] = shfl_val<FACT>(v_k[jj / LPR < K ? jj / LPR : 0], gbase + jj % LPR);
                c[u] = jj < len ? cc : 0; // an absent entry re-reads row 0 and is not accumulated
            }
#pragma unroll
            for (int u = 0; u < U; ++u) x[u] = load_x<V, S32>(a, c[u], colc);
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (j0 + u < len) acc.fma(v[u], x[u]);
        }
        if (dst != NO_UNIT && col_ok) store_result<V>(acc, a, row, dst, col);
        beg = nbeg;
        end = nend;
#pragma unroll
        for (int k = 0; k < K; ++k) { c_k[k] = c_n[k]; v_k[k] = v_n[k]; }
    }
}

// Rows of at most TINY_ROW entries, 64 consecutive positions of the schedule per wavefront (consecutive
// rows in natural order).
template <int LPR, int V, bool S32, bool FACT>
__device__ __forceinline__ void tiny_rows_body(const SpmmArgs &a, int block)
{
    constexpr int UNITS = 8 * (64 / LPR); // rows per wavefront
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int first = (block * 4 + wave) * UNITS;
    if (first >= a.n) return; // uniform per wavefront
    int beg_l = 0, end_l = 0, row_l = 0, dst_l = NO_UNIT;
    if (lane < UNITS && first + lane < a.n) {
        const int row = a.order ? a.order[first + lane] : first + lane;
        const int b = a.rowptr[row], e = a.rowptr[row + 1];
        if (e - b <= TINY_ROW) { row_l = row; beg_l = b; end_l = e; dst_l = row; }
    }
    batch_units<LPR, V, S32, FACT>(a, beg_l, end_l, row_l, dst_l, lane);
}

template <int LPR, int V, bool S32, bool FACT>
__global__ __launch_bounds__(256) void spmm_wave_items_kernel(const SpmmArgs a) { wave_items_body<LPR, V, S32, FACT>(a, blockIdx.x); }

template <int LPR, int V, bool S32, int GI_MAX, bool FACT>
__global__ __launch_bounds__(256) void spmm_group_items_kernel(const SpmmArgs a) { group_items_body<LPR, V, S32, GI_MAX, FACT>(a, blockIdx.x); }

template <int LPR, int V, bool S32, bool FACT>
__global__ __launch_bounds__(256) void spmm_tiny_rows_kernel(const SpmmArgs a) { tiny_rows_body<LPR, V, S32, FACT>(a, blockIdx.x); }

// All three item kinds in one launch: workgroups [0, g1) take wavefront items, [g1, g1 + g2)
// lane-group items, the rest tiny rows (g1 and g2 are multiples of n_classes, so workgroup b still
// serves class b mod n_classes).  For graphs that stay in cache a call takes tens of microseconds and
// each of three launches would pay its own ramp-up and its own chain of dependent loads; in one launch
// they overlap (cfg2: 0.075 -> 0.056 ms per call).  Large graphs keep the three launches: there the
// class pieces must have the L2s to themselves before the whole rows start (merged: cfg5 4.09 -> 4.30 ms).
template <int LPR, int V, bool S32, bool FACT>
__global__ __launch_bounds__(256) void spmm_merged_kernel(const SpmmArgs a, int g1, int g2)
{
    const int b = blockIdx.x; // uniform per workgroup
    if (b < g1) wave_items_run_body<LPR, V, S32, FACT>(a, b);
    else if (b < g1 + g2) group_items_body<LPR, V, S32, ITEM_SHORT, FACT>(a, b - g1);
    else tiny_rows_body<LPR, V, S32, FACT>(a, b - g1 - g2);
}

// Rows with several items: add the partial slots in order.  One thread per (row, column); eight
// independent slot reads are in flight at a time, the additions stay in slot order.
__global__ __launch_bounds__(256) void spmm_fix_kernel(const SpmmArgs a, int32_t n_fix)
{
    const int w = a.col_end - a.col0;
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t r = t / w;
    if (r >= n_fix) return;
    const int j = (int)(t - r * w);
    const int4 f = *reinterpret_cast<const int4 *>(a.fix + r);
    const float *p = a.scratch + j;
    float acc = 0.f;
    int s = f.y;
    for (; s + 8 <= f.z; s += 8) {
        float q[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) q[i] = p[(int64_t)(s + i) * a.slot_cols];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc += q[i];
    }
    for (; s < f.z; ++s) acc += p[(int64_t)s * a.slot_cols];
    if (a.dinv) acc *= a.dinv[f.x]; // factored form: the row's own factor
    const int col = a.col0 + j;
    if (a.Add) acc += a.Add[(int64_t)f.x * a.ldadd + col];
    a.Y[(int64_t)f.x * a.ldy + col] = acc;
}

template <int LPR, int V, bool S32, bool FACT>
int launch_variant(const SpmmArgs &a, hipStream_t stream)
{
    constexpr int units_per_block = 4 * 8 * (64 / LPR);
    const int64_t g1 = (int64_t)a.n_classes * a.big_blocks;
    const int64_t g2 = (int64_t)a.n_classes * a.small_blocks;
    const int64_t g3 = (a.n + units_per_block - 1) / units_per_block;
    SG_REQUIRE(g1 <= INT32_MAX && g2 <= INT32_MAX && g3 <= INT32_MAX, SLICEGCN_ERANGE, "spmm: grid too large");
    if (a.item_max <= ITEM_SHORT) { // cache-resident graph: one launch (big_blocks counts runs of 4 * ipw items)
        SG_REQUIRE(g1 + g2 + g3 <= INT32_MAX, SLICEGCN_ERANGE, "spmm: grid too large");
        spmm_merged_kernel<LPR, V, S32, FACT><<<(unsigned)(g1 + g2 + g3), 256, 0, stream>>>(a, (int)g1, (int)g2);
        SG_LAUNCH_CHECK();
        return SLICEGCN_OK;
    }
    if (g1 > 0) {
        spmm_wave_items_kernel<LPR, V, S32, FACT><<<(unsigned)g1, 256, 0, stream>>>(a);
        SG_LAUNCH_CHECK();
    }
    if (g2 > 0) {
        spmm_group_items_kernel<LPR, V, S32, ITEM_LONG, FACT><<<(unsigned)g2, 256, 0, stream>>>(a);
        SG_LAUNCH_CHECK();
    }
    spmm_tiny_rows_kernel<LPR, V, S32, FACT><<<(unsigned)g3, 256, 0, stream>>>(a);
    SG_LAUNCH_CHECK();
    return SLICEGCN_OK;
}

template <int LPR, int V>
int launch_kernels(const SpmmArgs &a, hipStream_t stream)
{
    if (a.dinv) { // factored form
        if (V == 4 && a.ldx_bytes != 0) return launch_variant<LPR, V, V == 4, true>(a, stream);
        return launch_variant<LPR, V, false, true>(a, stream);
    }
    if (V == 4 && a.ldx_bytes != 0) return launch_variant<LPR, V, V == 4, false>(a, stream);
    return launch_variant<LPR, V, false, false>(a, stream);
}

template <int V>
int launch_pass(const SpmmArgs &a, int lpr, hipStream_t stream)
{
    switch (lpr) {
    case 8: return launch_kernels<8, V>(a, stream);
    case 16: return launch_kernels<16, V>(a, stream);
    case 32: return launch_kernels<32, V>(a, stream);
    default: return launch_kernels<64, V>(a, stream);
    }
}

} // namespace

// Bytes of partial-sum workspace an aggregation of `width` columns over pattern `m` may need: the larger
// of the two schedules (which one runs depends on the operand layout, unknown here), one slot of
// min(width rounded up to 4, pass width) floats per item of every row cut into several items.
size_t spmm_workspace_bytes(const Csr &m, int32_t width)
{
    const int64_t w4 = round_up(width, 4);
    const int64_t a = m.wide.n_slots * (w4 < WIDE_SLOT_COLS ? w4 : WIDE_SLOT_COLS);
    const int64_t b = m.xcd.n_slots * (w4 < XCD_SLOT_COLS ? w4 : XCD_SLOT_COLS);
    return (size_t)round_up((a > b ? a : b) * (int64_t)sizeof(float), 256);
}

int launch_spmm(const slicegcn_graph *g, const Csr &m, const float *X, int64_t ldx, int32_t width,
                float *Y, int64_t ldy, const float *Add, int64_t ldadd, void *ws, size_t ws_bytes, hipStream_t stream,
                bool prescaled)
{
    // 16-byte gathers need an aligned base, ld % 4 == 0 and room for the last vector of a row
    const bool vec_load = aligned16(X) && (ldx % 4 == 0) && ldx >= round_up(width, 4);
    const int V = vec_load ? 4 : 1;
    // 16-byte gathers use the 8-class schedule in passes of at most 128 columns (32 lanes per row):
    // narrower passes re-read the index streams more often, wider ones make the set of hot rows of
    // the operand too large for the L2s (301 columns: 7.8 / 7.4 / 7.7 ms for passes of 64 / 128 / 256);
    // the scalar path keeps the single-class schedule
    const bool use_xcd = vec_load;
    const Schedule &sc = use_xcd ? m.xcd : m.wide;
    const int slot_cols = use_xcd ? XCD_SLOT_COLS : WIDE_SLOT_COLS;
    const int64_t used_cols = width < slot_cols ? round_up(width, 4) : slot_cols; // one pass: slots packed densely
    const size_t need = (size_t)(sc.n_slots * used_cols) * sizeof(float);
    SG_REQUIRE(need == 0 || (ws != nullptr && ws_bytes >= need), SLICEGCN_EWORKSPACE,
               "aggregation: workspace of %zu bytes, %zu needed", ws_bytes, need);
    SG_REQUIRE(need == 0 || (reinterpret_cast<uintptr_t>(ws) & 255u) == 0, SLICEGCN_EINVAL,
               "aggregation: workspace not 256-byte aligned");
    SpmmArgs a;
    a.rowptr = m.rowptr; a.colidx = m.colidx; a.vals = m.vals; a.items = sc.items; a.fix = sc.fix; a.order = g->order;
    a.X = X; a.Y = Y; a.Add = Add; a.scratch = static_cast<float *>(ws);
    a.dinv = prescaled ? g->dinv : nullptr;
    a.ldx = ldx; a.ldy = ldy; a.ldadd = Add ? ldadd : 0;
    const bool s32 = g->n < (1 << 24) && ldx * 4 < (1 << 24) && (int64_t)g->n * ldx * 4 < ((int64_t)1 << 32);
    a.ldx_bytes = s32 ? (uint32_t)(ldx * 4) : 0u;
    a.n = (int32_t)g->n;
    a.n_classes = sc.n_classes;
    a.item_max = sc.item_max;
    a.slot_cols = slot_cols; // narrowed below to the pass width
    a.vec_store = aligned16(Y) && (ldy % 4 == 0) && (!Add || (aligned16(Add) && ldadd % 4 == 0));
    a.wbig_off = sc.wbig_off; a.wbig_cnt = sc.wbig_cnt;
    a.wsmall_off = sc.wsmall_off; a.wsmall_cnt = sc.wsmall_cnt;
    // workgroups per class: the class's own pieces, then its share of the whole-row chunks
    a.ipw = sc.item_max <= ITEM_SHORT ? 4 : 1; // the one-launch kernel works through runs of items
    const int64_t ipb = 4 * a.ipw;
    const int64_t wbig_chunks = ((int64_t)sc.wbig_cnt + ipb - 1) / ipb;
    int64_t big_blocks = 0;
    for (int c = 0; c < MAX_CLASSES; ++c) {
        a.big_off[c] = sc.big_off[c]; a.big_cnt[c] = sc.big_cnt[c];
        a.small_off[c] = sc.small_off[c]; a.small_cnt[c] = sc.small_cnt[c];
        if (c >= sc.n_classes) continue;
        const int64_t b = (sc.big_cnt[c] + ipb - 1) / ipb + (wbig_chunks + sc.n_classes - 1 - c) / sc.n_classes;
        big_blocks = b > big_blocks ? b : big_blocks;
    }
    SG_REQUIRE(big_blocks * sc.n_classes <= INT32_MAX, SLICEGCN_ERANGE, "spmm: grid too large");
    a.big_blocks = (int32_t)big_blocks;
    ProfScope prof(Add ? SLICEGCN_PROF_SPMM_ADD : SLICEGCN_PROF_SPMM, width, stream);
    const int pass_cols = vec_load ? slot_cols : 64;
    a.slot_cols = (int32_t)used_cols;
    for (int32_t c0 = 0; c0 < width; c0 += pass_cols) {
        a.col0 = c0;
        a.col_end = width < c0 + pass_cols ? width : c0 + pass_cols;
        const int lanes_needed = (a.col_end - c0 + V - 1) / V;
        int lpr = 8;
        while (lpr < lanes_needed) lpr <<= 1; // 8, 16, 32 or 64
        const int64_t run = 4 * 8 * (64 / lpr); // lane-group items per workgroup: runs of consecutive items
        const int64_t wsmall_runs = ((int64_t)sc.wsmall_cnt + run - 1) / run;
        int64_t small_blocks = 0;
        for (int c = 0; c < sc.n_classes; ++c) { // the class's own pieces, then its share of the whole-row runs
            const int64_t b = (sc.small_cnt[c] + run - 1) / run + (wsmall_runs + sc.n_classes - 1 - c) / sc.n_classes;
            small_blocks = b > small_blocks ? b : small_blocks;
        }
        SG_REQUIRE(small_blocks * sc.n_classes <= INT32_MAX, SLICEGCN_ERANGE, "spmm: grid too large");
        a.small_blocks = (int32_t)small_blocks;
        if (int rc = vec_load ? launch_pass<4>(a, lpr, stream) : launch_pass<1>(a, lpr, stream)) return rc;
        if (sc.n_fix > 0) {
            const int64_t threads = sc.n_fix * (int64_t)(a.col_end - c0);
            spmm_fix_kernel<<<(unsigned)((threads + 255) / 256), 256, 0, stream>>>(a, (int32_t)sc.n_fix);
            SG_LAUNCH_CHECK();
        }
    }
    return SLICEGCN_OK;
}

} // namespace slicegcn

using namespace slicegcn;

// ---- aggregation without a caller workspace --------------------------------------------------
// The partial sums go to this fixed array instead (one copy per GPU the library runs on, held until the
// process ends).  In host code `scratch` is only a handle for the symbol: the device address comes from
// hipGetSymbolAddress, once per device, and only that address is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[SLICEGCN_STATIC_WS_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[MAX_DEVICES] = {nullptr};

// device address of `scratch` on the current device (looked up on the first call per device)
int static_scratch(void **out)
{
    int dev = -1;
    SG_HIP(hipGetDevice(&dev));
    SG_REQUIRE(dev >= 0 && dev < MAX_DEVICES, SLICEGCN_EUNSUPPORTED, "spmm_slice_static: device index %d not supported", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *ptr = nullptr;
        SG_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        SG_REQUIRE(ptr != nullptr, SLICEGCN_EHIP, "spmm_slice_static: hipGetSymbolAddress returned NULL");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SLICEGCN_OK;
}
} // namespace

extern "C" int slicegcn_spmm_slice_static(const slicegcn_graph *g, int op, const float *X, int64_t ldx,
                                          int32_t width, float *Y, int64_t ldy, void *stream)
{
    SG_REQUIRE(g && X && Y, SLICEGCN_EINVAL, "spmm_slice_static: NULL argument");
    SG_REQUIRE((op & ~(SLICEGCN_SPMM_TRANSPOSE | SLICEGCN_SPMM_PRESCALED)) == 0, SLICEGCN_EINVAL, "spmm_slice_static: unknown op bits 0x%x", op);
    SG_REQUIRE(width >= 1, SLICEGCN_EINVAL, "spmm_slice_static: width = %d < 1", width);
    SG_REQUIRE(ldx >= width && ldy >= width, SLICEGCN_EINVAL, "spmm_slice_static: leading dimension smaller than width");
    const Csr &m = (op & SLICEGCN_SPMM_TRANSPOSE) ? g->tr : g->fwd;
    const size_t need = spmm_workspace_bytes(m, width);
    SG_REQUIRE(need <= (size_t)SLICEGCN_STATIC_WS_BYTES, SLICEGCN_EWORKSPACE,
               "spmm_slice_static: this graph and width need %zu bytes of partial sums, the built-in buffer holds %zu; "
               "use slicegcn_spmm_slice with a workspace", need, (size_t)SLICEGCN_STATIC_WS_BYTES);
    void *ptr = nullptr;
    if (need > 0)
        if (int rc = static_scratch(&ptr)) return rc;
    return launch_spmm(g, m, X, ldx, width, Y, ldy, nullptr, 0, ptr, need, as_stream(stream), (op & SLICEGCN_SPMM_PRESCALED) != 0);
}

extern "C" size_t slicegcn_spmm_workspace_bytes(const slicegcn_graph *g, int op, int32_t width)
{
    if (!g || width < 1) return 0;
    return spmm_workspace_bytes((op & SLICEGCN_SPMM_TRANSPOSE) ? g->tr : g->fwd, width);
}

extern "C" int slicegcn_spmm_slice(const slicegcn_graph *g, int op, const float *X, int64_t ldx,
                                   int32_t width, float *Y, int64_t ldy, void *ws, size_t ws_bytes, void *stream)
{
    SG_REQUIRE(g && X && Y, SLICEGCN_EINVAL, "spmm_slice: NULL argument");
    SG_REQUIRE((op & ~(SLICEGCN_SPMM_TRANSPOSE | SLICEGCN_SPMM_PRESCALED)) == 0, SLICEGCN_EINVAL, "spmm_slice: unknown op bits 0x%x", op);
    SG_REQUIRE(width >= 1, SLICEGCN_EINVAL, "spmm_slice: width = %d < 1", width);
    SG_REQUIRE(ldx >= width && ldy >= width, SLICEGCN_EINVAL, "spmm_slice: leading dimension smaller than width");
    return launch_spmm(g, (op & SLICEGCN_SPMM_TRANSPOSE) ? g->tr : g->fwd, X, ldx, width, Y, ldy, nullptr, 0, ws, ws_bytes,
                       as_stream(stream), (op & SLICEGCN_SPMM_PRESCALED) != 0);
}
