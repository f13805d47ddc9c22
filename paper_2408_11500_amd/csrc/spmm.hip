// Slice aggregation Y = A^ X (+ Add): the neighbour sum of the SliceGCN layer equation.
//
// Work split (fixed per graph when it is built):
//   * rows with at most LONG_ROW stored entries: a group of LPR lanes per row, rows in natural
//     order, so index/value reads and the output stream stay contiguous;
//   * longer rows: one wavefront per segment of at most SEG_NNZ entries; the 64/LPR lane groups
//     stride over the segment (four gathers in flight per group) and are combined with
//     cross-lane shuffles; a row cut into several segments stores per-segment partial sums that
//     a small fix-up kernel adds in segment order.
// No floating-point atomics anywhere: the summation order is a function of the graph only.
//
// Lanes map to columns: with vector width V (4 floats when the operand layout allows 16-byte
// loads, else 1), lane `sub` of a group owns columns [V*sub, V*sub + V) of the current column
// pass; a pass covers at most SCRATCH_COLS columns and wider operands take several passes.
#include "common.h"

namespace slicegcn {

namespace {

struct SpmmArgs {
    const int32_t *rowptr;
    const int32_t *colidx;
    const float *vals;
    const Segment *segs;
    const FixRow *fix;
    const float *X;
    float *Y;
    const float *Add;
    float *scratch;
    int64_t ldx, ldy, ldadd;
    int32_t n;
    int32_t n_segs;
    int32_t n_seg_blocks;
    int32_t col0;    // first column of this pass
    int32_t col_end; // one past the last column of this pass (<= width)
    int32_t vec_store; // Y (and Add) allow 16-byte accesses
};

template <int V> struct Acc;
template <> struct Acc<4> {
    float4 v;
    __device__ Acc() : v(make_float4(0.f, 0.f, 0.f, 0.f)) {}
    __device__ void fma(float a, const float4 &x) { v.x += a * x.x; v.y += a * x.y; v.z += a * x.z; v.w += a * x.w; }
    __device__ void add(const Acc &o) { v.x += o.v.x; v.y += o.v.y; v.z += o.v.z; v.w += o.v.w; }
    __device__ float get(int i) const { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }
};
template <> struct Acc<1> {
    float v;
    __device__ Acc() : v(0.f) {}
    __device__ void fma(float a, float x) { v += a * x; }
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

// Accumulate entries e = first, first + step, ... < end, four gathers in flight.
template <int V>
__device__ inline void gather_accumulate(Acc<V> &acc, const SpmmArgs &a, int first, int end, int step, int col)
{
    using L = Ld<V>;
    int e = first;
    for (; e + 3 * step < end; e += 4 * step) {
        const int c0 = a.colidx[e], c1 = a.colidx[e + step], c2 = a.colidx[e + 2 * step], c3 = a.colidx[e + 3 * step];
        const float v0 = a.vals[e], v1 = a.vals[e + step], v2 = a.vals[e + 2 * step], v3 = a.vals[e + 3 * step];
        const typename L::T x0 = L::load(a.X + (int64_t)c0 * a.ldx + col);
        const typename L::T x1 = L::load(a.X + (int64_t)c1 * a.ldx + col);
        const typename L::T x2 = L::load(a.X + (int64_t)c2 * a.ldx + col);
        const typename L::T x3 = L::load(a.X + (int64_t)c3 * a.ldx + col);
        acc.fma(v0, x0);
        acc.fma(v1, x1);
        acc.fma(v2, x2);
        acc.fma(v3, x3);
    }
    for (; e < end; e += step) {
        const int c = a.colidx[e];
        const float v = a.vals[e];
        acc.fma(v, L::load(a.X + (int64_t)c * a.ldx + col));
    }
}

template <int LPR, int V>
__global__ __launch_bounds__(256) void spmm_kernel(const SpmmArgs a)
{
    constexpr int GROUPS = 64 / LPR;       // lane groups per wavefront
    constexpr int ROWS_PER_BLOCK = 256 / LPR;
    const int blk = blockIdx.x;
    if (blk < a.n_seg_blocks) {
        // ---- long rows: one wavefront per segment ----
        const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
        const int seg = blk * 4 + wave;
        if (seg >= a.n_segs) return; // uniform per wavefront
        const int4 s = *reinterpret_cast<const int4 *>(a.segs + seg);
        const int row = s.x, beg = s.y, end = s.z, dst = s.w;
        const int grp = lane / LPR, sub = lane % LPR;
        const int col = a.col0 + sub * V;
        const bool active = col < a.col_end;
        Acc<V> acc;
        if (active) gather_accumulate<V>(acc, a, beg + grp, end, GROUPS, col);
#pragma unroll
        for (int m = LPR; m < 64; m <<= 1) acc.add(shfl_xor_acc<V>(acc, m));
        if (grp == 0 && active) {
            if (dst >= 0) {
                store_cols<V>(acc, a.Y + (int64_t)row * a.ldy, a.Add ? a.Add + (int64_t)row * a.ldadd : nullptr, col,
                              a.col_end, a.vec_store != 0);
            } else {
                float *p = a.scratch + (int64_t)(-(dst + 1)) * SCRATCH_COLS - a.col0; // slot row, pass-relative columns
                store_cols<V>(acc, p, nullptr, col, a.col_end, true);
            }
        }
    } else {
        // ---- short rows: one lane group per row, natural order ----
        const int row = (blk - a.n_seg_blocks) * ROWS_PER_BLOCK + threadIdx.x / LPR;
        const int sub = threadIdx.x % LPR;
        const int col = a.col0 + sub * V;
        if (row >= a.n || col >= a.col_end) return;
        const int beg = a.rowptr[row], end = a.rowptr[row + 1];
        if (end - beg > LONG_ROW) return; // a long row: written by the branch above
        Acc<V> acc;
        gather_accumulate<V>(acc, a, beg, end, 1, col);
        store_cols<V>(acc, a.Y + (int64_t)row * a.ldy, a.Add ? a.Add + (int64_t)row * a.ldadd : nullptr, col,
                      a.col_end, a.vec_store != 0);
    }
}

// Rows that were cut: add the partial slots in order.  One thread per (row, column).
__global__ __launch_bounds__(256) void spmm_fix_kernel(const SpmmArgs a, int32_t n_fix)
{
    const int w = a.col_end - a.col0;
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t r = t / w;
    if (r >= n_fix) return;
    const int j = (int)(t - r * w);
    const int4 f = *reinterpret_cast<const int4 *>(a.fix + r);
    float acc = 0.f;
    for (int s = f.y; s < f.z; ++s) acc += a.scratch[(int64_t)s * SCRATCH_COLS + j];
    const int col = a.col0 + j;
    if (a.Add) acc += a.Add[(int64_t)f.x * a.ldadd + col];
    a.Y[(int64_t)f.x * a.ldy + col] = acc;
}

template <int V>
int launch_pass(const SpmmArgs &a, int lpr, hipStream_t stream)
{
    const int rows_per_block = 256 / lpr;
    const unsigned grid = (unsigned)a.n_seg_blocks + (unsigned)((a.n + rows_per_block - 1) / rows_per_block);
    switch (lpr) {
    case 8: spmm_kernel<8, V><<<grid, 256, 0, stream>>>(a); break;
    case 16: spmm_kernel<16, V><<<grid, 256, 0, stream>>>(a); break;
    case 32: spmm_kernel<32, V><<<grid, 256, 0, stream>>>(a); break;
    default: spmm_kernel<64, V><<<grid, 256, 0, stream>>>(a); break;
    }
    SG_LAUNCH_CHECK();
    return SLICEGCN_OK;
}

} // namespace

int launch_spmm(const slicegcn_graph *g, const Csr &m, const float *X, int64_t ldx, int32_t width,
                float *Y, int64_t ldy, const float *Add, int64_t ldadd, hipStream_t stream)
{
    SG_REQUIRE(m.n_slots == 0 || g->scratch != nullptr, SLICEGCN_EINVAL, "spmm: graph handle has no scratch buffer");
    SpmmArgs a;
    a.rowptr = m.rowptr; a.colidx = m.colidx; a.vals = m.vals; a.segs = m.segs; a.fix = m.fix;
    a.X = X; a.Y = Y; a.Add = Add; a.scratch = g->scratch;
    a.ldx = ldx; a.ldy = ldy; a.ldadd = Add ? ldadd : 0;
    a.n = (int32_t)g->n;
    a.n_segs = (int32_t)m.n_segs;
    a.n_seg_blocks = (int32_t)((m.n_segs + 3) / 4);
    // 16-byte gathers need an aligned base, ld % 4 == 0 and room for the last vector of a row
    const bool vec_load = aligned16(X) && (ldx % 4 == 0) && ldx >= round_up(width, 4);
    a.vec_store = aligned16(Y) && (ldy % 4 == 0) && (!Add || (aligned16(Add) && ldadd % 4 == 0));
    ProfScope prof(Add ? SLICEGCN_PROF_SPMM_ADD : SLICEGCN_PROF_SPMM, width, stream);
    const int V = vec_load ? 4 : 1;
    const int pass_cols = vec_load ? SCRATCH_COLS : 64;
    for (int32_t c0 = 0; c0 < width; c0 += pass_cols) {
        a.col0 = c0;
        a.col_end = width < c0 + pass_cols ? width : c0 + pass_cols;
        const int lanes_needed = (a.col_end - c0 + V - 1) / V;
        int lpr = 8;
        while (lpr < lanes_needed) lpr <<= 1; // 8, 16, 32 or 64
        if (int rc = vec_load ? launch_pass<4>(a, lpr, stream) : launch_pass<1>(a, lpr, stream)) return rc;
        if (m.n_fix > 0) {
            const int64_t threads = m.n_fix * (int64_t)(a.col_end - c0);
            spmm_fix_kernel<<<(unsigned)((threads + 255) / 256), 256, 0, stream>>>(a, (int32_t)m.n_fix);
            SG_LAUNCH_CHECK();
        }
    }
    return SLICEGCN_OK;
}

} // namespace slicegcn

using namespace slicegcn;

extern "C" int slicegcn_spmm_slice(const slicegcn_graph *g, int transpose, const float *X, int64_t ldx,
                                   int32_t width, float *Y, int64_t ldy, void *stream)
{
    SG_REQUIRE(g && X && Y, SLICEGCN_EINVAL, "spmm_slice: NULL argument");
    SG_REQUIRE(width >= 1, SLICEGCN_EINVAL, "spmm_slice: width = %d < 1", width);
    SG_REQUIRE(ldx >= width && ldy >= width, SLICEGCN_EINVAL, "spmm_slice: leading dimension smaller than width");
    return launch_spmm(g, transpose ? g->tr : g->fwd, X, ldx, width, Y, ldy, nullptr, 0, as_stream(stream));
}
