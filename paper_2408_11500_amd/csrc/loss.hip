// Mean softmax cross-entropy over all nodes and its gradient: the paper's loss equation with every
// node labelled,  loss = -(1/n) sum_v log softmax(logits[v, :])[y_v],
// dlogits[v, j] = (softmax(logits[v, :])[j] - [j == y_v]) / n.
//
// One 16-lane group per row: the group sweeps the row three times (maximum, sum of exponentials,
// gradient), each lane taking columns sub, sub + 16, ...; the row was just read, so the second
// and third sweep hit L1/L2.  Row losses are added per workgroup (64 rows) in fp64 in a fixed
// order, and a single-workgroup kernel adds the workgroup sums in fp64 in a fixed order: no
// floating-point atomics, bitwise reproducible.  A label outside [0, c) cannot be reported to the
// host without a synchronisation, so it poisons the result instead: the loss becomes NaN.
#include "common.h"

namespace slicegcn {

namespace {

constexpr int CE_LPR = 16;                // lanes per row
constexpr int CE_ROWS = 256 / CE_LPR;     // rows per workgroup pass
constexpr int CE_ROWS_PER_BLOCK = 4 * CE_ROWS; // each group handles four rows

// logits and dlogits may be the same buffer (gradient in place), so neither is declared restrict: every
// read of a row element, the label's logit included, precedes in program order the store that replaces it.
__global__ __launch_bounds__(256) void softmax_ce_kernel(const float *logits, int64_t ld, int64_t n, int32_t c,
                                                         const int32_t *__restrict__ labels, float *dlogits,
                                                         int64_t ldd, double *__restrict__ partial)
{
    __shared__ double row_loss[CE_ROWS_PER_BLOCK];
    const int grp = threadIdx.x / CE_LPR, sub = threadIdx.x % CE_LPR;
    const float inv_n = 1.0f / (float)n;
    const bool vec = c <= 64 && c % 4 == 0 && ld % 4 == 0 && aligned16(logits) &&
                     (dlogits == nullptr || (ldd % 4 == 0 && aligned16(dlogits)));
    for (int q = 0; q < 4; ++q) {
        const int local = q * CE_ROWS + grp;
        const int64_t v = (int64_t)blockIdx.x * CE_ROWS_PER_BLOCK + local;
        double loss = 0.0;
        if (v < n) { // uniform within the 16-lane group
            const float *x = logits + v * ld;
            int y = labels[v];
            const bool bad = y < 0 || y >= c;
            if (bad) y = 0;
            if (vec) { // at most 64 classes, 16-byte accesses: the row lives in one float4 per lane, one exp per element
                const int j = 4 * sub;
                float4 q = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
                if (j < c) q = *reinterpret_cast<const float4 *>(x + j);
                float m = fmaxf(fmaxf(q.x, q.y), fmaxf(q.z, q.w));
#pragma unroll
                for (int s = 1; s < CE_LPR; s <<= 1) m = fmaxf(m, __shfl_xor(m, s, 64));
                float4 e = make_float4(0.f, 0.f, 0.f, 0.f);
                if (j < c) e = make_float4(expf(q.x - m), expf(q.y - m), expf(q.z - m), expf(q.w - m));
                float sum = (e.x + e.y) + (e.z + e.w);
#pragma unroll
                for (int s = 1; s < CE_LPR; s <<= 1) sum += __shfl_xor(sum, s, 64);
                loss = bad ? (double)NAN : (double)(m + logf(sum)) - (double)x[y];
                if (dlogits && j < c) {
                    const float inv_sum = 1.0f / sum;
                    float4 g4 = make_float4(e.x * inv_sum, e.y * inv_sum, e.z * inv_sum, e.w * inv_sum);
                    if (y == j) g4.x -= 1.f;
                    if (y == j + 1) g4.y -= 1.f;
                    if (y == j + 2) g4.z -= 1.f;
                    if (y == j + 3) g4.w -= 1.f;
                    g4.x *= inv_n; g4.y *= inv_n; g4.z *= inv_n; g4.w *= inv_n;
                    *reinterpret_cast<float4 *>(dlogits + v * ldd + j) = g4;
                }
            } else {
                float m = -INFINITY;
                for (int j = sub; j < c; j += CE_LPR) m = fmaxf(m, x[j]);
#pragma unroll
                for (int s = 1; s < CE_LPR; s <<= 1) m = fmaxf(m, __shfl_xor(m, s, 64));
                float sum = 0.f;
                for (int j = sub; j < c; j += CE_LPR) sum += expf(x[j] - m);
#pragma unroll
                for (int s = 1; s < CE_LPR; s <<= 1) sum += __shfl_xor(sum, s, 64);
                loss = bad ? (double)NAN : (double)(m + logf(sum)) - (double)x[y];
                if (dlogits) {
                    float *g = dlogits + v * ldd;
                    const float inv_sum = 1.0f / sum;
                    for (int j = sub; j < c; j += CE_LPR) g[j] = (expf(x[j] - m) * inv_sum - (j == y ? 1.f : 0.f)) * inv_n;
                }
            }
        }
        if (sub == 0) row_loss[local] = loss;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = 0.0;
        for (int i = 0; i < CE_ROWS_PER_BLOCK; ++i) s += row_loss[i];
        partial[blockIdx.x] = s;
    }
}

// loss = (sum of the workgroup sums) / n, fp64, fixed order: thread t adds every 256th sum, then the
// 256 thread sums are added in thread order.
__global__ __launch_bounds__(256) void ce_final_kernel(const double *__restrict__ partial, int64_t n_blocks, int64_t n,
                                                       float *__restrict__ loss)
{
    __shared__ double red[256];
    double s = 0.0;
    for (int64_t b = threadIdx.x; b < n_blocks; b += 256) s += partial[b];
    red[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int i = 0; i < 256; ++i) t += red[i];
        *loss = (float)(t / (double)n);
    }
}

inline int64_t ce_blocks(int64_t n) { return (n + CE_ROWS_PER_BLOCK - 1) / CE_ROWS_PER_BLOCK; }

} // namespace

} // namespace slicegcn

using namespace slicegcn;

extern "C" size_t slicegcn_softmax_ce_workspace_bytes(int64_t n)
{
    if (n < 1) return 0;
    return (size_t)round_up(ce_blocks(n) * (int64_t)sizeof(double), 256);
}

extern "C" int slicegcn_softmax_ce(const float *logits, int64_t ld, int64_t n, int32_t n_classes, const int32_t *labels,
                                   float *loss, float *dlogits, int64_t ldd, void *ws, size_t ws_bytes, void *stream_)
{
    SG_REQUIRE(logits && labels && loss, SLICEGCN_EINVAL, "softmax_ce: NULL logits, labels or loss");
    SG_REQUIRE(n >= 1 && n_classes >= 1, SLICEGCN_EINVAL, "softmax_ce: sizes must be >= 1");
    SG_REQUIRE(ld >= n_classes && (dlogits == nullptr || ldd >= n_classes), SLICEGCN_EINVAL,
               "softmax_ce: leading dimension smaller than the number of classes");
    const size_t need = slicegcn_softmax_ce_workspace_bytes(n);
    SG_REQUIRE(ws != nullptr && ws_bytes >= need, SLICEGCN_EWORKSPACE, "softmax_ce: workspace of %zu bytes, %zu needed",
               ws_bytes, need);
    SG_REQUIRE((reinterpret_cast<uintptr_t>(ws) & 255u) == 0, SLICEGCN_EINVAL, "softmax_ce: workspace not 256-byte aligned");
    hipStream_t stream = as_stream(stream_);
    const int64_t nb = ce_blocks(n);
    SG_REQUIRE(nb <= INT32_MAX, SLICEGCN_ERANGE, "softmax_ce: too many rows for one launch");
    double *partial = static_cast<double *>(ws);
    ProfScope prof(SLICEGCN_PROF_LOSS, n_classes, stream);
    softmax_ce_kernel<<<(unsigned)nb, 256, 0, stream>>>(logits, ld, n, n_classes, labels, dlogits, ldd, partial);
    SG_LAUNCH_CHECK();
    ce_final_kernel<<<1, 256, 0, stream>>>(partial, nb, n, loss);
    SG_LAUNCH_CHECK();
    return SLICEGCN_OK;
}
