// Host-side slice strategy, direct feature slicing, slice encoding + concatenation and the
// error-text plumbing of the C ABI.
#include "common.h"

#include <cmath>

#include <algorithm>
#include <cstdarg>
#include <map>
#include <mutex>
#include <utility>
#include <vector>

namespace slicegcn {

namespace {
thread_local char g_err[512] = "";
}

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

// ---- per-kernel event timing --------------------------------------------------------------
namespace {
struct ProfRecord { int kind, width; hipEvent_t start, stop; bool closed; };
std::mutex g_prof_mutex;
bool g_prof_on = false;
std::vector<ProfRecord> g_prof;
std::vector<hipEvent_t> g_prof_pool; // events created ahead of time by slicegcn_profile_reserve

bool take_event(hipEvent_t *e)
{
    if (!g_prof_pool.empty()) {
        *e = g_prof_pool.back();
        g_prof_pool.pop_back();
        return true;
    }
    return hipEventCreate(e) == hipSuccess;
}
} // namespace

ProfScope::ProfScope(int kind, int width, hipStream_t stream) : slot_(-1), stream_(stream)
{
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (!g_prof_on) return;
    ProfRecord r{kind, width, nullptr, nullptr, false};
    if (!take_event(&r.start)) return;
    if (!take_event(&r.stop)) { (void)hipEventDestroy(r.start); return; }
    (void)hipEventRecord(r.start, stream);
    g_prof.push_back(r);
    slot_ = (int)g_prof.size() - 1;
}

ProfScope::~ProfScope()
{
    if (slot_ < 0) return;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (slot_ < (int)g_prof.size() && !g_prof[slot_].closed) {
        (void)hipEventRecord(g_prof[slot_].stop, stream_);
        g_prof[slot_].closed = true;
    }
}

namespace {

// dst[r, c] = src[r, c] (+ e[c]) for c < w, 0 for w <= c < w_pad.  One thread per element of
// the padded destination row, rows strided over the grid.  src and dst may be the same view (slice
// encoding in place), so they are not declared restrict: a thread reads only the element it writes.
__global__ __launch_bounds__(256) void copy_cols_kernel(const float *src, int64_t lds_, float *dst,
                                                        int64_t ldd, int64_t n, int32_t w, int32_t w_pad,
                                                        const float *__restrict__ e)
{
    const int64_t total = n * (int64_t)w_pad;
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
        const int64_t r = t / w_pad;
        const int c = (int)(t - r * w_pad);
        float v = 0.f;
        if (c < w) {
            v = src[r * lds_ + c];
            if (e) v += e[c];
        }
        dst[r * ldd + c] = v;
    }
}

// Same copy, 16 bytes per thread: needs aligned bases, leading dimensions, w and w_pad all multiples of 4.
__global__ __launch_bounds__(256) void copy_cols_vec_kernel(const float *src, int64_t lds_, float *dst,
                                                            int64_t ldd, int64_t n, int32_t w, int32_t w_pad,
                                                            const float *__restrict__ e)
{
    const int q = w_pad >> 2; // float4 per destination row
    const int64_t total = n * (int64_t)q;
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
        const int64_t r = t / q;
        const int c = (int)(t - r * q) * 4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (c < w) {
            v = *reinterpret_cast<const float4 *>(src + r * lds_ + c);
            if (e) {
                const float4 b = *reinterpret_cast<const float4 *>(e + c);
                v.x += b.x; v.y += b.y; v.z += b.z; v.w += b.w;
            }
        }
        *reinterpret_cast<float4 *>(dst + r * ldd + c) = v;
    }
}

// dst[r, c] = scale[r] * src[r, c] for c < w, 0 for w <= c < w_pad (one thread per element of the padded row)
// src and dst may be the same view (scaling in place): a thread reads only the element it writes.
__global__ __launch_bounds__(256) void scale_rows_kernel(const float *src, int64_t lds_, float *dst, int64_t ldd,
                                                         int64_t n, int32_t w, int32_t w_pad, const float *__restrict__ scale)
{
    const int64_t total = n * (int64_t)w_pad;
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
        const int64_t r = t / w_pad;
        const int c = (int)(t - r * w_pad);
        dst[r * ldd + c] = c < w ? scale[r] * src[r * lds_ + c] : 0.f;
    }
}

// dst[r, c] += src[r, c] for c < w; 16 bytes per thread when VEC (aligned bases, lds and w multiples of 4).
template <bool VEC>
__global__ __launch_bounds__(256) void accumulate_kernel(float *__restrict__ dst, int64_t ldd, const float *__restrict__ src,
                                                         int64_t lds_, int64_t n, int32_t w)
{
    const int q = VEC ? w >> 2 : w; // elements (float4 or float) per row
    const int64_t total = n * (int64_t)q;
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
        const int64_t r = t / q;
        const int c = (int)(t - r * q);
        if (VEC) {
            float4 d = *reinterpret_cast<const float4 *>(dst + r * ldd + 4 * c);
            const float4 v = *reinterpret_cast<const float4 *>(src + r * lds_ + 4 * c);
            d.x += v.x; d.y += v.y; d.z += v.z; d.w += v.w;
            *reinterpret_cast<float4 *>(dst + r * ldd + 4 * c) = d;
        } else {
            dst[r * ldd + c] += src[r * lds_ + c];
        }
    }
}

// One Adam step on `count` contiguous parameters (bias-corrected, optional L2 weight decay).
// c1 = 1 - beta1^t and c2 = 1 - beta2^t are computed on the host in fp64.
__global__ __launch_bounds__(256) void adam_kernel(float *__restrict__ p, const float *__restrict__ g, float *__restrict__ m,
                                                   float *__restrict__ v, int64_t count, float lr, float beta1, float omb1,
                                                   float beta2, float omb2, float eps, float wd, float inv_c1, float inv_c2)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) {
        const float pi = p[i];
        const float gi = g[i] + wd * pi;
        const float mi = beta1 * m[i] + omb1 * gi; // omb = 1 - beta, rounded from fp64 on the host
        const float vi = beta2 * v[i] + omb2 * gi * gi;
        m[i] = mi;
        v[i] = vi;
        p[i] = pi - lr * (mi * inv_c1) / (sqrtf(vi * inv_c2) + eps);
    }
}

inline unsigned grid_for(int64_t total)
{
    const int64_t b = (total + 255) / 256;
    return (unsigned)(b < 1 ? 1 : (b > 1048576 ? 1048576 : b));
}

int launch_copy_cols(const float *src, int64_t lds_, float *dst, int64_t ldd, int64_t n, int32_t w, int32_t w_pad,
                     const float *e, hipStream_t stream)
{
    const bool vec = aligned16(src) && aligned16(dst) && (!e || aligned16(e)) && lds_ % 4 == 0 && ldd % 4 == 0 &&
                     w % 4 == 0 && w_pad % 4 == 0;
    if (vec)
        copy_cols_vec_kernel<<<grid_for(n * (w_pad / 4)), 256, 0, stream>>>(src, lds_, dst, ldd, n, w, w_pad, e);
    else
        copy_cols_kernel<<<grid_for(n * w_pad), 256, 0, stream>>>(src, lds_, dst, ldd, n, w, w_pad, e);
    SG_LAUNCH_CHECK();
    return SLICEGCN_OK;
}

} // namespace
} // namespace slicegcn

using namespace slicegcn;

extern "C" int slicegcn_accumulate(float *dst, int64_t ldd, const float *src, int64_t lds_, int64_t n, int32_t w, void *stream)
{
    SG_REQUIRE(dst && src, SLICEGCN_EINVAL, "accumulate: NULL pointer");
    SG_REQUIRE(n >= 1 && w >= 1 && ldd >= w && lds_ >= w, SLICEGCN_EINVAL, "accumulate: sizes or leading dimensions too small");
    ProfScope prof(SLICEGCN_PROF_ACCUM, w, as_stream(stream));
    const bool vec = aligned16(dst) && aligned16(src) && ldd % 4 == 0 && lds_ % 4 == 0 && w % 4 == 0;
    if (vec) accumulate_kernel<true><<<grid_for(n * (w / 4)), 256, 0, as_stream(stream)>>>(dst, ldd, src, lds_, n, w);
    else accumulate_kernel<false><<<grid_for(n * (int64_t)w), 256, 0, as_stream(stream)>>>(dst, ldd, src, lds_, n, w);
    SG_LAUNCH_CHECK();
    return SLICEGCN_OK;
}

extern "C" int slicegcn_adam_step(float *param, const float *grad, float *m, float *v, int64_t count, double lr, double beta1,
                                  double beta2, double eps, double weight_decay, int32_t step, void *stream)
{
    SG_REQUIRE(param && grad && m && v, SLICEGCN_EINVAL, "adam_step: NULL pointer");
    SG_REQUIRE(count >= 1 && step >= 1, SLICEGCN_EINVAL, "adam_step: count and step must be >= 1");
    SG_REQUIRE(beta1 >= 0.0 && beta1 < 1.0 && beta2 >= 0.0 && beta2 < 1.0 && eps >= 0.0, SLICEGCN_EINVAL,
               "adam_step: betas must lie in [0, 1) and eps must not be negative");
    const double c1 = 1.0 - pow(beta1, (double)step), c2 = 1.0 - pow(beta2, (double)step);
    adam_kernel<<<grid_for(count), 256, 0, as_stream(stream)>>>(param, grad, m, v, count, (float)lr, (float)beta1,
                                                                (float)(1.0 - beta1), (float)beta2, (float)(1.0 - beta2), (float)eps,
                                                                (float)weight_decay, (float)(1.0 / c1), (float)(1.0 / c2));
    SG_LAUNCH_CHECK();
    return SLICEGCN_OK;
}

extern "C" double slicegcn_cosine_lr(double lr_max, double lr_min, int32_t t, int32_t t_max)
{
    if (t_max < 1) return lr_max;
    return lr_min + 0.5 * (lr_max - lr_min) * (1.0 + cos(3.14159265358979323846 * (double)t / (double)t_max));
}

extern "C" int slicegcn_slice_strategy(int32_t in_d, int32_t p, double slice_size_scale,
                                       int32_t *starts, int32_t *ends, int32_t *slice_size)
{
    SG_REQUIRE(starts && ends && slice_size, SLICEGCN_EINVAL, "slice_strategy: NULL output");
    SG_REQUIRE(in_d >= 1 && p >= 1 && p <= in_d, SLICEGCN_EINVAL, "slice_strategy: need 1 <= p <= in_d (p=%d, in_d=%d)", p, in_d);
    SG_REQUIRE(slice_size_scale > 0.0, SLICEGCN_EINVAL, "slice_strategy: slice_size_scale must be positive");
    const int32_t size = in_d / p + (in_d % p != 0);
    const double scaled = (double)size * slice_size_scale;
    SG_REQUIRE(scaled >= 1.0 && scaled <= (double)in_d, SLICEGCN_EINVAL,
               "slice_strategy: scaled slice width %.3f outside [1, in_d]", scaled);
    const int64_t width = (int64_t)scaled; // truncation, as the algorithm's int() does
    for (int32_t i = 0; i < p; ++i) {
        int64_t s = (int64_t)i * size, e = s + width;
        if (e > in_d) { // the slice that passes the end moves left to end at in_d
            s -= e - in_d;
            e = in_d;
        }
        SG_REQUIRE(s >= 0, SLICEGCN_EINVAL, "slice_strategy: slice %d would start before column 0", i);
        starts[i] = (int32_t)s;
        ends[i] = (int32_t)e;
    }
    *slice_size = size;
    return SLICEGCN_OK;
}

extern "C" int slicegcn_slice_feature(const float *X, int64_t n, int64_t ldx, int32_t start, int32_t end,
                                      float *Xs, int64_t ldxs, void *stream)
{
    SG_REQUIRE(X && Xs, SLICEGCN_EINVAL, "slice_feature: NULL pointer");
    SG_REQUIRE(n >= 1, SLICEGCN_EINVAL, "slice_feature: n < 1");
    SG_REQUIRE(start >= 0 && start < end && end <= ldx, SLICEGCN_EINVAL,
               "slice_feature: need 0 <= start < end <= ldx (start=%d, end=%d, ldx=%lld)", start, end, (long long)ldx);
    SG_REQUIRE(ldxs >= end - start, SLICEGCN_EINVAL, "slice_feature: ldxs smaller than the slice width");
    SG_REQUIRE(ldxs <= INT32_MAX, SLICEGCN_EINVAL, "slice_feature: ldxs too large");
    return launch_copy_cols(X + start, ldx, Xs, ldxs, n, end - start, (int32_t)ldxs, nullptr, as_stream(stream));
}

extern "C" int slicegcn_scale_rows(const slicegcn_graph *g, const float *X, int64_t ldx, int32_t width, float *Xs, int64_t ldxs,
                                   void *stream)
{
    SG_REQUIRE(g && X && Xs, SLICEGCN_EINVAL, "scale_rows: NULL pointer");
    SG_REQUIRE(width >= 1 && ldx >= width && ldxs >= width && ldxs <= INT32_MAX, SLICEGCN_EINVAL,
               "scale_rows: need 1 <= width <= ldx, ldxs");
    scale_rows_kernel<<<grid_for(g->n * ldxs), 256, 0, as_stream(stream)>>>(X, ldx, Xs, ldxs, g->n, width, (int32_t)ldxs, g->dinv);
    SG_LAUNCH_CHECK();
    return SLICEGCN_OK;
}

extern "C" int slicegcn_concat(int32_t k, const float *const *Hs, const int64_t *lds, const int32_t *widths,
                               const float *E, int64_t lde, int64_t n, float *H, int64_t ldh, void *stream)
{
    SG_REQUIRE(Hs && lds && widths && H, SLICEGCN_EINVAL, "concat: NULL pointer");
    SG_REQUIRE(k >= 1 && n >= 1, SLICEGCN_EINVAL, "concat: k and n must be >= 1");
    int64_t total = 0;
    int32_t wmax = 0;
    for (int32_t i = 0; i < k; ++i) {
        SG_REQUIRE(Hs[i] != nullptr, SLICEGCN_EINVAL, "concat: Hs[%d] is NULL", i);
        SG_REQUIRE(widths[i] >= 1 && lds[i] >= widths[i], SLICEGCN_EINVAL, "concat: bad width or ld of slice %d", i);
        total += widths[i];
        wmax = widths[i] > wmax ? widths[i] : wmax;
    }
    SG_REQUIRE(total <= ldh, SLICEGCN_EINVAL, "concat: sum of widths %lld exceeds ldh %lld", (long long)total, (long long)ldh);
    SG_REQUIRE(E == nullptr || lde >= wmax, SLICEGCN_EINVAL, "concat: lde smaller than the widest slice");
    int64_t off = 0;
    ProfScope prof(SLICEGCN_PROF_CONCAT, wmax, as_stream(stream));
    for (int32_t i = 0; i < k; ++i) {
        const bool in_place = Hs[i] == H + off && lds[i] == ldh;
        if (!(in_place && E == nullptr)) {
            if (int rc = launch_copy_cols(Hs[i], lds[i], H + off, ldh, n, widths[i], widths[i],
                                          E ? E + (int64_t)i * lde : nullptr, as_stream(stream)))
                return rc;
        }
        off += widths[i];
    }
    return SLICEGCN_OK;
}

extern "C" size_t slicegcn_concat_bwd_workspace_bytes(int64_t n, int32_t k, const int32_t *widths)
{
    if (n < 1 || k < 1 || !widths) return 0;
    int64_t total = 0;
    for (int32_t i = 0; i < k; ++i) total += widths[i] > 0 ? widths[i] : 0;
    if (total < 1 || total > INT32_MAX) return 0;
    return (size_t)round_up((int64_t)colsum_workspace_bytes(n, (int32_t)total), 256);
}

extern "C" int slicegcn_concat_bwd(int32_t k, const float *dH, int64_t ldh, int64_t n, const int32_t *widths,
                                   float *const *dHs, const int64_t *lds, float *dE, int64_t lde,
                                   void *ws, size_t ws_bytes, void *stream)
{
    SG_REQUIRE(dH && widths, SLICEGCN_EINVAL, "concat_bwd: NULL pointer");
    SG_REQUIRE(k >= 1 && n >= 1, SLICEGCN_EINVAL, "concat_bwd: k and n must be >= 1");
    int64_t total = 0;
    int32_t wmax = 0;
    for (int32_t i = 0; i < k; ++i) {
        SG_REQUIRE(widths[i] >= 1, SLICEGCN_EINVAL, "concat_bwd: width of slice %d < 1", i);
        if (dHs && dHs[i]) SG_REQUIRE(lds && lds[i] >= widths[i], SLICEGCN_EINVAL, "concat_bwd: bad ld of slice %d", i);
        total += widths[i];
        wmax = widths[i] > wmax ? widths[i] : wmax;
    }
    SG_REQUIRE(total <= ldh, SLICEGCN_EINVAL, "concat_bwd: sum of widths exceeds ldh");
    if (dE) {
        SG_REQUIRE(lde >= wmax, SLICEGCN_EINVAL, "concat_bwd: lde smaller than the widest slice");
        const size_t need = slicegcn_concat_bwd_workspace_bytes(n, k, widths);
        SG_REQUIRE(ws && ws_bytes >= need, SLICEGCN_EWORKSPACE, "concat_bwd: workspace of %zu bytes, %zu needed", ws_bytes, need);
    }
    int64_t off = 0;
    ProfScope prof(SLICEGCN_PROF_CONCAT, wmax, as_stream(stream));
    for (int32_t i = 0; i < k; ++i) {
        if (dHs && dHs[i] && !(dHs[i] == dH + off && lds[i] == ldh)) {
            if (int rc = launch_copy_cols(dH + off, ldh, dHs[i], lds[i], n, widths[i], widths[i], nullptr, as_stream(stream)))
                return rc;
        }
        off += widths[i];
    }
    if (dE) { // one pass over dH gives the column sums of every slice; each slice then takes its block
        if (int rc = launch_colsum_partial(dH, ldh, n, (int32_t)total, static_cast<float *>(ws), as_stream(stream))) return rc;
        off = 0;
        for (int32_t i = 0; i < k; ++i) {
            if (int rc = launch_colsum_final(static_cast<float *>(ws) + off, n, (int32_t)total, widths[i],
                                             dE + (int64_t)i * lde, as_stream(stream)))
                return rc;
            off += widths[i];
        }
    }
    return SLICEGCN_OK;
}

extern "C" int slicegcn_profile_begin(void)
{
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    for (auto &r : g_prof) { g_prof_pool.push_back(r.start); g_prof_pool.push_back(r.stop); }
    g_prof.clear();
    g_prof_on = true;
    return SLICEGCN_OK;
}

extern "C" int slicegcn_profile_reserve(int32_t scopes)
{
    SG_REQUIRE(scopes >= 0, SLICEGCN_EINVAL, "profile_reserve: negative count");
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    while ((int64_t)g_prof_pool.size() < 2 * (int64_t)scopes) {
        hipEvent_t e;
        SG_HIP(hipEventCreate(&e));
        g_prof_pool.push_back(e);
    }
    return SLICEGCN_OK;
}

extern "C" int slicegcn_profile_end(slicegcn_profile_entry *entries, int32_t capacity, int32_t *count)
{
    SG_REQUIRE(count != nullptr && (entries != nullptr || capacity == 0), SLICEGCN_EINVAL, "profile_end: NULL output");
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    g_prof_on = false;
    SG_HIP(hipDeviceSynchronize());
    struct Acc { int64_t launches = 0; double total = 0.0, lo = 0.0, hi = 0.0; std::vector<float> all; };
    std::map<std::pair<int, int>, Acc> sum;
    for (auto &r : g_prof) {
        float ms = 0.f;
        if (r.closed && hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess) {
            auto &e = sum[{r.kind, r.width}];
            if (e.launches == 0 || ms < e.lo) e.lo = ms;
            if (e.launches == 0 || ms > e.hi) e.hi = ms;
            e.launches += 1;
            e.total += (double)ms;
            e.all.push_back(ms);
        }
        g_prof_pool.push_back(r.start); // kept for the next profiled region
        g_prof_pool.push_back(r.stop);
    }
    g_prof.clear();
    int32_t i = 0;
    for (auto &kv : sum) {
        if (i < capacity) {
            entries[i].kind = kv.first.first;
            entries[i].width = kv.first.second;
            entries[i].launches = kv.second.launches;
            entries[i].total_ms = kv.second.total;
            entries[i].min_ms = kv.second.lo;
            entries[i].max_ms = kv.second.hi;
            std::vector<float> &v = kv.second.all;
            std::sort(v.begin(), v.end());
            const size_t h = v.size() / 2;
            entries[i].median_ms = v.empty() ? 0.0 : (v.size() % 2 ? (double)v[h] : 0.5 * ((double)v[h - 1] + (double)v[h]));
        }
        ++i;
    }
    *count = i;
    return SLICEGCN_OK;
}

extern "C" const char *slicegcn_strerror(int status)
{
    switch (status) {
    case SLICEGCN_OK: return "ok";
    case SLICEGCN_EINVAL: return "invalid argument";
    case SLICEGCN_ERANGE: return "value out of range";
    case SLICEGCN_ENOMEM: return "out of memory";
    case SLICEGCN_EHIP: return "HIP runtime error";
    case SLICEGCN_EUNSUPPORTED: return "unsupported request";
    case SLICEGCN_EWORKSPACE: return "workspace missing or too small";
    default: return "unknown status";
    }
}

extern "C" const char *slicegcn_last_error(void) { return g_err; }
