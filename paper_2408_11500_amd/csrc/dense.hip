// Dense half of a SliceGCN layer (the layer equation's weight products, bias, ReLU and self
// term) and of its backward pass, plus the layer entry points that chain it with the
// aggregation kernels.
//
//   forward :  Hout = act(Z W_agg + b) + Hin W_self + b_self,  mask = [P > 0] bit-packed
//   backward:  dZ = (dHout * mask) W_agg^T,  T = dHout W_self^T            (pair kernel, transposed)
//              dW_agg = Z^T (dHout * mask), dW_self = Hin^T dHout, db, db_self   (reduce kernels)
//
// This file holds the portable fp32 FMA version of the pair kernel: register-blocked 4x4
// micro-tiles, operands staged through LDS in K-steps of 16.
#include "common.h"

namespace slicegcn {

namespace {

constexpr int KT = 16;

struct PairArgs {
    const float *A1; int64_t lda1; // forward: Z          backward: dHout (masked on load)
    const float *A2; int64_t lda2; // forward: Hin        backward: dHout           (NULL: no second product)
    const float *B1;               // W_agg  (w_in x w_out row-major)
    const float *B2;               // W_self (same shape) or NULL
    const float *bias1;            // forward only
    const float *bias2;            // forward only
    float *O1; int64_t ldo1;       // forward: Hout       backward: dZ
    float *O2; int64_t ldo2;       // backward: T (may be NULL)
    uint32_t *mask; int64_t mask_words; // forward: written (act = ReLU); backward: read
    int64_t n;
    int32_t K;     // reduction length: w_in forward, w_out backward
    int32_t Nout;  // output width:     w_out forward, w_in backward
    int32_t ldw;   // leading dimension of W (= w_out)
    int32_t act;
};

// CGP: column groups (of 4 columns) per block, 8 / 16 / 32.  Rows per block = (256 / CGP) * 4.
template <int CGP, bool BWD>
__global__ __launch_bounds__(256) void pair_gemm_kernel(const PairArgs a)
{
    constexpr int BM = (256 / CGP) * 4;
    constexpr int BN = CGP * 4;
    __shared__ float As1[BM][KT + 1];
    __shared__ float As2[BM][KT + 1];
    __shared__ __attribute__((aligned(16))) float Bs1[KT][BN];
    __shared__ __attribute__((aligned(16))) float Bs2[KT][BN];

    const int tid = threadIdx.x;
    const int rg = tid / CGP, cg = tid % CGP;
    const int64_t row0 = (int64_t)blockIdx.x * BM;
    const int col0 = blockIdx.y * BN;
    const bool two = a.A2 != nullptr && a.B2 != nullptr;

    float acc1[4][4], acc2[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) { acc1[i][j] = 0.f; acc2[i][j] = 0.f; }

    for (int k0 = 0; k0 < a.K; k0 += KT) {
        // ---- stage A tiles (BM x KT) ----
        for (int t = tid; t < BM * KT; t += 256) {
            const int r = t / KT, k = t % KT;
            const int64_t row = row0 + r;
            const int kk = k0 + k;
            float v1 = 0.f, v2 = 0.f;
            if (row < a.n && kk < a.K) {
                v1 = a.A1[row * a.lda1 + kk];
                if (BWD) {
                    if (a.mask) {
                        const uint32_t w = a.mask[row * a.mask_words + (kk >> 5)];
                        if (((w >> (kk & 31)) & 1u) == 0u) v1 = 0.f;
                    }
                }
                if (two) v2 = a.A2[row * a.lda2 + kk];
            }
            As1[r][k] = v1;
            As2[r][k] = v2;
        }
        // ---- stage B tiles (KT x BN) ----
        for (int t = tid; t < KT * BN; t += 256) {
            const int k = t / BN, j = t % BN;
            const int kk = k0 + k, col = col0 + j;
            float w1 = 0.f, w2 = 0.f;
            if (kk < a.K && col < a.Nout) {
                const int64_t idx = BWD ? (int64_t)col * a.ldw + kk : (int64_t)kk * a.ldw + col;
                w1 = a.B1[idx];
                if (two) w2 = a.B2[idx];
            }
            Bs1[k][j] = w1;
            Bs2[k][j] = w2;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < KT; ++k) {
            const float4 b1 = *reinterpret_cast<const float4 *>(&Bs1[k][cg * 4]);
            float x1[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) x1[i] = As1[rg * 4 + i][k];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc1[i][0] += x1[i] * b1.x; acc1[i][1] += x1[i] * b1.y;
                acc1[i][2] += x1[i] * b1.z; acc1[i][3] += x1[i] * b1.w;
            }
            if (two) {
                const float4 b2 = *reinterpret_cast<const float4 *>(&Bs2[k][cg * 4]);
                float x2[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) x2[i] = As2[rg * 4 + i][k];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    acc2[i][0] += x2[i] * b2.x; acc2[i][1] += x2[i] * b2.y;
                    acc2[i][2] += x2[i] * b2.z; acc2[i][3] += x2[i] * b2.w;
                }
            }
        }
        __syncthreads();
    }

    // ---- epilogue ----
    const int colb = col0 + cg * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t row = row0 + rg * 4 + i;
        float o1[4], o2[4];
        uint32_t bits = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = colb + j;
            if (!BWD) {
                float p = acc1[i][j] + ((a.bias1 && col < a.Nout) ? a.bias1[col] : 0.f);
                if (p > 0.f && col < a.Nout) bits |= 1u << j;
                const float r = (a.act == SLICEGCN_ACT_RELU) ? (p > 0.f ? p : 0.f) : p;
                float s = 0.f;
                if (two) s = acc2[i][j] + ((a.bias2 && col < a.Nout) ? a.bias2[col] : 0.f);
                o1[j] = r + s;
                o2[j] = 0.f;
            } else {
                o1[j] = acc1[i][j];
                o2[j] = acc2[i][j];
            }
        }
        if (!BWD && a.act == SLICEGCN_ACT_RELU) {
            // eight neighbouring lanes hold the 32 columns of one mask word of this row
            uint32_t word = bits << ((cg & 7) * 4);
            word |= __shfl_xor(word, 1, 64);
            word |= __shfl_xor(word, 2, 64);
            word |= __shfl_xor(word, 4, 64);
            const int widx = (col0 >> 5) + (cg >> 3);
            if ((cg & 7) == 0 && row < a.n && widx * 32 < a.Nout) a.mask[row * a.mask_words + widx] = word;
        }
        if (row < a.n) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int col = colb + j;
                if (col < a.Nout) {
                    a.O1[row * a.ldo1 + col] = o1[j];
                    if (BWD && a.O2) a.O2[row * a.ldo2 + col] = o2[j];
                }
            }
        }
    }
}

template <bool BWD>
int launch_pair(const PairArgs &a, hipStream_t stream)
{
    int cgp = 8;
    while (cgp < 32 && cgp * 4 < a.Nout) cgp <<= 1;
    const int bm = (256 / cgp) * 4, bn = cgp * 4;
    dim3 grid((unsigned)((a.n + bm - 1) / bm), (unsigned)((a.Nout + bn - 1) / bn));
    switch (cgp) {
    case 8: pair_gemm_kernel<8, BWD><<<grid, 256, 0, stream>>>(a); break;
    case 16: pair_gemm_kernel<16, BWD><<<grid, 256, 0, stream>>>(a); break;
    default: pair_gemm_kernel<32, BWD><<<grid, 256, 0, stream>>>(a); break;
    }
    SG_LAUNCH_CHECK();
    return SLICEGCN_OK;
}

// ---- weight-gradient reductions over the node axis ----------------------------------------
constexpr int RED_ROWS = 1024; // rows per block: fp32 chains stay this short
constexpr int RED_TILE = 32;   // output tile edge
constexpr int RED_RK = 32;     // rows staged per step

struct ReduceArgs {
    const float *Z; int64_t ldz;
    const float *Hin; int64_t ldi;      // NULL: no self term
    const float *dHout; int64_t ldo;
    const uint32_t *mask; int64_t mask_words; // NULL: all ones
    float *partial;                     // [n_row_blocks][stride]
    int64_t n;
    int32_t w_in, w_out;
    int32_t stride;                     // 2*w_in*w_out + 2*w_out
};

__global__ __launch_bounds__(256) void grad_partial_kernel(const ReduceArgs a)
{
    __shared__ float Zs[RED_RK][RED_TILE + 1];
    __shared__ float Hs[RED_RK][RED_TILE + 1];
    __shared__ float Ps[RED_RK][RED_TILE + 1];
    __shared__ float Gs[RED_RK][RED_TILE + 1];
    const int tid = threadIdx.x;
    const int ty = tid / 16, tx = tid % 16;
    const int i_base = blockIdx.y * RED_TILE, j_base = blockIdx.z * RED_TILE;
    const int64_t r_begin = (int64_t)blockIdx.x * RED_ROWS;
    const int64_t r_end = r_begin + RED_ROWS < a.n ? r_begin + RED_ROWS : a.n;
    const bool self = a.Hin != nullptr;

    float accA[2][2] = {{0.f, 0.f}, {0.f, 0.f}}, accS[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
    float accb[2] = {0.f, 0.f}, accbs[2] = {0.f, 0.f};

    for (int64_t r0 = r_begin; r0 < r_end; r0 += RED_RK) {
        for (int t = tid; t < RED_RK * RED_TILE; t += 256) {
            const int r = t / RED_TILE, c = t % RED_TILE;
            const int64_t row = r0 + r;
            float z = 0.f, h = 0.f, p = 0.f, gq = 0.f;
            if (row < r_end) {
                const int i = i_base + c, j = j_base + c;
                if (i < a.w_in) {
                    z = a.Z[row * a.ldz + i];
                    if (self) h = a.Hin[row * a.ldi + i];
                }
                if (j < a.w_out) {
                    gq = a.dHout[row * a.ldo + j];
                    p = gq;
                    if (a.mask) {
                        const uint32_t w = a.mask[row * a.mask_words + (j >> 5)];
                        if (((w >> (j & 31)) & 1u) == 0u) p = 0.f;
                    }
                }
            }
            Zs[r][c] = z; Hs[r][c] = h; Ps[r][c] = p; Gs[r][c] = gq;
        }
        __syncthreads();
#pragma unroll 8
        for (int r = 0; r < RED_RK; ++r) {
            const float z0 = Zs[r][ty * 2], z1 = Zs[r][ty * 2 + 1];
            const float p0 = Ps[r][tx * 2], p1 = Ps[r][tx * 2 + 1];
            accA[0][0] += z0 * p0; accA[0][1] += z0 * p1; accA[1][0] += z1 * p0; accA[1][1] += z1 * p1;
            const float g0 = Gs[r][tx * 2], g1 = Gs[r][tx * 2 + 1];
            if (self) {
                const float h0 = Hs[r][ty * 2], h1 = Hs[r][ty * 2 + 1];
                accS[0][0] += h0 * g0; accS[0][1] += h0 * g1; accS[1][0] += h1 * g0; accS[1][1] += h1 * g1;
            }
            if (ty == 0) { accb[0] += p0; accb[1] += p1; accbs[0] += g0; accbs[1] += g1; }
        }
        __syncthreads();
    }

    float *out = a.partial + (int64_t)blockIdx.x * a.stride;
    const int ww = a.w_in * a.w_out;
#pragma unroll
    for (int di = 0; di < 2; ++di)
#pragma unroll
        for (int dj = 0; dj < 2; ++dj) {
            const int i = i_base + ty * 2 + di, j = j_base + tx * 2 + dj;
            if (i < a.w_in && j < a.w_out) {
                out[i * a.w_out + j] = accA[di][dj];
                out[ww + i * a.w_out + j] = accS[di][dj];
            }
        }
    if (blockIdx.y == 0 && ty == 0) {
#pragma unroll
        for (int dj = 0; dj < 2; ++dj) {
            const int j = j_base + tx * 2 + dj;
            if (j < a.w_out) {
                out[2 * ww + j] = accb[dj];
                out[2 * ww + a.w_out + j] = accbs[dj];
            }
        }
    }
}

// Column sums of an n x w matrix (slice-encoding gradient): partial[block][w].
__global__ __launch_bounds__(256) void colsum_partial_kernel(const float *__restrict__ M, int64_t ld, int64_t n, int32_t w,
                                                             float *__restrict__ partial)
{
    const int64_t r_begin = (int64_t)blockIdx.x * RED_ROWS;
    const int64_t r_end = r_begin + RED_ROWS < n ? r_begin + RED_ROWS : n;
    // thread t owns column (t % cw) of every (256 / cw)-th row, cw = columns rounded up to a power of two <= 256
    __shared__ float red[256];
    for (int c0 = 0; c0 < w; c0 += 256) {
        const int cols = w - c0 < 256 ? w - c0 : 256;
        int cw = 1;
        while (cw < cols) cw <<= 1;
        const int lanes_r = 256 / cw;
        const int c = threadIdx.x % cw, rr = threadIdx.x / cw;
        float acc = 0.f;
        if (c < cols)
            for (int64_t r = r_begin + rr; r < r_end; r += lanes_r) acc += M[r * ld + c0 + c];
        red[threadIdx.x] = acc;
        __syncthreads();
        if (rr == 0 && c < cols) {
            float s = 0.f;
            for (int q = 0; q < lanes_r; ++q) s += red[q * cw + c];
            partial[(int64_t)blockIdx.x * w + c0 + c] = s;
        }
        __syncthreads();
    }
}

// Final stage: out[e] = sum over row blocks of partial[b][e], in fp64, fixed order.
// 32 elements x 32 parts per block of 1024 threads.
struct FinalDst { float *ptr[4]; int32_t begin[5]; }; // element ranges [begin[q], begin[q+1]) go to ptr[q]

__global__ __launch_bounds__(1024) void reduce_final_kernel(const float *__restrict__ partial, int64_t n_blocks,
                                                            int32_t stride, const FinalDst dst)
{
    __shared__ double red[32][33];
    const int el = threadIdx.x % 32, part = threadIdx.x / 32;
    const int64_t e = (int64_t)blockIdx.x * 32 + el;
    const int64_t per = (n_blocks + 31) / 32;
    const int64_t b0 = part * per, b1 = b0 + per < n_blocks ? b0 + per : n_blocks;
    double acc = 0.0;
    if (e < stride)
        for (int64_t b = b0; b < b1; ++b) acc += (double)partial[b * stride + e];
    red[part][el] = acc;
    __syncthreads();
    if (part == 0 && e < stride) {
        double s = 0.0;
        for (int q = 0; q < 32; ++q) s += red[q][el];
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (e >= dst.begin[q] && e < dst.begin[q + 1] && dst.ptr[q]) dst.ptr[q][e - dst.begin[q]] = (float)s;
    }
}

inline int64_t red_blocks(int64_t n) { return (n + RED_ROWS - 1) / RED_ROWS; }

int check_layer(const slicegcn_graph *g, const slicegcn_layer_desc *d, const slicegcn_layer_params *p, const char *who)
{
    SG_REQUIRE(g && d && p, SLICEGCN_EINVAL, "%s: NULL graph, desc or params", who);
    SG_REQUIRE(d->w_in >= 1 && d->w_out >= 1, SLICEGCN_EINVAL, "%s: widths must be >= 1", who);
    SG_REQUIRE(d->act == SLICEGCN_ACT_NONE || d->act == SLICEGCN_ACT_RELU, SLICEGCN_EINVAL, "%s: unknown act %d", who, d->act);
    SG_REQUIRE(p->W_agg != nullptr, SLICEGCN_EINVAL, "%s: W_agg is NULL", who);
    SG_REQUIRE(p->W_self != nullptr || p->b_self == nullptr, SLICEGCN_EINVAL, "%s: b_self without W_self", who);
    return SLICEGCN_OK;
}

int check_saved(const slicegcn_layer_desc *d, const slicegcn_layer_saved *s, const char *who)
{
    SG_REQUIRE(s && s->Z, SLICEGCN_EINVAL, "%s: saved or saved->Z is NULL", who);
    SG_REQUIRE(s->ldz >= d->w_in && s->ldz % 4 == 0 && aligned16(s->Z), SLICEGCN_EINVAL,
               "%s: saved->Z needs ldz >= w_in, ldz %% 4 == 0 and a 16-byte aligned base", who);
    if (d->act == SLICEGCN_ACT_RELU)
        SG_REQUIRE(s->mask && s->mask_words >= (d->w_out + 31) / 32, SLICEGCN_EINVAL,
                   "%s: mask is NULL or mask_words < ceil(w_out / 32)", who);
    return SLICEGCN_OK;
}

} // namespace

// shared with concat.hip
int launch_colsum(const float *M, int64_t ld, int64_t n, int32_t w, float *out, float *ws, hipStream_t stream)
{
    const int64_t nb = red_blocks(n);
    colsum_partial_kernel<<<(unsigned)nb, 256, 0, stream>>>(M, ld, n, w, ws);
    SG_LAUNCH_CHECK();
    FinalDst dst;
    dst.ptr[0] = out; dst.ptr[1] = dst.ptr[2] = dst.ptr[3] = nullptr;
    dst.begin[0] = 0; dst.begin[1] = dst.begin[2] = dst.begin[3] = dst.begin[4] = w;
    reduce_final_kernel<<<(unsigned)((w + 31) / 32), 1024, 0, stream>>>(ws, nb, w, dst);
    SG_LAUNCH_CHECK();
    return SLICEGCN_OK;
}

size_t colsum_workspace_bytes(int64_t n, int32_t w) { return (size_t)red_blocks(n) * (size_t)w * sizeof(float); }

} // namespace slicegcn

using namespace slicegcn;

extern "C" int slicegcn_layer_fwd(const slicegcn_graph *g, const slicegcn_layer_desc *desc,
                                  const slicegcn_layer_params *params, const float *Hin, int64_t ldi,
                                  float *Hout, int64_t ldo, slicegcn_layer_saved *saved, void *stream_)
{
    if (int rc = check_layer(g, desc, params, "layer_fwd")) return rc;
    SG_REQUIRE(Hin && Hout, SLICEGCN_EINVAL, "layer_fwd: NULL Hin or Hout");
    SG_REQUIRE(ldi >= desc->w_in && ldo >= desc->w_out, SLICEGCN_EINVAL, "layer_fwd: leading dimension too small");
    if (int rc = check_saved(desc, saved, "layer_fwd")) return rc;
    hipStream_t stream = as_stream(stream_);

    if (int rc = launch_spmm(g, g->fwd, Hin, ldi, desc->w_in, saved->Z, saved->ldz, nullptr, 0, stream)) return rc;

    PairArgs a;
    a.A1 = saved->Z; a.lda1 = saved->ldz;
    a.A2 = params->W_self ? Hin : nullptr; a.lda2 = ldi;
    a.B1 = params->W_agg; a.B2 = params->W_self;
    a.bias1 = params->b; a.bias2 = params->b_self;
    a.O1 = Hout; a.ldo1 = ldo; a.O2 = nullptr; a.ldo2 = 0;
    a.mask = desc->act == SLICEGCN_ACT_RELU ? saved->mask : nullptr; a.mask_words = saved->mask_words;
    a.n = g->n; a.K = desc->w_in; a.Nout = desc->w_out; a.ldw = desc->w_out; a.act = desc->act;
    ProfScope prof(SLICEGCN_PROF_DENSE_FWD, desc->w_out, stream);
    return launch_pair<false>(a, stream);
}

extern "C" size_t slicegcn_layer_bwd_workspace_bytes(int64_t n_nodes, const slicegcn_layer_desc *desc, int need_dHin)
{
    if (!desc || n_nodes < 1 || desc->w_in < 1 || desc->w_out < 1) return 0;
    const size_t stride = 2 * (size_t)desc->w_in * desc->w_out + 2 * (size_t)desc->w_out;
    size_t bytes = (size_t)round_up((int64_t)(red_blocks(n_nodes) * stride * sizeof(float)), 256);
    if (need_dHin) bytes += (size_t)round_up(n_nodes * round_up(desc->w_in, 4) * (int64_t)sizeof(float), 256);
    return bytes;
}

extern "C" int slicegcn_layer_bwd(const slicegcn_graph *g, const slicegcn_layer_desc *desc,
                                  const slicegcn_layer_params *params, const float *Hin, int64_t ldi,
                                  const slicegcn_layer_saved *saved, const float *dHout, int64_t ldo,
                                  float *dHin, int64_t ldgi, slicegcn_layer_grads *grads,
                                  void *ws, size_t ws_bytes, void *stream_)
{
    if (int rc = check_layer(g, desc, params, "layer_bwd")) return rc;
    SG_REQUIRE(Hin && dHout && grads, SLICEGCN_EINVAL, "layer_bwd: NULL Hin, dHout or grads");
    SG_REQUIRE(ldi >= desc->w_in && ldo >= desc->w_out, SLICEGCN_EINVAL, "layer_bwd: leading dimension too small");
    SG_REQUIRE(dHin == nullptr || ldgi >= desc->w_in, SLICEGCN_EINVAL, "layer_bwd: ldgi < w_in");
    if (int rc = check_saved(desc, saved, "layer_bwd")) return rc;
    const size_t need = slicegcn_layer_bwd_workspace_bytes(g->n, desc, dHin != nullptr);
    SG_REQUIRE(ws != nullptr && ws_bytes >= need, SLICEGCN_EWORKSPACE, "layer_bwd: workspace of %zu bytes, %zu needed",
               ws_bytes, need);
    SG_REQUIRE((reinterpret_cast<uintptr_t>(ws) & 255u) == 0, SLICEGCN_EINVAL, "layer_bwd: workspace not 256-byte aligned");
    hipStream_t stream = as_stream(stream_);
    const uint32_t *mask = desc->act == SLICEGCN_ACT_RELU ? saved->mask : nullptr;
    const int w_in = desc->w_in, w_out = desc->w_out;

    // ---- parameter gradients: per-row-block partial sums, then an fp64 combination ----
    float *partial = static_cast<float *>(ws);
    const int64_t nb = red_blocks(g->n);
    const int32_t stride = 2 * w_in * w_out + 2 * w_out;
    {
        ProfScope prof(SLICEGCN_PROF_GRAD_REDUCE, w_out, stream);
        ReduceArgs r;
        r.Z = saved->Z; r.ldz = saved->ldz;
        r.Hin = params->W_self ? Hin : nullptr; r.ldi = ldi;
        r.dHout = dHout; r.ldo = ldo;
        r.mask = mask; r.mask_words = saved->mask_words;
        r.partial = partial; r.n = g->n; r.w_in = w_in; r.w_out = w_out; r.stride = stride;
        dim3 grid((unsigned)nb, (unsigned)((w_in + RED_TILE - 1) / RED_TILE), (unsigned)((w_out + RED_TILE - 1) / RED_TILE));
        grad_partial_kernel<<<grid, 256, 0, stream>>>(r);
        SG_LAUNCH_CHECK();
        FinalDst dst;
        const int ww = w_in * w_out;
        dst.ptr[0] = grads->dW_agg;
        dst.ptr[1] = params->W_self ? grads->dW_self : nullptr;
        dst.ptr[2] = grads->db;
        dst.ptr[3] = params->W_self ? grads->db_self : nullptr;
        dst.begin[0] = 0; dst.begin[1] = ww; dst.begin[2] = 2 * ww; dst.begin[3] = 2 * ww + w_out; dst.begin[4] = stride;
        reduce_final_kernel<<<(unsigned)((stride + 31) / 32), 1024, 0, stream>>>(partial, nb, stride, dst);
        SG_LAUNCH_CHECK();
    }

    // ---- input gradient: dHin = A^^T (dP W_agg^T) + dHout W_self^T ----
    if (dHin) {
        const int64_t ldz = round_up(w_in, 4);
        float *dZ = reinterpret_cast<float *>(static_cast<char *>(ws) +
                                              round_up((int64_t)(nb * stride * sizeof(float)), 256));
        PairArgs a;
        a.A1 = dHout; a.lda1 = ldo;
        a.A2 = params->W_self ? dHout : nullptr; a.lda2 = ldo;
        a.B1 = params->W_agg; a.B2 = params->W_self;
        a.bias1 = a.bias2 = nullptr;
        a.O1 = dZ; a.ldo1 = ldz;
        a.O2 = params->W_self ? dHin : nullptr; a.ldo2 = ldgi;
        a.mask = const_cast<uint32_t *>(mask); a.mask_words = saved->mask_words;
        a.n = g->n; a.K = w_out; a.Nout = w_in; a.ldw = w_out; a.act = desc->act;
        {
            ProfScope prof(SLICEGCN_PROF_DENSE_BWD, w_in, stream);
            if (int rc = launch_pair<true>(a, stream)) return rc;
        }
        // padding columns of dZ are never read as data: the aggregation masks them on store
        if (int rc = launch_spmm(g, g->tr, dZ, ldz, w_in, dHin, ldgi, params->W_self ? dHin : nullptr, ldgi, stream)) return rc;
    }
    return SLICEGCN_OK;
}
