// Dense half of a SliceGCN layer (the layer equation's weight products, bias, ReLU and self
// term) and of its backward pass, plus the layer entry points that chain it with the
// aggregation kernels.
//
//   forward :  Hout = act(Z W_agg + b) + Hin W_self + b_self,  mask = [P > 0] bit-packed
//   backward:  dZ = (dHout * mask) W_agg^T,  T = dHout W_self^T            (pair kernel, transposed)
//              dW_agg = Z^T (dHout * mask), dW_self = Hin^T dHout, db, db_self   (reduce kernels)
//
// Every product runs on v_mfma_f32_32x32x2_f32 tiles (fp32 in, fp32 accumulate), one 32-row strip per
// wavefront, operands staged through LDS with coalesced 16-byte loads.
// Lane layout of the 32x32x2 fp32 MFMA (64 lanes, l = lane): A operand = A[m = l % 32][k = l / 32],
// B operand = B[k = l / 32][n = l % 32], accumulator register r (0..15) = C[8*(r/4) + 4*(l/32) + r%4][l % 32].
#include "common.h"

namespace slicegcn {

namespace {

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
    // Scaled layout (activations stored as D~^-1/2 H, the operand form the aggregation wants): per-row factors.
    const float *scale2 = nullptr;   // forward: rows of A2 are multiplied by scale2[row] when read (sqrt(d~): undoes the scaling of Hin)
    const float *scale_o1 = nullptr; // rows of O1 are multiplied by scale_o1[row] (forward: on store; backward: dZ rows, folded into dP)
};

__device__ inline void scale4(float4 &v, float s) { v.x *= s; v.y *= s; v.z *= s; v.w *= s; }

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Four floats of row `row` starting at column k (k % 4 == 0), zero beyond column K.
__device__ inline float4 load_k4(const float *__restrict__ base, int64_t ld, int64_t row, int k, int K, bool vec_ok)
{
    const float *p = base + row * ld + k;
    if (vec_ok && k + 4 <= K) return *reinterpret_cast<const float4 *>(p);
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (k < K) v.x = p[0];
    if (k + 1 < K) v.y = p[1];
    if (k + 2 < K) v.z = p[2];
    if (k + 3 < K) v.w = p[3];
    return v;
}

__device__ inline float pick(const float4 &v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }

// MFMA pair kernel.  Workgroup = 4 wavefronts = 128 rows (32 per wavefront) x NT*32 output
// columns.  The reduction axis is walked in chunks of 32: the A tile(s) (128 x 32) and the B
// tile(s) (32 x NT*32) are staged in LDS; a lane then reads 4 consecutive k of its row with one
// 16-byte LDS read and feeds them to four MFMA steps (the k pairing of a step is (k, k+4), the B
// tile is read with the same pairing).  The global loads of chunk c+1 are issued into registers
// before the MFMAs of chunk c and written to LDS after them, so memory latency hides behind the
// matrix instructions.  TWO: second product A2 B2 (self term / T output) present.
// Workgroups are numbered so that the column tiles of one row tile run back to back on the same
// XCD (workgroup b goes to XCD b mod 8): the A tile is fetched from HBM once and re-read from L2.
template <int NT, bool BWD, bool TWO>
__global__ __launch_bounds__(256) void pair_mfma_kernel(const PairArgs a, int n_col_tiles)
{
    constexpr int BM = 128, KC = 32, AS = KC + 4, BN = NT * 32;
    constexpr int BPT = KC * BN / 256; // B-tile elements per thread and chunk
    __shared__ __attribute__((aligned(16))) float As1[BM][AS];
    __shared__ __attribute__((aligned(16))) float As2[TWO ? BM : 1][AS];
    // the B tiles are kept column-major ([column][k], the A tiles' row stride), so that a lane reads the four
    // consecutive k of its column with one 16-byte LDS read, as it does for A: one LDS read per four MFMAs
    __shared__ __attribute__((aligned(16))) float Bt1[BN][AS];
    __shared__ __attribute__((aligned(16))) float Bt2[TWO ? BN : 1][AS];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int m = lane & 31, h = lane >> 5;
    const int64_t b = blockIdx.x;
    const int64_t row_tile = (b / (8 * n_col_tiles)) * 8 + (b % 8);
    const int col_tile = (int)((b / 8) % n_col_tiles);
    const int64_t row0 = row_tile * BM;
    if (row0 >= a.n) return; // uniform per workgroup (the last group of 8 row tiles may be partial)
    const int col0 = col_tile * BN;
    const bool vec1 = aligned16(a.A1) && (a.lda1 % 4 == 0);
    const bool vec2 = TWO && !BWD && aligned16(a.A2) && (a.lda2 % 4 == 0);

    floatx16 acc1[NT], acc2[TWO ? NT : 1];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc1[t][r] = 0.f; if (TWO) acc2[t][r] = 0.f; }

    float4 ra1[4], ra2[TWO ? 4 : 1];
    float rs[4]; // per-row factor of this thread's four rows (applied when the registers go to LDS, so that the loads stay in flight)
    float rb1[BPT], rb2[TWO ? BPT : 1];
    auto fetch = [&](int k0) { // this thread's share of the tiles of chunk k0, into registers
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int idx = tid + it * 256;
            const int r = idx >> 3, c4 = (idx & 7) * 4;
            const int64_t row = row0 + r;
            const int kk = k0 + c4;
            float4 v1 = make_float4(0.f, 0.f, 0.f, 0.f), v2 = v1;
            float f = 1.f;
            if (row < a.n && kk < a.K) {
                v1 = load_k4(a.A1, a.lda1, row, kk, a.K, vec1);
                if (!BWD) {
                    if (TWO) {
                        v2 = load_k4(a.A2, a.lda2, row, kk, a.K, vec2);
                        if (a.scale2) f = a.scale2[row];
                    }
                } else {
                    if (TWO) v2 = v1;
                    if (a.mask) { // four mask bits of this row; kk % 4 == 0 keeps them inside one word
                        const uint32_t bits = a.mask[row * a.mask_words + (kk >> 5)] >> (kk & 31);
                        if (!(bits & 1u)) v1.x = 0.f;
                        if (!(bits & 2u)) v1.y = 0.f;
                        if (!(bits & 4u)) v1.z = 0.f;
                        if (!(bits & 8u)) v1.w = 0.f;
                    }
                    if (a.scale_o1) f = a.scale_o1[row];
                }
            }
            ra1[it] = v1;
            rs[it] = f;
            if (TWO) ra2[it] = v2;
        }
#pragma unroll
        for (int it = 0; it < BPT; ++it) {
            const int idx = tid + it * 256;
            // consecutive threads walk the contiguous axis of W: columns forward, k backward (W^T)
            const int kk = BWD ? idx % KC : idx / BN, j = BWD ? idx / KC : idx % BN;
            const int gk = k0 + kk, col = col0 + j;
            float w1 = 0.f, w2 = 0.f;
            if (gk < a.K && col < a.Nout) {
                const int64_t id = BWD ? (int64_t)col * a.ldw + gk : (int64_t)gk * a.ldw + col;
                w1 = a.B1[id];
                if (TWO) w2 = a.B2[id];
            }
            rb1[it] = w1;
            if (TWO) rb2[it] = w2;
        }
    };
    auto stash = [&]() { // registers -> LDS
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int idx = tid + it * 256;
            const int r = idx >> 3, c4 = (idx & 7) * 4;
            if (BWD && a.scale_o1) scale4(ra1[it], rs[it]);         // rows of the first product only (dZ rows)
            if (!BWD && TWO && a.scale2) scale4(ra2[it], rs[it]);   // rows of Hin kept scaled
            *reinterpret_cast<float4 *>(&As1[r][c4]) = ra1[it];
            if (TWO) *reinterpret_cast<float4 *>(&As2[r][c4]) = ra2[it];
        }
#pragma unroll
        for (int it = 0; it < BPT; ++it) {
            const int idx = tid + it * 256;
            const int kk = BWD ? idx % KC : idx / BN, j = BWD ? idx / KC : idx % BN;
            Bt1[j][kk] = rb1[it];
            if (TWO) Bt2[j][kk] = rb2[it];
        }
    };

    fetch(0);
    for (int k0 = 0; k0 < a.K; k0 += KC) {
        stash();
        __syncthreads();
        if (k0 + KC < a.K) fetch(k0 + KC);
#pragma unroll
        for (int j8 = 0; j8 < 4; ++j8) {
            const float4 a1 = *reinterpret_cast<const float4 *>(&As1[wave * 32 + m][8 * j8 + 4 * h]);
            float4 a2 = a1;
            if (TWO) a2 = *reinterpret_cast<const float4 *>(&As2[wave * 32 + m][8 * j8 + 4 * h]);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const float4 b1 = *reinterpret_cast<const float4 *>(&Bt1[t * 32 + m][8 * j8 + 4 * h]);
                float4 b2 = b1;
                if (TWO) b2 = *reinterpret_cast<const float4 *>(&Bt2[t * 32 + m][8 * j8 + 4 * h]);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    acc1[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(pick(a1, i), pick(b1, i), acc1[t], 0, 0, 0);
                    if (TWO) acc2[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(pick(a2, i), pick(b2, i), acc2[t], 0, 0, 0);
                }
            }
        }
        __syncthreads();
    }

    // ---- epilogue: register r of a lane is row 8*(r/4) + 4*h + r%4 of the strip, column m of tile t ----
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int col = col0 + t * 32 + m;
        const bool col_ok = col < a.Nout;
        const float bias1 = (!BWD && a.bias1 && col_ok) ? a.bias1[col] : 0.f;
        const float bias2 = (!BWD && TWO && a.bias2 && col_ok) ? a.bias2[col] : 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t row = row0 + wave * 32 + 8 * (r / 4) + 4 * h + (r % 4);
            if (!BWD) {
                const float p = acc1[t][r] + bias1;
                const bool pos = p > 0.f && col_ok;
                if (a.act == SLICEGCN_ACT_RELU) {
                    // lanes 0..31 hold one row of this tile, lanes 32..63 the row four below it
                    const unsigned long long bal = __ballot(pos);
                    if (m == 0 && row < a.n && col0 + t * 32 < a.Nout)
                        a.mask[row * a.mask_words + ((col0 + t * 32) >> 5)] = h ? (uint32_t)(bal >> 32) : (uint32_t)bal;
                }
                const float rl = (a.act == SLICEGCN_ACT_RELU) ? (p > 0.f ? p : 0.f) : p;
                const float o = rl + (TWO ? acc2[t][r] + bias2 : 0.f);
                if (row < a.n && col_ok) a.O1[row * a.ldo1 + col] = a.scale_o1 ? o * a.scale_o1[row] : o;
            } else {
                if (row < a.n && col_ok) {
                    a.O1[row * a.ldo1 + col] = acc1[t][r];
                    if (TWO && a.O2) a.O2[row * a.ldo2 + col] = acc2[t][r];
                }
            }
        }
    }
}

// Variant for reduction lengths K <= 64 (every layer of the narrow-slice workloads): the weight
// tiles are staged in LDS once per workgroup, which then walks over row tiles; each lane loads the
// k values it feeds to the MFMA straight from global memory (16-byte loads, 32 contiguous bytes
// per row and instruction), so there is no LDS round trip or barrier per row tile and all loads of
// a tile are in flight at once.
template <int NT, int KCH, bool BWD> // KCH: number of 32-wide K chunks (1 or 2)
__global__ __launch_bounds__(256) void pair_mfma_direct_kernel(const PairArgs a)
{
    constexpr int BN = NT * 32, KK = KCH * 32;
    __shared__ float Bs1[KK][BN];
    __shared__ float Bs2[KK][BN];
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int m = lane & 31, h = lane >> 5;
    const int col0 = blockIdx.y * BN;
    const bool two = a.A2 != nullptr && a.B2 != nullptr;
    const bool vec1 = aligned16(a.A1) && (a.lda1 % 4 == 0);
    const bool vec2 = two && aligned16(a.A2) && (a.lda2 % 4 == 0);

    for (int idx = tid; idx < KK * BN; idx += 256) {
        const int kk = idx / BN, j = idx % BN;
        const int col = col0 + j;
        float w1 = 0.f, w2 = 0.f;
        if (kk < a.K && col < a.Nout) {
            const int64_t id = BWD ? (int64_t)col * a.ldw + kk : (int64_t)kk * a.ldw + col;
            w1 = a.B1[id];
            if (two) w2 = a.B2[id];
        }
        Bs1[kk][j] = w1;
        Bs2[kk][j] = w2;
    }
    __syncthreads();

    const int64_t n_tiles = (a.n + 127) / 128;
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        // the weight tiles are re-read from LDS for every row tile: keeping them in registers across
        // the loop would cost 64 registers per product and halve the wavefronts per SIMD
        asm volatile("" ::: "memory");
        const int64_t row = tile * 128 + wave * 32 + m; // the row this lane feeds as A operand
        float4 a1[KCH * 4], a2[KCH * 4];
#pragma unroll
        for (int q = 0; q < KCH * 4; ++q) {
            const int kk = 8 * q + 4 * h;
            float4 v1 = make_float4(0.f, 0.f, 0.f, 0.f), v2 = v1;
            if (row < a.n && kk < a.K) {
                v1 = load_k4(a.A1, a.lda1, row, kk, a.K, vec1);
                if (!BWD) {
                    if (two) {
                        v2 = load_k4(a.A2, a.lda2, row, kk, a.K, vec2);
                        if (a.scale2) scale4(v2, a.scale2[row]);
                    }
                } else {
                    if (two) v2 = v1;
                    if (a.mask) {
                        const uint32_t bits = a.mask[row * a.mask_words + (kk >> 5)] >> (kk & 31);
                        if (!(bits & 1u)) v1.x = 0.f;
                        if (!(bits & 2u)) v1.y = 0.f;
                        if (!(bits & 4u)) v1.z = 0.f;
                        if (!(bits & 8u)) v1.w = 0.f;
                    }
                    if (a.scale_o1) scale4(v1, a.scale_o1[row]); // scales the rows of the first product only
                }
            }
            a1[q] = v1;
            a2[q] = v2;
        }
        floatx16 acc1[NT], acc2[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) { acc1[t][r] = 0.f; acc2[t][r] = 0.f; }
#pragma unroll
        for (int q = 0; q < KCH * 4; ++q)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int kk = 8 * q + 4 * h + i;
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    acc1[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(pick(a1[q], i), Bs1[kk][t * 32 + m], acc1[t], 0, 0, 0);
                    if (two) acc2[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(pick(a2[q], i), Bs2[kk][t * 32 + m], acc2[t], 0, 0, 0);
                }
            }
        const int64_t row0 = tile * 128;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int col = col0 + t * 32 + m;
            const bool col_ok = col < a.Nout;
            const float bias1 = (!BWD && a.bias1 && col_ok) ? a.bias1[col] : 0.f;
            const float bias2 = (!BWD && two && a.bias2 && col_ok) ? a.bias2[col] : 0.f;
            uint32_t my_word = 0u; // lane L < 32 collects the activation word of strip row L
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t orow = row0 + wave * 32 + 8 * (r / 4) + 4 * h + (r % 4);
                if (!BWD) {
                    const float p = acc1[t][r] + bias1;
                    const bool pos = p > 0.f && col_ok;
                    if (a.act == SLICEGCN_ACT_RELU) {
                        // lanes 0..31 hold strip row 8*(r/4) + r%4 of this tile, lanes 32..63 the row four below it
                        const unsigned long long bal = __ballot(pos);
                        if (lane < 32 && r == 4 * (lane >> 3) + (lane & 3))
                            my_word = ((lane >> 2) & 1) ? (uint32_t)(bal >> 32) : (uint32_t)bal;
                    }
                    const float rl = (a.act == SLICEGCN_ACT_RELU) ? (p > 0.f ? p : 0.f) : p;
                    const float o = rl + (two ? acc2[t][r] + bias2 : 0.f);
                    if (orow < a.n && col_ok) a.O1[orow * a.ldo1 + col] = a.scale_o1 ? o * a.scale_o1[orow] : o;
                } else {
                    if (orow < a.n && col_ok) {
                        a.O1[orow * a.ldo1 + col] = acc1[t][r];
                        if (a.O2) a.O2[orow * a.ldo2 + col] = acc2[t][r];
                    }
                }
            }
            if (!BWD && a.act == SLICEGCN_ACT_RELU && lane < 32 && col0 + t * 32 < a.Nout) {
                const int64_t wrow = row0 + wave * 32 + lane; // one coalesced store of the strip's 32 words
                if (wrow < a.n) a.mask[wrow * a.mask_words + ((col0 + t * 32) >> 5)] = my_word;
            }
        }
    }
}

// Variant for the narrowest layers (K <= 32, at most 32 output columns: every layer of the workload
// with slices and hidden width 32).  These layers are HBM bound (about 10 flop per byte), so the kernel
// is built around the memory accesses: a wavefront owns strips of 32 rows; it reads a strip with fully
// coalesced 16-byte loads (eight lanes per 128-byte row), parks it in its own LDS tile, and reads it
// back in the MFMA operand layout (lane = row, four consecutive k per 16-byte LDS read; the row
// stride of 36 floats keeps those reads conflict free).  The next strip's loads are issued before
// the current strip's MFMAs.  The weight operands never change, so every lane keeps its 16 values per
// product in registers.  No workgroup barrier anywhere: a wavefront only touches its own tile, and
// its LDS accesses execute in program order.
template <bool BWD, bool TWO>
__global__ __launch_bounds__(256) void pair_strip32_kernel(const PairArgs a)
{
    constexpr int ST = 36;
    __shared__ __attribute__((aligned(16))) float T1[4][32][ST];
    __shared__ __attribute__((aligned(16))) float T2[(TWO && !BWD) ? 4 : 1][32][ST];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int m = lane & 31, h = lane >> 5;
    const int lr = lane >> 3, lc = (lane & 7) * 4; // coalesced layout: row lr + 8 * it, columns lc..lc+3
    const bool vec1 = aligned16(a.A1) && (a.lda1 % 4 == 0);
    const bool vec2 = TWO && !BWD && aligned16(a.A2) && (a.lda2 % 4 == 0);
    float (*t1)[ST] = T1[wave];
    float (*t2)[ST] = T2[(TWO && !BWD) ? wave : 0];

    float b1[16], b2[16];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int kk = 8 * q + 4 * h + i;
            float w1 = 0.f, w2 = 0.f;
            if (kk < a.K && m < a.Nout) {
                const int64_t id = BWD ? (int64_t)m * a.ldw + kk : (int64_t)kk * a.ldw + m;
                w1 = a.B1[id];
                if (TWO) w2 = a.B2[id];
            }
            b1[q * 4 + i] = w1;
            b2[q * 4 + i] = w2;
        }
    const bool col_ok = m < a.Nout;
    const float bias1 = (!BWD && a.bias1 && col_ok) ? a.bias1[m] : 0.f;
    const float bias2 = (!BWD && TWO && a.bias2 && col_ok) ? a.bias2[m] : 0.f;

    const int64_t n_strips = (a.n + 31) / 32;
    const int64_t first = (int64_t)blockIdx.x * 4 + wave, step = (int64_t)gridDim.x * 4;
    float4 p1[4], p2[4];
    uint32_t pw = ~0u; // backward: activation word of strip row m (the row this lane feeds to the MFMAs)
    float ps = 1.f;    // backward: scale_o1 of strip row m
    // forward, scaled layout: factors of the rows lr + 8 it this lane loads and stores (only fetched here; they are
    // applied where the strip is consumed, so that the next strip's loads stay in flight behind the MFMAs).  One
    // load per lane and strip handed on by cross-lane reads was measured slower (the LDS pipe carries the tiles).
    float f2[4] = {1.f, 1.f, 1.f, 1.f}, fo[4] = {1.f, 1.f, 1.f, 1.f};
    auto fetch = [&](int64_t strip) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int64_t row = strip * 32 + lr + 8 * it;
            float4 v1 = make_float4(0.f, 0.f, 0.f, 0.f), v2 = v1;
            if (row < a.n && lc < a.K) {
                v1 = load_k4(a.A1, a.lda1, row, lc, a.K, vec1);
                if (!BWD && TWO) v2 = load_k4(a.A2, a.lda2, row, lc, a.K, vec2);
            }
            if (!BWD && row < a.n) {
                if (TWO && a.scale2) f2[it] = a.scale2[row];
                if (a.scale_o1) fo[it] = a.scale_o1[row];
            }
            p1[it] = v1;
            p2[it] = v2;
        }
        if (BWD && a.mask) pw = strip * 32 + m < a.n ? a.mask[(strip * 32 + m) * a.mask_words] : 0u;
        if (BWD && a.scale_o1) ps = strip * 32 + m < a.n ? a.scale_o1[strip * 32 + m] : 1.f;
    };
    if (first < n_strips) fetch(first);
    for (int64_t strip = first; strip < n_strips; strip += step) {
        float out_f[4]; // output factors of the rows lr + 8 it of this strip (the fetch below overwrites fo)
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            if (TWO && !BWD && a.scale2) scale4(p2[it], f2[it]);
            out_f[it] = fo[it];
            *reinterpret_cast<float4 *>(&t1[lr + 8 * it][lc]) = p1[it];
            if (TWO && !BWD) *reinterpret_cast<float4 *>(&t2[lr + 8 * it][lc]) = p2[it];
        }
        __builtin_amdgcn_wave_barrier();
        float4 a1[4], a2[4];
        const uint32_t word = pw;
        const float so = ps;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            a1[q] = *reinterpret_cast<const float4 *>(&t1[m][8 * q + 4 * h]);
            if (TWO && !BWD) a2[q] = *reinterpret_cast<const float4 *>(&t2[m][8 * q + 4 * h]);
            if (BWD) { // second product: dHout as it is; first product: dP = dHout * mask (times the row's output factor)
                a2[q] = a1[q];
                const uint32_t bits = word >> (8 * q + 4 * h);
                if (!(bits & 1u)) a1[q].x = 0.f;
                if (!(bits & 2u)) a1[q].y = 0.f;
                if (!(bits & 4u)) a1[q].z = 0.f;
                if (!(bits & 8u)) a1[q].w = 0.f;
                if (a.scale_o1) scale4(a1[q], so);
            }
        }
        __builtin_amdgcn_wave_barrier();
        if (strip + step < n_strips) fetch(strip + step); // flies during the MFMAs and the stores below
        floatx16 acc1, acc2;
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc1[r] = 0.f; acc2[r] = 0.f; }
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(pick(a1[q], i), b1[q * 4 + i], acc1, 0, 0, 0);
                if (TWO) acc2 = __builtin_amdgcn_mfma_f32_32x32x2f32(pick(a2[q], i), b2[q * 4 + i], acc2, 0, 0, 0);
            }
        const int64_t row0 = strip * 32;
        uint32_t my_word = 0u; // lane L < 32 collects the activation word of strip row L
        float o1[16], o2[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if (!BWD) {
                const float p = acc1[r] + bias1;
                const bool pos = p > 0.f && col_ok;
                if (a.act == SLICEGCN_ACT_RELU) {
                    const unsigned long long bal = __ballot(pos);
                    if (lane < 32 && r == 4 * (lane >> 3) + (lane & 3))
                        my_word = ((lane >> 2) & 1) ? (uint32_t)(bal >> 32) : (uint32_t)bal;
                }
                const float rl = (a.act == SLICEGCN_ACT_RELU) ? (p > 0.f ? p : 0.f) : p;
                o1[r] = rl + (TWO ? acc2[r] + bias2 : 0.f);
            } else {
                o1[r] = acc1[r];
                o2[r] = acc2[r];
            }
        }
        // Outputs leave through the wavefront's tile so that a row goes out as eight 16-byte stores
        // (register r of lane (m, h) is strip row 8*(r/4) + 4*h + r%4, column m); layouts that do not
        // allow 16-byte stores write the registers directly.
        // `rs`: per-row factor applied on the way out (forward outputs kept in the scaled layout), or NULL; the
        // 16-byte path takes the factors from out_f, fetched a strip ahead.
        auto store_tile = [&](const float (&o)[16], float *O, int64_t ldo, bool vec_ok, const float *rs) {
            if (vec_ok) {
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int r = 0; r < 16; ++r) t1[8 * (r / 4) + 4 * h + (r % 4)][m] = o[r];
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int64_t row = row0 + lr + 8 * it;
                    float4 v = *reinterpret_cast<const float4 *>(&t1[lr + 8 * it][lc]);
                    if (row < a.n && lc < a.Nout) {
                        if (rs) scale4(v, out_f[it]);
                        *reinterpret_cast<float4 *>(O + row * ldo + lc) = v;
                    }
                }
                __builtin_amdgcn_wave_barrier();
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t orow = row0 + 8 * (r / 4) + 4 * h + (r % 4);
                    if (orow < a.n && col_ok) O[orow * ldo + m] = rs ? o[r] * rs[orow] : o[r];
                }
            }
        };
        const bool nout4 = a.Nout % 4 == 0;
        store_tile(o1, a.O1, a.ldo1, nout4 && aligned16(a.O1) && a.ldo1 % 4 == 0, BWD ? nullptr : a.scale_o1);
        if (BWD && TWO && a.O2) store_tile(o2, a.O2, a.ldo2, nout4 && aligned16(a.O2) && a.ldo2 % 4 == 0, nullptr);
        if (!BWD && a.act == SLICEGCN_ACT_RELU && lane < 32 && row0 + lane < a.n)
            a.mask[(row0 + lane) * a.mask_words] = my_word;
    }
}

// The same idea for layers up to 64 wide (K <= 32 * KC, at most 32 * NC output columns).  The weights no
// longer fit in registers next to the accumulators, so the workgroup keeps them (zero padded, already
// transposed for the backward products) in LDS and every MFMA reads its B operand from there; the
// two operand strips of the forward pass go through the wavefront's one tile in turn.  Compiled for
// two wavefronts per SIMD: one computes while the other moves its strip.
template <int KC, int NC, bool BWD, bool TWO>
__global__ __launch_bounds__(256, 2) void pair_strip64_kernel(const PairArgs a)
{
    constexpr int KW = 32 * KC, NW = 32 * NC;
    constexpr int ST = (KW > NW ? KW : NW) + 4; // tile row stride: 16-byte reads with lane = row stay conflict free
    constexpr int LK = KW / 4, LN = NW / 4;     // lanes per row, operand strips / output strips
    constexpr int PK = 32 * LK / 64, PN = 32 * LN / 64; // 16-byte accesses per lane and strip
    constexpr int QN = 4 * KC;                  // float4 of the reduction axis per row
    __shared__ __attribute__((aligned(16))) float Tl[4][32][ST];
    __shared__ float W1s[KW][NW];
    __shared__ float W2s[TWO ? KW : 1][NW];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int m = lane & 31, h = lane >> 5;
    const int rk = lane / LK, ck = (lane % LK) * 4; // coalesced layout of an operand strip
    const int rn = lane / LN, cn = (lane % LN) * 4; // and of an output strip
    const bool vec1 = aligned16(a.A1) && (a.lda1 % 4 == 0);
    const bool vec2 = TWO && !BWD && aligned16(a.A2) && (a.lda2 % 4 == 0);
    float (*tl)[ST] = Tl[wave];

    for (int idx = threadIdx.x; idx < KW * NW; idx += 256) {
        // consecutive threads walk the contiguous axis of W: columns forward, k backward (W^T)
        const int kk = BWD ? idx % KW : idx / NW, j = BWD ? idx / KW : idx % NW;
        float w1 = 0.f, w2 = 0.f;
        if (kk < a.K && j < a.Nout) {
            const int64_t id = BWD ? (int64_t)j * a.ldw + kk : (int64_t)kk * a.ldw + j;
            w1 = a.B1[id];
            if (TWO) w2 = a.B2[id];
        }
        W1s[kk][j] = w1;
        if (TWO) W2s[kk][j] = w2;
    }
    __syncthreads(); // the only workgroup barrier: from here on a wavefront touches its own tile only

    float bias1[NC], bias2[NC];
#pragma unroll
    for (int t = 0; t < NC; ++t) {
        const bool ok = 32 * t + m < a.Nout;
        bias1[t] = (!BWD && a.bias1 && ok) ? a.bias1[32 * t + m] : 0.f;
        bias2[t] = (!BWD && TWO && a.bias2 && ok) ? a.bias2[32 * t + m] : 0.f;
    }

    const int64_t n_strips = (a.n + 31) / 32;
    const int64_t first = (int64_t)blockIdx.x * 4 + wave, step = (int64_t)gridDim.x * 4;
    float4 p1[PK], p2[(TWO && !BWD) ? PK : 1];
    uint32_t pw[KC]; // backward: activation words of strip row m
    // forward, scaled layout: factors of the rows this lane loads (f2) and stores (fo); fetched a strip ahead, applied
    // where the strip is consumed
    float f2[(TWO && !BWD) ? PK : 1], fo[BWD ? 1 : PN];
#pragma unroll
    for (int w = 0; w < KC; ++w) pw[w] = ~0u;
    auto fetch = [&](int64_t strip) {
#pragma unroll
        for (int it = 0; it < PK; ++it) {
            const int64_t row = strip * 32 + rk + (64 / LK) * it;
            float4 v1 = make_float4(0.f, 0.f, 0.f, 0.f), v2 = v1;
            if (row < a.n && ck < a.K) {
                v1 = load_k4(a.A1, a.lda1, row, ck, a.K, vec1);
                if (!BWD && TWO) v2 = load_k4(a.A2, a.lda2, row, ck, a.K, vec2);
            }
            if (!BWD && TWO) f2[it] = (a.scale2 && row < a.n) ? a.scale2[row] : 1.f;
            p1[it] = v1;
            if (!BWD && TWO) p2[it] = v2;
        }
        if (BWD && a.mask) {
#pragma unroll
            for (int w = 0; w < KC; ++w)
                pw[w] = (strip * 32 + m < a.n && 32 * w < a.K) ? a.mask[(strip * 32 + m) * a.mask_words + w] : 0u;
        }
        if (!BWD) {
#pragma unroll
            for (int it = 0; it < PN; ++it) {
                const int64_t row = strip * 32 + rn + (64 / LN) * it;
                fo[it] = (a.scale_o1 && row < a.n) ? a.scale_o1[row] : 1.f;
            }
        }
    };
    if (first < n_strips) fetch(first);
    for (int64_t strip = first; strip < n_strips; strip += step) {
        float out_f[BWD ? 1 : PN]; // output factors of this strip's rows (the fetch below overwrites fo)
        if (!BWD) {
#pragma unroll
            for (int it = 0; it < PN; ++it) out_f[it] = fo[it];
        }
#pragma unroll
        for (int it = 0; it < PK; ++it) *reinterpret_cast<float4 *>(&tl[rk + (64 / LK) * it][ck]) = p1[it];
        __builtin_amdgcn_wave_barrier();
        float4 a1[QN];
#pragma unroll
        for (int q = 0; q < QN; ++q) a1[q] = *reinterpret_cast<const float4 *>(&tl[m][8 * q + 4 * h]);
        __builtin_amdgcn_wave_barrier();
        if (TWO && !BWD) { // the second operand strip takes the tile while the first product runs from registers
#pragma unroll
            for (int it = 0; it < PK; ++it) {
                if (a.scale2) scale4(p2[it], f2[it]);
                *reinterpret_cast<float4 *>(&tl[rk + (64 / LK) * it][ck]) = p2[it];
            }
            __builtin_amdgcn_wave_barrier();
        }
        const bool more = strip + step < n_strips;
        uint32_t word[KC];
#pragma unroll
        for (int w = 0; w < KC; ++w) word[w] = pw[w];
        if (more) fetch(strip + step); // flies during the MFMAs and the stores below
        floatx16 acc1[NC], acc2[NC];
#pragma unroll
        for (int t = 0; t < NC; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) { acc1[t][r] = 0.f; acc2[t][r] = 0.f; }
        if (BWD) { // both products read dHout; the first one through the activation bits (dP = dHout * mask)
#pragma unroll
            for (int q = 0; q < QN; ++q)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int kk = 8 * q + 4 * h + i;
                    const float g = pick(a1[q], i);
                    const float gp = ((word[q >> 2] >> (8 * (q & 3) + 4 * h + i)) & 1u) ? g : 0.f;
#pragma unroll
                    for (int t = 0; t < NC; ++t)
                        acc1[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(gp, W1s[kk][32 * t + m], acc1[t], 0, 0, 0);
                }
            if (TWO) {
#pragma unroll
                for (int q = 0; q < QN; ++q)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int kk = 8 * q + 4 * h + i;
#pragma unroll
                        for (int t = 0; t < NC; ++t)
                            acc2[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(pick(a1[q], i), W2s[kk][32 * t + m], acc2[t], 0, 0, 0);
                    }
            }
        } else {
#pragma unroll
            for (int q = 0; q < QN; ++q)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int kk = 8 * q + 4 * h + i;
#pragma unroll
                    for (int t = 0; t < NC; ++t)
                        acc1[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(pick(a1[q], i), W1s[kk][32 * t + m], acc1[t], 0, 0, 0);
                }
            if (TWO) {
#pragma unroll
                for (int q = 0; q < QN; ++q) a1[q] = *reinterpret_cast<const float4 *>(&tl[m][8 * q + 4 * h]);
#pragma unroll
                for (int q = 0; q < QN; ++q)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int kk = 8 * q + 4 * h + i;
#pragma unroll
                        for (int t = 0; t < NC; ++t)
                            acc2[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(pick(a1[q], i), W2s[kk][32 * t + m], acc2[t], 0, 0, 0);
                    }
            }
        }
        const int64_t row0 = strip * 32;
        uint32_t my_word[NC]; // lane L < 32 collects the activation words of strip row L
        if (!BWD) { // the forward result replaces the first accumulator
#pragma unroll
            for (int t = 0; t < NC; ++t) {
                my_word[t] = 0u;
                const bool col_ok = 32 * t + m < a.Nout;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float p = acc1[t][r] + bias1[t];
                    const bool pos = p > 0.f && col_ok;
                    if (a.act == SLICEGCN_ACT_RELU) {
                        const unsigned long long bal = __ballot(pos);
                        if (lane < 32 && r == 4 * (lane >> 3) + (lane & 3))
                            my_word[t] = ((lane >> 2) & 1) ? (uint32_t)(bal >> 32) : (uint32_t)bal;
                    }
                    const float rl = (a.act == SLICEGCN_ACT_RELU) ? (p > 0.f ? p : 0.f) : p;
                    acc1[t][r] = rl + (TWO ? acc2[t][r] + bias2[t] : 0.f);
                }
            }
        }
        // Outputs leave through the wavefront's tile so that a row goes out as 16-byte stores
        // (register r of lane (m, h) is strip row 8*(r/4) + 4*h + r%4, column 32 t + m); layouts that
        // do not allow 16-byte stores write the registers directly.
        // `rs`: per-row factor applied on the way out (forward outputs kept in the scaled layout), or NULL.
        auto store_tile = [&](const floatx16 (&o)[NC], float *O, int64_t ldo, bool vec_ok, const float *rs) {
            if (vec_ok) {
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int t = 0; t < NC; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r) tl[8 * (r / 4) + 4 * h + (r % 4)][32 * t + m] = o[t][r];
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int it = 0; it < PN; ++it) {
                    const int64_t row = row0 + rn + (64 / LN) * it;
                    float4 v = *reinterpret_cast<const float4 *>(&tl[rn + (64 / LN) * it][cn]);
                    if (row < a.n && cn < a.Nout) {
                        if constexpr (!BWD) {
                            if (rs) scale4(v, out_f[it]);
                        } else { // backward: the accumulators leave no register for a factor fetched ahead
                            if (rs) scale4(v, rs[row]);
                        }
                        *reinterpret_cast<float4 *>(O + row * ldo + cn) = v;
                    }
                }
                __builtin_amdgcn_wave_barrier();
            } else {
#pragma unroll
                for (int t = 0; t < NC; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int64_t orow = row0 + 8 * (r / 4) + 4 * h + (r % 4);
                        if (orow < a.n && 32 * t + m < a.Nout) O[orow * ldo + 32 * t + m] = rs ? o[t][r] * rs[orow] : o[t][r];
                    }
            }
        };
        const bool nout4 = a.Nout % 4 == 0;
        store_tile(acc1, a.O1, a.ldo1, nout4 && aligned16(a.O1) && a.ldo1 % 4 == 0, a.scale_o1);
        if constexpr (BWD && TWO) {
            if (a.O2) store_tile(acc2, a.O2, a.ldo2, nout4 && aligned16(a.O2) && a.ldo2 % 4 == 0, nullptr);
        }
        if (!BWD && a.act == SLICEGCN_ACT_RELU && lane < 32 && row0 + lane < a.n) {
#pragma unroll
            for (int t = 0; t < NC; ++t)
                if (32 * t < a.Nout) a.mask[(row0 + lane) * a.mask_words + t] = my_word[t];
        }
    }
}

template <int KC, int NC, bool BWD>
void launch_strip64(const PairArgs &a, unsigned gb, hipStream_t stream)
{
    if (a.A2 != nullptr && a.B2 != nullptr) pair_strip64_kernel<KC, NC, BWD, true><<<gb, 256, 0, stream>>>(a);
    else pair_strip64_kernel<KC, NC, BWD, false><<<gb, 256, 0, stream>>>(a);
}

template <int NT, bool BWD>
void launch_direct(const PairArgs &a, dim3 grid, hipStream_t stream)
{
    if (a.K <= 32) pair_mfma_direct_kernel<NT, 1, BWD><<<grid, 256, 0, stream>>>(a);
    else pair_mfma_direct_kernel<NT, 2, BWD><<<grid, 256, 0, stream>>>(a);
}

template <bool BWD>
int launch_pair(const PairArgs &a, hipStream_t stream)
{
    const int nt = a.Nout <= 32 ? 1 : a.Nout <= 64 ? 2 : a.Nout <= 96 ? 3 : 4;
    dim3 grid((unsigned)((a.n + 127) / 128), (unsigned)((a.Nout + nt * 32 - 1) / (nt * 32)));
    if (a.K <= 32 && a.Nout <= 32) { // narrowest layers: per-wavefront strips, no barriers
        const int64_t strips = (a.n + 31) / 32;
        const unsigned gb = (unsigned)((strips + 3) / 4 < 2048 ? (strips + 3) / 4 : 2048);
        const bool two = a.A2 != nullptr && a.B2 != nullptr;
        if (two) pair_strip32_kernel<BWD, true><<<gb, 256, 0, stream>>>(a);
        else pair_strip32_kernel<BWD, false><<<gb, 256, 0, stream>>>(a);
        SG_LAUNCH_CHECK();
        return SLICEGCN_OK;
    }
    if (a.K <= 64 && a.Nout <= 64 && a.n >= 262144) { // up to 64 wide: strips, weights in LDS
        const int64_t strips = (a.n + 31) / 32;
        // as many workgroups as the chip holds at once (two per CU): each stages the weights once
        const unsigned gb = (unsigned)((strips + 3) / 4 < 512 ? (strips + 3) / 4 : 512);
        if (a.K <= 32) launch_strip64<1, 2, BWD>(a, gb, stream);
        else if (a.Nout <= 32) launch_strip64<2, 1, BWD>(a, gb, stream);
        else launch_strip64<2, 2, BWD>(a, gb, stream);
        SG_LAUNCH_CHECK();
        return SLICEGCN_OK;
    }
    if (a.K <= 64 && nt == 1) { // short reduction, one output tile: weights resident in LDS, workgroups walk over row tiles
        const unsigned tiles = grid.x;
        grid.x = tiles < 2048u ? tiles : 2048u;
        switch (nt) {
        case 1: launch_direct<1, BWD>(a, grid, stream); break;
        case 2: launch_direct<2, BWD>(a, grid, stream); break;
        case 3: launch_direct<3, BWD>(a, grid, stream); break;
        default: launch_direct<4, BWD>(a, grid, stream); break;
        }
        SG_LAUNCH_CHECK();
        return SLICEGCN_OK;
    }
    // staged kernel: 1-D grid, 8 row tiles x all column tiles per group of workgroups (see the kernel)
    const bool two = a.A2 != nullptr && a.B2 != nullptr;
    // Column tiles per workgroup: 4 for a single product and 2 for a pair, which keeps two workgroups on a CU (64 and
    // 2 x 32 accumulator registers): the other workgroup's MFMAs fill the barrier waits.  Wider tiles (256 columns,
    // or 128 for a pair) run one workgroup per CU and are 20 % and 16 % slower on 256 -> 256 and 301 -> 128.
    const int cap = two ? 2 : 4;
    const int nt2 = nt > cap ? cap : nt;
    const int bn = nt2 * 32;
    const int n_col = (a.Nout + bn - 1) / bn;
    const int64_t row_tiles = (a.n + 127) / 128;
    const int64_t blocks = (row_tiles + 7) / 8 * 8 * n_col;
    SG_REQUIRE(blocks <= INT32_MAX, SLICEGCN_ERANGE, "dense product: grid too large");
    const unsigned gb = (unsigned)blocks;
    if (two) {
        if (nt2 == 1) pair_mfma_kernel<1, BWD, true><<<gb, 256, 0, stream>>>(a, n_col);
        else pair_mfma_kernel<2, BWD, true><<<gb, 256, 0, stream>>>(a, n_col);
    } else {
        switch (nt2) {
        case 1: pair_mfma_kernel<1, BWD, false><<<gb, 256, 0, stream>>>(a, n_col); break;
        case 2: pair_mfma_kernel<2, BWD, false><<<gb, 256, 0, stream>>>(a, n_col); break;
        case 3: pair_mfma_kernel<3, BWD, false><<<gb, 256, 0, stream>>>(a, n_col); break;
        default: pair_mfma_kernel<4, BWD, false><<<gb, 256, 0, stream>>>(a, n_col); break;
        }
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
    int32_t stride;                     // 2*w_in*w_out + 2*w_out; compact: w_in*w_out + w_out
    int32_t compact;                    // 1: no self term and no slot for it: [Z^T dP | colsum dP]
    int32_t rows_per_block = RED_ROWS;  // tiled kernels: node rows per workgroup (one partial each)
    const float *hin_scale = nullptr;   // rows of Hin are multiplied by hin_scale[row] when read (Hin stored as D~^-1/2 Hin)
};

// Partial weight gradients, tiled: grid = (row blocks, w_in tiles, w_out tiles), every workgroup writes its
// tile of the four results [Z^T dP | Hin^T dHout | colsum dP | colsum dHout] of its row block into
// partial[row block][...].  Per step the workgroup stages 32 rows of the four operand tiles in LDS;
// wavefront w multiplies rows 8w..8w+7 (the node axis is the MFMA's k axis: A[m][k] = Z[k][m]),
// and the four wavefronts' accumulators are added in wavefront order at the end.
__global__ __launch_bounds__(256) void grad_partial_mfma_kernel(const ReduceArgs a)
{
    // one LDS block: the four operand tiles during the row loop, the accumulators of wavefronts 1..3 after it
    constexpr int TILE_FLOATS = RED_RK * RED_TILE;
    __shared__ __attribute__((aligned(16))) float lds[3 * 2 * RED_TILE * RED_TILE];
    float (*Zs)[RED_TILE] = reinterpret_cast<float (*)[RED_TILE]>(lds);
    float (*Hs)[RED_TILE] = reinterpret_cast<float (*)[RED_TILE]>(lds + TILE_FLOATS);
    float (*Ps)[RED_TILE] = reinterpret_cast<float (*)[RED_TILE]>(lds + 2 * TILE_FLOATS);
    float (*Gs)[RED_TILE] = reinterpret_cast<float (*)[RED_TILE]>(lds + 3 * TILE_FLOATS);
    float (*red)[2][RED_TILE * RED_TILE] = reinterpret_cast<float (*)[2][RED_TILE * RED_TILE]>(lds);
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int m = lane & 31, h = lane >> 5;
    const int i_base = blockIdx.y * RED_TILE, j_base = blockIdx.z * RED_TILE;
    const int64_t r_begin = (int64_t)blockIdx.x * a.rows_per_block;
    const int64_t r_end = r_begin + a.rows_per_block < a.n ? r_begin + a.rows_per_block : a.n;
    const bool self = a.Hin != nullptr;
    const bool vz = aligned16(a.Z) && a.ldz % 4 == 0, vh = self && aligned16(a.Hin) && a.ldi % 4 == 0;
    const bool vg = aligned16(a.dHout) && a.ldo % 4 == 0;

    floatx16 accA, accS;
#pragma unroll
    for (int r = 0; r < 16; ++r) { accA[r] = 0.f; accS[r] = 0.f; }
    float accb = 0.f; // lanes 0..31: column (j_base + m) of dP, lanes 32..63: of dH_out; rows of this wavefront only

    const int lr = tid >> 3, lc = (tid & 7) * 4; // this thread's float4 of each 32 x 32 tile
    float4 z, hh, p, g;
    float hf = 1.f; // factor of this thread's row of Hin (scaled layout); applied when the registers go to LDS
    auto fetch = [&](int64_t r0) { // this thread's share of the four tiles of rows [r0, r0 + 32)
        const int64_t row = r0 + lr;
        z = make_float4(0.f, 0.f, 0.f, 0.f); hh = z; p = z; g = z;
        if (row < r_end) {
            if (i_base + lc < a.w_in) {
                z = load_k4(a.Z, a.ldz, row, i_base + lc, a.w_in, vz);
                if (self) {
                    hh = load_k4(a.Hin, a.ldi, row, i_base + lc, a.w_in, vh);
                    if (a.hin_scale) hf = a.hin_scale[row];
                }
            }
            if (j_base + lc < a.w_out) {
                g = load_k4(a.dHout, a.ldo, row, j_base + lc, a.w_out, vg);
                p = g;
                if (a.mask) {
                    const int j = j_base + lc;
                    const uint32_t bits = a.mask[row * a.mask_words + (j >> 5)] >> (j & 31);
                    if (!(bits & 1u)) p.x = 0.f;
                    if (!(bits & 2u)) p.y = 0.f;
                    if (!(bits & 4u)) p.z = 0.f;
                    if (!(bits & 8u)) p.w = 0.f;
                }
            }
        }
    };
    fetch(r_begin);
    for (int64_t r0 = r_begin; r0 < r_end; r0 += RED_RK) {
        if (a.hin_scale) scale4(hh, hf);
        *reinterpret_cast<float4 *>(&Zs[lr][lc]) = z;
        *reinterpret_cast<float4 *>(&Hs[lr][lc]) = hh;
        *reinterpret_cast<float4 *>(&Ps[lr][lc]) = p;
        *reinterpret_cast<float4 *>(&Gs[lr][lc]) = g;
        __syncthreads();
        if (r0 + RED_RK < r_end) fetch(r0 + RED_RK); // next step's loads fly during this step's MFMAs
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
            const int k = wave * 8 + s4 * 2 + h;
            accA = __builtin_amdgcn_mfma_f32_32x32x2f32(Zs[k][m], Ps[k][m], accA, 0, 0, 0);
            if (self) accS = __builtin_amdgcn_mfma_f32_32x32x2f32(Hs[k][m], Gs[k][m], accS, 0, 0, 0);
        }
        if (blockIdx.y == 0) {
            float (*T)[RED_TILE] = h ? Gs : Ps;
#pragma unroll
            for (int r = 0; r < 8; ++r) accb += T[wave * 8 + r][m];
        }
        __syncthreads();
    }

    // ---- add the four wavefronts' tiles in order, then store (the tile memory is free now) ----
    __shared__ float bsum[4][64];
    bsum[wave][lane] = accb;
    if (wave > 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int i = 8 * (r / 4) + 4 * h + (r % 4);
            red[wave - 1][0][i * RED_TILE + m] = accA[r];
            red[wave - 1][1][i * RED_TILE + m] = accS[r];
        }
    }
    __syncthreads();
    float *out = a.partial + (int64_t)blockIdx.x * a.stride;
    const int ww = a.w_in * a.w_out;
    if (wave == 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int il = 8 * (r / 4) + 4 * h + (r % 4);
            float va = accA[r], vs = accS[r];
            for (int q = 0; q < 3; ++q) { va += red[q][0][il * RED_TILE + m]; vs += red[q][1][il * RED_TILE + m]; }
            const int i = i_base + il, j = j_base + m;
            if (i < a.w_in && j < a.w_out) {
                out[i * a.w_out + j] = va;
                if (!a.compact) out[ww + i * a.w_out + j] = vs;
            }
        }
        if (blockIdx.y == 0) {
            const int j = j_base + m;
            const float sum = ((bsum[0][lane] + bsum[1][lane]) + bsum[2][lane]) + bsum[3][lane];
            if (j < a.w_out && !(a.compact && h)) out[(a.compact ? ww : 2 * ww) + (h ? a.w_out : 0) + j] = sum;
        }
    }
}

// Partial weight gradients of the narrowest layers (w_in, w_out <= 32, large n): every wavefront owns
// its own accumulators and every n_waves-th strip of 32 rows (so that the chip reads one contiguous
// window at a time), reads a strip with coalesced 16-byte loads into wave-private LDS tiles (the
// next strip's loads in flight during the MFMAs), and writes one partial result.  The node axis is the MFMA's k axis (lane (m, h) feeds
// column m of node row 2s + h).  No workgroup barrier; same output layout as grad_partial_mfma_kernel,
// one partial per wavefront.
__global__ __launch_bounds__(256) void grad_strip32_kernel(const ReduceArgs a, int64_t n_waves)
{
    __shared__ __attribute__((aligned(16))) float Zs[4][32][32];
    __shared__ __attribute__((aligned(16))) float Hs[4][32][32];
    __shared__ __attribute__((aligned(16))) float Gs[4][32][32];
    __shared__ uint32_t Ms[4][32];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int m = lane & 31, h = lane >> 5;
    const int lr = lane >> 3, lc = (lane & 7) * 4;
    const int64_t w_id = (int64_t)blockIdx.x * 4 + wave;
    const int64_t n_strips = (a.n + 31) / 32, r_end = a.n;
    if (w_id >= n_waves) return; // uniform per wavefront; no barriers below (n_waves <= n_strips)
    const bool self = a.Hin != nullptr;
    const bool vz = aligned16(a.Z) && a.ldz % 4 == 0, vh = self && aligned16(a.Hin) && a.ldi % 4 == 0;
    const bool vg = aligned16(a.dHout) && a.ldo % 4 == 0;
    float (*zs)[32] = Zs[wave];
    float (*hs)[32] = Hs[wave];
    float (*gs)[32] = Gs[wave];
    uint32_t *ms = Ms[wave];

    floatx16 accA, accS;
#pragma unroll
    for (int r = 0; r < 16; ++r) { accA[r] = 0.f; accS[r] = 0.f; }
    float sum_p = 0.f, sum_g = 0.f; // column m of dP and of dHout over the node rows 2s + h

    float4 pz[4], ph[4], pg[4];
    float hf[4] = {1.f, 1.f, 1.f, 1.f}; // factors of the rows of Hin this lane loads (scaled layout); applied on the way to LDS
    uint32_t pw = ~0u;
    auto fetch = [&](int64_t r0) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int64_t row = r0 + lr + 8 * it;
            float4 z = make_float4(0.f, 0.f, 0.f, 0.f), hh = z, g = z;
            if (row < r_end) {
                if (lc < a.w_in) {
                    z = load_k4(a.Z, a.ldz, row, lc, a.w_in, vz);
                    if (self) {
                        hh = load_k4(a.Hin, a.ldi, row, lc, a.w_in, vh);
                        if (a.hin_scale) hf[it] = a.hin_scale[row];
                    }
                }
                if (lc < a.w_out) g = load_k4(a.dHout, a.ldo, row, lc, a.w_out, vg);
            }
            pz[it] = z; ph[it] = hh; pg[it] = g;
        }
        if (a.mask && lane < 32) pw = r0 + lane < r_end ? a.mask[(r0 + lane) * a.mask_words] : 0u;
    };
    fetch(w_id * 32);
    for (int64_t strip = w_id; strip < n_strips; strip += n_waves) { // wavefront w takes strips w, w + n_waves, ...
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            if (a.hin_scale) scale4(ph[it], hf[it]);
            *reinterpret_cast<float4 *>(&zs[lr + 8 * it][lc]) = pz[it];
            *reinterpret_cast<float4 *>(&hs[lr + 8 * it][lc]) = ph[it];
            *reinterpret_cast<float4 *>(&gs[lr + 8 * it][lc]) = pg[it];
        }
        if (lane < 32) ms[lane] = pw;
        __builtin_amdgcn_wave_barrier();
        if (strip + n_waves < n_strips) fetch((strip + n_waves) * 32);
#pragma unroll
        for (int s2 = 0; s2 < 16; ++s2) {
            const int k = 2 * s2 + h;
            const float g = gs[k][m];
            const float p = ((ms[k] >> m) & 1u) ? g : 0.f;
            accA = __builtin_amdgcn_mfma_f32_32x32x2f32(zs[k][m], p, accA, 0, 0, 0);
            if (self) accS = __builtin_amdgcn_mfma_f32_32x32x2f32(hs[k][m], g, accS, 0, 0, 0);
            sum_p += p;
            sum_g += g;
        }
        __builtin_amdgcn_wave_barrier();
    }
    sum_p += __shfl_xor(sum_p, 32, 64);
    sum_g += __shfl_xor(sum_g, 32, 64);
    float *out = a.partial + w_id * a.stride;
    const int ww = a.w_in * a.w_out;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int i = 8 * (r / 4) + 4 * h + (r % 4);
        if (i < a.w_in && m < a.w_out) {
            out[i * a.w_out + m] = accA[r];
            if (!a.compact) out[ww + i * a.w_out + m] = accS[r];
        }
    }
    if (lane < 32 && m < a.w_out) {
        out[(a.compact ? ww : 2 * ww) + m] = sum_p;
        if (!a.compact) out[2 * ww + a.w_out + m] = sum_g;
    }
}

// Backward pass of a narrow layer (w_in, w_out <= 32, self term present, input gradient wanted) in one sweep over the
// node rows: the weight-gradient sums of grad_strip32_kernel and the two input-gradient products of
// pair_strip32_kernel<true, true> from the same wavefront-private tiles, so that dHout (and the mask) are read once
// instead of twice.  Per strip of 32 rows: Z, Hin and dHout go to LDS with coalesced 16-byte loads (the next strip's
// loads in flight behind the MFMAs); the node axis is the k axis of Z^T dP and Hin^T dHout (column reads of the
// tiles), the column axis that of dZ = dP W_agg^T and T = dHout W_self^T (row reads, weights in registers); dZ and T
// leave through the Z and Hin tiles as 16-byte stores.  Partial sums: one per wavefront, layout of
// grad_partial_mfma_kernel.  `a` carries the input-gradient half: B1 / B2 = W_agg / W_self (ldw), O1 = dZ (rows
// scaled by scale_o1), O2 = T, K = w_out, Nout = w_in.
__global__ __launch_bounds__(256, 2) void bwd_strip32_kernel(const ReduceArgs r, const PairArgs a, int64_t n_waves)
{
    constexpr int ST = 36; // row stride: 16-byte row reads and 4-byte column reads are both conflict free
    __shared__ __attribute__((aligned(16))) float Zs[4][32][ST];
    __shared__ __attribute__((aligned(16))) float Hs[4][32][ST];
    __shared__ __attribute__((aligned(16))) float Gs[4][32][ST];
    __shared__ uint32_t Ms[4][32];
    __shared__ __attribute__((aligned(16))) float W1s[32][ST]; // W_agg and W_self, zero padded to 32 x 32: row i, k contiguous
    __shared__ __attribute__((aligned(16))) float W2s[32][ST];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int m = lane & 31, h = lane >> 5;
    const int lr = lane >> 3, lc = (lane & 7) * 4;
    for (int idx = threadIdx.x; idx < 32 * 32; idx += 256) {
        const int i = idx >> 5, kk = idx & 31;
        const bool ok = i < r.w_in && kk < r.w_out;
        W1s[i][kk] = ok ? a.B1[(int64_t)i * a.ldw + kk] : 0.f;
        W2s[i][kk] = ok ? a.B2[(int64_t)i * a.ldw + kk] : 0.f;
    }
    __syncthreads(); // the only workgroup barrier: before any wavefront leaves
    const int64_t w_id = (int64_t)blockIdx.x * 4 + wave;
    const int64_t n_strips = (r.n + 31) / 32, r_end = r.n;
    if (w_id >= n_waves) return; // uniform per wavefront (n_waves <= n_strips)
    const bool vz = aligned16(r.Z) && r.ldz % 4 == 0, vh = aligned16(r.Hin) && r.ldi % 4 == 0;
    const bool vg = aligned16(r.dHout) && r.ldo % 4 == 0;
    float (*zs)[ST] = Zs[wave];
    float (*hs)[ST] = Hs[wave];
    float (*gs)[ST] = Gs[wave];
    uint32_t *ms = Ms[wave];

    floatx16 accA, accS;
#pragma unroll
    for (int x = 0; x < 16; ++x) { accA[x] = 0.f; accS[x] = 0.f; }
    float sum_p = 0.f, sum_g = 0.f;

    float4 pz[4], ph[4], pg[4];
    float hf[4] = {1.f, 1.f, 1.f, 1.f};
    uint32_t pw = ~0u;
    float ps = 1.f; // scale_o1 of strip row m
    auto fetch = [&](int64_t r0) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int64_t row = r0 + lr + 8 * it;
            float4 z = make_float4(0.f, 0.f, 0.f, 0.f), hh = z, g = z;
            if (row < r_end) {
                if (lc < r.w_in) {
                    z = load_k4(r.Z, r.ldz, row, lc, r.w_in, vz);
                    hh = load_k4(r.Hin, r.ldi, row, lc, r.w_in, vh);
                    if (r.hin_scale) hf[it] = r.hin_scale[row];
                }
                if (lc < r.w_out) g = load_k4(r.dHout, r.ldo, row, lc, r.w_out, vg);
            }
            pz[it] = z; ph[it] = hh; pg[it] = g;
        }
        if (lane < 32) pw = r0 + lane < r_end ? (r.mask ? r.mask[(r0 + lane) * r.mask_words] : ~0u) : 0u;
        if (a.scale_o1) ps = r0 + m < r_end ? a.scale_o1[r0 + m] : 1.f;
    };
    fetch(w_id * 32);
    for (int64_t strip = w_id; strip < n_strips; strip += n_waves) {
        const int64_t row0 = strip * 32;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            if (r.hin_scale) scale4(ph[it], hf[it]);
            *reinterpret_cast<float4 *>(&zs[lr + 8 * it][lc]) = pz[it];
            *reinterpret_cast<float4 *>(&hs[lr + 8 * it][lc]) = ph[it];
            *reinterpret_cast<float4 *>(&gs[lr + 8 * it][lc]) = pg[it];
        }
        if (lane < 32) ms[lane] = pw;
        const float so = ps;
        __builtin_amdgcn_wave_barrier();
        if (strip + n_waves < n_strips) fetch((strip + n_waves) * 32); // flies during the MFMAs and the stores below
#pragma unroll 4
        for (int s2 = 0; s2 < 16; ++s2) { // node rows 2 s2 + h: Z^T dP, Hin^T dHout and the bias sums
            const int k = 2 * s2 + h;
            const float g = gs[k][m];
            const float p = ((ms[k] >> m) & 1u) ? g : 0.f;
            accA = __builtin_amdgcn_mfma_f32_32x32x2f32(zs[k][m], p, accA, 0, 0, 0);
            accS = __builtin_amdgcn_mfma_f32_32x32x2f32(hs[k][m], g, accS, 0, 0, 0);
            sum_p += p;
            sum_g += g;
        }
        __builtin_amdgcn_sched_barrier(0); // keep the two halves apart: interleaved they do not fit the register file
        floatx16 acc1, acc2;
#pragma unroll
        for (int x = 0; x < 16; ++x) { acc1[x] = 0.f; acc2[x] = 0.f; }
        const uint32_t word = ms[m];
#pragma unroll
        for (int q = 0; q < 4; ++q) { // columns 8 q + 4 h + i: dZ = dP W_agg^T and T = dHout W_self^T for strip row m
            const float4 g4 = *reinterpret_cast<const float4 *>(&gs[m][8 * q + 4 * h]);
            float4 p4 = g4; // dP = dHout * mask, times the row's output factor
            const uint32_t bits = word >> (8 * q + 4 * h);
            if (!(bits & 1u)) p4.x = 0.f;
            if (!(bits & 2u)) p4.y = 0.f;
            if (!(bits & 4u)) p4.z = 0.f;
            if (!(bits & 8u)) p4.w = 0.f;
            if (a.scale_o1) scale4(p4, so);
            const float4 w1 = *reinterpret_cast<const float4 *>(&W1s[m][8 * q + 4 * h]);
            const float4 w2 = *reinterpret_cast<const float4 *>(&W2s[m][8 * q + 4 * h]);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(pick(p4, i), pick(w1, i), acc1, 0, 0, 0);
                acc2 = __builtin_amdgcn_mfma_f32_32x32x2f32(pick(g4, i), pick(w2, i), acc2, 0, 0, 0);
            }
        }
        // dZ leaves through the Z tile and T through the Hin tile (register x of lane (m, h) is strip row
        // 8*(x/4) + 4*h + x%4, column m); layouts without 16-byte stores write the registers directly
        auto store_tile = [&](const floatx16 &o, float (*t)[ST], float *O, int64_t ldo, bool vec_ok) {
            if (vec_ok) {
#pragma unroll
                for (int x = 0; x < 16; ++x) t[8 * (x / 4) + 4 * h + (x % 4)][m] = o[x];
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int64_t row = row0 + lr + 8 * it;
                    if (row < r_end && lc < r.w_in)
                        *reinterpret_cast<float4 *>(O + row * ldo + lc) = *reinterpret_cast<const float4 *>(&t[lr + 8 * it][lc]);
                }
            } else {
#pragma unroll
                for (int x = 0; x < 16; ++x) {
                    const int64_t orow = row0 + 8 * (x / 4) + 4 * h + (x % 4);
                    if (orow < r_end && m < r.w_in) O[orow * ldo + m] = o[x];
                }
            }
        };
        const bool nout4 = r.w_in % 4 == 0;
        __builtin_amdgcn_wave_barrier(); // every lane is done reading the tiles
        store_tile(acc1, zs, a.O1, a.ldo1, nout4 && aligned16(a.O1) && a.ldo1 % 4 == 0);
        store_tile(acc2, hs, a.O2, a.ldo2, nout4 && aligned16(a.O2) && a.ldo2 % 4 == 0);
        __builtin_amdgcn_wave_barrier();
    }
    sum_p += __shfl_xor(sum_p, 32, 64);
    sum_g += __shfl_xor(sum_g, 32, 64);
    float *out = r.partial + w_id * r.stride;
    const int ww = r.w_in * r.w_out;
#pragma unroll
    for (int x = 0; x < 16; ++x) {
        const int i = 8 * (x / 4) + 4 * h + (x % 4);
        if (i < r.w_in && m < r.w_out) {
            out[i * r.w_out + m] = accA[x];
            out[ww + i * r.w_out + m] = accS[x];
        }
    }
    if (lane < 32 && m < r.w_out) {
        out[2 * ww + m] = sum_p;
        out[2 * ww + r.w_out + m] = sum_g;
    }
}

// The same for layers up to 64 wide (w_in <= 32 * MI, w_out <= 32 * NJ, large n): a wavefront owns the
// whole w_in x w_out gradient pair (2 * MI * NJ accumulators), so every operand row is read from
// memory exactly once.  Strips are dealt to the wavefronts round-robin, so at any moment the chip
// reads one contiguous window of the operands.  Short strips (8 node rows; 4, 16 and 32 are no
// faster, nor is keeping two or three strips in flight) keep the staging registers and the
// wave-private LDS tiles small enough for two wavefronts per SIMD beside the 128 accumulator
// registers of the full-width variant, three for the half-width ones.
template <int MI, int NJ, int SR, int WPS> // SR: node rows per strip; WPS: wavefronts per SIMD to compile for
__global__ __launch_bounds__(256, WPS) void grad_strip64_kernel(const ReduceArgs a, int64_t n_waves)
{
    constexpr int WI = 32 * MI, WJ = 32 * NJ; // padded widths
    constexpr int LI = WI / 4, LJ = WJ / 4;   // lanes per row (16-byte accesses)
    constexpr int PI = SR * LI / 64, PJ = SR * LJ / 64; // passes over a strip
    __shared__ __attribute__((aligned(16))) float Zs[4][SR][WI];
    __shared__ __attribute__((aligned(16))) float Hs[4][SR][WI];
    __shared__ __attribute__((aligned(16))) float Gs[4][SR][WJ];
    __shared__ uint32_t Ms[4][SR][NJ];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int m = lane & 31, h = lane >> 5;
    const int ri = lane / LI, ci = (lane % LI) * 4; // coalesced layout of the w_in-wide operands
    const int rj = lane / LJ, cj = (lane % LJ) * 4; // and of dHout
    const int64_t w_id = (int64_t)blockIdx.x * 4 + wave;
    const int64_t n_strips = (a.n + SR - 1) / SR;
    if (w_id >= n_waves) return; // uniform per wavefront; no workgroup barriers below (n_waves <= n_strips)
    const bool self = a.Hin != nullptr;
    const bool vz = aligned16(a.Z) && a.ldz % 4 == 0, vh = self && aligned16(a.Hin) && a.ldi % 4 == 0;
    const bool vg = aligned16(a.dHout) && a.ldo % 4 == 0;
    float (*zs)[WI] = Zs[wave];
    float (*hs)[WI] = Hs[wave];
    float (*gs)[WJ] = Gs[wave];
    uint32_t (*ms)[NJ] = Ms[wave];

    floatx16 accA[MI][NJ], accS[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) { accA[i][j][r] = 0.f; accS[i][j][r] = 0.f; }
    float sum_p[NJ], sum_g[NJ]; // column 32 j + m of dP and of dHout over the node rows 2 s + h
#pragma unroll
    for (int j = 0; j < NJ; ++j) { sum_p[j] = 0.f; sum_g[j] = 0.f; }

    float4 pz[PI], ph[PI], pg[PJ];
    float hf[PI]; // factors of the rows of Hin this lane loads (scaled layout); applied on the way to LDS
    uint32_t pw = ~0u; // lane l < SR * NJ: word l % NJ of strip row l / NJ
    auto fetch = [&](int64_t r0) {
#pragma unroll
        for (int it = 0; it < PI; ++it) {
            const int64_t row = r0 + ri + (64 / LI) * it;
            float4 z = make_float4(0.f, 0.f, 0.f, 0.f), hh = z;
            hf[it] = 1.f;
            if (row < a.n && ci < a.w_in) {
                z = load_k4(a.Z, a.ldz, row, ci, a.w_in, vz);
                if (self) {
                    hh = load_k4(a.Hin, a.ldi, row, ci, a.w_in, vh);
                    if (a.hin_scale) hf[it] = a.hin_scale[row];
                }
            }
            pz[it] = z; ph[it] = hh;
        }
#pragma unroll
        for (int it = 0; it < PJ; ++it) {
            const int64_t row = r0 + rj + (64 / LJ) * it;
            float4 g = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < a.n && cj < a.w_out) g = load_k4(a.dHout, a.ldo, row, cj, a.w_out, vg);
            pg[it] = g;
        }
        if (a.mask && lane < SR * NJ) {
            const int64_t row = r0 + lane / NJ;
            const int word = lane % NJ;
            pw = (row < a.n && 32 * word < a.w_out) ? a.mask[row * a.mask_words + word] : 0u;
        }
    };
    fetch(w_id * SR);
    for (int64_t strip = w_id; strip < n_strips; strip += n_waves) { // wavefront w takes strips w, w + n_waves, ...
#pragma unroll
        for (int it = 0; it < PI; ++it) {
            if (a.hin_scale) scale4(ph[it], hf[it]);
            *reinterpret_cast<float4 *>(&zs[ri + (64 / LI) * it][ci]) = pz[it];
            *reinterpret_cast<float4 *>(&hs[ri + (64 / LI) * it][ci]) = ph[it];
        }
#pragma unroll
        for (int it = 0; it < PJ; ++it) *reinterpret_cast<float4 *>(&gs[rj + (64 / LJ) * it][cj]) = pg[it];
        if (lane < SR * NJ) ms[lane / NJ][lane % NJ] = pw;
        __builtin_amdgcn_wave_barrier();
        if (strip + n_waves < n_strips) fetch((strip + n_waves) * SR);
#pragma unroll
        for (int s2 = 0; s2 < SR / 2; ++s2) {
            const int k = 2 * s2 + h;
            float g[NJ], pp[NJ], z[MI], hh[MI];
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                g[j] = gs[k][32 * j + m];
                pp[j] = ((ms[k][j] >> m) & 1u) ? g[j] : 0.f;
                sum_p[j] += pp[j];
                sum_g[j] += g[j];
            }
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                z[i] = zs[k][32 * i + m];
                hh[i] = hs[k][32 * i + m];
            }
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    accA[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(z[i], pp[j], accA[i][j], 0, 0, 0);
                    if (self) accS[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(hh[i], g[j], accS[i][j], 0, 0, 0);
                }
        }
        __builtin_amdgcn_wave_barrier();
    }
    float *out = a.partial + w_id * a.stride;
    const int ww = a.w_in * a.w_out;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = 32 * i + 8 * (r / 4) + 4 * h + (r % 4), col = 32 * j + m;
                if (row < a.w_in && col < a.w_out) {
                    out[row * a.w_out + col] = accA[i][j][r];
                    if (!a.compact) out[ww + row * a.w_out + col] = accS[i][j][r];
                }
            }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const float sp = sum_p[j] + __shfl_xor(sum_p[j], 32, 64);
        const float sg = sum_g[j] + __shfl_xor(sum_g[j], 32, 64);
        const int col = 32 * j + m;
        if (lane < 32 && col < a.w_out) {
            out[(a.compact ? ww : 2 * ww) + col] = sp;
            if (!a.compact) out[2 * ww + a.w_out + col] = sg;
        }
    }
}

// Partial weight gradient of a single product (compact layout: [X^T dP | colsum dP]) for wide
// layers: one workgroup per 128 x 128 output tile and block of RED_ROWS rows, each wavefront owning a
// 64 x 64 quarter (four MFMA accumulators).  Per step 32 rows of the X tile and of the dP tile are
// staged in LDS (the next step's loads are issued into registers before this step's MFMAs); the
// node axis is the MFMA's k axis.  32 flop per staged byte instead of 8 for 32 x 32 tiles.
constexpr int GB_T = 128;

__global__ __launch_bounds__(256) void grad_big_mfma_kernel(const ReduceArgs a)
{
    __shared__ __attribute__((aligned(16))) float Xs[RED_RK][GB_T];
    __shared__ __attribute__((aligned(16))) float Ps[RED_RK][GB_T];
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int m = lane & 31, h = lane >> 5;
    const int i_base = blockIdx.y * GB_T, j_base = blockIdx.z * GB_T;
    const int wi = (wave >> 1) * 64, wj = (wave & 1) * 64;
    const int64_t r_begin = (int64_t)blockIdx.x * RED_ROWS;
    const int64_t r_end = r_begin + RED_ROWS < a.n ? r_begin + RED_ROWS : a.n;
    const bool vz = aligned16(a.Z) && a.ldz % 4 == 0, vg = aligned16(a.dHout) && a.ldo % 4 == 0;
    const bool bias_wave = blockIdx.y == 0 && (wave >> 1) == 0;

    floatx16 acc[2][2];
#pragma unroll
    for (int ti = 0; ti < 2; ++ti)
#pragma unroll
        for (int tj = 0; tj < 2; ++tj)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[ti][tj][r] = 0.f;
    float accb = 0.f; // column j_base + wj + lane of dP

    float4 rx[4], rp[4];
    auto fetch = [&](int64_t r0) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int idx = tid + it * 256;
            const int r = idx >> 5, c4 = (idx & 31) * 4;
            const int64_t row = r0 + r;
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f), p = x;
            if (row < r_end) {
                if (i_base + c4 < a.w_in) x = load_k4(a.Z, a.ldz, row, i_base + c4, a.w_in, vz);
                if (j_base + c4 < a.w_out) {
                    p = load_k4(a.dHout, a.ldo, row, j_base + c4, a.w_out, vg);
                    if (a.mask) {
                        const int j = j_base + c4;
                        const uint32_t bits = a.mask[row * a.mask_words + (j >> 5)] >> (j & 31);
                        if (!(bits & 1u)) p.x = 0.f;
                        if (!(bits & 2u)) p.y = 0.f;
                        if (!(bits & 4u)) p.z = 0.f;
                        if (!(bits & 8u)) p.w = 0.f;
                    }
                }
            }
            rx[it] = x;
            rp[it] = p;
        }
    };
    fetch(r_begin);
    for (int64_t r0 = r_begin; r0 < r_end; r0 += RED_RK) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int idx = tid + it * 256;
            const int r = idx >> 5, c4 = (idx & 31) * 4;
            *reinterpret_cast<float4 *>(&Xs[r][c4]) = rx[it];
            *reinterpret_cast<float4 *>(&Ps[r][c4]) = rp[it];
        }
        __syncthreads();
        if (r0 + RED_RK < r_end) fetch(r0 + RED_RK);
#pragma unroll
        for (int kp = 0; kp < RED_RK / 2; ++kp) {
            const int k = 2 * kp + h;
            const float a0 = Xs[k][wi + m], a1 = Xs[k][wi + 32 + m];
            const float b0 = Ps[k][wj + m], b1 = Ps[k][wj + 32 + m];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
        }
        if (bias_wave) {
#pragma unroll
            for (int r = 0; r < RED_RK; ++r) accb += Ps[r][wj + lane];
        }
        __syncthreads();
    }

    float *out = a.partial + (int64_t)blockIdx.x * a.stride;
#pragma unroll
    for (int ti = 0; ti < 2; ++ti)
#pragma unroll
        for (int tj = 0; tj < 2; ++tj)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = i_base + wi + 32 * ti + 8 * (r / 4) + 4 * h + (r % 4);
                const int j = j_base + wj + 32 * tj + m;
                if (i < a.w_in && j < a.w_out) out[i * a.w_out + j] = acc[ti][tj][r];
            }
    if (bias_wave) {
        const int j = j_base + wj + lane;
        if (j < a.w_out) out[a.w_in * a.w_out + j] = accb;
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

// Same sums with 16-byte loads (aligned base, ld % 4 == 0, w % 4 == 0): thread t owns four
// columns of every (256 / q)-th row, q = float4 per row rounded up to a power of two.
__global__ __launch_bounds__(256) void colsum_partial_vec_kernel(const float *__restrict__ M, int64_t ld, int64_t n, int32_t w,
                                                                 float *__restrict__ partial)
{
    const int64_t r_begin = (int64_t)blockIdx.x * RED_ROWS;
    const int64_t r_end = r_begin + RED_ROWS < n ? r_begin + RED_ROWS : n;
    __shared__ float4 red[256];
    for (int c0 = 0; c0 < w; c0 += 1024) {
        const int cols4 = (w - c0 < 1024 ? w - c0 : 1024) >> 2;
        int q = 1;
        while (q < cols4) q <<= 1;
        const int lanes_r = 256 / q;
        const int c = threadIdx.x % q, rr = threadIdx.x / q;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        if (c < cols4) {
            const float *p = M + c0 + c * 4;
            int64_t r = r_begin + rr;
            for (; r + 3 * lanes_r < r_end; r += 4 * lanes_r) {
                const float4 v0 = *reinterpret_cast<const float4 *>(p + r * ld);
                const float4 v1 = *reinterpret_cast<const float4 *>(p + (r + lanes_r) * ld);
                const float4 v2 = *reinterpret_cast<const float4 *>(p + (r + 2 * lanes_r) * ld);
                const float4 v3 = *reinterpret_cast<const float4 *>(p + (r + 3 * lanes_r) * ld);
                acc.x += v0.x; acc.y += v0.y; acc.z += v0.z; acc.w += v0.w;
                acc.x += v1.x; acc.y += v1.y; acc.z += v1.z; acc.w += v1.w;
                acc.x += v2.x; acc.y += v2.y; acc.z += v2.z; acc.w += v2.w;
                acc.x += v3.x; acc.y += v3.y; acc.z += v3.z; acc.w += v3.w;
            }
            for (; r < r_end; r += lanes_r) {
                const float4 v = *reinterpret_cast<const float4 *>(p + r * ld);
                acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
            }
        }
        red[threadIdx.x] = acc;
        __syncthreads();
        if (rr == 0 && c < cols4) {
            float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int k = 0; k < lanes_r; ++k) {
                const float4 v = red[k * q + c];
                s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
            }
            *reinterpret_cast<float4 *>(partial + (int64_t)blockIdx.x * w + c0 + c * 4) = s;
        }
        __syncthreads();
    }
}

// Final stage: out[e] = sum over row blocks of partial[b][e], in fp64, fixed order.
// 32 elements x 32 parts per block of 1024 threads.
struct FinalDst { float *ptr[4]; int32_t begin[5]; }; // element ranges [begin[q], begin[q+1]) go to ptr[q]

__global__ __launch_bounds__(1024) void reduce_final_kernel(const float *__restrict__ partial, int64_t n_blocks,
                                                            int32_t row_stride, int32_t stride, const FinalDst dst)
{
    __shared__ double red[32][33];
    const int el = threadIdx.x % 32, part = threadIdx.x / 32;
    const int64_t e = (int64_t)blockIdx.x * 32 + el;
    const int64_t per = (n_blocks + 31) / 32;
    const int64_t b0 = part * per, b1 = b0 + per < n_blocks ? b0 + per : n_blocks;
    double acc = 0.0;
    if (e < stride) {
        int64_t b = b0;
        for (; b + 8 <= b1; b += 8) { // eight independent loads in flight; the additions stay in block order
            float q[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) q[i] = partial[(b + i) * row_stride + e];
#pragma unroll
            for (int i = 0; i < 8; ++i) acc += (double)q[i];
        }
        for (; b < b1; ++b) acc += (double)partial[b * row_stride + e];
    }
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

// Node rows per partial sum of a slice layer's weight gradients: RED_ROWS, or a quarter of it when that
// would give the tiled kernel fewer than 2048 workgroups (a workgroup walks its rows in dependent steps
// of 32, so on small graphs shorter walks in more workgroups finish sooner: cfg2 80 -> 35 us).
inline int32_t layer_grad_rows(int64_t n, int32_t w_in, int32_t w_out)
{
    const int64_t tiles = (int64_t)((w_in + RED_TILE - 1) / RED_TILE) * ((w_out + RED_TILE - 1) / RED_TILE);
    return red_blocks(n) * tiles < 2048 ? RED_ROWS / 4 : RED_ROWS;
}
inline int64_t layer_grad_blocks(int64_t n, int32_t w_in, int32_t w_out)
{
    const int32_t rows = layer_grad_rows(n, w_in, w_out);
    return (n + rows - 1) / rows;
}


// ---- pieces of the transform-first layer order -------------------------------------------------
// Hout[v, j] = act(P[v, j] + bias[j]) (+ Hout[v, j] when add), mask bit j of row v = [P + bias > 0].
// One thread per element of the row padded to a multiple of 32 columns, so every half wavefront lies
// inside one mask word of one row and a ballot assembles the word.
__global__ __launch_bounds__(256) void bias_act_add_kernel(const float *__restrict__ P, int64_t ldp, const float *__restrict__ bias,
                                                           float *__restrict__ Hout, int64_t ldo, int add, uint32_t *__restrict__ mask,
                                                           int64_t mask_words, int64_t n, int32_t w_out, int32_t act)
{
    const int wpad = (w_out + 31) / 32 * 32;
    const int64_t total = n * (int64_t)wpad;
    const int64_t padded_total = (total + 63) / 64 * 64; // whole wavefronts take part in every ballot
    const int lane = threadIdx.x & 63;
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < padded_total; t += (int64_t)gridDim.x * 256) {
        const int64_t row = t / wpad;
        const int col = (int)(t - row * wpad);
        const bool valid = t < total && col < w_out;
        const float p = valid ? P[row * ldp + col] + (bias ? bias[col] : 0.f) : 0.f;
        const bool pos = valid && p > 0.f;
        const unsigned long long bits = __ballot(pos);
        if (valid) {
            float r = act == SLICEGCN_ACT_RELU ? (pos ? p : 0.f) : p;
            if (add) r += Hout[row * ldo + col];
            Hout[row * ldo + col] = r;
        }
        if (act == SLICEGCN_ACT_RELU && (lane & 31) == 0 && t < total)
            mask[row * mask_words + (col >> 5)] = (uint32_t)(bits >> (lane & 32));
    }
}

// dP[v, j] = dHout[v, j] where the activation passed (all of it when mask == NULL)
__global__ __launch_bounds__(256) void mask_apply_kernel(const float *__restrict__ dHout, int64_t ldo, const uint32_t *__restrict__ mask,
                                                         int64_t mask_words, float *__restrict__ dP, int64_t ldp, int64_t n, int32_t w_out)
{
    const int64_t total = n * (int64_t)w_out;
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
        const int64_t row = t / w_out;
        const int col = (int)(t - row * w_out);
        float v = dHout[row * ldo + col];
        if (mask && ((mask[row * mask_words + (col >> 5)] >> (col & 31)) & 1u) == 0u) v = 0.f;
        dP[row * ldp + col] = v;
    }
}

// Wt[j][i] = W[i][j] for a rows x cols row-major W (weights are small: one thread per element)
__global__ __launch_bounds__(256) void transpose_kernel(const float *__restrict__ W, int32_t rows, int32_t cols, float *__restrict__ Wt)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= rows * cols) return;
    const int i = t / cols, j = t - i * cols;
    Wt[(int64_t)j * rows + i] = W[t];
}

inline unsigned ew_grid(int64_t total)
{
    const int64_t b = (total + 255) / 256;
    return (unsigned)(b < 1 ? 1 : (b > 262144 ? 262144 : b));
}

// aggregate first: Z = A^ Hin, then the weight products; transform first: T = Hin W_agg, then P = A^ T.
// Equal in exact arithmetic; the second gathers rows of w_out instead of w_in columns.
inline bool transform_first(const slicegcn_layer_desc *d)
{
    if (d->flags & SLICEGCN_LAYER_TRANSFORM_FIRST) return true;
    return (d->flags & SLICEGCN_LAYER_ORDER_AUTO) && d->w_out < d->w_in;
}

int check_layer(const slicegcn_graph *g, const slicegcn_layer_desc *d, const slicegcn_layer_params *p, const char *who)
{
    SG_REQUIRE(g && d && p, SLICEGCN_EINVAL, "%s: NULL graph, desc or params", who);
    SG_REQUIRE(d->w_in >= 1 && d->w_out >= 1, SLICEGCN_EINVAL, "%s: widths must be >= 1", who);
    SG_REQUIRE(d->act == SLICEGCN_ACT_NONE || d->act == SLICEGCN_ACT_RELU, SLICEGCN_EINVAL, "%s: unknown act %d", who, d->act);
    SG_REQUIRE((d->flags & ~(SLICEGCN_LAYER_Z_VALID | SLICEGCN_LAYER_TRANSFORM_FIRST | SLICEGCN_LAYER_ORDER_AUTO |
                             SLICEGCN_LAYER_IN_SCALED | SLICEGCN_LAYER_OUT_SCALED)) == 0, SLICEGCN_EINVAL,
               "%s: unknown flag bits 0x%x", who, d->flags);
    SG_REQUIRE(!((d->flags & (SLICEGCN_LAYER_IN_SCALED | SLICEGCN_LAYER_OUT_SCALED)) && transform_first(d)), SLICEGCN_EINVAL,
               "%s: the scaled layout needs the aggregate-first order", who);
    SG_REQUIRE(!((d->flags & SLICEGCN_LAYER_TRANSFORM_FIRST) && (d->flags & SLICEGCN_LAYER_ORDER_AUTO)), SLICEGCN_EINVAL,
               "%s: TRANSFORM_FIRST and ORDER_AUTO exclude each other", who);
    SG_REQUIRE(!((d->flags & SLICEGCN_LAYER_Z_VALID) && transform_first(d)), SLICEGCN_EINVAL,
               "%s: Z_VALID needs the aggregate-first order (no aggregation of the input is kept by the transform-first order)", who);
    SG_REQUIRE(p->W_agg != nullptr, SLICEGCN_EINVAL, "%s: W_agg is NULL", who);
    SG_REQUIRE(p->W_self != nullptr || p->b_self == nullptr, SLICEGCN_EINVAL, "%s: b_self without W_self", who);
    return SLICEGCN_OK;
}

int check_saved(const slicegcn_layer_desc *d, const slicegcn_layer_saved *s, const char *who)
{
    SG_REQUIRE(s != nullptr, SLICEGCN_EINVAL, "%s: saved is NULL", who);
    if (!transform_first(d)) { // the transform-first order keeps no aggregation: Z is neither written nor read
        SG_REQUIRE(s->Z != nullptr, SLICEGCN_EINVAL, "%s: saved->Z is NULL", who);
        SG_REQUIRE(s->ldz >= d->w_in && s->ldz % 4 == 0 && aligned16(s->Z), SLICEGCN_EINVAL,
                   "%s: saved->Z needs ldz >= w_in, ldz %% 4 == 0 and a 16-byte aligned base", who);
    }
    if (d->act == SLICEGCN_ACT_RELU)
        SG_REQUIRE(s->mask && s->mask_words >= (d->w_out + 31) / 32, SLICEGCN_EINVAL,
                   "%s: mask is NULL or mask_words < ceil(w_out / 32)", who);
    return SLICEGCN_OK;
}

} // namespace

// shared with misc.hip
int launch_colsum_partial(const float *M, int64_t ld, int64_t n, int32_t w, float *ws, hipStream_t stream)
{
    const int64_t nb = red_blocks(n);
    if (aligned16(M) && ld % 4 == 0 && w % 4 == 0)
        colsum_partial_vec_kernel<<<(unsigned)nb, 256, 0, stream>>>(M, ld, n, w, ws);
    else
        colsum_partial_kernel<<<(unsigned)nb, 256, 0, stream>>>(M, ld, n, w, ws);
    SG_LAUNCH_CHECK();
    return SLICEGCN_OK;
}

int launch_colsum_final(const float *ws_first, int64_t n, int32_t ws_row, int32_t count, float *out, hipStream_t stream)
{
    FinalDst dst;
    dst.ptr[0] = out; dst.ptr[1] = dst.ptr[2] = dst.ptr[3] = nullptr;
    dst.begin[0] = 0; dst.begin[1] = dst.begin[2] = dst.begin[3] = dst.begin[4] = count;
    reduce_final_kernel<<<(unsigned)((count + 31) / 32), 1024, 0, stream>>>(ws_first, red_blocks(n), ws_row, count, dst);
    SG_LAUNCH_CHECK();
    return SLICEGCN_OK;
}

size_t colsum_workspace_bytes(int64_t n, int32_t w) { return (size_t)red_blocks(n) * (size_t)w * sizeof(float); }

} // namespace slicegcn

using namespace slicegcn;

// partial sums of a dense layer's weight and bias gradients: one [w_in*w_out + w_out] row per block of 1024 rows
static size_t linear_partial_bytes(int64_t n, int32_t w_in, int32_t w_out)
{
    const size_t stride = (size_t)w_in * w_out + (size_t)w_out;
    return (size_t)round_up((int64_t)(red_blocks(n) * stride * sizeof(float)), 256);
}

// dW = X^T (dY * mask) (w_in x w_out), db = colsum(dY * mask); NULL outputs are skipped.  ws: linear_partial_bytes bytes.
static int launch_linear_grads(const float *X, int64_t ldx, int64_t n, int32_t w_in, int32_t w_out, const uint32_t *m,
                               int64_t mask_words, const float *dY, int64_t lddy, float *dW, float *db, void *ws, hipStream_t stream)
{
    const int64_t nb = red_blocks(n);
    const int ww = w_in * w_out;
    const int32_t stride = ww + w_out;
    ReduceArgs r;
    r.Z = X; r.ldz = ldx; r.Hin = nullptr; r.ldi = 0; r.dHout = dY; r.ldo = lddy;
    r.mask = m; r.mask_words = mask_words;
    r.partial = static_cast<float *>(ws); r.n = n; r.w_in = w_in; r.w_out = w_out; r.stride = stride; r.compact = 1;
    dim3 grid((unsigned)nb, (unsigned)((w_in + RED_TILE - 1) / RED_TILE), (unsigned)((w_out + RED_TILE - 1) / RED_TILE));
    if (w_in > 64 || w_out > 64) { // wide layer: 128 x 128 output tiles
        dim3 big((unsigned)nb, (unsigned)((w_in + GB_T - 1) / GB_T), (unsigned)((w_out + GB_T - 1) / GB_T));
        grad_big_mfma_kernel<<<big, 256, 0, stream>>>(r);
    } else {
        grad_partial_mfma_kernel<<<grid, 256, 0, stream>>>(r);
    }
    SG_LAUNCH_CHECK();
    FinalDst dst;
    dst.ptr[0] = dW; dst.ptr[1] = db; dst.ptr[2] = dst.ptr[3] = nullptr;
    dst.begin[0] = 0; dst.begin[1] = ww; dst.begin[2] = dst.begin[3] = dst.begin[4] = stride;
    reduce_final_kernel<<<(unsigned)((stride + 31) / 32), 1024, 0, stream>>>(r.partial, nb, stride, stride, dst);
    SG_LAUNCH_CHECK();
    return SLICEGCN_OK;
}

// ---- transform-first order of a slice layer ------------------------------------------------
// forward : T = Hin W_agg;  S = Hin W_self + b_self (stored straight into Hout);  P = A^ T;
//           Hout = act(P + b) + S,  mask = [P + b > 0]
// backward: dP = dHout * mask;  db = colsum dP;  G = A^^T dP;  dW_agg = Hin^T G;
//           dW_self = Hin^T dHout, db_self = colsum dHout;  dHin = G W_agg^T + dHout W_self^T
// Nothing of the forward pass but the mask is kept: the backward pass aggregates dP instead of re-using A^ Hin.
static size_t tf_mat_bytes(int64_t n, int32_t w) { return (size_t)round_up(n * round_up(w, 32) * (int64_t)sizeof(float), 256); }
static size_t tf_wt_bytes(const slicegcn_layer_desc *d) { return (size_t)round_up((int64_t)d->w_in * d->w_out * (int64_t)sizeof(float), 256); }
static size_t tf_red_bytes(int64_t n, const slicegcn_layer_desc *d)
{
    const size_t a = linear_partial_bytes(n, d->w_in, d->w_out), b = (size_t)round_up((int64_t)colsum_workspace_bytes(n, d->w_out), 256);
    return a > b ? a : b;
}
// backward workspace: [dP | G | W_agg^T | W_self^T | reduction partials | aggregation workspace]
static size_t tf_bwd_bytes(const slicegcn_graph *g, const slicegcn_layer_desc *d)
{
    return 2 * tf_mat_bytes(g->n, d->w_out) + 2 * tf_wt_bytes(d) + tf_red_bytes(g->n, d) + spmm_workspace_bytes(g->tr, d->w_out);
}

static int layer_fwd_transform_first(const slicegcn_graph *g, const slicegcn_layer_desc *desc, const slicegcn_layer_params *params,
                                     const float *Hin, int64_t ldi, float *Hout, int64_t ldo, slicegcn_layer_saved *saved,
                                     void *ws, size_t ws_bytes, hipStream_t stream)
{
    const int w_in = desc->w_in, w_out = desc->w_out;
    const size_t need = slicegcn_layer_fwd_workspace_bytes(g, desc);
    SG_REQUIRE(ws != nullptr && ws_bytes >= need, SLICEGCN_EWORKSPACE, "layer_fwd: workspace of %zu bytes, %zu needed", ws_bytes, need);
    SG_REQUIRE((reinterpret_cast<uintptr_t>(ws) & 255u) == 0, SLICEGCN_EINVAL, "layer_fwd: workspace not 256-byte aligned");
    const int64_t ldt = round_up(w_out, 32);
    float *T = static_cast<float *>(ws);
    float *P = reinterpret_cast<float *>(static_cast<char *>(ws) + tf_mat_bytes(g->n, w_out));
    void *agg_ws = static_cast<char *>(ws) + 2 * tf_mat_bytes(g->n, w_out);
    {
        ProfScope prof(SLICEGCN_PROF_DENSE_FWD, w_out, stream);
        PairArgs a;
        a.A1 = Hin; a.lda1 = ldi; a.A2 = nullptr; a.lda2 = 0;
        a.B1 = params->W_agg; a.B2 = nullptr; a.bias1 = a.bias2 = nullptr;
        a.O1 = T; a.ldo1 = ldt; a.O2 = nullptr; a.ldo2 = 0;
        a.mask = nullptr; a.mask_words = 0;
        a.n = g->n; a.K = w_in; a.Nout = w_out; a.ldw = w_out; a.act = SLICEGCN_ACT_NONE;
        if (int rc = launch_pair<false>(a, stream)) return rc;
        if (params->W_self) { // the self term goes straight to the output; the epilogue below adds the activated part
            a.B1 = params->W_self; a.bias1 = params->b_self; a.O1 = Hout; a.ldo1 = ldo;
            if (int rc = launch_pair<false>(a, stream)) return rc;
        }
    }
    if (int rc = launch_spmm(g, g->fwd, T, ldt, w_out, P, ldt, nullptr, 0, agg_ws, spmm_workspace_bytes(g->fwd, w_out), stream)) return rc;
    ProfScope prof(SLICEGCN_PROF_DENSE_FWD, w_out, stream);
    const int64_t total = g->n * round_up(w_out, 32);
    bias_act_add_kernel<<<ew_grid(total), 256, 0, stream>>>(P, ldt, params->b, Hout, ldo, params->W_self != nullptr,
                                                            desc->act == SLICEGCN_ACT_RELU ? saved->mask : nullptr, saved->mask_words,
                                                            g->n, w_out, desc->act);
    SG_LAUNCH_CHECK();
    return SLICEGCN_OK;
}

static int layer_bwd_transform_first(const slicegcn_graph *g, const slicegcn_layer_desc *desc, const slicegcn_layer_params *params,
                                     const float *Hin, int64_t ldi, const uint32_t *mask, int64_t mask_words, const float *dHout,
                                     int64_t ldo, float *dHin, int64_t ldgi, slicegcn_layer_grads *grads, void *ws, hipStream_t stream)
{
    const int w_in = desc->w_in, w_out = desc->w_out;
    const int64_t n = g->n, ldp = round_up(w_out, 32);
    char *base = static_cast<char *>(ws);
    float *dP = reinterpret_cast<float *>(base);
    float *G = reinterpret_cast<float *>(base + tf_mat_bytes(n, w_out));
    float *WaT = reinterpret_cast<float *>(base + 2 * tf_mat_bytes(n, w_out));
    float *WsT = reinterpret_cast<float *>(base + 2 * tf_mat_bytes(n, w_out) + tf_wt_bytes(desc));
    void *red = base + 2 * tf_mat_bytes(n, w_out) + 2 * tf_wt_bytes(desc);
    void *agg_ws = static_cast<char *>(red) + tf_red_bytes(n, desc);
    {
        ProfScope prof(SLICEGCN_PROF_DENSE_BWD, w_out, stream);
        mask_apply_kernel<<<ew_grid(n * w_out), 256, 0, stream>>>(dHout, ldo, mask, mask_words, dP, ldp, n, w_out);
        SG_LAUNCH_CHECK();
    }
    if (int rc = launch_spmm(g, g->tr, dP, ldp, w_out, G, ldp, nullptr, 0, agg_ws, spmm_workspace_bytes(g->tr, w_out), stream)) return rc;
    {
        ProfScope prof(SLICEGCN_PROF_GRAD_REDUCE, w_out, stream);
        if (grads->db) {
            if (int rc = launch_colsum_partial(dP, ldp, n, w_out, static_cast<float *>(red), stream)) return rc;
            if (int rc = launch_colsum_final(static_cast<float *>(red), n, w_out, w_out, grads->db, stream)) return rc;
        }
        if (grads->dW_agg)
            if (int rc = launch_linear_grads(Hin, ldi, n, w_in, w_out, nullptr, 0, G, ldp, grads->dW_agg, nullptr, red, stream)) return rc;
        if (params->W_self && (grads->dW_self || grads->db_self))
            if (int rc = launch_linear_grads(Hin, ldi, n, w_in, w_out, nullptr, 0, dHout, ldo, grads->dW_self, grads->db_self, red, stream))
                return rc;
    }
    if (dHin) { // dHin = G W_agg^T + dHout W_self^T: one forward-form launch over the transposed weights
        ProfScope prof(SLICEGCN_PROF_DENSE_BWD, w_in, stream);
        const int count = w_in * w_out;
        transpose_kernel<<<(count + 255) / 256, 256, 0, stream>>>(params->W_agg, w_in, w_out, WaT);
        if (params->W_self) transpose_kernel<<<(count + 255) / 256, 256, 0, stream>>>(params->W_self, w_in, w_out, WsT);
        SG_LAUNCH_CHECK();
        PairArgs a;
        a.A1 = G; a.lda1 = ldp;
        a.A2 = params->W_self ? dHout : nullptr; a.lda2 = ldo;
        a.B1 = WaT; a.B2 = params->W_self ? WsT : nullptr;
        a.bias1 = a.bias2 = nullptr;
        a.O1 = dHin; a.ldo1 = ldgi; a.O2 = nullptr; a.ldo2 = 0;
        a.mask = nullptr; a.mask_words = 0;
        a.n = n; a.K = w_out; a.Nout = w_in; a.ldw = w_in; a.act = SLICEGCN_ACT_NONE;
        if (int rc = launch_pair<false>(a, stream)) return rc;
    }
    return SLICEGCN_OK;
}

extern "C" int slicegcn_layer_fwd(const slicegcn_graph *g, const slicegcn_layer_desc *desc,
                                  const slicegcn_layer_params *params, const float *Hin, int64_t ldi,
                                  float *Hout, int64_t ldo, slicegcn_layer_saved *saved, void *ws, size_t ws_bytes,
                                  void *stream_)
{
    if (int rc = check_layer(g, desc, params, "layer_fwd")) return rc;
    SG_REQUIRE(Hin && Hout, SLICEGCN_EINVAL, "layer_fwd: NULL Hin or Hout");
    SG_REQUIRE(ldi >= desc->w_in && ldo >= desc->w_out, SLICEGCN_EINVAL, "layer_fwd: leading dimension too small");
    if (int rc = check_saved(desc, saved, "layer_fwd")) return rc;
    hipStream_t stream = as_stream(stream_);
    if (transform_first(desc)) return layer_fwd_transform_first(g, desc, params, Hin, ldi, Hout, ldo, saved, ws, ws_bytes, stream);

    if (!(desc->flags & SLICEGCN_LAYER_Z_VALID))
        if (int rc = launch_spmm(g, g->fwd, Hin, ldi, desc->w_in, saved->Z, saved->ldz, nullptr, 0, ws, ws_bytes, stream,
                                 (desc->flags & SLICEGCN_LAYER_IN_SCALED) != 0))
            return rc;

    PairArgs a;
    a.A1 = saved->Z; a.lda1 = saved->ldz;
    a.A2 = params->W_self ? Hin : nullptr; a.lda2 = ldi;
    a.B1 = params->W_agg; a.B2 = params->W_self;
    a.bias1 = params->b; a.bias2 = params->b_self;
    a.O1 = Hout; a.ldo1 = ldo; a.O2 = nullptr; a.ldo2 = 0;
    a.mask = desc->act == SLICEGCN_ACT_RELU ? saved->mask : nullptr; a.mask_words = saved->mask_words;
    a.n = g->n; a.K = desc->w_in; a.Nout = desc->w_out; a.ldw = desc->w_out; a.act = desc->act;
    a.scale2 = ((desc->flags & SLICEGCN_LAYER_IN_SCALED) && params->W_self) ? g->sqrtd : nullptr;
    a.scale_o1 = (desc->flags & SLICEGCN_LAYER_OUT_SCALED) ? g->dinv : nullptr;
    ProfScope prof(SLICEGCN_PROF_DENSE_FWD, desc->w_out, stream);
    return launch_pair<false>(a, stream);
}

extern "C" size_t slicegcn_layer_fwd_workspace_bytes(const slicegcn_graph *g, const slicegcn_layer_desc *desc)
{
    if (!g || !desc || desc->w_in < 1 || desc->w_out < 1) return 0;
    if (transform_first(desc)) return 2 * tf_mat_bytes(g->n, desc->w_out) + spmm_workspace_bytes(g->fwd, desc->w_out);
    return spmm_workspace_bytes(g->fwd, desc->w_in);
}

// layout of the backward workspace: [partial weight gradients | dZ (only with dHin) | aggregation workspace (only with dHin)]
static size_t bwd_partial_bytes(int64_t n, const slicegcn_layer_desc *desc)
{
    const size_t stride = 2 * (size_t)desc->w_in * desc->w_out + 2 * (size_t)desc->w_out;
    return (size_t)round_up((int64_t)(layer_grad_blocks(n, desc->w_in, desc->w_out) * stride * sizeof(float)), 256);
}
static size_t bwd_dz_bytes(int64_t n, const slicegcn_layer_desc *desc)
{
    return (size_t)round_up(n * round_up(desc->w_in, 32) * (int64_t)sizeof(float), 256);
}

extern "C" size_t slicegcn_layer_bwd_workspace_bytes(const slicegcn_graph *g, const slicegcn_layer_desc *desc, int need_dHin)
{
    if (!g || !desc || desc->w_in < 1 || desc->w_out < 1) return 0;
    if (transform_first(desc)) return tf_bwd_bytes(g, desc);
    size_t bytes = bwd_partial_bytes(g->n, desc);
    if (need_dHin) bytes += bwd_dz_bytes(g->n, desc) + spmm_workspace_bytes(g->tr, desc->w_in);
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
    const size_t need = slicegcn_layer_bwd_workspace_bytes(g, desc, dHin != nullptr);
    SG_REQUIRE(ws != nullptr && ws_bytes >= need, SLICEGCN_EWORKSPACE, "layer_bwd: workspace of %zu bytes, %zu needed",
               ws_bytes, need);
    SG_REQUIRE((reinterpret_cast<uintptr_t>(ws) & 255u) == 0, SLICEGCN_EINVAL, "layer_bwd: workspace not 256-byte aligned");
    hipStream_t stream = as_stream(stream_);
    const uint32_t *mask = desc->act == SLICEGCN_ACT_RELU ? saved->mask : nullptr;
    const int w_in = desc->w_in, w_out = desc->w_out;
    if (transform_first(desc)) return layer_bwd_transform_first(g, desc, params, Hin, ldi, mask, saved->mask_words, dHout, ldo, dHin, ldgi, grads, ws, stream);

    // ---- input gradient, dense half: dZ = dP W_agg^T (staged, rows scaled by D~^-1/2) and T = dHout W_self^T (into dHin) ----
    const int64_t ldz_in = round_up(w_in, 32); // rows of the gathered operand start on 128-byte boundaries
    char *after_partials = static_cast<char *>(ws) + bwd_partial_bytes(g->n, desc);
    float *dZ = reinterpret_cast<float *>(after_partials);
    auto input_gradient_args = [&]() {
        PairArgs a;
        a.A1 = dHout; a.lda1 = ldo;
        a.A2 = params->W_self ? dHout : nullptr; a.lda2 = ldo;
        a.B1 = params->W_agg; a.B2 = params->W_self;
        a.bias1 = a.bias2 = nullptr;
        a.O1 = dZ; a.ldo1 = ldz_in;
        a.O2 = params->W_self ? dHin : nullptr; a.ldo2 = ldgi;
        a.mask = const_cast<uint32_t *>(mask); a.mask_words = saved->mask_words;
        a.n = g->n; a.K = w_out; a.Nout = w_in; a.ldw = w_out; a.act = desc->act;
        a.scale_o1 = g->dinv; // dZ is staged as D~^-1/2 dZ: its aggregation then skips the stored values
        return a;
    };
    // narrow layers with a self term: the kernel that forms the weight gradients also forms dZ and T (one read of dHout)
    const bool fused_inputs = dHin && params->W_self && w_in <= 32 && w_out <= 32 && g->n >= 65536;

    // ---- parameter gradients: per-row-block partial sums, then an fp64 combination ----
    float *partial = static_cast<float *>(ws);
    const int64_t nb = layer_grad_blocks(g->n, w_in, w_out); // partial sums the workspace has room for
    const int32_t stride = 2 * w_in * w_out + 2 * w_out;
    {
        ProfScope prof(SLICEGCN_PROF_GRAD_REDUCE, w_out, stream);
        ReduceArgs r;
        r.Z = saved->Z; r.ldz = saved->ldz;
        r.Hin = params->W_self ? Hin : nullptr; r.ldi = ldi;
        r.dHout = dHout; r.ldo = ldo;
        r.mask = mask; r.mask_words = saved->mask_words;
        r.partial = partial; r.n = g->n; r.w_in = w_in; r.w_out = w_out; r.stride = stride; r.compact = 0;
        r.rows_per_block = layer_grad_rows(g->n, w_in, w_out);
        r.hin_scale = (desc->flags & SLICEGCN_LAYER_IN_SCALED) ? g->sqrtd : nullptr;
        dim3 grid((unsigned)nb, (unsigned)((w_in + RED_TILE - 1) / RED_TILE), (unsigned)((w_out + RED_TILE - 1) / RED_TILE));
        int64_t n_partials = nb;
        if (w_in <= 32 && w_out <= 32 && g->n >= 65536) {
            // one partial per wavefront, at most as many as the workspace has rows (nb) and as fill the chip
            int64_t waves = nb < 8192 ? nb : 8192;
            const int64_t n_strips = (g->n + 31) / 32;
            if (waves > n_strips) waves = n_strips;
            n_partials = waves;
            if (fused_inputs) { // weight gradients and the two input-gradient products in one sweep over the rows
                PairArgs a = input_gradient_args();
                bwd_strip32_kernel<<<(unsigned)((waves + 3) / 4), 256, 0, stream>>>(r, a, waves);
            } else {
                grad_strip32_kernel<<<(unsigned)((waves + 3) / 4), 256, 0, stream>>>(r, waves);
            }
        } else if (w_in <= 64 && w_out <= 64 && g->n >= ((int64_t)1 << 21)) {
            // whole waves of resident workgroups (256 CUs x 3 workgroups x 4 wavefronts) when the workspace allows
            const int64_t resident = 3072;
            int64_t waves = nb >= resident ? nb / resident * resident : nb >= 2048 ? 2048 : nb;
            const int64_t n_strips = (g->n + 7) / 8; // strips of 8 rows in every variant launched here
            if (waves > n_strips) waves = n_strips;
            n_partials = waves;
            const unsigned gb = (unsigned)((waves + 3) / 4);
            if (w_in <= 32) grad_strip64_kernel<1, 2, 8, 3><<<gb, 256, 0, stream>>>(r, waves);
            else if (w_out <= 32) grad_strip64_kernel<2, 1, 8, 3><<<gb, 256, 0, stream>>>(r, waves);
            else grad_strip64_kernel<2, 2, 8, 2><<<gb, 256, 0, stream>>>(r, waves);
        } else {
            grad_partial_mfma_kernel<<<grid, 256, 0, stream>>>(r);
        }
        SG_LAUNCH_CHECK();
        FinalDst dst;
        const int ww = w_in * w_out;
        dst.ptr[0] = grads->dW_agg;
        dst.ptr[1] = params->W_self ? grads->dW_self : nullptr;
        dst.ptr[2] = grads->db;
        dst.ptr[3] = params->W_self ? grads->db_self : nullptr;
        dst.begin[0] = 0; dst.begin[1] = ww; dst.begin[2] = 2 * ww; dst.begin[3] = 2 * ww + w_out; dst.begin[4] = stride;
        reduce_final_kernel<<<(unsigned)((stride + 31) / 32), 1024, 0, stream>>>(partial, n_partials, stride, stride, dst);
        SG_LAUNCH_CHECK();
    }

    // ---- input gradient: dHin = A^^T (dP W_agg^T) + dHout W_self^T ----
    if (dHin) {
        void *agg_ws = after_partials + bwd_dz_bytes(g->n, desc);
        const size_t agg_ws_bytes = spmm_workspace_bytes(g->tr, w_in);
        const int64_t ldz = ldz_in;
        if (!fused_inputs) {
            PairArgs a = input_gradient_args();
            ProfScope prof(SLICEGCN_PROF_DENSE_BWD, w_in, stream);
            if (int rc = launch_pair<true>(a, stream)) return rc;
        }
        // padding columns of dZ are never read as data: the aggregation masks them on store
        if (int rc = launch_spmm(g, g->tr, dZ, ldz, w_in, dHin, ldgi, params->W_self ? dHin : nullptr, ldgi, agg_ws, agg_ws_bytes, stream,
                                 true))
            return rc;
    }
    return SLICEGCN_OK;
}

// ---- dense layer Y = act(X W + b): the unit of the paper's classifier MLP_CLS and of MLP_FF ----

extern "C" int slicegcn_linear_fwd(const float *X, int64_t ldx, int64_t n, int32_t w_in, int32_t w_out, const float *W,
                                   const float *b, int32_t act, float *Y, int64_t ldy, uint32_t *mask, int64_t mask_words,
                                   void *stream_)
{
    SG_REQUIRE(X && W && Y, SLICEGCN_EINVAL, "linear_fwd: NULL X, W or Y");
    SG_REQUIRE(n >= 1 && w_in >= 1 && w_out >= 1, SLICEGCN_EINVAL, "linear_fwd: sizes must be >= 1");
    SG_REQUIRE(ldx >= w_in && ldy >= w_out, SLICEGCN_EINVAL, "linear_fwd: leading dimension too small");
    SG_REQUIRE(act == SLICEGCN_ACT_NONE || act == SLICEGCN_ACT_RELU, SLICEGCN_EINVAL, "linear_fwd: unknown act %d", act);
    if (act == SLICEGCN_ACT_RELU)
        SG_REQUIRE(mask && mask_words >= (w_out + 31) / 32, SLICEGCN_EINVAL,
                   "linear_fwd: mask is NULL or mask_words < ceil(w_out / 32)");
    hipStream_t stream = as_stream(stream_);
    PairArgs a;
    a.A1 = X; a.lda1 = ldx; a.A2 = nullptr; a.lda2 = 0;
    a.B1 = W; a.B2 = nullptr; a.bias1 = b; a.bias2 = nullptr;
    a.O1 = Y; a.ldo1 = ldy; a.O2 = nullptr; a.ldo2 = 0;
    a.mask = act == SLICEGCN_ACT_RELU ? mask : nullptr; a.mask_words = mask_words;
    a.n = n; a.K = w_in; a.Nout = w_out; a.ldw = w_out; a.act = act;
    ProfScope prof(SLICEGCN_PROF_LINEAR_FWD, w_out, stream);
    return launch_pair<false>(a, stream);
}

extern "C" size_t slicegcn_linear_bwd_workspace_bytes(int64_t n, int32_t w_in, int32_t w_out)
{
    if (n < 1 || w_in < 1 || w_out < 1) return 0;
    return linear_partial_bytes(n, w_in, w_out);
}

extern "C" int slicegcn_linear_bwd(const float *X, int64_t ldx, int64_t n, int32_t w_in, int32_t w_out, const float *W,
                                   int32_t act, const uint32_t *mask, int64_t mask_words, const float *dY, int64_t lddy,
                                   float *dX, int64_t lddx, float *dW, float *db, void *ws, size_t ws_bytes, void *stream_)
{
    SG_REQUIRE(X && W && dY, SLICEGCN_EINVAL, "linear_bwd: NULL X, W or dY");
    SG_REQUIRE(n >= 1 && w_in >= 1 && w_out >= 1, SLICEGCN_EINVAL, "linear_bwd: sizes must be >= 1");
    SG_REQUIRE(ldx >= w_in && lddy >= w_out && (dX == nullptr || lddx >= w_in), SLICEGCN_EINVAL,
               "linear_bwd: leading dimension too small");
    SG_REQUIRE(act == SLICEGCN_ACT_NONE || act == SLICEGCN_ACT_RELU, SLICEGCN_EINVAL, "linear_bwd: unknown act %d", act);
    if (act == SLICEGCN_ACT_RELU)
        SG_REQUIRE(mask && mask_words >= (w_out + 31) / 32, SLICEGCN_EINVAL,
                   "linear_bwd: mask is NULL or mask_words < ceil(w_out / 32)");
    hipStream_t stream = as_stream(stream_);
    const uint32_t *m = act == SLICEGCN_ACT_RELU ? mask : nullptr;
    if (dW || db) {
        const size_t need = linear_partial_bytes(n, w_in, w_out);
        SG_REQUIRE(ws != nullptr && ws_bytes >= need, SLICEGCN_EWORKSPACE, "linear_bwd: workspace of %zu bytes, %zu needed",
                   ws_bytes, need);
        SG_REQUIRE((reinterpret_cast<uintptr_t>(ws) & 255u) == 0, SLICEGCN_EINVAL, "linear_bwd: workspace not 256-byte aligned");
        ProfScope prof(SLICEGCN_PROF_LINEAR_GRAD, w_out, stream);
        if (int rc = launch_linear_grads(X, ldx, n, w_in, w_out, m, mask_words, dY, lddy, dW, db, ws, stream)) return rc;
    }
    if (dX) {
        PairArgs a;
        a.A1 = dY; a.lda1 = lddy; a.A2 = nullptr; a.lda2 = 0;
        a.B1 = W; a.B2 = nullptr; a.bias1 = a.bias2 = nullptr;
        a.O1 = dX; a.ldo1 = lddx; a.O2 = nullptr; a.ldo2 = 0;
        a.mask = const_cast<uint32_t *>(m); a.mask_words = mask_words;
        a.n = n; a.K = w_out; a.Nout = w_in; a.ldw = w_out; a.act = act;
        ProfScope prof(SLICEGCN_PROF_LINEAR_BWD, w_in, stream);
        if (int rc = launch_pair<true>(a, stream)) return rc;
    }
    return SLICEGCN_OK;
}
