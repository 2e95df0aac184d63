// Bandwidth-bound kernels: dense-layer (T = 1) squared norms, clip factors,
// fixed-order folds of partial results, zero fill, Philox Gaussian noise.
#include "dp_common.h"
#include "dp_internal.h"
#include "dp_noise.h"
#include <atomic>

namespace dpk {

// ---------------------------------------------------------------------------
// T = 1: s_i = ||A_i||^2 * ||G_i||^2 (closed form of Section 4).  One wave per
// example; each lane streams 16-byte pieces of the row, then a wave shuffle
// reduction.  Rows whose length is not a multiple of the vector width (or
// whose start is therefore unaligned) take the scalar loop.
// ---------------------------------------------------------------------------

// Sum of squares of one row by the `lpe` lanes (a power of two, 4 .. 64) that share an example; `sl` = this lane's
// place among them.  Short rows get few lanes, so that a wave takes several examples at once and every lane has a
// load of its own in flight (a whole wave on a 256-byte row would leave three quarters of its lanes idle).
__device__ __forceinline__ float group_sum(float v, int lpe) {
    for (int off = lpe >> 1; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// The 16-byte loads of four steps of the row are issued together, from clamped (valid) positions and without a branch
// between them, and added in the order of the plain loop: a guarded load per step costs a memory round trip each.
__device__ __forceinline__ float row_sumsq_f32(const float* __restrict__ row, int d, int sl, int lpe) {
    float acc = 0.f;
    if ((d & 3) == 0) {
        const float4* r4 = reinterpret_cast<const float4*>(row);
        const int n4 = d >> 2;
        for (int c0 = sl; c0 < n4; c0 += 4 * lpe) {
            float4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = r4[min(c0 + u * lpe, n4 - 1)];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (c0 + u * lpe < n4) acc += v[u].x * v[u].x + v[u].y * v[u].y + v[u].z * v[u].z + v[u].w * v[u].w;
        }
    } else {
        for (int c = sl; c < d; c += lpe) { float v = row[c]; acc += v * v; }
    }
    return group_sum(acc, lpe);
}

template <bool F16>
__device__ __forceinline__ float row_sumsq_16(const uint16_t* __restrict__ row, int d, int sl, int lpe) {
    float acc = 0.f;
    if ((d & 7) == 0) {
        const uint4* r8 = reinterpret_cast<const uint4*>(row);
        const int n8 = d >> 3;
        for (int c0 = sl; c0 < n8; c0 += 4 * lpe) {
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = r8[min(c0 + u * lpe, n8 - 1)];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (c0 + u * lpe >= n8) continue;
                const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float lo = In16<F16>::lo(w[j]), hi = In16<F16>::hi(w[j]);
                    acc += lo * lo + hi * hi;
                }
            }
        }
    } else {
        for (int c = sl; c < d; c += lpe) { float v = In16<F16>::lo(row[c]); acc += v * v; }
    }
    return group_sum(acc, lpe);
}

// Lanes per example for rows of d_max elements of `es` bytes: enough for one 16-byte piece per lane, between 4 and 64.
inline int dense_lanes_per_example(int d_max, int es) {
    const int pieces = (int)(((int64_t)d_max * es + 15) / 16);
    int lpe = 4;
    while (lpe < 64 && lpe < pieces) lpe <<= 1;
    return lpe;
}

// DT: 0 = float32, 1 = bf16, 2 = fp16.  lpe lanes per example: example = (global wave) * (64 / lpe) + lane / lpe.
template <int DT>
__global__ __launch_bounds__(kThreads) void k_sqnorm_dense(const void* __restrict__ A, const void* __restrict__ G,
                                                           int B, int d_in, int d_out, int accumulate,
                                                           float* __restrict__ sqnorm, float C, float* __restrict__ clip, int lpe) {
    const int lane = threadIdx.x & (kWave - 1), sl = lane & (lpe - 1);
    const int64_t gwave = (int64_t)blockIdx.x * (kThreads / kWave) + (threadIdx.x >> 6);
    const int64_t ex64 = gwave * (kWave / lpe) + lane / lpe;
    // lanes past the last example run on the last one (the shuffles need every lane) and write nothing
    const int ex = (int)(ex64 < B ? ex64 : B - 1);
    float sa, sg;
    if (DT != 0) {
        sa = row_sumsq_16<DT == 2>(static_cast<const uint16_t*>(A) + (size_t)ex * d_in, d_in, sl, lpe);
        sg = row_sumsq_16<DT == 2>(static_cast<const uint16_t*>(G) + (size_t)ex * d_out, d_out, sl, lpe);
    } else {
        sa = row_sumsq_f32(static_cast<const float*>(A) + (size_t)ex * d_in, d_in, sl, lpe);
        sg = row_sumsq_f32(static_cast<const float*>(G) + (size_t)ex * d_out, d_out, sl, lpe);
    }
    if (sl == 0 && ex64 < B) {
        float s = sa * sg;
        s = accumulate ? sqnorm[ex] + s : s;
        sqnorm[ex] = s;
        if (clip) clip[ex] = clip_factor_of(s, C);
    }
}

// The same for several dense layers at once: s_i (+)= sum over the layers, in the order given, of
// ||a_l,i||^2 ||g_l,i||^2  (one launch instead of one per layer: these layers are a few microseconds each).
template <int DT>
__global__ __launch_bounds__(kThreads) void k_sqnorm_dense_layers(DenseLayers t, int B, int accumulate, float* __restrict__ sqnorm,
                                                                  float C, float* __restrict__ clip, int lpe) {
    const int lane = threadIdx.x & (kWave - 1), sl = lane & (lpe - 1);
    const int64_t gwave = (int64_t)blockIdx.x * (kThreads / kWave) + (threadIdx.x >> 6);
    const int64_t ex64 = gwave * (kWave / lpe) + lane / lpe;
    const int ex = (int)(ex64 < B ? ex64 : B - 1);
    float s = 0.f;
    for (int l = 0; l < t.n_layers; ++l) {
        const int d_in = t.d_in[l], d_out = t.d_out[l];
        float sa, sg;
        if (DT != 0) {
            sa = row_sumsq_16<DT == 2>(static_cast<const uint16_t*>(t.A[l]) + (size_t)ex * d_in, d_in, sl, lpe);
            sg = row_sumsq_16<DT == 2>(static_cast<const uint16_t*>(t.G[l]) + (size_t)ex * d_out, d_out, sl, lpe);
        } else {
            sa = row_sumsq_f32(static_cast<const float*>(t.A[l]) + (size_t)ex * d_in, d_in, sl, lpe);
            sg = row_sumsq_f32(static_cast<const float*>(t.G[l]) + (size_t)ex * d_out, d_out, sl, lpe);
        }
        s += sa * sg;
    }
    if (sl == 0 && ex64 < B) {
        s = accumulate ? sqnorm[ex] + s : s;
        sqnorm[ex] = s;
        if (clip) clip[ex] = clip_factor_of(s, C);
    }
}

// The same sums for a small batch: one workgroup per example, its lane groups take the 2 * n_layers rows of the example
// (row 2 l: a_l,i; row 2 l + 1: g_l,i) side by side instead of one after the other, so that a model of a few layers
// costs one or two memory round trips and not two per layer; the row sums meet in LDS and thread 0 adds the layers'
// products in the order given.  Every row is summed by `lpe` lanes exactly as in the kernel above: same bits.
template <int DT>
__global__ __launch_bounds__(kThreads) void k_sqnorm_dense_layers_rows(DenseLayers t, int accumulate, float* __restrict__ sqnorm,
                                                                       float C, float* __restrict__ clip, int lpe) {
    __shared__ float rs[2 * kDenseBatch];
    const int ex = blockIdx.x, sl = threadIdx.x & (lpe - 1), groups = kThreads / lpe;
    for (int r = threadIdx.x / lpe; r < 2 * t.n_layers; r += groups) {
        const int l = r >> 1;
        const int d = (r & 1) ? t.d_out[l] : t.d_in[l];
        const void* base = (r & 1) ? t.G[l] : t.A[l];
        float v;
        if (DT != 0) v = row_sumsq_16<DT == 2>(static_cast<const uint16_t*>(base) + (size_t)ex * d, d, sl, lpe);
        else         v = row_sumsq_f32(static_cast<const float*>(base) + (size_t)ex * d, d, sl, lpe);
        if (sl == 0) rs[r] = v;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        float s = 0.f;
        for (int l = 0; l < t.n_layers; ++l) s += rs[2 * l] * rs[2 * l + 1];
        s = accumulate ? sqnorm[ex] + s : s;
        sqnorm[ex] = s;
        if (clip) clip[ex] = clip_factor_of(s, C);
    }
}
constexpr int kDenseRowsMaxB = 1024;     // beyond this the batch fills the chip with one wave per example

// Short rows (every row of every layer at most 512 bytes, a whole number of 16-byte pieces): a lane holds at most one
// piece of a row, so the loads of ITER examples per lane group are issued together before anything is added: rows of
// a few hundred bytes otherwise leave one or two loads in flight per wave, far from what HBM needs.
template <int DT> __device__ __forceinline__ float piece_sumsq(const uint4& v) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (DT == 0) { const float x = __uint_as_float(w[j]); acc += x * x; }
        else { const float lo = In16<DT == 2>::lo(w[j]), hi = In16<DT == 2>::hi(w[j]); acc += lo * lo + hi * hi; }
    }
    return acc;
}
template <int DT, int ITER>
__global__ __launch_bounds__(kThreads) void k_sqnorm_dense_short(DenseLayers t, int B, int accumulate, float* __restrict__ sqnorm,
                                                                 float C, float* __restrict__ clip, int lpe) {
    constexpr int ES = DT == 0 ? 4 : 2;
    const int lane = threadIdx.x & (kWave - 1), sl = lane & (lpe - 1), epw = kWave / lpe;
    const int64_t gwave = (int64_t)blockIdx.x * (kThreads / kWave) + (threadIdx.x >> 6);
    const int64_t ex0 = gwave * epw * ITER + lane / lpe;            // this lane group's examples: ex0 + k * epw
    float s[ITER];
#pragma unroll
    for (int k = 0; k < ITER; ++k) s[k] = 0.f;
    for (int l = 0; l < t.n_layers; ++l) {
        const int rba = t.d_in[l] * ES, rbg = t.d_out[l] * ES;       // row bytes
        const unsigned char* A = static_cast<const unsigned char*>(t.A[l]);
        const unsigned char* G = static_cast<const unsigned char*>(t.G[l]);
        uint4 a[ITER], g[ITER];
#pragma unroll
        for (int k = 0; k < ITER; ++k) {
            const int64_t ex = ex0 + (int64_t)k * epw;
            // unconditional loads from clamped positions, zeroed afterwards: no branch between the 2 ITER loads
            const size_t exc = (size_t)(ex < B ? ex : B - 1);
            const uint4 ra = *reinterpret_cast<const uint4*>(A + exc * rba + (sl * 16 < rba ? sl * 16 : 0));
            const uint4 rg = *reinterpret_cast<const uint4*>(G + exc * rbg + (sl * 16 < rbg ? sl * 16 : 0));
            const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
            a[k] = (ex < B && sl * 16 < rba) ? ra : zero;
            g[k] = (ex < B && sl * 16 < rbg) ? rg : zero;
        }
#pragma unroll
        for (int k = 0; k < ITER; ++k) s[k] += group_sum(piece_sumsq<DT>(a[k]), lpe) * group_sum(piece_sumsq<DT>(g[k]), lpe);
    }
#pragma unroll
    for (int k = 0; k < ITER; ++k) {
        const int64_t ex = ex0 + (int64_t)k * epw;
        if (sl == 0 && ex < B) {
            const float v = accumulate ? sqnorm[ex] + s[k] : s[k];
            sqnorm[ex] = v;
            if (clip) clip[ex] = clip_factor_of(v, C);
        }
    }
}
constexpr int kShortIter = 4;
// every row of every layer a whole number of 16-byte pieces, at most 32 of them
bool dense_rows_short(const DenseLayers& t, int es) {
    for (int l = 0; l < t.n_layers; ++l)
        for (int d : {t.d_in[l], t.d_out[l]})
            if (((int64_t)d * es) % 16 != 0 || (int64_t)d * es > 512) return false;
    return t.n_layers > 0;
}

hipError_t launch_sqnorm_dense_layers(const DenseLayers& t, int B, int dt, bool accumulate, float* sqnorm, hipStream_t st,
                                      const ClipOut* co) {
    int d_max = 1;
    for (int l = 0; l < t.n_layers; ++l) d_max = t.d_in[l] > d_max ? t.d_in[l] : d_max, d_max = t.d_out[l] > d_max ? t.d_out[l] : d_max;
    const int lpe = dense_lanes_per_example(d_max, dt == 0 ? 4 : 2);
    const float C = co ? co->C : 0.f;
    float* clip = co ? co->clip : nullptr;
    if (dense_rows_short(t, dt == 0 ? 4 : 2)) {
        const int64_t per_blk = (int64_t)(kThreads / kWave) * (kWave / lpe) * kShortIter;
        dim3 g((unsigned)((B + per_blk - 1) / per_blk));
        if (dt == 2)      k_sqnorm_dense_short<2, kShortIter><<<g, kThreads, 0, st>>>(t, B, accumulate ? 1 : 0, sqnorm, C, clip, lpe);
        else if (dt == 1) k_sqnorm_dense_short<1, kShortIter><<<g, kThreads, 0, st>>>(t, B, accumulate ? 1 : 0, sqnorm, C, clip, lpe);
        else              k_sqnorm_dense_short<0, kShortIter><<<g, kThreads, 0, st>>>(t, B, accumulate ? 1 : 0, sqnorm, C, clip, lpe);
        return hipGetLastError();
    }
    if (t.n_layers > 1 && B <= kDenseRowsMaxB) {
        if (dt == 2)      k_sqnorm_dense_layers_rows<2><<<B, kThreads, 0, st>>>(t, accumulate ? 1 : 0, sqnorm, C, clip, lpe);
        else if (dt == 1) k_sqnorm_dense_layers_rows<1><<<B, kThreads, 0, st>>>(t, accumulate ? 1 : 0, sqnorm, C, clip, lpe);
        else              k_sqnorm_dense_layers_rows<0><<<B, kThreads, 0, st>>>(t, accumulate ? 1 : 0, sqnorm, C, clip, lpe);
        return hipGetLastError();
    }
    const int64_t per_block = (int64_t)(kThreads / kWave) * (kWave / lpe);
    dim3 grid((unsigned)((B + per_block - 1) / per_block));
    if (dt == 2)      k_sqnorm_dense_layers<2><<<grid, kThreads, 0, st>>>(t, B, accumulate ? 1 : 0, sqnorm, C, clip, lpe);
    else if (dt == 1) k_sqnorm_dense_layers<1><<<grid, kThreads, 0, st>>>(t, B, accumulate ? 1 : 0, sqnorm, C, clip, lpe);
    else              k_sqnorm_dense_layers<0><<<grid, kThreads, 0, st>>>(t, B, accumulate ? 1 : 0, sqnorm, C, clip, lpe);
    return hipGetLastError();
}

hipError_t launch_sqnorm_dense(const void* A, const void* G, int B, int d_in, int d_out, int dt,
                               bool accumulate, float* sqnorm, hipStream_t st, const ClipOut* co) {
    {
        DenseLayers one;
        one.n_layers = 1; one.A[0] = A; one.G[0] = G; one.d_in[0] = d_in; one.d_out[0] = d_out;
        if (dense_rows_short(one, dt == 0 ? 4 : 2)) return launch_sqnorm_dense_layers(one, B, dt, accumulate, sqnorm, st, co);
    }
    const int lpe = dense_lanes_per_example(d_in > d_out ? d_in : d_out, dt == 0 ? 4 : 2);
    const int64_t per_block = (int64_t)(kThreads / kWave) * (kWave / lpe);
    dim3 grid((unsigned)((B + per_block - 1) / per_block));
    const float C = co ? co->C : 0.f;
    float* clip = co ? co->clip : nullptr;
    if (dt == 2)      k_sqnorm_dense<2><<<grid, kThreads, 0, st>>>(A, G, B, d_in, d_out, accumulate ? 1 : 0, sqnorm, C, clip, lpe);
    else if (dt == 1) k_sqnorm_dense<1><<<grid, kThreads, 0, st>>>(A, G, B, d_in, d_out, accumulate ? 1 : 0, sqnorm, C, clip, lpe);
    else              k_sqnorm_dense<0><<<grid, kThreads, 0, st>>>(A, G, B, d_in, d_out, accumulate ? 1 : 0, sqnorm, C, clip, lpe);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// s_i (+)= sum_j partial[i][j], j ascending: the fixed-order second stage of
// the tiled norm kernels.  One thread per example (n is tens at most).
// ---------------------------------------------------------------------------
__global__ void k_finalize_partials(const float* __restrict__ partial, int B, int n, int accumulate,
                                    float* __restrict__ sqnorm, float C, float* __restrict__ clip) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B) return;
    const float* p = partial + (size_t)i * n;
    float s = 0.f;
    for (int j0 = 0; j0 < n; j0 += 8) {             // eight loads in flight, added in order
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = p[min(j0 + u, n - 1)];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (j0 + u < n) s += v[u];
    }
    s = accumulate ? sqnorm[i] + s : s;
    sqnorm[i] = s;
    if (clip) clip[i] = clip_factor_of(s, C);
}

// The partial sums of several layers, each [B][n_l]: one wave per example; lane j adds entries j, j + 64, ... of every
// layer in the order of the queue, then the lanes' sums are added in the fixed order of wave_sum.
__global__ __launch_bounds__(64) void k_finalize_queue(FinalizeQueue q, int accumulate, float* __restrict__ sqnorm, float C,
                                                       float* __restrict__ clip) {
    const int i = blockIdx.x, lane = threadIdx.x;
    float v = 0.f;
#pragma unroll 4
    for (int l = 0; l < q.count; ++l) {
        const float* p = q.partial[l] + (size_t)i * q.n[l];
        for (int j = lane; j < q.n[l]; j += 64) v += p[j];
    }
    v = wave_sum(v);
    if (lane == 0) {
        const float s = accumulate ? sqnorm[i] + v : v;
        sqnorm[i] = s;
        if (clip) clip[i] = clip_factor_of(s, C);
    }
}

hipError_t launch_finalize_queue(const FinalizeQueue& q, int B, bool accumulate, float* sqnorm, hipStream_t st, const ClipOut* co) {
    if (q.count < 1 || q.count > FinalizeQueue::kMax || B < 1) return hipErrorInvalidValue;
    k_finalize_queue<<<(unsigned)B, 64, 0, st>>>(q, accumulate ? 1 : 0, sqnorm, co ? co->C : 0.f, co ? co->clip : nullptr);
    return hipGetLastError();
}

hipError_t launch_finalize_partials(const float* partial, int B, int n, bool accumulate, float* sqnorm, hipStream_t st,
                                    const ClipOut* co) {
    if (co && co->defer && co->defer->count < FinalizeQueue::kMax) {
        FinalizeQueue& q = *co->defer;
        q.partial[q.count] = partial; q.n[q.count] = n; ++q.count;
        return hipSuccess;
    }
    k_finalize_partials<<<(B + 63) / 64, 64, 0, st>>>(partial, B, n, accumulate ? 1 : 0, sqnorm, co ? co->C : 0.f, co ? co->clip : nullptr);
    return hipGetLastError();
}

// The same over the item lists of several layers (batched Gram launch), layer after layer.  clip != nullptr: the
// finished norms are the whole model's, and their clip factors for threshold C are written too.
// This launch sits between the two big phases of a step, so what counts is its latency: 64 examples per workgroup,
// four threads per example that take every fourth layer and request a layer's partial sums eight at a time (one
// thread walking all layers one load after the other took 6.4 us for 4 layers of 10 sums); the layers' sums meet
// in LDS and the example's first thread adds them in the order given, so the result is the same sum.
__global__ __launch_bounds__(256) void k_finalize_layers(const float* __restrict__ partial, FinalizeLayers f, int B, int accumulate,
                                                         float* __restrict__ sqnorm, float C, float* __restrict__ clip) {
    __shared__ float tl[kGramBatch][64];
    const int e = threadIdx.x & 63, k = threadIdx.x >> 6;
    const int i = blockIdx.x * 64 + e;
    if (i < B) {
        for (int l = k; l < f.n_layers; l += 4) {
            const int n = f.n[l];
            const float* p = partial + (size_t)f.first[l] + (size_t)i * n;
            float t = 0.f;
            for (int j0 = 0; j0 < n; j0 += 8) {
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = p[min(j0 + u, n - 1)];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (j0 + u < n) t += v[u];
            }
            tl[l][e] = t;
        }
    }
    __syncthreads();
    if (k != 0 || i >= B) return;
    float s = accumulate ? sqnorm[i] : 0.f;
    for (int l = 0; l < f.n_layers; ++l) s += tl[l][e];
    sqnorm[i] = s;
    if (clip) clip[i] = clip_factor_of(s, C);
}

hipError_t launch_finalize_layers(const float* partial, const FinalizeLayers& f, int B, bool accumulate, float* sqnorm, hipStream_t st,
                                  float C, float* clip) {
    k_finalize_layers<<<(B + 63) / 64, 256, 0, st>>>(partial, f, B, accumulate ? 1 : 0, sqnorm, C, clip);
    return hipGetLastError();
}

// One output array per layer; arrays may repeat (layers of one group), so they are read and written layer after
// layer by the example's one thread and are not declared restrict.
__global__ __launch_bounds__(256) void k_finalize_each(const float* __restrict__ partial, FinalizeEach f, int B) {
    // the layers' sums as in k_finalize_layers (four threads per example), then the example's first thread walks the
    // output arrays in the order given
    __shared__ float tl[kGramBatch][64];
    const int e = threadIdx.x & 63, k = threadIdx.x >> 6;
    const int i = blockIdx.x * 64 + e;
    if (i < B) {
        for (int l = k; l < f.n_layers; l += 4) {
            const int n = f.n[l];
            const float* p = partial + (size_t)f.first[l] + (size_t)i * n;
            float t = 0.f;
            for (int j0 = 0; j0 < n; j0 += 8) {
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = p[min(j0 + u, n - 1)];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (j0 + u < n) t += v[u];
            }
            tl[l][e] = t;
        }
    }
    __syncthreads();
    if (k != 0 || i >= B) return;
    for (int l = 0; l < f.n_layers; ++l) {
        const float t = tl[l][e];
        float* out = f.out[l];
        const float s = f.acc[l] ? out[i] + t : t;
        out[i] = s;
        if (f.clip[l]) f.clip[l][i] = clip_factor_of(s, f.C[l]);
    }
}

hipError_t launch_finalize_each(const float* partial, const FinalizeEach& f, int B, hipStream_t st) {
    k_finalize_each<<<(B + 63) / 64, 256, 0, st>>>(partial, f, B);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// nu_i = 1 / max(1, sqrt(s_i) / C)   (clip function of Section 3.2)
// ---------------------------------------------------------------------------
__global__ void k_clip_factors(const float* __restrict__ sqnorm, int B, float C, float* __restrict__ clip) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B) return;
    clip[i] = clip_factor_of(sqnorm[i], C);
}

hipError_t launch_clip_factors(const float* sqnorm, int B, float C, float* clip, hipStream_t st) {
    k_clip_factors<<<(B + 255) / 256, 256, 0, st>>>(sqnorm, B, C, clip);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// grad[j] (+)= sum_z ws[z][j], z ascending: second stage of the split-K GEMM.
// ---------------------------------------------------------------------------
// NOISE: n and nz.offset are multiples of 4; element j gets stddev * N(0,1)[seed, offset + j] on top.
template <bool NOISE>
__global__ __launch_bounds__(256) void k_splitk_reduce(const float* __restrict__ ws, int64_t n, int64_t slice, int splits,
                                                       int accumulate, float* __restrict__ grad, NoiseArgs nz) {
    const int64_t n4 = n >> 2;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; c < n4; c += stride) {
        float4 acc = reinterpret_cast<const float4*>(ws)[c];
        for (int z = 1; z < splits; ++z) {
            float4 v = reinterpret_cast<const float4*>(ws + (size_t)z * slice)[c];
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
        float4* o = reinterpret_cast<float4*>(grad) + c;
        if (accumulate) { float4 g = *o; acc.x += g.x; acc.y += g.y; acc.z += g.z; acc.w += g.w; }
        if (NOISE) add_noise4(acc, (nz.offset >> 2) + (uint64_t)c, nz);
        *o = acc;
    }
    // tail (n not a multiple of 4)
    for (int64_t j = (n4 << 2) + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < n; j += stride) {
        float acc = ws[j];
        for (int z = 1; z < splits; ++z) acc += ws[(size_t)z * slice + j];
        grad[j] = accumulate ? grad[j] + acc : acc;
    }
}

// Same sum for many slices of a small matrix, where one thread per output would leave most of the chip idle and
// walk its slices one load at a time: 8 threads share an output column group, thread g adds slices g, g + 8, ...
// in ascending order, and the 8 partial sums are added in the order g = 0 .. 7.  The order is fixed, so the
// result is reproducible; it differs from the one-thread order only by rounding.
template <bool NOISE>
__global__ __launch_bounds__(256) void k_splitk_reduce_wide(const float* __restrict__ ws, int64_t n4, int64_t slice, int splits,
                                                            int accumulate, float* __restrict__ grad, NoiseArgs nz) {
    __shared__ float4 part[8][32];
    const int g = threadIdx.x >> 5, cl = threadIdx.x & 31;
    const int64_t c = (int64_t)blockIdx.x * 32 + cl;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (c < n4) {
        int z = g;
        for (; z + 24 < splits; z += 32) {
            const float4 v0 = reinterpret_cast<const float4*>(ws + (size_t)z * slice)[c];
            const float4 v1 = reinterpret_cast<const float4*>(ws + (size_t)(z + 8) * slice)[c];
            const float4 v2 = reinterpret_cast<const float4*>(ws + (size_t)(z + 16) * slice)[c];
            const float4 v3 = reinterpret_cast<const float4*>(ws + (size_t)(z + 24) * slice)[c];
            acc.x += v0.x; acc.y += v0.y; acc.z += v0.z; acc.w += v0.w;
            acc.x += v1.x; acc.y += v1.y; acc.z += v1.z; acc.w += v1.w;
            acc.x += v2.x; acc.y += v2.y; acc.z += v2.z; acc.w += v2.w;
            acc.x += v3.x; acc.y += v3.y; acc.z += v3.z; acc.w += v3.w;
        }
        for (; z < splits; z += 8) {
            const float4 v = reinterpret_cast<const float4*>(ws + (size_t)z * slice)[c];
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
    }
    part[g][cl] = acc;
    __syncthreads();
    if (g == 0 && c < n4) {
#pragma unroll
        for (int k = 1; k < 8; ++k) { const float4 v = part[k][cl]; acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w; }
        float4* o = reinterpret_cast<float4*>(grad) + c;
        if (accumulate) { const float4 q = *o; acc.x += q.x; acc.y += q.y; acc.z += q.z; acc.w += q.w; }
        if (NOISE) add_noise4(acc, (nz.offset >> 2) + (uint64_t)c, nz);
        *o = acc;
    }
}

bool splitk_noise_ok(int64_t n, uint64_t offset) { return (n & 3) == 0 && (offset & 3) == 0; }

// noise: nullptr or stddev == 0 for none; otherwise splitk_noise_ok(n, noise->offset) must hold
hipError_t launch_splitk_reduce(const float* ws, int64_t n, int splits, bool accumulate, float* grad, hipStream_t st,
                                const NoiseArgs* noise) {
    // slices are spaced splitk_slice_elems(n) apart, a multiple of 4 floats, so each starts 16-byte aligned
    const int64_t n4 = n >> 2;
    const bool nz = noise != nullptr && noise->stddev != 0.0f;
    if (nz && !splitk_noise_ok(n, noise->offset)) return hipErrorInvalidValue;
    const NoiseArgs na = nz ? *noise : NoiseArgs{0.f, 0u, 0u, 0u};
    if (splits >= 16 && (n & 3) == 0 && n4 <= (int64_t)256 * 1024) {
        const unsigned grid = (unsigned)((n4 + 31) / 32);
        if (nz) k_splitk_reduce_wide<true><<<grid, 256, 0, st>>>(ws, n4, splitk_slice_elems(n), splits, accumulate ? 1 : 0, grad, na);
        else    k_splitk_reduce_wide<false><<<grid, 256, 0, st>>>(ws, n4, splitk_slice_elems(n), splits, accumulate ? 1 : 0, grad, na);
        return hipGetLastError();
    }
    int64_t blocks = (n4 + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 4096) blocks = 4096;
    if (nz) k_splitk_reduce<true><<<(unsigned)blocks, 256, 0, st>>>(ws, n, splitk_slice_elems(n), splits, accumulate ? 1 : 0, grad, na);
    else    k_splitk_reduce<false><<<(unsigned)blocks, 256, 0, st>>>(ws, n, splitk_slice_elems(n), splits, accumulate ? 1 : 0, grad, na);
    return hipGetLastError();
}

// The same fold for the layers of a joint launch in ONE launch (z ascending for every entry, as k_splitk_reduce):
// a fold per layer is a launch of a few microseconds each, which for a dozen small layers is longer than their sums
// took.  A workgroup takes 256 groups of 4 entries of one layer.
template <bool NOISE>
__global__ __launch_bounds__(256) void k_splitk_reduce_layers(FoldLayers f, int accumulate, NoiseArgs nz) {
    int l = 0;
    while (l + 1 < f.n_layers && blockIdx.x >= f.first_block[l + 1]) ++l;
    const int64_t c = (int64_t)(blockIdx.x - f.first_block[l]) * 256 + threadIdx.x;
    if (c >= (f.n[l] >> 2)) return;
    const float* ws = f.ws[l];
    const int64_t slice = f.slice[l];
    const int splits = f.splits[l];
    float4 acc = reinterpret_cast<const float4*>(ws)[c];
    int z = 1;
    for (; z + 3 < splits; z += 4) {
        const float4 v0 = reinterpret_cast<const float4*>(ws + (size_t)z * slice)[c];
        const float4 v1 = reinterpret_cast<const float4*>(ws + (size_t)(z + 1) * slice)[c];
        const float4 v2 = reinterpret_cast<const float4*>(ws + (size_t)(z + 2) * slice)[c];
        const float4 v3 = reinterpret_cast<const float4*>(ws + (size_t)(z + 3) * slice)[c];
        acc.x += v0.x; acc.y += v0.y; acc.z += v0.z; acc.w += v0.w;
        acc.x += v1.x; acc.y += v1.y; acc.z += v1.z; acc.w += v1.w;
        acc.x += v2.x; acc.y += v2.y; acc.z += v2.z; acc.w += v2.w;
        acc.x += v3.x; acc.y += v3.y; acc.z += v3.z; acc.w += v3.w;
    }
    for (; z < splits; ++z) {
        const float4 v = reinterpret_cast<const float4*>(ws + (size_t)z * slice)[c];
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    float4* o = reinterpret_cast<float4*>(f.grad[l]) + c;
    if (accumulate) { const float4 g = *o; acc.x += g.x; acc.y += g.y; acc.z += g.z; acc.w += g.w; }
    if (NOISE) add_noise4(acc, (f.noise_offset[l] >> 2) + (uint64_t)c, nz);
    *o = acc;
}

// every layer: n a multiple of 4, slices spaced splitk_slice_elems(n) apart; with noise, noise_offset a multiple of 4
hipError_t launch_splitk_reduce_layers(FoldLayers& f, bool accumulate, hipStream_t st, float stddev, uint64_t seed) {
    if (f.n_layers < 1 || f.n_layers > kJointLayers) return hipErrorInvalidValue;
    int64_t blocks = 0;
    for (int l = 0; l < f.n_layers; ++l) {
        if ((f.n[l] & 3) != 0 || (stddev != 0.0f && (f.noise_offset[l] & 3) != 0)) return hipErrorInvalidValue;
        f.first_block[l] = (unsigned)blocks;
        f.slice[l] = splitk_slice_elems(f.n[l]);
        blocks += ((f.n[l] >> 2) + 255) / 256;
        if (blocks >= (int64_t(1) << 31)) return hipErrorInvalidValue;
    }
    for (int l = f.n_layers; l < kJointLayers; ++l) { f.first_block[l] = (unsigned)blocks; f.slice[l] = 0; }
    const NoiseArgs nz{stddev, (uint32_t)seed, (uint32_t)(seed >> 32), 0};
    if (stddev != 0.0f) k_splitk_reduce_layers<true><<<(unsigned)blocks, 256, 0, st>>>(f, accumulate ? 1 : 0, nz);
    else                k_splitk_reduce_layers<false><<<(unsigned)blocks, 256, 0, st>>>(f, accumulate ? 1 : 0, nz);
    return hipGetLastError();
}

// Direct norm of few, long examples of a small layer (the first convolution of an image model: thousands of
// positions, 27 or 147 patch columns, 64 channels, 20-32 examples): one workgroup per (example, tile) is a few dozen
// workgroups that each walk thousands of rows.  The positions are cut into chunks instead (mode 2 of k_tn_bf16_rows / k_tn_f32), every
// chunk stores its share of the small matrix A_i^T G_i, and this kernel adds an example's shares entry by entry in
// the order of the chunks, squares and sums: partial[ex][block].  The layer's per-example gradients exist for a
// moment, as in the paper's own implementation, but only where they are small next to the inputs.
__global__ __launch_bounds__(kThreads) void k_direct_chunks_finish(const float* __restrict__ ws, int64_t slice, int S, int n,
                                                                   int nblk, float* __restrict__ partial) {
    __shared__ float red[4];
    const int ex = blockIdx.y;
    const float* base = ws + (size_t)ex * S * slice;
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int e = blockIdx.x * 1024 + k * kThreads + threadIdx.x;
        const int ec = e < n ? e : 0;
        float v = 0.f;
#pragma unroll 4
        for (int z = 0; z < S; ++z) v += base[(size_t)z * slice + ec];
        s += e < n ? v * v : 0.f;
    }
    s = block_sum_256(s, red);
    if (threadIdx.x == 0) partial[(size_t)ex * nblk + blockIdx.x] = s;
}

hipError_t launch_direct_chunks_finish(const float* shares, int64_t slice, int S, int n, int B, float* sums, hipStream_t st) {
    const int nblk = (n + 1023) / 1024;
    if (S < 1 || n < 1 || B < 1 || B > 65535) return hipErrorInvalidValue;
    k_direct_chunks_finish<<<dim3((unsigned)nblk, (unsigned)B), kThreads, 0, st>>>(shares, slice, S, n, nblk, sums);
    return hipGetLastError();
}

// few long examples of a small layer: about 1024 workgroups of at least 256 rows, as long as the chunks' shares are
// written and read in fewer bytes than the inputs (esize: bytes per input element; stage: rows per stage of the kernel)
void plan_direct_chunks(TnPlan& p, int B, int T, int M, int N, int esize, int stage) {
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    if (T < 1024 || (int64_t)B * tiles >= 256 || B > 4096) return;
    int64_t S = (1024 + B * tiles - 1) / (B * tiles);
    if (S > T / 256) S = T / 256;
    const int64_t kchunk = ((T + S - 1) / S + stage - 1) / stage * stage;
    S = (T + kchunk - 1) / kchunk;
    const int64_t in_bytes = (int64_t)B * T * ((int64_t)M + N) * esize;
    if (S >= 2 && B * S <= 65535 && B * S * (int64_t)M * N * 8 <= in_bytes) { p.splits = (int)S; p.kchunk = (int)kchunk; }
}

__global__ void k_fill_zero(float* __restrict__ p, int64_t n) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < n; j += stride) p[j] = 0.f;
}

// 8-bit floats -> fp16, exactly: e5m2 is the upper byte of an fp16, and e4m3's values (2^-9 .. 448) lie inside
// fp16's normal range.  NaN codes become fp16 NaNs.  16 elements per thread and step while whole 16-byte pieces
// remain (src and dst 16-byte aligned), then single elements.
template <bool E5M2> __device__ __forceinline__ uint32_t widen2_f8(uint32_t w, int pair) {
    if (E5M2) {
        const uint32_t two = pair ? (w >> 16) : (w & 0xffffu);
        return ((two & 0xffu) << 8) | ((two & 0xff00u) << 16);
    }
    const float lo = pair ? __builtin_amdgcn_cvt_f32_fp8((int)w, 2) : __builtin_amdgcn_cvt_f32_fp8((int)w, 0);
    const float hi = pair ? __builtin_amdgcn_cvt_f32_fp8((int)w, 3) : __builtin_amdgcn_cvt_f32_fp8((int)w, 1);
    return In16<true>::pack(lo, hi);
}
template <bool E5M2>
__global__ __launch_bounds__(256) void k_widen_f8(const unsigned char* __restrict__ src, uint16_t* __restrict__ dst, int64_t n) {
    const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x, stride = (int64_t)gridDim.x * 256;
    const int64_t nv = n >> 4;
    for (int64_t i = tid; i < nv; i += stride) {
        const uint4 w = reinterpret_cast<const uint4*>(src)[i];
        uint4 o0, o1;
        o0.x = widen2_f8<E5M2>(w.x, 0); o0.y = widen2_f8<E5M2>(w.x, 1); o0.z = widen2_f8<E5M2>(w.y, 0); o0.w = widen2_f8<E5M2>(w.y, 1);
        o1.x = widen2_f8<E5M2>(w.z, 0); o1.y = widen2_f8<E5M2>(w.z, 1); o1.z = widen2_f8<E5M2>(w.w, 0); o1.w = widen2_f8<E5M2>(w.w, 1);
        reinterpret_cast<uint4*>(dst)[2 * i] = o0;
        reinterpret_cast<uint4*>(dst)[2 * i + 1] = o1;
    }
    for (int64_t i = (nv << 4) + tid; i < n; i += stride) dst[i] = (uint16_t)(widen2_f8<E5M2>(src[i], 0) & 0xffffu);
}

hipError_t launch_widen_f8(const void* src, uint16_t* dst, int64_t n, bool e5m2, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n / 16 + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 8192) blocks = 8192;
    if (e5m2) k_widen_f8<true><<<(unsigned)blocks, 256, 0, st>>>(static_cast<const unsigned char*>(src), dst, n);
    else      k_widen_f8<false><<<(unsigned)blocks, 256, 0, st>>>(static_cast<const unsigned char*>(src), dst, n);
    return hipGetLastError();
}

// A line of zeros in the device image (never written), one copy per GPU: what the copy-pipeline kernels read where a
// stage reaches past an example's rows or into the padding of an image.  In host code the array's name is only a
// handle for the lookup.
static __device__ __align__(256) unsigned char zero_line[kZeroHeadFloats * sizeof(float)];

const void* device_zero_line(hipStream_t st) {
    constexpr int kDevices = 64;
    static std::atomic<void*> cache[kDevices];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kDevices) return nullptr;
    void* p = cache[dev].load(std::memory_order_acquire);
    if (p) return p;
    // the first lookup on a device may load the code object: not while the caller's stream is being captured
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cs) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
    if (cs != hipStreamCaptureStatusNone) return nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(zero_line)) != hipSuccess || !p) { (void)hipGetLastError(); return nullptr; }
    cache[dev].store(p, std::memory_order_release);
    return p;
}

hipError_t launch_fill_zero(float* p, int64_t n, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    k_fill_zero<<<(unsigned)blocks, 256, 0, st>>>(p, n);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void k_add_noise(float* __restrict__ grad, int64_t n, float stddev,
                                                   uint32_t k0, uint32_t k1, uint64_t offset) {
    const uint64_t q_first = offset >> 2;
    const uint64_t nq = ((offset + (uint64_t)n - 1) >> 2) - q_first + 1;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t qi = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; qi < nq; qi += stride) {
        const uint64_t q = q_first + qi;
        const U4 w = philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), 0u, 0u, k0, k1);
        float z[4];
        box_muller(w.x, w.y, z[0], z[1]);
        box_muller(w.z, w.w, z[2], z[3]);
        const int64_t j0 = (int64_t)(q << 2) - (int64_t)offset;   // index of slot 0 in grad (may be < 0 on the first block)
        float* p = grad + j0;
        if (j0 >= 0 && j0 + 3 < n && ((reinterpret_cast<uintptr_t>(p) & 15) == 0)) {
            float4 g = *reinterpret_cast<float4*>(p);
            g.x += stddev * z[0]; g.y += stddev * z[1]; g.z += stddev * z[2]; g.w += stddev * z[3];
            *reinterpret_cast<float4*>(p) = g;
        } else {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int64_t j = j0 + r;
                if (j >= 0 && j < n) grad[j] += stddev * z[r];
            }
        }
    }
}

hipError_t launch_add_noise(float* grad, int64_t n, float stddev, uint64_t seed, uint64_t offset, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    const uint64_t nq = ((offset + (uint64_t)n - 1) >> 2) - (offset >> 2) + 1;
    uint64_t blocks = (nq + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    k_add_noise<<<(unsigned)blocks, 256, 0, st>>>(grad, n, stddev, (uint32_t)seed, (uint32_t)(seed >> 32), offset);
    return hipGetLastError();
}

__global__ void k_philox_raw(uint32_t* __restrict__ out, int64_t nq, uint32_t k0, uint32_t k1, uint64_t first) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t qi = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; qi < nq; qi += stride) {
        const uint64_t q = first + (uint64_t)qi;
        const U4 w = philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), 0u, 0u, k0, k1);
        out[4 * qi + 0] = w.x; out[4 * qi + 1] = w.y; out[4 * qi + 2] = w.z; out[4 * qi + 3] = w.w;
    }
}

hipError_t launch_philox_raw(uint32_t* out, int64_t nq, uint64_t seed, uint64_t first, hipStream_t st) {
    if (nq <= 0) return hipSuccess;
    int64_t blocks = (nq + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    k_philox_raw<<<(unsigned)blocks, 256, 0, st>>>(out, nq, (uint32_t)seed, (uint32_t)(seed >> 32), first);
    return hipGetLastError();
}

}  // namespace dpk
