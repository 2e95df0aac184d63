// Bias parameters: per-example bias gradients u_i = sum_t G_i[t, :] (dL/db = dL/dz for a
// fully-connected layer, Section 5.1; summed over the positions that share the bias,
// Section 5.3), their squared norms, and the clipped sum  sum_i nu_i u_i.
// All three are bandwidth-bound; every sum runs in a fixed order (no atomics).
#include "dp_common.h"
#include "dp_internal.h"

namespace dpk {

namespace {

// One workgroup per (example, chunk of columns).  The 256 threads form rg row groups x ct column
// threads (ct = 1 << ctl); a thread owns VEC consecutive columns (one 16-byte load per row) and
// adds rows rgid, rgid + rg, ... in ascending order; the rg partial sums are then added in the
// order 0 .. rg-1.  Needs D % VEC == 0 (with the 16-byte aligned base every load is aligned).
template <bool BF16>
__global__ __launch_bounds__(kThreads) void k_bias_rows(const void* __restrict__ G, int T, int D, int ctl,
                                                        float* __restrict__ u) {
    constexpr int VEC = BF16 ? 8 : 4;
    __shared__ float part[kThreads][VEC];
    const int tid = threadIdx.x, ct = 1 << ctl, rg = kThreads >> ctl;
    const int ctid = tid & (ct - 1), rgid = tid >> ctl;
    const int ex = blockIdx.y;
    const int col0 = (blockIdx.x * ct + ctid) * VEC;
    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
    auto add = [&](const uint4& w) {
        if (BF16) {
            const uint32_t d[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) { acc[2 * j] += bf16_lo(d[j]); acc[2 * j + 1] += bf16_hi(d[j]); }
        } else {
            acc[0] += __uint_as_float(w.x); acc[1] += __uint_as_float(w.y);
            acc[2] += __uint_as_float(w.z); acc[3] += __uint_as_float(w.w);
        }
    };
    if (col0 < D) {
        const size_t row_bytes = (size_t)D * (BF16 ? 2 : 4);
        const unsigned char* p = static_cast<const unsigned char*>(G) + ((size_t)ex * T) * row_bytes + (size_t)col0 * (BF16 ? 2 : 4);
        int t = rgid;
        for (; t + 7 * rg < T; t += 8 * rg) {          // eight loads in flight, added in row order
            uint4 w[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) w[k] = *reinterpret_cast<const uint4*>(p + (size_t)(t + k * rg) * row_bytes);
#pragma unroll
            for (int k = 0; k < 8; ++k) add(w[k]);
        }
        for (; t < T; t += rg) add(*reinterpret_cast<const uint4*>(p + (size_t)t * row_bytes));
    }
#pragma unroll
    for (int v = 0; v < VEC; ++v) part[tid][v] = acc[v];
    __syncthreads();
    if (rgid == 0 && col0 < D) {
        for (int r = 1; r < rg; ++r)
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[v] += part[r * ct + ctid][v];
        float* o = u + (size_t)ex * D + col0;
#pragma unroll
        for (int v = 0; v < VEC; ++v) o[v] = acc[v];
    }
}

// Any D: one thread per column, rows in ascending order.
template <bool BF16>
__global__ __launch_bounds__(kThreads) void k_bias_rows_scalar(const void* __restrict__ G, int T, int D, float* __restrict__ u) {
    const int q = blockIdx.x * kThreads + threadIdx.x;
    const int ex = blockIdx.y;
    if (q >= D) return;
    float acc = 0.f;
    if (BF16) {
        const uint16_t* p = static_cast<const uint16_t*>(G) + (size_t)ex * T * D + q;
        for (int t = 0; t < T; ++t) acc += bf16_to_f32(p[(size_t)t * D]);
    } else {
        const float* p = static_cast<const float*>(G) + (size_t)ex * T * D + q;
        for (int t = 0; t < T; ++t) acc += p[(size_t)t * D];
    }
    u[(size_t)ex * D + q] = acc;
}

// s_i (+)= sum_q u[i, q]^2: one wave per example, lane l adds columns l, l + 64, ..., then a shuffle tree.
__global__ __launch_bounds__(kWave) void k_rows_sqnorm(const float* __restrict__ u, int D, int accumulate, float* __restrict__ sqnorm) {
    const int ex = blockIdx.x, lane = threadIdx.x;
    const float* p = u + (size_t)ex * D;
    float acc = 0.f;
    for (int q = lane; q < D; q += kWave) { const float v = p[q]; acc += v * v; }
    acc = wave_sum(acc);
    if (lane == 0) sqnorm[ex] = accumulate ? sqnorm[ex] + acc : acc;
}

// grad_b[q] (+)= sum_i nu_i u[i, q], i ascending; one thread per column.
__global__ __launch_bounds__(kThreads) void k_clipped_bias(const float* __restrict__ u, const float* __restrict__ clip, int B, int D,
                                                           int accumulate, float* __restrict__ grad_b) {
    const int q = blockIdx.x * kThreads + threadIdx.x;
    if (q >= D) return;
    float acc = 0.f;
    int i = 0;
    for (; i + 3 < B; i += 4) {
        const float v0 = u[(size_t)i * D + q], v1 = u[(size_t)(i + 1) * D + q];
        const float v2 = u[(size_t)(i + 2) * D + q], v3 = u[(size_t)(i + 3) * D + q];
        acc += clip[i] * v0; acc += clip[i + 1] * v1; acc += clip[i + 2] * v2; acc += clip[i + 3] * v3;
    }
    for (; i < B; ++i) acc += clip[i] * u[(size_t)i * D + q];
    grad_b[q] = accumulate ? grad_b[q] + acc : acc;
}

}  // namespace

hipError_t launch_bias_rows(const void* G, int B, int T, int D, bool bf16, float* u, hipStream_t st) {
    const int vec = bf16 ? 8 : 4;
    if (B > 65535) return hipErrorInvalidValue;          // grid.y
    if (D % vec == 0) {
        const int nvec = D / vec;
        int ctl = 0;
        while (ctl < 6 && (1 << ctl) < nvec) ++ctl;      // column threads: next power of two, at most 64 ...
        // ... but narrower column chunks (down to 16 threads = 256-byte row pieces) while the grid is too small
        // to keep enough loads in flight for HBM
        while (ctl > 4 && (int64_t)((nvec + (1 << ctl) - 1) >> ctl) * B < 1024) --ctl;
        const dim3 grid((unsigned)((nvec + (1 << ctl) - 1) >> ctl), (unsigned)B);
        if (bf16) k_bias_rows<true><<<grid, kThreads, 0, st>>>(G, T, D, ctl, u);
        else      k_bias_rows<false><<<grid, kThreads, 0, st>>>(G, T, D, ctl, u);
    } else {
        const dim3 grid((unsigned)((D + kThreads - 1) / kThreads), (unsigned)B);
        if (bf16) k_bias_rows_scalar<true><<<grid, kThreads, 0, st>>>(G, T, D, u);
        else      k_bias_rows_scalar<false><<<grid, kThreads, 0, st>>>(G, T, D, u);
    }
    return hipGetLastError();
}

hipError_t launch_rows_sqnorm(const float* u, int B, int D, bool accumulate, float* sqnorm, hipStream_t st) {
    k_rows_sqnorm<<<(unsigned)B, kWave, 0, st>>>(u, D, accumulate ? 1 : 0, sqnorm);
    return hipGetLastError();
}

hipError_t launch_clipped_bias(const float* u, const float* clip, int B, int D, bool accumulate, float* grad_b, hipStream_t st) {
    k_clipped_bias<<<(unsigned)((D + kThreads - 1) / kThreads), kThreads, 0, st>>>(u, clip, B, D, accumulate ? 1 : 0, grad_b);
    return hipGetLastError();
}

}  // namespace dpk
