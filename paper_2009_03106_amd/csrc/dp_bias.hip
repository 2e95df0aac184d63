// Parameters whose per-example gradients are column sums, small enough ([B, d] floats) to
// materialise: bias vectors, u_i = sum_t G_i[t, :] (dL/db = dL/dz for a fully-connected
// layer, Section 5.1; summed over the positions that share the bias, Section 5.3), and
// LayerNorm scale / shift, sum_t G_i[t, :] (*) Hbar_i[t, :] and sum_t G_i[t, :] (Section 5.5,
// Algorithm 5); their squared norms; and the clipped sum  sum_i nu_i u_i.
// All of it is bandwidth-bound; every sum runs in a fixed order (no atomics).
#include "dp_common.h"
#include "dp_internal.h"
#include <type_traits>

namespace dpk {

namespace {

// One workgroup per (example, chunk of columns).  The 256 threads form rg row groups x ct column
// threads (ct = 1 << ctl); a thread owns VEC consecutive columns (one 16-byte load per row) and
// adds rows rgid, rgid + rg, ... in ascending order; the rg partial sums are then added in the
// order 0 .. rg-1.  Needs D % VEC == 0 (with the 16-byte aligned base every load is aligned).
// PROD: a second input Hb of the same shape; u2 gets the plain column sums and u the sums of G (*) Hb.
// DT (type of G), DTH (type of Hb): 0 = float32, 1 = bf16, 2 = fp16, 3 = e4m3, 4 = e5m2; both of the same width
template <int DT> struct ElemBytes { static constexpr int value = DT == 0 ? 4 : (DT >= 3 ? 1 : 2); };
// one 8-bit float -> float32 (e5m2 is the upper byte of an fp16)
template <int DT> __device__ __forceinline__ float f8_byte(uint32_t word, int which) {
    if (DT == 4) return (float)__builtin_bit_cast(_Float16, (uint16_t)(((word >> (8 * which)) & 0xffu) << 8));
    return which == 0 ? __builtin_amdgcn_cvt_f32_fp8((int)word, 0) : which == 1 ? __builtin_amdgcn_cvt_f32_fp8((int)word, 1)
         : which == 2 ? __builtin_amdgcn_cvt_f32_fp8((int)word, 2) : __builtin_amdgcn_cvt_f32_fp8((int)word, 3);
}
template <int DT, bool PROD, int DTH = DT>
__global__ __launch_bounds__(kThreads) void k_bias_rows(const void* __restrict__ G, const void* __restrict__ Hb, int T, int D, int ctl,
                                                        float* __restrict__ u, float* __restrict__ u2) {
    constexpr int ES = ElemBytes<DT>::value;          // bytes per element
    static_assert(ElemBytes<DTH>::value == ES, "G and Hb of one width");
    constexpr int VEC = 16 / ES;
    __shared__ float part[kThreads][PROD ? 2 * VEC : VEC];
    const int tid = threadIdx.x, ct = 1 << ctl, rg = kThreads >> ctl;
    const int ctid = tid & (ct - 1), rgid = tid >> ctl;
    const int ex = blockIdx.y;
    const int col0 = (blockIdx.x * ct + ctid) * VEC;
    float acc[VEC], acc2[VEC];                        // acc2 (PROD only): plain sums
#pragma unroll
    for (int v = 0; v < VEC; ++v) { acc[v] = 0.f; acc2[v] = 0.f; }
    auto widen = [&](const uint4& w, float (&x)[VEC], auto tag) {
        constexpr int E = decltype(tag)::value;
        const uint32_t d[4] = {w.x, w.y, w.z, w.w};
        if constexpr (E >= 3) {
            // two conversions per instruction (v_cvt_pk_f32_fp8 / _bf8: the low or the high 16 bits of the word)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f32x2 lo, hi;
                if constexpr (E == 3) { lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)d[j], false); hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)d[j], true); }
                else                  { lo = __builtin_amdgcn_cvt_pk_f32_bf8((int)d[j], false); hi = __builtin_amdgcn_cvt_pk_f32_bf8((int)d[j], true); }
                x[4 * j] = lo[0]; x[4 * j + 1] = lo[1]; x[4 * j + 2] = hi[0]; x[4 * j + 3] = hi[1];
            }
        } else if constexpr (E != 0) {
#pragma unroll
            for (int j = 0; j < 4; ++j) { x[2 * j] = In16<E == 2>::lo(d[j]); x[2 * j + 1] = In16<E == 2>::hi(d[j]); }
        } else {
            x[0] = __uint_as_float(w.x); x[1] = __uint_as_float(w.y); x[2] = __uint_as_float(w.z); x[3] = __uint_as_float(w.w);
        }
    };
    auto add = [&](const uint4& w) {
        float x[VEC];
        widen(w, x, std::integral_constant<int, DT>{});
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] += x[v];
    };
    auto add_prod = [&](const uint4& w, const uint4& h) {
        float x[VEC], y[VEC];
        widen(w, x, std::integral_constant<int, DT>{});
        widen(h, y, std::integral_constant<int, DTH>{});
#pragma unroll
        for (int v = 0; v < VEC; ++v) { acc[v] += x[v] * y[v]; acc2[v] += x[v]; }
    };
    if (col0 < D) {
        const size_t row_bytes = (size_t)D * ES;
        const unsigned char* p = static_cast<const unsigned char*>(G) + ((size_t)ex * T) * row_bytes + (size_t)col0 * ES;
        int t = rgid;
        if (PROD) {
            const unsigned char* q = static_cast<const unsigned char*>(Hb) + ((size_t)ex * T) * row_bytes + (size_t)col0 * ES;
            for (; t + 3 * rg < T; t += 4 * rg) {      // eight loads in flight, added in row order
                uint4 w[4], h[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    w[k] = *reinterpret_cast<const uint4*>(p + (size_t)(t + k * rg) * row_bytes);
                    h[k] = *reinterpret_cast<const uint4*>(q + (size_t)(t + k * rg) * row_bytes);
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) add_prod(w[k], h[k]);
            }
            for (; t < T; t += rg)
                add_prod(*reinterpret_cast<const uint4*>(p + (size_t)t * row_bytes), *reinterpret_cast<const uint4*>(q + (size_t)t * row_bytes));
        } else {
            for (; t + 7 * rg < T; t += 8 * rg) {      // eight loads in flight, added in row order
                uint4 w[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) w[k] = *reinterpret_cast<const uint4*>(p + (size_t)(t + k * rg) * row_bytes);
#pragma unroll
                for (int k = 0; k < 8; ++k) add(w[k]);
            }
            for (; t < T; t += rg) add(*reinterpret_cast<const uint4*>(p + (size_t)t * row_bytes));
        }
    }
#pragma unroll
    for (int v = 0; v < VEC; ++v) { part[tid][v] = acc[v]; if (PROD) part[tid][VEC + v] = acc2[v]; }
    __syncthreads();
    if (rgid == 0 && col0 < D) {
        for (int r = 1; r < rg; ++r)
#pragma unroll
            for (int v = 0; v < VEC; ++v) { acc[v] += part[r * ct + ctid][v]; if (PROD) acc2[v] += part[r * ct + ctid][VEC + v]; }
        float* o = u + (size_t)ex * D + col0;
#pragma unroll
        for (int v = 0; v < VEC; ++v) o[v] = acc[v];
        if (PROD) {
            float* o2 = u2 + (size_t)ex * D + col0;
#pragma unroll
            for (int v = 0; v < VEC; ++v) o2[v] = acc2[v];
        }
    }
}

// Any D: one thread per column, rows in ascending order.
template <int DT> __device__ __forceinline__ float load_elem(const void* p, size_t k) {
    if (DT >= 3) return f8_byte<DT>(static_cast<const unsigned char*>(p)[k], 0);
    if (DT != 0) return In16<DT == 2>::lo(static_cast<const uint16_t*>(p)[k]);
    return static_cast<const float*>(p)[k];
}
template <int DT, bool PROD, int DTH = DT>
__global__ __launch_bounds__(kThreads) void k_bias_rows_scalar(const void* __restrict__ G, const void* __restrict__ Hb, int T, int D,
                                                               float* __restrict__ u, float* __restrict__ u2) {
    const int q = blockIdx.x * kThreads + threadIdx.x;
    const int ex = blockIdx.y;
    if (q >= D) return;
    float acc = 0.f, acc2 = 0.f;
    const size_t base = (size_t)ex * T * D + q;
    for (int t = 0; t < T; ++t) {
        const size_t k = base + (size_t)t * D;
        const float g = load_elem<DT>(G, k);
        if (PROD) {
            const float h = load_elem<DTH>(Hb, k);
            acc += g * h; acc2 += g;
        } else {
            acc += g;
        }
    }
    u[(size_t)ex * D + q] = acc;
    if (PROD) u2[(size_t)ex * D + q] = acc2;
}

// s_i (+)= sum_q u[i, q]^2 (+ sum_q u2[i, q]^2 when u2 is given: LayerNorm's scale and shift rows in one launch):
// one wave per example, four per workgroup; lane l adds the 16-byte pieces l, l + 64, ... of the row (four loads in
// flight), then a shuffle tree.  The order of the additions is fixed.
__device__ __forceinline__ float row_sq(const float* __restrict__ p, int D, int lane) {
    float acc = 0.f;
    if ((D & 3) == 0 && (reinterpret_cast<uintptr_t>(p) & 15) == 0) {
        const float4* p4 = reinterpret_cast<const float4*>(p);
        const int n4 = D >> 2;
        int q = lane;
        for (; q + 3 * kWave < n4; q += 4 * kWave) {
            const float4 a = p4[q], b = p4[q + kWave], c = p4[q + 2 * kWave], d = p4[q + 3 * kWave];
            acc += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
            acc += b.x * b.x + b.y * b.y + b.z * b.z + b.w * b.w;
            acc += c.x * c.x + c.y * c.y + c.z * c.z + c.w * c.w;
            acc += d.x * d.x + d.y * d.y + d.z * d.z + d.w * d.w;
        }
        for (; q < n4; q += kWave) { const float4 a = p4[q]; acc += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w; }
    } else {
        for (int q = lane; q < D; q += kWave) { const float v = p[q]; acc += v * v; }
    }
    return wave_sum(acc);
}
__global__ __launch_bounds__(kThreads) void k_rows_sqnorm(const float* __restrict__ u, const float* __restrict__ u2, int B, int D,
                                                          int accumulate, float* __restrict__ sqnorm) {
    const int lane = threadIdx.x & (kWave - 1);
    const int ex = blockIdx.x * (kThreads / kWave) + (threadIdx.x >> 6);
    if (ex >= B) return;
    const float a = row_sq(u + (size_t)ex * D, D, lane);
    const float b = u2 ? row_sq(u2 + (size_t)ex * D, D, lane) : 0.f;
    if (lane == 0) {
        float s = accumulate ? sqnorm[ex] + a : a;
        if (u2) s += b;
        sqnorm[ex] = s;
    }
}

// grad_b[q] (+)= sum_i nu_i u[i, q].  A workgroup owns 32 columns; its NG row groups add examples g, g + NG, ... in
// ascending order (four loads in flight each), and the NG partial sums are added in the order g = 0 .. NG - 1: a
// fixed order, so the result is reproducible.  (One thread per column walking all B examples one dependent load
// after the other took 17 us for 256 examples.)  NG = 8 for small batches; 32 (1024 threads per workgroup) from
// 2048 examples on: the grid is only d_out / 32 workgroups, so a long batch needs the loads of many threads in
// flight per workgroup (B = 65536, d_out = 512: 0.70 ms with 8 groups).
template <int NG>
__global__ __launch_bounds__(NG * 32) void k_clipped_bias(const float* __restrict__ u, const float* __restrict__ clip, int B, int D,
                                                          int accumulate, float* __restrict__ grad_b) {
    __shared__ float part[NG][32];
    const int g = threadIdx.x >> 5, cl = threadIdx.x & 31;
    const int q = blockIdx.x * 32 + cl;
    float acc = 0.f;
    if (q < D) {
        int i = g;
        for (; i + 3 * NG < B; i += 4 * NG) {
            const float v0 = u[(size_t)i * D + q], v1 = u[(size_t)(i + NG) * D + q];
            const float v2 = u[(size_t)(i + 2 * NG) * D + q], v3 = u[(size_t)(i + 3 * NG) * D + q];
            acc += clip[i] * v0; acc += clip[i + NG] * v1; acc += clip[i + 2 * NG] * v2; acc += clip[i + 3 * NG] * v3;
        }
        for (; i < B; i += NG) acc += clip[i] * u[(size_t)i * D + q];
    }
    part[g][cl] = acc;
    __syncthreads();
    if (g == 0 && q < D) {
#pragma unroll
        for (int k = 1; k < NG; ++k) acc += part[k][cl];
        grad_b[q] = accumulate ? grad_b[q] + acc : acc;
    }
}

template <int DT, int DTH = DT> void launch_bias_rows_dt(const void* G, const void* Hb, int B, int T, int D, float* u, float* u2, hipStream_t st) {
    constexpr int vec = 16 / ElemBytes<DT>::value;
    const bool prod = Hb != nullptr;
    if (D % vec == 0) {
        const int nvec = D / vec;
        int ctl = 0;
        while (ctl < 6 && (1 << ctl) < nvec) ++ctl;      // column threads: next power of two, at most 64 ...
        // ... but narrower column chunks (down to 16 threads = 256-byte row pieces) while the grid is too small
        // to keep enough loads in flight for HBM
        while (ctl > 4 && (int64_t)((nvec + (1 << ctl) - 1) >> ctl) * B < 1024) --ctl;
        const dim3 grid((unsigned)((nvec + (1 << ctl) - 1) >> ctl), (unsigned)B);
        if (prod) k_bias_rows<DT, true, DTH><<<grid, kThreads, 0, st>>>(G, Hb, T, D, ctl, u, u2);
        else      k_bias_rows<DT, false><<<grid, kThreads, 0, st>>>(G, Hb, T, D, ctl, u, u2);
    } else {
        const dim3 grid((unsigned)((D + kThreads - 1) / kThreads), (unsigned)B);
        if (prod) k_bias_rows_scalar<DT, true, DTH><<<grid, kThreads, 0, st>>>(G, Hb, T, D, u, u2);
        else      k_bias_rows_scalar<DT, false><<<grid, kThreads, 0, st>>>(G, Hb, T, D, u, u2);
    }
}

}  // namespace

// Hb == nullptr: u = column sums of G.  Otherwise u = column sums of G (*) Hb and u2 = column sums of G.
// dt: type of G and Hb as above; 5: G e5m2 with Hb e4m3.
hipError_t launch_bias_rows(const void* G, const void* Hb, int B, int T, int D, int dt, float* u, float* u2, hipStream_t st) {
    // the examples are the grid's y dimension (at most 65535): larger batches go in several launches
    const size_t es = dt == 0 ? 4 : (dt >= 3 ? 1 : 2);
    for (int b0 = 0; b0 < B; b0 += 65535) {
        const int nb = (B - b0 < 65535) ? (B - b0) : 65535;
        const size_t in_off = (size_t)b0 * T * D * es, out_off = (size_t)b0 * D;
        const void* g = static_cast<const unsigned char*>(G) + in_off;
        const void* h = Hb ? static_cast<const unsigned char*>(Hb) + in_off : nullptr;
        float* pu = u + out_off;
        float* pu2 = u2 ? u2 + out_off : nullptr;
        if (dt == 5)      launch_bias_rows_dt<4, 3>(g, h, nb, T, D, pu, pu2, st);
        else if (dt == 4) launch_bias_rows_dt<4>(g, h, nb, T, D, pu, pu2, st);
        else if (dt == 3) launch_bias_rows_dt<3>(g, h, nb, T, D, pu, pu2, st);
        else if (dt == 2) launch_bias_rows_dt<2>(g, h, nb, T, D, pu, pu2, st);
        else if (dt == 1) launch_bias_rows_dt<1>(g, h, nb, T, D, pu, pu2, st);
        else              launch_bias_rows_dt<0>(g, h, nb, T, D, pu, pu2, st);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Bias rows from the per-row-tile column sums that the Gram kernel leaves behind:
//     u[i, q] = sum_tt upart[i, tt, q]  (tt ascending),   s_i (+)= sum_q u[i, q]^2.
// One workgroup of 1024 threads per example; thread t takes columns t, t + 1024, ... (the loads of a column's
// tiles are independent, four in flight); the squares are added per thread in column order, then over each wave
// and over the 16 waves in a fixed order.
constexpr int kFoldThreads = 1024;
__global__ __launch_bounds__(kFoldThreads) void k_bias_fold(const float* __restrict__ upart, int nt, int D, int accumulate,
                                                            float* __restrict__ u, float* __restrict__ sqnorm) {
    __shared__ float red[kFoldThreads / kWave];
    const int ex = blockIdx.x, tid = threadIdx.x;
    const float* p = upart + (size_t)ex * nt * D;
    float acc = 0.f;
    for (int q = tid; q < D; q += kFoldThreads) {
        float v = 0.f;
        int tt = 0;
        for (; tt + 3 < nt; tt += 4) {
            const float v0 = p[(size_t)tt * D + q], v1 = p[(size_t)(tt + 1) * D + q];
            const float v2 = p[(size_t)(tt + 2) * D + q], v3 = p[(size_t)(tt + 3) * D + q];
            v += v0; v += v1; v += v2; v += v3;
        }
        for (; tt < nt; ++tt) v += p[(size_t)tt * D + q];
        u[(size_t)ex * D + q] = v;
        acc += v * v;
    }
    acc = wave_sum(acc);
    if ((tid & (kWave - 1)) == 0) red[tid >> 6] = acc;
    __syncthreads();
    if (tid == 0) {
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < kFoldThreads / kWave; ++w) t += red[w];
        sqnorm[ex] = accumulate ? sqnorm[ex] + t : t;
    }
}

hipError_t launch_bias_fold(const float* upart, int B, int nt, int D, bool accumulate, float* u, float* sqnorm, hipStream_t st) {
    k_bias_fold<<<(unsigned)B, kFoldThreads, 0, st>>>(upart, nt, D, accumulate ? 1 : 0, u, sqnorm);
    return hipGetLastError();
}

hipError_t launch_rows_sqnorm(const float* u, int B, int D, bool accumulate, float* sqnorm, hipStream_t st, const float* u2) {
    const int per_block = kThreads / kWave;
    k_rows_sqnorm<<<(unsigned)((B + per_block - 1) / per_block), kThreads, 0, st>>>(u, u2, B, D, accumulate ? 1 : 0, sqnorm);
    return hipGetLastError();
}

hipError_t launch_clipped_bias(const float* u, const float* clip, int B, int D, bool accumulate, float* grad_b, hipStream_t st) {
    if (B >= 2048) k_clipped_bias<32><<<(unsigned)((D + 31) / 32), 1024, 0, st>>>(u, clip, B, D, accumulate ? 1 : 0, grad_b);
    else           k_clipped_bias<8><<<(unsigned)((D + 31) / 32), kThreads, 0, st>>>(u, clip, B, D, accumulate ? 1 : 0, grad_b);
    return hipGetLastError();
}

}  // namespace dpk
