// Gram path for the per-example squared norm of a layer whose weights are shared by T positions (Sections 5.2 and
// 5.3: g_i = A_i^T G_i; its squared Frobenius norm is the sum over position pairs of (A_i A_i^T)_{ts} (G_i G_i^T)_{ts})
// for layers of few positions (T <= 64) and wide rows in a small batch: the late
// convolutions of an image model (4 x 4 or 8 x 8 positions, 2304 -> 256 or 4608 -> 512 unfolded columns, 20 to 32
// examples).  One workgroup per example walks thousands of columns alone there and leaves most of the chip idle, so
// here the COLUMNS are split: every wave takes a range of the columns of A and G (one after the other), forms its
// share of A_i A_i^T and of G_i G_i^T straight from registers, the four waves of a workgroup add their shares
// through LDS, and a second kernel adds the workgroups' shares of an example in a fixed order, multiplies the two
// T x T products entry by entry and sums.
//
// No LDS staging of the inputs: both operands of a Gram product are rows of the same matrix, so a lane's 16-byte
// piece of global memory serves the left and the right side of the MFMA alike.  16-bit inputs: the piece (8
// consecutive columns of one row) is one operand of the 32 x 32 x 16 instruction (row = lane % 32, columns
// 8 * (lane / 32) .. + 7 of a 16-column step).  float32: the piece (4 columns) feeds four 32 x 32 x 2 instructions,
// entry j of lanes 0-31 and of lanes 32-63 being the two columns of the j-th; which columns meet in an instruction
// does not matter to the sum, and both sides use the same register.  A wave issues the loads of 8 steps before the
// first MFMA, so a range of 128 (64) columns is one memory round trip.
#include "dp_common.h"
#include "dp_internal.h"

namespace dpk {

namespace {

constexpr int kColsSteps = 8;        // 16-column steps whose loads are in flight together

struct GramColsLayer {
    const void* A;
    const void* G;
    size_t part_off;     // floats: where the layer's shares start in the scratch
    int T, d_in, d_out;
    int steps_a;         // steps (16 columns of 16-bit inputs, 8 of float32) of A; the steps of G follow them
    int steps;           // of A and G together
    int W;               // workgroups per example
    int per_wave;        // steps per wave
    unsigned first_block;
};
// Several layers in one launch (the same number of 32-row blocks NB for all): a layer alone is a few hundred
// workgroups that each make one memory round trip, so the launches of a model's layers mostly wait.
struct GramColsArgs {
    GramColsLayer layer[kGramColsLayers];
    float* part;         // per layer [B][W][2][NT][16][64]: the workgroups' shares of the two products, in accumulator layout
    int n_layers;
};

// acc[tile] += X[rows of block b0] . X[rows of block b1]^T over the steps [kb, ke) of X_i[T, D]; tiles in the
// order (0,0), (0,1), (1,1) for two 32-row blocks.  Rows >= T and columns >= D read as zero (loads go to clamped,
// valid addresses).
template <int NB, bool F16>
__device__ __forceinline__ void gram_cols_run16(const uint16_t* __restrict__ X, int T, int D, int kb, int ke, int lane,
                                                f32x16 (&acc)[NB * (NB + 1) / 2]) {
    const int row = lane & 31, half = lane >> 5;
    const uint16_t* p[NB];
    bool in[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int r = b * 32 + row;
        in[b] = r < T;
        p[b] = X + (size_t)(r < T ? r : T - 1) * D;
    }
    for (int k = kb; k < ke; k += kColsSteps) {
        uint4 f[kColsSteps][NB];
#pragma unroll
        for (int u = 0; u < kColsSteps; ++u) {
            const int col = (k + u) * 16 + half * 8;
            const bool ok = (k + u) < ke && col < D;                 // D is a multiple of 8: a piece is inside or outside
            const int c = ok ? col : 0;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const uint4 v = *reinterpret_cast<const uint4*>(p[b] + c);
                const bool keep = ok && in[b];
                f[u][b] = make_uint4(keep ? v.x : 0u, keep ? v.y : 0u, keep ? v.z : 0u, keep ? v.w : 0u);
            }
        }
#pragma unroll
        for (int u = 0; u < kColsSteps; ++u) {
            if (k + u >= ke) break;                                  // uniform: the steps past the range hold zeros
            const bf16x8 f0 = __builtin_bit_cast(bf16x8, f[u][0]);
            acc[0] = In16<F16>::mfma(f0, f0, acc[0]);
            if constexpr (NB == 2) {
                const bf16x8 f1 = __builtin_bit_cast(bf16x8, f[u][1]);
                acc[1] = In16<F16>::mfma(f0, f1, acc[1]);
                acc[2] = In16<F16>::mfma(f1, f1, acc[2]);
            }
        }
    }
}

// float32: a step is 8 columns, the lane's piece columns 4 * (lane / 32) .. + 3 of it; where D is not a multiple of 4
// (rows then start at any 4-byte address) the piece is four clamped 4-byte loads
template <int NB, bool VEC>
__device__ __forceinline__ void gram_cols_run32(const float* __restrict__ X, int T, int D, int kb, int ke, int lane,
                                                f32x16 (&acc)[NB * (NB + 1) / 2]) {
    const int row = lane & 31, half = lane >> 5;
    const float* p[NB];
    bool in[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int r = b * 32 + row;
        in[b] = r < T;
        p[b] = X + (size_t)(r < T ? r : T - 1) * D;
    }
    for (int k = kb; k < ke; k += kColsSteps) {
        float4 f[kColsSteps][NB];
#pragma unroll
        for (int u = 0; u < kColsSteps; ++u) {
            const int col = (k + u) * 8 + half * 4;
            const bool ok = (k + u) < ke && col < D;
            const int c = ok ? col : 0;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const bool keep = ok && in[b];
                if (VEC) {
                    const float4 v = *reinterpret_cast<const float4*>(p[b] + c);
                    f[u][b] = make_float4(keep ? v.x : 0.f, keep ? v.y : 0.f, keep ? v.z : 0.f, keep ? v.w : 0.f);
                } else {
                    const float x = p[b][c], y = p[b][min(c + 1, D - 1)], z = p[b][min(c + 2, D - 1)], w = p[b][min(c + 3, D - 1)];
                    f[u][b] = make_float4(keep ? x : 0.f, (keep && c + 1 < D) ? y : 0.f, (keep && c + 2 < D) ? z : 0.f, (keep && c + 3 < D) ? w : 0.f);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kColsSteps; ++u) {
            if (k + u >= ke) break;                                  // uniform: the steps past the range hold zeros
            const float a0[4] = {f[u][0].x, f[u][0].y, f[u][0].z, f[u][0].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[e], a0[e], acc[0], 0, 0, 0);
            if constexpr (NB == 2) {
                const float a1[4] = {f[u][1].x, f[u][1].y, f[u][1].z, f[u][1].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[e], a1[e], acc[1], 0, 0, 0);
                    acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[e], a1[e], acc[2], 0, 0, 0);
                }
            }
        }
    }
}

// X_i of whichever type: DT 0 = float32, 1 = bf16, 2 = fp16 (the values of dp_dtype)
template <int NB, int DT>
__device__ __forceinline__ void gram_cols_run(const void* X, size_t ex, int T, int D, int kb, int ke, int lane,
                                              f32x16 (&acc)[NB * (NB + 1) / 2]) {
    if constexpr (DT == 0) {
        // (the choice sits outside the loops: a branch around every load would make each wait for the one before)
        if ((D & 3) == 0) gram_cols_run32<NB, true>(static_cast<const float*>(X) + ex * T * D, T, D, kb, ke, lane, acc);
        else              gram_cols_run32<NB, false>(static_cast<const float*>(X) + ex * T * D, T, D, kb, ke, lane, acc);
    }
    else gram_cols_run16<NB, DT == 2>(static_cast<const uint16_t*>(X) + ex * T * D, T, D, kb, ke, lane, acc);
}

// NB: 32-row blocks of positions (1: T <= 32, 2: T <= 64)
template <int NB, int DT>
__global__ __launch_bounds__(kThreads, 2) void k_gram_cols(GramColsArgs j) {
    constexpr int NT = NB * (NB + 1) / 2;            // tiles of the upper triangle
    constexpr int SHARE = 2 * NT * 16 * 64;          // floats of one wave's share (both products)
    __shared__ float red[2 * SHARE];
    int li = 0;
    while (li + 1 < j.n_layers && blockIdx.x >= j.layer[li + 1].first_block) ++li;
    const GramColsLayer& a = j.layer[li];
    const int item = blockIdx.x - a.first_block;
    const int ex = item / a.W, w = item - ex * a.W;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    f32x16 acc[2][NT];
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[q][t][r] = 0.f;

    const int k0 = (w * 4 + wave) * a.per_wave;
    const int k1 = min(k0 + a.per_wave, a.steps);
    if (k0 < a.steps_a)
        gram_cols_run<NB, DT>(a.A, (size_t)ex, a.T, a.d_in, k0, min(k1, a.steps_a), lane, acc[0]);
    if (k1 > a.steps_a)
        gram_cols_run<NB, DT>(a.G, (size_t)ex, a.T, a.d_out, max(k0, a.steps_a) - a.steps_a, k1 - a.steps_a, lane, acc[1]);

    // waves 2, 3 -> LDS; waves 0, 1 add them; wave 1 -> LDS; wave 0 adds it and stores the workgroup's share
    auto put = [&](float* slot) {
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) slot[((q * NT + t) * 16 + r) * 64 + lane] = acc[q][t][r];
    };
    auto add = [&](const float* slot) {
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[q][t][r] += slot[((q * NT + t) * 16 + r) * 64 + lane];
    };
    if (wave >= 2) put(red + (wave - 2) * SHARE);
    __syncthreads();
    if (wave < 2) add(red + wave * SHARE);
    __syncthreads();
    if (wave == 1) put(red);
    __syncthreads();
    if (wave == 0) {
        add(red);
        put(j.part + a.part_off + (size_t)item * SHARE);
    }
}

// sqnorm[ex] (+)= sum over the layers of the sum over the entries of (sum_w P_w) * (sum_w Q_w), the tile (0,1)
// counted twice (it stands for its mirror image too); one workgroup of 1024 threads per example, the shares added in
// the order of the workgroups, the layers in the order of the launch
constexpr int kFinishThreads = 1024;
template <int NB>
__global__ __launch_bounds__(kFinishThreads) void k_gram_cols_finish(GramColsArgs j, int accumulate,
                                                                       float* __restrict__ sqnorm, float C, float* __restrict__ clip) {
    constexpr int NT = NB * (NB + 1) / 2;
    constexpr int HALF = NT * 16 * 64;
    constexpr int PER = HALF / kFinishThreads;       // entries per thread: 1 or 3 (one of each tile)
    __shared__ float red[kFinishThreads / 64];
    const int ex = blockIdx.x;
    float s = 0.f;
    for (int li = 0; li < j.n_layers; ++li) {
        const int W = j.layer[li].W;
        const float* base = j.part + j.layer[li].part_off + (size_t)ex * W * 2 * HALF + threadIdx.x;
        float p[PER], q[PER];
#pragma unroll
        for (int i = 0; i < PER; ++i) { p[i] = 0.f; q[i] = 0.f; }
#pragma unroll 4
        for (int w = 0; w < W; ++w) {
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                p[i] += base[(size_t)w * 2 * HALF + i * kFinishThreads];
                q[i] += base[(size_t)w * 2 * HALF + HALF + i * kFinishThreads];
            }
        }
        float t = 0.f;
#pragma unroll
        for (int i = 0; i < PER; ++i) t += (NB == 2 && i == 1) ? 2.0f * (p[i] * q[i]) : p[i] * q[i];
        s += t;
    }
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        float v = 0.f;
#pragma unroll
        for (int i = 0; i < kFinishThreads / 64; ++i) v += red[i];
        const float t = accumulate ? sqnorm[ex] + v : v;
        sqnorm[ex] = t;
        if (clip) clip[ex] = clip_factor_of(t, C);
    }
}

}  // namespace

GramColsPlan plan_gram_cols(int B, int T, int d_in, int d_out, int dt) {
    GramColsPlan p{};
    const int piece = dt == 0 ? 4 : 8;                   // columns of a 16-byte piece; a step is two pieces
    if (B < 1 || T < 2 || T > 64 || dt < 0 || dt > 2 || d_in < 1 || d_out < 1) return p;
    if (dt != 0 && ((d_in | d_out) % piece) != 0) return p;     // 16-bit rows: whole 16-byte pieces only
    const int steps = ceil_div(d_in, 2 * piece) + ceil_div(d_out, 2 * piece);
    // fill the chip (2 workgroups on each of 256 compute units) with waves of at least kColsSteps steps
    int W = ceil_div(512, B);
    const int w_max = steps / (4 * kColsSteps);
    if (W > w_max) W = w_max;
    if (W > 64) W = 64;
    if (W < 2) return p;                                 // enough examples, or rows too narrow to split
    p.use = true;
    p.nb = T <= 32 ? 1 : 2;
    p.per_wave = ceil_div(steps, 4 * W);
    p.W = ceil_div(steps, 4 * p.per_wave);               // no workgroup without a step
    const int nt = p.nb * (p.nb + 1) / 2;
    p.ws_floats = (size_t)B * p.W * 2 * nt * 16 * 64;
    return p;
}

namespace {
template <int NB> hipError_t launch_cols_nb(const GramColsArgs& a, unsigned grid, int dt, hipStream_t st) {
    if (dt == 0)      k_gram_cols<NB, 0><<<grid, kThreads, 0, st>>>(a);
    else if (dt == 1) k_gram_cols<NB, 1><<<grid, kThreads, 0, st>>>(a);
    else              k_gram_cols<NB, 2><<<grid, kThreads, 0, st>>>(a);
    return hipGetLastError();
}
}  // namespace

// layers: every one with plan_gram_cols(...).use and the same .nb; ws: the sum of their ws_floats; dt: 0 float32, 1 bf16, 2 fp16
hipError_t launch_gram_cols_layers(const GramLayerDesc* layers, int n_layers, int B, bool accumulate, float* sqnorm, float* ws,
                                   hipStream_t st, int dt, const ClipOut* co) {
    if (n_layers < 1 || n_layers > kGramColsLayers || dt < 0 || dt > 2) return hipErrorInvalidValue;
    GramColsArgs a;
    a.part = ws; a.n_layers = n_layers;
    const int step = dt == 0 ? 8 : 16;
    int nb = 0;
    int64_t blocks = 0;
    size_t off = 0;
    for (int l = 0; l < n_layers; ++l) {
        const GramLayerDesc& y = layers[l];
        const GramColsPlan p = plan_gram_cols(B, y.T, y.d_in, y.d_out, dt);
        if (!p.use || (l > 0 && p.nb != nb)) return hipErrorInvalidValue;
        nb = p.nb;
        GramColsLayer& g = a.layer[l];
        g.A = y.A; g.G = y.G;
        g.part_off = off;
        g.T = y.T; g.d_in = y.d_in; g.d_out = y.d_out;
        g.steps_a = ceil_div(y.d_in, step); g.steps = g.steps_a + ceil_div(y.d_out, step);
        g.W = p.W; g.per_wave = p.per_wave;
        g.first_block = (unsigned)blocks;
        blocks += (int64_t)B * p.W;
        off += p.ws_floats;
    }
    for (int l = n_layers; l < kGramColsLayers; ++l) a.layer[l] = a.layer[0];
    if (blocks >= (int64_t(1) << 31)) return hipErrorInvalidValue;
    const hipError_t e = nb == 1 ? launch_cols_nb<1>(a, (unsigned)blocks, dt, st) : launch_cols_nb<2>(a, (unsigned)blocks, dt, st);
    if (e != hipSuccess) return e;
    const float C = co ? co->C : 0.f;
    float* clip = co ? co->clip : nullptr;
    if (nb == 1) k_gram_cols_finish<1><<<B, kFinishThreads, 0, st>>>(a, accumulate ? 1 : 0, sqnorm, C, clip);
    else         k_gram_cols_finish<2><<<B, kFinishThreads, 0, st>>>(a, accumulate ? 1 : 0, sqnorm, C, clip);
    return hipGetLastError();
}

hipError_t launch_gram_cols(const GramColsPlan& p, const void* A, const void* G, int B, int T, int d_in, int d_out,
                            bool accumulate, float* sqnorm, float* ws, hipStream_t st, int dt, const ClipOut* co) {
    if (!p.use) return hipErrorInvalidValue;
    GramLayerDesc y{A, G, T, d_in, d_out, nullptr, nullptr};
    return launch_gram_cols_layers(&y, 1, B, accumulate, sqnorm, ws, st, dt, co);
}

}  // namespace dpk
