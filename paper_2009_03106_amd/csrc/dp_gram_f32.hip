// Gram path of the per-example squared norm for float32 inputs:
//     ||A_i^T G_i||_F^2 = sum_{t,s} (A_i A_i^T)_{ts} (G_i G_i^T)_{ts}.
// Same decomposition as the 16-bit Gram kernels: one workgroup per example and
// pair of row tiles (t-tile <= s-tile, 64 rows each), the tile of A_i A_i^T
// (contraction over d_in) and then the tile of G_i G_i^T (contraction over
// d_out) kept in MFMA accumulators of identical layout, multiplied lane by lane
// and reduced; off-diagonal pairs count twice.  The matrix instruction is the
// fp32 one (v_mfma_f32_32x32x2_f32: one k per lane and instruction, lanes 0-31
// take k, lanes 32-63 take k + 1), so a lane reads its operands straight from the
// row-major LDS tiles; the rows are padded to 33 floats, which puts the 32 rows
// that one read touches into 32 different banks.
#include "dp_common.h"
#include "dp_internal.h"

namespace dpk {

namespace {

constexpr int FT = 64;        // rows of T per tile
constexpr int FK = 32;        // contraction elements per LDS stage
constexpr int FP = FK + 1;    // padded row length in LDS

struct GramArgsF {
    const float* A;
    const float* G;
    float* partial;      // [B][npairs]
    int T, d_in, d_out;
    int nt, npairs;
};

// One Gram product tile: acc += X[t-tile rows] . X[s-tile rows]^T over the D columns of X_i[T, D].
// VEC: D % 4 == 0 (every 16-byte piece lies inside a row or outside it).
template <bool VEC>
__device__ __forceinline__ void gram_product_f32(const float* __restrict__ Xi, int T, int D, int t0, int s0, bool diag,
                                                 float (*sT)[FP], float (*sS)[FP], f32x16& acc) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = lane & 31, lhalf = lane >> 5;
    // global -> LDS: a thread moves two 4-column pieces of either tile per stage (rows lr and lr + 32)
    const int lr = tid >> 3, lc = (tid & 7) * 4;
    float xt[2][4], xs[2][4];
    bool in_t[2], in_s[2];
    // loads are issued from clamped (valid) addresses and zeroed when they are committed, one stage of MFMAs
    // later, so that nothing waits for them in between
    auto fetch = [&](int k0) {
#pragma unroll
        for (int v = 0; v < 2; ++v) {
            const int rt = t0 + lr + 32 * v, rs = s0 + lr + 32 * v;
            in_t[v] = rt < T; in_s[v] = rs < T;
            const float* pt = Xi + (size_t)(in_t[v] ? rt : T - 1) * D;
            const float* ps = Xi + (size_t)(in_s[v] ? rs : T - 1) * D;
            if (VEC) {
                const int c = (k0 + lc < D) ? k0 + lc : 0;
                const float4 q = *reinterpret_cast<const float4*>(pt + c);
                xt[v][0] = q.x; xt[v][1] = q.y; xt[v][2] = q.z; xt[v][3] = q.w;
                if (!diag) {
                    const float4 r = *reinterpret_cast<const float4*>(ps + c);
                    xs[v][0] = r.x; xs[v][1] = r.y; xs[v][2] = r.z; xs[v][3] = r.w;
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int c = (k0 + lc + j < D) ? k0 + lc + j : 0;
                    xt[v][j] = pt[c];
                    if (!diag) xs[v][j] = ps[c];
                }
            }
        }
    };
    auto commit = [&](int k0) {
#pragma unroll
        for (int v = 0; v < 2; ++v)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool col_ok = k0 + lc + j < D;
                sT[lr + 32 * v][lc + j] = (in_t[v] && col_ok) ? xt[v][j] : 0.f;
                if (!diag) sS[lr + 32 * v][lc + j] = (in_s[v] && col_ok) ? xs[v][j] : 0.f;
            }
    };
    float (*sB)[FP] = diag ? sT : sS;
    if (D > 0) fetch(0);
    for (int k0 = 0; k0 < D; k0 += FK) {
        commit(k0);
        __syncthreads();
        if (k0 + FK < D) fetch(k0 + FK);
        // the operands of 8 MFMAs are read together, so that their LDS latency is paid once per group
#pragma unroll
        for (int k8 = 0; k8 < FK / 2; k8 += 8) {
            float fa[8], fb[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                fa[j] = sT[wm * 32 + lrow][(k8 + j) * 2 + lhalf];
                fb[j] = sB[wn * 32 + lrow][(k8 + j) * 2 + lhalf];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[j], fb[j], acc, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
    }
}

template <bool VEC>
__global__ __launch_bounds__(kThreads) void k_gram_f32(GramArgsF a) {
    __shared__ float sT[FT][FP];
    __shared__ float sS[FT][FP];
    __shared__ float red[4];

    const int ex = blockIdx.x / a.npairs;
    int pair = blockIdx.x - ex * a.npairs;
    // pair -> (tt, ss), tt <= ss, rows of the upper triangle in order
    int tt = 0;
    while (pair >= a.nt - tt) { pair -= a.nt - tt; ++tt; }
    const int ss = tt + pair;
    const bool diag = (tt == ss);

    f32x16 accP, accQ;
#pragma unroll
    for (int r = 0; r < 16; ++r) { accP[r] = 0.f; accQ[r] = 0.f; }
    gram_product_f32<VEC>(a.A + (size_t)ex * a.T * a.d_in, a.T, a.d_in, tt * FT, ss * FT, diag, sT, sS, accP);
    gram_product_f32<VEC>(a.G + (size_t)ex * a.T * a.d_out, a.T, a.d_out, tt * FT, ss * FT, diag, sT, sS, accQ);

    // rows beyond T were stored as zeros, so their entries of both tiles are zero
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) s += accP[r] * accQ[r];
    s = block_sum_256(s, red);
    if (threadIdx.x == 0) a.partial[blockIdx.x] = diag ? s : 2.0f * s;
}

// Short sequences (T <= 32: the late convolutions of an image model, 16 positions of 2304 to 4608 inputs): the kernel
// above would give the one useful 32 x 32 tile to one wave, a chain of d / 2 dependent 64-cycle MFMAs (75 to 135 us
// for such layers), while three waves multiply zeros.  Here the four waves split the contraction: every stage holds
// 128 columns of the example's rows, wave w takes columns 32 w .. 32 w + 31 of it, and the four partial tiles are
// added through LDS in the order w = 0 .. 3, first for A A^T, then for G G^T; the tile is diagonal, so both MFMA
// operands are the same fragment.  One workgroup per example.
constexpr int SK = 128;       // contraction elements per stage
constexpr int SP = SK + 1;    // padded row length in LDS
template <bool VEC>
__device__ __forceinline__ void gram_small_product(const float* __restrict__ Xi, int T, int D, float (*sX)[SP],
                                                   float (*part)[32][33], float (*out)[33]) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lrow = lane & 31, lhalf = lane >> 5;
    // global -> LDS: a thread moves four 4-column pieces per stage: rows lr + 8 v, columns lc .. lc + 3
    const int lr = tid >> 5, lc = (tid & 31) * 4;
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    float x[2][4][4];
    auto fetch = [&](int b, int k0) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = lr + 8 * v;
            const float* p = Xi + (size_t)(row < T ? row : T - 1) * D;
            if (VEC) {
                const int c = (k0 + lc < D) ? k0 + lc : 0;
                const float4 q = *reinterpret_cast<const float4*>(p + c);
                x[b][v][0] = q.x; x[b][v][1] = q.y; x[b][v][2] = q.z; x[b][v][3] = q.w;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) x[b][v][j] = p[(k0 + lc + j < D) ? k0 + lc + j : 0];
            }
        }
    };
    auto commit = [&](int b, int k0) {
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                sX[lr + 8 * v][lc + j] = (lr + 8 * v < T && k0 + lc + j < D) ? x[b][v][j] : 0.f;
    };
    // two stages of loads in flight
    if (D > 0) fetch(0, 0);
    if (D > SK) fetch(1, SK);
    for (int k0 = 0; k0 < D; k0 += 2 * SK) {
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int kb = k0 + b * SK;
            if (kb >= D) break;
            commit(b, kb);
            __syncthreads();
            if (kb + 2 * SK < D) fetch(b, kb + 2 * SK);
            float f[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) f[j] = sX[lrow][wave * 32 + 2 * j + lhalf];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < 16; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(f[j], f[j], acc, 0, 0, 0);
            __syncthreads();
        }
    }
    // accumulator element r of a lane: row 8 (r / 4) + 4 lhalf + r % 4, column lrow
#pragma unroll
    for (int r = 0; r < 16; ++r) part[wave][8 * (r >> 2) + 4 * lhalf + (r & 3)][lrow] = acc[r];
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int idx = tid + 256 * e, mr = idx >> 5, nc = idx & 31;
        out[mr][nc] = ((part[0][mr][nc] + part[1][mr][nc]) + part[2][mr][nc]) + part[3][mr][nc];
    }
    __syncthreads();
}

template <bool VEC>
__global__ __launch_bounds__(kThreads) void k_gram_f32_small(GramArgsF a) {
    __shared__ float sX[32][SP];
    __shared__ float part[4][32][33];
    __shared__ float P[32][33], Q[32][33];
    __shared__ float red[4];
    const int ex = blockIdx.x;
    gram_small_product<VEC>(a.A + (size_t)ex * a.T * a.d_in, a.T, a.d_in, sX, part, P);
    gram_small_product<VEC>(a.G + (size_t)ex * a.T * a.d_out, a.T, a.d_out, sX, part, Q);
    // rows beyond T were stored as zeros, so their entries of both tiles are zero
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int idx = threadIdx.x + 256 * e, mr = idx >> 5, nc = idx & 31;
        s += P[mr][nc] * Q[mr][nc];
    }
    s = block_sum_256(s, red);
    if (threadIdx.x == 0) a.partial[ex] = s;
}

}  // namespace

GramPlan plan_gram_f32(int T) {
    GramPlan p;
    p.tile = FT;
    p.nt = (T + FT - 1) / FT;
    p.npairs = p.nt * (p.nt + 1) / 2;
    return p;
}

hipError_t launch_gram_f32(const GramPlan& p, const float* A, const float* G, int B, int T, int d_in, int d_out,
                           bool accumulate, float* sqnorm, float* partial, hipStream_t st, const ClipOut* co) {
    GramArgsF a;
    a.A = A; a.G = G; a.partial = partial;
    a.T = T; a.d_in = d_in; a.d_out = d_out;
    a.nt = p.nt; a.npairs = p.npairs;
    const int64_t grid = (int64_t)B * p.npairs;
    if (grid >= (int64_t(1) << 31)) return hipErrorInvalidValue;
    if (T <= 32) {              // one tile pair per example (p.npairs == 1): the four waves split the contraction
        if (((d_in | d_out) & 3) == 0) k_gram_f32_small<true><<<(unsigned)B, kThreads, 0, st>>>(a);
        else                           k_gram_f32_small<false><<<(unsigned)B, kThreads, 0, st>>>(a);
    } else if (((d_in | d_out) & 3) == 0) k_gram_f32<true><<<(unsigned)grid, kThreads, 0, st>>>(a);
    else                                  k_gram_f32<false><<<(unsigned)grid, kThreads, 0, st>>>(a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_finalize_partials(partial, B, p.npairs, accumulate, sqnorm, st, co);
}

}  // namespace dpk
