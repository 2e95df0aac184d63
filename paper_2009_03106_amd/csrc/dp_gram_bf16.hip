// Gram path for the per-example squared norm (16-bit inputs: bf16 or fp16):
//     ||A_i^T G_i||_F^2 = sum_{t,s} (A_i A_i^T)_{ts} (G_i G_i^T)_{ts}.
// One workgroup owns one (example, t-tile, s-tile) with t-tile <= s-tile.  It
// forms the tile of A_i A_i^T (contraction over d_in) and then the tile of
// G_i G_i^T (contraction over d_out) in MFMA accumulators that share one
// register layout, multiplies them lane by lane, and reduces to one float.
// Off-diagonal tile pairs stand for their mirror image too and are weighted by
// two.  Nothing of size T x T leaves the chip; the per-pair partial sums are
// folded per example in a fixed order by a second small kernel.
//
// Both Gram products contract over the contiguous axis of their operand, so
// the 16-byte global pieces are already what an MFMA lane needs (8 consecutive
// k for one row): tiles are copied to LDS unchanged (swizzled by row).
#include "dp_common.h"
#include "dp_internal.h"

namespace dpk {

namespace {

constexpr int GBK = 64;      // contraction elements per LDS stage

struct GramArgs {
    const uint16_t* A;
    const uint16_t* G;
    float* partial;      // [B][npairs]
    int T, d_in, d_out;
    int nt, npairs;
    // one tile pair per example (T <= 64): the kernel completes the norm itself, no second launch
    float* sqnorm;       // nullptr: write partial[]
    int accumulate;
    float C; float* clip;
};

// Rows [row0, row0 + TT) x columns [k0, k0 + 64) of X_i[T, D] -> LDS tile (zero padded).  For widths that are not
// multiples of 8 the loads are issued unconditionally from clamped (valid) addresses and zeroed afterwards (with a
// branch around each of the 8 scalar loads of a piece they went out one memory round trip after the other); widths
// that are multiples of 4 take 8-byte pieces.
template <int TT>
__device__ __forceinline__ void gram_fetch(const uint16_t* __restrict__ Xi, int T, int D, bool vec_ok,
                                           int row0, int k0, int tid, uint4 (&st)[TT / 32]) {
    const int c = tid & 7;
    const int col = k0 + c * 8;
#pragma unroll
    for (int it = 0; it < TT / 32; ++it) {
        const int row = row0 + (tid >> 3) + it * 32;
        const bool in = row < T;
        const uint16_t* p = Xi + (size_t)min(row, T - 1) * D;
        if (vec_ok) {
            // (16-byte pieces: the guarded form is the faster one here, measured)
            st[it] = make_uint4(0u, 0u, 0u, 0u);
            if (in && col < D) st[it] = *reinterpret_cast<const uint4*>(Xi + (size_t)row * D + col);
        } else if ((D & 3) == 0) {
            const bool ok0 = col < D, ok1 = col + 4 < D;
            const uint2 lo = *reinterpret_cast<const uint2*>(p + (ok0 ? col : 0)), hi = *reinterpret_cast<const uint2*>(p + (ok1 ? col + 4 : 0));
            st[it] = make_uint4((in && ok0) ? lo.x : 0u, (in && ok0) ? lo.y : 0u, (in && ok1) ? hi.x : 0u, (in && ok1) ? hi.y : 0u);
        } else {
            uint32_t e[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) e[j] = p[min(col + j, D - 1)];
            uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int j = 0; j < 8; ++j) w[j >> 1] |= ((in && col + j < D) ? e[j] : 0u) << ((j & 1) * 16);
            st[it] = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
}

template <int TT>
__device__ __forceinline__ void gram_commit(unsigned char* lds_tile, int tid, const uint4 (&st)[TT / 32]) {
    const int c = tid & 7;
#pragma unroll
    for (int it = 0; it < TT / 32; ++it) {
        const int r = (tid >> 3) + it * 32;
        *reinterpret_cast<uint4*>(lds_tile + lds_off_bytes(r, c)) = st[it];
    }
}

// One Gram product tile: acc[i][j] += X[t-tile rows] . X[s-tile rows]^T over D.
template <int TT, bool F16>
__device__ __forceinline__ void gram_product(const uint16_t* __restrict__ Xi, int T, int D, int t0, int s0, bool diag,
                                             unsigned char* lds, f32x16 (&acc)[TT / 64][TT / 64]) {
    constexpr int WT = TT / 2;       // rows (and columns) per wave
    constexpr int NF = WT / 32;      // MFMA tiles per wave per side
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = lane & 31, lhalf = lane >> 5;
    const bool vec_ok = (D & 7) == 0;
    unsigned char* lds_t = lds;
    unsigned char* lds_s = diag ? lds : lds + TT * 128;

    uint4 st_t[TT / 32], st_s[TT / 32];
    gram_fetch<TT>(Xi, T, D, vec_ok, t0, 0, tid, st_t);
    if (!diag) gram_fetch<TT>(Xi, T, D, vec_ok, s0, 0, tid, st_s);
    for (int k0 = 0; k0 < D; k0 += GBK) {
        gram_commit<TT>(lds_t, tid, st_t);
        if (!diag) gram_commit<TT>(lds_s, tid, st_s);
        __syncthreads();
        if (k0 + GBK < D) {
            gram_fetch<TT>(Xi, T, D, vec_ok, t0, k0 + GBK, tid, st_t);
            if (!diag) gram_fetch<TT>(Xi, T, D, vec_ok, s0, k0 + GBK, tid, st_s);
        }
#pragma unroll
        for (int ks = 0; ks < GBK / 16; ++ks) {
            bf16x8 fa[NF], fb[NF];
#pragma unroll
            for (int i = 0; i < NF; ++i)
                fa[i] = *reinterpret_cast<const bf16x8*>(lds_t + lds_off_bytes(wm * WT + i * 32 + lrow, ks * 2 + lhalf));
#pragma unroll
            for (int j = 0; j < NF; ++j)
                fb[j] = *reinterpret_cast<const bf16x8*>(lds_s + lds_off_bytes(wn * WT + j * 32 + lrow, ks * 2 + lhalf));
#pragma unroll
            for (int i = 0; i < NF; ++i)
#pragma unroll
                for (int j = 0; j < NF; ++j)
                    acc[i][j] = In16<F16>::mfma(fa[i], fb[j], acc[i][j]);
        }
        __syncthreads();
    }
}

template <int TT, bool F16>
__global__ __launch_bounds__(kThreads, 2) void k_gram_bf16(GramArgs a) {
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * TT * 128];
    __shared__ float red[4];
    constexpr int NF = TT / 64;

    const int ex = blockIdx.x / a.npairs;
    int pair = blockIdx.x - ex * a.npairs;
    // pair -> (tt, ss), tt <= ss, rows of the upper triangle in order
    int tt = 0;
    while (pair >= a.nt - tt) { pair -= a.nt - tt; ++tt; }
    const int ss = tt + pair;
    const bool diag = (tt == ss);

    f32x16 accP[NF][NF], accQ[NF][NF];
#pragma unroll
    for (int i = 0; i < NF; ++i)
#pragma unroll
        for (int j = 0; j < NF; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) { accP[i][j][r] = 0.f; accQ[i][j][r] = 0.f; }

    gram_product<TT, F16>(a.A + (size_t)ex * a.T * a.d_in, a.T, a.d_in, tt * TT, ss * TT, diag, lds, accP);
    gram_product<TT, F16>(a.G + (size_t)ex * a.T * a.d_out, a.T, a.d_out, tt * TT, ss * TT, diag, lds, accQ);

    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NF; ++i)
#pragma unroll
        for (int j = 0; j < NF; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) s += accP[i][j][r] * accQ[i][j][r];
    s = block_sum_256(s, red);
    if (threadIdx.x == 0) {
        const float v = diag ? s : 2.0f * s;
        if (a.sqnorm) {
            const float t = a.accumulate ? a.sqnorm[ex] + v : v;
            a.sqnorm[ex] = t;
            if (a.clip) a.clip[ex] = clip_factor_of(t, a.C);
        } else {
            a.partial[blockIdx.x] = v;
        }
    }
}

// One tile pair per example (T <= 64), 8 waves: waves 0-3 form A_i A_i^T while waves 4-7 form G_i G_i^T, each
// wave a 32 x 32 block of its 64 x 64 product, and the two meet through LDS at the end.  A launch of B workgroups is a
// chain of memory round trips, one per 64-column stage, and this halves the chain.
template <bool F16>
__global__ __launch_bounds__(512) void k_gram_bf16_two(GramArgs a) {
    __shared__ __attribute__((aligned(16))) unsigned char lds[2][64 * 128];
    __shared__ float xq[4][16][64];
    __shared__ float red[4];
    const int ex = blockIdx.x;
    const int side = threadIdx.x >> 8;                       // 0: A, 1: G
    const int tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int D = side ? a.d_out : a.d_in;
    const uint16_t* Xi = side ? a.G + (size_t)ex * a.T * a.d_out : a.A + (size_t)ex * a.T * a.d_in;
    const int Dmax = a.d_in > a.d_out ? a.d_in : a.d_out;
    const bool vec_ok = (D & 7) == 0;
    unsigned char* tile = lds[side];

    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    uint4 st[2];
    gram_fetch<64>(Xi, a.T, D, vec_ok, 0, 0, tid, st);
    for (int k0 = 0; k0 < Dmax; k0 += GBK) {
        const bool on = k0 < D;                              // uniform over a side's waves
        if (on) gram_commit<64>(tile, tid, st);
        __syncthreads();
        if (k0 + GBK < D) gram_fetch<64>(Xi, a.T, D, vec_ok, 0, k0 + GBK, tid, st);
        if (on) {
#pragma unroll
            for (int ks = 0; ks < GBK / 16; ++ks) {
                const bf16x8 fa = *reinterpret_cast<const bf16x8*>(tile + lds_off_bytes(wm * 32 + lrow, ks * 2 + lhalf));
                const bf16x8 fb = *reinterpret_cast<const bf16x8*>(tile + lds_off_bytes(wn * 32 + lrow, ks * 2 + lhalf));
                acc = In16<F16>::mfma(fa, fb, acc);
            }
        }
        __syncthreads();
    }
    if (side == 1) {
#pragma unroll
        for (int r = 0; r < 16; ++r) xq[wave][r][lane] = acc[r];
    }
    __syncthreads();
    float s = 0.f;
    if (side == 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[r] * xq[wave][r][lane];
        s = wave_sum(s);
        if (lane == 0) red[wave] = s;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const float v = (red[0] + red[1]) + (red[2] + red[3]);
        const float t = a.accumulate ? a.sqnorm[ex] + v : v;
        a.sqnorm[ex] = t;
        if (a.clip) a.clip[ex] = clip_factor_of(t, a.C);
    }
}

}  // namespace

GramPlan plan_gram_bf16(int T, int d_in, int d_out) {
    (void)d_in; (void)d_out;
    GramPlan p;
    p.tile = (T <= 64) ? 64 : 128;
    p.nt = (T + p.tile - 1) / p.tile;
    p.npairs = p.nt * (p.nt + 1) / 2;
    return p;
}

hipError_t launch_gram_bf16(const GramPlan& p, const uint16_t* A, const uint16_t* G, int B, int T, int d_in, int d_out,
                            bool accumulate, float* sqnorm, float* partial, hipStream_t st, bool f16, const ClipOut* co) {
    if (gram_dma_ok(T, d_in, d_out)) return launch_gram_bf16_dma(p, A, G, B, T, d_in, d_out, accumulate, sqnorm, partial, st, f16, co);
    GramArgs a;
    a.A = A; a.G = G; a.partial = partial;
    a.T = T; a.d_in = d_in; a.d_out = d_out;
    a.nt = p.nt; a.npairs = p.npairs;
    const bool direct = p.npairs == 1;
    a.sqnorm = direct ? sqnorm : nullptr; a.accumulate = accumulate ? 1 : 0;
    a.C = co ? co->C : 0.f; a.clip = co ? co->clip : nullptr;
    const unsigned grid = (unsigned)((int64_t)B * p.npairs);
    if (p.tile == 64) { if (f16) k_gram_bf16_two<true><<<grid, 512, 0, st>>>(a); else k_gram_bf16_two<false><<<grid, 512, 0, st>>>(a); }
    else              { if (f16) k_gram_bf16<128, true><<<grid, kThreads, 0, st>>>(a); else k_gram_bf16<128, false><<<grid, kThreads, 0, st>>>(a); }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || direct) return e;
    return launch_finalize_partials(partial, B, p.npairs, accumulate, sqnorm, st, co);
}

}  // namespace dpk
