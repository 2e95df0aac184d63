// float32 K-major products  P = sum_k A[k, m-tile]^T G[k, n-tile]  on the
// fp32 MFMA (v_mfma_f32_32x32x2_f32).  That instruction takes one k per lane
// (lanes 0-31: k, lanes 32-63: k+1), so the K-major tiles are used as they lie
// in memory: LDS holds [k][col] and consecutive lanes read consecutive floats.
// Same two uses as the bf16 file: clipped sum (rows of A scaled by their
// example's clip factor, exactly, in fp32) and direct squared norm.
#include "dp_common.h"
#include "dp_internal.h"

namespace dpk {

namespace {

constexpr int FBK = 16;               // k rows per stage
constexpr int FBM = 64, FBN = 64;     // block tile; 2 x 2 waves, one 32 x 32 MFMA tile each

struct TnArgsF {
    const float* A;
    const float* G;
    const float* clip;
    float* out;
    int64_t slice;
    int K, T, M, N;
    int tiles_m, tiles_n;
    int kchunk;
    int accumulate;
};

__device__ __forceinline__ float4 load4_guarded(const float* __restrict__ X, int D, bool vec_ok,
                                                int row, int k_end, int col0) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (row >= k_end) return v;
    const float* p = X + (size_t)row * D;
    if (vec_ok) {
        if (col0 < D) v = *reinterpret_cast<const float4*>(p + col0);
    } else {
        if (col0 + 0 < D) v.x = p[col0 + 0];
        if (col0 + 1 < D) v.y = p[col0 + 1];
        if (col0 + 2 < D) v.z = p[col0 + 2];
        if (col0 + 3 < D) v.w = p[col0 + 3];
    }
    return v;
}

template <int MODE>
__global__ __launch_bounds__(kThreads) void k_tn_f32(TnArgsF a) {
    __shared__ __attribute__((aligned(16))) float sA[FBK][FBM];
    __shared__ __attribute__((aligned(16))) float sG[FBK][FBN];
    __shared__ float red[4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tile = blockIdx.x;
    const int tm = tile / a.tiles_n, tn = tile % a.tiles_n;
    const int m0 = tm * FBM, n0 = tn * FBN;
    const int z = blockIdx.y;
    int k_begin, k_end;
    if (MODE == 0) { k_begin = z * a.kchunk; k_end = min(a.K, k_begin + a.kchunk); }
    else { k_begin = z * a.T; k_end = k_begin + a.T; }

    // each thread moves one float4 of A and one of G per stage
    const int lr = tid >> 4;            // row in stage, 0..15
    const int lc = (tid & 15) * 4;      // column in tile
    const bool vecA = (a.M & 3) == 0, vecG = (a.N & 3) == 0;

    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = lane & 31, lhalf = lane >> 5;
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;

    float4 va, vg;
    auto fetch = [&](int k0) {
        const int row = k0 + lr;
        va = load4_guarded(a.A, a.M, vecA, row, k_end, m0 + lc);
        vg = load4_guarded(a.G, a.N, vecG, row, k_end, n0 + lc);
        if (MODE == 0 && row < k_end) {
            const float c = a.clip[a.T == 1 ? row : row / a.T];
            va.x *= c; va.y *= c; va.z *= c; va.w *= c;
        }
    };

    if (k_begin < k_end) fetch(k_begin);
    for (int k0 = k_begin; k0 < k_end; k0 += FBK) {
        *reinterpret_cast<float4*>(&sA[lr][lc]) = va;
        *reinterpret_cast<float4*>(&sG[lr][lc]) = vg;
        __syncthreads();
        if (k0 + FBK < k_end) fetch(k0 + FBK);
#pragma unroll
        for (int ks = 0; ks < FBK / 2; ++ks) {
            const float fa = sA[ks * 2 + lhalf][wm * 32 + lrow];
            const float fb = sG[ks * 2 + lhalf][wn * 32 + lrow];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa, fb, acc, 0, 0, 0);
        }
        __syncthreads();
    }

    if (MODE == 0) {
        float* out = a.out + (size_t)z * a.slice;
        const int n = n0 + wn * 32 + lrow;
        if (n < a.N) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
                if (m < a.M) {
                    float* p = out + (size_t)m * a.N + n;
                    *p = a.accumulate ? *p + acc[r] : acc[r];
                }
            }
        }
    } else {
        float s = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[r] * acc[r];
        s = block_sum_256(s, red);
        if (tid == 0) a.out[(size_t)z * (a.tiles_m * a.tiles_n) + tile] = s;
    }
}

inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

}  // namespace

TnPlan plan_clipped_f32(int B, int T, int M, int N) {
    const int64_t K = (int64_t)B * T;
    TnPlan p;
    p.segmented = false; p.epu = 0; p.big = false; p.dma = false;
    p.tile_m = FBM; p.tile_n = FBN;
    p.tiles_m = ceil_div(M, FBM); p.tiles_n = ceil_div(N, FBN);
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    int64_t want = (512 + tiles - 1) / tiles;
    int64_t max_splits = (K + 4 * FBK - 1) / (4 * FBK);
    if (want > max_splits) want = max_splits;
    if (want < 1) want = 1;
    int64_t kchunk = (K + want - 1) / want;
    kchunk = ((kchunk + FBK - 1) / FBK) * FBK;
    if (kchunk < FBK) kchunk = FBK;
    p.kchunk = (int)kchunk;
    p.splits = (int)((K + kchunk - 1) / kchunk);
    if (p.splits < 1) p.splits = 1;
    return p;
}

TnPlan plan_direct_f32(int T, int M, int N) {
    (void)T;
    TnPlan p;
    p.segmented = false; p.epu = 0; p.big = false; p.dma = false;
    p.tile_m = FBM; p.tile_n = FBN;
    p.tiles_m = ceil_div(M, FBM); p.tiles_n = ceil_div(N, FBN);
    p.splits = 1; p.kchunk = 0;
    return p;
}

hipError_t launch_clipped_f32(const TnPlan& p, const float* A, const float* G, const float* clip,
                              int B, int T, int M, int N, bool accumulate, float* grad, float* ws, hipStream_t st) {
    TnArgsF a;
    a.A = A; a.G = G; a.clip = clip;
    a.K = B * T; a.T = T; a.M = M; a.N = N;
    a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n; a.kchunk = p.kchunk;
    const int64_t n = (int64_t)M * N;
    if (p.splits == 1) { a.out = grad; a.slice = 0; a.accumulate = accumulate ? 1 : 0; }
    else { a.out = ws; a.slice = splitk_slice_elems(n); a.accumulate = 0; }
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)p.splits);
    k_tn_f32<0><<<grid, kThreads, 0, st>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.splits == 1) return e;
    return launch_splitk_reduce(ws, n, p.splits, accumulate, grad, st);
}

hipError_t launch_direct_f32(const TnPlan& p, const float* A, const float* G, int B, int T, int M, int N,
                             bool accumulate, float* sqnorm, float* partial, hipStream_t st) {
    TnArgsF a;
    a.clip = nullptr;
    a.K = B * T; a.T = T; a.M = M; a.N = N;
    a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n; a.kchunk = 0;
    a.slice = 0; a.accumulate = 0;
    const int tiles = p.tiles_m * p.tiles_n;
    for (int b0 = 0; b0 < B; b0 += 65535) {
        const int nb = (B - b0 < 65535) ? (B - b0) : 65535;
        a.A = A + (size_t)b0 * T * M;
        a.G = G + (size_t)b0 * T * N;
        a.out = partial + (size_t)b0 * tiles;
        dim3 grid((unsigned)tiles, (unsigned)nb);
        k_tn_f32<1><<<grid, kThreads, 0, st>>>(a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return launch_finalize_partials(partial, B, tiles, accumulate, sqnorm, st);
}

}  // namespace dpk
