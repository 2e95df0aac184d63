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

// k rows per stage: 64 where the contraction is long enough (a stage costs a global-load latency and two barriers
// whatever its size, so short stages make the loop latency-bound), 16 for short ones (direct norm of short sequences,
// where a 64-row stage would be mostly zero padding)
inline int stage_rows(int64_t k) { return k >= 128 ? 64 : 16; }
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
    int slices_per_example = 1;     // mode 2
};

// The loads of a stage are issued unconditionally from clamped (valid) addresses and zeroed afterwards: no branch
// sits between them, so they are all in flight together (a guarded load costs one memory round trip each).
// VECA / VECG: d_in / d_out is a multiple of 4, so every 16-byte piece of that operand is all inside or all outside a
// row and is one load; otherwise a piece is four 4-byte loads (each operand by itself: a 256 -> 10 classifier head
// still reads its wide operand in 16-byte pieces).
template <int MODE, int FBK, bool VECA, bool VECG>
__global__ __launch_bounds__(kThreads) void k_tn_f32(TnArgsF a) {
    constexpr int NV = FBK / 16;        // float4 pieces of either operand per thread and stage
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
    else if (MODE == 2) {
        // slice z = (example, chunk of its positions), its share of A_i^T G_i stored unscaled (direct norm of few long
        // examples of a small layer, see plan_direct_chunks)
        const int ex = z / a.slices_per_example, ch = z - ex * a.slices_per_example;
        k_begin = ex * a.T + ch * a.kchunk;
        k_end = min(ex * a.T + a.T, k_begin + a.kchunk);
    }
    else { k_begin = z * a.T; k_end = k_begin + a.T; }

    // each thread moves NV float4 of A and of G per stage: rows lr, lr + 16, ..., columns lc .. lc + 3 of the tile
    const int lr = tid >> 4;            // 0..15
    const int lc = (tid & 15) * 4;
    bool okA[4], okG[4];                // the column lies inside the matrix
    int colA[4], colG[4];               // a valid column to load from
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        okA[j] = m0 + lc + j < a.M; okG[j] = n0 + lc + j < a.N;
        colA[j] = okA[j] ? m0 + lc + j : 0; colG[j] = okG[j] ? n0 + lc + j : 0;
    }

    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = lane & 31, lhalf = lane >> 5;
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;

    float xa[NV][4], xg[NV][4];         // what fetch() loaded; scaled and zeroed in commit(), one stage of MFMAs
    float cl[NV];                       // later, so that the loads stay in flight behind them
    bool inr[NV];                       // the row lies inside the slice
    auto fetch = [&](int k0) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int row = k0 + lr + 16 * v;
            inr[v] = row < k_end;
            const int rc = inr[v] ? row : k_end - 1;                    // k_begin < k_end whenever a stage is fetched
            const float* pa = a.A + (size_t)rc * a.M;
            const float* pg = a.G + (size_t)rc * a.N;
            if (VECA) {
                const float4 qa = *reinterpret_cast<const float4*>(pa + colA[0]);
                xa[v][0] = qa.x; xa[v][1] = qa.y; xa[v][2] = qa.z; xa[v][3] = qa.w;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) xa[v][j] = pa[colA[j]];
            }
            if (VECG) {
                const float4 qg = *reinterpret_cast<const float4*>(pg + colG[0]);
                xg[v][0] = qg.x; xg[v][1] = qg.y; xg[v][2] = qg.z; xg[v][3] = qg.w;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) xg[v][j] = pg[colG[j]];
            }
            cl[v] = (MODE == 0) ? a.clip[a.T == 1 ? rc : rc / a.T] : 1.0f;
        }
    };
    auto commit = [&]() {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            float ya[4], yg[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                ya[j] = (inr[v] && okA[j]) ? xa[v][j] * cl[v] : 0.f;
                yg[j] = (inr[v] && okG[j]) ? xg[v][j] : 0.f;
            }
            *reinterpret_cast<float4*>(&sA[lr + 16 * v][lc]) = make_float4(ya[0], ya[1], ya[2], ya[3]);
            *reinterpret_cast<float4*>(&sG[lr + 16 * v][lc]) = make_float4(yg[0], yg[1], yg[2], yg[3]);
        }
    };

    if (k_begin < k_end) fetch(k_begin);
    for (int k0 = k_begin; k0 < k_end; k0 += FBK) {
        commit();
        __syncthreads();
        if (k0 + FBK < k_end) fetch(k0 + FBK);
        // the operands of 8 MFMAs are read together, so that their LDS latency is paid once per group
#pragma unroll
        for (int k8 = 0; k8 < FBK / 2; k8 += 8) {
            float fa[8], fb[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                fa[j] = sA[(k8 + j) * 2 + lhalf][wm * 32 + lrow];
                fb[j] = sG[(k8 + j) * 2 + lhalf][wn * 32 + lrow];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[j], fb[j], acc, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
    }

    if (MODE == 0 || MODE == 2) {
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

// Clipped sum over a short contraction (dense layers: K = B, a few hundred rows): 32 x 32 output tile per workgroup,
// the four waves split the rows of every 64-row stage between them (wave w: rows 16 w .. 16 w + 15) and their four
// partial tiles are added through LDS in the order w = 0 .. 3.  The fp32 MFMA is a chain of dependent 64-cycle
// instructions per wave, so the 64 x 64 kernel above, one wave per 32 x 32 tile, needs K / 2 of them in a row and
// fills only (d_in / 64)(d_out / 64) compute units; here a wave runs K / 8 and there are four times as many
// workgroups.  No K slices: the whole sum is finished in the kernel.
constexpr int SBK = 64, STM = 32, STN = 32;
#define SHORT_LDS                                                          \
    __shared__ __attribute__((aligned(16))) float sA[SBK][STM];            \
    __shared__ __attribute__((aligned(16))) float sG[SBK][STN];            \
    __shared__ __attribute__((aligned(16))) float part[4][STM][STN + 1]
template <bool VECA, bool VECG>
__device__ __forceinline__ void tn_f32_short_tile(const TnArgsF& a, int tile, float (*sA)[STM], float (*sG)[STN],
                                                  float (*part)[STM][STN + 1]) {
    constexpr int NV = 2;               // float4 pieces of either operand per thread and stage

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tm = tile / a.tiles_n, tn = tile % a.tiles_n;
    const int m0 = tm * STM, n0 = tn * STN;
    const int k_end = a.K;

    // each thread moves NV float4 of A and of G per stage: rows lr, lr + 32, columns lc .. lc + 3 of the tile
    const int lr = tid >> 3;            // 0..31
    const int lc = (tid & 7) * 4;
    bool okA[4], okG[4];
    int colA[4], colG[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        okA[j] = m0 + lc + j < a.M; okG[j] = n0 + lc + j < a.N;
        colA[j] = okA[j] ? m0 + lc + j : 0; colG[j] = okG[j] ? n0 + lc + j : 0;
    }
    const int lrow = lane & 31, lhalf = lane >> 5;
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;

    // The loads of GS stages (256 rows: a whole contraction of the dense configurations) are issued before any of
    // them is used, so that a workgroup waits for memory once per 256 rows and not once per stage: with K = B = 256
    // the kernel is one memory latency, four short MFMA chains and the epilogue.
    constexpr int GS = 4;
    float xa[GS][NV][4], xg[GS][NV][4], cl[GS][NV];
    auto fetch = [&](int g, int k0) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int row = k0 + lr + 32 * v;
            const int rc = row < k_end ? row : k_end - 1;
            const float* pa = a.A + (size_t)rc * a.M;
            const float* pg = a.G + (size_t)rc * a.N;
            if (VECA) {
                const float4 qa = *reinterpret_cast<const float4*>(pa + colA[0]);
                xa[g][v][0] = qa.x; xa[g][v][1] = qa.y; xa[g][v][2] = qa.z; xa[g][v][3] = qa.w;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) xa[g][v][j] = pa[colA[j]];
            }
            if (VECG) {
                const float4 qg = *reinterpret_cast<const float4*>(pg + colG[0]);
                xg[g][v][0] = qg.x; xg[g][v][1] = qg.y; xg[g][v][2] = qg.z; xg[g][v][3] = qg.w;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) xg[g][v][j] = pg[colG[j]];
            }
            cl[g][v] = a.clip[a.T == 1 ? rc : rc / a.T];
        }
    };
    auto commit = [&](int g, int k0) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const bool inr = k0 + lr + 32 * v < k_end;
            float ya[4], yg[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                ya[j] = (inr && okA[j]) ? xa[g][v][j] * cl[g][v] : 0.f;
                yg[j] = (inr && okG[j]) ? xg[g][v][j] : 0.f;
            }
            *reinterpret_cast<float4*>(&sA[lr + 32 * v][lc]) = make_float4(ya[0], ya[1], ya[2], ya[3]);
            *reinterpret_cast<float4*>(&sG[lr + 32 * v][lc]) = make_float4(yg[0], yg[1], yg[2], yg[3]);
        }
    };

    for (int kg = 0; kg < k_end; kg += GS * SBK) {
#pragma unroll
        for (int g = 0; g < GS; ++g)
            if (kg + g * SBK < k_end) fetch(g, kg + g * SBK);
#pragma unroll
        for (int g = 0; g < GS; ++g) {
            const int k0 = kg + g * SBK;
            if (k0 >= k_end) break;
            commit(g, k0);
            __syncthreads();
            float fa[8], fb[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                fa[j] = sA[wave * 16 + j * 2 + lhalf][lrow];
                fb[j] = sG[wave * 16 + j * 2 + lhalf][lrow];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[j], fb[j], acc, 0, 0, 0);
            __syncthreads();
        }
    }

    // accumulator element r of a lane: row 8 (r / 4) + 4 lhalf + r % 4, column lrow of the 32 x 32 tile
#pragma unroll
    for (int r = 0; r < 16; ++r) part[wave][8 * (r >> 2) + 4 * lhalf + (r & 3)][lrow] = acc[r];
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int idx = tid + 256 * e;              // 1024 outputs, 4 per thread; consecutive threads: consecutive columns
        const int mr = idx >> 5, nc = idx & 31;
        const int m = m0 + mr, n = n0 + nc;
        if (m < a.M && n < a.N) {
            const float v = ((part[0][mr][nc] + part[1][mr][nc]) + part[2][mr][nc]) + part[3][mr][nc];
            float* p = a.out + (size_t)m * a.N + n;
            *p = a.accumulate ? *p + v : v;
        }
    }
}

// 16-byte loads for each operand whose width allows them (a 256 -> 10 head must not cost a wide layer its loads,
// nor its own wide operand)
__device__ __forceinline__ void tn_f32_short_dispatch(const TnArgsF& a, int tile, float (*sA)[STM], float (*sG)[STN],
                                                      float (*part)[STM][STN + 1]) {
    const bool va = (a.M & 3) == 0, vg = (a.N & 3) == 0;
    if (va) { if (vg) tn_f32_short_tile<true, true>(a, tile, sA, sG, part); else tn_f32_short_tile<true, false>(a, tile, sA, sG, part); }
    else    { if (vg) tn_f32_short_tile<false, true>(a, tile, sA, sG, part); else tn_f32_short_tile<false, false>(a, tile, sA, sG, part); }
}
__global__ __launch_bounds__(kThreads) void k_tn_f32_short(TnArgsF a) {
    SHORT_LDS;
    tn_f32_short_dispatch(a, blockIdx.x, sA, sG, part);
}

// The same for several layers in one launch (a model of small dense layers is a chain of launches of a few
// microseconds each otherwise): the layers' tiles form one list, in the order given.
constexpr int kShortBatch = 8;
struct TnShortLayers { int n_layers; int first_tile[kShortBatch + 1]; TnArgsF layer[kShortBatch]; };
__global__ __launch_bounds__(kThreads) void k_tn_f32_short_layers(TnShortLayers t) {
    SHORT_LDS;
    int li = 0;
    while (li + 1 < t.n_layers && (int)blockIdx.x >= t.first_tile[li + 1]) ++li;
    const TnArgsF a = t.layer[li];
    tn_f32_short_dispatch(a, (int)blockIdx.x - t.first_tile[li], sA, sG, part);
}

// the short-contraction kernel takes K up to this many rows
constexpr int kShortK = 512;

template <int MODE, int FBK> void launch_f32_k(bool veca, bool vecg, dim3 grid, const TnArgsF& a, hipStream_t st) {
    if (veca) { if (vecg) k_tn_f32<MODE, FBK, true, true><<<grid, kThreads, 0, st>>>(a); else k_tn_f32<MODE, FBK, true, false><<<grid, kThreads, 0, st>>>(a); }
    else      { if (vecg) k_tn_f32<MODE, FBK, false, true><<<grid, kThreads, 0, st>>>(a); else k_tn_f32<MODE, FBK, false, false><<<grid, kThreads, 0, st>>>(a); }
}
template <int MODE> void launch_f32(bool deep, bool veca, bool vecg, dim3 grid, const TnArgsF& a, hipStream_t st) {
    if (deep) launch_f32_k<MODE, 64>(veca, vecg, grid, a, st);
    else      launch_f32_k<MODE, 16>(veca, vecg, grid, a, st);
}

}  // namespace

TnPlan plan_clipped_f32(int B, int T, int M, int N) {
    const int64_t K = (int64_t)B * T;
    TnPlan p;
    p.segmented = false; p.epu = 0; p.big = false; p.dma = false;
    if (K <= kShortK) {
        p.tile_m = STM; p.tile_n = STN;
        p.tiles_m = ceil_div(M, STM); p.tiles_n = ceil_div(N, STN);
        p.splits = 1; p.kchunk = (int)K;
        return p;
    }
    if (f32_dma_ok(K, M, N) && K < (int64_t(1) << 31)) {
        // 128 x 128 tiles on the copy pipeline: two workgroups per compute unit, slices of at least 16 stages
        const int t = f32_dma_tile(), dk = f32_dma_stage_rows();
        p.dma = true;
        p.tile_m = p.tile_n = t;
        p.tiles_m = ceil_div(M, t); p.tiles_n = ceil_div(N, t);
        const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
        // K slices: the (tile, slice) items run 512 at a time (two workgroups per compute unit); an item costs its
        // stages plus about 16 stage times of start-up, store and fold.  Take the slice count with the smallest
        // rounds x (stages per slice + 16): a count that just spills into one more round (540 items) costs a whole
        // extra round, many short slices cost their overheads.
        const int64_t stages = (K + dk - 1) / dk;
        int64_t max_splits = stages / 16;
        if (max_splits < 1) max_splits = 1;
        if (max_splits > 256) max_splits = 256;
        int64_t best = 1, best_cost = -1;
        for (int64_t sp = 1; sp <= max_splits; ++sp) {
            const int64_t sps = (stages + sp - 1) / sp, real = (stages + sps - 1) / sps;
            const int64_t rounds = (tiles * real + 511) / 512;
            const int64_t cost = rounds * (sps + 16);
            if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = sp; }
        }
        const int64_t kchunk = ((stages + best - 1) / best) * dk;
        p.kchunk = (int)kchunk;
        p.splits = (int)((K + kchunk - 1) / kchunk);
        return p;
    }
    p.tile_m = FBM; p.tile_n = FBN;
    p.tiles_m = ceil_div(M, FBM); p.tiles_n = ceil_div(N, FBN);
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    const int FBK = stage_rows(K);
    int64_t want = (512 + tiles - 1) / tiles;
    int64_t max_splits = (K + 4 * FBK - 1) / (4 * FBK);      // at least 4 stages per slice
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

TnPlan plan_direct_f32(int B, int T, int M, int N) {
    TnPlan p;
    p.segmented = false; p.epu = 0; p.big = false; p.dma = false;
    if (f32_dma_ok(T, M, N)) {
        const int t = f32_dma_tile();
        p.dma = true;
        p.tile_m = p.tile_n = t;
        p.tiles_m = ceil_div(M, t); p.tiles_n = ceil_div(N, t);
        p.splits = 1; p.kchunk = 0;
        return p;
    }
    p.tile_m = FBM; p.tile_n = FBN;
    p.tiles_m = ceil_div(M, FBM); p.tiles_n = ceil_div(N, FBN);
    p.splits = 1; p.kchunk = 0;
    plan_direct_chunks(p, B, T, M, N, 4, 64);
    return p;
}

hipError_t launch_clipped_f32(const TnPlan& p, const float* A, const float* G, const float* clip,
                              int B, int T, int M, int N, bool accumulate, float* grad, float* ws, hipStream_t st,
                              const NoiseArgs* noise) {
    TnArgsF a;
    a.A = A; a.G = G; a.clip = clip;
    a.K = B * T; a.T = T; a.M = M; a.N = N;
    a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n; a.kchunk = p.kchunk;
    const int64_t n = (int64_t)M * N;
    if (p.splits == 1) { a.out = grad; a.slice = 0; a.accumulate = accumulate ? 1 : 0; }
    else { a.out = ws; a.slice = splitk_slice_elems(n); a.accumulate = 0; }
    if (p.dma) {
        hipError_t e = launch_tn_f32_dma(0, p, A, G, clip, B, T, M, N, a.out, a.slice, a.accumulate != 0, st);
        if (e != hipSuccess || p.splits == 1) return e;
        return launch_splitk_reduce(ws, n, p.splits, accumulate, grad, st, noise);
    }
    if (p.tile_m == STM) {
        a.out = grad; a.slice = 0; a.accumulate = accumulate ? 1 : 0;
        const unsigned tiles = (unsigned)(p.tiles_m * p.tiles_n);
        k_tn_f32_short<<<tiles, kThreads, 0, st>>>(a);
        return hipGetLastError();
    }
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)p.splits);
    launch_f32<0>(stage_rows(a.K) == 64, (M & 3) == 0, (N & 3) == 0, grid, a, st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.splits == 1) return e;
    return launch_splitk_reduce(ws, n, p.splits, accumulate, grad, st, noise);
}

bool clipped_f32_is_short(const TnPlan& p) { return p.tile_m == STM && p.splits == 1; }

hipError_t launch_clipped_f32_short_layers(const ShortLayerDesc* layers, int n_layers, int B, bool accumulate, hipStream_t st) {
    if (n_layers < 1 || n_layers > kShortBatch) return hipErrorInvalidValue;
    TnShortLayers t;
    t.n_layers = n_layers;
    int64_t first = 0;
    // the layers that cannot use 16-byte loads first: their workgroups take about twice as long, and the workgroups of
    // a launch start in the order of their ids (536 of them for the MLP configuration start over several microseconds)
    int order[kShortBatch], no = 0;
    for (int pass = 0; pass < 2; ++pass)
        for (int l = 0; l < n_layers; ++l)
            if ((((layers[l].M | layers[l].N) & 3) != 0) == (pass == 0)) order[no++] = l;
    for (int l = 0; l < kShortBatch; ++l) {
        t.first_tile[l] = (int)first;
        if (l >= n_layers) { t.layer[l] = TnArgsF{nullptr, nullptr, nullptr, nullptr, 0, 0, 1, 0, 0, 0, 0, 0, 0}; continue; }
        const ShortLayerDesc& y = layers[order[l]];
        TnArgsF& a = t.layer[l];
        a.A = y.A; a.G = y.G; a.clip = y.clip;
        a.K = B * y.T; a.T = y.T; a.M = y.M; a.N = y.N;
        a.tiles_m = ceil_div(y.M, STM); a.tiles_n = ceil_div(y.N, STN); a.kchunk = a.K;
        a.out = y.grad; a.slice = 0; a.accumulate = accumulate ? 1 : 0;
        first += (int64_t)a.tiles_m * a.tiles_n;
        if (first >= (int64_t(1) << 31)) return hipErrorInvalidValue;
    }
    t.first_tile[kShortBatch] = (int)first;
    k_tn_f32_short_layers<<<(unsigned)first, kThreads, 0, st>>>(t);
    return hipGetLastError();
}

hipError_t launch_direct_f32(const TnPlan& p, const float* A, const float* G, int B, int T, int M, int N,
                             bool accumulate, float* sqnorm, float* partial, hipStream_t st, const ClipOut* co) {
    TnArgsF a;
    a.clip = nullptr;
    a.K = B * T; a.T = T; a.M = M; a.N = N;
    a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n; a.kchunk = 0;
    a.slice = 0; a.accumulate = 0;
    const int tiles = p.tiles_m * p.tiles_n;
    if (p.dma) {
        // one launch of (example, tile) items; batches beyond the 32-bit item count go in pieces
        const int64_t per = ((int64_t(1) << 30) / tiles);
        for (int64_t b0 = 0; b0 < B; b0 += per) {
            const int nb = (int)((B - b0 < per) ? (B - b0) : per);
            hipError_t e = launch_tn_f32_dma(1, p, A + (size_t)b0 * T * M, G + (size_t)b0 * T * N, nullptr, nb, T, M, N,
                                             partial + (size_t)b0 * tiles, 0, false, st);
            if (e != hipSuccess) return e;
        }
        return launch_finalize_partials(partial, B, tiles, accumulate, sqnorm, st, co);
    }
    if (p.splits > 1) {
        // chunks of positions: workspace = the chunks' shares [B][S][slice], then sums[B][nblk]
        const int64_t n = (int64_t)M * N, slice = splitk_slice_elems(n);
        const int nblk = (int)((n + 1023) / 1024);
        float* sums = partial + (size_t)B * p.splits * slice;
        a.A = A; a.G = G;
        a.kchunk = p.kchunk; a.out = partial; a.slice = slice; a.slices_per_example = p.splits;
        dim3 grid((unsigned)tiles, (unsigned)(B * p.splits));
        launch_f32<2>(true, (M & 3) == 0, (N & 3) == 0, grid, a, st);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        e = launch_direct_chunks_finish(partial, slice, p.splits, (int)n, B, sums, st);
        if (e != hipSuccess) return e;
        return launch_finalize_partials(sums, B, nblk, accumulate, sqnorm, st, co);
    }
    for (int b0 = 0; b0 < B; b0 += 65535) {
        const int nb = (B - b0 < 65535) ? (B - b0) : 65535;
        a.A = A + (size_t)b0 * T * M;
        a.G = G + (size_t)b0 * T * N;
        a.out = partial + (size_t)b0 * tiles;
        dim3 grid((unsigned)tiles, (unsigned)nb);
        launch_f32<1>(stage_rows(T) == 64, (M & 3) == 0, (N & 3) == 0, grid, a, st);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return launch_finalize_partials(partial, B, tiles, accumulate, sqnorm, st, co);
}

}  // namespace dpk
