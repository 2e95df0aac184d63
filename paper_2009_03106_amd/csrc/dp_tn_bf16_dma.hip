// Large-tile bf16 clipped sum  sum_i c_i A_i^T G_i  for big aligned layers.
//
// gfx950-specific data path, no VALU work in the main loop:
//   * global -> LDS copies go straight into LDS (global_load_lds_dwordx4): a
//     wave instruction moves two 512-byte rows of a K-major tile, as they lie
//     in memory, into 1 KB of LDS.  Four 32-row stages are kept in LDS, three
//     of them in flight while one is consumed.
//   * the 16-bit transpose the MFMA needs (a lane must hold consecutive k for
//     one column, memory has consecutive columns for one k) is done by the
//     LDS read itself (ds_read_b64_tr_b16): 16 lanes read a 4(k) x 16(col)
//     patch and each lane gets the 4 k values of one column.
//   * 256 x 256 output tile per workgroup, one workgroup per compute unit,
//     each of the 4 waves owns 128 x 128 (256 accumulator registers).
//
// Clip factors are applied to the fp32 accumulators, not to the bf16 inputs:
// the tile holds  (1 / c_cur) * sum_{j <= cur} c_j g_j ; when the rows of the
// next example start it is multiplied by c_cur / c_next (one multiply per
// accumulator register per example, skipped when the two factors are equal),
// and by the last example's factor at the end.  This is exact up to one fp32
// rounding per example.  It needs every 32-row stage to lie inside one
// example, hence T % 32 == 0.  K slices are arbitrary ranges of stages.
#include "dp_common.h"
#include "dp_internal.h"

namespace dpk {

namespace {

constexpr int DM = 256, DN = 256;     // output tile
constexpr int DK = 32;                // rows per stage
constexpr int NST = 4;                // stages resident in LDS
constexpr int STAGE_BYTES = 2 * DK * DM * 2;     // A part then G part: 32 KB
constexpr int OPND_BYTES = DK * DM * 2;          // 16 KB

typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef short v8i16 __attribute__((ext_vector_type(8)));
#define LDS_PTR(T) __attribute__((address_space(3))) T*
#define GLB_PTR(T) const __attribute__((address_space(1))) T*

struct DmaArgs {
    const uint16_t* A;
    const uint16_t* G;
    const float* clip;
    float* out;            // slice base (stride `slice` per K slice) or grad
    int64_t slice;
    int B, T, M, N;
    int tiles_m, tiles_n;
    int splits;
    int stages_total;      // B*T / 32
    int stages_per_split;
    int per_xcd;
    int accumulate;
};

// 16-byte chunk c of tile row r sits at chunk position c ^ ((r & 3) << 1): the four rows a
// transposing read touches then fall into four different 32-byte bank windows.
__device__ __forceinline__ int chunk_swz(int r) { return (r & 3) << 1; }

__global__ __launch_bounds__(kThreads, 1) void k_tn_bf16_dma(DmaArgs a) {
    __shared__ __attribute__((aligned(1024))) unsigned char lds[NST * STAGE_BYTES];   // 128 KB

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tiles = a.tiles_m * a.tiles_n;
    const int L = (blockIdx.x & 7) * a.per_xcd + (blockIdx.x >> 3);
    if (L >= tiles * a.splits) return;
    const int z = L / tiles, tile = L - z * tiles;
    const int tm = tile / a.tiles_n, tn = tile - tm * a.tiles_n;
    const int m0 = tm * DM, n0 = tn * DN;
    const int s_begin = z * a.stages_per_split;
    const int s_end = min(a.stages_total, s_begin + a.stages_per_split);
    const int n_stages = s_end - s_begin;
    if (n_stages <= 0) return;
    const int spe = a.T / DK;                       // stages per example

    // ---- global -> LDS: wave w copies rows 8w..8w+7 of the A part and of the G part of a stage,
    //      4 instructions each; instruction u covers rows 8w+2u, 8w+2u+1 (lane / 32 picks the row)
    const int lr = lane >> 5, cp = lane & 31;
    int offA[2], offG[2];                           // element offsets of this lane's source chunk for u even / odd
#pragma unroll
    for (int par = 0; par < 2; ++par) {
        const int r = 2 * par + lr;                 // r & 3 of the row this lane fills
        const int c = cp ^ chunk_swz(r);
        int ca = m0 + c * 8, cgn = n0 + c * 8;
        if (ca >= a.M) ca = m0;                     // out-of-range columns only feed output rows that are never stored
        if (cgn >= a.N) cgn = n0;
        offA[par] = ca;
        offG[par] = cgn;
    }
    const uint16_t* pA = a.A + ((size_t)s_begin * DK + wave * 8 + lr) * a.M;    // row of this lane for u = 0
    const uint16_t* pG = a.G + ((size_t)s_begin * DK + wave * 8 + lr) * a.N;
    const size_t stepA = (size_t)DK * a.M, stepG = (size_t)DK * a.N;            // per stage
    const size_t row2A = (size_t)2 * a.M, row2G = (size_t)2 * a.N;              // per instruction (two rows)

    auto issue = [&](int buf) {
        LDS_PTR(unsigned char) base = (LDS_PTR(unsigned char))lds + buf * STAGE_BYTES + wave * 8 * 512;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            __builtin_amdgcn_global_load_lds((GLB_PTR(void))(pA + u * row2A + offA[u & 1]),
                                             (LDS_PTR(void))(base + u * 1024), 16, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            __builtin_amdgcn_global_load_lds((GLB_PTR(void))(pG + u * row2G + offG[u & 1]),
                                             (LDS_PTR(void))(base + OPND_BYTES + u * 1024), 16, 0, 0);
        }
        pA += stepA;
        pG += stepG;
    };

    // ---- LDS -> MFMA operands.  Lane l of a 16-lane group: source row j = (l % 16) / 4, source column
    //      piece q = l % 4; after the transposing read the lane holds 4 k values of column l % 16.
    const int wm = wave >> 1, wn = wave & 1;
    const int g16 = lane >> 4, s16 = lane & 15;
    const int half = g16 >> 1;                      // lanes 32..63 hold k + 8 .. k + 15 of a 16-wide k step
    const int rsrc = 8 * half + (s16 >> 2);         // row inside the k step for the first read (second read: + 4)
    int rdA[4], rdG[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int ma = wm * 128 + i * 32 + 16 * (g16 & 1) + 4 * (s16 & 3);      // column (element) of the 8-byte piece
        const int na = wn * 128 + i * 32 + 16 * (g16 & 1) + 4 * (s16 & 3);
        rdA[i] = rsrc * 512 + ((((ma >> 3) ^ chunk_swz(rsrc)) << 4) | ((ma & 7) << 1));
        rdG[i] = OPND_BYTES + rsrc * 512 + ((((na >> 3) ^ chunk_swz(rsrc)) << 4) | ((na & 7) << 1));
    }

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // prologue: up to NST - 1 stages in flight
#pragma unroll
    for (int p = 0; p < NST - 1; ++p)
        if (p < n_stages) issue(p);

    int ex = s_begin / spe;
    int sub = s_begin - ex * spe;
    float c_cur = a.clip[ex];

    int st = 0;
    while (st < n_stages) {
        // the stages left in the current example: plain copy / read / MFMA loop, no other vector work
        const int run_end = min(n_stages, st + (spe - sub));
        for (; st < run_end; ++st) {
            // stage st must have landed; the copies of later stages may stay in flight (8 per stage and wave)
            const int ahead = min(n_stages - 1 - st, NST - 2);
            if (ahead >= 2) __builtin_amdgcn_s_waitcnt(0x4F70);        // vmcnt(16)
            else if (ahead == 1) __builtin_amdgcn_s_waitcnt(0x0F78);   // vmcnt(8)
            else __builtin_amdgcn_s_waitcnt(0x0F70);                   // vmcnt(0)
            __syncthreads();
            if (st + NST - 1 < n_stages) issue((st + NST - 1) % NST);

            LDS_PTR(unsigned char) sb = (LDS_PTR(unsigned char))lds + (st % NST) * STAGE_BYTES;
#pragma unroll
            for (int ks = 0; ks < DK / 16; ++ks) {
                bf16x8 fa[4], fb[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(v4i16))(sb + rdA[i] + ks * 16 * 512));
                    const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(v4i16))(sb + rdA[i] + ks * 16 * 512 + 4 * 512));
                    fa[i] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(v4i16))(sb + rdG[j] + ks * 16 * 512));
                    const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(v4i16))(sb + rdG[j] + ks * 16 * 512 + 4 * 512));
                    fb[j] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
            }
        }
        sub = 0;
        ++ex;
        if (st < n_stages) {
            // the next example starts: rescale the running tile
            const float c_next = a.clip[ex];
            if (c_next != c_cur) {
                const float ratio = c_cur / c_next;
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[i][j][r] *= ratio;
            }
            c_cur = c_next;
        }
    }

    // the tile holds (1 / c_cur) * sum: finish with the last example's factor
    float* out = a.out + (size_t)z * a.slice;
    const int lrow = lane & 31, lhalf = lane >> 5;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + wn * 128 + j * 32 + lrow;
            if (n >= a.N) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * 128 + i * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
                if (m < a.M) {
                    float* p = out + (size_t)m * a.N + n;
                    const float v = acc[i][j][r] * c_cur;
                    *p = a.accumulate ? *p + v : v;
                }
            }
        }
}

inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

}  // namespace

bool dma_clipped_ok(int B, int T, int M, int N) {
    (void)B;
    if ((T % DK) != 0 || ((M | N) & 7) != 0) return false;
    const int64_t padded = (int64_t)ceil_div(M, DM) * DM * ceil_div(N, DN) * DN;
    return padded * 4 <= (int64_t)M * N * 5;          // at most a quarter of the padded tiles is waste
}

TnPlan plan_clipped_bf16_dma(int B, int T, int M, int N) {
    TnPlan p;
    p.tile_m = DM; p.tile_n = DN;
    p.tiles_m = ceil_div(M, DM); p.tiles_n = ceil_div(N, DN);
    p.segmented = false; p.epu = 0; p.big = false; p.dma = true;
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    const int64_t stages = (int64_t)B * T / DK;
    // one workgroup per compute unit: as many K slices as fit into 256 workgroups, at least 8 stages each
    int64_t splits = 256 / tiles;
    if (splits < 1) splits = 1;
    const int64_t max_splits = (stages + 7) / 8;
    if (splits > max_splits) splits = max_splits;
    const int64_t sps = (stages + splits - 1) / splits;
    p.kchunk = (int)(sps * DK);
    p.splits = (int)((stages + sps - 1) / sps);
    return p;
}

hipError_t launch_clipped_bf16_dma(const TnPlan& p, const uint16_t* A, const uint16_t* G, const float* clip,
                                   int B, int T, int M, int N, bool accumulate, float* grad, float* ws, hipStream_t st) {
    DmaArgs a;
    a.A = A; a.G = G; a.clip = clip;
    a.B = B; a.T = T; a.M = M; a.N = N;
    a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n; a.splits = p.splits;
    a.stages_total = (int)((int64_t)B * T / DK);
    a.stages_per_split = p.kchunk / DK;
    const int64_t n = (int64_t)M * N;
    const int tiles = p.tiles_m * p.tiles_n;
    a.per_xcd = ceil_div((int64_t)tiles * p.splits, 8);
    if (p.splits == 1) { a.out = grad; a.slice = 0; a.accumulate = accumulate ? 1 : 0; }
    else { a.out = ws; a.slice = splitk_slice_elems(n); a.accumulate = 0; }
    k_tn_bf16_dma<<<8u * (unsigned)a.per_xcd, kThreads, 0, st>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.splits == 1) return e;
    return launch_splitk_reduce(ws, n, p.splits, accumulate, grad, st);
}

}  // namespace dpk
