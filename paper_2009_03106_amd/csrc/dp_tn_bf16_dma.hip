// Large-tile bf16 clipped sum  sum_i c_i A_i^T G_i  for big aligned layers.
//
// gfx950-specific data path with (almost) no VALU work in the main loop:
//   * global -> LDS copies go straight into LDS (global_load_lds_dwordx4): a
//     wave instruction moves 1 KB of a K-major tile, as it lies in memory
//     (two 512-byte rows of A or four 256-byte rows of G).  Three 32-row
//     stages are kept in LDS, two of them in flight while one is consumed.
//   * the 16-bit transpose the MFMA needs (a lane must hold consecutive k for
//     one column, memory has consecutive columns for one k) is done by the
//     LDS read itself (ds_read_b64_tr_b16): 16 lanes read a 4(k) x 16(col)
//     patch and each lane gets the 4 k values of one column.
//   * 256 x 128 output tile per workgroup (4 waves, 128 x 64 each = 128
//     accumulator registers), two workgroups per compute unit so that one
//     can compute while the other waits at its stage barrier.
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

constexpr int DM = 256, DN = 128;     // output tile
constexpr int DK = 32;                // rows per stage
constexpr int NST = 3;                // stages resident in LDS
constexpr int A_BYTES = DK * DM * 2;             // 16 KB, rows of 512 B
constexpr int G_BYTES = DK * DN * 2;             //  8 KB, rows of 256 B
constexpr int STAGE_BYTES = A_BYTES + G_BYTES;   // 24 KB
constexpr int LOADS_PER_STAGE = 6;               // per wave: 4 of A, 2 of G

typedef short v4i16 __attribute__((ext_vector_type(4)));
#define LDS_PTR(T) __attribute__((address_space(3))) T*
#define GLB_PTR(T) const __attribute__((address_space(1))) T*
#define TR_READ(dst, addr, off) asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "i"(off))

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

__global__ __launch_bounds__(kThreads, 2) void k_tn_bf16_dma(DmaArgs a) {
    __shared__ __attribute__((aligned(1024))) unsigned char lds[NST * STAGE_BYTES];   // 72 KB

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tiles = a.tiles_m * a.tiles_n;
    // workgroup b runs on XCD b % 8: give each XCD a contiguous run of (slice, tile) pairs so that
    // its workgroups stream the same rows of A and G through one L2
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

    // ---- global -> LDS.  Wave w copies rows 8w..8w+7 of a stage.
    //   A: 4 instructions, instruction u covers rows 8w+2u, 8w+2u+1 (lane / 32 picks the row, lane % 32 the chunk)
    //   G: 2 instructions, instruction u covers rows 8w+4u .. 8w+4u+3 (lane / 16 picks the row, lane % 16 the chunk)
    int offA[2];                                    // element offset of this lane's source chunk for u even / odd
#pragma unroll
    for (int par = 0; par < 2; ++par) {
        const int r = 2 * par + (lane >> 5);        // r & 3 of the row this lane fills
        int ca = m0 + ((lane & 31) ^ chunk_swz(r)) * 8;
        if (ca >= a.M) ca = m0;                     // out-of-range columns only feed output rows that are never stored
        offA[par] = ca;
    }
    int offG = n0 + ((lane & 15) ^ chunk_swz(lane >> 4)) * 8;
    if (offG >= a.N) offG = n0;
    const uint16_t* pA = a.A + ((size_t)s_begin * DK + wave * 8 + (lane >> 5)) * a.M;
    const uint16_t* pG = a.G + ((size_t)s_begin * DK + wave * 8 + (lane >> 4)) * a.N + offG;
    const size_t stepA = (size_t)DK * a.M, stepG = (size_t)DK * a.N;            // per stage
    const size_t row2A = (size_t)2 * a.M, row4G = (size_t)4 * a.N;              // per instruction

    auto issue = [&](int buf) {
        LDS_PTR(unsigned char) base = (LDS_PTR(unsigned char))lds + buf * STAGE_BYTES;
#pragma unroll
        for (int u = 0; u < 4; ++u)
            __builtin_amdgcn_global_load_lds((GLB_PTR(void))(pA + u * row2A + offA[u & 1]),
                                             (LDS_PTR(void))(base + wave * 4096 + u * 1024), 16, 0, 0);
#pragma unroll
        for (int u = 0; u < 2; ++u)
            __builtin_amdgcn_global_load_lds((GLB_PTR(void))(pG + u * row4G),
                                             (LDS_PTR(void))(base + A_BYTES + wave * 2048 + u * 1024), 16, 0, 0);
        pA += stepA;
        pG += stepG;
    };

    // ---- LDS -> MFMA operands.  Lane l of a 16-lane group: source row j = (l % 16) / 4, source column
    //      piece q = l % 4; after the transposing read the lane holds 4 k values of column l % 16.
    const int wm = wave >> 1, wn = wave & 1;
    const int g16 = lane >> 4, s16 = lane & 15;
    const int half = g16 >> 1;                      // lanes 32..63 hold k + 8 .. k + 15 of a 16-wide k step
    const int rsrc = 8 * half + (s16 >> 2);         // row inside the k step for the first read (second read: + 4)
    const uint32_t lds_base = (uint32_t)(uintptr_t)(LDS_PTR(unsigned char))lds;
    uint32_t rdA[4], rdG[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int ma = wm * 128 + i * 32 + 16 * (g16 & 1) + 4 * (s16 & 3);      // column (element) of the 8-byte piece
        rdA[i] = lds_base + rsrc * 512 + ((((ma >> 3) ^ chunk_swz(rsrc)) << 4) | ((ma & 7) << 1));
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int na = wn * 64 + j * 32 + 16 * (g16 & 1) + 4 * (s16 & 3);
        rdG[j] = lds_base + A_BYTES + rsrc * 256 + ((((na >> 3) ^ chunk_swz(rsrc)) << 4) | ((na & 7) << 1));
    }

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // prologue: NST - 1 stages in flight
#pragma unroll
    for (int p = 0; p < NST - 1; ++p)
        if (p < n_stages) issue(p);

    int ex = s_begin / spe;
    int sub = s_begin - ex * spe;
    // clip factors are read with scalar loads (constant address space, uniform index): a vector load here
    // would tie every later vmcnt wait to the copies in flight
    const __attribute__((address_space(4))) float* clip_s = (const __attribute__((address_space(4))) float*)a.clip;
    float c_cur = clip_s[ex];

    for (int st = 0; st < n_stages; ++st) {
        // stage st must have landed; the copies of the next stage may stay in flight
        if (st + 1 < n_stages) __builtin_amdgcn_s_waitcnt(0x0F70 | LOADS_PER_STAGE);     // vmcnt(6)
        else __builtin_amdgcn_s_waitcnt(0x0F70);                                         // vmcnt(0)
        __builtin_amdgcn_s_barrier();
        if (st + NST - 1 < n_stages) issue((st + NST - 1) % NST);

        if (sub == spe) {
            // first stage of the next example: rescale the running tile
            sub = 0;
            ++ex;
            const float c_next = clip_s[ex];
            if (c_next != c_cur) {
                const float ratio = c_cur / c_next;
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[i][j][r] *= ratio;
            }
            c_cur = c_next;
        }
        ++sub;

        const uint32_t sb = (uint32_t)(st % NST) * STAGE_BYTES;
        uint32_t adA[4], adG[2];
#pragma unroll
        for (int i = 0; i < 4; ++i) adA[i] = sb + rdA[i];
#pragma unroll
        for (int j = 0; j < 2; ++j) adG[j] = sb + rdG[j];
        // The transposing reads are issued as inline assembly so that they are ordered by the explicit
        // lgkmcnt waits below and are not tied to the completion of the copies still in flight.
        // k step ks covers rows 16 ks .. 16 ks + 15 of the stage (A rows are 512 B, G rows 256 B apart).
        v4i16 lo[2][6], hi[2][6];
#pragma unroll
        for (int i = 0; i < 4; ++i) { TR_READ(lo[0][i], adA[i], 0); TR_READ(hi[0][i], adA[i], 4 * 512); }
#pragma unroll
        for (int j = 0; j < 2; ++j) { TR_READ(lo[0][4 + j], adG[j], 0); TR_READ(hi[0][4 + j], adG[j], 4 * 256); }
#pragma unroll
        for (int i = 0; i < 4; ++i) { TR_READ(lo[1][i], adA[i], 16 * 512); TR_READ(hi[1][i], adA[i], 20 * 512); }
#pragma unroll
        for (int j = 0; j < 2; ++j) { TR_READ(lo[1][4 + j], adG[j], 16 * 256); TR_READ(hi[1][4 + j], adG[j], 20 * 256); }
        // LDS reads return in order: 24 issued, the first 12 are back once at most 12 are outstanding
        asm volatile("s_waitcnt lgkmcnt(12)" : "+v"(lo[0][0]), "+v"(hi[0][0]), "+v"(lo[0][1]), "+v"(hi[0][1]),
                     "+v"(lo[0][2]), "+v"(hi[0][2]), "+v"(lo[0][3]), "+v"(hi[0][3]), "+v"(lo[0][4]), "+v"(hi[0][4]),
                     "+v"(lo[0][5]), "+v"(hi[0][5]));
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            if (ks == 1)
                asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(lo[1][0]), "+v"(hi[1][0]), "+v"(lo[1][1]), "+v"(hi[1][1]),
                             "+v"(lo[1][2]), "+v"(hi[1][2]), "+v"(lo[1][3]), "+v"(hi[1][3]), "+v"(lo[1][4]), "+v"(hi[1][4]),
                             "+v"(lo[1][5]), "+v"(hi[1][5]));
            bf16x8 f[6];
#pragma unroll
            for (int x = 0; x < 6; ++x)
                f[x] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo[ks][x], hi[ks][x], 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i], f[4 + j], acc[i][j], 0, 0, 0);
        }
    }

    // the tile holds (1 / c_cur) * sum: finish with the last example's factor
    float* out = a.out + (size_t)z * a.slice;
    const int lrow = lane & 31, lhalf = lane >> 5;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + wn * 64 + j * 32 + lrow;
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
    // two workgroups per compute unit: as many K slices as fit into 512 workgroups, at least 8 stages each
    int64_t splits = 512 / tiles;
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
