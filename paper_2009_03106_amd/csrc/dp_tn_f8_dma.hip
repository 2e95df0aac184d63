// Copy-pipeline kernels for aligned layers with 8-bit floating-point inputs (OCP e4m3 and e5m2, one byte per
// element): clipped sum  sum_i c_i A_i^T G_i  and direct squared norm, on the 64-deep 8-bit MFMA
// (v_mfma_f32_32x32x64_f8f6f4: twice the rate of the 16-bit instructions for half the bytes).
//
// Same structure as the 16-bit copy-pipeline kernels:
//   * global -> LDS copies go straight into LDS (global_load_lds_dwordx4, 1 KB per wave instruction: 16 elements per
//     lane), a ring of 64-row stages, all but one of them in flight while one is consumed;
//   * the transpose that the MFMA needs (a lane holds 32 consecutive-in-k bytes of one column, memory has consecutive
//     columns for one k) is done by the LDS read (ds_read_b64_tr_b8: the 16 lanes of a group read 8 rows x 16 bytes,
//     lanes 2 e and 2 e + 1 the two halves of row e, and lane i receives the 8 bytes of column i);
//   * the clip factors are applied to the fp32 accumulators at the example boundaries, so every stage lies inside one
//     example: T % 64 == 0, or the ragged mode, which pads every example with rows of zeros.
// One stage is one k step of the MFMA.  Which k a byte position of the operand registers stands for does not matter
// as long as the A and the G fragment agree; both are read with the same row pattern (lanes 0-31: rows 0-31 of the
// stage, lanes 32-63: rows 32-63, 8 rows per read).
#include "dp_common.h"
#include "dp_internal.h"
#include <type_traits>

namespace dpk {

namespace {

constexpr int DK8 = 64;               // rows of A and of G per stage

typedef int v2i32 __attribute__((ext_vector_type(2)));
typedef int v8i32 __attribute__((ext_vector_type(8)));
#define LDS_PTR(T) __attribute__((address_space(3))) T*

// Tile geometry: WM x WN waves, each owning FM x FN MFMA tiles of 32 x 32; NST stages resident in LDS; OCC
// workgroups per compute unit.
template <int WM_, int WN_, int FM_, int FN_, int NST_, int OCC_>
struct Geo8 {
    static constexpr int WM = WM_, WN = WN_, FM = FM_, FN = FN_, NST = NST_, OCC = OCC_;
    static constexpr int WAVES = WM * WN, THREADS = 64 * WAVES;
    static constexpr int TM = WM * FM * 32, TN = WN * FN * 32;        // output tile
    static constexpr int RBA = TM, RBG = TN;                          // bytes of one stage row of either operand
    static constexpr int IPA = RBA * DK8 / 1024 / WAVES, IPG = RBG * DK8 / 1024 / WAVES;   // 1 KB copies per operand, stage and wave
    static constexpr int LPS = IPA + IPG;                             // copies per stage and wave
    static constexpr int OPA = DK8 * RBA, STAGE_BYTES = DK8 * (RBA + RBG);
    static_assert(IPA * 1024 * WAVES == RBA * DK8 && IPG * 1024 * WAVES == RBG * DK8, "a stage must be a whole number of copies per wave");
    static_assert(NST >= 2 && OCC * NST * STAGE_BYTES <= 160 * 1024, "stages must fit the 160 KB of LDS");
    static_assert(3 * LPS <= 63, "vmcnt range");
};
// 256 x 256 tile, 8 waves of 128 x 64, four 32 KB stages, one workgroup per compute unit
using Geo8L = Geo8<2, 4, 4, 2, 4, 1>;
// 128 x 128 tile, 4 waves of 64 x 64, four 16 KB stages, two workgroups per compute unit
using Geo8T = Geo8<2, 2, 2, 2, 4, 2>;

struct Dma8Args {
    const unsigned char* A;
    const unsigned char* G;
    const float* clip;
    float* out;            // slice base (stride `slice` per K slice) or grad; direct norm: partial[B][tiles]
    int64_t slice;
    int B, T, M, N;
    int tiles_m, tiles_n;
    int splits;
    int stages_total;      // B * ceil(T / DK8)
    int stages_per_split;
    int per_xcd;
    int accumulate;
    const unsigned char* zero;  // ragged mode: at least 16 bytes of zeros
};

// Rows of RB bytes; the 16-byte chunk c of row r sits at chunk position c ^ chunk_swz8<RB>(r).  A transposing read of
// 32 lanes touches 8 consecutive rows x 32 bytes.  Banks repeat every 256 bytes: when RB is a multiple of 256 the 8
// rows start in the same bank and the xor moves them to 8 different 32-byte windows; when RB = 128 mod 256 rows r and
// r + 2 collide and the xor spreads r / 2 over the four windows of a 128-byte half.
template <int RB> __device__ __forceinline__ int chunk_swz8(int r) {
    static_assert(RB % 128 == 0, "row bytes");
    if (RB % 256 == 0) return (r & 7) << 1;         // needs 16 | chunks per row
    return ((r >> 1) & 3) << 1;                     // needs 8 | chunks per row
}

template <int N> __device__ __forceinline__ void wait_vmcnt8() { __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14)); }

// FA, FG: 0 = e4m3, 1 = e5m2 (the format fields of the MFMA).
// MODE 0: clipped sum over a K slice (any range of stages).  MODE 1: direct squared norm: the K slice is one
// example (stages_per_split = ceil(T / DK8), splits = B), no scaling, and the finished tile of A_i^T G_i is squared
// and reduced to one float per (example, tile) instead of being stored (Algorithm 3 / 4 without their output).
// RAG: T is not a multiple of the 64-row stage.  Every example then takes ceil(T / 64) stages, and the rows past
// its end in the last one are copied from the line of zeros (rows of zeros add nothing to the product).
// `L`: the (slice, tile) pair of this workgroup among the layer's tiles * splits
template <class GEO, int MODE, bool RAG, int FA, int FG>
__device__ __forceinline__ void tn_f8_tile(const Dma8Args& a, const int L) {
    constexpr int NST = GEO::NST, FM = GEO::FM, FN = GEO::FN, NF = FM + FN;
    constexpr int RBA = GEO::RBA, RBG = GEO::RBG, IPA = GEO::IPA, IPG = GEO::IPG, LPS = GEO::LPS;
    constexpr int OPA = GEO::OPA, STAGE_BYTES = GEO::STAGE_BYTES;
    static_assert((RBA % 256 == 0 ? (RBA / 16) % 16 : (RBA / 16) % 8) == 0 && (RBG % 256 == 0 ? (RBG / 16) % 16 : (RBG / 16) % 8) == 0, "swizzle range");
    __shared__ __attribute__((aligned(1024))) unsigned char lds[NST * STAGE_BYTES];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tiles = a.tiles_m * a.tiles_n;
    if (L >= tiles * a.splits) return;
    const int z = L / tiles, tile = L - z * tiles;
    // Consecutive items walk the short side of the tile grid first: the workgroups that run at the same time on an
    // XCD then form a block of whole columns (or rows) of tiles, and a run of items that ends inside a slice's tile
    // set leaves few panels of A and G to be fetched a second time by the items behind it.
    int tm, tn;
    if (a.tiles_m < a.tiles_n) { tn = tile / a.tiles_m; tm = tile - tn * a.tiles_m; }
    else { tm = tile / a.tiles_n; tn = tile - tm * a.tiles_n; }
    const int m0 = tm * GEO::TM, n0 = tn * GEO::TN;
    const int s_begin = z * a.stages_per_split;
    const int s_end = min(a.stages_total, s_begin + a.stages_per_split);
    const int n_stages = s_end - s_begin;
    if (n_stages <= 0) return;
    const int spe = (a.T + DK8 - 1) / DK8;          // stages per example (T % 64 != 0 only in the ragged mode)

    // ---- global -> LDS.  The A part of a stage (DK8 rows of RBA bytes) and its G part are each a linear run of
    //      16-byte chunks; copy u of wave w moves chunks 64 (w IP + u) .. + 63, one per lane.
    uint32_t offA[IPA], offG[IPG];
    int rowA[IPA], rowG[IPG];                        // RAG: row inside the stage of each copy's lane
    const int sub_begin = s_begin - (s_begin / spe) * spe;
#pragma unroll
    for (int u = 0; u < IPA; ++u) {
        const int idx = (wave * IPA + u) * 64 + lane;
        const int r = idx / (RBA / 16);                               // row inside the stage
        int col = m0 + (((idx % (RBA / 16)) ^ chunk_swz8<RBA>(r)) << 4);
        if (col >= a.M) col = m0;                   // out-of-range columns only feed output rows that are never stored
        rowA[u] = r;
        offA[u] = (uint32_t)r * (uint32_t)a.M + (uint32_t)col;
    }
#pragma unroll
    for (int u = 0; u < IPG; ++u) {
        const int idx = (wave * IPG + u) * 64 + lane;
        const int r = idx / (RBG / 16);
        int col = n0 + (((idx % (RBG / 16)) ^ chunk_swz8<RBG>(r)) << 4);
        if (col >= a.N) col = n0;
        rowG[u] = r;
        offG[u] = (uint32_t)r * (uint32_t)a.N + (uint32_t)col;
    }
    const size_t stepA = (size_t)DK8 * a.M, stepG = (size_t)DK8 * a.N;  // bytes per stage
    const unsigned char* baseA = RAG ? a.A + (size_t)(s_begin / spe) * a.T * a.M + (size_t)sub_begin * stepA
                                     : a.A + (size_t)s_begin * stepA;                    // uniform
    const unsigned char* baseG = RAG ? a.G + (size_t)(s_begin / spe) * a.T * a.N + (size_t)sub_begin * stepG
                                     : a.G + (size_t)s_begin * stepG;
    int rag_sub = sub_begin;                                          // RAG: stage inside the example of the next copy

    // The copies are inline assembly: the compiler then does not make every LDS read wait for all copies in
    // flight; the waits for them are the explicit vmcnt waits in front of the stage barriers below.
    const uint32_t lds_base = (uint32_t)(uintptr_t)(LDS_PTR(unsigned char))lds;
    const uint32_t wave_ldsA = __builtin_amdgcn_readfirstlane(lds_base + wave * IPA * 1024);
    const uint32_t wave_ldsG = __builtin_amdgcn_readfirstlane(lds_base + OPA + wave * IPG * 1024);
    auto issue = [&](int buf) {
        if (RAG) {
            const int rows_valid = a.T - rag_sub * DK8;               // rows of this stage inside the example (may exceed 64)
#pragma unroll
            for (int u = 0; u < IPA; ++u) {
                const uint64_t addr = rowA[u] < rows_valid ? (uint64_t)(uintptr_t)baseA + offA[u] : (uint64_t)(uintptr_t)a.zero;
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                             :: "s"(wave_ldsA + buf * STAGE_BYTES + u * 1024), "v"(addr) : "memory", "m0");
            }
#pragma unroll
            for (int u = 0; u < IPG; ++u) {
                const uint64_t addr = rowG[u] < rows_valid ? (uint64_t)(uintptr_t)baseG + offG[u] : (uint64_t)(uintptr_t)a.zero;
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                             :: "s"(wave_ldsG + buf * STAGE_BYTES + u * 1024), "v"(addr) : "memory", "m0");
            }
            // the next stage: 64 rows further, or the first rows of the next example (which start T rows after this one's)
            if (++rag_sub == spe) {
                baseA += (size_t)(a.T - (spe - 1) * DK8) * a.M;
                baseG += (size_t)(a.T - (spe - 1) * DK8) * a.N;
                rag_sub = 0;
            } else {
                baseA += stepA;
                baseG += stepG;
            }
            return;
        }
#pragma unroll
        for (int u = 0; u < IPA; ++u)
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :: "s"(wave_ldsA + buf * STAGE_BYTES + u * 1024), "v"(offA[u]), "s"(baseA) : "memory", "m0");
        baseA += stepA;
#pragma unroll
        for (int u = 0; u < IPG; ++u)
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :: "s"(wave_ldsG + buf * STAGE_BYTES + u * 1024), "v"(offG[u]), "s"(baseG) : "memory", "m0");
        baseG += stepG;
    };

    // ---- LDS -> MFMA operands.  Lane l of a 16-lane group: source row (l % 16) / 2, source half l % 2 of the
    //      row's 16 bytes; after the transposing read the lane holds 8 k values of column l % 16.
    const int wm = wave / GEO::WN, wn = wave % GEO::WN;
    const int g16 = lane >> 4, s16 = lane & 15;
    const int half = g16 >> 1;                      // lanes 32..63 hold rows 32 .. 63 of the stage
    const int rsrc = 32 * half + (s16 >> 1);        // row of the first read (read x: + 8 x)
    uint32_t rd[NF];                                // 0 .. FM-1: A fragments, FM ..: G fragments
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int ma = (wm * FM + i) * 32 + 16 * (g16 & 1) + 8 * (s16 & 1);     // column (byte) of the 8-byte piece
        rd[i] = rsrc * RBA + ((((ma >> 4) ^ chunk_swz8<RBA>(rsrc)) << 4) | (ma & 15));
    }
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const int na = (wn * FN + j) * 32 + 16 * (g16 & 1) + 8 * (s16 & 1);
        rd[FM + j] = OPA + rsrc * RBG + ((((na >> 4) ^ chunk_swz8<RBG>(rsrc)) << 4) | (na & 15));
    }

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    int ex = s_begin / spe;
    int sub = s_begin - ex * spe;
    // The clip factors of the examples this workgroup walks through are kept one per lane in a register
    // (loaded before the copies start) and picked with v_readlane.
    const int ex0 = ex;                             // a K slice spans at most 64 examples (see the plan)
    float vclip = 1.0f;
    if (MODE == 0) vclip = a.clip[min(ex0 + lane, a.B - 1)];
    float c_cur = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, vclip), 0));
    bool skip = false;                              // the current example is left out (zero factor, see below)
    float c_ref = c_cur;                            // the largest factor accumulated so far

    // prologue: all NST buffers are free, fill them
#pragma unroll
    for (int p = 0; p < NST; ++p)
        if (p < n_stages) issue(p);

    // rows 8 x .. 8 x + 7 of this lane half's 32 rows come with read x; the swizzle of a row depends on r % 8 only,
    // so the four reads differ by whole rows
    auto read_stage = [&](v8i32 (&f)[NF], uint32_t sb) {
        LDS_PTR(unsigned char) b = (LDS_PTR(unsigned char))lds + sb;
#pragma unroll
        for (int x = 0; x < NF; ++x) {
            const int rb = x < FM ? RBA : RBG;
            v2i32 q[4];
#pragma unroll
            for (int y = 0; y < 4; ++y) q[y] = __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_PTR(v2i32))(b + rd[x] + y * 8 * rb));
            f[x] = v8i32{q[0][0], q[0][1], q[1][0], q[1][1], q[2][0], q[2][1], q[3][0], q[3][1]};
        }
    };
    auto mfma_stage = [&](const v8i32 (&f)[NF]) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(f[i], f[FM + j], acc[i][j], FA, FG, 0, 0, 0, 0);
    };
    // stage s (relative) landed once at most `ahead` later stages' copies are outstanding
    auto wait_stage = [&](int ahead) {
        if (NST >= 4 && ahead >= 3) wait_vmcnt8<3 * LPS>();
        else if (NST >= 3 && ahead == 2) wait_vmcnt8<2 * LPS>();
        else if (ahead == 1) wait_vmcnt8<LPS>();
        else wait_vmcnt8<0>();
    };

    wait_stage(min(n_stages - 1, NST - 1));
    __builtin_amdgcn_s_barrier();
    v8i32 f[2][NF];                                 // fragments of the current / next stage
    read_stage(f[0], 0u);

    // One stage: its fragments were requested while the stage before it was multiplied.  The barrier that makes
    // stage st + 1 visible sits in front of the MFMAs of stage st, so that the reads of stage st + 1 are in flight
    // under them; behind it the buffer of stage st (all reads retired) takes the copies of stage st + NST.
    auto step = [&](int st, auto cur_tag) {
        constexpr int CUR = decltype(cur_tag)::value;
        if (MODE == 0 && sub == spe) {
            // first stage of the next example: rescale the running tile
            sub = 0;
            ++ex;
            const float c_next = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, vclip), ex - ex0));
            const float ratio = c_cur / c_next;
            // a zero factor, or one below 2^-40 of the largest so far (the tile in that unit would leave the float32
            // range), after a non-zero one cannot become the tile's unit: the example's MFMAs are skipped and the unit
            // stays, i.e. it counts with factor 0
            skip = __builtin_isinf(ratio) || c_next < c_ref * 0x1p-40f;
            if (c_next != c_cur && !skip) {
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[i][j][r] *= ratio;
            }
            if (!skip) { c_cur = c_next; c_ref = fmaxf(c_ref, c_next); }
        }
        ++sub;
        __builtin_amdgcn_s_waitcnt(0xC07F);                                              // lgkmcnt(0): this stage's fragments
        if (st + 1 < n_stages) {
            // stage st + 1 must have landed (later stages may stay in flight), for every wave; every wave has
            // also retired its reads of stage st, so that buffer can take stage st + NST
            wait_stage(min(n_stages - 2 - st, NST - 2));
            __builtin_amdgcn_s_barrier();
            if (st + NST < n_stages) issue(st % NST);
            read_stage(f[CUR ^ 1], (uint32_t)((st + 1) % NST) * STAGE_BYTES);
        }
        if (MODE != 0 || !skip) mfma_stage(f[CUR]);
        __builtin_amdgcn_sched_barrier(0);
    };
    for (int st = 0; st < n_stages; st += 2) {
        step(st, std::integral_constant<int, 0>{});
        if (st + 1 < n_stages) step(st + 1, std::integral_constant<int, 1>{});
    }

    const int lrow = lane & 31, lhalf = lane >> 5;
    if (MODE == 1) {
        // sum of squares over the valid part of the tile (columns / rows beyond d_out / d_in hold clamped copies)
        float sq = 0.f;
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int n = n0 + (wn * FN + j) * 32 + lrow;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = m0 + (wm * FM + i) * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
                    const float v = acc[i][j][r];
                    sq += (m < a.M && n < a.N) ? v * v : 0.f;
                }
            }
        sq = wave_sum(sq);
        __syncthreads();                            // every wave is done with the stage buffers: reuse them for the reduction
        float* red = reinterpret_cast<float*>(lds);
        if (lane == 0) red[wave] = sq;
        __syncthreads();
        if (tid == 0) {
            float t = 0.f;
#pragma unroll
            for (int w = 0; w < GEO::WAVES; ++w) t += red[w];
            a.out[(size_t)z * tiles + tile] = t;
        }
        return;
    }
    // the tile holds (1 / c_cur) * sum: finish with the last example's factor
    float* out = a.out + (size_t)z * a.slice;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int n = n0 + (wn * FN + j) * 32 + lrow;
            if (n >= a.N) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + (wm * FM + i) * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
                if (m < a.M) {
                    float* p = out + (size_t)m * a.N + n;
                    const float v = acc[i][j][r] * c_cur;
                    *p = a.accumulate ? *p + v : v;
                }
            }
        }
}


template <class GEO, int MODE, bool RAG, int FA, int FG>
__global__ __launch_bounds__(GEO::THREADS, GEO::OCC) void k_tn_f8_dma(Dma8Args a) {
    // workgroup b runs on XCD b % 8: give each XCD a contiguous run of (slice, tile) pairs so that
    // its workgroups stream the same rows of A and G through one L2
    tn_f8_tile<GEO, MODE, RAG, FA, FG>(a, (blockIdx.x & 7) * a.per_xcd + (blockIdx.x >> 3));
}

// Several layers' clipped sums in one launch (256 x 256 tiles, T a multiple of 64), as for the 16-bit inputs: a list
// of (layer, K slice, tile) items, all layers' slices of about one length, filling the chip a whole number of times.
struct Joint8Layer {
    const unsigned char* A; const unsigned char* G; const float* clip;
    float* slices;       // the layer's K slices; the gradient itself where one slice is the whole sum (then `accumulate` applies)
    int T, M, N, tiles_m, tiles_n, splits, stages_total, stages_per_split, first_item, accumulate;
};
struct Joint8Args {
    Joint8Layer layer[kJointLayers];
    int n_layers, n_items, per_xcd, B;
};
template <int FA, int FG>
__global__ __launch_bounds__(Geo8L::THREADS, Geo8L::OCC) void k_tn_f8_dma_joint(Joint8Args j) {
    const int L = (blockIdx.x & 7) * j.per_xcd + (blockIdx.x >> 3);
    if (L >= j.n_items) return;
    int l = 0;
    while (l + 1 < j.n_layers && L >= j.layer[l + 1].first_item) ++l;
    const Joint8Layer& y = j.layer[l];
    Dma8Args a;
    a.A = y.A; a.G = y.G; a.clip = y.clip;
    a.out = y.slices; a.slice = (((int64_t)y.M * y.N) + 3) & ~(int64_t)3;        // splitk_slice_elems
    a.B = j.B; a.T = y.T; a.M = y.M; a.N = y.N;
    a.tiles_m = y.tiles_m; a.tiles_n = y.tiles_n; a.splits = y.splits;
    a.stages_total = y.stages_total; a.stages_per_split = y.stages_per_split;
    a.per_xcd = 0; a.accumulate = y.accumulate; a.zero = nullptr;
    tn_f8_tile<Geo8L, 0, false, FA, FG>(a, L - y.first_item);
}

// 0: not for this kernel; 1: Geo8L; 2: Geo8T
int dma8_geometry(int T, int M, int N) {
    if (((M | N) & 15) != 0) return 0;
    if ((T % DK8) != 0 && (int64_t)ceil_div(T, DK8) * DK8 * 4 > (int64_t)T * 5) return 0;   // ragged T: at most a quarter of zero rows
    if ((int64_t)DK8 * (M > N ? M : N) >= (int64_t(1) << 31)) return 0;           // 32-bit lane offsets inside a stage
    if (tiles_fit(M, N, Geo8L::TM, Geo8L::TN)) return 1;
    if (tiles_fit(M, N, Geo8T::TM, Geo8T::TN)) return 2;
    return 0;
}

struct Geo8Dims { int tm, tn, occ; };
Geo8Dims geo8_dims(int id) {
    if (id == 1) return {Geo8L::TM, Geo8L::TN, Geo8L::OCC};
    return {Geo8T::TM, Geo8T::TN, Geo8T::OCC};
}
// the first geometry that fits (largest tile) unless it leaves most of the chip idle: a launch of fewer than 128
// workgroups gives way to the geometry with the most workgroups.  `units` = what multiplies the tile count:
// K slices available (clipped sum) or examples (direct norm).
int pick_geometry8(int T, int M, int N, int64_t units) {
    const int first = dma8_geometry(T, M, N);
    if (first == 0) return 0;
    int best = first;
    int64_t best_blocks = -1;
    for (int id = first; id <= 2; ++id) {
        const Geo8Dims g = geo8_dims(id);
        if (!tiles_fit(M, N, g.tm, g.tn)) continue;
        const int64_t tiles = (int64_t)ceil_div(M, g.tm) * ceil_div(N, g.tn);
        int64_t per_tile = 256 * g.occ / tiles;
        if (per_tile < 1) per_tile = 1;
        const int64_t blocks = tiles * (units < per_tile ? units : per_tile);
        if (id == first && blocks >= 128) return first;
        if (blocks > best_blocks) { best_blocks = blocks; best = id; }
    }
    return best;
}

template <class GEO, int MODE, int FA, int FG> hipError_t launch_rag8(const Dma8Args& a, bool rag, hipStream_t st) {
    if (rag) k_tn_f8_dma<GEO, MODE, true, FA, FG><<<8u * (unsigned)a.per_xcd, GEO::THREADS, 0, st>>>(a);
    else     k_tn_f8_dma<GEO, MODE, false, FA, FG><<<8u * (unsigned)a.per_xcd, GEO::THREADS, 0, st>>>(a);
    return hipGetLastError();
}
template <class GEO, int MODE> hipError_t launch_fmt8(const Dma8Args& a, bool rag, int fmt, hipStream_t st) {
    if (fmt == 2) return launch_rag8<GEO, MODE, 0, 0>(a, rag, st);
    if (fmt == 3) return launch_rag8<GEO, MODE, 1, 1>(a, rag, st);
    if (fmt == 4) return launch_rag8<GEO, MODE, 0, 1>(a, rag, st);
    return hipErrorInvalidValue;
}
template <int MODE> hipError_t launch_any8(bool big, const Dma8Args& a, bool rag, int fmt, hipStream_t st) {
    return big ? launch_fmt8<Geo8L, MODE>(a, rag, fmt, st) : launch_fmt8<Geo8T, MODE>(a, rag, fmt, st);
}

}  // namespace

bool dma8_clipped_ok(int T, int M, int N) { return dma8_geometry(T, M, N) != 0; }
bool dma8_direct_ok(int T, int M, int N) { return T >= 64 && dma8_geometry(T, M, N) != 0; }

TnPlan plan_clipped_f8_dma(int B, int T, int M, int N) {
    const int64_t spe = ceil_div(T, DK8);
    const int64_t stages = (int64_t)B * spe;
    const Geo8Dims gd = geo8_dims(pick_geometry8(T, M, N, (stages + 3) / 4));
    TnPlan p;
    p.tile_m = gd.tm; p.tile_n = gd.tn;
    p.tiles_m = ceil_div(M, p.tile_m); p.tiles_n = ceil_div(N, p.tile_n);
    p.segmented = false; p.epu = 0; p.big = gd.tm == Geo8L::TM; p.dma = true;
    p.zero_head = (T % DK8) != 0;
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    // fill the chip once (256 compute units x workgroups per unit) with K slices of at least 4 stages (256 rows) each
    int64_t splits = 256 * gd.occ / tiles;
    if (splits < 1) splits = 1;
    const int64_t max_splits = (stages + 3) / 4;
    if (splits > max_splits) splits = max_splits;
    int64_t sps = (stages + splits - 1) / splits;
    if (sps > 63 * spe) sps = 63 * spe;               // a slice may touch at most 64 examples (one clip factor per lane)
    p.kchunk = (int)(sps * DK8);
    p.splits = (int)((stages + sps - 1) / sps);
    return p;
}

hipError_t launch_clipped_f8_dma(const TnPlan& p, const void* A, const void* G, const float* clip,
                                 int B, int T, int M, int N, bool accumulate, float* grad, float* ws, hipStream_t st,
                                 int fmt, const NoiseArgs* noise) {
    Dma8Args a;
    a.zero = nullptr;
    if (p.zero_head) {
        // ragged T: the head of the workspace is the line of zeros
        a.zero = static_cast<const unsigned char*>(device_zero_line(st));
        if (!a.zero) {
            const hipError_t ez = launch_fill_zero(ws, kZeroHeadFloats, st);
            if (ez != hipSuccess) return ez;
            a.zero = reinterpret_cast<const unsigned char*>(ws);
        }
        ws += kZeroHeadFloats;
    }
    a.A = static_cast<const unsigned char*>(A); a.G = static_cast<const unsigned char*>(G); a.clip = clip;
    a.B = B; a.T = T; a.M = M; a.N = N;
    a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n; a.splits = p.splits;
    a.stages_total = (int)((int64_t)B * ceil_div(T, DK8));
    a.stages_per_split = p.kchunk / DK8;
    const int64_t n = (int64_t)M * N;
    const int tiles = p.tiles_m * p.tiles_n;
    a.per_xcd = ceil_div((int64_t)tiles * p.splits, 8);
    if (p.splits == 1) { a.out = grad; a.slice = 0; a.accumulate = accumulate ? 1 : 0; }
    else { a.out = ws; a.slice = splitk_slice_elems(n); a.accumulate = 0; }
    const hipError_t e = launch_any8<0>(p.big, a, p.zero_head, fmt, st);
    if (e != hipSuccess || p.splits == 1) return e;
    return launch_splitk_reduce(ws, n, p.splits, accumulate, grad, st, noise);
}

// ---- joint launch of several layers' clipped sums
bool dma8_joint_ok(int T, int M, int N) { return T > 0 && (T % DK8) == 0 && dma8_geometry(T, M, N) == 1; }

size_t joint8_workspace_floats(const JointShape* sh, int n_layers, int B) {
    const JointPlan p = plan_joint(sh, n_layers, B, DK8, Geo8L::TM);
    size_t slices = 0;
    for (int l = 0; l < n_layers; ++l) slices += (size_t)p.splits[l] * (size_t)splitk_slice_elems((int64_t)sh[l].M * sh[l].N);
    return slices;
}

hipError_t launch_clipped_f8_dma_joint(const JointShape* sh, const JointOperands* op, int n_layers, int B, bool accumulate,
                                       float stddev, uint64_t seed, float* ws, hipStream_t st, int fmt) {
    if (n_layers < 1 || n_layers > kJointLayers) return hipErrorInvalidValue;
    const JointPlan p = plan_joint(sh, n_layers, B, DK8, Geo8L::TM);
    if (p.items >= (int64_t(1) << 28)) return hipErrorInvalidValue;
    Joint8Args j;
    float* slices = ws;
    int64_t first = 0;
    for (int l = 0; l < n_layers; ++l) {
        Joint8Layer& y = j.layer[l];
        y.A = reinterpret_cast<const unsigned char*>(op[l].A); y.G = reinterpret_cast<const unsigned char*>(op[l].G); y.clip = op[l].clip;
        // one slice and no noise to add: the launch writes the gradient itself, nothing to fold
        const bool whole = p.splits[l] == 1 && stddev == 0.0f;
        y.slices = whole ? op[l].grad : slices;
        y.accumulate = whole && accumulate ? 1 : 0;
        y.T = sh[l].T; y.M = sh[l].M; y.N = sh[l].N;
        y.tiles_m = p.tiles_m[l]; y.tiles_n = p.tiles_n[l]; y.splits = p.splits[l];
        y.stages_total = (int)((int64_t)B * (sh[l].T / DK8)); y.stages_per_split = p.sps[l];
        y.first_item = (int)first;
        first += (int64_t)p.tiles_m[l] * p.tiles_n[l] * p.splits[l];
        slices += (size_t)p.splits[l] * (size_t)splitk_slice_elems((int64_t)sh[l].M * sh[l].N);
    }
    for (int l = n_layers; l < kJointLayers; ++l) j.layer[l] = j.layer[0];
    j.n_layers = n_layers; j.n_items = (int)p.items; j.per_xcd = ceil_div(p.items, 8);
    j.B = B;
    const unsigned grid = 8u * (unsigned)j.per_xcd;
    if (fmt == 2)      k_tn_f8_dma_joint<0, 0><<<grid, Geo8L::THREADS, 0, st>>>(j);
    else if (fmt == 3) k_tn_f8_dma_joint<1, 1><<<grid, Geo8L::THREADS, 0, st>>>(j);
    else if (fmt == 4) k_tn_f8_dma_joint<0, 1><<<grid, Geo8L::THREADS, 0, st>>>(j);
    else return hipErrorInvalidValue;
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // one launch folds the slices of all layers (+ noise)
    FoldLayers f;
    int nf = 0;
    for (int l = 0; l < n_layers; ++l) {
        if (j.layer[l].slices == op[l].grad) continue;                 // written by the launch itself
        f.ws[nf] = j.layer[l].slices; f.grad[nf] = op[l].grad; f.n[nf] = (int64_t)sh[l].M * sh[l].N;
        f.splits[nf] = p.splits[l]; f.noise_offset[nf] = op[l].noise_offset;
        ++nf;
    }
    if (nf == 0) return hipSuccess;
    f.n_layers = nf;
    for (int l = nf; l < kJointLayers; ++l) { f.ws[l] = f.ws[0]; f.grad[l] = f.grad[0]; f.n[l] = 0; f.splits[l] = 0; f.noise_offset[l] = 0; }
    return launch_splitk_reduce_layers(f, accumulate, st, stddev, seed);
}

TnPlan plan_direct_f8_dma(int B, int T, int M, int N) {
    const Geo8Dims gd = geo8_dims(pick_geometry8(T, M, N, B));      // one workgroup per (example, tile)
    TnPlan p;
    p.tile_m = gd.tm; p.tile_n = gd.tn;
    p.tiles_m = ceil_div(M, p.tile_m); p.tiles_n = ceil_div(N, p.tile_n);
    p.segmented = false; p.big = gd.tm == Geo8L::TM; p.dma = true;
    p.zero_head = (T % DK8) != 0;
    p.splits = 1; p.kchunk = 0; p.epu = 1;
    return p;
}

hipError_t launch_direct_f8_dma(const TnPlan& p, const void* A, const void* G, int B, int T, int M, int N,
                                bool accumulate, float* sqnorm, float* partial, hipStream_t st, int fmt, const ClipOut* co) {
    Dma8Args a;
    a.zero = nullptr;
    if (p.zero_head) {
        a.zero = static_cast<const unsigned char*>(device_zero_line(st));
        if (!a.zero) {
            const hipError_t ez = launch_fill_zero(partial, kZeroHeadFloats, st);
            if (ez != hipSuccess) return ez;
            a.zero = reinterpret_cast<const unsigned char*>(partial);
        }
        partial += kZeroHeadFloats;
    }
    a.A = static_cast<const unsigned char*>(A); a.G = static_cast<const unsigned char*>(G); a.clip = nullptr;
    a.B = B; a.T = T; a.M = M; a.N = N;
    a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n;
    a.splits = B;
    a.stages_total = (int)((int64_t)B * ceil_div(T, DK8));
    a.stages_per_split = ceil_div(T, DK8);
    a.out = partial; a.slice = 0; a.accumulate = 0;
    const int tiles = a.tiles_m * a.tiles_n;
    const int64_t total = (int64_t)tiles * B;
    if (total >= (int64_t(1) << 28)) return hipErrorInvalidValue;
    a.per_xcd = ceil_div(total, 8);
    const hipError_t e = launch_any8<1>(p.big, a, p.zero_head, fmt, st);
    if (e != hipSuccess) return e;
    return launch_finalize_partials(partial, B, tiles, accumulate, sqnorm, st, co);
}

}  // namespace dpk
