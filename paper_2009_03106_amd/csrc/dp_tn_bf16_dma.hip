// Large-tile bf16 clipped sum  sum_i c_i A_i^T G_i  for big aligned layers.
//
// gfx950-specific data path with (almost) no VALU work in the main loop:
//   * global -> LDS copies go straight into LDS (global_load_lds_dwordx4): a
//     wave instruction moves 1 KB of a K-major tile, as it lies in memory
//     (two 512-byte rows).  Four 32-row stages are kept in LDS, three of them
//     in flight while one is consumed.
//   * the 16-bit transpose the MFMA needs (a lane must hold consecutive k for
//     one column, memory has consecutive columns for one k) is done by the
//     LDS read itself (ds_read_b64_tr_b16): 16 lanes read a 4(k) x 16(col)
//     patch and each lane gets the 4 k values of one column.
//   * 256 x 256 output tile per workgroup of 8 waves (128 x 64 each = 128
//     accumulator registers, two waves per SIMD), one workgroup per compute
//     unit.  The tile size is set by the L2: at 256 x 128 the kernel ran into
//     the ~10 TB/s the L2s deliver to the compute units (85 flop per byte);
//     256 x 256 needs 128 flop per byte.
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
constexpr int DTHREADS = 512;         // 8 waves: 2 (M) x 4 (N)
constexpr int ROW_BYTES = 512;        // one tile row of either operand in LDS

typedef short v4i16 __attribute__((ext_vector_type(4)));
#define LDS_PTR(T) __attribute__((address_space(3))) T*

struct DmaArgs {
    const uint16_t* A;
    const uint16_t* G;
    const float* clip;
    float* out;            // slice base (stride `slice` per K slice) or grad
    int64_t slice;
    int B, T, M, N;
    int tiles_m, tiles_n;
    int splits;
    int stages_total;      // B*T / DK
    int stages_per_split;
    int per_xcd;
    int accumulate;
};

// 16-byte chunk c of tile row r sits at chunk position c ^ ((r & 3) << 2).  A transposing read of 32
// lanes touches 4 rows x two 32-byte pieces (columns m .. m+15 and m+16 .. m+31); rows are 512 B apart, so
// without the xor all of them would start in the same bank.  With it the 8 pieces cover 256 consecutive
// bytes modulo the bank period and the read is conflict free.
__device__ __forceinline__ int chunk_swz(int r) { return (r & 3) << 2; }

template <int N> __device__ __forceinline__ void wait_vmcnt() { __builtin_amdgcn_s_waitcnt(0x0F70 | N); }

// DK rows per stage, NST stages resident in LDS (DK * NST * 1 KB <= 128 KB).
// MODE 0: clipped sum over a K slice (any range of stages).  MODE 1: direct squared norm: the K slice is one
// example (stages_per_split = T / DK, splits = B), no scaling, and the finished tile of A_i^T G_i is squared
// and reduced to one float per (example, tile) instead of being stored (Algorithm 3 / 4 without their output).
template <int DK, int NST, int MODE>
__global__ __launch_bounds__(DTHREADS, 1) void k_tn_bf16_dma(DmaArgs a) {
    constexpr int OPND_BYTES = DK * ROW_BYTES;       // one operand of one stage
    constexpr int STAGE_BYTES = 2 * OPND_BYTES;      // A part then G part
    constexpr int KS = DK / 16;                      // k steps per stage
    constexpr int IPO = DK / 16;                     // copy instructions per operand, stage and wave (2 rows each)
    constexpr int LPS = 2 * IPO;                     // copies per stage and wave
    static_assert(KS % 2 == 0 && NST >= 2 && NST * STAGE_BYTES <= 131072, "stage geometry");
    __shared__ __attribute__((aligned(1024))) unsigned char lds[NST * STAGE_BYTES];

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

    // ---- global -> LDS.  Wave w copies rows (DK/8) w .. of the A part and of the G part of a stage, two rows
    //      per instruction (lane / 32 picks the row, lane % 32 the chunk position).  Addresses are a uniform
    //      64-bit stage base (SGPR) plus a 32-bit per-lane byte offset that never changes.
    uint32_t offA[IPO], offG[IPO];
#pragma unroll
    for (int u = 0; u < IPO; ++u) {
        const int r = wave * (DK / 8) + 2 * u + (lane >> 5);          // row inside the stage
        const int c = (lane & 31) ^ chunk_swz(r);
        int ca = m0 + c * 8, cn = n0 + c * 8;
        if (ca >= a.M) ca = m0;                     // out-of-range columns only feed output rows / columns that are never stored
        if (cn >= a.N) cn = n0;
        offA[u] = ((uint32_t)r * (uint32_t)a.M + (uint32_t)ca) * 2u;
        offG[u] = ((uint32_t)r * (uint32_t)a.N + (uint32_t)cn) * 2u;
    }
    const uint16_t* baseA = a.A + (size_t)s_begin * DK * a.M;         // uniform
    const uint16_t* baseG = a.G + (size_t)s_begin * DK * a.N;
    const size_t stepA = (size_t)DK * a.M, stepG = (size_t)DK * a.N;  // per stage

    // The copies are issued as inline assembly: the compiler then does not know that they write LDS and
    // does not make every LDS read wait for all copies in flight; the waits for them are the explicit
    // vmcnt waits in front of the stage barriers below.
    const uint32_t lds_base = (uint32_t)(uintptr_t)(LDS_PTR(unsigned char))lds;
    const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(lds_base + wave * (DK / 8) * ROW_BYTES);
    auto issue = [&](int buf) {
#if defined(DPK_EXP) && DPK_EXP == 2
        (void)buf; return;                          // scratch timing experiment: no copies at all
#endif
        const uint32_t base = wave_lds + buf * STAGE_BYTES;
#pragma unroll
        for (int u = 0; u < IPO; ++u)
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :: "s"(base + u * 1024), "v"(offA[u]), "s"(baseA) : "memory", "m0");
#pragma unroll
        for (int u = 0; u < IPO; ++u)
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :: "s"(base + OPND_BYTES + u * 1024), "v"(offG[u]), "s"(baseG) : "memory", "m0");
        baseA += stepA;
        baseG += stepG;
    };

    // ---- LDS -> MFMA operands.  Lane l of a 16-lane group: source row j = (l % 16) / 4, source column
    //      piece q = l % 4; after the transposing read the lane holds 4 k values of column l % 16.
    const int wm = wave >> 2, wn = wave & 3;
    const int g16 = lane >> 4, s16 = lane & 15;
    const int half = g16 >> 1;                      // lanes 32..63 hold k + 8 .. k + 15 of a 16-wide k step
    const int rsrc = 8 * half + (s16 >> 2);         // row inside the k step for the first read (second read: + 4)
    uint32_t rdA[4], rdG[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int ma = wm * 128 + i * 32 + 16 * (g16 & 1) + 4 * (s16 & 3);      // column (element) of the 8-byte piece
        rdA[i] = rsrc * ROW_BYTES + ((((ma >> 3) ^ chunk_swz(rsrc)) << 4) | ((ma & 7) << 1));
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int na = wn * 64 + j * 32 + 16 * (g16 & 1) + 4 * (s16 & 3);
        rdG[j] = OPND_BYTES + rsrc * ROW_BYTES + ((((na >> 3) ^ chunk_swz(rsrc)) << 4) | ((na & 7) << 1));
    }

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    int ex = s_begin / spe;
    int sub = s_begin - ex * spe;
    // The clip factors of the examples this workgroup walks through are kept one per lane in a register
    // (loaded before the copies start) and picked with v_readlane: a scalar or vector load inside the loop
    // would make the compiler wait for every LDS read / copy in flight at each use.
    const int ex0 = ex;                             // a K slice spans at most 64 examples (see the plan)
    float vclip = 1.0f;
    if (MODE == 0) vclip = a.clip[min(ex0 + lane, a.B - 1)];
    float c_cur = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, vclip), 0));

    // prologue: all NST buffers are free, fill them
#pragma unroll
    for (int p = 0; p < NST; ++p)
        if (p < n_stages) issue(p);

    // Software pipeline over k steps: while the MFMAs of one k step run, the LDS reads of the next one are
    // in flight, also across the stage boundary.  The barrier that makes stage st + 1 visible therefore
    // sits in front of the last k step of stage st.
    auto read_kstep = [&](bf16x8 (&f)[6], uint32_t sb, int ks) {
        LDS_PTR(unsigned char) b = (LDS_PTR(unsigned char))lds + sb + ks * 16 * ROW_BYTES;
#pragma unroll
        for (int x = 0; x < 6; ++x) {
            const uint32_t off = x < 4 ? rdA[x & 3] : rdG[x & 1];
            const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(v4i16))(b + off));
            const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(v4i16))(b + off + 4 * ROW_BYTES));
            f[x] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
    };
    auto mfma_kstep = [&](const bf16x8 (&f)[6]) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i], f[4 + j], acc[i][j], 0, 0, 0);
    };
    // stage s (relative) landed once at most `ahead` later stages' copies are outstanding
    auto wait_stage = [&](int ahead) {
#if defined(DPK_EXP) && (DPK_EXP == 1 || DPK_EXP == 2)
        (void)ahead; return;                        // scratch timing experiment: no waits for the copies
#endif
        if (NST >= 4 && ahead >= 3) wait_vmcnt<3 * LPS>();
        else if (NST >= 3 && ahead == 2) wait_vmcnt<2 * LPS>();
        else if (ahead == 1) wait_vmcnt<LPS>();
        else wait_vmcnt<0>();
    };

    wait_stage(min(n_stages - 1, NST - 1));
    __builtin_amdgcn_s_barrier();
    bf16x8 f[2][6];                                 // fragments of the current / next k step: 0..3 of A, 4..5 of G
    read_kstep(f[0], 0u, 0);

    for (int st = 0; st < n_stages; ++st) {
        const uint32_t sb = (uint32_t)(st % NST) * STAGE_BYTES;
        if (MODE == 0 && sub == spe) {
            // first stage of the next example: rescale the running tile
            sub = 0;
            ++ex;
            const float c_next = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, vclip), ex - ex0));
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
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            // the fragments of this k step were requested a whole k step ago: retire them before queueing the
            // next ones, so that the MFMAs below never wait for reads issued here (LDS reads return in order)
            __builtin_amdgcn_s_waitcnt(0xC07F);                                          // lgkmcnt(0)
            if (ks + 1 < KS) {
                read_kstep(f[(ks + 1) & 1], sb, ks + 1);
            } else if (st + 1 < n_stages) {
                // stage st + 1 must have landed (later stages may stay in flight), for every wave; every wave
                // has also retired its last reads of stage st, so that buffer can take stage st + NST
                wait_stage(min(n_stages - 2 - st, NST - 2));
                __builtin_amdgcn_s_barrier();
                if (st + NST < n_stages) issue(st % NST);
                read_kstep(f[0], (uint32_t)((st + 1) % NST) * STAGE_BYTES, 0);
            }
            mfma_kstep(f[ks & 1]);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    const int lrow = lane & 31, lhalf = lane >> 5;
    if (MODE == 1) {
        // sum of squares over the valid part of the tile (columns / rows beyond d_out / d_in hold clamped copies)
        float sq = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int n = n0 + wn * 64 + j * 32 + lrow;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = m0 + wm * 128 + i * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
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
            for (int w = 0; w < DTHREADS / 64; ++w) t += red[w];
            a.out[(size_t)z * tiles + tile] = t;
        }
        return;
    }
    // the tile holds (1 / c_cur) * sum: finish with the last example's factor
    float* out = a.out + (size_t)z * a.slice;
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

// rows per stage: 64 when every example is a whole number of 64-row stages, else 32
inline int dma_dk(int T) { (void)T; return 32; }

inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

}  // namespace

bool dma_clipped_ok(int B, int T, int M, int N) {
    (void)B;
    if ((T % 32) != 0 || ((M | N) & 7) != 0) return false;
    if ((int64_t)64 * (M > N ? M : N) * 2 >= (int64_t(1) << 31)) return false;     // 32-bit lane offsets inside a stage
    const int64_t padded = (int64_t)ceil_div(M, DM) * DM * ceil_div(N, DN) * DN;
    return padded * 4 <= (int64_t)M * N * 5;                              // at most a quarter of the padded tiles is waste
}

TnPlan plan_clipped_bf16_dma(int B, int T, int M, int N) {
    TnPlan p;
    p.tile_m = DM; p.tile_n = DN;
    p.tiles_m = ceil_div(M, DM); p.tiles_n = ceil_div(N, DN);
    p.segmented = false; p.epu = 0; p.big = false; p.dma = true;
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    const int DK = dma_dk(T);
    const int64_t stages = (int64_t)B * T / DK;
    // one workgroup per compute unit: as many K slices as fit into 256 workgroups, at least 8 stages each
    int64_t splits = 256 / tiles;
    if (splits < 1) splits = 1;
    const int64_t max_splits = (stages + 7) / 8;
    if (splits > max_splits) splits = max_splits;
    int64_t sps = (stages + splits - 1) / splits;
    const int64_t spe = T / DK;
    if (sps > 63 * spe) sps = 63 * spe;               // a slice may touch at most 64 examples (one clip factor per lane)
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
    const int DK = dma_dk(T);
    a.stages_total = (int)((int64_t)B * T / DK);
    a.stages_per_split = p.kchunk / DK;
    const int64_t n = (int64_t)M * N;
    const int tiles = p.tiles_m * p.tiles_n;
    a.per_xcd = ceil_div((int64_t)tiles * p.splits, 8);
    if (p.splits == 1) { a.out = grad; a.slice = 0; a.accumulate = accumulate ? 1 : 0; }
    else { a.out = ws; a.slice = splitk_slice_elems(n); a.accumulate = 0; }
    if (DK == 64) k_tn_bf16_dma<64, 2, 0><<<8u * (unsigned)a.per_xcd, DTHREADS, 0, st>>>(a);
    else k_tn_bf16_dma<32, 4, 0><<<8u * (unsigned)a.per_xcd, DTHREADS, 0, st>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.splits == 1) return e;
    return launch_splitk_reduce(ws, n, p.splits, accumulate, grad, st);
}

bool dma_direct_ok(int T, int M, int N) {
    if (T < 64 || (T % 32) != 0 || ((M | N) & 7) != 0) return false;
    if ((int64_t)64 * (M > N ? M : N) * 2 >= (int64_t(1) << 31)) return false;     // 32-bit lane offsets inside a stage
    const int64_t padded = (int64_t)ceil_div(M, DM) * DM * ceil_div(N, DN) * DN;
    return padded * 4 <= (int64_t)M * N * 5;                              // at most a quarter of the padded tiles is waste
}

hipError_t launch_direct_bf16_dma(const uint16_t* A, const uint16_t* G, int B, int T, int M, int N,
                                  bool accumulate, float* sqnorm, float* partial, hipStream_t st) {
    DmaArgs a;
    a.A = A; a.G = G; a.clip = nullptr;
    a.B = B; a.T = T; a.M = M; a.N = N;
    a.tiles_m = ceil_div(M, DM); a.tiles_n = ceil_div(N, DN);
    a.splits = B;
    a.stages_total = (int)((int64_t)B * T / 32);
    a.stages_per_split = T / 32;
    a.out = partial; a.slice = 0; a.accumulate = 0;
    const int tiles = a.tiles_m * a.tiles_n;
    const int64_t total = (int64_t)tiles * B;
    if (total >= (int64_t(1) << 28)) return hipErrorInvalidValue;
    a.per_xcd = ceil_div(total, 8);
    k_tn_bf16_dma<32, 4, 1><<<8u * (unsigned)a.per_xcd, DTHREADS, 0, st>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_finalize_partials(partial, B, tiles, accumulate, sqnorm, st);
}

}  // namespace dpk
