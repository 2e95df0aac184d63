// Copy-pipeline kernels for aligned layers with 16-bit inputs (bf16 or fp16; the kernels only move the bits, the
// format decides which MFMA instruction consumes them): clipped sum  sum_i c_i A_i^T G_i  and direct squared norm.
//
// gfx950-specific data path with (almost) no VALU work in the main loop:
//   * global -> LDS copies go straight into LDS (global_load_lds_dwordx4): a
//     wave instruction moves 1 KB of a K-major tile, as it lies in memory.
//     A ring of 32-row stages is kept in LDS, all but one of them in flight
//     while one is consumed.
//   * the 16-bit transpose the MFMA needs (a lane must hold consecutive k for
//     one column, memory has consecutive columns for one k) is done by the
//     LDS read itself (ds_read_b64_tr_b16): 16 lanes read a 4(k) x 16(col)
//     patch and each lane gets the 4 k values of one column.
//   * four tile geometries (struct Geo below): 256 x 256 per workgroup of 8
//     waves, one workgroup per compute unit, for layers whose clipped sum is
//     bound by the MFMA rate; 192 x 128 per workgroup of 4 waves, two
//     workgroups per compute unit, for narrow layers bound by HBM; 128 x 128
//     for the mid-size layers that neither tiles without much padding; 64 x 64
//     for the clipped sum of a small matrix over many rows.
//
// Clip factors are applied to the fp32 accumulators, not to the 16-bit inputs:
// the tile holds  (1 / c_cur) * sum_{j <= cur} c_j g_j ; when the rows of the
// next example start it is multiplied by c_cur / c_next (one multiply per
// accumulator register per example, skipped when the two factors are equal),
// and by the last example's factor at the end.  This is exact up to one fp32
// rounding per example.  It needs every 32-row stage to lie inside one
// example: T % 32 == 0, or the ragged mode below, which pads every example
// with rows of zeros.  K slices are arbitrary ranges of stages.
// An example whose factor is zero (a masked example, or the factor that
// dp_clip_factors gives an overflowed norm), or below 2^-40 of the largest
// factor the K slice has accumulated so far, cannot become the unit (the tile
// in that unit, sum / c_next, would leave the float32 range): its MFMAs are
// skipped instead and the unit stays, i.e. the example counts with factor 0,
// as the weighted sum defines for a zero factor; a factor 10^12 times below
// another one of the same sum is below that sum's float32 resolution.
#include <algorithm>
#include "dp_common.h"
#include "dp_internal.h"

namespace dpk {

namespace {

constexpr int DK = 32;                // rows of A and of G per stage

typedef short v4i16 __attribute__((ext_vector_type(4)));
#define LDS_PTR(T) __attribute__((address_space(3))) T*

// Tile geometry: WM x WN waves, each owning FM x FN MFMA tiles of 32 x 32; NST stages resident in LDS; OCC
// workgroups per compute unit.
template <int WM_, int WN_, int FM_, int FN_, int NST_, int OCC_>
struct Geo {
    static constexpr int WM = WM_, WN = WN_, FM = FM_, FN = FN_, NST = NST_, OCC = OCC_;
    static constexpr int WAVES = WM * WN, THREADS = 64 * WAVES;
    static constexpr int TM = WM * FM * 32, TN = WN * FN * 32;        // output tile
    static constexpr int RBA = TM * 2, RBG = TN * 2;                  // bytes of one stage row of either operand
    static constexpr int IPA = RBA / 32 / WAVES, IPG = RBG / 32 / WAVES;   // 1 KB copies per operand, stage and wave
    static constexpr int LPS = IPA + IPG;                             // copies per stage and wave
    static constexpr int OPA = DK * RBA, STAGE_BYTES = DK * (RBA + RBG);
    static_assert(IPA * 32 * WAVES == RBA && IPG * 32 * WAVES == RBG, "a stage must be a whole number of copies per wave");
    static_assert(NST >= 2 && OCC * NST * STAGE_BYTES <= 160 * 1024, "stages must fit the 160 KB of LDS");
    static_assert(3 * LPS <= 63, "vmcnt range");
};
// MFMA-bound layers: 256 x 256 tile (128 flop per byte copied), 8 waves of 128 x 64, four 32 KB stages, one
// workgroup per compute unit.  At 256 x 128 the kernel ran into the ~10 TB/s the L2s deliver to the compute units.
using GeoL = Geo<2, 4, 4, 2, 4, 1>;
// narrow, HBM-bound layers (e.g. the unfolded 3 x 3 convolution, 576 x 128): 192 x 128 tile, 4 waves of 96 x 64,
// three 20 KB stages, two workgroups per compute unit: more workgroups to spread over the chip, and as many bytes
// in flight per compute unit
using GeoS = Geo<2, 2, 3, 2, 3, 2>;
// layers of a few hundred columns that neither of the above tiles without much padding (256 x 128, 128 x 128,
// 640 x 384, ...): 128 x 128 tile, 4 waves of 64 x 64, four 16 KB stages, two workgroups per compute unit
using GeoT = Geo<2, 2, 2, 2, 4, 2>;
// clipped sums of a small matrix over many rows (a recurrent layer: 256 x 256 from 8192 rows): a handful of tiles,
// so the chip is filled with K slices, every one a partial matrix to store and to fold.  64 x 64 tiles, 4 waves of
// 32 x 32, four 8 KB stages: four times the tiles, a quarter of the slices.
using GeoU = Geo<2, 2, 1, 1, 4, 4>;

struct DmaArgs {
    const uint16_t* A;
    const uint16_t* G;
    const float* clip;
    float* out;            // slice base (stride `slice` per K slice) or grad; direct norm: partial[B][tiles]
    int64_t slice;
    int B, T, M, N;
    int tiles_m, tiles_n;
    int splits;
    int stages_total;      // B * ceil(T / DK)
    int stages_per_split;
    int per_xcd;
    int accumulate;
    // AM = 1: A is the image X[B, H, W, C] (channels last); column (kh * KW + kw) * C + c of the patch matrix at
    // output position (y, x) is X[y + kh - pad, x + kw - pad, c], zero outside the image; T = Hout * Wout.
    int H, W, C, KW, pad, Wout;
    const uint16_t* zero;  // AM = 1, 2: at least 16 bytes of zeros
};

// Rows of RB bytes; the 16-byte chunk c of row r sits at chunk position c ^ chunk_swz<RB>(r).  A transposing read
// of 32 lanes touches 4 consecutive rows x 64 bytes (two 32-byte pieces side by side).  Banks repeat every 256
// bytes: when RB is a multiple of 256 the 4 rows start in the same bank and the xor moves them to 4 different
// 64-byte windows; when RB = 128 mod 256 rows r and r + 2 collide and the xor separates those.
template <int RB> __device__ __forceinline__ int chunk_swz(int r) {
    static_assert(RB % 128 == 0, "row bytes");
    if (RB % 256 == 0) return (r & 3) << 2;         // needs 16 | chunks per row
    return ((r >> 1) & 1) << 2;                     // needs 8 | chunks per row
}

template <int N> __device__ __forceinline__ void wait_vmcnt() { __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14)); }

// MODE 0: clipped sum over a K slice (any range of stages).  MODE 1: direct squared norm: the K slice is one
// example (stages_per_split = ceil(T / DK), splits = B), no scaling, and the finished tile of A_i^T G_i is squared
// and reduced to one float per (example, tile) instead of being stored (Algorithm 3 / 4 without their output).
// AM = 1 (CONV): the A operand is never unfolded in memory (implicit unfolding of Algorithm 3's patch matrix): every lane of
// a copy instruction computes the address of its 16-byte piece of the image, or points at a line of zeros where
// the patch reaches into the padding; the LDS tile, the MFMA loop and the epilogues are the same.
// AM = 2 (ragged): T is not a multiple of the 32-row stage.  Every example then takes ceil(T / 32) stages, and
// the rows past its end in the last one are copied from the line of zeros (rows of zeros add nothing to the
// product); the per-lane addresses are 64-bit as in the convolution mode.
// `L`: the (slice, tile) pair of this workgroup among the layer's tiles * splits
template <class GEO, int MODE, int AM, bool F16>
__device__ __forceinline__ void tn_dma_tile(const DmaArgs& a, const int L) {
    constexpr bool CONV = AM == 1, RAG = AM == 2;
    constexpr int NST = GEO::NST, FM = GEO::FM, FN = GEO::FN, NF = FM + FN;
    constexpr int RBA = GEO::RBA, RBG = GEO::RBG, IPA = GEO::IPA, IPG = GEO::IPG, LPS = GEO::LPS;
    constexpr int OPA = GEO::OPA, STAGE_BYTES = GEO::STAGE_BYTES;
    constexpr int KS = DK / 16;                      // k steps per stage
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
    const int spe = (a.T + DK - 1) / DK;            // stages per example (T % 32 != 0 only in the ragged mode)

    // ---- global -> LDS.  The A part of a stage (DK rows of RBA bytes) and its G part are each a linear run of
    //      16-byte chunks; copy u of wave w moves chunks 64 (w IP + u) .. + 63, one per lane.  Addresses are a
    //      uniform 64-bit stage base (SGPR) plus a 32-bit per-lane byte offset that never changes.
    uint32_t offA[IPA], offG[IPG];
    int rowA[IPA], rowG[IPG];                        // RAG: row inside the stage of each copy's lane
    int cdy[IPA], cdx[IPA], cy0[IPA], cx0[IPA], cy[IPA], cx[IPA];    // CONV: tap offsets, position at an example's start, current position
    const int sub_begin = s_begin - (s_begin / spe) * spe;
#pragma unroll
    for (int u = 0; u < IPA; ++u) {
        const int idx = (wave * IPA + u) * 64 + lane;
        const int r = idx / (RBA / 16);                               // row inside the stage
        int col = m0 + (((idx % (RBA / 16)) ^ chunk_swz<RBA>(r)) << 3);
        if (col >= a.M) col = m0;                   // out-of-range columns only feed output rows that are never stored
        rowA[u] = r;
        if (CONV) {
            const int tap = col / a.C, kh = tap / a.KW;
            offA[u] = (uint32_t)(col - tap * a.C) * 2u;               // channel offset inside the pixel, bytes
            cdy[u] = kh - a.pad; cdx[u] = tap - kh * a.KW - a.pad;
            cy0[u] = r / a.Wout; cx0[u] = r - cy0[u] * a.Wout;
            const int t = sub_begin * DK + r;
            cy[u] = t / a.Wout; cx[u] = t - cy[u] * a.Wout;
        } else {
            offA[u] = ((uint32_t)r * (uint32_t)a.M + (uint32_t)col) * 2u;
        }
    }
#pragma unroll
    for (int u = 0; u < IPG; ++u) {
        const int idx = (wave * IPG + u) * 64 + lane;
        const int r = idx / (RBG / 16);
        int col = n0 + (((idx % (RBG / 16)) ^ chunk_swz<RBG>(r)) << 3);
        if (col >= a.N) col = n0;
        rowG[u] = r;
        offG[u] = ((uint32_t)r * (uint32_t)a.N + (uint32_t)col) * 2u;
    }
    const size_t stepA = (size_t)DK * a.M, stepG = (size_t)DK * a.N;  // per stage
    const uint16_t* baseA = CONV ? a.A + (size_t)(s_begin / spe) * a.H * a.W * a.C       // the example's image
                          : RAG  ? a.A + (size_t)(s_begin / spe) * a.T * a.M + (size_t)sub_begin * stepA
                                 : a.A + (size_t)s_begin * stepA;                        // uniform
    const uint16_t* baseG = (RAG || CONV) ? a.G + (size_t)(s_begin / spe) * a.T * a.N + (size_t)sub_begin * stepG
                                : a.G + (size_t)s_begin * stepG;
    int conv_sub = sub_begin;                                          // CONV, RAG: stage inside the example of the next copy

    // The copies are issued as inline assembly: the compiler then does not know that they write LDS and
    // does not make every LDS read wait for all copies in flight; the waits for them are the explicit
    // vmcnt waits in front of the stage barriers below.
    const uint32_t lds_base = (uint32_t)(uintptr_t)(LDS_PTR(unsigned char))lds;
    const uint32_t wave_ldsA = __builtin_amdgcn_readfirstlane(lds_base + wave * IPA * 1024);
    const uint32_t wave_ldsG = __builtin_amdgcn_readfirstlane(lds_base + OPA + wave * IPG * 1024);
    auto issue = [&](int buf) {
        if (CONV) {
            const int hout = a.T / a.Wout;
#pragma unroll
            for (int u = 0; u < IPA; ++u) {
                const int py = cy[u] + cdy[u], px = cx[u] + cdx[u];
                // inside the image, and an output position of this example (the last stage may run past T)
                const bool inside = (unsigned)py < (unsigned)a.H && (unsigned)px < (unsigned)a.W && cy[u] < hout;
                const uint64_t addr = inside ? (uint64_t)(uintptr_t)baseA + ((uint32_t)(py * a.W + px) * (uint32_t)a.C * 2u + offA[u])
                                             : (uint64_t)(uintptr_t)a.zero;
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                             :: "s"(wave_ldsA + buf * STAGE_BYTES + u * 1024), "v"(addr) : "memory", "m0");
            }
            const int rows_valid = a.T - conv_sub * DK;
#pragma unroll
            for (int u = 0; u < IPG; ++u) {
                const uint64_t addr = rowG[u] < rows_valid ? (uint64_t)(uintptr_t)baseG + offG[u] : (uint64_t)(uintptr_t)a.zero;
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                             :: "s"(wave_ldsG + buf * STAGE_BYTES + u * 1024), "v"(addr) : "memory", "m0");
            }
            // the next stage: 32 positions further, or the start of the next example's image
            if (++conv_sub == spe) {
                conv_sub = 0;
                baseA += (size_t)a.H * a.W * a.C;
                baseG += (size_t)(a.T - (spe - 1) * DK) * a.N;
#pragma unroll
                for (int u = 0; u < IPA; ++u) { cy[u] = cy0[u]; cx[u] = cx0[u]; }
            } else {
                baseG += stepG;
#pragma unroll
                for (int u = 0; u < IPA; ++u) {
                    cx[u] += DK;
                    while (cx[u] >= a.Wout) { cx[u] -= a.Wout; ++cy[u]; }
                }
            }
            return;
        } else if (RAG) {
            const int rows_valid = a.T - conv_sub * DK;               // rows of this stage inside the example (may exceed 32)
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
            // the next stage: 32 rows further, or the first rows of the next example (which start T rows after this one's)
            if (++conv_sub == spe) {
                baseA += (size_t)(a.T - (spe - 1) * DK) * a.M;
                baseG += (size_t)(a.T - (spe - 1) * DK) * a.N;
                conv_sub = 0;
            } else {
                baseA += stepA;
                baseG += stepG;
            }
            return;
        } else {
#pragma unroll
            for (int u = 0; u < IPA; ++u)
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                             :: "s"(wave_ldsA + buf * STAGE_BYTES + u * 1024), "v"(offA[u]), "s"(baseA) : "memory", "m0");
            baseA += stepA;
        }
#pragma unroll
        for (int u = 0; u < IPG; ++u)
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :: "s"(wave_ldsG + buf * STAGE_BYTES + u * 1024), "v"(offG[u]), "s"(baseG) : "memory", "m0");
        baseG += stepG;
    };

    // ---- LDS -> MFMA operands.  Lane l of a 16-lane group: source row j = (l % 16) / 4, source column
    //      piece q = l % 4; after the transposing read the lane holds 4 k values of column l % 16.
    const int wm = wave / GEO::WN, wn = wave % GEO::WN;
    const int g16 = lane >> 4, s16 = lane & 15;
    const int half = g16 >> 1;                      // lanes 32..63 hold k + 8 .. k + 15 of a 16-wide k step
    const int rsrc = 8 * half + (s16 >> 2);         // row inside the k step for the first read (second read: + 4)
    uint32_t rd[NF];                                // 0 .. FM-1: A fragments, FM ..: G fragments
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int ma = (wm * FM + i) * 32 + 16 * (g16 & 1) + 4 * (s16 & 3);     // column (element) of the 8-byte piece
        rd[i] = rsrc * RBA + ((((ma >> 3) ^ chunk_swz<RBA>(rsrc)) << 4) | ((ma & 7) << 1));
    }
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const int na = (wn * FN + j) * 32 + 16 * (g16 & 1) + 4 * (s16 & 3);
        rd[FM + j] = OPA + rsrc * RBG + ((((na >> 3) ^ chunk_swz<RBG>(rsrc)) << 4) | ((na & 7) << 1));
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
    // (loaded before the copies start) and picked with v_readlane: a scalar or vector load inside the loop
    // would make the compiler wait for every LDS read / copy in flight at each use.
    const int ex0 = ex;                             // a K slice spans at most 64 examples (see the plan)
    float vclip = 1.0f;
    if (MODE == 0) vclip = a.clip[min(ex0 + lane, a.B - 1)];
    float c_cur = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, vclip), 0));
    bool skip = false;                              // the current example is left out (see the head of this file)
    float c_ref = c_cur;                            // the largest factor accumulated so far

    // prologue: all NST buffers are free, fill them
#pragma unroll
    for (int p = 0; p < NST; ++p)
        if (p < n_stages) issue(p);

    // Software pipeline over k steps: while the MFMAs of one k step run, the LDS reads of the next one are
    // in flight, also across the stage boundary.  The barrier that makes stage st + 1 visible therefore
    // sits in front of the last k step of stage st.
    auto read_kstep = [&](bf16x8 (&f)[NF], uint32_t sb, int ks) {
        LDS_PTR(unsigned char) b = (LDS_PTR(unsigned char))lds + sb;
#pragma unroll
        for (int x = 0; x < NF; ++x) {
            const uint32_t off = rd[x] + ks * 16 * (x < FM ? RBA : RBG);
            const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(v4i16))(b + off));
            const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(v4i16))(b + off + 4 * (x < FM ? RBA : RBG)));
            f[x] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
    };
    auto mfma_kstep = [&](const bf16x8 (&f)[NF]) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
                acc[i][j] = In16<F16>::mfma(f[i], f[FM + j], acc[i][j]);
    };
    // stage s (relative) landed once at most `ahead` later stages' copies are outstanding
    auto wait_stage = [&](int ahead) {
        if (NST >= 4 && ahead >= 3) wait_vmcnt<3 * LPS>();
        else if (NST >= 3 && ahead == 2) wait_vmcnt<2 * LPS>();
        else if (ahead == 1) wait_vmcnt<LPS>();
        else wait_vmcnt<0>();
    };

    wait_stage(min(n_stages - 1, NST - 1));
    __builtin_amdgcn_s_barrier();
    bf16x8 f[2][NF];                                // fragments of the current / next k step
    read_kstep(f[0], 0u, 0);

    for (int st = 0; st < n_stages; ++st) {
        const uint32_t sb = (uint32_t)(st % NST) * STAGE_BYTES;
        if (MODE == 0 && sub == spe) {
            // first stage of the next example: rescale the running tile
            sub = 0;
            ++ex;
            const float c_next = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, vclip), ex - ex0));
            const float ratio = c_cur / c_next;
            // a zero factor, or one far below the largest so far, after a non-zero one: leave this example out
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
            if (MODE != 0 || !skip) mfma_kstep(f[ks & 1]);
            __builtin_amdgcn_sched_barrier(0);
        }
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

template <class GEO, int MODE, int AM, bool F16>
__global__ __launch_bounds__(GEO::THREADS, GEO::OCC) void k_tn_bf16_dma(DmaArgs a) {
    // workgroup b runs on XCD b % 8: give each XCD a contiguous run of (slice, tile) pairs so that
    // its workgroups stream the same rows of A and G through one L2
    tn_dma_tile<GEO, MODE, AM, F16>(a, (blockIdx.x & 7) * a.per_xcd + (blockIdx.x >> 3));
}

// Several layers' clipped sums in one launch (256 x 256 tiles, flat operands): the launch is a list of (layer, K slice,
// tile) items, a layer's items slice-major, dealt to the XCDs in contiguous runs like a single layer's.  All layers
// cut their K range into slices of about the same length, chosen so that the items fill the chip a whole number of
// times: a launch per layer has to fill it exactly once, which takes more and shorter slices (more partial tiles to
// store and to fold) and leaves a gap between the layers.
constexpr int kJointMax = kJointLayers;
struct JointLayer {
    const uint16_t* A; const uint16_t* G; const float* clip;
    float* slices;       // the layer's K slices; the gradient itself where one slice is the whole sum (then `accumulate` applies)
    int T, M, N, tiles_m, tiles_n, splits, stages_total, stages_per_split, first_item, accumulate;
};
struct JointArgs {
    JointLayer layer[kJointMax];
    int n_layers, n_items, per_xcd, B;
};
// the ragged mode's line of zeros (never written)
__device__ __attribute__((aligned(256))) unsigned int g_zero_line[64];

// AM: 0 = every layer's T is a multiple of the 32-row stage, 2 = ragged T (stages padded with the line of zeros)
// MODE 1: the layers' direct squared norms (a layer's "K slices" are its examples, `slices` is partial[B][tiles])
template <class GEO, bool F16, int AM, int MODE = 0>
__global__ __launch_bounds__(GEO::THREADS, GEO::OCC) void k_tn_bf16_dma_joint(JointArgs j) {
    const int L = (blockIdx.x & 7) * j.per_xcd + (blockIdx.x >> 3);
    if (L >= j.n_items) return;
    int l = 0;
    while (l + 1 < j.n_layers && L >= j.layer[l + 1].first_item) ++l;
    const JointLayer& y = j.layer[l];
    DmaArgs a;
    a.A = y.A; a.G = y.G; a.clip = y.clip;
    a.out = y.slices; a.slice = (((int64_t)y.M * y.N) + 3) & ~(int64_t)3;        // splitk_slice_elems
    a.B = j.B; a.T = y.T; a.M = y.M; a.N = y.N;
    a.tiles_m = y.tiles_m; a.tiles_n = y.tiles_n; a.splits = y.splits;
    a.stages_total = y.stages_total; a.stages_per_split = y.stages_per_split;
    a.per_xcd = 0; a.accumulate = y.accumulate;
    a.H = a.W = a.C = a.KW = a.Wout = 1; a.pad = 0;
    a.zero = AM == 2 ? reinterpret_cast<const uint16_t*>(g_zero_line) : nullptr;
    tn_dma_tile<GEO, MODE, AM, F16>(a, L - y.first_item);
}


// 0: not for this kernel; 1: GeoL; 2: GeoS; 3: GeoT (the first that fits, in the order of flop per copied byte)
int dma_geometry(int T, int M, int N) {
    if (((M | N) & 7) != 0) return 0;
    if ((T % DK) != 0 && (int64_t)ceil_div(T, DK) * DK * 4 > (int64_t)T * 5) return 0;   // ragged T: at most a quarter of zero rows
    if ((int64_t)DK * (M > N ? M : N) * 2 >= (int64_t(1) << 31)) return 0;        // 32-bit lane offsets inside a stage
    if (tiles_fit(M, N, GeoL::TM, GeoL::TN)) return 1;
    if (tiles_fit(M, N, GeoS::TM, GeoS::TN)) return 2;
    if (tiles_fit(M, N, GeoT::TM, GeoT::TN)) return 3;
    return 0;
}

// Among the geometries that fit, the first one (largest tile) unless it leaves most of the chip idle: a launch
// of fewer than 128 workgroups gives way to the geometry with the most workgroups.  `units` = what multiplies
// the tile count: K slices available (clipped sum) or examples (direct norm).
struct GeoDims { int tm, tn, occ; };
GeoDims geo_dims(int id) {
    if (id == 1) return {GeoL::TM, GeoL::TN, GeoL::OCC};
    if (id == 2) return {GeoS::TM, GeoS::TN, GeoS::OCC};
    return {GeoT::TM, GeoT::TN, GeoT::OCC};
}
int pick_geometry(int T, int M, int N, int64_t units) {
    const int first = dma_geometry(T, M, N);
    if (first == 0) return 0;
    int best = first;
    int64_t best_blocks = -1;
    for (int id = first; id <= 3; ++id) {
        const GeoDims g = geo_dims(id);
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

// the plan names its geometry by the tile shape
int geo_of_plan(const TnPlan& p) { return p.tile_m == GeoL::TM ? 1 : (p.tile_m == GeoS::TM ? 2 : (p.tile_m == GeoT::TM ? 3 : 4)); }

// am: 0 = rows of A as they lie in memory, 1 = implicit unfolding of an image, 2 = ragged T
template <class GEO, int MODE, bool F16> hipError_t launch_geo(const DmaArgs& a, int am, hipStream_t st) {
    if (am == 1)      k_tn_bf16_dma<GEO, MODE, 1, F16><<<8u * (unsigned)a.per_xcd, GEO::THREADS, 0, st>>>(a);
    else if (am == 2) k_tn_bf16_dma<GEO, MODE, 2, F16><<<8u * (unsigned)a.per_xcd, GEO::THREADS, 0, st>>>(a);
    else              k_tn_bf16_dma<GEO, MODE, 0, F16><<<8u * (unsigned)a.per_xcd, GEO::THREADS, 0, st>>>(a);
    return hipGetLastError();
}
template <int MODE, bool F16> hipError_t launch_fmt(int geo, const DmaArgs& a, int am, hipStream_t st) {
    if (geo == 1) return launch_geo<GeoL, MODE, F16>(a, am, st);
    if (geo == 2) return launch_geo<GeoS, MODE, F16>(a, am, st);
    return launch_geo<GeoT, MODE, F16>(a, am, st);
}
template <int MODE> hipError_t launch_any(int geo, const DmaArgs& a, int am, bool f16, hipStream_t st) {
    return f16 ? launch_fmt<MODE, true>(geo, a, am, st) : launch_fmt<MODE, false>(geo, a, am, st);
}

void set_conv(DmaArgs& a, const ConvGeom* cg, const uint16_t* zero) {
    a.zero = zero;

    if (cg) { a.H = cg->H; a.W = cg->W; a.C = cg->C; a.KW = cg->KW; a.pad = cg->pad; a.Wout = cg->W + 2 * cg->pad - cg->KW + 1; }
    else { a.H = a.W = a.C = a.KW = a.Wout = 1; a.pad = 0; }
}

}  // namespace

bool dma_clipped_ok(int B, int T, int M, int N) { (void)B; return dma_geometry(T, M, N) != 0; }

TnPlan plan_clipped_bf16_dma(int B, int T, int M, int N, bool flat) {
    const int64_t spe = ceil_div(T, DK);
    const int64_t stages = (int64_t)B * spe;
    const GeoDims gd = geo_dims(pick_geometry(T, M, N, (stages + 7) / 8));
    TnPlan p;
    // A small matrix (at most 16 tiles of 128 x 128) whose rows lie flat in memory, T a multiple of the stage, and so
    // many stages that the larger tiles would be cut into 16 slices or more: 64 x 64 tiles, slices of at least 16 stages
    if (flat && (T % DK) == 0 && ((M | N) & 63) == 0 && (int64_t)M * N <= 16 * 128 * 128 && stages >= 256 &&
        (int64_t)ceil_div(M, gd.tm) * ceil_div(N, gd.tn) * 16 <= 256 * gd.occ) {
        p.tile_m = GeoU::TM; p.tile_n = GeoU::TN;
        p.tiles_m = M / GeoU::TM; p.tiles_n = N / GeoU::TN;
        p.segmented = false; p.epu = 0; p.big = false; p.dma = true; p.zero_head = false;
        const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
        int64_t splits = 512 / tiles;                 // two workgroups per compute unit
        if (splits < 1) splits = 1;
        if (splits > stages / 16) splits = stages / 16;
        int64_t sps = (stages + splits - 1) / splits;
        if (sps > 63 * spe) sps = 63 * spe;
        p.kchunk = (int)(sps * DK);
        p.splits = (int)((stages + sps - 1) / sps);
        return p;
    }
    p.tile_m = gd.tm; p.tile_n = gd.tn;
    p.tiles_m = ceil_div(M, p.tile_m); p.tiles_n = ceil_div(N, p.tile_n);
    p.segmented = false; p.epu = 0; p.big = false; p.dma = true;
    p.zero_head = (T % DK) != 0;
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    // fill the chip once (256 compute units x workgroups per unit) with K slices of at least 8 stages each
    int64_t splits = 256 * gd.occ / tiles;
    if (splits < 1) splits = 1;
    const int64_t max_splits = (stages + 7) / 8;
    if (splits > max_splits) splits = max_splits;
    int64_t sps = (stages + splits - 1) / splits;
    if (sps > 63 * spe) sps = 63 * spe;               // a slice may touch at most 64 examples (one clip factor per lane)
    p.kchunk = (int)(sps * DK);
    p.splits = (int)((stages + sps - 1) / sps);
    return p;
}

hipError_t launch_clipped_bf16_dma(const TnPlan& p, const uint16_t* A, const uint16_t* G, const float* clip,
                                   int B, int T, int M, int N, bool accumulate, float* grad, float* ws, hipStream_t st,
                                   const ConvGeom* cg, const uint16_t* zero, bool f16, const NoiseArgs* noise) {
    int am = cg ? 1 : 0;
    if (!cg && p.zero_head) {
        // ragged T: the head of the workspace is the line of zeros
        zero = static_cast<const uint16_t*>(device_zero_line(st));
        if (!zero) {
            const hipError_t ez = launch_fill_zero(ws, kZeroHeadFloats, st);
            if (ez != hipSuccess) return ez;
            zero = reinterpret_cast<const uint16_t*>(ws);
        }
        ws += kZeroHeadFloats;
        am = 2;
    }
    DmaArgs a;
    set_conv(a, cg, zero);
    a.A = A; a.G = G; a.clip = clip;
    a.B = B; a.T = T; a.M = M; a.N = N;
    a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n; a.splits = p.splits;
    a.stages_total = (int)((int64_t)B * ceil_div(T, DK));
    a.stages_per_split = p.kchunk / DK;
    const int64_t n = (int64_t)M * N;
    const int tiles = p.tiles_m * p.tiles_n;
    a.per_xcd = ceil_div((int64_t)tiles * p.splits, 8);
    if (p.splits == 1) { a.out = grad; a.slice = 0; a.accumulate = accumulate ? 1 : 0; }
    else { a.out = ws; a.slice = splitk_slice_elems(n); a.accumulate = 0; }
    hipError_t e;
    if (geo_of_plan(p) == 4) {
        if (am != 0) return hipErrorInvalidValue;     // the 64 x 64 tiles are planned for flat rows only
        if (f16) k_tn_bf16_dma<GeoU, 0, 0, true><<<8u * (unsigned)a.per_xcd, GeoU::THREADS, 0, st>>>(a);
        else     k_tn_bf16_dma<GeoU, 0, 0, false><<<8u * (unsigned)a.per_xcd, GeoU::THREADS, 0, st>>>(a);
        e = hipGetLastError();
    } else {
        e = launch_any<0>(geo_of_plan(p), a, am, f16, st);
    }
    if (e != hipSuccess || p.splits == 1) return e;
    return launch_splitk_reduce(ws, n, p.splits, accumulate, grad, st, noise);
}

// ---- joint launch of several layers' clipped sums.  Two classes of layers, each with launches of its own:
//      geo 1: 256 x 256 tiles (one workgroup per compute unit), layers whose clipped sum is bound by the MFMA rate;
//      geo 3: 128 x 128 tiles (two workgroups per compute unit) for the aligned layers of a few hundred columns
//             that the first class does not take (the 3 x 3 convolutions of an image model, unfolded: 576 -> 64,
//             1152 -> 128, ...): alone each of them is a launch of 10 to 30 us that fills a fraction of the chip and
//             a fold behind it; tiles may be mostly padding, these layers are bound by latency and bandwidth.
bool dma_joint_ok(int T, int M, int N) { return T > 0 && (T % DK) == 0 && dma_geometry(T, M, N) == 1; }
//      geo 4: the same tiles for such layers whose T is not a multiple of the 32-row stage (at least 16 positions:
//             4 x 4 positions of a late convolution); the stages of an example's last rows are filled up with zeros.
bool dma_joint_mid_ok(int T, int M, int N) {
    if (T <= 0 || (T % DK) != 0 || ((M | N) & 7) != 0 || M < 64 || N < 64) return false;
    if ((int64_t)DK * (M > N ? M : N) * 2 >= (int64_t(1) << 31)) return false;        // 32-bit lane offsets inside a stage
    return dma_geometry(T, M, N) != 1;
}
bool dma_joint_ragged_ok(int T, int M, int N) {
    if (T < 16 || (T % DK) == 0 || ((M | N) & 7) != 0 || M < 64 || N < 64) return false;
    return (int64_t)T * (M > N ? M : N) * 2 < (int64_t(1) << 31);                      // 32-bit lane offsets inside an example
}
namespace {
inline int joint_tile(int geo) { return geo == 1 ? GeoL::TM : GeoT::TM; }
inline int joint_slots(int geo) { return geo == 1 ? 256 * GeoL::OCC : 256 * GeoT::OCC; }
// A group of the first class whose 256 x 256 tiles are so few and whose contractions are so short that the tiles
// would be cut into 4 or more K slices of at most 16 stages (a few examples of 64 positions into 2304 x 256: 9 tiles
// per layer, slices of 8 stages) runs on the second class's tiles: four times the tiles, half the slices to store
// and fold, and nothing there is bound by the MFMA rate.
inline int joint_group_geo(const JointShape* sh, int n_layers, int B, int geo) {
    if (geo != 1) return geo;
    const JointPlan p = plan_joint(sh, n_layers, B, DK, GeoL::TM, 256 * GeoL::OCC);
    int most = 1, longest = 1;
    for (int l = 0; l < n_layers; ++l) {
        most = most > p.splits[l] ? most : p.splits[l];
        longest = longest > p.sps[l] ? longest : p.sps[l];
    }
    return (most >= 4 && longest <= 16) ? 3 : 1;
}
}

// floats of workspace: every layer's slices, one layer after the other
size_t joint_workspace_floats(const JointShape* sh, int n_layers, int B, int geo) {
    geo = joint_group_geo(sh, n_layers, B, geo);
    const JointPlan p = plan_joint(sh, n_layers, B, DK, joint_tile(geo), joint_slots(geo));
    size_t slices = 0;
    for (int l = 0; l < n_layers; ++l) slices += (size_t)p.splits[l] * (size_t)splitk_slice_elems((int64_t)sh[l].M * sh[l].N);
    return slices;
}

hipError_t launch_clipped_bf16_dma_joint(const JointShape* sh, const JointOperands* op, int n_layers, int B, bool accumulate,
                                         float stddev, uint64_t seed, float* ws, hipStream_t st, bool f16, int geo) {
    if (n_layers < 1 || n_layers > kJointMax || (geo != 1 && geo != 3 && geo != 4)) return hipErrorInvalidValue;
    geo = joint_group_geo(sh, n_layers, B, geo);
    const JointPlan p = plan_joint(sh, n_layers, B, DK, joint_tile(geo), joint_slots(geo));
    if (p.items >= (int64_t(1) << 28)) return hipErrorInvalidValue;
    JointArgs j;
    float* slices = ws;
    int64_t first = 0;
    for (int l = 0; l < n_layers; ++l) {
        JointLayer& y = j.layer[l];
        y.A = op[l].A; y.G = op[l].G; y.clip = op[l].clip;
        // one slice and no noise to add: the launch writes the gradient itself, nothing to fold
        const bool whole = p.splits[l] == 1 && stddev == 0.0f;
        y.slices = whole ? op[l].grad : slices;
        y.accumulate = whole && accumulate ? 1 : 0;
        y.T = sh[l].T; y.M = sh[l].M; y.N = sh[l].N;
        y.tiles_m = p.tiles_m[l]; y.tiles_n = p.tiles_n[l]; y.splits = p.splits[l];
        y.stages_total = (int)((int64_t)B * ceil_div(sh[l].T, DK)); y.stages_per_split = p.sps[l];
        y.first_item = (int)first;
        first += (int64_t)p.tiles_m[l] * p.tiles_n[l] * p.splits[l];
        slices += (size_t)p.splits[l] * (size_t)splitk_slice_elems((int64_t)sh[l].M * sh[l].N);
    }
    for (int l = n_layers; l < kJointMax; ++l) j.layer[l] = j.layer[0];
    j.n_layers = n_layers; j.n_items = (int)p.items; j.per_xcd = ceil_div(p.items, 8);
    j.B = B;
    const unsigned grid = 8u * (unsigned)j.per_xcd;
    if (geo == 1) {
        if (f16) k_tn_bf16_dma_joint<GeoL, true, 0><<<grid, GeoL::THREADS, 0, st>>>(j);
        else     k_tn_bf16_dma_joint<GeoL, false, 0><<<grid, GeoL::THREADS, 0, st>>>(j);
    } else if (geo == 3) {
        if (f16) k_tn_bf16_dma_joint<GeoT, true, 0><<<grid, GeoT::THREADS, 0, st>>>(j);
        else     k_tn_bf16_dma_joint<GeoT, false, 0><<<grid, GeoT::THREADS, 0, st>>>(j);
    } else {
        if (f16) k_tn_bf16_dma_joint<GeoT, true, 2><<<grid, GeoT::THREADS, 0, st>>>(j);
        else     k_tn_bf16_dma_joint<GeoT, false, 2><<<grid, GeoT::THREADS, 0, st>>>(j);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // one launch folds the slices of all layers (+ noise): a fold per layer is a launch of a few microseconds each
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

// implicit unfolding: whole 16-byte pieces must stay inside one pixel's channels, image offsets must fit 32 bits
bool dma_conv_ok(const ConvGeom& g, int N) {
    const int64_t Hout = (int64_t)g.H + 2 * g.pad - g.KH + 1, Wout = (int64_t)g.W + 2 * g.pad - g.KW + 1;
    if (Hout < 1 || Wout < 1 || (g.C & 7) != 0) return false;
    if ((int64_t)g.H * g.W * g.C * 2 >= (int64_t(1) << 31)) return false;
    const int64_t T = Hout * Wout, M = (int64_t)g.KH * g.KW * g.C;
    if (T >= (int64_t(1) << 31) || M >= (int64_t(1) << 24)) return false;
    return T >= 64 && dma_geometry((int)T, (int)M, N) != 0;
}

// The direct norm stores nothing, and for long examples of few columns (positions x (576 -> 64) of an unfolded
// convolution) it is bound by reading them: there 128 x 128 tiles that are up to 60 % padding still beat the kernels
// that repack through registers (clamped columns are read again from L2, their products are masked out).
static bool direct_padded_ok(int T, int M, int N) {
    if (((M | N) & 7) != 0 || M < 32 || N < 32 || T < 4 * DK) return false;
    if ((T % DK) != 0 && (int64_t)ceil_div(T, DK) * DK * 4 > (int64_t)T * 5) return false;
    if ((int64_t)DK * (M > N ? M : N) * 2 >= (int64_t(1) << 31)) return false;
    const int64_t padded = (int64_t)ceil_div(M, GeoT::TM) * GeoT::TM * ceil_div(N, GeoT::TN) * GeoT::TN;
    return padded * 2 <= (int64_t)M * N * 5;
}
bool dma_direct_ok(int T, int M, int N) { return T >= 64 && (dma_geometry(T, M, N) != 0 || direct_padded_ok(T, M, N)); }

// Several layers' direct norms in one launch of 128 x 128 tiles (the long, narrow convolutions of an image model:
// a launch each is a few hundred workgroups and a tail; together they stream).  partial: per layer [B][tiles].
bool dma_direct_joint_ok(int B, int T, int M, int N) {
    if (!dma_direct_ok(T, M, N)) return false;
    // layers that tile well with 192 x 128 do better alone on those tiles once they are large (more flop per copied byte)
    if (dma_geometry(T, M, N) == 2 && (int64_t)B * T * ((int64_t)M + N) * 2 > (int64_t(32) << 20)) return false;
    if ((int64_t)T * (M > N ? M : N) * 2 >= (int64_t(1) << 31)) return false;       // ragged mode: lane offsets inside an example
    if (dma_geometry(T, M, N) == 1) return false;     // layers that fill 256 x 256 tiles are bound by the MFMA rate: their own launch
    return tiles_fit(M, N, GeoT::TM, GeoT::TN) || direct_padded_ok(T, M, N);
}
int direct_joint_tiles(int M, int N) { return ceil_div(M, GeoT::TM) * ceil_div(N, GeoT::TN); }

hipError_t launch_direct_bf16_dma_joint(const JointShape* sh, const JointOperands* op, float* const* partial, int n_layers,
                                        int B, hipStream_t st, bool f16) {
    if (n_layers < 1 || n_layers > kJointMax) return hipErrorInvalidValue;
    JointArgs j;
    int64_t first = 0;
    bool ragged = false;
    for (int l = 0; l < n_layers; ++l) {
        JointLayer& y = j.layer[l];
        y.A = op[l].A; y.G = op[l].G; y.clip = nullptr;
        y.slices = partial[l];
        y.accumulate = 0;
        y.T = sh[l].T; y.M = sh[l].M; y.N = sh[l].N;
        y.tiles_m = ceil_div(sh[l].M, GeoT::TM); y.tiles_n = ceil_div(sh[l].N, GeoT::TN);
        y.splits = B;                                   // one "slice" per example
        y.stages_per_split = ceil_div(sh[l].T, DK);
        y.stages_total = (int)((int64_t)B * y.stages_per_split);
        y.first_item = (int)first;
        first += (int64_t)y.tiles_m * y.tiles_n * B;
        ragged = ragged || (sh[l].T % DK) != 0;
    }
    if (first >= (int64_t(1) << 28)) return hipErrorInvalidValue;
    for (int l = n_layers; l < kJointMax; ++l) j.layer[l] = j.layer[0];
    j.n_layers = n_layers; j.n_items = (int)first; j.per_xcd = ceil_div(first, 8);
    j.B = B;
    const unsigned grid = 8u * (unsigned)j.per_xcd;
    if (ragged) {
        if (f16) k_tn_bf16_dma_joint<GeoT, true, 2, 1><<<grid, GeoT::THREADS, 0, st>>>(j);
        else     k_tn_bf16_dma_joint<GeoT, false, 2, 1><<<grid, GeoT::THREADS, 0, st>>>(j);
    } else {
        if (f16) k_tn_bf16_dma_joint<GeoT, true, 0, 1><<<grid, GeoT::THREADS, 0, st>>>(j);
        else     k_tn_bf16_dma_joint<GeoT, false, 0, 1><<<grid, GeoT::THREADS, 0, st>>>(j);
    }
    return hipGetLastError();
}

TnPlan plan_direct_bf16_dma(int B, int T, int M, int N) {
    const int geo = dma_geometry(T, M, N) != 0 ? pick_geometry(T, M, N, B) : 3;
    const GeoDims gd = geo_dims(geo);      // one workgroup per (example, tile)
    TnPlan p;
    p.tile_m = gd.tm; p.tile_n = gd.tn;
    p.tiles_m = ceil_div(M, p.tile_m); p.tiles_n = ceil_div(N, p.tile_n);
    p.segmented = false; p.big = false; p.dma = true;
    p.zero_head = (T % DK) != 0;
    p.splits = 1; p.kchunk = 0; p.epu = 1;
    return p;
}

hipError_t launch_direct_bf16_dma(const TnPlan& p, const uint16_t* A, const uint16_t* G, int B, int T, int M, int N,
                                  bool accumulate, float* sqnorm, float* partial, hipStream_t st,
                                  const ConvGeom* cg, const uint16_t* zero, bool f16, const ClipOut* co) {
    int am = cg ? 1 : 0;
    if (!cg && p.zero_head) {
        zero = static_cast<const uint16_t*>(device_zero_line(st));
        if (!zero) {
            const hipError_t ez = launch_fill_zero(partial, kZeroHeadFloats, st);
            if (ez != hipSuccess) return ez;
            zero = reinterpret_cast<const uint16_t*>(partial);
        }
        partial += kZeroHeadFloats;
        am = 2;
    }
    DmaArgs a;
    set_conv(a, cg, zero);
    a.A = A; a.G = G; a.clip = nullptr;
    a.B = B; a.T = T; a.M = M; a.N = N;
    a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n;
    a.splits = B;
    a.stages_total = (int)((int64_t)B * ceil_div(T, DK));
    a.stages_per_split = ceil_div(T, DK);
    a.out = partial; a.slice = 0; a.accumulate = 0;
    const int tiles = a.tiles_m * a.tiles_n;
    const int64_t total = (int64_t)tiles * B;
    if (total >= (int64_t(1) << 28)) return hipErrorInvalidValue;
    a.per_xcd = ceil_div(total, 8);
    const hipError_t e = launch_any<1>(geo_of_plan(p), a, am, f16, st);
    if (e != hipSuccess) return e;
    return launch_finalize_partials(partial, B, tiles, accumulate, sqnorm, st, co);
}

}  // namespace dpk
