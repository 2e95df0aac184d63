// Gram path of the per-example squared norm for aligned 16-bit (bf16 or fp16) and 8-bit (OCP e4m3 / e5m2) layers
// (d_in and d_out multiples of 128 bytes of elements: 64 for the 16-bit types, 128 for the 8-bit ones; T > 64):
//     ||A_i^T G_i||_F^2 = sum_{t,s} (A_i A_i^T)_{ts} (G_i G_i^T)_{ts}.
// Same decomposition as the generic Gram kernel (one workgroup per example
// and upper-triangular pair of 128-row tiles, both Gram tiles kept in MFMA
// accumulators of identical layout, multiplied lane by lane and reduced), with
// the gfx950 data path:
//   * row tiles are copied global -> LDS directly (global_load_lds_dwordx4, a
//     wave instruction moves 8 rows x 128 B), double buffered and one stage
//     ahead; the LDS reads run one k step ahead of the MFMAs; the chunk
//     permutation that makes the 16-byte LDS reads conflict free is applied to
//     the source addresses of the copy;
//   * workgroups of one example are dealt to the same XCD (workgroup b runs on
//     XCD b % 8), so the up to four re-reads of every row tile hit that XCD's
//     L2 instead of going out to memory;
//   * two workgroups per compute unit, so one computes while the other waits
//     at its stage barrier.
// Rows t >= T of a ragged last tile are read from a clamped (valid) row and
// masked out of the final product.
#include "dp_common.h"
#include "dp_internal.h"
#include <type_traits>

namespace dpk {

namespace {

constexpr int GT = 128;                 // rows of T per tile
constexpr int GK = 64;                  // contraction elements per stage, 16-bit types (128 B per row = one cache line)
constexpr int GK8 = 128;                // ... 8-bit types: the same 128 B
constexpr int ROWB = GK * 2;            // bytes per tile row in LDS
constexpr int CPR = ROWB / 16;          // 16-byte chunks per row
constexpr int RPI = 64 / CPR;           // rows per copy instruction (1 KB)
constexpr int IPT = GT / RPI / 4;       // copy instructions per tile and wave
constexpr int TILE_BYTES = GT * ROWB;
constexpr int GSTAGE = 2 * TILE_BYTES;  // t-tile then s-tile
constexpr int GNST = 2;                 // stages resident in LDS (64 KB: two workgroups per compute unit).  Measured
                                        // alternatives: GK = 32 with a 4-stage ring (half cache lines per row) 14 % slower,
                                        // 3 stages of GK = 64 with one workgroup per compute unit 7 % slower
#define LDS_PTR(T) __attribute__((address_space(3))) T*

// One launch covers up to kGramBatch layers: their (example, pair) work items form one list, so that the tail of
// one layer's work (10 items per example at T = 512 against 512 resident workgroups) is filled by the next layer's.
struct GramDmaLayer {
    const unsigned char* A;
    const unsigned char* G;
    int T, d_in, d_out;
    int nt, npairs;
    int first;           // index of the layer's first item in partial[]; its items are partial[first + ex * npairs + slot]
    int per_xcd;         // items of this layer per XCD queue: ceil(B * npairs / 8)
    float* upart;        // BIAS kernels: [B][nt][d_out] column sums of G over each row tile (nullptr: not wanted)
};
struct GramDmaArgs {
    GramDmaLayer layer[kGramBatch];
    int n_layers;
    float* partial;
    int B;
    int per_xcd;         // length of one XCD's queue: sum of the layers' per_xcd
};

// chunk c (16 B) of tile row r sits at chunk position c ^ swz(r) so that 16 consecutive rows reading the same
// logical chunk cover all 64 banks once: with 128-byte rows the row parity selects the upper or lower 128 bytes
// and (r >> 1) & 7 spreads the rest; with 64-byte rows r & 3 selects a 64-byte window and (r >> 2) & 3 spreads.
template <int N> __device__ __forceinline__ void wait_vm() { __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70); }

__device__ __forceinline__ int gram_swz(int r) { return CPR == 8 ? ((r >> 1) & 7) : ((r >> 2) & 3); }

typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef int v8i32 __attribute__((ext_vector_type(8)));

// Input formats.  0: bf16, 1: fp16 (v_mfma_f32_32x32x16_{bf16,f16}); 2: A and G e4m3, 3: A and G e5m2, 4: A e4m3 and
// G e5m2 (v_mfma_f32_32x32x64_f8f6f4, whose format fields take 0 for e4m3 and 1 for e5m2).  Both operands of a Gram
// product come from the same matrix, so one field value per phase serves both.
__host__ __device__ constexpr bool fmt_is8(int fmt) { return fmt >= 2; }
__host__ __device__ constexpr int fmt8_of_A(int fmt) { return fmt == 3 ? 1 : 0; }
__host__ __device__ constexpr int fmt8_of_G(int fmt) { return fmt >= 3 ? 1 : 0; }
template <int F8> __device__ __forceinline__ f32x16 mfma8(v8i32 x, v8i32 y, f32x16 c) {
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(x, y, c, F8, F8, 0, 0, 0, 0);
}

// BIAS: the diagonal pairs (every row tile belongs to exactly one) also take the column sums of their 128 rows of
// G, sum_t G_i[t, :] over the tile, which is the tile's share of the example's bias gradient (Section 5.1: the
// bias gradient is dLoss/dz, summed over the positions that share the bias): while a 64-column stage of G sits in
// LDS, each wave multiplies a row of ones (zeros for rows beyond T) with the transpose of its 32 rows -- read with
// the transposing LDS load -- on the matrix unit, 4 extra MFMAs next to the 16 of the stage; the four partial sums
// meet in LDS and wave 0 writes the stage's 64 sums to upart.  The pass over G that a separate bias kernel needs
// is saved.
template <int FMT, bool BIAS>
__global__ __launch_bounds__(kThreads, GNST * GSTAGE <= 65536 ? 2 : 1) void k_gram_bf16_dma(GramDmaArgs a) {
    constexpr bool F16 = FMT == 1, F8 = fmt_is8(FMT);
    constexpr int ES = F8 ? 1 : 2;                       // bytes per element
    constexpr int GKE = ROWB / ES;                       // elements per stage
    static_assert(!(F8 && BIAS), "the column sums are built for the 16-bit types");
    __shared__ __attribute__((aligned(1024))) unsigned char lds[GNST * GSTAGE];
    __shared__ float red[4];
    __shared__ float ub[BIAS ? 2 * 4 * GK : 1];          // [stage parity][wave][column of the stage]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // Work order.  Consecutive workgroup ids go round the 8 XCDs, so id & 7 names the XCD (and its L2) and
    // id >> 3 the position in that XCD's queue.  Each XCD takes a contiguous eighth of every layer's
    // (example, pair) list, example-major, one layer after the other: the pairs of one example run on one XCD at
    // about the same time and share its L2 (measured: 1.09x the algorithmic bytes from HBM; with the diagonal
    // pairs moved to the end of the queue 1.5x for the same run time), and every XCD gets the same mix of layers.
    const int xcd = blockIdx.x & 7;
    int q = blockIdx.x >> 3;
    int li = 0;
    while (li < a.n_layers && q >= a.layer[li].per_xcd) { q -= a.layer[li].per_xcd; ++li; }
    if (li >= a.n_layers) return;
    const GramDmaLayer ly = a.layer[li];
    const int L = xcd * ly.per_xcd + q;                 // item of this layer
    if (L >= a.B * ly.npairs) return;
    const int ex = L / ly.npairs;
    const int slot = L - ex * ly.npairs;                // position in the row-major list of (tt, ss), tt <= ss
    int pair = slot, tt = 0;
    while (pair >= ly.nt - tt) { pair -= ly.nt - tt; ++tt; }
    const int ss = tt + pair;
    const bool diag = (tt == ss);

    const int sa = ly.d_in / GKE, sg = ly.d_out / GKE;    // stages of the A phase and of the G phase
    const int n_stages = sa + sg;

    // ---- copies: wave w moves rows 32w .. 32w+31 of the t-tile and of the s-tile, 4 instructions each
    //      (instruction u: rows 32w + 8u .. + 7; lane / 8 picks the row, lane % 8 the chunk position)
    const int lrow8 = lane / CPR, cp = lane % CPR;
    // per-lane byte offsets inside the example (tile rows clamped to valid rows), fixed for the whole kernel:
    // [0] = A phase, [1] = G phase
    uint32_t off_t[2][IPT], off_s[2][IPT];
#pragma unroll
    for (int u = 0; u < IPT; ++u) {
        const int r = wave * 32 + u * RPI + lrow8;                     // row inside the tile
        const uint32_t c16 = (uint32_t)((cp ^ gram_swz(r)) << 4);      // source chunk for this LDS slot
        const uint32_t rt = (uint32_t)min(tt * GT + r, ly.T - 1), rs = (uint32_t)min(ss * GT + r, ly.T - 1);
        off_t[0][u] = rt * (uint32_t)ly.d_in * ES + c16;  off_s[0][u] = rs * (uint32_t)ly.d_in * ES + c16;
        off_t[1][u] = rt * (uint32_t)ly.d_out * ES + c16; off_s[1][u] = rs * (uint32_t)ly.d_out * ES + c16;
    }
    const unsigned char* baseA = ly.A + (size_t)ex * ly.T * ly.d_in * ES;    // uniform example bases; lane offsets stay 32-bit
    const unsigned char* baseG = ly.G + (size_t)ex * ly.T * ly.d_out * ES;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(LDS_PTR(unsigned char))lds;
    const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(lds_base + wave * 32 * ROWB);
    // The copies are inline assembly so that the compiler does not tie every LDS read to them; they are
    // waited for with the explicit vmcnt wait in front of the stage barrier.
    auto issue_phase = [&](const unsigned char* sbase, const uint32_t (&ot)[IPT], const uint32_t (&os)[IPT], int buf) {
        const uint32_t base = wave_lds + buf * GSTAGE;
#pragma unroll
        for (int u = 0; u < IPT; ++u)
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(base + u * 1024), "v"(ot[u]), "s"(sbase) : "memory", "m0");
        if (!diag) {
#pragma unroll
            for (int u = 0; u < IPT; ++u)
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(base + TILE_BYTES + u * 1024), "v"(os[u]), "s"(sbase) : "memory", "m0");
        }
    };
    auto issue = [&](int st, int buf) {
        if (st < sa) issue_phase(baseA + st * ROWB, off_t[0], off_s[0], buf);
        else issue_phase(baseG + (st - sa) * ROWB, off_t[1], off_s[1], buf);
    };

    // ---- MFMA roles: 2 x 2 waves, each owns 64 x 64 of the 128 x 128 tile pair
    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = lane & 31, lhalf = lane >> 5;
    int rd_t[2], rd_s[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int rt = wm * 64 + i * 32 + lrow, rs = wn * 64 + i * 32 + lrow;
        rd_t[i] = rt * ROWB + ((lhalf ^ gram_swz(rt)) << 4);
        rd_s[i] = (diag ? 0 : TILE_BYTES) + rs * ROWB + ((lhalf ^ gram_swz(rs)) << 4);
    }
    f32x16 accP[2][2], accQ[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) { accP[i][j][r] = 0.f; accQ[i][j][r] = 0.f; }
    // A diagonal pair is symmetric: the 64 x 64 block of wave (0, 1) is the transpose of wave (1, 0)'s, and inside the
    // blocks of waves (0, 0) and (1, 1) the 32 x 32 block (0, 1) is the transpose of block (1, 0).  The upper ones are
    // not computed (wave (0, 1) issues no MFMA and reads no fragment, it only copies and keeps the barriers) and the
    // lower ones count twice: 10 of the 16 MFMAs of a k step.  (Letting waves (0, 0) and (1, 1) also use their t
    // fragments as s fragments, two LDS reads fewer per k step, made the kernel 50 % slower: a second MFMA sequence
    // on other registers in the pipelined loop.)
    const bool skip_wave = __builtin_amdgcn_readfirstlane((int)(diag && wm < wn)) != 0;
    const bool skip_upper = __builtin_amdgcn_readfirstlane((int)(diag && wm == wn)) != 0;

    // ---- BIAS: operands of the column sums.  Wave w takes rows 32 w .. 32 w + 31 of the t-tile as two 16-row k steps.
    const bool do_bias = BIAS && diag && ly.upart != nullptr;
    bf16x8 ones[2];
    int rdu[2];                                       // byte offset in the t-tile of this lane's piece: rows +0 / +4 of the first
                                                      // k step, columns 0-31; second k step: + 16 rows, columns 32-63: ^ 64
    f32x16 au[2];
    bf16x8 fu[2];
    if (BIAS) {
        const int g16 = lane >> 4, s16 = lane & 15, half = g16 >> 1;
        const uint32_t one = F16 ? 0x3C00u : 0x3F80u;
#pragma unroll
        for (int kl = 0; kl < 2; ++kl) {
            const int k0 = (2 * wave + kl) * 16 + 8 * half;          // first of this lane's 8 rows
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t lo = (tt * GT + k0 + 2 * e < ly.T) ? one : 0u, hi = (tt * GT + k0 + 2 * e + 1 < ly.T) ? one : 0u;
                w[e] = lo | (hi << 16);
            }
            ones[kl] = __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
        }
        const int na = 16 * (g16 & 1) + 4 * (s16 & 3);               // column (element) of the 8-byte piece
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int r = 2 * wave * 16 + 8 * half + (s16 >> 2) + 4 * h;
            rdu[h] = r * ROWB + ((((na >> 3) ^ gram_swz(r)) << 4) | ((na & 7) << 1));
        }
    }
    // this wave's 16 rows of k step kl, transposed: 8 rows x 32 columns per lane half, both 32-column blocks.
    // Rows + 16 keep their chunk permutation ((r >> 1) & 7), columns + 32 flip bit 2 of the chunk index.
    auto read_u = [&](int buf, int kl) {
        LDS_PTR(unsigned char) b = (LDS_PTR(unsigned char))lds + buf * GSTAGE + kl * 16 * ROWB;
#pragma unroll
        for (int nf = 0; nf < 2; ++nf) {
            const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(v4i16))(b + (rdu[0] ^ (nf << 6))));
            const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(v4i16))(b + (rdu[1] ^ (nf << 6))));
            fu[nf] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
    };
    // sums of stage `st` (written to ub by the four waves before the barrier that ended it) -> upart; wave 0 only
    auto flush_u = [&](int st) {
        const float* p = ub + (st & 1) * 4 * GK;
        const float v = ((p[lane] + p[GK + lane]) + p[2 * GK + lane]) + p[3 * GK + lane];
        ly.upart[((size_t)ex * ly.nt + tt) * ly.d_out + (size_t)(st - sa) * GK + lane] = v;
    };

    // Software pipeline over k steps (4 per stage): the LDS reads of the next k step are in flight while the
    // MFMAs of the current one run, also across the stage boundary; the stage barrier sits in front of the
    // last k step of a stage, when every wave has retired its reads of that stage.
    auto read_kstep = [&](bf16x8 (&f)[4], int buf, int ks) {
        if (skip_wave) return;
        const unsigned char* sb = lds + buf * GSTAGE;
        // chunk (2 ks + lhalf) ^ swz == (lhalf ^ swz) ^ (2 ks): flip bits 5-6 of the byte offset
#pragma unroll
        for (int i = 0; i < 2; ++i) f[i] = *reinterpret_cast<const bf16x8*>(sb + (rd_t[i] ^ (ks << 5)));
#pragma unroll
        for (int j = 0; j < 2; ++j) f[2 + j] = *reinterpret_cast<const bf16x8*>(sb + (rd_s[j] ^ (ks << 5)));
    };
    auto mfma_kstep = [&](const bf16x8 (&f)[4], f32x16 (&acc)[2][2]) {
        if (skip_wave) return;
        acc[0][0] = In16<F16>::mfma(f[0], f[2], acc[0][0]);
        acc[1][0] = In16<F16>::mfma(f[1], f[2], acc[1][0]);
        acc[1][1] = In16<F16>::mfma(f[1], f[3], acc[1][1]);
        if (!skip_upper) acc[0][1] = In16<F16>::mfma(f[0], f[3], acc[0][1]);
    };
    bf16x8 f[2][4];
    // wait until at most `stages` later stages' copies are outstanding (4 per wave and stage on a diagonal pair, else 8)
    auto wait_copies = [&](int stages) {
        // copies per wave and stage: IPT on a diagonal pair, else 2 * IPT
        if (stages <= 0) wait_vm<0>();
        else if (stages == 1) { if (diag) wait_vm<IPT>(); else wait_vm<2 * IPT>(); }
        else if (stages == 2) { if (diag) wait_vm<2 * IPT>(); else wait_vm<4 * IPT>(); }
        else { if (diag) wait_vm<3 * IPT>(); else wait_vm<6 * IPT>(); }
    };
    auto stage = [&](int st, f32x16 (&acc)[2][2]) {
#pragma unroll
        for (int ks = 0; ks < GK / 16; ++ks) {
            if (BIAS && ks == GK / 16 - 1 && do_bias && st >= sa) {
                // hand the stage's 64 column sums over, in front of the barrier that ends the stage (the MFMAs that
                // made them were issued a k step ago).  Every row of the 32 x 32 result is the same; element 0 of
                // lanes 0-31 is row 0, column lane.
#pragma unroll
                for (int nf = 0; nf < 2; ++nf)
                    if (lane < 32) ub[(st & 1) * 4 * GK + wave * GK + nf * 32 + lane] = au[nf][0];
            }
            __builtin_amdgcn_s_waitcnt(0xC07F);              // lgkmcnt(0): this k step's fragments (requested a k step ago)
            if (ks + 1 < GK / 16) {
                read_kstep(f[(ks + 1) & 1], st % GNST, ks + 1);
            } else if (st + 1 < n_stages) {
                // the copies of stage st + 1 must have landed; those of stage st + 2 (4 per wave on a diagonal
                // pair, else 8) may stay in flight
                wait_copies(min(n_stages - 2 - st, GNST - 2));
                __builtin_amdgcn_s_barrier();                // ... for every wave, and every wave is done reading stage st
                if (st + GNST < n_stages) issue(st + GNST, st % GNST);
                read_kstep(f[0], (st + 1) % GNST, 0);
            }
            mfma_kstep(f[ks & 1], acc);
            if (BIAS && do_bias && st >= sa) {
                // k step 0: request this wave's first 16 rows of the stage (transposed); 1 and 2: one 16-row step each
                // on the matrix unit (1 also requests the second 16 rows).  All before the barrier in k step 3 that
                // frees the buffer.
                if (ks == 0) {
                    if (wave == 0 && st > sa) flush_u(st - 1);
                    read_u(st % GNST, 0);
                } else if (ks == 1) {
#pragma unroll
                    for (int nf = 0; nf < 2; ++nf) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) au[nf][r] = 0.f;
                        au[nf] = In16<F16>::mfma(ones[0], fu[nf], au[nf]);
                    }
                    read_u(st % GNST, 1);
                } else if (ks == 2) {
#pragma unroll
                    for (int nf = 0; nf < 2; ++nf) au[nf] = In16<F16>::mfma(ones[1], fu[nf], au[nf]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // 8-bit types: a stage row holds 128 elements = two k steps of the 64-deep MFMA.  A lane's 32 bytes of a k step
    // are the two 16-byte pieces that the 16-bit path reads in its k steps 2 K and 2 K + 1 (elements 16 h .. 16 h + 15
    // and 32 + 16 h .. of the 64, h = lane / 32): which k a byte position stands for does not matter as long as both
    // operands agree, and they are read the same way.
    v8i32 f8[2][4];
    auto read_k8 = [&](v8i32 (&g)[4], int buf, int K) {
        if (skip_wave) return;
        const unsigned char* sb = lds + buf * GSTAGE;
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int o = x < 2 ? rd_t[x] : rd_s[x - 2];
            const uint4 lo = *reinterpret_cast<const uint4*>(sb + (o ^ ((2 * K) << 5)));
            const uint4 hi = *reinterpret_cast<const uint4*>(sb + (o ^ ((2 * K + 1) << 5)));
            g[x] = v8i32{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
        }
    };
    auto stage8 = [&](int st, f32x16 (&acc)[2][2], auto tag) {
        constexpr int F = decltype(tag)::value;
#pragma unroll
        for (int K = 0; K < 2; ++K) {
            __builtin_amdgcn_s_waitcnt(0xC07F);              // lgkmcnt(0): this k step's fragments (requested a k step ago)
            if (K == 0) {
                read_k8(f8[1], st % GNST, 1);
            } else if (st + 1 < n_stages) {
                wait_copies(min(n_stages - 2 - st, GNST - 2));
                __builtin_amdgcn_s_barrier();
                if (st + GNST < n_stages) issue(st + GNST, st % GNST);
                read_k8(f8[0], (st + 1) % GNST, 0);
            }
            if (!skip_wave) {
                acc[0][0] = mfma8<F>(f8[K][0], f8[K][2], acc[0][0]);
                acc[1][0] = mfma8<F>(f8[K][1], f8[K][2], acc[1][0]);
                acc[1][1] = mfma8<F>(f8[K][1], f8[K][3], acc[1][1]);
                if (!skip_upper) acc[0][1] = mfma8<F>(f8[K][0], f8[K][3], acc[0][1]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

#pragma unroll
    for (int p = 0; p < GNST; ++p)
        if (p < n_stages) issue(p, p);
    wait_copies(min(n_stages, GNST) - 1);                        // stage 0 must have landed
    __builtin_amdgcn_s_barrier();
    if constexpr (F8) {
        read_k8(f8[0], 0, 0);
        for (int st = 0; st < sa; ++st) stage8(st, accP, std::integral_constant<int, fmt8_of_A(FMT)>{});
        for (int st = sa; st < n_stages; ++st) stage8(st, accQ, std::integral_constant<int, fmt8_of_G(FMT)>{});
    } else {
        read_kstep(f[0], 0, 0);
        for (int st = 0; st < sa; ++st) stage(st, accP);              // A A^T tile
        for (int st = sa; st < n_stages; ++st) stage(st, accQ);       // G G^T tile
    }

    // ---- sum of the elementwise product; rows / columns beyond T are masked (their tiles hold clamped rows)
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = ss * GT + wn * 64 + j * 32 + lrow;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = tt * GT + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
                const float v = accP[i][j][r] * accQ[i][j][r];
                const float wgt = !diag ? 1.f : wm > wn ? 2.f : (i == j ? 1.f : i > j ? 2.f : 0.f);   // skipped blocks hold zeros
                s += (row < ly.T && col < ly.T) ? wgt * v : 0.f;
            }
        }
    __syncthreads();
    if (BIAS && do_bias && wave == 0) flush_u(n_stages - 1);
    s = block_sum_256(s, red);
    if (tid == 0) a.partial[(size_t)ly.first + (size_t)ex * ly.npairs + slot] = diag ? s : 2.0f * s;
}

}  // namespace

bool gram_dma_ok(int T, int d_in, int d_out, int fmt) {
    const int64_t dmax = d_in > d_out ? d_in : d_out;
    const int es = fmt_is8(fmt) ? 1 : 2, gke = ROWB / es;
    return T > 64 && (d_in % gke) == 0 && (d_out % gke) == 0 && (int64_t)T * dmax * es < (int64_t(1) << 31);   // 32-bit lane offsets
}

// Several layers in one launch (at most kGramBatch, every one passing gram_dma_ok); partial gets the layers' item
// lists one after the other, in the order given, and the sums go to sqnorm in that order.
hipError_t launch_gram_bf16_dma_layers(const GramLayerDesc* layers, int n_layers, int B, bool accumulate, float* sqnorm,
                                       float* partial, hipStream_t st, int fmt, float C, float* clip) {
    if (n_layers < 1 || n_layers > kGramBatch || fmt < 0 || fmt > 4) return hipErrorInvalidValue;
    GramDmaArgs a;
    FinalizeLayers fin;
    a.n_layers = n_layers; a.partial = partial; a.B = B;
    fin.n_layers = n_layers;
    int64_t first = 0, queue = 0;
    bool any_bias = false;
    for (int l = 0; l < n_layers; ++l) {
        const GramPlan p = plan_gram_bf16(layers[l].T, layers[l].d_in, layers[l].d_out);
        GramDmaLayer& y = a.layer[l];
        y.A = static_cast<const unsigned char*>(layers[l].A); y.G = static_cast<const unsigned char*>(layers[l].G);
        y.T = layers[l].T; y.d_in = layers[l].d_in; y.d_out = layers[l].d_out;
        y.nt = p.nt; y.npairs = p.npairs;
        const int64_t items = (int64_t)B * p.npairs;
        if (first + items >= (int64_t(1) << 31)) return hipErrorInvalidValue;
        y.first = (int)first;
        y.per_xcd = (int)((items + 7) / 8);
        y.upart = layers[l].upart;
        any_bias = any_bias || y.upart != nullptr;
        fin.first[l] = (int)first; fin.n[l] = p.npairs;
        first += items;
        queue += y.per_xcd;
    }
    for (int l = n_layers; l < kGramBatch; ++l) a.layer[l] = GramDmaLayer{nullptr, nullptr, 0, 0, 0, 0, 0, 0, 0, nullptr};
    if (queue * 8 >= (int64_t(1) << 31)) return hipErrorInvalidValue;
    a.per_xcd = (int)queue;
    const unsigned grid = 8u * (unsigned)a.per_xcd;
    if (any_bias) {
        if (fmt == 0) k_gram_bf16_dma<0, true><<<grid, kThreads, 0, st>>>(a);
        else if (fmt == 1) k_gram_bf16_dma<1, true><<<grid, kThreads, 0, st>>>(a);
        else return hipErrorInvalidValue;                     // 8-bit types: the caller takes the bias rows in a pass of their own
    } else if (fmt == 0) k_gram_bf16_dma<0, false><<<grid, kThreads, 0, st>>>(a);
    else if (fmt == 1) k_gram_bf16_dma<1, false><<<grid, kThreads, 0, st>>>(a);
    else if (fmt == 2) k_gram_bf16_dma<2, false><<<grid, kThreads, 0, st>>>(a);
    else if (fmt == 3) k_gram_bf16_dma<3, false><<<grid, kThreads, 0, st>>>(a);
    else               k_gram_bf16_dma<4, false><<<grid, kThreads, 0, st>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (layers[0].out) {
        // an output array per layer (groups share one): the bias folds first, then the layers' sums, each adding to
        // its array if the array holds a value by then; a group's clip factors go with its last layer
        int canon[kGramBatch];
        bool holds[kGramBatch];
        for (int l = 0; l < n_layers; ++l) {
            if (!layers[l].out) return hipErrorInvalidValue;
            canon[l] = l;
            for (int j = 0; j < l; ++j)
                if (layers[j].out == layers[l].out) { canon[l] = canon[j]; break; }
            holds[l] = layers[l].out_acc;
        }
        for (int l = 0; l < n_layers; ++l) {
            if (!layers[l].upart) continue;
            e = launch_bias_fold(layers[l].upart, B, a.layer[l].nt, layers[l].d_out, holds[canon[l]], layers[l].bias_rows, layers[l].out, st);
            if (e != hipSuccess) return e;
            holds[canon[l]] = true;
        }
        FinalizeEach fe;
        fe.n_layers = n_layers;
        for (int l = 0; l < kGramBatch; ++l) { fe.first[l] = 0; fe.n[l] = 0; fe.acc[l] = 0; fe.C[l] = 0.f; fe.out[l] = nullptr; fe.clip[l] = nullptr; }
        for (int l = 0; l < n_layers; ++l) {
            fe.first[l] = fin.first[l]; fe.n[l] = fin.n[l];
            fe.out[l] = layers[l].out;
            fe.acc[l] = holds[canon[l]] ? 1 : 0;
            holds[canon[l]] = true;
            bool last = true;
            for (int j = l + 1; j < n_layers; ++j) last = last && layers[j].out != layers[l].out;
            fe.C[l] = layers[l].out_C;
            fe.clip[l] = last ? layers[l].out_clip : nullptr;
        }
        return launch_finalize_each(partial, fe, B, st);
    }
    // bias rows and their share of the norms first, so that the finalize kernel below (which may write the clip
    // factors) sees complete sums
    for (int l = 0; l < n_layers; ++l) {
        if (!layers[l].upart) continue;
        e = launch_bias_fold(layers[l].upart, B, a.layer[l].nt, layers[l].d_out, accumulate, layers[l].bias_rows, sqnorm, st);
        if (e != hipSuccess) return e;
        accumulate = true;
    }
    return launch_finalize_layers(partial, fin, B, accumulate, sqnorm, st, C, clip);
}

hipError_t launch_gram_bf16_dma(const GramPlan& p, const void* A, const void* G, int B, int T, int d_in, int d_out,
                                bool accumulate, float* sqnorm, float* partial, hipStream_t st, int fmt, const ClipOut* co) {
    (void)p;
    const GramLayerDesc one{A, G, T, d_in, d_out, nullptr, nullptr};
    return launch_gram_bf16_dma_layers(&one, 1, B, accumulate, sqnorm, partial, st, fmt, co ? co->C : 0.f, co ? co->clip : nullptr);
}

}  // namespace dpk
