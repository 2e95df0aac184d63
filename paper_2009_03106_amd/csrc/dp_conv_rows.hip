// 3 x 3 stride-1 convolution layers from their input image, with the image rows resident in LDS: direct squared
// norm and clipped sum of  A_i^T G_i  where A_i is the unfolded patch matrix of Algorithm 3 (Section 5.2, column
// order (kh, kw, c)) that is never formed.
//
// The general copy-pipeline kernel gathers every patch element from the image again (nine copies of each pixel,
// global -> LDS).  Here a workgroup keeps a ring of padded image rows in LDS (64 channels of every pixel, zeros
// around the image written by the same copies) and copies each pixel once; the nine taps are nine LDS addresses of
// the same pixels: the fragment of tap (kh, kw) for output position (y, x) is read at padded pixel (y + kh, x + kw).
//
// Work split: a workgroup owns 64 input channels x 9 taps = 576 rows of the gradient and 64 of its columns.  It has
// 8 waves, two per SIMD: waves 0 .. 3 compute, wave w owns channels 16 w .. 16 w + 15 of every tap (nine
// 16 x 16 x 32 MFMA row blocks, the tap is the block index, so the tap offsets are constants of the code) and all
// four 16-column blocks of G; a stage is 32 output positions = one MFMA step, per stage a wave reads 9 + 4
// fragments for 36 MFMAs.  Waves 4 .. 7 only copy (global -> LDS needs no registers): the address arithmetic of the
// copies then runs beside the MFMAs of the computing wave on the same SIMD instead of in front of them - with one
// wave per SIMD a stage took the time of its ~300 other instructions, not of its 36 MFMAs.  The two kinds of waves
// meet at one barrier per stage: behind it stage st + 1 has landed (the copying waves waited for it) and stage st
// is in the computing waves' registers, so its LDS may be written again.
//
// LDS: pixels are 160 bytes apart (128 bytes of channels + 32): eight consecutive pixels then start in eight
// different 32-byte bank windows, which is what a transposing read of 32 lanes touches.  The image is a stream of
// padded rows (example after example of a K slice), cut into 1 KB units that the waves copy in order into a ring
// of `ring_rows` rows; a unit may only be written when the rows it replaces are dead, and must have been issued
// together with (or before) the G rows of the first stage that reads it, so that the stage's wait on the copy
// counter covers it.  The host simulates that schedule for a geometry before it chooses this kernel.
#include <algorithm>
#include <type_traits>
#include "dp_common.h"
#include "dp_internal.h"

namespace dpk {

namespace {

constexpr int DK = 32;                 // output positions per stage
constexpr int TAPS = 9, KW3 = 3;
constexpr int CW = 4;                  // computing waves: 4 (each all 64 columns) or 8 (two per SIMD, 32 columns each)
constexpr int FNB = 16 / CW, TN = 64;  // 16-column blocks per computing wave, columns per workgroup
constexpr int THREADS = 64 * (CW + 4);
constexpr int CG = 64;                 // input channels per workgroup
constexpr int PITCH = 2 * CG + 32;     // bytes from a pixel to the next in LDS
constexpr int CPP = PITCH / 16;        // 16-byte chunks per pixel (the last two are padding)
constexpr int NSTG = 4;                // stages of G resident
constexpr int G_STAGE = DK * TN * 2;   // bytes
constexpr int NI = 4;                  // image copies per wave and stage
constexpr int LPS = 1 + NI;            // copies per wave and stage
constexpr int TABLE_BYTES = 4096;      // copy offsets of the 16-byte chunks of a padded row
constexpr int LDS_TABLE = NSTG * G_STAGE + 1024;
constexpr int LDS_FIXED = LDS_TABLE + TABLE_BYTES;   // G stages, the 1 KB that takes the copies with nothing to bring, the table
constexpr int LDS_MAX = 152 * 1024;  // one workgroup per compute unit (its 8 waves take the registers anyway)

typedef short v4i16 __attribute__((ext_vector_type(4)));
#define LDS_PTR(T) __attribute__((address_space(3))) T*

struct ConvRowsArgs {
    const uint16_t* X;     // [B, H, W, C]
    const uint16_t* G;     // [B, T, N]
    const float* clip;
    float* out;            // clipped sum: slice base (stride `slice`) or grad; direct norm: partial[B][tiles]
    int64_t slice;
    const uint16_t* zero;  // at least 16 bytes of zeros
    int B, T, N, C, H, W, pad, Wout, Hp, Wp;
    int rowbytes;          // bytes of a padded row in LDS, a multiple of the 1 KB copy unit
    int cpr, rps;          // copies per wave and row (units per row / 4, rounded up), rows per round: cpr * rps = NI
    int dx32, dy32;        // 32 % Wout, 32 / Wout: how a position moves from a stage to the next
    int ring_rows;         // power of two
    int pre_rounds;        // rounds of image copies before the first stage's
    uint32_t mg_wout, mg_upr, mg_hp, mg_ring;      // reciprocals (see fastdiv) of Wout, units per row, Hp, ring units
    int tiles_m, tiles_n, ex_per_slice, splits, per_xcd, accumulate;
};

// n / d for n * d < 2^32, with mg = 2^32 / d + 1 (d >= 2)
__device__ __forceinline__ uint32_t fastdiv(uint32_t n, uint32_t mg) { return __umulhi(n, mg); }
inline uint32_t magic_of(uint32_t d) { return (uint32_t)((uint64_t(1) << 32) / d) + 1u; }

#ifdef DP_CONV_ROWS_TRACE
__device__ unsigned long long g_trace[8 * 256];
#define TRACE(k, st) do { if (L == 0 && lane == 0 && (wave12 == 0 || wave12 == CW) && (st) < 256) g_trace[(k) * 256 + (st)] = __builtin_amdgcn_s_memtime(); } while (0)
#else
#define TRACE(k, st) do {} while (0)
#endif
template <int N> __device__ __forceinline__ void wait_vmcnt() { __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14)); }

// MODE 0: clipped sum over the examples of a K slice.  MODE 1: direct squared norm of one example's tile.
// RAG: the output positions of an example are not a multiple of the 32-position stage (28 x 28, 14 x 14, 7 x 7 ...):
// every example takes ceil(T / 32) stages; the rows of G past its end are copied from the line of zeros, and the
// image fragments of those positions are whatever the ring holds there - finite values, since the ring is cleared
// before the first copy - so their products are exact zeros.
template <int MODE, bool F16, bool RAG>
__global__ __launch_bounds__(THREADS, 1) void k_conv3x3_rows(ConvRowsArgs a) {
    __shared__ __attribute__((aligned(1024))) unsigned char lds[LDS_MAX];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave12 = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool copier = wave12 >= CW;
    const int wave = wave12 & 3;                    // copying: which quarter of the units; computing: which 16 channels
    const int hcol = CW == 8 ? (wave12 >> 2) & 1 : 0;    // computing, 8 waves: which 32 of the 64 columns
    const int L = (blockIdx.x & 7) * a.per_xcd + (blockIdx.x >> 3);
    const int tiles = a.tiles_m * a.tiles_n;
    if (L >= tiles * a.splits) return;
    const int z = L / tiles, tile = L - z * tiles;
    const int tm = tile / a.tiles_n, tn = tile - tm * a.tiles_n;
    const int cbase = tm * CG, n0 = tn * TN;
    const int ex0 = z * a.ex_per_slice;
    const int E = min(a.ex_per_slice, a.B - ex0);
    const int spe = RAG ? (a.T + DK - 1) / DK : a.T / DK;
    const int n_stages = E * spe;
    const uint32_t upr = (uint32_t)a.rowbytes >> 10;                  // copy units per padded row
    const uint32_t ring_units = (uint32_t)a.ring_rows * upr;
    const uint32_t u_total = (uint32_t)E * (uint32_t)a.Hp * upr;

    const uint32_t lds_base = (uint32_t)(uintptr_t)(LDS_PTR(unsigned char))lds;
    const uint32_t lds_g = lds_base + wave * 1024;
    const uint32_t lds_dump = lds_base + NSTG * G_STAGE;
    const uint32_t lds_ring = lds_base + LDS_FIXED;

    // Where the 16-byte chunks of a padded row come from: byte offset inside the image row, or all ones for the
    // chunks of the zero border, of the padding behind a pixel's channels and behind the row.
    LDS_PTR(uint32_t) table = (LDS_PTR(uint32_t))((LDS_PTR(unsigned char))lds + LDS_TABLE);
    for (uint32_t c = tid; c < (upr << 6); c += THREADS) {
        const uint32_t px = c / CPP, ch = c - px * CPP, ix = px - (uint32_t)a.pad;
        table[c] = (ch < CG / 8 && ix < (uint32_t)a.W) ? (ix * (uint32_t)a.C + ch * 8u) * 2u : 0xFFFFFFFFu;
    }
    if (RAG) {
        const uint32_t n16 = ((uint32_t)a.ring_rows * (uint32_t)a.rowbytes) >> 4;
        LDS_PTR(f32x4) ring16 = (LDS_PTR(f32x4))((LDS_PTR(unsigned char))lds + LDS_FIXED);
        for (uint32_t c = tid; c < n16; c += THREADS) ring16[c] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    __syncthreads();

    // ---- copies.  G: a stage is 32 rows of 128 bytes = 4 units, one per wave; the 32-byte window v of row r sits at
    //      window v ^ ((r >> 1) & 3), so that rows r .. r + 7 of one window land in eight different bank windows.
    uint32_t offG;
    {
        const int idx = wave * 64 + lane, r = idx >> 3, pos = idx & 7;
        const int win = (pos >> 1) ^ ((r >> 1) & 3);
        int col = n0 + (((win << 1) | (pos & 1)) << 3);
        if (col >= a.N) col = n0;                   // columns past d_out feed outputs that are never used
        offG = ((uint32_t)r * (uint32_t)a.N + (uint32_t)col) * 2u;
    }
    const uint16_t* baseG = a.G + (size_t)ex0 * a.T * a.N;
    const size_t stepG = (size_t)DK * a.N;
    const int rowG = (wave * 64 + lane) >> 3;       // RAG: this lane's row of the stage, and the stage being issued
    int ie = 0, isub = 0;
    const uint16_t* baseX = a.X + (size_t)ex0 * a.H * a.W * a.C + cbase;
    int oe = 0, osub = 0;                           // the oldest stage that still reads the ring: example, stage in it

    // Image: a stream of padded rows, example after example.  A round issues the next a.rps image rows (none when
    // the ring is full): copy c < a.cpr of wave w moves unit 4 c + w of a row, so a lane's source offsets inside a
    // row are constants, and which row comes next is a few scalar additions - every copy instruction takes the
    // compute unit's address path some 64 cycles, so the copies that bring nothing are the ones to avoid.  The rows
    // of the zero border above and below the image are not copied but written (ds_write) when the stream passes
    // them; the border pixels left and right and the units' tails read the line of zeros.
    uint32_t rnext = 0;                             // stream rows issued so far
    uint32_t rho = 0;                               // padded row inside its example of stream row rnext
    uint64_t rowptr = (uint64_t)(uintptr_t)baseX;   // the next image row to copy
    const uint32_t rowstride = (uint32_t)a.W * (uint32_t)a.C * 2u;
    const uint32_t rows_total = (uint32_t)E * (uint32_t)a.Hp;
    // copy i of a round moves unit 4 (i % cpr) + wave of its row, if the row has that many units
    uint32_t toffc[NI], part10[NI];
    bool has[NI], row_end[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const uint32_t c = (uint32_t)i % (uint32_t)a.cpr, part = 4 * c + (uint32_t)wave;
        has[i] = i < a.cpr * a.rps && part < upr;
        row_end[i] = i < a.cpr * a.rps && c + 1 == (uint32_t)a.cpr;
        part10[i] = part << 10;
        toffc[i] = has[i] ? table[(part << 6) + lane] : 0xFFFFFFFFu;
    }
    uint32_t limit = 0;
    // copies this wave issued in the last three rounds, the latest first: a round copies as many rows as the ring
    // takes, so what may stay in flight while a stage is waited for is counted, not constant
    int c1 = 0, c2 = 0, c3 = 0;
    // rows of the zero border at the head of the stream: this wave zeroes its units of them
    auto zero_rows = [&]() {
        while (rnext < limit && !(rho - (uint32_t)a.pad < (uint32_t)a.H)) {
            LDS_PTR(unsigned char) row = (LDS_PTR(unsigned char))lds + LDS_FIXED + (rnext & (uint32_t)(a.ring_rows - 1)) * (uint32_t)a.rowbytes;
            for (uint32_t part = (uint32_t)wave; part < upr; part += 4)
                *(LDS_PTR(f32x4))(row + (part << 10) + lane * 16) = f32x4{0.f, 0.f, 0.f, 0.f};
            ++rnext;
            if (++rho == (uint32_t)a.Hp) rho = 0;
        }
    };
    auto issue_image = [&]() {
        // rows up to the first one the oldest live stage reads, plus a ring, may be in LDS
        const uint32_t ya = fastdiv((uint32_t)(osub * DK), a.mg_wout) + (uint32_t)oe * (uint32_t)a.Hp;
        limit = min(ya + (uint32_t)a.ring_rows, rows_total);
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            if (i == 0 || row_end[i - 1]) zero_rows();
            const bool in = rnext < limit;
            if (has[i] && in) {
                const uint64_t addr = toffc[i] != 0xFFFFFFFFu ? rowptr + toffc[i] : (uint64_t)(uintptr_t)a.zero;
                const uint32_t dst = lds_ring + (rnext & (uint32_t)(a.ring_rows - 1)) * (uint32_t)a.rowbytes + part10[i];
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" :: "s"(dst), "v"(addr) : "memory", "m0");
                ++c1;
            }
            if (row_end[i] && in) {
                rowptr += rowstride;
                ++rnext;
                if (++rho == (uint32_t)a.Hp) rho = 0;
            }
        }
        zero_rows();
    };
    auto issue_stage = [&](int buf) {
        c3 = c2; c2 = c1; c1 = 1;
        if (RAG) {
            // rows past the example's end come from the line of zeros; the next example starts T rows, not a whole
            // number of stages, behind this one
            const uint64_t src = (uint64_t)(uintptr_t)(a.G + ((size_t)(ex0 + ie) * a.T + (size_t)isub * DK) * a.N) + offG;
            const uint64_t addr = isub * DK + rowG < a.T ? src : (uint64_t)(uintptr_t)a.zero;
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                         :: "s"(lds_g + buf * G_STAGE), "v"(addr) : "memory", "m0");
            if (++isub == spe) { isub = 0; ++ie; }
        } else {
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :: "s"(lds_g + buf * G_STAGE), "v"(offG), "s"(baseG) : "memory", "m0");
            baseG += stepG;
        }
        issue_image();
    };
    // stage s (relative) landed once at most `ahead` later stages' copies are outstanding
    auto wait_stage = [&](int ahead) {
        switch ((ahead >= 1 ? c1 : 0) + (ahead >= 2 ? c2 : 0) + (ahead >= 3 ? c3 : 0)) {
            case 0: wait_vmcnt<0>(); break;
            case 1: wait_vmcnt<1>(); break;
            case 2: wait_vmcnt<2>(); break;
            case 3: wait_vmcnt<3>(); break;
            case 4: wait_vmcnt<4>(); break;
            case 5: wait_vmcnt<5>(); break;
            case 6: wait_vmcnt<6>(); break;
            case 7: wait_vmcnt<7>(); break;
            case 8: wait_vmcnt<8>(); break;
            case 9: wait_vmcnt<9>(); break;
            case 10: wait_vmcnt<10>(); break;
            case 11: wait_vmcnt<11>(); break;
            case 12: wait_vmcnt<12>(); break;
            case 13: wait_vmcnt<13>(); break;
            case 14: wait_vmcnt<14>(); break;
            default: wait_vmcnt<15>(); break;
        }
    };
    static_assert(NSTG <= 4 && 3 * LPS <= 15, "wait_stage counts the copies of up to three rounds");

    // ---- LDS -> MFMA operands.  A lane of 16-lane group g reads row j = (lane % 16) / 4, 8-byte piece q = lane % 4
    //      of a 4 x 32-byte patch and receives the four rows' values of one column.  The two reads of a fragment
    //      take positions 4 g + j and 16 + 4 g + j of the stage (for A and for G alike, the order inside the
    //      contraction is free): lanes 0 .. 31 then touch eight consecutive positions.
    const int g16 = lane >> 4, j4 = (lane & 15) >> 2, q4 = lane & 3;
    const uint32_t kk0 = 4 * g16 + j4;
    const uint32_t lane_a = 32 * wave + 8 * q4;     // the wave's 16 channels inside the pixel
    uint32_t rdG[2][FNB];
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int jn = 0; jn < FNB; ++jn) {
            const uint32_t row = 16 * r + kk0;
            rdG[r][jn] = row * (TN * 2) + (((uint32_t)(FNB * hcol + jn) ^ ((row >> 1) & 3)) << 5) + 8 * q4;
        }
    uint32_t ad[2][3];                              // ring offsets of the stage's two positions, per kernel row
    // a lane's two positions of a stage: column, its byte offset, ring offset of the padded row of kernel row 0
    uint32_t px_[2], xoff[2], roff[2];
    const uint32_t ringbytes = (uint32_t)a.ring_rows * (uint32_t)a.rowbytes;
    const uint32_t rb0 = (uint32_t)a.dy32 * (uint32_t)a.rowbytes, rb1 = rb0 + (uint32_t)a.rowbytes;
    auto set_ad = [&]() {
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            uint32_t o = roff[r];
#pragma unroll
            for (int kh = 0; kh < 3; ++kh) {
                ad[r][kh] = o + xoff[r] + lane_a;
                o += (uint32_t)a.rowbytes;
                if (o >= ringbytes) o -= ringbytes;
            }
        }
    };
    // a lane's two positions in the first stage of an example
    uint32_t x0_[2], y0_[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const uint32_t k = 16 * r + kk0;
        y0_[r] = fastdiv(k, a.mg_wout); x0_[r] = k - y0_[r] * (uint32_t)a.Wout;
    }
    // The addresses of stage (e, sub): the first stage of an example from the lane's constants, any other one from
    // the stage before it, 32 positions earlier.  No branch and no full-rate-blocking multiplication, so that the
    // compiler can spread these operations between the MFMAs.
    auto stage_addr = [&](int e, int sub) {
        const bool first = sub == 0;
        const uint32_t srow0 = (uint32_t)e * (uint32_t)a.Hp;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const uint32_t xn = px_[r] + (uint32_t)a.dx32;
            const bool carry = xn >= (uint32_t)a.Wout;
            const uint32_t xs = carry ? xn - (uint32_t)a.Wout : xn;
            uint32_t rs = roff[r] + (carry ? rb1 : rb0);
            if (rs >= ringbytes) rs -= ringbytes;
            const uint32_t rf = __umul24((srow0 + y0_[r]) & (uint32_t)(a.ring_rows - 1), (uint32_t)a.rowbytes);
            px_[r] = first ? x0_[r] : xs;
            roff[r] = first ? rf : rs;
            xoff[r] = __umul24(px_[r], PITCH);
        }
        set_ad();
    };
    LDS_PTR(unsigned char) ringp = (LDS_PTR(unsigned char))lds + LDS_FIXED;
    auto read_a = [&](int tap) -> bf16x8 {
        const int kh = tap / KW3, kw = tap - kh * KW3;
        const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(v4i16))(ringp + ad[0][kh] + kw * PITCH));
        const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(v4i16))(ringp + ad[1][kh] + kw * PITCH));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    auto read_b = [&](int jn, int buf) -> bf16x8 {
        LDS_PTR(unsigned char) p = (LDS_PTR(unsigned char))lds + buf * G_STAGE;
        const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(v4i16))(p + rdG[0][jn]));
        const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(v4i16))(p + rdG[1][jn]));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };

    int e = 0, sub = 0;
    if (copier) {
        __builtin_amdgcn_s_setprio(3);
        for (int p = 0; p < a.pre_rounds; ++p) issue_image();
#pragma unroll
        for (int p = 0; p < NSTG; ++p)
            if (p < n_stages) issue_stage(p);
        wait_stage(min(n_stages - 1, NSTG - 1));
        __builtin_amdgcn_s_waitcnt(0xC07F);         // the rows of zeros are written: lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
        for (int st = 0; st + 1 < n_stages; ++st) {
            if (++sub == spe) { sub = 0; ++e; }     // stage st + 1
            TRACE(0, st);
            wait_stage(min(n_stages - 2 - st, NSTG - 2));
            __builtin_amdgcn_s_waitcnt(0xC07F);
            TRACE(1, st);
            __builtin_amdgcn_s_barrier();
            TRACE(2, st);
            if (st + NSTG < n_stages) { oe = e; osub = sub; issue_stage(st % NSTG); }
            TRACE(3, st);
        }
        if (MODE == 1) { __syncthreads(); __syncthreads(); }      // the reduction of the computing waves below
        return;
    }

    f32x4 acc[TAPS][FNB];
#pragma unroll
    for (int t = 0; t < TAPS; ++t)
#pragma unroll
        for (int jn = 0; jn < FNB; ++jn)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[t][jn][r] = 0.f;

    // clip factors of the slice's examples, one per lane (a slice is at most 64 examples)
    float vclip = 1.0f;
    if (MODE == 0) vclip = a.clip[min(ex0 + lane, a.B - 1)];
    float c_cur = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, vclip), 0));
    bool skip = false;
    float c_ref = c_cur;                            // the largest factor accumulated so far

    __builtin_amdgcn_s_barrier();                   // stage 0 has landed
    px_[0] = px_[1] = 0; roff[0] = roff[1] = 0;
    stage_addr(0, 0);
    // Fragments are requested a stage ahead: the MFMAs run tap by tap, and the image fragment of tap t is read again
    // for stage st + 1 behind the tap's four MFMAs (32 MFMAs before its next use), so the LDS reads are spread evenly
    // over the stage; the four G fragments serve every tap and have a second set.  The switch to the next stage sits
    // behind tap SW - 1, when the reads queued at the end of the previous stage have long returned.
    constexpr int SW = 3;
    bf16x8 fa[TAPS], fb[FNB];
#pragma unroll
    for (int jn = 0; jn < FNB; ++jn) fb[jn] = read_b(jn, 0);
#pragma unroll
    for (int t = 0; t < TAPS; ++t) fa[t] = read_a(t);

    // one stage; `more`: another stage follows (the last one is peeled, so that the loop body has no branch around
    // its reads and the compiler's wait counts stay exact)
    auto stage = [&](int st, auto more_tag) {
        constexpr bool more = decltype(more_tag)::value;
        if (MODE == 0 && sub == 0 && st > 0) {
            // first stage of the next example: the tile holds (1 / c_cur) * sum, move it to the new unit
            const float c_next = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, vclip), e));
            const float ratio = c_cur / c_next;
            // a zero factor, or one below 2^-40 of the largest so far (the tile in that unit would leave the float32
            // range), after a non-zero one: the example is left out
            skip = __builtin_isinf(ratio) || c_next < c_ref * 0x1p-40f;
            if (c_next != c_cur && !skip) {
#pragma unroll
                for (int t = 0; t < TAPS; ++t)
#pragma unroll
                    for (int jn = 0; jn < FNB; ++jn)
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[t][jn][r] *= ratio;
            }
            if (!skip) { c_cur = c_next; c_ref = fmaxf(c_ref, c_next); }
        }
        int ne = e, nsub = sub + 1;
        if (nsub == spe) { nsub = 0; ++ne; }
        const int nbuf = (st + 1) % NSTG;
        // a skipped example multiplies by a zero operand instead of branching around its MFMAs
        bf16x8 b[FNB];
#pragma unroll
        for (int jn = 0; jn < FNB; ++jn) {
            b[jn] = fb[jn];
            if (MODE == 0 && skip) {
#pragma unroll
                for (int i = 0; i < 8; ++i) b[jn][i] = (__bf16)0.0f;
            }
        }
        bf16x8 bn[FNB];
#pragma unroll
        for (int t = 0; t < TAPS; ++t) {
            if (more && t == SW) {
                // every computing wave holds stage st in registers once its reads have returned (the last ones were
                // queued SW taps ago): behind the barrier the copying waves may overwrite it, and stage st + 1 has landed
                TRACE(4, st);
                __builtin_amdgcn_s_waitcnt(0xC07F);                              // lgkmcnt(0)
                TRACE(5, st);
                __builtin_amdgcn_s_barrier();
                TRACE(6, st);
                stage_addr(ne, nsub);
#pragma unroll
                for (int jn = 0; jn < FNB; ++jn) bn[jn] = read_b(jn, nbuf);
#pragma unroll
                for (int u = 0; u < SW; ++u) fa[u] = read_a(u);
            }
#pragma unroll
            for (int jn = 0; jn < FNB; ++jn) acc[t][jn] = In16<F16>::mfma16(fa[t], b[jn], acc[t][jn]);
            if (more && t >= SW) fa[t] = read_a(t);
        }
        if (more) {
#pragma unroll
            for (int jn = 0; jn < FNB; ++jn) fb[jn] = bn[jn];
        }
        e = ne; sub = nsub;
    };
    for (int st = 0; st + 1 < n_stages; ++st) stage(st, std::true_type{});
    stage(n_stages - 1, std::false_type{});

    // accumulator layout of a 16 x 16 block: lane holds column lane % 16, rows 4 (lane / 16) + r
    const int ncol = lane & 15, mrow = 4 * g16;
    if (MODE == 1) {
        float sq = 0.f;
#pragma unroll
        for (int t = 0; t < TAPS; ++t)
#pragma unroll
            for (int jn = 0; jn < FNB; ++jn) {
                const bool in = n0 + 16 * (FNB * hcol + jn) + ncol < a.N;
#pragma unroll
                for (int r = 0; r < 4; ++r) sq += in ? acc[t][jn][r] * acc[t][jn][r] : 0.f;
            }
        sq = wave_sum(sq);
        __syncthreads();
        float* red = reinterpret_cast<float*>(lds);
        if (lane == 0) red[wave12] = sq;
        __syncthreads();
        if (tid == 0) {
            float t = (red[0] + red[1]) + (red[2] + red[3]);
            if (CW == 8) t += (red[4] + red[5]) + (red[6] + red[7]);
            a.out[(size_t)z * tiles + tile] = t;
        }
        return;
    }
    float* out = a.out + (size_t)z * a.slice;
#pragma unroll
    for (int t = 0; t < TAPS; ++t)
#pragma unroll
        for (int jn = 0; jn < FNB; ++jn) {
            const int n = n0 + 16 * (FNB * hcol + jn) + ncol;
            if (n >= a.N) continue;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = t * a.C + cbase + 16 * wave + mrow + r;
                float* p = out + (size_t)m * a.N + n;
                const float v = acc[t][jn][r] * c_cur;
                *p = a.accumulate ? *p + v : v;
            }
        }
}

// The copy schedule of the kernel, replayed on the host for a slice of E examples: true when every stage finds its
// rows issued in time.  Fills the rounds of image copies needed before the first stage.
bool schedule_ok(const ConvGeom& g, int E, int rps, int ring_rows, int* pre_rounds) {
    const int Hp = g.H + 2 * g.pad, Wout = g.W + 2 * g.pad - 2, Hout = g.H + 2 * g.pad - 2;
    const int T = Hout * Wout, spe = (T + DK - 1) / DK;
    const int64_t rows_total = (int64_t)E * Hp;
    auto need = [&](int e, int sub) {
        const int64_t yb = std::min<int64_t>((int64_t)(sub * DK + DK - 1) / Wout, Hout - 1);   // positions past T need no rows
        return std::min(rows_total, (int64_t)e * Hp + yb + 3);
    };
    auto limit = [&](int oe, int osub) {
        const int64_t ya = (int64_t)(osub * DK) / Wout + (int64_t)oe * Hp;
        return std::min(rows_total, ya + ring_rows);
    };
    auto border = [&](int64_t row) { const int64_t rho = row % Hp; return rho < g.pad || rho >= g.pad + g.H; };
    // a round: rps image rows, and the rows of the zero border on the way for free
    auto round = [&](int64_t next, int64_t lim) {
        for (int i = 0; i < rps; ++i) {
            while (next < lim && border(next)) ++next;
            if (next < lim) ++next;
        }
        while (next < lim && border(next)) ++next;
        return next;
    };
    const int64_t n_stages = (int64_t)E * spe;
    // before the first stage everything is issued with stage 0 as the oldest one
    const int64_t need0 = need(0, 0);
    if (need0 > limit(0, 0)) return false;
    int64_t next = 0;
    *pre_rounds = 0;
    while (round(next, limit(0, 0)) < need0) {
        const int64_t n2 = round(next, limit(0, 0));
        if (n2 == next) return false;
        next = n2;
        ++*pre_rounds;
    }
    for (int64_t j = 0; j < n_stages; ++j) {
        const int64_t o = std::max<int64_t>(0, j - (NSTG - 1));
        next = round(next, limit((int)(o / spe), (int)(o % spe)));
        if (next < need((int)(j / spe), (int)(j % spe))) return false;
    }
    return true;
}

struct RowsPlan { bool ok; int rowbytes, cpr, rps, ring_rows, pre_rounds, tiles_m, tiles_n, ex_per_slice, splits; size_t lds; };

// E = 0: choose the examples per K slice (clipped sum); E = 1: direct norm
RowsPlan plan_rows(const ConvGeom& g, int N, int B, int E) {
    RowsPlan p{};
    if (g.KH != 3 || g.KW != 3 || g.C < CG || (g.C % CG) != 0 || N < 8 || (N & 7) != 0 || B < 1) return p;
    const int64_t Hout = (int64_t)g.H + 2 * g.pad - 2, Wout = (int64_t)g.W + 2 * g.pad - 2;
    if (Hout < 1 || Wout < 2) return p;
    const int64_t T = Hout * Wout, Hp = g.H + 2 * g.pad, Wp = g.W + 2 * g.pad;
    // whole stages of 32 positions, or at most a quarter of a ragged example's stages beyond its end (49, 196, 784 ...)
    const int64_t Tp = (T + DK - 1) / DK * DK;
    if (Tp * 3 > T * 4 || T >= (int64_t(1) << 24) || Wp > 4096 || Hp > 4096) return p;
    const int64_t rowbytes = (Wp * PITCH + 1023) / 1024 * 1024;
    if (rowbytes < 2048 || rowbytes * 64 / 1024 * 4 > TABLE_BYTES) return p;      // 2 .. 16 copy units per row
    p.tiles_m = g.C / CG;
    p.tiles_n = (N + TN - 1) / TN;
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    if (E == 0) {
        // two workgroups per compute unit, at most 64 examples per slice (their clip factors sit one per lane)
        E = (int)std::min<int64_t>(64, std::max<int64_t>(1, (int64_t)B * tiles / 512));
        // the 32-bit arithmetic of the copies: chunks of the slice's stream times chunks per row, and the image offsets
        // the 32-bit arithmetic of the copies: the image offsets inside a slice
        while (E > 1 && (int64_t)E * g.H * g.W * g.C >= (int64_t(1) << 30)) --E;
    }
    if ((int64_t)E * g.H * g.W * g.C >= (int64_t(1) << 30)) return p;
    if ((int64_t)E * Hp * rowbytes >= (int64_t(1) << 31) || T * Wout >= (int64_t(1) << 32)) return p;
    p.ex_per_slice = E;
    p.splits = (B + E - 1) / E;
    if (tiles * p.splits >= (int64_t(1) << 28)) return p;
    p.rowbytes = (int)rowbytes;
    p.cpr = (int)((rowbytes / 1024 + 3) / 4);
    // as many image rows per round as the copy counter of a wave allows (a round stops at the ring's end anyway), in
    // the smallest ring that works
    {
        const int rps = NI / p.cpr;
        for (int R = 8; R <= 64; R *= 2) {
            const int64_t lds = LDS_FIXED + (int64_t)R * rowbytes;
            if (lds > LDS_MAX) break;
            if (DK / Wout + 1 > R) continue;          // a stage's step through the rows wraps the ring at most once
            int pre = 0;
            if (schedule_ok(g, E, rps, R, &pre)) {
                p.ok = true; p.rps = rps; p.ring_rows = R; p.pre_rounds = pre; p.lds = (size_t)lds;
                return p;
            }
        }
    }
    return p;
}

void fill_args(ConvRowsArgs& a, const RowsPlan& p, const ConvGeom& g, const uint16_t* X, const uint16_t* G, int B, int N,
               const uint16_t* zero) {
    a.X = X; a.G = G; a.zero = zero;
    a.B = B; a.N = N; a.C = g.C; a.H = g.H; a.W = g.W; a.pad = g.pad;
    a.Wout = g.W + 2 * g.pad - 2; a.Hp = g.H + 2 * g.pad; a.Wp = g.W + 2 * g.pad;
    a.T = (g.H + 2 * g.pad - 2) * a.Wout;
    a.rowbytes = p.rowbytes; a.cpr = p.cpr; a.rps = p.rps; a.ring_rows = p.ring_rows; a.pre_rounds = p.pre_rounds;
    a.mg_wout = magic_of((uint32_t)a.Wout); a.mg_upr = magic_of((uint32_t)p.rowbytes / 1024u);
    a.dx32 = DK % a.Wout; a.dy32 = DK / a.Wout;
    a.mg_hp = magic_of((uint32_t)a.Hp); a.mg_ring = magic_of((uint32_t)((int64_t)p.ring_rows * p.rowbytes / 1024));
    a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n; a.ex_per_slice = p.ex_per_slice; a.splits = p.splits;
    a.per_xcd = (int)(((int64_t)p.tiles_m * p.tiles_n * p.splits + 7) / 8);
}

}  // namespace

// This kernel spends about 7 stage times per workgroup outside its stages, and its norm mode takes one example per
// workgroup: with fewer than 16 stages per example (images below about 23 x 23) the general copy-pipeline kernel with
// implicit unfolding is as fast or faster where it takes the geometry at all (measured from the image, bf16, this
// kernel against that one: 32 x 32 x 64 -> 128, B = 128: 26 / 40 us against 39 / 47; 28 x 28: 26 / 36 against
// 33 / 41; 16 x 16 x 128 -> 128, B = 256: 39 / 51 against 38 / 46; 8 x 8 x 256 -> 256, B = 256: 81 / 60 against 57 / 49).
bool conv_rows_ok(const ConvGeom& g, int d_out, int B) {
    if (!plan_rows(g, d_out, B, 1).ok || !plan_rows(g, d_out, B, 0).ok) return false;
    const int64_t T = (int64_t)(g.H + 2 * g.pad - 2) * (g.W + 2 * g.pad - 2);
    return T >= 16 * DK || !dma_conv_ok(g, d_out);
}
int conv_rows_tiles(const ConvGeom& g, int d_out) { return (g.C / CG) * ((d_out + TN - 1) / TN); }
int conv_rows_splits(const ConvGeom& g, int d_out, int B) { return plan_rows(g, d_out, B, 0).splits; }

hipError_t launch_direct_conv_rows(const ConvGeom& g, const uint16_t* X, const uint16_t* G, int B, int N, bool accumulate,
                                   float* sqnorm, float* partial, hipStream_t st, const uint16_t* zero, bool f16,
                                   const ClipOut* co) {
    const RowsPlan p = plan_rows(g, N, B, 1);
    if (!p.ok) return hipErrorInvalidValue;
    ConvRowsArgs a;
    fill_args(a, p, g, X, G, B, N, zero);
    a.clip = nullptr; a.out = partial; a.slice = 0; a.accumulate = 0;
    const unsigned grid = 8u * (unsigned)a.per_xcd;
    const bool rag = (a.T % DK) != 0;
    if (rag) {
        if (f16) k_conv3x3_rows<1, true, true><<<grid, THREADS, 0, st>>>(a);
        else     k_conv3x3_rows<1, false, true><<<grid, THREADS, 0, st>>>(a);
    } else {
        if (f16) k_conv3x3_rows<1, true, false><<<grid, THREADS, 0, st>>>(a);
        else     k_conv3x3_rows<1, false, false><<<grid, THREADS, 0, st>>>(a);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_finalize_partials(partial, B, p.tiles_m * p.tiles_n, accumulate, sqnorm, st, co);
}

hipError_t launch_clipped_conv_rows(const ConvGeom& g, const uint16_t* X, const uint16_t* G, const float* clip, int B, int N,
                                    bool accumulate, float* grad, float* ws, hipStream_t st, const uint16_t* zero, bool f16,
                                    const NoiseArgs* noise) {
    const RowsPlan p = plan_rows(g, N, B, 0);
    if (!p.ok) return hipErrorInvalidValue;
    ConvRowsArgs a;
    fill_args(a, p, g, X, G, B, N, zero);
    a.clip = clip;
    const int64_t n = (int64_t)9 * g.C * N;
    if (p.splits == 1) { a.out = grad; a.slice = 0; a.accumulate = accumulate ? 1 : 0; }
    else { a.out = ws; a.slice = splitk_slice_elems(n); a.accumulate = 0; }
    const unsigned grid = 8u * (unsigned)a.per_xcd;
    const bool rag = (a.T % DK) != 0;
    if (rag) {
        if (f16) k_conv3x3_rows<0, true, true><<<grid, THREADS, 0, st>>>(a);
        else     k_conv3x3_rows<0, false, true><<<grid, THREADS, 0, st>>>(a);
    } else {
        if (f16) k_conv3x3_rows<0, true, false><<<grid, THREADS, 0, st>>>(a);
        else     k_conv3x3_rows<0, false, false><<<grid, THREADS, 0, st>>>(a);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.splits == 1) return e;
    return launch_splitk_reduce(ws, n, p.splits, accumulate, grad, st, noise);
}

}  // namespace dpk
