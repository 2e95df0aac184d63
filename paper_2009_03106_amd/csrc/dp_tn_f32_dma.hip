// float32 K-major products  P = sum_k A[k, m-tile]^T G[k, n-tile]  for long contractions, on the fp32 MFMA
// (v_mfma_f32_32x32x2_f32), with the data path of the 16-bit copy-pipeline kernels:
//   * 128 x 128 output tile per workgroup of 4 waves (64 x 64 = 2 x 2 MFMA tiles per wave): 32 flop per byte copied,
//     against 16 for the 64 x 64 kernel of dp_tn_f32.hip, which at the fp32 matrix rate asks the L2s for about
//     10 TB/s, all they deliver;
//   * 16-row stages copied global -> LDS directly (global_load_lds_dwordx4), a ring of four, two workgroups per
//     compute unit; the fp32 MFMA takes one k per lane half, so the K-major rows are used as they lie in memory
//     and the fragments are plain 4-byte LDS reads of consecutive floats;
//   * the clip factors of a stage's rows are copied into LDS by the same mechanism (global_load_lds_dword, one per
//     wave and stage, each wave into a copy of its own) and multiplied into the A fragments after the LDS read:
//     one multiply per fragment register, the same a * c rounded once to float32 as in the row-scaling kernels.
//     Rows past the end of the K slice read a clamped valid row and get the factor 0.
// Two uses, as in the 16-bit file: clipped sum (Eq. weighted_loss) over K slices, and direct squared norm (Algorithm
// 3 / 4 without their output tensor): the slice is one example and the finished tile is squared and summed.
// Needs d_in and d_out multiples of 4 (16-byte pieces) and 16-byte aligned operands.
#include <algorithm>
#include "dp_common.h"
#include "dp_internal.h"

namespace dpk {

namespace {

constexpr int TMF = 128, TNF = 128;     // output tile
constexpr int DKF = 16;                 // rows of K per stage
constexpr int NSTF = 4;                 // stages resident in LDS
constexpr int ROWB = TMF * 4;           // bytes of one stage row of either operand (TMF == TNF)
constexpr int OPB = DKF * ROWB;         // bytes of one operand's part of a stage
constexpr int STAGE_B = 2 * OPB;
constexpr int CSB = 256;                // one wave's copy of a stage's factors (a dword copy instruction writes 64 x 4 bytes)
constexpr int LPSF = 5;                 // copies per stage and wave: 2 of A, 2 of G, 1 of factors
#define LDS_PTR(T) __attribute__((address_space(3))) T*

struct F32DmaArgs {
    const float* A;
    const float* G;
    const float* clip;
    float* out;            // slice base (stride `slice` per K slice) or grad; direct norm: partial[B][tiles]
    int64_t slice;
    int K, T, M, N;
    int tiles_m, tiles_n;
    int splits;            // K slices (direct norm: examples)
    int kchunk;            // rows per K slice, a multiple of DKF
    int per_xcd;
    int accumulate;
};

__device__ float g_factor_consts[2] = {0.0f, 1.0f};

template <int N> __device__ __forceinline__ void wait_vm() { __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14)); }

// MODE 0: clipped sum over K slice z = rows [z kchunk, (z + 1) kchunk).  MODE 1: direct squared norm of example z.
// item L of the launch: (slice, tile), slice-major
template <int MODE>
__device__ __forceinline__ void tn_f32_dma_tile(const F32DmaArgs& a, const int L) {
    __shared__ __attribute__((aligned(1024))) unsigned char lds[NSTF * STAGE_B + NSTF * 4 * CSB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tiles = a.tiles_m * a.tiles_n;
    if (L >= (int64_t)tiles * a.splits) return;
    const int z = L / tiles, tile = L - z * tiles;
    int tm, tn;                                          // consecutive items walk the short side of the tile grid first
    if (a.tiles_m < a.tiles_n) { tn = tile / a.tiles_m; tm = tile - tn * a.tiles_m; }
    else { tm = tile / a.tiles_n; tn = tile - tm * a.tiles_n; }
    const int m0 = tm * TMF, n0 = tn * TNF;
    int k_begin, k_end;
    if (MODE == 0) { k_begin = z * a.kchunk; k_end = min(a.K, k_begin + a.kchunk); }
    else { k_begin = z * a.T; k_end = k_begin + a.T; }
    const int n_stages = (k_end - k_begin + DKF - 1) / DKF;
    if (n_stages <= 0) return;

    // ---- global -> LDS.  A stage row is 32 pieces of 16 bytes; copy u of wave w moves rows 2 (2 w + u) and + 1, one
    //      piece per lane (lane / 32: the row, lane % 32: the position).  Piece c of row r sits at position
    //      c ^ (8 (r & 1)): odd rows are shifted by 32 floats, so that the two lane halves of a fragment read (rows k
    //      and k + 1, the same columns) use different banks.
    const int crow = lane >> 5, cpos = lane & 31;
    const int cpiece = cpos ^ (crow << 3);
    int colA = m0 + 4 * cpiece, colG = n0 + 4 * cpiece;
    if (colA >= a.M) colA = m0;                          // columns outside the matrix only feed outputs that are never stored
    if (colG >= a.N) colG = n0;
    // the factor copy: lane i < 16 fetches the factor of row 2 (i % 8) + i / 8 of the stage, i.e. the copy holds the
    // factors of the even rows, then those of the odd rows: what the lower / upper lane half of a fragment needs
    const int frow = 2 * (lane & 7) + ((lane >> 3) & 1);
    int fex = 0, fpos = 0;                               // example and position inside it of this lane's row of the next stage to copy
    if (MODE == 0 && a.T > 1) { fex = (k_begin + frow) / a.T; fpos = (k_begin + frow) - fex * a.T; }
    const int adv_ex = DKF / a.T, adv_pos = DKF - adv_ex * a.T;
    int next_row = k_begin;                              // first row of the next stage to copy

    const uint32_t lds_base = (uint32_t)(uintptr_t)(LDS_PTR(unsigned char))lds;
    const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(lds_base + wave * 2048);
    const uint32_t wave_cs = __builtin_amdgcn_readfirstlane(lds_base + NSTF * STAGE_B + wave * CSB);
    // The copies are inline assembly: the compiler then does not know that they write LDS and does not make every
    // LDS read wait for all copies in flight; they are waited for with the explicit vmcnt waits below.
    auto issue = [&](int buf) {
        const float* f;
        {
            const int row = next_row + frow;
            if (row >= k_end) f = &g_factor_consts[0];
            else if (MODE != 0) f = &g_factor_consts[1];
            else f = a.clip + (a.T == 1 ? row : fex);
        }
        asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, off"
                     :: "s"(wave_cs + buf * 4 * CSB), "v"((uint64_t)(uintptr_t)f) : "memory", "m0");
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int row = min(next_row + 2 * (2 * wave + u) + crow, k_end - 1);
            const uint64_t pa = (uint64_t)(uintptr_t)(a.A + ((size_t)row * a.M + colA));
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                         :: "s"(wave_lds + buf * STAGE_B + u * 1024), "v"(pa) : "memory", "m0");
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int row = min(next_row + 2 * (2 * wave + u) + crow, k_end - 1);
            const uint64_t pg = (uint64_t)(uintptr_t)(a.G + ((size_t)row * a.N + colG));
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                         :: "s"(wave_lds + buf * STAGE_B + OPB + u * 1024), "v"(pg) : "memory", "m0");
        }
        next_row += DKF;
        if (MODE == 0 && a.T > 1) {
            fex += adv_ex; fpos += adv_pos;
            if (fpos >= a.T) { fpos -= a.T; ++fex; }
        }
    };

    // ---- LDS -> MFMA operands: lane (lrow, lhalf) takes column lrow of a 32-wide block and row 2 j + lhalf
    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = lane & 31, lhalf = lane >> 5;
    uint32_t rdA[2], rdG[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int m = wm * 64 + i * 32 + lrow, n = wn * 64 + i * 32 + lrow;
        rdA[i] = lhalf * ROWB + ((((m >> 2) ^ (lhalf << 3)) << 4) | ((m & 3) << 2));
        rdG[i] = OPB + lhalf * ROWB + ((((n >> 2) ^ (lhalf << 3)) << 4) | ((n & 3) << 2));
    }
    const uint32_t rdC = NSTF * STAGE_B + wave * CSB + lhalf * 32;

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // a half stage: 4 pairs of rows = 16 MFMAs per wave; its 16 fragment values and 4 factors are requested while
    // the MFMAs of the half before it run, also across the stage boundary
    struct Half { float fa[4][2], fg[4][2]; f32x4 c; };
    auto read_half = [&](Half& h, int buf, int half) {
        const unsigned char* sb = lds + buf * STAGE_B + half * 8 * ROWB;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                h.fa[jj][i] = *reinterpret_cast<const float*>(sb + jj * 2 * ROWB + rdA[i]);
                h.fg[jj][i] = *reinterpret_cast<const float*>(sb + jj * 2 * ROWB + rdG[i]);
            }
        }
        h.c = *reinterpret_cast<const f32x4*>(lds + rdC + buf * 4 * CSB + half * 16);
    };
    auto mfma_half = [&](const Half& h) {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const float a0 = h.fa[jj][0] * h.c[jj], a1 = h.fa[jj][1] * h.c[jj];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, h.fg[jj][0], acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, h.fg[jj][1], acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, h.fg[jj][0], acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, h.fg[jj][1], acc[1][1], 0, 0, 0);
        }
    };
    // stage s landed once at most `ahead` later stages' copies are outstanding
    auto wait_stage = [&](int ahead) {
        if (ahead >= 3) wait_vm<3 * LPSF>();
        else if (ahead == 2) wait_vm<2 * LPSF>();
        else if (ahead == 1) wait_vm<LPSF>();
        else wait_vm<0>();
    };

#pragma unroll
    for (int p = 0; p < NSTF; ++p)
        if (p < n_stages) issue(p);
    wait_stage(min(n_stages - 1, NSTF - 1));
    __builtin_amdgcn_s_barrier();
    Half hf[2];
    read_half(hf[0], 0, 0);

    for (int st = 0; st < n_stages; ++st) {
        const int buf = st % NSTF;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            __builtin_amdgcn_s_waitcnt(0xC07F);                  // lgkmcnt(0): this half's operands, requested a half stage ago
            if (half == 0) {
                read_half(hf[1], buf, 1);
            } else if (st + 1 < n_stages) {
                // stage st + 1 must have landed, for every wave; every wave has retired its reads of stage st, so its
                // buffer can take stage st + NSTF
                wait_stage(min(n_stages - 2 - st, NSTF - 2));
                __builtin_amdgcn_s_barrier();
                if (st + NSTF < n_stages) issue(buf);
                read_half(hf[0], (st + 1) % NSTF, 0);
            }
            mfma_half(hf[half]);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    if (MODE == 1) {
        float sq = 0.f;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int n = n0 + wn * 64 + j * 32 + lrow;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = m0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
                    const float v = acc[i][j][r];
                    sq += (m < a.M && n < a.N) ? v * v : 0.f;
                }
            }
        sq = wave_sum(sq);
        __syncthreads();                                         // every wave is done with the stage buffers
        float* red = reinterpret_cast<float*>(lds);
        if (lane == 0) red[wave] = sq;
        __syncthreads();
        if (tid == 0) a.out[(size_t)z * tiles + tile] = (red[0] + red[1]) + (red[2] + red[3]);
        return;
    }
    float* out = a.out + (size_t)z * a.slice;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + wn * 64 + j * 32 + lrow;
            if (n >= a.N) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
                if (m < a.M) {
                    float* p = out + (size_t)m * a.N + n;
                    *p = a.accumulate ? *p + acc[i][j][r] : acc[i][j][r];
                }
            }
        }
}

template <int MODE>
__global__ __launch_bounds__(kThreads, 2) void k_tn_f32_dma(F32DmaArgs a) {
    // workgroup b runs on XCD b % 8: each XCD takes a contiguous run of (slice, tile) items, slice-major, so that
    // its workgroups stream the same rows of A and G through one L2
    tn_f32_dma_tile<MODE>(a, (blockIdx.x & 7) * a.per_xcd + (blockIdx.x >> 3));
}

// Several layers' clipped sums in one launch, as for the 16-bit inputs (dp_tn_bf16_dma.hip): the launch is a list of
// (layer, K slice, tile) items, a layer's items slice-major, dealt to the XCDs in contiguous runs.
struct F32JointLayer {
    const float* A; const float* G; const float* clip;
    float* out;            // the layer's K slices; the gradient itself where one slice is the whole sum
    int K, T, M, N, tiles_m, tiles_n, splits, kchunk, first_item, accumulate;
};
struct F32JointArgs {
    F32JointLayer layer[kJointLayers];
    int n_layers, n_items, per_xcd;
};
// MODE 1: the layers' direct squared norms (a layer's "K slices" are its examples, `out` is partial[B][tiles])
template <int MODE>
__global__ __launch_bounds__(kThreads, 2) void k_tn_f32_dma_joint(F32JointArgs j) {
    const int L = (blockIdx.x & 7) * j.per_xcd + (blockIdx.x >> 3);
    if (L >= j.n_items) return;
    int l = 0;
    while (l + 1 < j.n_layers && L >= j.layer[l + 1].first_item) ++l;
    const F32JointLayer& y = j.layer[l];
    F32DmaArgs a;
    a.A = y.A; a.G = y.G; a.clip = y.clip;
    a.out = y.out; a.slice = (((int64_t)y.M * y.N) + 3) & ~(int64_t)3;          // splitk_slice_elems
    a.K = y.K; a.T = y.T; a.M = y.M; a.N = y.N;
    a.tiles_m = y.tiles_m; a.tiles_n = y.tiles_n; a.splits = y.splits; a.kchunk = y.kchunk;
    a.per_xcd = 0; a.accumulate = y.accumulate;
    tn_f32_dma_tile<MODE>(a, L - y.first_item);
}

// One slice length (in 16-row stages) for all layers of a joint launch, each layer rounding it to equal slices:
// minimise  rounds of 512 workgroups x (stages of the longest slice + what an item costs besides its stages).
struct F32JointPlan { int splits[kJointLayers], kchunk[kJointLayers], tiles_m[kJointLayers], tiles_n[kJointLayers]; int64_t items; };
F32JointPlan plan_joint_f32(const JointShape* sh, int n_layers, int B) {
    constexpr int64_t kItemOverhead = 16, kSlots = 512;
    F32JointPlan best{};
    int64_t best_cost = -1, stages_max = 1;
    for (int l = 0; l < n_layers; ++l) stages_max = std::max<int64_t>(stages_max, ceil_div((int64_t)B * sh[l].T, DKF));
    for (int64_t S = 1; S <= 512 && S <= stages_max; ++S) {
        const int64_t len = (stages_max + S - 1) / S;
        if (len < 8 && S > 1) break;
        F32JointPlan p{};
        int64_t longest = 0;
        for (int l = 0; l < n_layers; ++l) {
            const int64_t stages = ceil_div((int64_t)B * sh[l].T, DKF);
            int64_t splits = (stages + len - 1) / len;
            const int64_t sps = (stages + splits - 1) / splits;
            splits = (stages + sps - 1) / sps;
            p.tiles_m[l] = ceil_div(sh[l].M, TMF); p.tiles_n[l] = ceil_div(sh[l].N, TNF);
            p.splits[l] = (int)splits; p.kchunk[l] = (int)(sps * DKF);
            p.items += (int64_t)p.tiles_m[l] * p.tiles_n[l] * splits;
            longest = std::max(longest, sps);
        }
        const int64_t cost = ((p.items + kSlots - 1) / kSlots) * (longest + kItemOverhead);
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = p; }
    }
    return best;
}

}  // namespace

size_t joint_f32_workspace_floats(const JointShape* sh, int n_layers, int B) {
    const F32JointPlan p = plan_joint_f32(sh, n_layers, B);
    size_t slices = 0;
    for (int l = 0; l < n_layers; ++l) slices += (size_t)p.splits[l] * (size_t)splitk_slice_elems((int64_t)sh[l].M * sh[l].N);
    return slices;
}

// noise: stddev == 0 for none, else every layer's d_in * d_out and noise_offset are multiples of 4.  A, G of the
// operands are float pointers here.
hipError_t launch_clipped_f32_dma_joint(const JointShape* sh, const JointOperands* op, int n_layers, int B, bool accumulate,
                                        float stddev, uint64_t seed, float* ws, hipStream_t st) {
    if (n_layers < 1 || n_layers > kJointLayers) return hipErrorInvalidValue;
    const F32JointPlan p = plan_joint_f32(sh, n_layers, B);
    if (p.items >= (int64_t(1) << 28)) return hipErrorInvalidValue;
    F32JointArgs j;
    FoldLayers f;
    int nf = 0;
    float* slices = ws;
    int64_t first = 0;
    for (int l = 0; l < n_layers; ++l) {
        F32JointLayer& y = j.layer[l];
        y.A = reinterpret_cast<const float*>(op[l].A); y.G = reinterpret_cast<const float*>(op[l].G); y.clip = op[l].clip;
        // one slice and no noise to add: the launch writes the gradient itself, nothing to fold
        const bool whole = p.splits[l] == 1 && stddev == 0.0f;
        y.out = whole ? op[l].grad : slices;
        y.accumulate = whole && accumulate ? 1 : 0;
        y.K = B * sh[l].T; y.T = sh[l].T; y.M = sh[l].M; y.N = sh[l].N;
        y.tiles_m = p.tiles_m[l]; y.tiles_n = p.tiles_n[l]; y.splits = p.splits[l]; y.kchunk = p.kchunk[l];
        y.first_item = (int)first;
        first += (int64_t)p.tiles_m[l] * p.tiles_n[l] * p.splits[l];
        if (!whole) {
            f.ws[nf] = slices; f.grad[nf] = op[l].grad; f.n[nf] = (int64_t)sh[l].M * sh[l].N;
            f.splits[nf] = p.splits[l]; f.noise_offset[nf] = op[l].noise_offset;
            ++nf;
        }
        slices += (size_t)p.splits[l] * (size_t)splitk_slice_elems((int64_t)sh[l].M * sh[l].N);
    }
    for (int l = n_layers; l < kJointLayers; ++l) j.layer[l] = j.layer[0];
    j.n_layers = n_layers; j.n_items = (int)p.items; j.per_xcd = ceil_div(p.items, 8);
    k_tn_f32_dma_joint<0><<<8u * (unsigned)j.per_xcd, kThreads, 0, st>>>(j);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess || nf == 0) return e;
    f.n_layers = nf;
    for (int l = nf; l < kJointLayers; ++l) { f.ws[l] = f.ws[0]; f.grad[l] = f.grad[0]; f.n[l] = 0; f.splits[l] = 0; f.noise_offset[l] = 0; }
    return launch_splitk_reduce_layers(f, accumulate, st, stddev, seed);
}

// Shapes for this kernel: 16-byte pieces, and tiles of 128 that are not mostly padding.
bool f32_dma_ok(int64_t K, int M, int N) {
    if (((M | N) & 3) != 0 || K < 16 * DKF) return false;
    const int64_t pm = (int64_t)ceil_div(M, TMF) * TMF, pn = (int64_t)ceil_div(N, TNF) * TNF;
    return pm * pn * 3 <= (int64_t)M * N * 4;           // at most a third more than the matrix
}
int f32_dma_tile() { return TMF; }
int f32_dma_stage_rows() { return DKF; }

// mode 0: clipped sum, p.splits K slices of p.kchunk rows to out (+ z * slice); mode 1: direct norm, one item per
// (example, tile) to out[B][tiles].
hipError_t launch_tn_f32_dma(int mode, const TnPlan& p, const float* A, const float* G, const float* clip, int B, int T,
                             int M, int N, float* out, int64_t slice, bool accumulate, hipStream_t st) {
    F32DmaArgs a;
    a.A = A; a.G = G; a.clip = clip; a.out = out; a.slice = slice;
    a.K = B * T; a.T = T; a.M = M; a.N = N;
    a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n;
    a.splits = mode == 0 ? p.splits : B;
    a.kchunk = mode == 0 ? p.kchunk : T;
    a.accumulate = accumulate ? 1 : 0;
    const int64_t items = (int64_t)p.tiles_m * p.tiles_n * a.splits;
    if (items <= 0 || items >= (int64_t(1) << 31) - 8) return hipErrorInvalidValue;
    if (mode == 0 && (p.kchunk % DKF) != 0) return hipErrorInvalidValue;
    a.per_xcd = (int)((items + 7) / 8);
    const unsigned grid = 8u * (unsigned)a.per_xcd;
    if (mode == 0) k_tn_f32_dma<0><<<grid, kThreads, 0, st>>>(a);
    else           k_tn_f32_dma<1><<<grid, kThreads, 0, st>>>(a);
    return hipGetLastError();
}

// Several layers' direct norms in one launch; partial[l]: the layer's [B][tiles of 128 x 128] sums of squares, to be
// added by the caller.  Every layer: f32_dma_ok(T, M, N).
hipError_t launch_direct_f32_dma_joint(const JointShape* sh, const JointOperands* op, float* const* partial, int n_layers,
                                       int B, hipStream_t st) {
    if (n_layers < 1 || n_layers > kJointLayers) return hipErrorInvalidValue;
    F32JointArgs j;
    int64_t first = 0;
    for (int l = 0; l < n_layers; ++l) {
        F32JointLayer& y = j.layer[l];
        y.A = reinterpret_cast<const float*>(op[l].A); y.G = reinterpret_cast<const float*>(op[l].G); y.clip = nullptr;
        y.out = partial[l]; y.accumulate = 0;
        y.K = B * sh[l].T; y.T = sh[l].T; y.M = sh[l].M; y.N = sh[l].N;
        y.tiles_m = ceil_div(sh[l].M, TMF); y.tiles_n = ceil_div(sh[l].N, TNF);
        y.splits = B; y.kchunk = sh[l].T;
        y.first_item = (int)first;
        first += (int64_t)y.tiles_m * y.tiles_n * B;
    }
    if (first >= (int64_t(1) << 28)) return hipErrorInvalidValue;
    for (int l = n_layers; l < kJointLayers; ++l) j.layer[l] = j.layer[0];
    j.n_layers = n_layers; j.n_items = (int)first; j.per_xcd = ceil_div(first, 8);
    k_tn_f32_dma_joint<1><<<8u * (unsigned)j.per_xcd, kThreads, 0, st>>>(j);
    return hipGetLastError();
}

}  // namespace dpk
