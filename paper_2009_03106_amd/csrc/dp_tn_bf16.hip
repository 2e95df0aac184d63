// K-major products  P = sum_k A[k, m-tile]^T G[k, n-tile]  of 16-bit inputs (bf16 or fp16) on MFMA.
//
// Both operands are stored with the contraction index k (example-major rows
// of the flattened [B*T, d] matrices) as the slow axis, while the MFMA wants
// each lane to hold 8 consecutive k for one m (or n).  The 16-bit transpose is
// done in registers on the way from global memory to LDS: a thread loads an
// 8(k) x 8(col) block as eight 16-byte row pieces, repacks it into eight
// 16-byte column pieces and stores those.  For the clipped sum the rows of A
// are multiplied by their example's clip factor in the same step (the values
// are in float registers anyway for the repack), then rounded back to 16 bits.
//
// Two kernels share the repack.  k_tn_bf16_seg (T >= 32) walks K example by
// example: a per-example accumulator tile is finished when the example's T
// rows are done and is then either folded into the running clipped sum with
// one float multiply-add per element (exact clip factor, no re-rounding of A)
// or squared and reduced.  k_tn_bf16_rows (small T, where an LDS stage would
// be mostly padding) walks K in plain 64-row stages and scales the rows of A
// by their clip factors during the repack, rounding them back to the input format.
//
// Two uses:
//   * clipped sum (dp_clipped_grad): grid = tiles x K-slices; every slice's
//     tile goes to the workspace and is folded in a fixed order afterwards.
//   * direct squared norm (dp_layer_sqnorm, DIRECT): grid = tiles x examples;
//     K = that example's T rows; the accumulator tile is squared and reduced,
//     never stored (Algorithm 3 / Algorithm 4 of the paper without their
//     output tensor).
#include "dp_common.h"
#include "dp_internal.h"

namespace dpk {

namespace {

constexpr int BK = 64;           // k rows per LDS stage
constexpr int BM = 128, BN = 128;

struct TnArgs {
    const uint16_t* A;
    const uint16_t* G;
    const float* clip;     // clipped sum only
    float* out;            // clipped: slice base [z][M][N] (slice stride `slice`); direct: partial[ex][tiles]
    int64_t slice;
    int K;                 // total rows B*T
    int T;
    int M, N;
    int tiles_m, tiles_n;
    int kchunk;            // clipped: rows per K slice
    int accumulate;        // clipped with one slice: add to out
    int slices_per_example = 1;    // MODE 2
};


// Load an 8(k) x 8(col) block starting at (row0, col0) of X[K, D]; rows >= k_end and
// columns >= D read as zero.  For widths that are not multiples of 8 every load is issued unconditionally from a
// clamped (valid) address and zeroed afterwards: with a branch around each of the 64 scalar loads, a thread's loads
// went out one memory round trip after the other (16-byte pieces: the guarded form is the faster one, measured).
// k_end >= 1 and D >= 1 (the launchers never start an empty slice).
__device__ __forceinline__ void load_block(const uint16_t* __restrict__ X, int D, bool vec_ok,
                                           int row0, int k_end, int col0, uint4 (&r)[8]) {
    if (vec_ok) {
        const bool col_ok = col0 < D;     // D % 8 == 0 and col0 % 8 == 0: the piece is all in or all out
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = row0 + i;
            if (col_ok && row < k_end) r[i] = *reinterpret_cast<const uint4*>(X + (size_t)row * D + col0);
            else r[i] = make_uint4(0u, 0u, 0u, 0u);
        }
    } else if ((D & 3) == 0) {
        // widths that are multiples of 4 only (300, 500, 20 ...): 8-byte pieces, each all in or all out, rows 8-byte aligned
        const bool ok0 = col0 < D, ok1 = col0 + 4 < D;
        const int c0 = ok0 ? col0 : 0, c1 = ok1 ? col0 + 4 : 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = row0 + i;
            const uint16_t* p = X + (size_t)min(row, k_end - 1) * D;
            const uint2 lo = *reinterpret_cast<const uint2*>(p + c0), hi = *reinterpret_cast<const uint2*>(p + c1);
            const bool in = row < k_end;
            r[i] = make_uint4((in && ok0) ? lo.x : 0u, (in && ok0) ? lo.y : 0u, (in && ok1) ? hi.x : 0u, (in && ok1) ? hi.y : 0u);
        }
    } else {
        int cc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) cc[j] = min(col0 + j, D - 1);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = row0 + i;
            const uint16_t* p = X + (size_t)min(row, k_end - 1) * D;
            uint32_t v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = p[cc[j]];
            uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t x = (row < k_end && col0 + j < D) ? v[j] : 0u;
                w[j >> 1] |= x << ((j & 1) * 16);
            }
            r[i] = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
}

// Repack rows r[0..7] (each 8 columns) into columns c[0..7] (each 8 k values), no scaling.
__device__ __forceinline__ void transpose8x8(const uint4 (&r)[8], uint4 (&c)[8]) {
    uint32_t in[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i) { in[i][0] = r[i].x; in[i][1] = r[i].y; in[i][2] = r[i].z; in[i][3] = r[i].w; }
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        uint32_t e[4], o[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            e[p] = pack_lo16(in[2 * p][d], in[2 * p + 1][d]);
            o[p] = pack_hi16(in[2 * p][d], in[2 * p + 1][d]);
        }
        c[2 * d] = make_uint4(e[0], e[1], e[2], e[3]);
        c[2 * d + 1] = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

// Same repack with row i multiplied by s[i] in float and rounded back to the input format (nearest even).
template <bool F16>
__device__ __forceinline__ void transpose8x8_scaled(const uint4 (&r)[8], const float (&s)[8], uint4 (&c)[8]) {
    uint32_t in[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i) { in[i][0] = r[i].x; in[i][1] = r[i].y; in[i][2] = r[i].z; in[i][3] = r[i].w; }
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        uint32_t e[4], o[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const uint32_t x = in[2 * p][d], y = in[2 * p + 1][d];
            e[p] = In16<F16>::pack(In16<F16>::lo(x) * s[2 * p], In16<F16>::lo(y) * s[2 * p + 1]);
            o[p] = In16<F16>::pack(In16<F16>::hi(x) * s[2 * p], In16<F16>::hi(y) * s[2 * p + 1]);
        }
        c[2 * d] = make_uint4(e[0], e[1], e[2], e[3]);
        c[2 * d + 1] = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

// MODE 0: clipped sum (scale A rows, store the tile).  MODE 1: direct squared norm.  MODE 2: a chunk of one example's
// positions, its share of A_i^T G_i stored unscaled (direct norm of few long examples, see k_direct_chunks_finish).
template <int MODE, bool F16>
__global__ __launch_bounds__(kThreads, 2) void k_tn_bf16_rows(TnArgs a) {
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * BM * 128];   // A^T tile then G^T tile: [col][64 k]
    __shared__ float red[4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tile = blockIdx.x;
    const int tm = tile / a.tiles_n, tn = tile % a.tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;
    const int z = blockIdx.y;
    int k_begin, k_end;
    if (MODE == 0) {
        k_begin = z * a.kchunk;
        k_end = min(a.K, k_begin + a.kchunk);
    } else if (MODE == 2) {
        // slice z = (example, chunk of its positions): a.slices_per_example chunks of a.kchunk rows
        const int ex = z / a.slices_per_example, ch = z - ex * a.slices_per_example;
        k_begin = ex * a.T + ch * a.kchunk;
        k_end = min(ex * a.T + a.T, k_begin + a.kchunk);
    } else {
        k_begin = z * a.T;
        k_end = k_begin + a.T;
    }

    // global -> LDS task of this thread: waves 0,1 move A, waves 2,3 move G
    const int opnd = tid >> 7;
    const int local = tid & 127;
    const int cg = local & 15;          // 8-column group inside the 128-column tile
    const int kc = local >> 4;          // 8-row chunk inside the 64-row stage
    const uint16_t* X = opnd ? a.G : a.A;
    const int D = opnd ? a.N : a.M;
    const int col0 = (opnd ? n0 : m0) + cg * 8;
    const bool vec_ok = (D & 7) == 0;
    unsigned char* lds_x = lds + opnd * (BM * 128);

    // MFMA roles: 2 x 2 waves, each owns a 64 x 64 piece made of 2 x 2 MFMA tiles
    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = lane & 31, lhalf = lane >> 5;
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    uint4 stage[8];
    float scl[8];
    auto fetch = [&](int k0) {
        const int row0 = k0 + kc * 8;
        load_block(X, D, vec_ok, row0, k_end, col0, stage);
        if (MODE == 0 && opnd == 0) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int row = row0 + i;
                scl[i] = (row < k_end) ? a.clip[a.T == 1 ? row : row / a.T] : 0.f;
            }
        }
    };
    auto commit = [&]() {
        uint4 cols[8];
        if (MODE == 0 && opnd == 0) transpose8x8_scaled<F16>(stage, scl, cols);
        else transpose8x8(stage, cols);
#pragma unroll
        for (int j = 0; j < 8; ++j)
            *reinterpret_cast<uint4*>(lds_x + lds_off_bytes(cg * 8 + j, kc)) = cols[j];
    };

    if (k_begin < k_end) fetch(k_begin);
    for (int k0 = k_begin; k0 < k_end; k0 += BK) {
        commit();
        __syncthreads();
        if (k0 + BK < k_end) fetch(k0 + BK);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int row = wm * 64 + i * 32 + lrow;
                fa[i] = *reinterpret_cast<const bf16x8*>(lds + lds_off_bytes(row, ks * 2 + lhalf));
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int row = wn * 64 + j * 32 + lrow;
                fb[j] = *reinterpret_cast<const bf16x8*>(lds + BM * 128 + lds_off_bytes(row, ks * 2 + lhalf));
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = In16<F16>::mfma(fa[i], fb[j], acc[i][j]);
        }
        __syncthreads();
    }

    if (MODE == 0 || MODE == 2) {
        // accumulator element r of lane: row 8*(r/4) + 4*lhalf + r%4, column lrow of the 32 x 32 MFMA tile
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
    } else {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) s += acc[i][j][r] * acc[i][j][r];
        s = block_sum_256(s, red);
        if (tid == 0) a.out[(size_t)z * (a.tiles_m * a.tiles_n) + tile] = s;
    }
}

// ---------------------------------------------------------------------------
// Example-segmented kernel (T >= 32).
// ---------------------------------------------------------------------------
struct SegArgs {
    const uint16_t* A;
    const uint16_t* G;
    const float* clip;     // clipped sum only
    float* out;            // clipped: slice base (stride `slice` per unit) or grad; direct: partial[B][tiles]
    int64_t slice;
    int B, T, M, N;
    int tiles_m, tiles_n;
    int epu;               // examples per unit of work (one unit = one K slice); direct: 1
    int units;
    int accumulate;        // clipped with a single unit: add to out
};

// Workgroup b runs on XCD b % 8 (round-robin dispatch).  Units are dealt to XCDs so that the
// workgroups resident on one XCD at a time work on the same rows of A and G (same unit,
// neighbouring tiles) and share them through that XCD's L2.
// FAST: d_in, d_out and T are multiples of 8, so every 16-byte piece and every thread's 8 rows are all in or all out.
template <int MODE, bool FAST, bool F16>
__global__ __launch_bounds__(kThreads, 2) void k_tn_bf16_seg(SegArgs a) {
    __shared__ __attribute__((aligned(16))) unsigned char lds[2][2 * BM * 128];
    __shared__ float red[4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tiles = a.tiles_m * a.tiles_n;
    const int xcd = blockIdx.x & 7, jj = blockIdx.x >> 3;
    const int z = xcd + 8 * (jj / tiles);
    const int tile = jj % tiles;
    if (z >= a.units) return;
    const int tm = tile / a.tiles_n, tn = tile % a.tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;
    const int ex_begin = z * a.epu;
    const int ex_end = min(a.B, ex_begin + a.epu);
    const int spe = (a.T + BK - 1) / BK;                 // stages per example
    const int n_stages = (ex_end - ex_begin) * spe;

    const int opnd = tid >> 7;
    const int local = tid & 127;
    const int cg = local & 15;
    const int kc = local >> 4;
    const uint16_t* X = opnd ? a.G : a.A;
    const int D = opnd ? a.N : a.M;
    const int col0 = (opnd ? n0 : m0) + cg * 8;
    const bool vec_ok = (D & 7) == 0;
    const int lds_x = opnd * (BM * 128);

    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = lane & 31, lhalf = lane >> 5;
    f32x16 acc[2][2], tot[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) { acc[i][j][r] = 0.f; tot[i][j][r] = 0.f; }

    uint4 stage[8];
    // fast path: 16-byte pieces, and a thread's 8 rows are inside the example together (T % 8 == 0)
    const bool col_ok = col0 < D;
    const size_t row_bytes = (size_t)D * 2;
    int f_e = 0, f_sub = 0;         // (example, stage in example) of the next fetch
    auto fetch = [&]() {
        const int row0 = f_sub * BK + kc * 8;
        const uint16_t* Xi = X + (size_t)(ex_begin + f_e) * a.T * D;
        if (FAST) {
            if (col_ok && row0 < a.T) {
                const unsigned char* p = reinterpret_cast<const unsigned char*>(Xi + (size_t)row0 * D + col0);
#pragma unroll
                for (int i = 0; i < 8; ++i) stage[i] = *reinterpret_cast<const uint4*>(p + i * row_bytes);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) stage[i] = make_uint4(0u, 0u, 0u, 0u);
            }
        } else {
            load_block(Xi, D, vec_ok, row0, a.T, col0, stage);
        }
        if (++f_sub == spe) { f_sub = 0; ++f_e; }
    };
    // LDS addresses are loop invariant: 8 write slots, 4 read rows (the k-step only flips bits 5-6)
    int wr_off[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) wr_off[j] = lds_x + lds_off_bytes(cg * 8 + j, kc);
    int rd_a[2], rd_b[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        rd_a[i] = lds_off_bytes(wm * 64 + i * 32 + lrow, lhalf);
        rd_b[i] = BM * 128 + lds_off_bytes(wn * 64 + i * 32 + lrow, lhalf);
    }
    auto commit = [&](int buf) {
        uint4 cols[8];
        transpose8x8(stage, cols);
#pragma unroll
        for (int j = 0; j < 8; ++j) *reinterpret_cast<uint4*>(&lds[buf][wr_off[j]]) = cols[j];
    };
    auto kstep = [&](int buf, int ks, bool fresh) {
        bf16x8 fa[2], fb[2];
        // chunk (2*ks + lhalf) ^ swz(row) == (lhalf ^ swz(row)) ^ (2*ks): flip bits 5-6 of the byte offset
#pragma unroll
        for (int i = 0; i < 2; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(&lds[buf][rd_a[i] ^ (ks << 5)]);
#pragma unroll
        for (int j = 0; j < 2; ++j) fb[j] = *reinterpret_cast<const bf16x8*>(&lds[buf][rd_b[j] ^ (ks << 5)]);
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = In16<F16>::mfma(fa[i], fb[j], fresh ? zero : acc[i][j]);
    };

    if (n_stages > 0) {
        fetch();
        commit(0);
        if (n_stages > 1) fetch();
    }
    __syncthreads();
    int sub = 0;                    // stage index inside the current example
    int ex = ex_begin;
    for (int st = 0; st < n_stages; ++st) {
        const int cur = st & 1;
        if (st + 1 < n_stages) commit(cur ^ 1);
        if (st + 2 < n_stages) fetch();
        if (sub == 0) kstep(cur, 0, true); else kstep(cur, 0, false);
#pragma unroll
        for (int ks = 1; ks < BK / 16; ++ks) kstep(cur, ks, false);
        if (++sub == spe) {
            // this example's tile of A_i^T G_i is complete
            if (MODE == 0) {
                const float c = a.clip[ex];
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) tot[i][j][r] += c * acc[i][j][r];
            } else {
                float s = 0.f;
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) s += acc[i][j][r] * acc[i][j][r];
                s = block_sum_256(s, red);
                if (tid == 0) a.out[(size_t)ex * tiles + tile] = s;
            }
            sub = 0;
            ++ex;
        }
        __syncthreads();
    }

    if (MODE == 0) {
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
                        *p = a.accumulate ? *p + tot[i][j][r] : tot[i][j][r];
                    }
                }
            }
    }
}

inline bool seg_fast(int T, int M, int N) { return ((T | M | N) & 7) == 0; }

template <int MODE> void launch_seg(bool fast, bool f16, unsigned grid, const SegArgs& a, hipStream_t st) {
    if (fast) { if (f16) k_tn_bf16_seg<MODE, true, true><<<grid, kThreads, 0, st>>>(a); else k_tn_bf16_seg<MODE, true, false><<<grid, kThreads, 0, st>>>(a); }
    else      { if (f16) k_tn_bf16_seg<MODE, false, true><<<grid, kThreads, 0, st>>>(a); else k_tn_bf16_seg<MODE, false, false><<<grid, kThreads, 0, st>>>(a); }
}

// ---------------------------------------------------------------------------
// Large-tile clipped sum: 256 x 256 output tile per workgroup, one workgroup
// per compute unit (128 KB of LDS, double buffered), each wave owning a
// 128 x 128 piece (4 x 4 MFMA tiles, 256 accumulator registers).  Per 64-row
// stage a workgroup reads 64 KB for 8.4 MFLOP, i.e. 32 bytes per clock and
// compute unit at full MFMA rate, half of what the 128 x 128 tiles need.
// Rows of A are scaled by their example's clip factor while they are
// repacked (all 8 rows of a thread's block belong to one example because
// T % 8 == 0 here).  K slices are arbitrary multiples of 64 rows.
// Requires d_in % 8 == 0, d_out % 8 == 0, T % 8 == 0.
// ---------------------------------------------------------------------------
constexpr int GM = 256, GN = 256;

struct BigArgs {
    const uint16_t* A;
    const uint16_t* G;
    const float* clip;
    float* out;            // slice base (stride `slice` per K slice) or grad
    int64_t slice;
    int B, T, K, M, N;
    int tiles_m, tiles_n;
    int splits, kchunk;
    int per_xcd;           // workgroups per XCD
    int accumulate;
};

// Same repack as transpose8x8_scaled with one factor for all 8 rows.
template <bool F16>
__device__ __forceinline__ void transpose8x8_scaled1(const uint4 (&r)[8], float s, uint4 (&c)[8]) {
    uint32_t in[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i) { in[i][0] = r[i].x; in[i][1] = r[i].y; in[i][2] = r[i].z; in[i][3] = r[i].w; }
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        uint32_t e[4], o[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const uint32_t x = in[2 * p][d], y = in[2 * p + 1][d];
            e[p] = In16<F16>::pack(In16<F16>::lo(x) * s, In16<F16>::lo(y) * s);
            o[p] = In16<F16>::pack(In16<F16>::hi(x) * s, In16<F16>::hi(y) * s);
        }
        c[2 * d] = make_uint4(e[0], e[1], e[2], e[3]);
        c[2 * d + 1] = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

template <bool F16>
__global__ __launch_bounds__(kThreads, 1) void k_tn_bf16_big(BigArgs a) {
    __shared__ __attribute__((aligned(16))) unsigned char lds[2][2 * GM * 128];   // [buffer][A^T tile | G^T tile]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tiles = a.tiles_m * a.tiles_n;
    // workgroup b runs on XCD b % 8: give each XCD a contiguous run of (slice, tile) pairs so that
    // its workgroups stream the same rows of A and G through one L2
    const int L = (blockIdx.x & 7) * a.per_xcd + (blockIdx.x >> 3);
    if (L >= tiles * a.splits) return;
    const int z = L / tiles, tile = L - z * tiles;
    const int tm = tile / a.tiles_n, tn = tile - tm * a.tiles_n;
    const int m0 = tm * GM, n0 = tn * GN;
    const int k_begin = z * a.kchunk;
    const int k_end = min(a.K, k_begin + a.kchunk);
    const int n_stages = (k_end - k_begin + BK - 1) / BK;

    // global -> LDS: every thread moves one 8 x 8 block of A and one of G per stage
    const int cg = tid & 31;            // 8-column group in the 256-column tile
    const int kc = tid >> 5;            // 8-row chunk in the 64-row stage
    const int colA = m0 + cg * 8, colG = n0 + cg * 8;
    const bool okA = colA < a.M, okG = colG < a.N;
    const size_t rbA = (size_t)a.M * 2, rbG = (size_t)a.N * 2;
    int row = k_begin + kc * 8;         // first row of this thread's block in the next stage to fetch
    int ex = row / a.T, rem = row - ex * a.T;

    uint4 stA[8], stG[8];
    float scl = 0.f;
    auto fetch = [&]() {
        const bool in = row < k_end;
        if (in && okA) {
            const unsigned char* p = reinterpret_cast<const unsigned char*>(a.A + (size_t)row * a.M + colA);
#pragma unroll
            for (int i = 0; i < 8; ++i) stA[i] = *reinterpret_cast<const uint4*>(p + i * rbA);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) stA[i] = make_uint4(0u, 0u, 0u, 0u);
        }
        if (in && okG) {
            const unsigned char* p = reinterpret_cast<const unsigned char*>(a.G + (size_t)row * a.N + colG);
#pragma unroll
            for (int i = 0; i < 8; ++i) stG[i] = *reinterpret_cast<const uint4*>(p + i * rbG);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) stG[i] = make_uint4(0u, 0u, 0u, 0u);
        }
        scl = a.clip[min(ex, a.B - 1)];
        row += BK; rem += BK;
        while (rem >= a.T) { rem -= a.T; ++ex; }
    };
    int wrA[8], wrG[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        wrA[j] = lds_off_bytes(cg * 8 + j, kc);
        wrG[j] = GM * 128 + wrA[j];
    }
    auto commit = [&](int buf) {
        uint4 cols[8];
        transpose8x8_scaled1<F16>(stA, scl, cols);
#pragma unroll
        for (int j = 0; j < 8; ++j) *reinterpret_cast<uint4*>(&lds[buf][wrA[j]]) = cols[j];
        transpose8x8(stG, cols);
#pragma unroll
        for (int j = 0; j < 8; ++j) *reinterpret_cast<uint4*>(&lds[buf][wrG[j]]) = cols[j];
    };

    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = lane & 31, lhalf = lane >> 5;
    int rdA[4], rdG[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        rdA[i] = lds_off_bytes(wm * 128 + i * 32 + lrow, lhalf);
        rdG[i] = GM * 128 + lds_off_bytes(wn * 128 + i * 32 + lrow, lhalf);
    }
    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    if (n_stages > 0) {
        fetch();
        commit(0);
        if (n_stages > 1) fetch();
    }
    __syncthreads();
    for (int st = 0; st < n_stages; ++st) {
        const int cur = st & 1;
        if (st + 1 < n_stages) commit(cur ^ 1);
        if (st + 2 < n_stages) fetch();
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fa[4], fb[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(&lds[cur][rdA[i] ^ (ks << 5)]);
#pragma unroll
            for (int j = 0; j < 4; ++j) fb[j] = *reinterpret_cast<const bf16x8*>(&lds[cur][rdG[j] ^ (ks << 5)]);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = In16<F16>::mfma(fa[i], fb[j], acc[i][j]);
        }
        __syncthreads();
    }

    float* out = a.out + (size_t)z * a.slice;
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
                    *p = a.accumulate ? *p + acc[i][j][r] : acc[i][j][r];
                }
            }
        }
}

// Use the 256 x 256 kernel when the shape is aligned and its padded tiles waste at most a quarter.
inline bool big_ok(int T, int M, int N) {
    if (((T | M | N) & 7) != 0) return false;
    const int64_t padded = (int64_t)ceil_div(M, GM) * GM * ceil_div(N, GN) * GN;
    return padded * 4 <= (int64_t)M * N * 5;
}

constexpr int kSegMinT = 32;      // below this an LDS stage would be mostly padding


}  // namespace

TnPlan plan_clipped_bf16(int B, int T, int M, int N) {
    if (dma_clipped_ok(B, T, M, N)) return plan_clipped_bf16_dma(B, T, M, N, true);
    TnPlan p;
    p.dma = false;
    p.tile_m = BM; p.tile_n = BN;
    p.tiles_m = ceil_div(M, BM); p.tiles_n = ceil_div(N, BN);
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    // Every K slice beyond the first costs a write and a read of M*N floats.  Where that outweighs the inputs (a short
    // contraction into a large matrix: a few examples of a few positions, thousands of columns), the layer is bound
    // by its output and slices of a few stages to fill the chip multiply exactly that: slices of at least 16 stages
    // there (a long contraction still gains more from the parallel slices than their traffic costs).
    const int64_t in_bytes = (int64_t)B * T * ((int64_t)M + N) * 2;
    int64_t traffic_cap = (int64_t)M * N * 8 > in_bytes ? (int64_t)B * T / (16 * BK) : (int64_t(1) << 40);
    if (traffic_cap < 1) traffic_cap = 1;
    p.big = big_ok(T, M, N);
    if (p.big) {
        // one workgroup per compute unit: as many K slices as fit in 256 workgroups
        const int64_t bt = (int64_t)ceil_div(M, GM) * ceil_div(N, GN);
        int64_t splits = 256 / bt;
        if (splits < 1) splits = 1;
        if (splits > traffic_cap) splits = traffic_cap;
        // few large tiles and no slices to multiply them: the 128 x 128 tiles below give four times the workgroups
        if (bt * splits < 128 && bt * splits < tiles) p.big = false;
    }
    if (p.big) {
        p.tile_m = GM; p.tile_n = GN;
        p.tiles_m = ceil_div(M, GM); p.tiles_n = ceil_div(N, GN);
        const int64_t bt = (int64_t)p.tiles_m * p.tiles_n;
        const int64_t K = (int64_t)B * T;
        int64_t splits = 256 / bt;
        if (splits < 1) splits = 1;
        if (splits > traffic_cap) splits = traffic_cap;
        const int64_t max_splits = (K + 2 * BK - 1) / (2 * BK);
        if (splits > max_splits) splits = max_splits;
        int64_t kchunk = (K + splits - 1) / splits;
        kchunk = ((kchunk + BK - 1) / BK) * BK;
        p.kchunk = (int)kchunk;
        p.splits = (int)((K + kchunk - 1) / kchunk);
        p.segmented = false; p.epu = 0;
        return p;
    }
    // the example-by-example kernel has at most one K slice per example: with few examples (a handful of long
    // sequences) it would leave most of the chip idle, and the kernel below, whose K slices are any rows, takes over
    p.segmented = (T >= kSegMinT) && (int64_t)B * tiles >= 64;
    if (p.segmented) {
        // K slices are whole examples.  Aim for a few workgroups per compute unit, in multiples of the
        // 8 XCDs, without multiplying the fp32 slice traffic more than needed.
        int64_t units = (768 + tiles - 1) / tiles;
        units = ((units + 7) / 8) * 8;
        // every slice costs a write and a read of M*N floats: keep that below a quarter of the input bytes
        const int64_t in_bytes = (int64_t)B * T * ((int64_t)M + N) * 2;
        int64_t cap = in_bytes / 4 / ((int64_t)M * N * 8);
        cap = (cap / 8) * 8;
        if (cap < 8) cap = 8;
        if (units > cap) units = cap;
        if (units > B) units = B;
        p.epu = ceil_div(B, units);
        p.splits = ceil_div(B, p.epu);
        p.kchunk = p.epu * T;
        return p;
    }
    const int64_t K = (int64_t)B * T;
    // enough K slices for about two workgroups per compute unit, each at least 4 stages long
    int64_t want = (512 + tiles - 1) / tiles;
    int64_t max_splits = (K + 4 * BK - 1) / (4 * BK);
    if (want > max_splits) want = max_splits;
    if (want > traffic_cap) want = traffic_cap;
    if (want < 1) want = 1;
    int64_t kchunk = (K + want - 1) / want;
    kchunk = ((kchunk + BK - 1) / BK) * BK;
    if (kchunk < BK) kchunk = BK;
    p.kchunk = (int)kchunk;
    p.epu = 0;
    p.splits = (int)((K + kchunk - 1) / kchunk);
    if (p.splits < 1) p.splits = 1;
    return p;
}

TnPlan plan_direct_bf16(int B, int T, int M, int N) {
    TnPlan p;
    if (dma_direct_ok(T, M, N)) return plan_direct_bf16_dma(B, T, M, N);
    p.tile_m = BM; p.tile_n = BN;
    p.tiles_m = ceil_div(M, BM); p.tiles_n = ceil_div(N, BN);
    p.segmented = (T >= kSegMinT);
    p.big = false; p.dma = false;
    p.splits = 1; p.kchunk = 0; p.epu = 1;
    plan_direct_chunks(p, B, T, M, N, 2, BK);
    return p;
}

hipError_t launch_clipped_bf16(const TnPlan& p, const uint16_t* A, const uint16_t* G, const float* clip,
                               int B, int T, int M, int N, bool accumulate, float* grad, float* ws, hipStream_t st, bool f16,
                               const NoiseArgs* noise) {
    const int64_t n = (int64_t)M * N;
    const int tiles = p.tiles_m * p.tiles_n;
    if (p.dma) return launch_clipped_bf16_dma(p, A, G, clip, B, T, M, N, accumulate, grad, ws, st, nullptr, nullptr, f16, noise);
    if (p.big) {
        BigArgs a;
        a.A = A; a.G = G; a.clip = clip;
        a.B = B; a.T = T; a.K = B * T; a.M = M; a.N = N;
        a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n; a.splits = p.splits; a.kchunk = p.kchunk;
        a.per_xcd = ceil_div((int64_t)tiles * p.splits, 8);
        if (p.splits == 1) { a.out = grad; a.slice = 0; a.accumulate = accumulate ? 1 : 0; }
        else { a.out = ws; a.slice = splitk_slice_elems(n); a.accumulate = 0; }
        if (f16) k_tn_bf16_big<true><<<8u * (unsigned)a.per_xcd, kThreads, 0, st>>>(a);
        else     k_tn_bf16_big<false><<<8u * (unsigned)a.per_xcd, kThreads, 0, st>>>(a);
    } else if (p.segmented) {
        SegArgs a;
        a.A = A; a.G = G; a.clip = clip;
        a.B = B; a.T = T; a.M = M; a.N = N;
        a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n; a.epu = p.epu; a.units = p.splits;
        if (p.splits == 1) { a.out = grad; a.slice = 0; a.accumulate = accumulate ? 1 : 0; }
        else { a.out = ws; a.slice = splitk_slice_elems(n); a.accumulate = 0; }
        const unsigned grid = 8u * (unsigned)ceil_div(p.splits, 8) * (unsigned)tiles;
        launch_seg<0>(seg_fast(T, M, N), f16, grid, a, st);
    } else {
        TnArgs a;
        a.A = A; a.G = G; a.clip = clip;
        a.K = B * T; a.T = T; a.M = M; a.N = N;
        a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n; a.kchunk = p.kchunk;
        if (p.splits == 1) { a.out = grad; a.slice = 0; a.accumulate = accumulate ? 1 : 0; }
        else { a.out = ws; a.slice = splitk_slice_elems(n); a.accumulate = 0; }
        dim3 grid((unsigned)tiles, (unsigned)p.splits);
        if (f16) k_tn_bf16_rows<0, true><<<grid, kThreads, 0, st>>>(a);
        else     k_tn_bf16_rows<0, false><<<grid, kThreads, 0, st>>>(a);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.splits == 1) return e;
    return launch_splitk_reduce(ws, n, p.splits, accumulate, grad, st, noise);
}

hipError_t launch_direct_bf16(const TnPlan& p, const uint16_t* A, const uint16_t* G, int B, int T, int M, int N,
                              bool accumulate, float* sqnorm, float* partial, hipStream_t st, bool f16, const ClipOut* co) {
    if (p.dma) return launch_direct_bf16_dma(p, A, G, B, T, M, N, accumulate, sqnorm, partial, st, nullptr, nullptr, f16, co);
    const int tiles = p.tiles_m * p.tiles_n;
    if (p.splits > 1) {
        // chunks of positions: workspace = the chunks' shares [B][S][slice], then partial[B][nblk]
        const int64_t n = (int64_t)M * N, slice = splitk_slice_elems(n);
        const int nblk = (int)((n + 1023) / 1024);
        float* shares = partial;
        float* sums = partial + (size_t)B * p.splits * slice;
        TnArgs a;
        a.A = A; a.G = G; a.clip = nullptr;
        a.K = B * T; a.T = T; a.M = M; a.N = N;
        a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n; a.kchunk = p.kchunk;
        a.out = shares; a.slice = slice; a.accumulate = 0; a.slices_per_example = p.splits;
        dim3 grid((unsigned)tiles, (unsigned)(B * p.splits));
        if (f16) k_tn_bf16_rows<2, true><<<grid, kThreads, 0, st>>>(a);
        else     k_tn_bf16_rows<2, false><<<grid, kThreads, 0, st>>>(a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        e = launch_direct_chunks_finish(shares, slice, p.splits, (int)n, B, sums, st);
        if (e != hipSuccess) return e;
        return launch_finalize_partials(sums, B, nblk, accumulate, sqnorm, st, co);
    }
    if (p.segmented) {
        // one launch covers at most 2^20 examples so that the workgroup count stays far below 2^31
        for (int b0 = 0; b0 < B; b0 += (1 << 20)) {
            const int nb = (B - b0 < (1 << 20)) ? (B - b0) : (1 << 20);
            SegArgs a;
            a.A = A + (size_t)b0 * T * M; a.G = G + (size_t)b0 * T * N; a.clip = nullptr;
            a.B = nb; a.T = T; a.M = M; a.N = N;
            a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n; a.epu = 1; a.units = nb;
            a.out = partial + (size_t)b0 * tiles; a.slice = 0; a.accumulate = 0;
            const int64_t grid = 8ll * ceil_div(nb, 8) * tiles;
            if (grid >= (int64_t(1) << 31)) return hipErrorInvalidValue;
            launch_seg<1>(seg_fast(T, M, N), f16, (unsigned)grid, a, st);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
        return launch_finalize_partials(partial, B, tiles, accumulate, sqnorm, st, co);
    }
    TnArgs a;
    a.A = A; a.G = G; a.clip = nullptr;
    a.K = B * T; a.T = T; a.M = M; a.N = N;
    a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n; a.kchunk = 0;
    a.out = partial; a.slice = 0; a.accumulate = 0;
    // grid.y is limited to 65535: fold larger batches into several launches
    for (int b0 = 0; b0 < B; b0 += 65535) {
        const int nb = (B - b0 < 65535) ? (B - b0) : 65535;
        TnArgs s = a;
        s.A = A + (size_t)b0 * T * M;
        s.G = G + (size_t)b0 * T * N;
        s.out = partial + (size_t)b0 * tiles;
        dim3 grid((unsigned)tiles, (unsigned)nb);
        if (f16) k_tn_bf16_rows<1, true><<<grid, kThreads, 0, st>>>(s);
        else     k_tn_bf16_rows<1, false><<<grid, kThreads, 0, st>>>(s);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return launch_finalize_partials(partial, B, tiles, accumulate, sqnorm, st, co);
}

}  // namespace dpk
