// Host-side launcher interface between the C-ABI layer (dp_api.hip) and the
// kernel translation units.  Every launcher validates nothing: dp_api.hip has
// already checked sizes and the workspace.  Each returns hipGetLastError().
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace dpk {

inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }
// an M x N output tiles into TM x TN blocks with at most a quarter of the padded area wasted
inline bool tiles_fit(int M, int N, int TM, int TN) {
    const int64_t padded = (int64_t)ceil_div(M, TM) * TM * ceil_div(N, TN) * TN;
    return padded * 4 <= (int64_t)M * N * 5;
}

// ---- small elementwise / reduction kernels (dp_small_kernels.hip)
// dt: 0 = float32, 1 = bf16, 2 = fp16 (the values of dp_dtype)
// Where a norm launcher's last kernel completes the norms of the whole model, it can write the clip factors
// clip[i] = 1 / max(1, sqrt(s_i) / C) too (co != nullptr), which saves the launch of their own kernel.
// defer: the several-layers call collects the partial sums of its layers that run one by one and folds them all in
// one launch at the end (launch_finalize_queue) instead of one small launch per layer; a launcher that ends in
// launch_finalize_partials then only records where its partial sums are.
struct FinalizeQueue { static constexpr int kMax = 16; const float* partial[kMax]; int n[kMax]; int count = 0; };
struct ClipOut { float C; float* clip; FinalizeQueue* defer = nullptr; };
hipError_t launch_finalize_queue(const FinalizeQueue& q, int B, bool accumulate, float* sqnorm, hipStream_t st, const ClipOut* co);
hipError_t launch_sqnorm_dense(const void* A, const void* G, int B, int d_in, int d_out, int dt,
                               bool accumulate, float* sqnorm, hipStream_t st, const ClipOut* co = nullptr);
constexpr int kDenseBatch = 16;        // dense (T = 1) layers per launch of the several-layers call
struct DenseLayers { int n_layers; const void* A[kDenseBatch]; const void* G[kDenseBatch]; int d_in[kDenseBatch]; int d_out[kDenseBatch]; };
hipError_t launch_sqnorm_dense_layers(const DenseLayers& t, int B, int dt, bool accumulate, float* sqnorm, hipStream_t st,
                                      const ClipOut* co = nullptr);
hipError_t launch_finalize_partials(const float* partial, int B, int n_per_example, bool accumulate,
                                    float* sqnorm, hipStream_t st, const ClipOut* co = nullptr);
// s_i (+)= sum over the layers l, then over j < n[l], of partial[first[l] + i * n[l] + j], in that order
constexpr int kGramBatch = 16;         // layers per batched Gram launch
struct FinalizeLayers { int n_layers; int first[kGramBatch]; int n[kGramBatch]; };
// clip != nullptr: also clip[i] = 1 / max(1, sqrt(s_i) / C) of the finished sums
hipError_t launch_finalize_layers(const float* partial, const FinalizeLayers& f, int B, bool accumulate, float* sqnorm, hipStream_t st,
                                  float C, float* clip);
// The same with an output array of its own per layer (per-layer or grouped norms; layers of one group name the same
// array and are added in the order given):  out[l][i] = (acc[l] ? out[l][i] : 0) + sum_j partial[first[l] + i n[l] + j],
// then clip[l][i] = 1 / max(1, sqrt(out[l][i]) / C[l]) where clip[l] != nullptr.
struct FinalizeEach { int n_layers; int first[kGramBatch]; int n[kGramBatch]; int acc[kGramBatch]; float C[kGramBatch];
                      float* out[kGramBatch]; float* clip[kGramBatch]; };
hipError_t launch_finalize_each(const float* partial, const FinalizeEach& f, int B, hipStream_t st);
hipError_t launch_clip_factors(const float* sqnorm, int B, float C, float* clip, hipStream_t st);
// distance in floats between consecutive split-K slices of an n-element output
inline int64_t splitk_slice_elems(int64_t n) { return (n + 3) & ~(int64_t)3; }
// Gaussian noise that the split-K reduce can add while it holds the sums (stddev == 0: none)
struct NoiseArgs { float stddev; uint32_t k0, k1; uint64_t offset; };
bool splitk_noise_ok(int64_t n, uint64_t offset);       // n and offset multiples of 4
hipError_t launch_splitk_reduce(const float* ws, int64_t n, int splits, bool accumulate, float* grad, hipStream_t st,
                                const NoiseArgs* noise);
// the folds of up to kJointLayers layers in one launch; the caller fills ws, grad, n, splits, noise_offset and n_layers
constexpr int kJointLayers = 16;
struct FoldLayers {
    const float* ws[kJointLayers]; float* grad[kJointLayers]; int64_t n[kJointLayers], slice[kJointLayers];
    uint64_t noise_offset[kJointLayers]; int splits[kJointLayers]; unsigned first_block[kJointLayers]; int n_layers;
};
hipError_t launch_splitk_reduce_layers(FoldLayers& f, bool accumulate, hipStream_t st, float stddev, uint64_t seed);
hipError_t launch_fill_zero(float* p, int64_t n, hipStream_t st);
// kZeroHeadFloats floats of zeros that live in the device image of the current GPU (nothing to fill, no launch), or
// nullptr when they cannot be looked up now (first use on this GPU while `st` is being captured): the caller then
// fills the head of its workspace as before.
const void* device_zero_line(hipStream_t st);
// dst[j] = fp16 bits of the 8-bit float src[j] (e4m3, or e5m2 when e5m2 is set), exact
hipError_t launch_widen_f8(const void* src, uint16_t* dst, int64_t n, bool e5m2, hipStream_t st);
hipError_t launch_add_noise(float* grad, int64_t n, float stddev, uint64_t seed, uint64_t offset, hipStream_t st);
// ---- bias parameters (dp_bias.hip)
hipError_t launch_bias_rows(const void* G, const void* Hb, int B, int T, int D, int dt, float* u, float* u2, hipStream_t st);
// u[i, :] = sum over nt row tiles of upart[i, tt, :];  s_i (+)= ||u[i, :]||^2
hipError_t launch_bias_fold(const float* upart, int B, int nt, int D, bool accumulate, float* u, float* sqnorm, hipStream_t st);
// s_i (+)= ||u[i, :]||^2, then + ||u2[i, :]||^2 where u2 is given
hipError_t launch_rows_sqnorm(const float* u, int B, int D, bool accumulate, float* sqnorm, hipStream_t st, const float* u2 = nullptr);
hipError_t launch_clipped_bias(const float* u, const float* clip, int B, int D, bool accumulate, float* grad_b, hipStream_t st);
hipError_t launch_philox_raw(uint32_t* out, int64_t n_counters, uint64_t seed, uint64_t first, hipStream_t st);

// ---- K-major ("TN") products  sum_k A[k,:]^T G[k,:]  (dp_tn_bf16.hip, dp_tn_f32.hip)
struct TnPlan {
    int tile_m, tile_n;     // block tile
    int tiles_m, tiles_n;
    int splits;             // clipped grad: number of K slices; direct sqnorm: unused
    int kchunk;             // rows of K per slice
    bool segmented;         // 16-bit inputs only: K is walked example by example (slices are whole examples)
    int epu;                // segmented: examples per K slice
    bool big;               // 16-bit clipped sum only: 256 x 256 tiles, one workgroup per compute unit
    bool zero_head = false; // the kernel needs a line of zeros: the first kZeroHeadFloats floats of the workspace are set aside for it
    bool dma;               // copy-pipeline kernel (direct-to-LDS copies); tile_m x tile_n names its geometry (16-bit inputs) or is 128 x 128 (float32)
};
constexpr int kZeroHeadFloats = 64;   // 256 bytes
// direct norm in chunks of positions (few long examples of a small layer): sets p.splits (chunks per example) and
// p.kchunk (rows per chunk) where that pays; the chunks' shares [B][splits][splitk_slice_elems(M N)] are added, squared
// and summed into sums[B][ceil(M N / 1024)] by launch_direct_chunks_finish
void plan_direct_chunks(TnPlan& p, int B, int T, int M, int N, int esize, int stage);
hipError_t launch_direct_chunks_finish(const float* shares, int64_t slice, int S, int n, int B, float* sums, hipStream_t st);
TnPlan plan_clipped_bf16(int B, int T, int M, int N);
TnPlan plan_clipped_f32(int B, int T, int M, int N);
TnPlan plan_direct_bf16(int B, int T, int M, int N);
// stride-1 convolution given by its channels-last input image (implicit unfolding in the copy-pipeline kernel)
struct ConvGeom { int H, W, C, KH, KW, pad; };
bool dma_conv_ok(const ConvGeom& g, int d_out);
// 3 x 3 kernels over at least 64 channels (a multiple of 64), a multiple of 32 output positions: the kernel that keeps
// the image rows in LDS and copies every pixel once (dp_conv_rows.hip)
bool conv_rows_ok(const ConvGeom& g, int d_out, int B);
int conv_rows_tiles(const ConvGeom& g, int d_out);              // partial sums per example of the direct norm
int conv_rows_splits(const ConvGeom& g, int d_out, int B);      // K slices of the clipped sum
bool dma_clipped_ok(int B, int T, int M, int N);
// flat: the rows of A lie in memory as they are (not the implicit unfolding of an image)
TnPlan plan_clipped_bf16_dma(int B, int T, int M, int N, bool flat = false);
TnPlan plan_direct_f32(int B, int T, int M, int N);
// float32 copy-pipeline kernel (dp_tn_f32_dma.hip): 128 x 128 tiles, 16-row stages; the plans above choose it (dma = true)
// for long contractions of shapes it fits
bool f32_dma_ok(int64_t K, int M, int N);
int f32_dma_tile();
int f32_dma_stage_rows();
hipError_t launch_tn_f32_dma(int mode, const TnPlan& p, const float* A, const float* G, const float* clip, int B, int T,
                             int M, int N, float* out, int64_t slice, bool accumulate, hipStream_t st);

// The 16-bit launchers below take bf16 bits, or fp16 bits when f16 is set.
// out: splits == 1 -> nullptr workspace allowed and the tile goes straight to `grad` (overwrite
// or accumulate); otherwise slices go to ws[splits][M][N] and a second kernel folds them.
hipError_t launch_clipped_bf16(const TnPlan& p, const uint16_t* A, const uint16_t* G, const float* clip,
                               int B, int T, int M, int N, bool accumulate, float* grad, float* ws, hipStream_t st, bool f16,
                               const NoiseArgs* noise);
hipError_t launch_clipped_bf16_dma(const TnPlan& p, const uint16_t* A, const uint16_t* G, const float* clip,
                                   int B, int T, int M, int N, bool accumulate, float* grad, float* ws, hipStream_t st,
                                   const ConvGeom* cg, const uint16_t* zero, bool f16, const NoiseArgs* noise);
hipError_t launch_direct_conv_rows(const ConvGeom& g, const uint16_t* X, const uint16_t* G, int B, int N, bool accumulate,
                                   float* sqnorm, float* partial, hipStream_t st, const uint16_t* zero, bool f16,
                                   const ClipOut* co = nullptr);
hipError_t launch_clipped_conv_rows(const ConvGeom& g, const uint16_t* X, const uint16_t* G, const float* clip, int B, int N,
                                    bool accumulate, float* grad, float* ws, hipStream_t st, const uint16_t* zero, bool f16,
                                    const NoiseArgs* noise);
// Several layers' clipped sums in one launch (16-bit inputs, 256 x 256 tiles, T a multiple of 32): the K slices of all
// layers are cut to about one length so that the launch fills the chip a whole number of times; the layers' slices
// are then folded (+ noise) by the split-K reduce kernel as after a launch per layer.  Same arithmetic per slice and
// the same ascending fold; the slices are cut differently, so the results agree with the per-layer launch up to the
// rounding of the float32 sum over slices.
struct JointShape { int T, M, N; };
struct JointOperands { const uint16_t* A; const uint16_t* G; const float* clip; float* grad; uint64_t noise_offset; };
// One slice length for all layers of a joint launch (each layer rounds it to a whole number of equal slices), chosen
// to minimise   rounds of 256 workgroups  x  (stages of the longest slice + what an item costs besides its stages):
// slices long enough that their start-up, their store and their fold stay small, and a number of items that fills
// the chip's 256 compute units a whole number of times.  dk: rows per stage; tile: the square output tile; slots:
// workgroups resident at a time (256 x workgroups per compute unit).
struct JointPlan { int n_layers; int tiles_m[kJointLayers], tiles_n[kJointLayers], splits[kJointLayers], sps[kJointLayers]; int64_t items; };
inline JointPlan plan_joint(const JointShape* sh, int n_layers, int B, int dk, int tile, int slots = 256) {
    constexpr int64_t kItemOverhead = 16;            // prologue + slice store + the slice's share of the fold, in stage times
    JointPlan best{};
    int64_t best_cost = -1, stages_max = 1;
    for (int l = 0; l < n_layers; ++l) stages_max = stages_max > (int64_t)B * ceil_div(sh[l].T, dk) ? stages_max : (int64_t)B * ceil_div(sh[l].T, dk);
    for (int64_t S = 1; S <= 512 && S <= stages_max; ++S) {
        const int64_t len = (stages_max + S - 1) / S;
        if (len < 8 && S > 1) break;
        JointPlan p{};
        p.n_layers = n_layers;
        int64_t longest = 0;
        for (int l = 0; l < n_layers; ++l) {
            const int64_t spe = ceil_div(sh[l].T, dk), stages = (int64_t)B * spe;
            const int64_t want = len < 63 * spe ? len : 63 * spe;   // a slice touches at most 64 examples (one clip factor per lane)
            int64_t splits = (stages + want - 1) / want;
            const int64_t sps = (stages + splits - 1) / splits;
            splits = (stages + sps - 1) / sps;                      // no empty slice
            p.tiles_m[l] = ceil_div(sh[l].M, tile); p.tiles_n[l] = ceil_div(sh[l].N, tile);
            p.splits[l] = (int)splits; p.sps[l] = (int)sps;
            p.items += (int64_t)p.tiles_m[l] * p.tiles_n[l] * splits;
            longest = longest > sps ? longest : sps;
        }
        const int64_t cost = ((p.items + slots - 1) / slots) * (longest + kItemOverhead);
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = p; }
    }
    return best;
}
bool dma_joint_ok(int T, int M, int N);
bool dma_joint_mid_ok(int T, int M, int N);      // the second class: 128 x 128 tiles, geo = 3 below
bool dma_joint_ragged_ok(int T, int M, int N);   // the same tiles, T not a multiple of the stage: geo = 4
size_t joint_workspace_floats(const JointShape* sh, int n_layers, int B, int geo = 1);
// the same for float32 inputs (dp_tn_f32_dma.hip; 128 x 128 tiles, any T); A, G of JointOperands are float pointers
size_t joint_f32_workspace_floats(const JointShape* sh, int n_layers, int B);
hipError_t launch_direct_f32_dma_joint(const JointShape* sh, const JointOperands* op, float* const* partial, int n_layers,
                                       int B, hipStream_t st);
hipError_t launch_clipped_f32_dma_joint(const JointShape* sh, const JointOperands* op, int n_layers, int B, bool accumulate,
                                        float stddev, uint64_t seed, float* ws, hipStream_t st);
// the same for 8-bit inputs (dp_tn_f8_dma.hip; 256 x 256 tiles, T a multiple of 64); A, G of JointOperands are byte pointers
bool dma8_joint_ok(int T, int M, int N);
size_t joint8_workspace_floats(const JointShape* sh, int n_layers, int B);
hipError_t launch_clipped_f8_dma_joint(const JointShape* sh, const JointOperands* op, int n_layers, int B, bool accumulate,
                                       float stddev, uint64_t seed, float* ws, hipStream_t st, int fmt);
// noise: stddev == 0 for none, else every layer's d_in * d_out and noise_offset are multiples of 4
hipError_t launch_clipped_bf16_dma_joint(const JointShape* sh, const JointOperands* op, int n_layers, int B, bool accumulate,
                                         float stddev, uint64_t seed, float* ws, hipStream_t st, bool f16, int geo = 1);
// several layers' direct norms in one launch (128 x 128 tiles; T >= 64, widths multiples of 8); partial[l]: the layer's
// [B][direct_joint_tiles(M, N)] sums of squares per (example, tile), to be added by the caller
bool dma_direct_joint_ok(int B, int T, int M, int N);
int direct_joint_tiles(int M, int N);
hipError_t launch_direct_bf16_dma_joint(const JointShape* sh, const JointOperands* op, float* const* partial, int n_layers,
                                        int B, hipStream_t st, bool f16);
// direct squared norm with the copy-pipeline kernel; partial[B][tiles_m * tiles_n]
bool dma_direct_ok(int T, int M, int N);
TnPlan plan_direct_bf16_dma(int B, int T, int M, int N);
hipError_t launch_direct_bf16_dma(const TnPlan& p, const uint16_t* A, const uint16_t* G, int B, int T, int M, int N,
                                  bool accumulate, float* sqnorm, float* partial, hipStream_t st,
                                  const ConvGeom* cg, const uint16_t* zero, bool f16, const ClipOut* co = nullptr);
// 8-bit inputs (dp_tn_f8_dma.hip); fmt: 2 = A and G e4m3, 3 = A and G e5m2, 4 = A e4m3 and G e5m2
bool dma8_clipped_ok(int T, int M, int N);
bool dma8_direct_ok(int T, int M, int N);
TnPlan plan_clipped_f8_dma(int B, int T, int M, int N);
TnPlan plan_direct_f8_dma(int B, int T, int M, int N);
hipError_t launch_clipped_f8_dma(const TnPlan& p, const void* A, const void* G, const float* clip,
                                 int B, int T, int M, int N, bool accumulate, float* grad, float* ws, hipStream_t st,
                                 int fmt, const NoiseArgs* noise);
hipError_t launch_direct_f8_dma(const TnPlan& p, const void* A, const void* G, int B, int T, int M, int N,
                                bool accumulate, float* sqnorm, float* partial, hipStream_t st, int fmt, const ClipOut* co = nullptr);
// float32 layers with a short contraction (B T <= 512: plan_clipped_f32 gives them one 32 x 32-tile kernel without K
// slices), up to 8 in one launch; per layer the same arithmetic as launch_clipped_f32
bool clipped_f32_is_short(const TnPlan& p);
struct ShortLayerDesc { const float* A; const float* G; const float* clip; float* grad; int T, M, N; };
hipError_t launch_clipped_f32_short_layers(const ShortLayerDesc* layers, int n_layers, int B, bool accumulate, hipStream_t st);
hipError_t launch_clipped_f32(const TnPlan& p, const float* A, const float* G, const float* clip,
                              int B, int T, int M, int N, bool accumulate, float* grad, float* ws, hipStream_t st,
                              const NoiseArgs* noise);
// partial[B][tiles_m*tiles_n] then finalize into sqnorm
hipError_t launch_direct_bf16(const TnPlan& p, const uint16_t* A, const uint16_t* G, int B, int T, int M, int N,
                              bool accumulate, float* sqnorm, float* partial, hipStream_t st, bool f16, const ClipOut* co = nullptr);
hipError_t launch_direct_f32(const TnPlan& p, const float* A, const float* G, int B, int T, int M, int N,
                             bool accumulate, float* sqnorm, float* partial, hipStream_t st, const ClipOut* co = nullptr);

// ---- Gram path, 16-bit inputs (dp_gram_bf16.hip, dp_gram_bf16_dma.hip)
struct GramPlan {
    int tile;     // rows of T per tile
    int nt;       // tiles along T
    int npairs;   // nt*(nt+1)/2 upper-triangular tile pairs per example
};
GramPlan plan_gram_bf16(int T, int d_in, int d_out);
// fmt (copy-pipeline launchers): 0 = bf16, 1 = fp16, 2 = A and G e4m3, 3 = A and G e5m2, 4 = A e4m3 and G e5m2
bool gram_dma_ok(int T, int d_in, int d_out, int fmt = 0);
// upart: nullptr, or [B][ceil(T / 128)][d_out] floats that receive the column sums of G over each 128-row tile
// bias_rows: nullptr, or float32[B, d_out] that receives sum_t G_i[t, :] (then upart is its scratch and ||bias_rows_i||^2 joins the norm)
// out: nullptr, or this layer's own output array (then every layer of the launch has one): out_acc = whether the array
// already holds a value to add to (the same for all layers naming the array), out_clip / out_C = nullptr, or where the
// array's clip factors go once the launch's last layer naming it has been added
struct GramLayerDesc { const void* A; const void* G; int T, d_in, d_out; float* upart; float* bias_rows;
                       float* out = nullptr; bool out_acc = false; float out_C = 0.f; float* out_clip = nullptr; };
// few positions (T <= 64), wide rows, small batch (dp_gram_cols.hip): the columns are split over workgroups.
// dt: 0 float32, 1 bf16, 2 fp16 (the values of dp_dtype); use: whether this kernel takes the shape; ws_floats: its scratch
struct GramColsPlan { bool use; int nb, W, per_wave; size_t ws_floats; };
GramColsPlan plan_gram_cols(int B, int T, int d_in, int d_out, int dt);
// several such layers (all with the same plan .nb) in one launch; ws: the sum of their ws_floats (A, G, T, d_in, d_out of
// the descriptors are used)
constexpr int kGramColsLayers = 16;
hipError_t launch_gram_cols_layers(const GramLayerDesc* layers, int n_layers, int B, bool accumulate, float* sqnorm, float* ws,
                                   hipStream_t st, int dt, const ClipOut* co = nullptr);
hipError_t launch_gram_cols(const GramColsPlan& p, const void* A, const void* G, int B, int T, int d_in, int d_out,
                            bool accumulate, float* sqnorm, float* ws, hipStream_t st, int dt, const ClipOut* co = nullptr);
hipError_t launch_gram_bf16_dma_layers(const GramLayerDesc* layers, int n_layers, int B, bool accumulate, float* sqnorm,
                                       float* partial, hipStream_t st, int fmt, float C = 0.f, float* clip = nullptr);
hipError_t launch_gram_bf16_dma(const GramPlan& p, const void* A, const void* G, int B, int T, int d_in, int d_out,
                                bool accumulate, float* sqnorm, float* partial, hipStream_t st, int fmt, const ClipOut* co = nullptr);
// float32 inputs (dp_gram_f32.hip): 64-row tiles
GramPlan plan_gram_f32(int T);
hipError_t launch_gram_f32(const GramPlan& p, const float* A, const float* G, int B, int T, int d_in, int d_out,
                           bool accumulate, float* sqnorm, float* partial, hipStream_t st, const ClipOut* co = nullptr);
hipError_t launch_gram_bf16(const GramPlan& p, const uint16_t* A, const uint16_t* G, int B, int T, int d_in, int d_out,
                            bool accumulate, float* sqnorm, float* partial, hipStream_t st, bool f16, const ClipOut* co = nullptr);

}  // namespace dpk
