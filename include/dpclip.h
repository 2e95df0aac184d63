/*
 * dpclip -- per-example gradient norms, clip factors and clipped gradient sums
 * for differentially private training, on one AMD MI355X (gfx950).
 *
 * The calls follow the problem statement of Lee & Kifer, "Scaling up
 * Differentially Private Deep Learning with Fast Per-Example Gradient
 * Clipping": for every layer only its mini-batch inputs X^(l) and the
 * gradients with respect to its pre-activations dLoss/dZ^(l) are needed
 * (Section 5, last paragraph before 5.1).  Here
 *     A[B, T, d_in]   layer inputs   (T = 1 dense; sequence length for a
 *                     recurrent / attention projection; number of output
 *                     positions for an unfolded convolution, Algorithm 3)
 *     G[B, T, d_out]  per-example pre-activation gradients, position-major
 * and example i's weight gradient is g_i = A_i^T G_i (Eq. grad_linear_layer,
 * Eq. recurrent_gradient, Algorithm 3, Section 5.6), which is never written
 * to memory by this library.
 *
 * Conventions for every entry point
 *  - All data pointers are DEVICE pointers owned by the caller, contiguous,
 *    row-major and 16-byte aligned.  The library never allocates, frees or
 *    synchronises.  Scratch space is passed in as `workspace`.
 *  - Every call is asynchronous on `hip_stream` (a hipStream_t passed as
 *    void*; NULL is the default stream).  Results are valid once the caller
 *    has synchronised that stream.
 *  - Errors come back as dp_status; on any error nothing is launched and the
 *    outputs are untouched.  Negative sizes, NULL required pointers, C <= 0,
 *    stddev < 0 or unknown enum values give DP_ERR_INVALID_ARG.  B*T must be
 *    below 2^31 and d_in, d_out below 2^24, else DP_ERR_UNSUPPORTED.
 *  - A zero B, T, d_in or d_out is a valid empty problem: DP_OK, and with
 *    accumulate == 0 the output is zero-filled.
 *  - NaN / Inf inputs are not detected; they propagate into the outputs.
 *  - Results are bit-reproducible for fixed inputs, sizes and build: all
 *    reductions run in a fixed order and no floating-point atomics are used.
 *  - bf16 inputs are the upper 16 bits of an IEEE float32, fp16 inputs are
 *    IEEE binary16; both run through the same kernels (the matrix
 *    instruction for the format is the only difference) and multiply exactly
 *    into float32.  All accumulation and all outputs are float32.  fp16
 *    subnormals (values below 6.1e-5) take part with their exact value.
 *    The 8-bit types are described at dp_dtype below.
 */
#ifndef DPCLIP_H
#define DPCLIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DP_OK = 0,
    DP_ERR_INVALID_ARG = 1,
    DP_ERR_UNSUPPORTED = 2,
    DP_ERR_WORKSPACE = 3,   /* workspace NULL or smaller than dp_workspace_bytes() */
    DP_ERR_HIP = 4          /* a kernel launch failed; hipGetLastError() has the cause */
} dp_status;

/* DP_F16 widens the library beyond what the paper ran (it used float32); it
 * is accepted wherever DP_BF16 is.
 * The 8-bit types (one byte per element, the OCP 8-bit floating-point formats:
 * e4m3 with bias 7, no infinities and the single NaN code S.1111.111; e5m2 with
 * bias 15 and IEEE-style infinities and NaNs; subnormals in both) run on the
 * 64-deep 8-bit matrix instruction, at twice the 16-bit rate:
 *   DP_F8_E4M3       A and G e4m3
 *   DP_F8_E5M2       A and G e5m2
 *   DP_F8_E4M3_E5M2  A e4m3 (activations), G e5m2 (backpropagated gradients)
 * Products of 8-bit values are exact in fp32, so the results differ from exact
 * arithmetic on the stored values only by the fp32 summation.
 * dp_layer_sqnorm, dp_clipped_grad(_noise) and the several-layers calls take
 * them for every shape.  The 8-bit kernels run: GRAM for T > 64 with d_in and
 * d_out multiples of 128; DIRECT and the clipped sum for d_in and d_out multiples
 * of 16 that tile into 256 x 256 or 128 x 128 blocks with at most a quarter of
 * padding and T >= 64 a multiple of 64 (or at most a quarter of padding up to the
 * next one); under DP_PATH_AUTO a layer goes to the other path where only that
 * one's kernel fits.  Every other shape (dense layers, other widths, short T) is
 * widened to fp16 -- which holds both formats exactly -- at the head of the
 * workspace and runs through the fp16 kernels: same result as the DP_F16 call on
 * the widened values, 2 bytes per input element more workspace (the size queries
 * include it).  dp_bias_sqnorm and dp_layernorm_sqnorm read 8-bit G (and
 * Hbar, stored like A) directly; bias_rows of dp_layers_sqnorm are then taken
 * in a pass of their own.  The convolution-from-image calls widen X and G to
 * fp16 in their workspace. */
typedef enum { DP_F32 = 0, DP_BF16 = 1, DP_F16 = 2, DP_F8_E4M3 = 3, DP_F8_E5M2 = 4, DP_F8_E4M3_E5M2 = 5 } dp_dtype;

/* How dp_layer_sqnorm evaluates ||A_i^T G_i||_F^2 when T > 1.
 *   DIRECT: a tile of g_i = sum_t outer(A_i[t], G_i[t]) is accumulated in
 *           registers, squared and reduced (Algorithm 3 / Algorithm 4 without
 *           storing their output).           2*T*d_in*d_out flops per example.
 *   GRAM:   sum_{t,s} (A_i A_i^T)_{ts} (G_i G_i^T)_{ts}, an identity of the
 *           Frobenius norm; T x T tiles stay on chip and only t <= s tiles are
 *           formed.                          T*(T+1)*(d_in+d_out) flops.
 *   AUTO:   GRAM iff its flop count is strictly smaller (dp_choose_path). */
typedef enum { DP_PATH_AUTO = 0, DP_PATH_GRAM = 1, DP_PATH_DIRECT = 2 } dp_path;

typedef enum { DP_OP_SQNORM = 0, DP_OP_CLIPPED_GRAD = 1 } dp_op;

/* Squared per-example gradient norms of one layer (Section 4 for T = 1;
 * Sections 5.2-5.6 otherwise):
 *     sqnorm[i]  =  (accumulate ? sqnorm[i] : 0) + ||A_i^T G_i||_F^2,  i in [0, B).
 * T == 1 always uses the closed form ||A_i||^2 ||G_i||^2 and ignores `path`.
 * Summing over the layers of a model (accumulate = 0 for the first layer, 1
 * for the rest) gives the squared norm of the whole parameter gradient
 * (Section 5, paragraph before 5.1; weights only).
 *   A, G       device, [B,T,d_in] and [B,T,d_out] of `dtype`, read only
 *   sqnorm     device, float32[B], written (read first if accumulate)
 *   workspace  device scratch of at least dp_workspace_bytes(DP_OP_SQNORM, ...)
 *              bytes; may be NULL when that size is 0 (T == 1)
 * Both paths exist for every input type. */
dp_status dp_layer_sqnorm(const void* A, const void* G,
                          int64_t B, int64_t T, int64_t d_in, int64_t d_out,
                          dp_dtype dtype, dp_path path, int accumulate,
                          float* sqnorm, void* workspace, size_t workspace_bytes,
                          void* hip_stream);

/* dp_layer_sqnorm for callers that cannot allocate or hand over device
 * memory of their own for scratch: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results
 * (bit for bit) as dp_layer_sqnorm, without `workspace`: the partial sums go
 * to a fixed array of DP_STATIC_SCRATCH_BYTES bytes inside the library's device
 * image (one copy per GPU, held until the process ends).  The call allocates
 * nothing and frees nothing; on the first call on a device it looks up that
 * device's copy of the array (no allocation either; make that first call outside
 * a graph capture).  A problem whose dp_workspace_bytes(DP_OP_SQNORM, ...)
 * exceeds DP_STATIC_SCRATCH_BYTES gives DP_ERR_WORKSPACE and launches nothing.
 * Every call on a GPU uses the same array: calls that may overlap on one GPU
 * (different streams, or a captured graph replayed next to an eager call) race
 * and must be ordered by the caller.  Nothing in the array has to start at
 * zero: every partial sum is written before it is read. */
#define DP_STATIC_SCRATCH_BYTES (4u << 20)
dp_status dp_layer_sqnorm_static(const void* A, const void* G,
                                 int64_t B, int64_t T, int64_t d_in, int64_t d_out,
                                 dp_dtype dtype, dp_path path, int accumulate,
                                 float* sqnorm, void* hip_stream);

/* The same for several layers of one model in one call (the whole-model norm
 * is the sum over the layers; Section 5, paragraph before 5.1):
 *     sqnorm[i] = (accumulate ? sqnorm[i] : 0) + sum_l ||A_l,i^T G_l,i||_F^2.
 * Layers on the Gram path whose widths are multiples of 64 (16-bit inputs;
 * multiples of 128 for 8-bit inputs) with T > 64 share kernel launches, up to 16 layers each: the workgroups of one
 * layer then fill the idle tail of another's, which a per-layer launch leaves
 * empty.  Dense layers (T == 1) share launches too, 16 each, and so do 16-bit
 * Gram layers of at most 64 positions with wide rows in a batch of fewer than
 * 512 (their columns are split over workgroups), and 16-bit layers on the
 * direct path with T >= 64 and widths that are multiples of 8, unless they
 * are large enough to do better alone.  Every other layer runs the
 * kernels dp_layer_sqnorm runs for it; where there are two or more of them,
 * their per-tile partial sums are added by one launch at the end instead of
 * one per layer.  The result equals per-layer calls up to the order of the
 * float32 additions (column-split Gram layers first, dense layers, then the
 * other layers, then the shared Gram launches, widest layer first).
 *   layers     HOST array of n_layers descriptors, read during the call only;
 *              A and G are device pointers as in dp_layer_sqnorm; all layers
 *              share B, dtype and path
 *   workspace  device scratch of at least dp_layers_workspace_bytes(...) bytes
 * n_layers == 0 (or only empty layers) zero-fills sqnorm unless accumulating.
 * A layer with bias_rows set also gets its bias term (Section 5.1, the bias
 * gradient; summed over the positions that share the bias as in Eq.
 * recurrent_gradient): bias_rows[i, :] = sum_t G_i[t, :] and ||bias_rows[i]||^2
 * joins sqnorm[i].  For the layers that share Gram launches the sums are taken by
 * the Gram kernel while G is on chip (no second pass over G); for the others
 * dp_bias_sqnorm is run.  dp_clipped_bias_grad then folds the rows. */
typedef struct {
    const void* A;              /* device, [B, T, d_in] */
    const void* G;              /* device, [B, T, d_out] */
    int64_t T, d_in, d_out;
    float* grad;                /* device, float32[d_in, d_out]: dp_layers_clipped_grad(_noise) only */
    uint64_t noise_offset;      /* position of grad[0] in the noise stream: dp_layers_clipped_grad_noise only */
    float* bias_rows;           /* NULL, or device float32[B, d_out]: dp_layers_sqnorm(_clip) also writes the layer's
                                   per-example bias gradients sum_t G_i[t, :] there and adds their squared norms (what
                                   dp_bias_sqnorm does), for layers that have a bias */
    /* Per-layer and grouped clipping (a threshold per layer, e.g. c / sqrt(m) for m layers, or per group of layers;
     * Section 4).  A layer that names an array of its own is added to that array instead of the call's sqnorm:
     * layers naming the same array form a group.  All NULL / 0: the layer belongs to the call's own array. */
    float* sqnorm;              /* NULL, or device float32[B]: dp_layers_sqnorm(_clip) adds this layer's squared norm
                                   (bias share included) here; `accumulate` applies to these arrays too */
    float* clip;                /* NULL, or device float32[B].  dp_layers_sqnorm_clip (with `sqnorm` set): receives
                                   min(1, clip_C / sqrt(.)) of the finished array; every layer of a group names the same
                                   clip and clip_C.  dp_layers_clipped_grad(_noise): the clip factors for this layer,
                                   in place of the call's */
    float clip_C;               /* threshold of this layer's group; > 0 when clip is set */
    float* grad_b;              /* NULL, or device float32[d_out]: dp_layers_clipped_grad(_noise) also writes the clipped
                                   sum of the layer's bias gradients, sum_i clip[i] bias_rows[i, :] (what
                                   dp_clipped_bias_grad does; bias_rows as dp_layers_sqnorm left them) */
    uint64_t bias_noise_offset; /* position of grad_b[0] in the noise stream: dp_layers_clipped_grad_noise only.  The
                                   stretches [noise_offset, + d_in*d_out) and [bias_noise_offset, + d_out) of all layers
                                   must be pairwise disjoint, or gradients share draws and the noise is no longer the
                                   independent N(0, sigma^2) per coordinate of the Gaussian mechanism (not checked here) */
} dp_layer_desc;

dp_status dp_layers_sqnorm(const dp_layer_desc* layers, int64_t n_layers, int64_t B,
                           dp_dtype dtype, dp_path path, int accumulate,
                           float* sqnorm, void* workspace, size_t workspace_bytes,
                           void* hip_stream);

size_t dp_layers_workspace_bytes(const dp_layer_desc* layers, int64_t n_layers, int64_t B,
                                 dp_dtype dtype, dp_path path);

/* dp_layers_sqnorm followed by dp_clip_factors(sqnorm, B, C, clip) (Algorithm 1,
 * the line defining nu_i), for the case that the layers given are the whole
 * model: the launch that completes the norms writes the clip factors too where it
 * can, else a clip-factor launch follows; the values are the same either way.
 * clip == NULL: exactly dp_layers_sqnorm.  C must be > 0 when clip is given.
 * Layers that name arrays of their own (dp_layer_desc.sqnorm / clip / clip_C) are
 * added to those instead, group by group, in the same launches; sqnorm and clip
 * of the call may then be NULL if no layer is left for them. */
dp_status dp_layers_sqnorm_clip(const dp_layer_desc* layers, int64_t n_layers, int64_t B,
                                dp_dtype dtype, dp_path path, int accumulate,
                                float* sqnorm, float C, float* clip,
                                void* workspace, size_t workspace_bytes, void* hip_stream);

/* dp_clipped_grad for several layers in one call, in the order given:
 *     layers[l].grad = (accumulate ? layers[l].grad : 0) + sum_i clip[i] * A_l,i^T G_l,i.
 * Same kernels as one dp_clipped_grad call per layer.  It saves the caller's
 * per-call cost, which is what bounds models made of many small layers, and
 * it lets layers share launches: float32 layers with a short contraction
 * (B*T <= 512), eight per launch, and 16-bit / 8-bit layers that run on 256 x
 * 256 tiles with T a multiple of the 32- / 64-row stage (groups of 2 to 16):
 * one launch whose work items fill the chip a whole number of times, where a
 * launch per layer has to fill it exactly once.  The other 16-bit layers whose
 * widths are multiples of 8 and at least 64, with T a multiple of 32 (the
 * unfolded convolutions of an image model: 576 -> 64, 1152 -> 128, ...), form
 * groups of their own (2 to 16 layers) on 128 x 128 tiles.  Results: bit for bit the
 * per-layer calls, except for those groups, whose contraction is cut into other K slices: the
 * float32 partial sums are then grouped differently (differences at the level
 * of float32 rounding; still bit-reproducible from call to call).  The groups
 * apply the clip factors to float32 sums, also for the shapes where the layer's
 * own kernel multiplies them into 16-bit inputs (dp_clipped_grad_rounds_inputs):
 * there the two differ by that rounding.
 *   workspace  device scratch of at least dp_layers_clipped_workspace_bytes(...)
 *              bytes (the largest single layer's need, or a group's slices).
 * A third kind of group takes such 16-bit layers whose T is at least 16 and not
 * a multiple of 32 (4 x 4 or 7 x 7 positions); float32 layers with at least 256
 * rows B*T and widths that are multiples of 4 form groups of their own. */
dp_status dp_layers_clipped_grad(const dp_layer_desc* layers, int64_t n_layers, int64_t B,
                                 const float* clip, dp_dtype dtype, int accumulate,
                                 void* workspace, size_t workspace_bytes, void* hip_stream);

size_t dp_layers_clipped_workspace_bytes(const dp_layer_desc* layers, int64_t n_layers, int64_t B,
                                         dp_dtype dtype);

/* dp_layers_clipped_grad followed by the Gaussian mechanism's noise (Algorithm 1,
 * the line that adds N(0, sigma^2 C^2 I)) on every layer's result:
 *     layers[l].grad[j] += stddev * z[layers[l].noise_offset + j],
 * z = the stream of dp_add_noise for `seed`.  Bit-identical to
 * dp_layers_clipped_grad followed by dp_add_noise(grad, d_in*d_out, stddev, seed,
 * noise_offset) per layer (for the groups that share a launch: to the same call without
 * noise followed by dp_add_noise); where a layer's clipped sum ends in the kernel that
 * folds its K slices (and d_in*d_out and noise_offset are multiples of 4), that
 * kernel adds the noise while it holds the sums, which saves the extra pass over
 * the gradient.  With the layers' noise_offset set to the positions of their
 * gradients in the model's flat parameter vector, the noise is the same as one
 * dp_add_noise call over that vector.  stddev == 0 adds nothing. */
dp_status dp_layers_clipped_grad_noise(const dp_layer_desc* layers, int64_t n_layers, int64_t B,
                                       const float* clip, dp_dtype dtype, int accumulate,
                                       float stddev, uint64_t seed,
                                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* One private step over a model's layers in a single call (the body of Algorithm 1's
 * loop after the backward pass: per-example norms, the factors nu_i, the clipped
 * sum, the noise):  dp_layers_sqnorm_clip(layers, ..., accumulate = 0, sqnorm, C,
 * clip, ...) followed by dp_layers_clipped_grad_noise(layers, ..., clip,
 * accumulate = 0, stddev, seed, ...) on the same stream, with the same launches and
 * bit-identical results; what it saves is one crossing of the boundary per step,
 * which is what bounds models of a few small layers.
 *   sqnorm, clip  device float32[B], written.
 *   workspace     device scratch of at least the larger of
 *                 dp_layers_workspace_bytes(...) and
 *                 dp_layers_clipped_workspace_bytes(...) bytes; the two stages use
 *                 it one after the other.
 * Errors: the arguments of the norm stage are checked before anything is launched;
 * if the clipped-sum stage then rejects its own (a layer without grad, a workspace
 * too small for it), sqnorm and clip have already been written. */
dp_status dp_layers_step(const dp_layer_desc* layers, int64_t n_layers, int64_t B,
                         dp_dtype dtype, dp_path path, float C, float* sqnorm, float* clip,
                         float stddev, uint64_t seed,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/* Clip factors (Algorithm 1, the line defining nu_i; Eq. per_example_weight;
 * clip function of Section 3.2):
 *     clip[i] = 1 / max(1, sqrt(sqnorm[i]) / C)  =  min(1, C / ||g_i||),
 * so a zero norm and a norm equal to C both give exactly 1.
 *   sqnorm  device float32[B], read only;  clip  device float32[B], written
 *   (clip may alias sqnorm).  C must be > 0. */
dp_status dp_clip_factors(const float* sqnorm, int64_t B, float C,
                          float* clip, void* hip_stream);

/* Clipped batch gradient of one layer (gradient of the re-weighted loss,
 * Eq. weighted_loss, without the 1/tau factor):
 *     grad  =  (accumulate ? grad : 0) + sum_i clip[i] * A_i^T G_i
 * as one GEMM over K = B*T rows with clip[i] folded into the rows of A.
 *   grad       device float32[d_in, d_out] row-major
 *   clip       device float32[B]
 *   workspace  device scratch of at least
 *              dp_workspace_bytes(DP_OP_CLIPPED_GRAD, ...) bytes
 * With 16-bit inputs the factor is applied either to the fp32 accumulators
 * (one fp32 rounding per example) or, in the kernels for unaligned shapes, to
 * the rows of A, which are then rounded back to the input format (relative
 * error at most 2^-8 per element for bf16, 2^-11 for fp16, unbiased).
 * clip[i] == 0 leaves example i out (finite inputs): masked examples, and the
 * factor that dp_clip_factors gives a norm that overflowed, are safe.  The
 * kernels that scale accumulators keep their running sum in units of the
 * current example's factor, which must stay in the float32 range: a factor
 * below 2^-40 (about 1e-12) of the largest earlier factor of the same K slice
 * (up to 64 consecutive examples) counts as 0 there.  Such a term is below the
 * float32 resolution of a sum in which the larger one takes part. */
dp_status dp_clipped_grad(const void* A, const void* G, const float* clip,
                          int64_t B, int64_t T, int64_t d_in, int64_t d_out,
                          dp_dtype dtype, int accumulate, float* grad,
                          void* workspace, size_t workspace_bytes,
                          void* hip_stream);

/* Bias parameters.  The per-example gradient of a layer's bias vector is
 * dL/dz itself for a fully-connected layer (Section 5.1) and its sum over the
 * T positions that share the bias otherwise (Section 5.3; the output positions
 * of a convolution likewise):
 *     bias_rows[i, :] = sum_t G_i[t, :]
 *     sqnorm[i]       = (accumulate ? sqnorm[i] : 0) + ||bias_rows[i, :]||^2
 * (the norm of the whole parameter gradient runs over weights and biases,
 * Section 5, paragraph before 5.1: call this with accumulate = 1 on the array
 * that dp_layer_sqnorm fills).
 *   G          device, [B,T,d_out] of `dtype`, read only
 *   bias_rows  device, float32[B, d_out], written; keep it for dp_clipped_bias_grad
 *   sqnorm     device, float32[B]
 * No workspace. */
dp_status dp_bias_sqnorm(const void* G, int64_t B, int64_t T, int64_t d_out,
                         dp_dtype dtype, int accumulate, float* sqnorm,
                         float* bias_rows, void* hip_stream);

/* LayerNorm scale and shift (Section 5.5, Algorithm 5): with G = dL/dh, the
 * gradient with respect to the layer's output, and Hbar the normalised input,
 * both [B, T, d] of `dtype`,
 *     gamma_rows[i, :] = sum_t G_i[t, :] * Hbar_i[t, :]   (elementwise product)
 *     beta_rows[i, :]  = sum_t G_i[t, :]
 *     sqnorm[i] = (accumulate ? sqnorm[i] : 0) + ||gamma_rows[i]||^2 + ||beta_rows[i]||^2
 * gamma_rows, beta_rows: device float32[B, d], written; their clipped sums
 * are two calls of dp_clipped_bias_grad.  No workspace.
 * With the 8-bit pair type DP_F8_E4M3_E5M2, G is e5m2 and Hbar e4m3. */
dp_status dp_layernorm_sqnorm(const void* G, const void* Hbar, int64_t B, int64_t T, int64_t d,
                              dp_dtype dtype, int accumulate, float* sqnorm,
                              float* gamma_rows, float* beta_rows, void* hip_stream);

/* Clipped batch gradient of the bias (Eq. weighted_loss applied to b; the same
 * call serves any per-example gradient rows [B, d_out], e.g. LayerNorm's):
 *     grad_b[q] = (accumulate ? grad_b[q] : 0) + sum_i clip[i] * bias_rows[i, q]
 *   bias_rows  device float32[B, d_out] from dp_bias_sqnorm, read only
 *   clip       device float32[B];  grad_b  device float32[d_out] */
dp_status dp_clipped_bias_grad(const float* bias_rows, const float* clip,
                               int64_t B, int64_t d_out, int accumulate,
                               float* grad_b, void* hip_stream);

/* Convolution layers given by their input image instead of the unfolded patch
 * matrix (Section 5.2; Algorithm 3 unfolds the image first, here the patches
 * are formed on the fly, so the kh*kw-fold larger matrix never exists in
 * memory).  Stride 1, zero padding `pad` on every side:
 *   X  device, [B, H, W, C] of bf16, fp16 or an 8-bit type, channels last
 *   G  device, [B, T, d_out] of the same type, T = H_out * W_out output positions in
 *      row-major (y, x) order, H_out = H + 2 pad - KH + 1, W_out likewise
 * The layer's weight gradient is [d_in, d_out] with d_in = KH*KW*C and row
 * index (kh*KW + kw)*C + c:  g_i[(kh,kw,c), o] = sum_{y,x} Xpad_i[y+kh, x+kw, c] * G_i[y*W_out + x, o].
 * dp_conv_sqnorm and dp_conv_clipped_grad compute exactly what
 * dp_layer_sqnorm (direct path) and dp_clipped_grad compute on the unfolded
 * A[B, T, d_in]; arguments not listed here mean the same as there.
 * Types: DP_BF16, DP_F16 and the 8-bit types (widened to fp16); d_out % 8 == 0.
 * Two families of geometries are taken, anything else is DP_ERR_UNSUPPORTED
 * (unfold and use the general entry points):
 * (1) C % 8 == 0, T >= 64 with at most a quarter of padding up to the next
 *     multiple of 32 (e.g. 784, 196, 1024), and a [d_in, d_out] that tiles into
 *     256 x 256, 192 x 128 or 128 x 128 blocks with at most a quarter of
 *     padding: the general kernels with the patches formed by their copies;
 * (2) 3 x 3 kernels with C a multiple of 64, a padded image row of at most
 *     about 100 pixels and T of at least three quarters of the next multiple
 *     of 32: a kernel of its own that keeps the padded image rows in LDS and
 *     fetches every pixel once instead of once per tap.  It is used for
 *     T >= 512 and wherever (1) does not apply (d_out or 9 C that do not tile,
 *     T < 64); dp_conv_rows_resident tells.  Its results are those of the
 *     general entry points up to the order of the float32 sums.
 * workspace: at least dp_conv_workspace_bytes(...). */
dp_status dp_conv_sqnorm(const void* X, const void* G,
                         int64_t B, int64_t H, int64_t W, int64_t C,
                         int64_t KH, int64_t KW, int64_t pad, int64_t d_out,
                         dp_dtype dtype, int accumulate, float* sqnorm,
                         void* workspace, size_t workspace_bytes, void* hip_stream);
dp_status dp_conv_clipped_grad(const void* X, const void* G, const float* clip,
                               int64_t B, int64_t H, int64_t W, int64_t C,
                               int64_t KH, int64_t KW, int64_t pad, int64_t d_out,
                               dp_dtype dtype, int accumulate, float* grad,
                               void* workspace, size_t workspace_bytes, void* hip_stream);
/* Scratch bytes for the two calls above (op as in dp_workspace_bytes); 0 for
 * invalid or unsupported arguments. */
size_t dp_conv_workspace_bytes(dp_op op, int64_t B, int64_t H, int64_t W, int64_t C,
                               int64_t KH, int64_t KW, int64_t pad, int64_t d_out, dp_dtype dtype);
/* Test hook: 1 when the two calls above run this geometry on the kernel that
 * keeps the image rows in LDS (then they equal the general entry points on the
 * unfolded matrix up to float32 summation order), 0 when they run the general
 * kernels with implicit unfolding (then bit for bit), -1 for invalid or
 * unsupported arguments. */
int dp_conv_rows_resident(int64_t B, int64_t H, int64_t W, int64_t C,
                          int64_t KH, int64_t KW, int64_t pad, int64_t d_out, dp_dtype dtype);

/* Gaussian mechanism (Section 2, Gaussian-mechanism lemma; Algorithm 1, the
 * update line): grad[j] += stddev * z[offset + j], j in [0, n), with z an
 * i.i.d. N(0,1) stream that is a pure function of (seed, element index):
 *   element e uses Philox4x32-10 with key = (lo32(seed), hi32(seed)) and
 *   counter = (lo32(e>>2), hi32(e>>2), 0, 0); output words (w0,w1) feed slots
 *   e&3 = 0,1 and (w2,w3) feed slots 2,3 through Box-Muller with
 *   u = ((w >> 9) + 0.5) * 2^-23:  r = sqrt(-2 ln u_a),
 *   z_even = r cos(2 pi u_b), z_odd = r sin(2 pi u_b).
 * Layers of one model use disjoint ranges: offset_l = sum of earlier n.
 * Resuming a run needs only (seed, offset).  stddev is absolute (sigma, not a
 * multiple of C). */
dp_status dp_add_noise(float* grad, int64_t n, float stddev,
                       uint64_t seed, uint64_t offset, void* hip_stream);

/* Scratch bytes needed by dp_layer_sqnorm (op = DP_OP_SQNORM, for the path
 * that `path` resolves to) or dp_clipped_grad (op = DP_OP_CLIPPED_GRAD; `path`
 * ignored).  Returns 0 for invalid arguments. */
size_t dp_workspace_bytes(dp_op op, int64_t B, int64_t T, int64_t d_in, int64_t d_out,
                          dp_dtype dtype, dp_path path);

/* The AUTO rule: DP_PATH_GRAM iff T*(T+1)*(d_in+d_out) < 2*T*d_in*d_out,
 * else DP_PATH_DIRECT (a tie goes to DIRECT). */
dp_path dp_choose_path(int64_t T, int64_t d_in, int64_t d_out);

/* Test hook: how dp_clipped_grad applies the clip factors for this shape and
 * type.  0: in float32 (to the accumulators or to a per-example tile; the
 * result differs from exact arithmetic on the stored inputs only by float32
 * rounding).  1: to the rows of A, which are rounded back to the 16-bit input
 * format (relative error at most 2^-8 per element for bf16, 2^-11 for fp16).  -1 for
 * invalid arguments.  Lets a test hold each kernel to the accuracy it should
 * reach instead of the loosest bound. */
int dp_clipped_grad_rounds_inputs(int64_t B, int64_t T, int64_t d_in, int64_t d_out, dp_dtype dtype);

/* Static, never-NULL description of a status code. */
const char* dp_status_string(dp_status status);

/* Test hook: raw Philox words.  out[4*q + r] = word r of the block with
 * counter first_counter + q, q in [0, n_counters).  out is a device pointer. */
dp_status dp_philox_raw(uint32_t* out, int64_t n_counters, uint64_t seed,
                        uint64_t first_counter, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DPCLIP_H */
