// C-ABI entry points declared in include/dpclip.h: argument checks, path
// choice, workspace carving and kernel launches.  No device allocation, no
// synchronisation, no host reads of device memory.
#include "../../include/dpclip.h"
#include "dp_internal.h"
#include <algorithm>
#include <mutex>
#include <vector>

using namespace dpk;

// Scratch of dp_layer_sqnorm_static: lives in the device image, one copy per GPU.  In host code this name is only a
// handle for hipGetSymbolAddress; kernels and launchers get the address that call returns.
static __device__ __align__(256) unsigned char scratch[DP_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};              // device address of `scratch` on each GPU, looked up once

// the current device's copy of `scratch`
dp_status static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return DP_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return DP_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return DP_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return DP_OK;
}

constexpr int64_t kMaxRows = (int64_t(1) << 31) - 1;   // B*T
constexpr int64_t kMaxDim = int64_t(1) << 24;          // d_in, d_out

bool is16(dp_dtype d) { return d == DP_BF16 || d == DP_F16; }
bool is8(dp_dtype d) { return d == DP_F8_E4M3 || d == DP_F8_E5M2 || d == DP_F8_E4M3_E5M2; }
bool valid_dtype(dp_dtype d) { return d == DP_F32 || is16(d) || is8(d); }
// format code of the copy-pipeline launchers (16-bit and 8-bit types)
int fmt_of(dp_dtype d) { return d == DP_BF16 ? 0 : d == DP_F16 ? 1 : d == DP_F8_E4M3 ? 2 : d == DP_F8_E5M2 ? 3 : 4; }
bool valid_path(dp_path p) { return p == DP_PATH_AUTO || p == DP_PATH_GRAM || p == DP_PATH_DIRECT; }

dp_status check_dims(int64_t B, int64_t T, int64_t d_in, int64_t d_out) {
    if (B < 0 || T < 0 || d_in < 0 || d_out < 0) return DP_ERR_INVALID_ARG;
    if (d_in >= kMaxDim || d_out >= kMaxDim) return DP_ERR_UNSUPPORTED;
    if (B > kMaxRows || T > kMaxRows) return DP_ERR_UNSUPPORTED;
    if (B > 0 && T > 0 && B > kMaxRows / T) return DP_ERR_UNSUPPORTED;
    return DP_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// 8-bit types: the shapes that a path's kernels take (T > 1)
bool f8_path_ok(dp_path p, dp_dtype dtype, int64_t T, int64_t d_in, int64_t d_out) {
    if (T <= 1) return false;
    if (p == DP_PATH_GRAM) return gram_dma_ok((int)T, (int)d_in, (int)d_out, fmt_of(dtype));
    return dma8_direct_ok((int)T, (int)d_in, (int)d_out);
}

dp_path resolve_path(dp_path path, dp_dtype dtype, int64_t T, int64_t d_in, int64_t d_out) {
    if (path != DP_PATH_AUTO) return path;
    const dp_path p = dp_choose_path(T, d_in, d_out);
    if (is8(dtype) && !f8_path_ok(p, dtype, T, d_in, d_out)) {
        // both paths give the same number: take the other one where only its kernels fit the shape
        const dp_path other = p == DP_PATH_GRAM ? DP_PATH_DIRECT : DP_PATH_GRAM;
        if (f8_path_ok(other, dtype, T, d_in, d_out)) return other;
    }
    return p;
}

// 8-bit inputs outside the shapes of their own kernels are widened to fp16 (exact for both formats) at the head of
// the workspace and run through the fp16 kernels
size_t widen_bytes(int64_t n) { return (size_t)((n * 2 + 255) & ~int64_t(255)); }
bool f8_fast_sqnorm(dp_dtype dtype, dp_path path, int64_t T, int64_t d_in, int64_t d_out) {
    return T > 1 && f8_path_ok(resolve_path(path, dtype, T, d_in, d_out), dtype, T, d_in, d_out);
}
bool a_is_e5m2(dp_dtype d) { return d == DP_F8_E5M2; }
bool g_is_e5m2(dp_dtype d) { return d != DP_F8_E4M3; }

// bytes of scratch for the squared-norm call on an already resolved path (T > 1)
size_t sqnorm_ws_bytes(int64_t B, int64_t T, int64_t d_in, int64_t d_out, dp_dtype dtype, dp_path path) {
    if (is8(dtype) && !f8_path_ok(path, dtype, T, d_in, d_out)) return 0;
    if (path == DP_PATH_GRAM) {
        if (!is8(dtype)) {
            const GramColsPlan c = plan_gram_cols((int)B, (int)T, (int)d_in, (int)d_out, (int)dtype);
            if (c.use) return c.ws_floats * sizeof(float);
        }
        GramPlan g = (is16(dtype) || is8(dtype)) ? plan_gram_bf16((int)T, (int)d_in, (int)d_out) : plan_gram_f32((int)T);
        return (size_t)B * g.npairs * sizeof(float);
    }
    TnPlan p = is8(dtype)  ? plan_direct_f8_dma((int)B, (int)T, (int)d_in, (int)d_out)
             : is16(dtype) ? plan_direct_bf16((int)B, (int)T, (int)d_in, (int)d_out)
                           : plan_direct_f32((int)B, (int)T, (int)d_in, (int)d_out);
    if (!is8(dtype) && !p.dma && p.splits > 1)         // chunks of positions: their shares of A_i^T G_i, then the blocks' sums
        return ((size_t)B * p.splits * (size_t)splitk_slice_elems(d_in * d_out) + (size_t)B * (size_t)((d_in * d_out + 1023) / 1024)) * sizeof(float);
    return (size_t)B * p.tiles_m * p.tiles_n * sizeof(float) + (p.zero_head ? kZeroHeadFloats * sizeof(float) : 0);
}

size_t clipped_ws_bytes(int64_t B, int64_t T, int64_t d_in, int64_t d_out, dp_dtype dtype) {
    if (is8(dtype) && !dma8_clipped_ok((int)T, (int)d_in, (int)d_out)) return 0;
    TnPlan p = is8(dtype)  ? plan_clipped_f8_dma((int)B, (int)T, (int)d_in, (int)d_out)
             : is16(dtype) ? plan_clipped_bf16((int)B, (int)T, (int)d_in, (int)d_out)
                           : plan_clipped_f32((int)B, (int)T, (int)d_in, (int)d_out);
    const size_t head = p.zero_head ? kZeroHeadFloats * sizeof(float) : 0;
    if (p.splits <= 1) return head;
    return head + (size_t)p.splits * (size_t)splitk_slice_elems(d_in * d_out) * sizeof(float);
}

// a layer that the batched Gram launch of dp_layers_sqnorm takes (everything else goes through dp_layer_sqnorm)
bool gram_batchable(int64_t T, int64_t d_in, int64_t d_out, dp_dtype dtype, dp_path path) {
    if (T <= 1 || d_in == 0 || d_out == 0 || !(is16(dtype) || is8(dtype))) return false;
    if (resolve_path(path, dtype, T, d_in, d_out) != DP_PATH_GRAM) return false;
    return gram_dma_ok((int)T, (int)d_in, (int)d_out, fmt_of(dtype));
}

// a layer that the shared column-split Gram launches of dp_layers_sqnorm take (few positions, wide rows, small batch):
// 0 = no, else the launch class (the plan's number of 32-row blocks)
int gram_cols_class(int64_t B, int64_t T, int64_t d_in, int64_t d_out, dp_dtype dtype, dp_path path) {
    if (is8(dtype) || T <= 1 || T > 64 || d_in == 0 || d_out == 0 || B >= (int64_t(1) << 20)) return 0;
    if (resolve_path(path, dtype, T, d_in, d_out) != DP_PATH_GRAM) return 0;
    const GramColsPlan c = plan_gram_cols((int)B, (int)T, (int)d_in, (int)d_out, (int)dtype);
    return c.use ? c.nb : 0;
}

size_t round16(size_t n) { return (n + 15) & ~size_t(15); }

// a layer whose direct norm the shared copy-pipeline launch of dp_layers_sqnorm can take (16-bit, direct path, T >= 64,
// aligned widths), and the scratch such a layer needs in the several-layers call: the larger of its own call's and
// the shared launch's (one sum per example and 128 x 128 tile)
bool direct_joinable(int64_t B, int64_t T, int64_t d_in, int64_t d_out, dp_dtype dtype, dp_path path) {
    if (is8(dtype) || T <= 1 || d_in == 0 || d_out == 0 || B >= (int64_t(1) << 20)) return false;
    if (gram_batchable(T, d_in, d_out, dtype, path) || gram_cols_class(B, T, d_in, d_out, dtype, path) != 0) return false;
    if (resolve_path(path, dtype, T, d_in, d_out) != DP_PATH_DIRECT) return false;
    if (!is16(dtype)) {
        // float32: the layers whose direct norm runs on the copy-pipeline kernel (128 x 128 tiles as well)
        if (B * T >= (int64_t(1) << 31)) return false;
        const TnPlan p = plan_direct_f32((int)B, (int)T, (int)d_in, (int)d_out);
        if (!p.dma) return false;
    } else if (!dma_direct_joint_ok((int)B, (int)T, (int)d_in, (int)d_out)) return false;
    return B * direct_joint_tiles((int)d_in, (int)d_out) < (int64_t(1) << 24);       // 16 layers' items stay below the launch's 2^28
}
size_t single_layer_need(int64_t B, const dp_layer_desc& y, dp_dtype dtype, dp_path path) {
    size_t n = dp_workspace_bytes(DP_OP_SQNORM, B, y.T, y.d_in, y.d_out, dtype, path);
    if (direct_joinable(B, y.T, y.d_in, y.d_out, dtype, path))
        n = std::max(n, (size_t)B * (size_t)direct_joint_tiles((int)y.d_in, (int)y.d_out) * sizeof(float));
    return round16(n);
}

// Which joint clipped-sum launch of dp_layers_clipped_grad(_noise) can take a layer (by shape and type): 0 none,
// 1 the 256 x 256-tile launch, 3 the 128 x 128-tile launch for aligned 16-bit layers of a few hundred columns, 4 the
// same for such layers whose T is not a multiple of the 32-row stage, 5 the float32 launch
int clipped_join_class(int64_t B, int64_t T, int64_t d_in, int64_t d_out, dp_dtype dtype) {
    if (B == 0 || T == 0 || d_in == 0 || d_out == 0) return 0;
    if (is8(dtype)) return (dma8_clipped_ok((int)T, (int)d_in, (int)d_out) && dma8_joint_ok((int)T, (int)d_in, (int)d_out)) ? 1 : 0;
    if (!is16(dtype)) {
        // float32: the layers of the copy-pipeline kernel (long contractions, widths multiples of 4) share launches too
        if (B * T >= (int64_t(1) << 31)) return 0;
        const TnPlan p = plan_clipped_f32((int)B, (int)T, (int)d_in, (int)d_out);
        return (p.dma && !clipped_f32_is_short(p)) ? 5 : 0;
    }
    if (plan_clipped_bf16((int)B, (int)T, (int)d_in, (int)d_out).dma && dma_joint_ok((int)T, (int)d_in, (int)d_out)) return 1;
    if (B * T < (int64_t(1) << 31) && dma_joint_mid_ok((int)T, (int)d_in, (int)d_out)) return 3;
    if (B * T < (int64_t(1) << 31) && dma_joint_ragged_ok((int)T, (int)d_in, (int)d_out)) return 4;
    return 0;
}
size_t joint_ws_bytes(const JointShape* sh, int n, int64_t B, dp_dtype dtype, int geo) {
    if (geo == 5) return joint_f32_workspace_floats(sh, n, (int)B) * sizeof(float);
    return (is8(dtype) ? joint8_workspace_floats(sh, n, (int)B) : joint_workspace_floats(sh, n, (int)B, geo)) * sizeof(float);
}

constexpr size_t kConvZeroBytes = 256;                // head of the conv workspace: a line of zeros for the padding

// geometry check shared by the conv entry points; fills T and d_in
dp_status conv_geometry(int64_t B, int64_t H, int64_t W, int64_t C, int64_t KH, int64_t KW, int64_t pad, int64_t d_out,
                        dp_dtype dtype, ConvGeom* g, int64_t* T, int64_t* d_in) {
    if (B < 0 || H < 0 || W < 0 || C < 0 || KH < 1 || KW < 1 || pad < 0 || d_out < 0) return DP_ERR_INVALID_ARG;
    if (!valid_dtype(dtype)) return DP_ERR_INVALID_ARG;
    if (H >= kMaxDim || W >= kMaxDim || C >= kMaxDim || KH >= 4096 || KW >= 4096 || pad >= 4096) return DP_ERR_UNSUPPORTED;
    const int64_t Hout = H + 2 * pad - KH + 1, Wout = W + 2 * pad - KW + 1;
    if (Hout < 1 || Wout < 1) return DP_ERR_INVALID_ARG;
    *T = Hout * Wout;
    *d_in = KH * KW * C;
    const dp_status st = check_dims(B, *T, *d_in, d_out);
    if (st != DP_OK) return st;
    g->H = (int)H; g->W = (int)W; g->C = (int)C; g->KH = (int)KH; g->KW = (int)KW; g->pad = (int)pad;
    return DP_OK;
}

dp_status layer_sqnorm_clip(const void* A, const void* G, int64_t B, int64_t T, int64_t d_in, int64_t d_out,
                            dp_dtype dtype, dp_path path, int accumulate, float* sqnorm,
                            void* workspace, size_t workspace_bytes, void* hip_stream, const ClipOut* co);

}  // namespace

extern "C" {

const char* dp_status_string(dp_status s) {
    switch (s) {
        case DP_OK: return "ok";
        case DP_ERR_INVALID_ARG: return "invalid argument";
        case DP_ERR_UNSUPPORTED: return "unsupported size, dtype or path";
        case DP_ERR_WORKSPACE: return "workspace missing or too small";
        case DP_ERR_HIP: return "HIP launch failed";
    }
    return "unknown status";
}

dp_path dp_choose_path(int64_t T, int64_t d_in, int64_t d_out) {
    if (T <= 0 || d_in <= 0 || d_out <= 0) return DP_PATH_DIRECT;
    // T*(T+1)*(d_in+d_out) < 2*T*d_in*d_out  <=>  (T+1)*(d_in+d_out) < 2*d_in*d_out ; values stay below 2^57
    const int64_t gram = (T + 1) * (d_in + d_out);
    const int64_t direct = 2 * d_in * d_out;
    return gram < direct ? DP_PATH_GRAM : DP_PATH_DIRECT;
}

size_t dp_workspace_bytes(dp_op op, int64_t B, int64_t T, int64_t d_in, int64_t d_out, dp_dtype dtype, dp_path path) {
    if (check_dims(B, T, d_in, d_out) != DP_OK || !valid_dtype(dtype) || !valid_path(path)) return 0;
    if (B == 0 || T == 0 || d_in == 0 || d_out == 0) return 0;
    if (is8(dtype) && (op == DP_OP_SQNORM || op == DP_OP_CLIPPED_GRAD)) {
        const bool fast = op == DP_OP_SQNORM ? f8_fast_sqnorm(dtype, path, T, d_in, d_out) : dma8_clipped_ok((int)T, (int)d_in, (int)d_out);
        if (!fast) return widen_bytes(B * T * d_in) + widen_bytes(B * T * d_out) + dp_workspace_bytes(op, B, T, d_in, d_out, DP_F16, path);
    }
    if (op == DP_OP_SQNORM) {
        if (T == 1) return 0;
        const dp_path p = resolve_path(path, dtype, T, d_in, d_out);
        return sqnorm_ws_bytes(B, T, d_in, d_out, dtype, p);
    }
    if (op == DP_OP_CLIPPED_GRAD) return clipped_ws_bytes(B, T, d_in, d_out, dtype);
    return 0;
}

int dp_clipped_grad_rounds_inputs(int64_t B, int64_t T, int64_t d_in, int64_t d_out, dp_dtype dtype) {
    if (check_dims(B, T, d_in, d_out) != DP_OK || !valid_dtype(dtype)) return -1;
    if (B == 0 || T == 0 || d_in == 0 || d_out == 0 || dtype == DP_F32) return 0;
    if (is8(dtype) && dma8_clipped_ok((int)T, (int)d_in, (int)d_out)) return 0;
    // 16-bit inputs, and 8-bit ones widened to fp16: the copy-pipeline and the example-by-example kernels scale in float32
    const TnPlan p = plan_clipped_bf16((int)B, (int)T, (int)d_in, (int)d_out);
    return (p.dma || (!p.big && p.segmented)) ? 0 : 1;
}

dp_status dp_layer_sqnorm(const void* A, const void* G, int64_t B, int64_t T, int64_t d_in, int64_t d_out,
                          dp_dtype dtype, dp_path path, int accumulate, float* sqnorm,
                          void* workspace, size_t workspace_bytes, void* hip_stream) {
    return layer_sqnorm_clip(A, G, B, T, d_in, d_out, dtype, path, accumulate, sqnorm, workspace, workspace_bytes, hip_stream, nullptr);
}

dp_status dp_layer_sqnorm_static(const void* A, const void* G, int64_t B, int64_t T, int64_t d_in, int64_t d_out,
                                 dp_dtype dtype, dp_path path, int accumulate, float* sqnorm, void* hip_stream) {
    const dp_status st = check_dims(B, T, d_in, d_out);
    if (st != DP_OK) return st;
    if (!valid_dtype(dtype) || !valid_path(path)) return DP_ERR_INVALID_ARG;
    // what dp_layer_sqnorm would ask of its workspace argument (0 for empty and dense problems)
    const size_t need = dp_workspace_bytes(DP_OP_SQNORM, B, T, d_in, d_out, dtype, path);
    if (need > (size_t)DP_STATIC_SCRATCH_BYTES) return DP_ERR_WORKSPACE;
    void* ws = nullptr;
    if (need > 0) {
        const dp_status s2 = static_scratch(&ws);
        if (s2 != DP_OK) return s2;
    }
    return layer_sqnorm_clip(A, G, B, T, d_in, d_out, dtype, path, accumulate, sqnorm, ws, need > 0 ? (size_t)DP_STATIC_SCRATCH_BYTES : 0,
                             hip_stream, nullptr);
}

}  // extern "C"

namespace {

// dp_layer_sqnorm; co != nullptr (non-empty problems only): the kernel that completes sqnorm also writes the clip factors
dp_status layer_sqnorm_clip(const void* A, const void* G, int64_t B, int64_t T, int64_t d_in, int64_t d_out,
                            dp_dtype dtype, dp_path path, int accumulate, float* sqnorm,
                            void* workspace, size_t workspace_bytes, void* hip_stream, const ClipOut* co) {
    dp_status st = check_dims(B, T, d_in, d_out);
    if (st != DP_OK) return st;
    if (!valid_dtype(dtype) || !valid_path(path)) return DP_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (B == 0) return DP_OK;
    if (!sqnorm) return DP_ERR_INVALID_ARG;
    if (T == 0 || d_in == 0 || d_out == 0) {
        if (!accumulate && launch_fill_zero(sqnorm, B, stream) != hipSuccess) return DP_ERR_HIP;
        return DP_OK;
    }
    if (!A || !G || !aligned16(A) || !aligned16(G)) return DP_ERR_INVALID_ARG;

    hipError_t e;
    if (is8(dtype) && !f8_fast_sqnorm(dtype, path, T, d_in, d_out)) {
        const size_t na = widen_bytes(B * T * d_in), ng = widen_bytes(B * T * d_out);
        const size_t inner = dp_workspace_bytes(DP_OP_SQNORM, B, T, d_in, d_out, DP_F16, path);
        if (!workspace || workspace_bytes < na + ng + inner || !aligned16(workspace)) return DP_ERR_WORKSPACE;
        unsigned char* w = static_cast<unsigned char*>(workspace);
        if (launch_widen_f8(A, reinterpret_cast<uint16_t*>(w), B * T * d_in, a_is_e5m2(dtype), stream) != hipSuccess) return DP_ERR_HIP;
        if (launch_widen_f8(G, reinterpret_cast<uint16_t*>(w + na), B * T * d_out, g_is_e5m2(dtype), stream) != hipSuccess) return DP_ERR_HIP;
        return layer_sqnorm_clip(w, w + na, B, T, d_in, d_out, DP_F16, path, accumulate, sqnorm, w + na + ng,
                                 workspace_bytes - na - ng, hip_stream, co);
    }
    if (T == 1) {
        e = launch_sqnorm_dense(A, G, (int)B, (int)d_in, (int)d_out, (int)dtype, accumulate != 0, sqnorm, stream, co);
        return e == hipSuccess ? DP_OK : DP_ERR_HIP;
    }
    const dp_path p = resolve_path(path, dtype, T, d_in, d_out);
    const size_t need = sqnorm_ws_bytes(B, T, d_in, d_out, dtype, p);
    if (need >= (size_t(1) << 33)) return DP_ERR_UNSUPPORTED;           // > 2^31 partial sums
    if (!workspace || workspace_bytes < need || !aligned16(workspace)) return DP_ERR_WORKSPACE;
    float* partial = static_cast<float*>(workspace);

    if (is8(dtype)) {
        if (p == DP_PATH_GRAM)
            e = launch_gram_bf16_dma(plan_gram_bf16((int)T, (int)d_in, (int)d_out), A, G, (int)B, (int)T, (int)d_in, (int)d_out,
                                     accumulate != 0, sqnorm, partial, stream, fmt_of(dtype), co);
        else
            e = launch_direct_f8_dma(plan_direct_f8_dma((int)B, (int)T, (int)d_in, (int)d_out), A, G, (int)B, (int)T, (int)d_in,
                                     (int)d_out, accumulate != 0, sqnorm, partial, stream, fmt_of(dtype), co);
    } else if (p == DP_PATH_GRAM && plan_gram_cols((int)B, (int)T, (int)d_in, (int)d_out, (int)dtype).use) {
        e = launch_gram_cols(plan_gram_cols((int)B, (int)T, (int)d_in, (int)d_out, (int)dtype), A, G, (int)B, (int)T, (int)d_in,
                             (int)d_out, accumulate != 0, sqnorm, partial, stream, (int)dtype, co);
    } else if (p == DP_PATH_GRAM && !is16(dtype)) {
        e = launch_gram_f32(plan_gram_f32((int)T), static_cast<const float*>(A), static_cast<const float*>(G), (int)B, (int)T,
                            (int)d_in, (int)d_out, accumulate != 0, sqnorm, partial, stream, co);
    } else if (p == DP_PATH_GRAM) {
        GramPlan g = plan_gram_bf16((int)T, (int)d_in, (int)d_out);
        e = launch_gram_bf16(g, static_cast<const uint16_t*>(A), static_cast<const uint16_t*>(G), (int)B, (int)T,
                             (int)d_in, (int)d_out, accumulate != 0, sqnorm, partial, stream, dtype == DP_F16, co);
    } else if (is16(dtype)) {
        TnPlan t = plan_direct_bf16((int)B, (int)T, (int)d_in, (int)d_out);
        e = launch_direct_bf16(t, static_cast<const uint16_t*>(A), static_cast<const uint16_t*>(G), (int)B, (int)T,
                               (int)d_in, (int)d_out, accumulate != 0, sqnorm, partial, stream, dtype == DP_F16, co);
    } else {
        TnPlan t = plan_direct_f32((int)B, (int)T, (int)d_in, (int)d_out);
        e = launch_direct_f32(t, static_cast<const float*>(A), static_cast<const float*>(G), (int)B, (int)T,
                              (int)d_in, (int)d_out, accumulate != 0, sqnorm, partial, stream, co);
    }
    return e == hipSuccess ? DP_OK : DP_ERR_HIP;
}

}  // namespace

extern "C" {

dp_status dp_clip_factors(const float* sqnorm, int64_t B, float C, float* clip, void* hip_stream) {
    if (B < 0 || !(C > 0.0f)) return DP_ERR_INVALID_ARG;
    if (B > kMaxRows) return DP_ERR_UNSUPPORTED;
    if (B == 0) return DP_OK;
    if (!sqnorm || !clip) return DP_ERR_INVALID_ARG;
    hipError_t e = launch_clip_factors(sqnorm, (int)B, C, clip, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? DP_OK : DP_ERR_HIP;
}

}  // extern "C"

namespace {

// dp_clipped_grad, optionally followed by  grad[j] += stddev * N(0,1)[seed, offset + j].  The noise is added by the
// split-K reduce kernel when there is one and the offsets are multiples of 4, else by the noise kernel.
dp_status clipped_grad_noise(const void* A, const void* G, const float* clip, int64_t B, int64_t T, int64_t d_in,
                             int64_t d_out, dp_dtype dtype, int accumulate, float* grad, void* workspace,
                             size_t workspace_bytes, void* hip_stream, float stddev, uint64_t seed, uint64_t offset);

}  // namespace

extern "C" dp_status dp_clipped_grad(const void* A, const void* G, const float* clip, int64_t B, int64_t T, int64_t d_in,
                                     int64_t d_out, dp_dtype dtype, int accumulate, float* grad, void* workspace,
                                     size_t workspace_bytes, void* hip_stream) {
    return clipped_grad_noise(A, G, clip, B, T, d_in, d_out, dtype, accumulate, grad, workspace, workspace_bytes, hip_stream,
                              0.0f, 0, 0);
}

namespace {

dp_status clipped_grad_noise(const void* A, const void* G, const float* clip, int64_t B, int64_t T, int64_t d_in,
                             int64_t d_out, dp_dtype dtype, int accumulate, float* grad, void* workspace,
                             size_t workspace_bytes, void* hip_stream, float stddev, uint64_t seed, uint64_t offset) {
    dp_status st = check_dims(B, T, d_in, d_out);
    if (st != DP_OK) return st;
    if (!valid_dtype(dtype)) return DP_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (d_in == 0 || d_out == 0) return DP_OK;
    if (!grad || !aligned16(grad)) return DP_ERR_INVALID_ARG;
    const int64_t n = d_in * d_out;
    const bool noisy = stddev != 0.0f;
    if (B == 0 || T == 0) {
        if (!accumulate && launch_fill_zero(grad, n, stream) != hipSuccess) return DP_ERR_HIP;
        if (noisy && launch_add_noise(grad, n, stddev, seed, offset, stream) != hipSuccess) return DP_ERR_HIP;
        return DP_OK;
    }
    if (!A || !G || !clip || !aligned16(A) || !aligned16(G)) return DP_ERR_INVALID_ARG;
    if (is8(dtype) && !dma8_clipped_ok((int)T, (int)d_in, (int)d_out)) {
        const size_t na = widen_bytes(B * T * d_in), ng = widen_bytes(B * T * d_out);
        const size_t inner = clipped_ws_bytes(B, T, d_in, d_out, DP_F16);
        if (!workspace || workspace_bytes < na + ng + inner || !aligned16(workspace)) return DP_ERR_WORKSPACE;
        unsigned char* w = static_cast<unsigned char*>(workspace);
        if (launch_widen_f8(A, reinterpret_cast<uint16_t*>(w), B * T * d_in, a_is_e5m2(dtype), stream) != hipSuccess) return DP_ERR_HIP;
        if (launch_widen_f8(G, reinterpret_cast<uint16_t*>(w + na), B * T * d_out, g_is_e5m2(dtype), stream) != hipSuccess) return DP_ERR_HIP;
        return clipped_grad_noise(w, w + na, clip, B, T, d_in, d_out, DP_F16, accumulate, grad, w + na + ng,
                                  workspace_bytes - na - ng, hip_stream, stddev, seed, offset);
    }
    const size_t need = clipped_ws_bytes(B, T, d_in, d_out, dtype);
    if (need > 0 && (!workspace || workspace_bytes < need || !aligned16(workspace))) return DP_ERR_WORKSPACE;
    float* ws = static_cast<float*>(workspace);

    const TnPlan p = is8(dtype)  ? plan_clipped_f8_dma((int)B, (int)T, (int)d_in, (int)d_out)
                   : is16(dtype) ? plan_clipped_bf16((int)B, (int)T, (int)d_in, (int)d_out)
                                 : plan_clipped_f32((int)B, (int)T, (int)d_in, (int)d_out);
    const NoiseArgs nz{stddev, (uint32_t)seed, (uint32_t)(seed >> 32), offset};
    const bool fused = noisy && p.splits > 1 && splitk_noise_ok(n, offset);
    hipError_t e;
    if (is8(dtype)) {
        e = launch_clipped_f8_dma(p, A, G, clip, (int)B, (int)T, (int)d_in, (int)d_out, accumulate != 0, grad, ws, stream,
                                  fmt_of(dtype), fused ? &nz : nullptr);
    } else if (is16(dtype)) {
        e = launch_clipped_bf16(p, static_cast<const uint16_t*>(A), static_cast<const uint16_t*>(G), clip, (int)B, (int)T,
                                (int)d_in, (int)d_out, accumulate != 0, grad, ws, stream, dtype == DP_F16, fused ? &nz : nullptr);
    } else {
        e = launch_clipped_f32(p, static_cast<const float*>(A), static_cast<const float*>(G), clip, (int)B, (int)T,
                               (int)d_in, (int)d_out, accumulate != 0, grad, ws, stream, fused ? &nz : nullptr);
    }
    if (e == hipSuccess && noisy && !fused) e = launch_add_noise(grad, n, stddev, seed, offset, stream);
    return e == hipSuccess ? DP_OK : DP_ERR_HIP;
}

}  // namespace

extern "C" {

dp_status dp_bias_sqnorm(const void* G, int64_t B, int64_t T, int64_t d_out, dp_dtype dtype, int accumulate,
                         float* sqnorm, float* bias_rows, void* hip_stream) {
    dp_status st = check_dims(B, T, 1, d_out);
    if (st != DP_OK) return st;
    if (!valid_dtype(dtype)) return DP_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (B == 0) return DP_OK;
    if (!sqnorm) return DP_ERR_INVALID_ARG;
    if (d_out == 0) {
        if (!accumulate && launch_fill_zero(sqnorm, B, stream) != hipSuccess) return DP_ERR_HIP;
        return DP_OK;
    }
    if (!bias_rows) return DP_ERR_INVALID_ARG;
    if (T == 0) {
        if (launch_fill_zero(bias_rows, B * d_out, stream) != hipSuccess) return DP_ERR_HIP;
        if (!accumulate && launch_fill_zero(sqnorm, B, stream) != hipSuccess) return DP_ERR_HIP;
        return DP_OK;
    }
    if (!G || !aligned16(G)) return DP_ERR_INVALID_ARG;
    // element type of G for the row kernels: the 8-bit pair types store G as e5m2 unless both are e4m3
    const int gdt = is8(dtype) ? (g_is_e5m2(dtype) ? 4 : 3) : (int)dtype;
    hipError_t e = launch_bias_rows(G, nullptr, (int)B, (int)T, (int)d_out, gdt, bias_rows, nullptr, stream);
    if (e == hipSuccess) e = launch_rows_sqnorm(bias_rows, (int)B, (int)d_out, accumulate != 0, sqnorm, stream);
    return e == hipSuccess ? DP_OK : DP_ERR_HIP;
}

dp_status dp_layernorm_sqnorm(const void* G, const void* Hbar, int64_t B, int64_t T, int64_t d, dp_dtype dtype, int accumulate,
                              float* sqnorm, float* gamma_rows, float* beta_rows, void* hip_stream) {
    dp_status st = check_dims(B, T, 1, d);
    if (st != DP_OK) return st;
    if (!valid_dtype(dtype)) return DP_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (B == 0) return DP_OK;
    if (!sqnorm) return DP_ERR_INVALID_ARG;
    if (d == 0) {
        if (!accumulate && launch_fill_zero(sqnorm, B, stream) != hipSuccess) return DP_ERR_HIP;
        return DP_OK;
    }
    if (!gamma_rows || !beta_rows) return DP_ERR_INVALID_ARG;
    if (T == 0) {
        if (launch_fill_zero(gamma_rows, B * d, stream) != hipSuccess) return DP_ERR_HIP;
        if (launch_fill_zero(beta_rows, B * d, stream) != hipSuccess) return DP_ERR_HIP;
        if (!accumulate && launch_fill_zero(sqnorm, B, stream) != hipSuccess) return DP_ERR_HIP;
        return DP_OK;
    }
    if (!G || !Hbar || !aligned16(G) || !aligned16(Hbar)) return DP_ERR_INVALID_ARG;
    // 8-bit types: Hbar is an activation (stored like A), G a backpropagated gradient
    const int gdt = dtype == DP_F8_E4M3 ? 3 : dtype == DP_F8_E5M2 ? 4 : dtype == DP_F8_E4M3_E5M2 ? 5 : (int)dtype;
    hipError_t e = launch_bias_rows(G, Hbar, (int)B, (int)T, (int)d, gdt, gamma_rows, beta_rows, stream);
    if (e == hipSuccess) e = launch_rows_sqnorm(gamma_rows, (int)B, (int)d, accumulate != 0, sqnorm, stream, beta_rows);
    return e == hipSuccess ? DP_OK : DP_ERR_HIP;
}

dp_status dp_clipped_bias_grad(const float* bias_rows, const float* clip, int64_t B, int64_t d_out, int accumulate,
                               float* grad_b, void* hip_stream) {
    dp_status st = check_dims(B, 1, 1, d_out);
    if (st != DP_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (d_out == 0) return DP_OK;
    if (!grad_b) return DP_ERR_INVALID_ARG;
    if (B == 0) {
        if (!accumulate && launch_fill_zero(grad_b, d_out, stream) != hipSuccess) return DP_ERR_HIP;
        return DP_OK;
    }
    if (!bias_rows || !clip) return DP_ERR_INVALID_ARG;
    hipError_t e = launch_clipped_bias(bias_rows, clip, (int)B, (int)d_out, accumulate != 0, grad_b, stream);
    return e == hipSuccess ? DP_OK : DP_ERR_HIP;
}

size_t dp_conv_workspace_bytes(dp_op op, int64_t B, int64_t H, int64_t W, int64_t C, int64_t KH, int64_t KW, int64_t pad,
                               int64_t d_out, dp_dtype dtype) {
    ConvGeom g; int64_t T, d_in;
    if (conv_geometry(B, H, W, C, KH, KW, pad, d_out, dtype, &g, &T, &d_in) != DP_OK) return 0;
    if (B == 0 || C == 0 || d_out == 0 || H == 0 || W == 0) return 0;
    if (is8(dtype)) {
        // widened to fp16 at the head of the workspace
        const size_t inner = dp_conv_workspace_bytes(op, B, H, W, C, KH, KW, pad, d_out, DP_F16);
        return inner == 0 ? 0 : widen_bytes(B * H * W * C) + widen_bytes(B * T * d_out) + inner;
    }
    if (!is16(dtype)) return 0;
    if (conv_rows_ok(g, (int)d_out, (int)B)) {
        if (op == DP_OP_SQNORM) return kConvZeroBytes + (size_t)B * conv_rows_tiles(g, (int)d_out) * sizeof(float);
        if (op == DP_OP_CLIPPED_GRAD) {
            const int splits = conv_rows_splits(g, (int)d_out, (int)B);
            return kConvZeroBytes + (splits <= 1 ? 0 : (size_t)splits * (size_t)splitk_slice_elems(d_in * d_out) * sizeof(float));
        }
        return 0;
    }
    if (!dma_conv_ok(g, (int)d_out)) return 0;
    if (op == DP_OP_SQNORM) {
        const TnPlan p = plan_direct_bf16_dma((int)B, (int)T, (int)d_in, (int)d_out);
        return kConvZeroBytes + (size_t)B * p.tiles_m * p.tiles_n * sizeof(float);
    }
    if (op == DP_OP_CLIPPED_GRAD) {
        const TnPlan p = plan_clipped_bf16_dma((int)B, (int)T, (int)d_in, (int)d_out);
        return kConvZeroBytes + (p.splits <= 1 ? 0 : (size_t)p.splits * (size_t)splitk_slice_elems(d_in * d_out) * sizeof(float));
    }
    return 0;
}

int dp_conv_rows_resident(int64_t B, int64_t H, int64_t W, int64_t C, int64_t KH, int64_t KW, int64_t pad, int64_t d_out,
                          dp_dtype dtype) {
    ConvGeom g; int64_t T, d_in;
    if (conv_geometry(B, H, W, C, KH, KW, pad, d_out, dtype, &g, &T, &d_in) != DP_OK) return -1;
    if (!(is16(dtype) || is8(dtype)) || B == 0 || T == 0 || d_in == 0 || d_out == 0) return -1;
    if (conv_rows_ok(g, (int)d_out, (int)B)) return 1;
    return dma_conv_ok(g, (int)d_out) ? 0 : -1;
}

dp_status dp_conv_sqnorm(const void* X, const void* G, int64_t B, int64_t H, int64_t W, int64_t C, int64_t KH, int64_t KW,
                         int64_t pad, int64_t d_out, dp_dtype dtype, int accumulate, float* sqnorm,
                         void* workspace, size_t workspace_bytes, void* hip_stream) {
    ConvGeom g; int64_t T, d_in;
    dp_status st = conv_geometry(B, H, W, C, KH, KW, pad, d_out, dtype, &g, &T, &d_in);
    if (st != DP_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (B == 0) return DP_OK;
    if (!sqnorm) return DP_ERR_INVALID_ARG;
    if (d_in == 0 || d_out == 0 || H == 0 || W == 0) {
        if (!accumulate && launch_fill_zero(sqnorm, B, stream) != hipSuccess) return DP_ERR_HIP;
        return DP_OK;
    }
    const bool rows = conv_rows_ok(g, (int)d_out, (int)B);
    if (!(is16(dtype) || is8(dtype)) || !(rows || dma_conv_ok(g, (int)d_out))) return DP_ERR_UNSUPPORTED;
    if (!X || !G || !aligned16(X) || !aligned16(G)) return DP_ERR_INVALID_ARG;
    if (is8(dtype)) {
        const size_t nx = widen_bytes(B * H * W * C), ng = widen_bytes(B * T * d_out);
        const size_t inner = dp_conv_workspace_bytes(DP_OP_SQNORM, B, H, W, C, KH, KW, pad, d_out, DP_F16);
        if (!workspace || workspace_bytes < nx + ng + inner || !aligned16(workspace)) return DP_ERR_WORKSPACE;
        unsigned char* w = static_cast<unsigned char*>(workspace);
        if (launch_widen_f8(X, reinterpret_cast<uint16_t*>(w), B * H * W * C, a_is_e5m2(dtype), stream) != hipSuccess) return DP_ERR_HIP;
        if (launch_widen_f8(G, reinterpret_cast<uint16_t*>(w + nx), B * T * d_out, g_is_e5m2(dtype), stream) != hipSuccess) return DP_ERR_HIP;
        return dp_conv_sqnorm(w, w + nx, B, H, W, C, KH, KW, pad, d_out, DP_F16, accumulate, sqnorm, w + nx + ng,
                              workspace_bytes - nx - ng, hip_stream);
    }
    const size_t need = dp_conv_workspace_bytes(DP_OP_SQNORM, B, H, W, C, KH, KW, pad, d_out, dtype);
    if (need >= (size_t(1) << 33)) return DP_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < need || !aligned16(workspace)) return DP_ERR_WORKSPACE;
    // the line of zeros for the padding: the one in the device image, else the head of the workspace
    const float* zero = static_cast<const float*>(device_zero_line(stream));
    float* partial = static_cast<float*>(workspace) + kConvZeroBytes / sizeof(float);
    if (!zero) {
        if (launch_fill_zero(static_cast<float*>(workspace), kConvZeroBytes / sizeof(float), stream) != hipSuccess) return DP_ERR_HIP;
        zero = static_cast<const float*>(workspace);
    }
    if (rows) {
        const hipError_t er = launch_direct_conv_rows(g, static_cast<const uint16_t*>(X), static_cast<const uint16_t*>(G), (int)B,
                                                      (int)d_out, accumulate != 0, sqnorm, partial, stream,
                                                      reinterpret_cast<const uint16_t*>(zero), dtype == DP_F16);
        return er == hipSuccess ? DP_OK : DP_ERR_HIP;
    }
    const TnPlan p = plan_direct_bf16_dma((int)B, (int)T, (int)d_in, (int)d_out);
    const hipError_t e = launch_direct_bf16_dma(p, static_cast<const uint16_t*>(X), static_cast<const uint16_t*>(G), (int)B, (int)T,
                                                (int)d_in, (int)d_out, accumulate != 0, sqnorm, partial, stream, &g,
                                                reinterpret_cast<const uint16_t*>(zero), dtype == DP_F16);
    return e == hipSuccess ? DP_OK : DP_ERR_HIP;
}

dp_status dp_conv_clipped_grad(const void* X, const void* G, const float* clip, int64_t B, int64_t H, int64_t W, int64_t C,
                               int64_t KH, int64_t KW, int64_t pad, int64_t d_out, dp_dtype dtype, int accumulate,
                               float* grad, void* workspace, size_t workspace_bytes, void* hip_stream) {
    ConvGeom g; int64_t T, d_in;
    dp_status st = conv_geometry(B, H, W, C, KH, KW, pad, d_out, dtype, &g, &T, &d_in);
    if (st != DP_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (d_in == 0 || d_out == 0) return DP_OK;
    if (!grad || !aligned16(grad)) return DP_ERR_INVALID_ARG;
    if (B == 0 || H == 0 || W == 0) {
        if (!accumulate && launch_fill_zero(grad, d_in * d_out, stream) != hipSuccess) return DP_ERR_HIP;
        return DP_OK;
    }
    const bool rows = conv_rows_ok(g, (int)d_out, (int)B);
    if (!(is16(dtype) || is8(dtype)) || !(rows || dma_conv_ok(g, (int)d_out))) return DP_ERR_UNSUPPORTED;
    if (!X || !G || !clip || !aligned16(X) || !aligned16(G)) return DP_ERR_INVALID_ARG;
    if (is8(dtype)) {
        const size_t nx = widen_bytes(B * H * W * C), ng = widen_bytes(B * T * d_out);
        const size_t inner = dp_conv_workspace_bytes(DP_OP_CLIPPED_GRAD, B, H, W, C, KH, KW, pad, d_out, DP_F16);
        if (!workspace || workspace_bytes < nx + ng + inner || !aligned16(workspace)) return DP_ERR_WORKSPACE;
        unsigned char* w = static_cast<unsigned char*>(workspace);
        if (launch_widen_f8(X, reinterpret_cast<uint16_t*>(w), B * H * W * C, a_is_e5m2(dtype), stream) != hipSuccess) return DP_ERR_HIP;
        if (launch_widen_f8(G, reinterpret_cast<uint16_t*>(w + nx), B * T * d_out, g_is_e5m2(dtype), stream) != hipSuccess) return DP_ERR_HIP;
        return dp_conv_clipped_grad(w, w + nx, clip, B, H, W, C, KH, KW, pad, d_out, DP_F16, accumulate, grad, w + nx + ng,
                                    workspace_bytes - nx - ng, hip_stream);
    }
    const size_t need = dp_conv_workspace_bytes(DP_OP_CLIPPED_GRAD, B, H, W, C, KH, KW, pad, d_out, dtype);
    if (!workspace || workspace_bytes < need || !aligned16(workspace)) return DP_ERR_WORKSPACE;
    const float* zero = static_cast<const float*>(device_zero_line(stream));
    float* ws = static_cast<float*>(workspace) + kConvZeroBytes / sizeof(float);
    if (!zero) {
        if (launch_fill_zero(static_cast<float*>(workspace), kConvZeroBytes / sizeof(float), stream) != hipSuccess) return DP_ERR_HIP;
        zero = static_cast<const float*>(workspace);
    }
    if (rows) {
        const hipError_t er = launch_clipped_conv_rows(g, static_cast<const uint16_t*>(X), static_cast<const uint16_t*>(G), clip,
                                                       (int)B, (int)d_out, accumulate != 0, grad, ws, stream,
                                                       reinterpret_cast<const uint16_t*>(zero), dtype == DP_F16, nullptr);
        return er == hipSuccess ? DP_OK : DP_ERR_HIP;
    }
    const TnPlan p = plan_clipped_bf16_dma((int)B, (int)T, (int)d_in, (int)d_out);
    const hipError_t e = launch_clipped_bf16_dma(p, static_cast<const uint16_t*>(X), static_cast<const uint16_t*>(G), clip, (int)B,
                                                 (int)T, (int)d_in, (int)d_out, accumulate != 0, grad, ws, stream, &g,
                                                 reinterpret_cast<const uint16_t*>(zero), dtype == DP_F16, nullptr);
    return e == hipSuccess ? DP_OK : DP_ERR_HIP;
}

dp_status dp_add_noise(float* grad, int64_t n, float stddev, uint64_t seed, uint64_t offset, void* hip_stream) {
    if (n < 0 || !(stddev >= 0.0f)) return DP_ERR_INVALID_ARG;
    if (n == 0) return DP_OK;
    if (!grad) return DP_ERR_INVALID_ARG;
    if (offset > ~uint64_t(0) - (uint64_t)n) return DP_ERR_INVALID_ARG;    // offset + n must not wrap
    if (stddev == 0.0f) return DP_OK;
    hipError_t e = launch_add_noise(grad, n, stddev, seed, offset, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? DP_OK : DP_ERR_HIP;
}

dp_status dp_philox_raw(uint32_t* out, int64_t n_counters, uint64_t seed, uint64_t first_counter, void* hip_stream) {
    if (n_counters < 0) return DP_ERR_INVALID_ARG;
    if (n_counters == 0) return DP_OK;
    if (!out) return DP_ERR_INVALID_ARG;
    hipError_t e = launch_philox_raw(out, n_counters, seed, first_counter, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? DP_OK : DP_ERR_HIP;
}

}  // extern "C"

namespace {

// checks shared by the several-layers calls and their size queries
// op: which call asks
dp_status check_layers(const dp_layer_desc* layers, int64_t n_layers, int64_t B, dp_dtype dtype, dp_path path, bool pointers,
                       dp_op op) {
    (void)op;
    if (n_layers < 0 || B < 0 || (n_layers > 0 && !layers)) return DP_ERR_INVALID_ARG;
    if (!valid_dtype(dtype) || !valid_path(path)) return DP_ERR_INVALID_ARG;
    if (n_layers > 4096) return DP_ERR_UNSUPPORTED;
    for (int64_t l = 0; l < n_layers; ++l) {
        const dp_layer_desc& y = layers[l];
        const dp_status st = check_dims(B, y.T, y.d_in, y.d_out);
        if (st != DP_OK) return st;
        if (B == 0 || y.T == 0 || y.d_in == 0 || y.d_out == 0) continue;
        if (pointers && (!y.A || !y.G || !aligned16(y.A) || !aligned16(y.G))) return DP_ERR_INVALID_ARG;
    }
    return DP_OK;
}

dp_status layers_sqnorm_grouped(const dp_layer_desc* layers, int64_t n_layers, int64_t B, dp_dtype dtype, dp_path path,
                                int accumulate, float* sqnorm, float C, float* clip, void* workspace, size_t workspace_bytes,
                                void* hip_stream);

// scratch: the layers that run one by one reuse one region, and so do the batched launches
size_t layers_ws_bytes(const dp_layer_desc* layers, int64_t n_layers, int64_t B, dp_dtype dtype, dp_path path) {
    size_t single = 0, single_sum = 0, batch = 0, batch_max = 0;
    int in_batch = 0;
    for (int64_t l = 0; l < n_layers; ++l) {
        const dp_layer_desc& y = layers[l];
        if (B == 0 || y.T == 0 || y.d_in == 0 || y.d_out == 0) continue;
        if (gram_cols_class(B, y.T, y.d_in, y.d_out, dtype, path) != 0) continue;      // below
        if (gram_batchable(y.T, y.d_in, y.d_out, dtype, path)) {
            if (in_batch == kGramBatch) { in_batch = 0; batch = 0; }
            const GramPlan g = plan_gram_bf16((int)y.T, (int)y.d_in, (int)y.d_out);
            batch += (size_t)B * g.npairs * sizeof(float);
            if (y.bias_rows && !is8(dtype)) batch += (size_t)B * g.nt * (size_t)y.d_out * sizeof(float);      // column sums per row tile
            ++in_batch;
            if (batch > batch_max) batch_max = batch;
        } else {
            const size_t n = single_layer_need(B, y, dtype, path);
            if (n > single) single = n;
            if (!(y.T == 1 && !is8(dtype))) single_sum += n;
        }
    }
    // the layers that run one by one keep their partial sums apart until one launch folds them (up to a limit: with
    // less scratch the fold comes earlier)
    if (!is8(dtype) && single_sum > single && single_sum <= (size_t(256) << 20)) single = single_sum;
    // the shared column-split Gram launches, one class after the other, kGramColsLayers layers each
    for (int cls = 1; cls <= 2; ++cls) {
        size_t group = 0;
        int in_group = 0;
        for (int64_t l = 0; l < n_layers; ++l) {
            const dp_layer_desc& y = layers[l];
            if (B == 0 || gram_cols_class(B, y.T, y.d_in, y.d_out, dtype, path) != cls) continue;
            if (in_group == kGramColsLayers) { in_group = 0; group = 0; }
            group += plan_gram_cols((int)B, (int)y.T, (int)y.d_in, (int)y.d_out, (int)dtype).ws_floats * sizeof(float);
            ++in_group;
            if (group > batch_max) batch_max = group;
        }
    }
    return round16(single > batch_max ? single : batch_max);
}

}  // namespace

extern "C" {

size_t dp_layers_workspace_bytes(const dp_layer_desc* layers, int64_t n_layers, int64_t B, dp_dtype dtype, dp_path path) {
    if (check_layers(layers, n_layers, B, dtype, path, false, DP_OP_SQNORM) != DP_OK) return 0;
    return layers_ws_bytes(layers, n_layers, B, dtype, path);
}

dp_status dp_layers_sqnorm(const dp_layer_desc* layers, int64_t n_layers, int64_t B, dp_dtype dtype, dp_path path,
                           int accumulate, float* sqnorm, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return dp_layers_sqnorm_clip(layers, n_layers, B, dtype, path, accumulate, sqnorm, 0.0f, nullptr, workspace, workspace_bytes,
                                 hip_stream);
}

dp_status dp_layers_sqnorm_clip(const dp_layer_desc* layers, int64_t n_layers, int64_t B, dp_dtype dtype, dp_path path,
                                int accumulate, float* sqnorm, float C, float* clip, void* workspace, size_t workspace_bytes,
                                void* hip_stream) {
    const dp_status st = check_layers(layers, n_layers, B, dtype, path, true, DP_OP_SQNORM);
    if (st != DP_OK) return st;
    if (clip && !(C > 0.0f)) return DP_ERR_INVALID_ARG;
    if (B == 0) return DP_OK;
    for (int64_t l = 0; l < n_layers; ++l)
        if (layers[l].sqnorm)
            return layers_sqnorm_grouped(layers, n_layers, B, dtype, path, accumulate, sqnorm, C, clip, workspace, workspace_bytes, hip_stream);
    if (!sqnorm) return DP_ERR_INVALID_ARG;
    const size_t need = layers_ws_bytes(layers, n_layers, B, dtype, path);
    if (need >= (size_t(1) << 33)) return DP_ERR_UNSUPPORTED;
    if (need > 0 && (!workspace || workspace_bytes < need || !aligned16(workspace))) return DP_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    int acc = accumulate != 0;
    bool launched = false;
    // Which kernel completes the norms and can write the clip factors with them: the last shared Gram launch if
    // there is one; else, unless a bias pass follows, the last layer that runs on its own; else the last launch
    // of dense layers.  Otherwise (bias passes at the end, or nothing to launch) the clip kernel runs.
    int64_t n_dense = 0, n_cols = 0, last_single = -1;
    bool any_gram = false, any_bias_pass = false;
    for (int64_t l = 0; l < n_layers; ++l) {
        const dp_layer_desc& y = layers[l];
        if (y.bias_rows && y.d_out != 0 &&
            !(!is8(dtype) && y.T > 1 && y.d_in > 0 && gram_batchable(y.T, y.d_in, y.d_out, dtype, path))) any_bias_pass = true;
        if (y.T == 0 || y.d_in == 0 || y.d_out == 0) continue;
        if (y.T == 1 && !is8(dtype)) ++n_dense;
        else if (gram_batchable(y.T, y.d_in, y.d_out, dtype, path)) any_gram = true;
        else if (gram_cols_class(B, y.T, y.d_in, y.d_out, dtype, path) != 0) ++n_cols;
        else last_single = l;
    }
    const ClipOut clip_out{C, clip};
    // layers of few positions and wide rows in a small batch: shared column-split Gram launches, first of all (they
    // write the clip factors only when nothing else follows)
    const bool clip_with_cols = clip && !any_gram && !any_bias_pass && last_single < 0 && n_dense == 0 && n_cols > 0;
    {
        int64_t cols_done = 0;
        for (int cls = 1; cls <= 2; ++cls) {
            GramLayerDesc group[kGramColsLayers];
            int ng = 0;
            auto flush_cols = [&]() -> hipError_t {
                if (ng == 0) return hipSuccess;
                cols_done += ng;
                const hipError_t e = launch_gram_cols_layers(group, ng, (int)B, acc != 0, sqnorm, static_cast<float*>(workspace), stream,
                                                             (int)dtype, (clip_with_cols && cols_done == n_cols) ? &clip_out : nullptr);
                ng = 0; acc = 1; launched = true;
                return e;
            };
            for (int64_t l = 0; l < n_layers; ++l) {
                const dp_layer_desc& y = layers[l];
                if (gram_cols_class(B, y.T, y.d_in, y.d_out, dtype, path) != cls) continue;
                group[ng++] = GramLayerDesc{y.A, y.G, (int)y.T, (int)y.d_in, (int)y.d_out, nullptr, nullptr};
                if (ng == kGramColsLayers && flush_cols() != hipSuccess) return DP_ERR_HIP;
            }
            if (flush_cols() != hipSuccess) return DP_ERR_HIP;
        }
    }
    const bool clip_with_single = clip && !any_gram && !any_bias_pass && last_single >= 0;
    const bool clip_with_dense = clip && !any_gram && !any_bias_pass && last_single < 0 && n_dense > 0;
    // dense layers (T = 1, closed form): up to kDenseBatch per launch, in the order given
    DenseLayers dense;
    dense.n_layers = 0;
    int64_t dense_done = 0;
    auto flush_dense = [&]() -> hipError_t {
        if (dense.n_layers == 0) return hipSuccess;
        dense_done += dense.n_layers;
        const hipError_t e = launch_sqnorm_dense_layers(dense, (int)B, (int)dtype, acc != 0, sqnorm, stream,
                                                        (clip_with_dense && dense_done == n_dense) ? &clip_out : nullptr);
        dense.n_layers = 0; acc = 1; launched = true;
        return e;
    };
    for (int64_t l = 0; l < n_layers; ++l) {
        const dp_layer_desc& y = layers[l];
        if (y.T != 1 || y.d_in == 0 || y.d_out == 0 || is8(dtype)) continue;      // 8-bit dense layers: one by one below
        const int k = dense.n_layers++;
        dense.A[k] = y.A; dense.G[k] = y.G; dense.d_in[k] = (int)y.d_in; dense.d_out[k] = (int)y.d_out;
        if (dense.n_layers == kDenseBatch && flush_dense() != hipSuccess) return DP_ERR_HIP;
    }
    if (flush_dense() != hipSuccess) return DP_ERR_HIP;
    // layers outside the batched launches, in the order given.  Two or more of them: their partial sums are folded by
    // one launch at the end (FinalizeQueue) instead of a launch of a few microseconds behind every layer.
    int64_t n_single = 0;
    for (int64_t l = 0; l < n_layers; ++l) {
        const dp_layer_desc& y = layers[l];
        if (y.T == 0 || (y.T == 1 && !is8(dtype)) || y.d_in == 0 || y.d_out == 0) continue;
        if (gram_batchable(y.T, y.d_in, y.d_out, dtype, path) || gram_cols_class(B, y.T, y.d_in, y.d_out, dtype, path) != 0) continue;
        ++n_single;
    }
    const bool defer_on = n_single >= 2 && !is8(dtype);
    FinalizeQueue queue;
    size_t ws_off = 0;
    auto flush_queue = [&](bool with_clip) -> hipError_t {
        if (queue.count == 0) return hipSuccess;
        const hipError_t e = launch_finalize_queue(queue, (int)B, acc != 0, sqnorm, stream, with_clip ? &clip_out : nullptr);
        queue.count = 0; ws_off = 0; acc = 1; launched = true;
        return e;
    };
    // Two or more of them with aligned widths on the direct path: their norms share copy-pipeline launches of up to
    // kJointLayers layers (a launch each is a few hundred workgroups and a tail), the sums join the queue.
    int64_t n_dj = 0;
    for (int64_t l = 0; l < n_layers; ++l)
        if (direct_joinable(B, layers[l].T, layers[l].d_in, layers[l].d_out, dtype, path)) ++n_dj;
    const bool join_direct = defer_on && n_dj >= 2;
    if (join_direct) {
        JointShape sh[kJointLayers];
        JointOperands op[kJointLayers];
        float* part[kJointLayers];
        int tiles[kJointLayers];
        int ng = 0;
        size_t group_bytes = 0;
        auto flush_group = [&]() -> hipError_t {
            if (ng == 0) return hipSuccess;
            if (queue.count + ng > FinalizeQueue::kMax || ws_off + group_bytes > workspace_bytes) {
                const hipError_t e = flush_queue(false);
                if (e != hipSuccess) return e;
            }
            for (int k = 0; k < ng; ++k) {
                part[k] = reinterpret_cast<float*>(static_cast<char*>(workspace) + ws_off);
                ws_off += round16((size_t)B * tiles[k] * sizeof(float));
            }
            const hipError_t e = is16(dtype) ? launch_direct_bf16_dma_joint(sh, op, part, ng, (int)B, stream, dtype == DP_F16)
                                             : launch_direct_f32_dma_joint(sh, op, part, ng, (int)B, stream);
            for (int k = 0; k < ng; ++k) { queue.partial[queue.count] = part[k]; queue.n[queue.count] = tiles[k]; ++queue.count; }
            ng = 0; group_bytes = 0;
            return e;
        };
        for (int64_t l = 0; l < n_layers; ++l) {
            const dp_layer_desc& y = layers[l];
            if (!direct_joinable(B, y.T, y.d_in, y.d_out, dtype, path)) continue;
            const int t = direct_joint_tiles((int)y.d_in, (int)y.d_out);
            // (a layer's sums alone always fit: the scratch is at least the largest single layer's need)
            if (ng > 0 && group_bytes + round16((size_t)B * t * sizeof(float)) > workspace_bytes && flush_group() != hipSuccess) return DP_ERR_HIP;
            sh[ng] = JointShape{(int)y.T, (int)y.d_in, (int)y.d_out};
            op[ng] = JointOperands{static_cast<const uint16_t*>(y.A), static_cast<const uint16_t*>(y.G), nullptr, nullptr, 0};
            tiles[ng] = t;
            group_bytes += round16((size_t)B * tiles[ng] * sizeof(float));
            ++ng;
            if (ng == kJointLayers && flush_group() != hipSuccess) return DP_ERR_HIP;
        }
        if (flush_group() != hipSuccess) return DP_ERR_HIP;
    }
    for (int64_t l = 0; l < n_layers; ++l) {
        const dp_layer_desc& y = layers[l];
        if (y.T == 0 || (y.T == 1 && !is8(dtype)) || y.d_in == 0 || y.d_out == 0) continue;     // empty layers add nothing
        if (gram_batchable(y.T, y.d_in, y.d_out, dtype, path)) continue;
        if (gram_cols_class(B, y.T, y.d_in, y.d_out, dtype, path) != 0) continue;
        if (join_direct && direct_joinable(B, y.T, y.d_in, y.d_out, dtype, path)) continue;
        if (!defer_on) {
            const dp_status s1 = layer_sqnorm_clip(y.A, y.G, B, y.T, y.d_in, y.d_out, dtype, path, acc, sqnorm, workspace, workspace_bytes,
                                                   hip_stream, (clip_with_single && l == last_single) ? &clip_out : nullptr);
            if (s1 != DP_OK) return s1;
            acc = 1; launched = true;
            continue;
        }
        // the layer's own region of the scratch: its partial sums stay there until the queue is folded
        const size_t need_l = single_layer_need(B, y, dtype, path);
        if ((queue.count == FinalizeQueue::kMax || ws_off + need_l > workspace_bytes) && flush_queue(false) != hipSuccess) return DP_ERR_HIP;
        const ClipOut co_defer{C, nullptr, &queue};
        const int before = queue.count;
        const dp_status s1 = layer_sqnorm_clip(y.A, y.G, B, y.T, y.d_in, y.d_out, dtype, path, acc, sqnorm,
                                               static_cast<char*>(workspace) + ws_off, workspace_bytes - ws_off, hip_stream, &co_defer);
        if (s1 != DP_OK) return s1;
        if (queue.count == before) { acc = 1; launched = true; }      // the layer's kernel added its norms itself
        else ws_off += need_l;
    }
    if (defer_on) {
        const bool queued = queue.count > 0;
        if (flush_queue(clip_with_single) != hipSuccess) return DP_ERR_HIP;
        if (clip_with_single && !queued && launch_clip_factors(sqnorm, (int)B, C, clip, stream) != hipSuccess) return DP_ERR_HIP;
    }
    // bias terms of the layers above (dense ones included): their own pass over G
    for (int64_t l = 0; l < n_layers; ++l) {
        const dp_layer_desc& y = layers[l];
        if (!y.bias_rows || y.d_out == 0) continue;
        // taken by the Gram kernel (16-bit types: the 8-bit Gram kernel has no column sums)
        if (!is8(dtype) && y.T > 1 && y.d_in > 0 && gram_batchable(y.T, y.d_in, y.d_out, dtype, path)) continue;
        const dp_status s1 = dp_bias_sqnorm(y.G, B, y.T, y.d_out, dtype, acc, sqnorm, y.bias_rows, hip_stream);
        if (s1 != DP_OK) return s1;
        acc = 1; launched = true;
    }
    // the others, up to kGramBatch per launch, heaviest first inside a launch (the light ones fill its tail)
    GramLayerDesc batch[kGramBatch];
    int nb = 0;
    // last: the launch that completes the norms also writes the clip factors
    auto flush = [&](bool last) -> hipError_t {
        if (nb == 0) return hipSuccess;
        for (int i = 1; i < nb; ++i) {                                          // stable insertion sort, descending work
            const GramLayerDesc v = batch[i];
            const int64_t wv = (int64_t)(v.d_in + v.d_out);
            int j = i;
            while (j > 0 && (int64_t)(batch[j - 1].d_in + batch[j - 1].d_out) < wv) { batch[j] = batch[j - 1]; --j; }
            batch[j] = v;
        }
        // workspace: the launch's partial sums, then the column-sum scratch of its layers that have a bias
        float* ws = static_cast<float*>(workspace);
        size_t used = 0;
        for (int i = 0; i < nb; ++i) used += (size_t)B * plan_gram_bf16(batch[i].T, batch[i].d_in, batch[i].d_out).npairs;
        for (int i = 0; i < nb; ++i) {
            if (!batch[i].bias_rows) continue;
            batch[i].upart = ws + used;
            used += (size_t)B * plan_gram_bf16(batch[i].T, batch[i].d_in, batch[i].d_out).nt * (size_t)batch[i].d_out;
        }
        const hipError_t e = launch_gram_bf16_dma_layers(batch, nb, (int)B, acc != 0, sqnorm, ws,
                                                         stream, fmt_of(dtype), C, last ? clip : nullptr);
        nb = 0; acc = 1; launched = true;
        return e;
    };
    for (int64_t l = 0; l < n_layers; ++l) {
        const dp_layer_desc& y = layers[l];
        if (y.T == 0 || y.d_in == 0 || y.d_out == 0) continue;
        if (!gram_batchable(y.T, y.d_in, y.d_out, dtype, path)) continue;
        if (nb == kGramBatch && flush(false) != hipSuccess) return DP_ERR_HIP;       // full, and another layer follows
        batch[nb++] = GramLayerDesc{y.A, y.G, (int)y.T, (int)y.d_in, (int)y.d_out, nullptr, is8(dtype) ? nullptr : y.bias_rows};
    }
    const bool clip_done = clip != nullptr && (nb > 0 || clip_with_single || clip_with_dense || clip_with_cols);
    if (flush(true) != hipSuccess) return DP_ERR_HIP;
    if (!launched && !accumulate && launch_fill_zero(sqnorm, B, stream) != hipSuccess) return DP_ERR_HIP;
    if (clip && !clip_done && launch_clip_factors(sqnorm, (int)B, C, clip, stream) != hipSuccess) return DP_ERR_HIP;
    return DP_OK;
}

}  // extern "C"

namespace {

// dp_layers_sqnorm_clip when layers name output arrays of their own (per-layer or grouped clipping, Section 4: a
// threshold per layer or per group of layers).  A group is an output array: the layers' `sqnorm` pointers, and the
// call's own array for the layers that name none.  Every group's norms are complete when its last layer (and bias
// pass) has been added; the kernel that adds it writes the group's clip factors where it can, else a clip-factor
// launch follows.  The shared Gram launches take layers of all groups together.
dp_status layers_sqnorm_grouped(const dp_layer_desc* layers, int64_t n_layers, int64_t B, dp_dtype dtype, dp_path path,
                                int accumulate, float* sqnorm, float C, float* clip, void* workspace, size_t workspace_bytes,
                                void* hip_stream) {
    struct Group { float* out; float C; float* clip; bool holds; int64_t ops; };
    std::vector<Group> groups;
    std::vector<int> group_of((size_t)n_layers, -1);
    auto bias_pass = [&](const dp_layer_desc& y) {     // the layer's bias rows need a pass of their own
        return y.bias_rows && y.d_out != 0 &&
               !(!is8(dtype) && y.T > 1 && y.d_in > 0 && gram_batchable(y.T, y.d_in, y.d_out, dtype, path));
    };
    for (int64_t l = 0; l < n_layers; ++l) {
        const dp_layer_desc& y = layers[l];
        Group g{y.sqnorm ? y.sqnorm : sqnorm, y.sqnorm ? y.clip_C : C, y.sqnorm ? y.clip : clip, accumulate != 0, 0};
        if (!g.out) return DP_ERR_INVALID_ARG;                         // no array of its own and none given to the call
        if (g.clip && !(g.C > 0.0f)) return DP_ERR_INVALID_ARG;
        int gi = -1;
        for (size_t k = 0; k < groups.size(); ++k)
            if (groups[k].out == g.out) { gi = (int)k; break; }
        if (gi < 0) { gi = (int)groups.size(); groups.push_back(g); }
        else if (groups[gi].clip != g.clip || (g.clip && groups[gi].C != g.C)) return DP_ERR_INVALID_ARG;   // one threshold per array
        group_of[l] = gi;
        const bool empty = y.T == 0 || y.d_in == 0 || y.d_out == 0;
        groups[gi].ops += (empty ? 0 : 1) + (bias_pass(y) ? 1 : 0);
    }
    const size_t need = layers_ws_bytes(layers, n_layers, B, dtype, path);
    if (need >= (size_t(1) << 33)) return DP_ERR_UNSUPPORTED;
    if (need > 0 && (!workspace || workspace_bytes < need || !aligned16(workspace))) return DP_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    // groups without any work: zero (unless accumulating) and, from that, their clip factors
    for (Group& g : groups) {
        if (g.ops > 0) continue;
        if (!g.holds && launch_fill_zero(g.out, B, stream) != hipSuccess) return DP_ERR_HIP;
        if (g.clip && launch_clip_factors(g.out, (int)B, g.C, g.clip, stream) != hipSuccess) return DP_ERR_HIP;
    }
    // dense layers and the layers outside the shared launches, one by one in the order given
    for (int64_t l = 0; l < n_layers; ++l) {
        const dp_layer_desc& y = layers[l];
        if (y.T == 0 || y.d_in == 0 || y.d_out == 0) continue;
        if (gram_batchable(y.T, y.d_in, y.d_out, dtype, path)) continue;
        Group& g = groups[group_of[l]];
        const ClipOut co{g.C, g.clip};
        const dp_status s1 = layer_sqnorm_clip(y.A, y.G, B, y.T, y.d_in, y.d_out, dtype, path, g.holds ? 1 : 0, g.out, workspace,
                                               workspace_bytes, hip_stream, (g.clip && g.ops == 1) ? &co : nullptr);
        if (s1 != DP_OK) return s1;
        g.holds = true; --g.ops;
    }
    // bias terms that need their own pass over G
    for (int64_t l = 0; l < n_layers; ++l) {
        const dp_layer_desc& y = layers[l];
        if (!bias_pass(y)) continue;
        Group& g = groups[group_of[l]];
        const dp_status s1 = dp_bias_sqnorm(y.G, B, y.T, y.d_out, dtype, g.holds ? 1 : 0, g.out, y.bias_rows, hip_stream);
        if (s1 != DP_OK) return s1;
        g.holds = true; --g.ops;
        if (g.ops == 0 && g.clip && launch_clip_factors(g.out, (int)B, g.C, g.clip, stream) != hipSuccess) return DP_ERR_HIP;
    }
    // the shared Gram launches, up to kGramBatch layers each, heaviest first inside a launch
    GramLayerDesc batch[kGramBatch];
    int batch_group[kGramBatch];
    int nb = 0;
    auto flush = [&]() -> hipError_t {
        if (nb == 0) return hipSuccess;
        for (int i = 1; i < nb; ++i) {                                          // stable insertion sort, descending work
            const GramLayerDesc v = batch[i];
            const int gv = batch_group[i];
            const int64_t wv = (int64_t)(v.d_in + v.d_out);
            int j = i;
            while (j > 0 && (int64_t)(batch[j - 1].d_in + batch[j - 1].d_out) < wv) { batch[j] = batch[j - 1]; batch_group[j] = batch_group[j - 1]; --j; }
            batch[j] = v; batch_group[j] = gv;
        }
        float* ws = static_cast<float*>(workspace);
        size_t used = 0;
        for (int i = 0; i < nb; ++i) used += (size_t)B * plan_gram_bf16(batch[i].T, batch[i].d_in, batch[i].d_out).npairs;
        for (int i = 0; i < nb; ++i) {
            if (batch[i].bias_rows) {
                batch[i].upart = ws + used;
                used += (size_t)B * plan_gram_bf16(batch[i].T, batch[i].d_in, batch[i].d_out).nt * (size_t)batch[i].d_out;
            }
            int64_t here = 0;                                                   // this group's layers in this launch
            for (int j = 0; j < nb; ++j) here += batch_group[j] == batch_group[i] ? 1 : 0;
            const Group& g = groups[batch_group[i]];
            batch[i].out = g.out; batch[i].out_acc = g.holds; batch[i].out_C = g.C;
            batch[i].out_clip = (g.ops == here) ? g.clip : nullptr;              // the group is complete after this launch
        }
        const hipError_t e = launch_gram_bf16_dma_layers(batch, nb, (int)B, false, nullptr, ws, stream, fmt_of(dtype), 0.f, nullptr);
        for (int i = 0; i < nb; ++i) { groups[batch_group[i]].holds = true; --groups[batch_group[i]].ops; }
        nb = 0;
        return e;
    };
    for (int64_t l = 0; l < n_layers; ++l) {
        const dp_layer_desc& y = layers[l];
        if (y.T == 0 || y.d_in == 0 || y.d_out == 0) continue;
        if (!gram_batchable(y.T, y.d_in, y.d_out, dtype, path)) continue;
        if (nb == kGramBatch && flush() != hipSuccess) return DP_ERR_HIP;
        batch_group[nb] = group_of[l];
        batch[nb++] = GramLayerDesc{y.A, y.G, (int)y.T, (int)y.d_in, (int)y.d_out, nullptr, is8(dtype) ? nullptr : y.bias_rows};
    }
    if (flush() != hipSuccess) return DP_ERR_HIP;
    return DP_OK;
}

}  // namespace

extern "C" {

size_t dp_layers_clipped_workspace_bytes(const dp_layer_desc* layers, int64_t n_layers, int64_t B, dp_dtype dtype) {
    if (check_layers(layers, n_layers, B, dtype, DP_PATH_DIRECT, false, DP_OP_CLIPPED_GRAD) != DP_OK) return 0;
    size_t need = 0;
    for (int64_t l = 0; l < n_layers; ++l) {
        const dp_layer_desc& y = layers[l];
        const size_t n = dp_workspace_bytes(DP_OP_CLIPPED_GRAD, B, y.T, y.d_in, y.d_out, dtype, DP_PATH_AUTO);
        if (n > need) need = n;
    }
    for (int geo : {1, 3, 4, 5}) {                              // the two classes of joint launches, each in groups of its own
        JointShape sh[kJointLayers];
        int nj = 0;
        auto joint_need = [&]() {
            if (nj >= 2) need = std::max(need, joint_ws_bytes(sh, nj, B, dtype, geo));
            nj = 0;
        };
        for (int64_t l = 0; l < n_layers; ++l) {
            const dp_layer_desc& y = layers[l];
            if (clipped_join_class(B, y.T, y.d_in, y.d_out, dtype) != geo) continue;
            sh[nj++] = JointShape{(int)y.T, (int)y.d_in, (int)y.d_out};
            if (nj == kJointLayers) joint_need();
        }
        joint_need();
    }
    return round16(need);
}

dp_status dp_layers_clipped_grad(const dp_layer_desc* layers, int64_t n_layers, int64_t B, const float* clip, dp_dtype dtype,
                                 int accumulate, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return dp_layers_clipped_grad_noise(layers, n_layers, B, clip, dtype, accumulate, 0.0f, 0, workspace, workspace_bytes, hip_stream);
}

dp_status dp_layers_step(const dp_layer_desc* layers, int64_t n_layers, int64_t B, dp_dtype dtype, dp_path path, float C,
                         float* sqnorm, float* clip, float stddev, uint64_t seed, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
    if (!clip || !(stddev >= 0.0f)) return DP_ERR_INVALID_ARG;
    const dp_status st = dp_layers_sqnorm_clip(layers, n_layers, B, dtype, path, 0, sqnorm, C, clip, workspace, workspace_bytes, hip_stream);
    if (st != DP_OK) return st;
    return dp_layers_clipped_grad_noise(layers, n_layers, B, clip, dtype, 0, stddev, seed, workspace, workspace_bytes, hip_stream);
}

dp_status dp_layers_clipped_grad_noise(const dp_layer_desc* layers, int64_t n_layers, int64_t B, const float* clip, dp_dtype dtype,
                                       int accumulate, float stddev, uint64_t seed, void* workspace, size_t workspace_bytes,
                                       void* hip_stream) {
    // everything is checked before the first launch: an error leaves every output untouched
    if (!(stddev >= 0.0f)) return DP_ERR_INVALID_ARG;
    const dp_status st = check_layers(layers, n_layers, B, dtype, DP_PATH_DIRECT, true, DP_OP_CLIPPED_GRAD);
    if (st != DP_OK) return st;
    size_t need = 0;
    for (int64_t l = 0; l < n_layers; ++l) {
        const dp_layer_desc& y = layers[l];
        if (y.d_in > 0 && y.d_out > 0 && (!y.grad || !aligned16(y.grad))) return DP_ERR_INVALID_ARG;
        if (stddev > 0.0f && y.noise_offset > ~uint64_t(0) - (uint64_t)(y.d_in * y.d_out)) return DP_ERR_INVALID_ARG;   // offset + n must not wrap
        if (y.grad_b && y.d_out > 0) {
            if (B > 0 && !y.bias_rows) return DP_ERR_INVALID_ARG;                  // the rows that dp_layers_sqnorm left
            if (stddev > 0.0f && y.bias_noise_offset > ~uint64_t(0) - (uint64_t)y.d_out) return DP_ERR_INVALID_ARG;
        }
        const size_t n = dp_workspace_bytes(DP_OP_CLIPPED_GRAD, B, y.T, y.d_in, y.d_out, dtype, DP_PATH_AUTO);
        if (n > need) need = n;
    }
    for (int64_t l = 0; l < n_layers; ++l)
        if (B > 0 && !clip && !layers[l].clip) return DP_ERR_INVALID_ARG;          // neither the layer's own factors nor the call's
    // Aligned 16-bit and 8-bit layers with 256 x 256 tiles share launches, up to kJointLayers each (groups of at least two):
    // one launch whose items fill the chip a whole number of times, the K slices folded (and the noise added) inside
    // it.  With noise the kernel adds it four elements at a time, so the layer's offset and size must be multiples of 4.
    // A second class of joint launches (128 x 128 tiles) takes the aligned 16-bit layers of a few hundred columns.
    std::vector<std::vector<int64_t>> joint_groups;
    std::vector<int> joint_geo;
    for (int geo : {1, 3, 4, 5}) {
        std::vector<int64_t> cur;
        const size_t first_group = joint_groups.size();
        for (int64_t l = 0; l < n_layers; ++l) {
            const dp_layer_desc& y = layers[l];
            if (clipped_join_class(B, y.T, y.d_in, y.d_out, dtype) != geo) continue;
            if (stddev > 0.0f && !splitk_noise_ok(y.d_in * y.d_out, y.noise_offset)) continue;
            cur.push_back(l);
            if ((int)cur.size() == kJointLayers) { joint_groups.push_back(cur); joint_geo.push_back(geo); cur.clear(); }
        }
        if (cur.size() >= 2) { joint_groups.push_back(cur); joint_geo.push_back(geo); }
        // the largest layers first: the tiles that are folded when the launch ends are then the smallest layer's
        for (size_t gi = first_group; gi < joint_groups.size(); ++gi) {
            auto& g = joint_groups[gi];
            std::stable_sort(g.begin(), g.end(), [&](int64_t a, int64_t b) {
                return layers[a].d_in * layers[a].d_out * layers[a].T > layers[b].d_in * layers[b].d_out * layers[b].T; });
            JointShape sh[kJointLayers];
            for (size_t k = 0; k < g.size(); ++k) {
                const dp_layer_desc& y = layers[g[k]];
                sh[k] = JointShape{(int)y.T, (int)y.d_in, (int)y.d_out};
            }
            need = std::max(need, joint_ws_bytes(sh, (int)g.size(), B, dtype, geo));
        }
    }
    if (need > 0 && (!workspace || workspace_bytes < need || !aligned16(workspace))) return DP_ERR_WORKSPACE;
    // float32 layers with a short contraction (a model of small dense layers) share launches, 8 layers each
    std::vector<char> done((size_t)n_layers, 0);
    for (size_t gi = 0; gi < joint_groups.size(); ++gi) {
        const auto& g = joint_groups[gi];
        JointShape sh[kJointLayers];
        JointOperands op[kJointLayers];
        for (size_t k = 0; k < g.size(); ++k) {
            const dp_layer_desc& y = layers[g[k]];
            sh[k] = JointShape{(int)y.T, (int)y.d_in, (int)y.d_out};
            op[k] = JointOperands{static_cast<const uint16_t*>(y.A), static_cast<const uint16_t*>(y.G), y.clip ? y.clip : clip, y.grad,
                                  y.noise_offset};
            done[(size_t)g[k]] = 1;
        }
        const hipError_t ej = joint_geo[gi] == 5
            ? launch_clipped_f32_dma_joint(sh, op, (int)g.size(), (int)B, accumulate != 0, stddev, seed, static_cast<float*>(workspace),
                                           static_cast<hipStream_t>(hip_stream))
            : is8(dtype)
            ? launch_clipped_f8_dma_joint(sh, op, (int)g.size(), (int)B, accumulate != 0, stddev, seed, static_cast<float*>(workspace),
                                          static_cast<hipStream_t>(hip_stream), fmt_of(dtype))
            : launch_clipped_bf16_dma_joint(sh, op, (int)g.size(), (int)B, accumulate != 0, stddev, seed, static_cast<float*>(workspace),
                                            static_cast<hipStream_t>(hip_stream), dtype == DP_F16, joint_geo[gi]);
        if (ej != hipSuccess) return DP_ERR_HIP;
    }
    if (dtype == DP_F32 && B > 0 && !(stddev > 0.0f)) {
        ShortLayerDesc batch[8];
        int64_t which[8];
        int nb = 0;
        auto flush = [&]() -> hipError_t {
            hipError_t e = hipSuccess;
            if (nb >= 2) {
                e = launch_clipped_f32_short_layers(batch, nb, (int)B, accumulate != 0, static_cast<hipStream_t>(hip_stream));
                for (int i = 0; i < nb; ++i) done[(size_t)which[i]] = 1;
            }
            nb = 0;
            return e;
        };
        for (int64_t l = 0; l < n_layers; ++l) {
            const dp_layer_desc& y = layers[l];
            if (y.T == 0 || y.d_in == 0 || y.d_out == 0) continue;
            if (!clipped_f32_is_short(plan_clipped_f32((int)B, (int)y.T, (int)y.d_in, (int)y.d_out))) continue;
            which[nb] = l;
            batch[nb++] = ShortLayerDesc{static_cast<const float*>(y.A), static_cast<const float*>(y.G), y.clip ? y.clip : clip, y.grad,
                                         (int)y.T, (int)y.d_in, (int)y.d_out};
            if (nb == 8 && flush() != hipSuccess) return DP_ERR_HIP;
        }
        if (flush() != hipSuccess) return DP_ERR_HIP;
    }
    for (int64_t l = 0; l < n_layers; ++l) {
        const dp_layer_desc& y = layers[l];
        const dp_status s1 = done[(size_t)l] ? DP_OK
                           : clipped_grad_noise(y.A, y.G, y.clip ? y.clip : clip, B, y.T, y.d_in, y.d_out, dtype, accumulate, y.grad, workspace,
                                                workspace_bytes, hip_stream, stddev, seed, y.noise_offset);
        if (s1 != DP_OK) return s1;
        if (y.grad_b && y.d_out > 0) {
            // the layer's bias: sum_i nu_i bias_rows[i, :], with its own stretch of the noise stream
            hipStream_t stream = static_cast<hipStream_t>(hip_stream);
            hipError_t e = hipSuccess;
            if (B == 0) { if (!accumulate) e = launch_fill_zero(y.grad_b, y.d_out, stream); }
            else e = launch_clipped_bias(y.bias_rows, y.clip ? y.clip : clip, (int)B, (int)y.d_out, accumulate != 0, y.grad_b, stream);
            if (e == hipSuccess && stddev > 0.0f) e = launch_add_noise(y.grad_b, y.d_out, stddev, seed, y.bias_noise_offset, stream);
            if (e != hipSuccess) return DP_ERR_HIP;
        }
    }
    return DP_OK;
}

}  // extern "C"
