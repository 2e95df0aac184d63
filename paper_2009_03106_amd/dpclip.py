"""Thin ctypes binding over libdpclip.so (see include/dpclip.h for the contract).

Argument marshalling only: tensors -> device pointers and sizes, the current
torch stream -> hipStream_t.  Every computation runs in the HIP kernels.  There
is no CPU fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libdpclip.so")

DP_OK = 0
DP_ERR_INVALID_ARG, DP_ERR_UNSUPPORTED, DP_ERR_WORKSPACE, DP_ERR_HIP = 1, 2, 3, 4
DP_F32, DP_BF16, DP_F16, DP_F8_E4M3, DP_F8_E5M2, DP_F8_E4M3_E5M2 = 0, 1, 2, 3, 4, 5
DP_PATH_AUTO, DP_PATH_GRAM, DP_PATH_DIRECT = 0, 1, 2
DP_OP_SQNORM, DP_OP_CLIPPED_GRAD = 0, 1
_PATHS = {"auto": DP_PATH_AUTO, "gram": DP_PATH_GRAM, "direct": DP_PATH_DIRECT}

EXPORTS = ("dp_layer_sqnorm", "dp_layer_sqnorm_static", "dp_layers_sqnorm", "dp_layers_sqnorm_clip", "dp_layers_workspace_bytes", "dp_layers_clipped_grad",
           "dp_layers_clipped_grad_noise", "dp_layers_step", "dp_layers_clipped_workspace_bytes", "dp_clip_factors", "dp_clipped_grad", "dp_bias_sqnorm", "dp_clipped_bias_grad", "dp_layernorm_sqnorm",
           "dp_conv_sqnorm", "dp_conv_clipped_grad", "dp_conv_workspace_bytes", "dp_conv_rows_resident", "dp_add_noise", "dp_workspace_bytes", "dp_choose_path", "dp_status_string", "dp_philox_raw",
           "dp_clipped_grad_rounds_inputs")

# the measurement probes of include/dpclip_probes.h
PROBE_EXPORTS = ("dp_probe_mfma", "dp_probe_read", "dp_probe_lds_read")
PROBE_SINK_FLOATS = 1024 * 256

_lib = None


class LayerDesc(ctypes.Structure):
    """dp_layer_desc of the header."""
    _fields_ = [("A", ctypes.c_void_p), ("G", ctypes.c_void_p), ("T", ctypes.c_int64), ("d_in", ctypes.c_int64),
                ("d_out", ctypes.c_int64), ("grad", ctypes.c_void_p), ("noise_offset", ctypes.c_uint64),
                ("bias_rows", ctypes.c_void_p), ("sqnorm", ctypes.c_void_p), ("clip", ctypes.c_void_p),
                ("clip_C", ctypes.c_float), ("grad_b", ctypes.c_void_p), ("bias_noise_offset", ctypes.c_uint64)]


class DpclipError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (dp_status {status})")


def load_library() -> ctypes.CDLL:
    """Load libdpclip.so from the package directory; raise if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not found: build it first (python -m paper_2009_03106_amd.build); "
                           "there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    i64, vp, sz, u64, f32, ci = (ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint64,
                                 ctypes.c_float, ctypes.c_int)
    lib.dp_layer_sqnorm.argtypes = [vp, vp, i64, i64, i64, i64, ci, ci, ci, vp, vp, sz, vp]
    lib.dp_layer_sqnorm.restype = ci
    lib.dp_layer_sqnorm_static.argtypes = [vp, vp, i64, i64, i64, i64, ci, ci, ci, vp, vp]
    lib.dp_layer_sqnorm_static.restype = ci
    lib.dp_layers_sqnorm.argtypes = [ctypes.POINTER(LayerDesc), i64, i64, ci, ci, ci, vp, vp, sz, vp]
    lib.dp_layers_sqnorm.restype = ci
    lib.dp_layers_sqnorm_clip.argtypes = [ctypes.POINTER(LayerDesc), i64, i64, ci, ci, ci, vp, f32, vp, vp, sz, vp]
    lib.dp_layers_sqnorm_clip.restype = ci
    lib.dp_layers_workspace_bytes.argtypes = [ctypes.POINTER(LayerDesc), i64, i64, ci, ci]
    lib.dp_layers_workspace_bytes.restype = sz
    lib.dp_layers_clipped_grad.argtypes = [ctypes.POINTER(LayerDesc), i64, i64, vp, ci, ci, vp, sz, vp]
    lib.dp_layers_clipped_grad.restype = ci
    lib.dp_layers_clipped_grad_noise.argtypes = [ctypes.POINTER(LayerDesc), i64, i64, vp, ci, ci, f32, u64, vp, sz, vp]
    lib.dp_layers_clipped_grad_noise.restype = ci
    lib.dp_layers_step.argtypes = [ctypes.POINTER(LayerDesc), i64, i64, ci, ci, f32, vp, vp, f32, u64, vp, sz, vp]
    lib.dp_layers_step.restype = ci
    lib.dp_layers_clipped_workspace_bytes.argtypes = [ctypes.POINTER(LayerDesc), i64, i64, ci]
    lib.dp_layers_clipped_workspace_bytes.restype = sz
    lib.dp_clip_factors.argtypes = [vp, i64, f32, vp, vp]
    lib.dp_clip_factors.restype = ci
    lib.dp_clipped_grad.argtypes = [vp, vp, vp, i64, i64, i64, i64, ci, ci, vp, vp, sz, vp]
    lib.dp_clipped_grad.restype = ci
    lib.dp_bias_sqnorm.argtypes = [vp, i64, i64, i64, ci, ci, vp, vp, vp]
    lib.dp_bias_sqnorm.restype = ci
    lib.dp_layernorm_sqnorm.argtypes = [vp, vp, i64, i64, i64, ci, ci, vp, vp, vp, vp]
    lib.dp_layernorm_sqnorm.restype = ci
    lib.dp_clipped_bias_grad.argtypes = [vp, vp, i64, i64, ci, vp, vp]
    lib.dp_clipped_bias_grad.restype = ci
    lib.dp_conv_sqnorm.argtypes = [vp, vp, i64, i64, i64, i64, i64, i64, i64, i64, ci, ci, vp, vp, sz, vp]
    lib.dp_conv_sqnorm.restype = ci
    lib.dp_conv_clipped_grad.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, i64, i64, i64, ci, ci, vp, vp, sz, vp]
    lib.dp_conv_clipped_grad.restype = ci
    lib.dp_conv_workspace_bytes.argtypes = [ci, i64, i64, i64, i64, i64, i64, i64, i64, ci]
    lib.dp_conv_workspace_bytes.restype = sz
    lib.dp_conv_rows_resident.argtypes = [i64, i64, i64, i64, i64, i64, i64, i64, ci]
    lib.dp_conv_rows_resident.restype = ci
    lib.dp_add_noise.argtypes = [vp, i64, f32, u64, u64, vp]
    lib.dp_add_noise.restype = ci
    lib.dp_workspace_bytes.argtypes = [ci, i64, i64, i64, i64, ci, ci]
    lib.dp_workspace_bytes.restype = sz
    lib.dp_choose_path.argtypes = [i64, i64, i64]
    lib.dp_choose_path.restype = ci
    lib.dp_status_string.argtypes = [ci]
    lib.dp_status_string.restype = ctypes.c_char_p
    lib.dp_philox_raw.argtypes = [vp, i64, u64, u64, vp]
    lib.dp_philox_raw.restype = ci
    lib.dp_clipped_grad_rounds_inputs.argtypes = [i64, i64, i64, i64, ci]
    lib.dp_clipped_grad_rounds_inputs.restype = ci
    lib.dp_probe_mfma.argtypes = [ci, ci, i64, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.dp_probe_mfma.restype = ci
    lib.dp_probe_read.argtypes = [vp, sz, vp, vp]
    lib.dp_probe_read.restype = ci
    lib.dp_probe_lds_read.argtypes = [ci, i64, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.dp_probe_lds_read.restype = ci
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().dp_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != DP_OK:
        raise DpclipError(status, where)


def _dtype_code(t: torch.Tensor, G: Optional[torch.Tensor] = None) -> int:
    """Library code of a tensor's type; with G, of the (A, G) pair: both of one type, or A e4m3 with G e5m2."""
    if G is not None and G.dtype != t.dtype:
        if t.dtype == torch.float8_e4m3fn and G.dtype == torch.float8_e5m2:
            return DP_F8_E4M3_E5M2
        raise TypeError(f"unsupported pair of dtypes {t.dtype}, {G.dtype}")
    if t.dtype == torch.float32:
        return DP_F32
    if t.dtype == torch.bfloat16:
        return DP_BF16
    if t.dtype == torch.float16:
        return DP_F16
    if t.dtype == torch.float8_e4m3fn:
        return DP_F8_E4M3
    if t.dtype == torch.float8_e5m2:
        return DP_F8_E5M2
    raise TypeError(f"unsupported dtype {t.dtype}")


# torch's raw handle of the current stream: building a torch.cuda.Stream object for it costs about 3 us per call,
# as much as the library call itself
_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    if stream is not None:
        return int(stream.cuda_stream)
    if _raw_stream is not None:
        return int(_raw_stream(torch.cuda.current_device()))
    return int(torch.cuda.current_stream().cuda_stream)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous device tensors")
    return t.data_ptr() if t.numel() > 0 else None


def _f32(t: Optional[torch.Tensor], shape, name: str) -> Optional[int]:
    """Pointer of a float32 device tensor that the library reads or writes as `shape`: a tensor of another type,
    size or layout would become an out-of-bounds access on the device, so it is refused here."""
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous float32 device tensor")
    n = 1
    for d in shape:
        n *= int(d)
    if t.numel() != n:
        raise ValueError(f"{name} must hold {tuple(shape)} = {n} elements, got {tuple(t.shape)}")
    return t.data_ptr() if n > 0 else None


def _on_stream(stream: Optional[torch.cuda.Stream], *tensors) -> None:
    """Temporaries that this module allocated (on torch's current stream) for a call issued on another stream:
    tell the caching allocator, or it could hand the block out again while the kernel still runs."""
    if stream is None or stream == torch.cuda.current_stream():
        return
    for t in tensors:
        if t is not None and t.numel() > 0:
            t.record_stream(stream)


def _shape3(A: torch.Tensor, G: torch.Tensor):
    if A.dim() == 2:
        A = A.unsqueeze(1)
    if G.dim() == 2:
        G = G.unsqueeze(1)
    if A.dim() != 3 or G.dim() != 3 or A.shape[:2] != G.shape[:2]:
        raise ValueError("A must be [B,T,d_in] and G [B,T,d_out]")
    _dtype_code(A, G)                       # one dtype, or the e4m3 / e5m2 pair
    B, T, d_in = A.shape
    return A, G, int(B), int(T), int(d_in), int(G.shape[2])


def choose_path(T: int, d_in: int, d_out: int) -> str:
    code = load_library().dp_choose_path(T, d_in, d_out)
    return {DP_PATH_GRAM: "gram", DP_PATH_DIRECT: "direct"}[code]


def workspace_bytes(op: int, B: int, T: int, d_in: int, d_out: int, dtype: int, path: str = "auto") -> int:
    return int(load_library().dp_workspace_bytes(op, B, T, d_in, d_out, dtype, _PATHS[path]))


def _workspace(nbytes, device, workspace: Optional[torch.Tensor]) -> Optional[torch.Tensor]:
    """The caller's workspace if there is one (the library checks its size), else a fresh one of nbytes() bytes."""
    if workspace is not None:
        return workspace
    n = nbytes()
    if n == 0:
        return None
    return torch.empty(n, dtype=torch.uint8, device=device)


def layer_sqnorm(A: torch.Tensor, G: torch.Tensor, sqnorm: Optional[torch.Tensor] = None, *,
                 path: str = "auto", accumulate: bool = False, workspace: Optional[torch.Tensor] = None,
                 stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """sqnorm[i] (+)= ||A_i^T G_i||_F^2 via dp_layer_sqnorm."""
    lib = load_library()
    A, G, B, T, d_in, d_out = _shape3(A, G)
    dt = _dtype_code(A, G)
    if sqnorm is None:
        if accumulate:
            raise ValueError("accumulate needs an existing sqnorm tensor")
        sqnorm = torch.empty(B, dtype=torch.float32, device=A.device)
    ws = _workspace(lambda: workspace_bytes(DP_OP_SQNORM, B, T, d_in, d_out, dt, path), A.device, workspace)
    _on_stream(stream, None if workspace is not None else ws)
    st = lib.dp_layer_sqnorm(_ptr(A), _ptr(G), B, T, d_in, d_out, dt, _PATHS[path], int(bool(accumulate)),
                             _f32(sqnorm, (B,), "sqnorm"), _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                             _stream_ptr(stream))
    _check(st, "dp_layer_sqnorm")
    return sqnorm


def check_noise_ranges(ranges) -> None:
    """Raise unless the [offset, offset + n) stretches of the noise stream are pairwise disjoint: two gradients that
    shared draws would not get the independent N(0, sigma^2) per coordinate that the Gaussian mechanism asks for."""
    end = -1
    for off, n in sorted(r for r in ranges if r[1] > 0):
        if off < end:
            raise ValueError("noise offsets overlap: every weight and bias gradient needs its own stretch of the stream")
        end = off + n


STATIC_SCRATCH_BYTES = 4 << 20


def layer_sqnorm_static(A: torch.Tensor, G: torch.Tensor, sqnorm: torch.Tensor, *, path: str = "auto",
                        accumulate: bool = False, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """layer_sqnorm through dp_layer_sqnorm_static: no workspace, nothing allocated (sqnorm is the caller's); problems
    needing more than STATIC_SCRATCH_BYTES of scratch raise DP_ERR_WORKSPACE."""
    lib = load_library()
    if not (A.is_contiguous() and G.is_contiguous()):
        raise ValueError("A and G must be contiguous")
    A, G, B, T, d_in, d_out = _shape3(A, G)
    st = lib.dp_layer_sqnorm_static(_ptr(A), _ptr(G), B, T, d_in, d_out, _dtype_code(A, G), _PATHS[path],
                                    int(bool(accumulate)), _f32(sqnorm, (B,), "sqnorm"), _stream_ptr(stream))
    _check(st, "dp_layer_sqnorm_static")
    return sqnorm


def noise_layout(sizes, has_bias, noise_offsets=None, bias_noise_offsets=None):
    """Positions in the noise stream of every layer's weight gradient and bias gradient.
    sizes: (d_in, d_out) per layer; has_bias: per layer, whether a bias gradient draws noise.
    Defaults: the weight gradients back to back from 0 in the order given, the bias gradients back to back behind
    the last weight gradient.  Returns (weight offsets, bias offsets (0 where there is no bias)); raises if any two
    stretches overlap."""
    w_offs, running = [], 0
    for i, (d_in, d_out) in enumerate(sizes):
        w_offs.append(running if noise_offsets is None else int(noise_offsets[i]))
        running += d_in * d_out
    bias_running = max([o + d_in * d_out for o, (d_in, d_out) in zip(w_offs, sizes)], default=0)
    b_offs = []
    for i, (d_in, d_out) in enumerate(sizes):
        if not has_bias[i]:
            b_offs.append(0)
            continue
        b_offs.append(bias_running if bias_noise_offsets is None else int(bias_noise_offsets[i]))
        bias_running += d_out
    check_noise_ranges([(o, d_in * d_out) for o, (d_in, d_out) in zip(w_offs, sizes)] +
                       [(o, d_out) for o, (_, d_out), hb in zip(b_offs, sizes, has_bias) if hb])
    return w_offs, b_offs


def layer_descs(layers, grads=None, noise_offsets=None, bias_rows=None, groups=None, grad_bs=None, bias_noise_offsets=None):
    """(ctypes array of dp_layer_desc, B, dtype code) for a list of (A, G) tensor pairs sharing B and dtype, with
    the float32 [d_in, d_out] output of each layer if grads is given (layers_clipped_grad needs them) and the position of
    each gradient in the noise stream if noise_offsets is given (default: the gradients laid out back to back in the order
    of the list).  bias_rows: one float32 [B, d_out] tensor (or None) per layer: layers_sqnorm then also writes the
    per-example bias gradients there and counts their norms.
    groups: per-layer or grouped clipping: one (sqnorm, clip, C) triple (or None) per layer, float32 [B] tensors (clip
    may be None) and the group's threshold; layers that give the same sqnorm tensor form a group, whose norms
    layers_sqnorm adds up in that tensor (and whose clip factors it writes to clip), and whose clip factors
    layers_clipped_grad uses for these layers.
    grad_bs: one float32 [d_out] tensor (or None) per layer: layers_clipped_grad then also writes the clipped sum of the
    layer's bias rows there.  bias_noise_offsets: their positions in the noise stream; by default the bias gradients
    follow the last weight gradient back to back, in the order of the list, so that every parameter of the model
    draws its own stretch of the stream (the Gaussian mechanism needs independent noise per coordinate).  Offsets
    given by the caller are checked: the ranges [offset, offset + n) of all weight and bias gradients must be
    pairwise disjoint.
    The tensors must stay alive (and contiguous: the pointers are taken here) while the array is used."""
    if len(layers) == 0:
        raise ValueError("no layers")
    if grads is not None and len(grads) != len(layers):
        raise ValueError("one gradient tensor per layer")
    arr = (LayerDesc * len(layers))()
    B0, dt0 = None, None
    w_offs, b_offs = noise_layout([(int(A.shape[-1]), int(G.shape[-1])) for A, G in layers],
                                  [grad_bs is not None and grad_bs[i] is not None for i in range(len(layers))],
                                  noise_offsets, bias_noise_offsets)
    for i, (A, G) in enumerate(layers):
        if not (A.is_contiguous() and G.is_contiguous()):
            raise ValueError("layer tensors must be contiguous")
        A, G, B, T, d_in, d_out = _shape3(A, G)
        dt = _dtype_code(A, G)
        if B0 is None:
            B0, dt0 = B, dt
        elif (B, dt) != (B0, dt0):
            raise ValueError("all layers must share the batch size and the dtype")
        gp = None
        if grads is not None:
            g = grads[i]
            if g.dtype != torch.float32 or tuple(g.shape) != (d_in, d_out):
                raise ValueError("gradients must be float32 [d_in, d_out]")
            gp = _ptr(g)
        bp = None
        if bias_rows is not None and bias_rows[i] is not None:
            if bias_rows[i].dtype != torch.float32 or tuple(bias_rows[i].shape) != (B, d_out):
                raise ValueError("bias rows must be float32 [B, d_out]")
            bp = _ptr(bias_rows[i])
        sp, cp, cC = None, None, 0.0
        if groups is not None and groups[i] is not None:
            gs, gc, cC = groups[i]
            for t in (gs, gc):
                if t is not None and (t.dtype != torch.float32 or tuple(t.shape) != (B,)):
                    raise ValueError("group arrays must be float32 [B]")
            sp, cp = _ptr(gs), _ptr(gc)
        gbp = None
        if grad_bs is not None and grad_bs[i] is not None:
            if grad_bs[i].dtype != torch.float32 or tuple(grad_bs[i].shape) != (d_out,):
                raise ValueError("bias gradients must be float32 [d_out]")
            gbp = _ptr(grad_bs[i])
        arr[i] = LayerDesc(_ptr(A), _ptr(G), T, d_in, d_out, gp, w_offs[i], bp, sp, cp, float(cC), gbp, b_offs[i])
    return arr, B0, dt0


def layers_workspace_bytes(descs, B: int, dtype: int, path: str = "auto") -> int:
    return int(load_library().dp_layers_workspace_bytes(descs, len(descs), B, dtype, _PATHS[path]))


def layers_sqnorm(layers, sqnorm: Optional[torch.Tensor] = None, *, path: str = "auto", accumulate: bool = False,
                  workspace: Optional[torch.Tensor] = None, descs=None, C: Optional[float] = None,
                  clip: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """sqnorm[i] (+)= sum over the (A, G) pairs of ||A_i^T G_i||_F^2 via dp_layers_sqnorm(_clip).
    With C and clip given, clip[i] = min(1, C / sqrt(sqnorm[i])) is written as well.
    descs: the result of layer_descs(layers), to skip rebuilding it on every call."""
    lib = load_library()
    arr, B, dt = descs if descs is not None else layer_descs(layers)
    dev = layers[0][0].device
    if sqnorm is None:
        if accumulate:
            raise ValueError("accumulate needs an existing sqnorm tensor")
        sqnorm = torch.empty(B, dtype=torch.float32, device=dev)
    ws = _workspace(lambda: layers_workspace_bytes(arr, B, dt, path), dev, workspace)
    _on_stream(stream, None if workspace is not None else ws)
    if (C is None) != (clip is None):
        raise ValueError("C and clip go together")
    st = lib.dp_layers_sqnorm_clip(arr, len(arr), B, dt, _PATHS[path], int(bool(accumulate)), _f32(sqnorm, (B,), "sqnorm"),
                                   0.0 if C is None else float(C), _f32(clip, (B,), "clip"), _ptr(ws),
                                   0 if ws is None else ws.numel() * ws.element_size(), _stream_ptr(stream))
    _check(st, "dp_layers_sqnorm_clip")
    return sqnorm


def layers_clipped_workspace_bytes(descs, B: int, dtype: int) -> int:
    return int(load_library().dp_layers_clipped_workspace_bytes(descs, len(descs), B, dtype))


def layers_clipped_grad(layers, clip: torch.Tensor, grads=None, *, accumulate: bool = False,
                        workspace: Optional[torch.Tensor] = None, descs=None, noise_std: float = 0.0, seed: int = 0,
                        stream: Optional[torch.cuda.Stream] = None):
    """grads[l] (+)= sum_i clip[i] A_l,i^T G_l,i for every (A, G) pair via dp_layers_clipped_grad(_noise); returns grads.
    noise_std > 0 also adds noise_std * N(0,1)[seed, noise_offset_l + j] to every grads[l][j] (see layer_descs).
    descs: the result of layer_descs(layers, grads), to skip rebuilding it on every call."""
    lib = load_library()
    if descs is None:
        if grads is None:
            if accumulate:
                raise ValueError("accumulate needs existing gradient tensors")
            grads = [torch.empty((A.shape[-1], G.shape[-1]), dtype=torch.float32, device=A.device) for A, G in layers]
        descs = layer_descs(layers, grads)
    arr, B, dt = descs
    ws = _workspace(lambda: layers_clipped_workspace_bytes(arr, B, dt), layers[0][0].device, workspace)
    _on_stream(stream, None if workspace is not None else ws)
    st = lib.dp_layers_clipped_grad_noise(arr, len(arr), B, _f32(clip, (B,), "clip"), dt, int(bool(accumulate)), float(noise_std),
                                          int(seed) & (2 ** 64 - 1), _ptr(ws),
                                          0 if ws is None else ws.numel() * ws.element_size(), _stream_ptr(stream))
    _check(st, "dp_layers_clipped_grad_noise")
    return grads


def layers_step(descs, C: float, sqnorm: torch.Tensor, clip: torch.Tensor, workspace: torch.Tensor, *, path: str = "auto",
                noise_std: float = 0.0, seed: int = 0, stream: Optional[torch.cuda.Stream] = None):
    """Norms, clip factors, clipped sums and noise of all layers in one call (dp_layers_step).  descs: the result of
    layer_descs(layers, grads, ...); workspace: at least max(layers_workspace_bytes, layers_clipped_workspace_bytes) bytes."""
    lib = load_library()
    arr, B, dt = descs
    _on_stream(stream, None)
    st = lib.dp_layers_step(arr, len(arr), B, dt, _PATHS[path], float(C), _f32(sqnorm, (B,), "sqnorm"), _f32(clip, (B,), "clip"),
                            float(noise_std), int(seed) & (2 ** 64 - 1), _ptr(workspace),
                            workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    _check(st, "dp_layers_step")


def clip_factors(sqnorm: torch.Tensor, C: float, clip: Optional[torch.Tensor] = None, *,
                 stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """clip[i] = min(1, C / sqrt(sqnorm[i])) via dp_clip_factors."""
    lib = load_library()
    if clip is None:
        clip = torch.empty_like(sqnorm)
    n = sqnorm.numel()
    st = lib.dp_clip_factors(_f32(sqnorm, (n,), "sqnorm"), n, float(C), _f32(clip, (n,), "clip"), _stream_ptr(stream))
    _check(st, "dp_clip_factors")
    return clip


def clipped_grad(A: torch.Tensor, G: torch.Tensor, clip: torch.Tensor, grad: Optional[torch.Tensor] = None, *,
                 accumulate: bool = False, workspace: Optional[torch.Tensor] = None,
                 stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """grad (+)= sum_i clip[i] A_i^T G_i, float32 [d_in, d_out], via dp_clipped_grad."""
    lib = load_library()
    A, G, B, T, d_in, d_out = _shape3(A, G)
    dt = _dtype_code(A, G)
    if grad is None:
        if accumulate:
            raise ValueError("accumulate needs an existing grad tensor")
        grad = torch.empty((d_in, d_out), dtype=torch.float32, device=A.device)
    ws = _workspace(lambda: workspace_bytes(DP_OP_CLIPPED_GRAD, B, T, d_in, d_out, dt), A.device, workspace)
    _on_stream(stream, None if workspace is not None else ws)
    st = lib.dp_clipped_grad(_ptr(A), _ptr(G), _f32(clip, (B,), "clip"), B, T, d_in, d_out, dt, int(bool(accumulate)),
                             _f32(grad, (d_in, d_out), "grad"), _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                             _stream_ptr(stream))
    _check(st, "dp_clipped_grad")
    return grad


def bias_sqnorm(G: torch.Tensor, sqnorm: Optional[torch.Tensor] = None, bias_rows: Optional[torch.Tensor] = None, *,
                accumulate: bool = False, stream: Optional[torch.cuda.Stream] = None):
    """bias_rows[i] = sum_t G_i[t]; sqnorm[i] (+)= ||bias_rows[i]||^2 via dp_bias_sqnorm.  Returns (sqnorm, bias_rows)."""
    lib = load_library()
    if G.dim() == 2:
        G = G.unsqueeze(1)
    if G.dim() != 3:
        raise ValueError("G must be [B, d_out] or [B, T, d_out]")
    Gc = G.contiguous()
    _on_stream(stream, None if Gc is G else Gc)
    G = Gc
    B, T, d_out = G.shape
    if sqnorm is None:
        if accumulate:
            raise ValueError("accumulate needs an existing sqnorm tensor")
        sqnorm = torch.empty(B, dtype=torch.float32, device=G.device)
    if bias_rows is None:
        bias_rows = torch.empty((B, d_out), dtype=torch.float32, device=G.device)
    st = lib.dp_bias_sqnorm(_ptr(G), B, T, d_out, _dtype_code(G), int(bool(accumulate)), _f32(sqnorm, (B,), "sqnorm"),
                            _f32(bias_rows, (B, d_out), "bias_rows"), _stream_ptr(stream))
    _check(st, "dp_bias_sqnorm")
    return sqnorm, bias_rows


def layernorm_sqnorm(G: torch.Tensor, Hbar: torch.Tensor, sqnorm: Optional[torch.Tensor] = None, *,
                     accumulate: bool = False, stream: Optional[torch.cuda.Stream] = None):
    """gamma_rows[i] = sum_t G_i[t] * Hbar_i[t], beta_rows[i] = sum_t G_i[t], sqnorm[i] (+)= their squared norms,
    via dp_layernorm_sqnorm.  Returns (sqnorm, gamma_rows, beta_rows)."""
    lib = load_library()
    if G.dim() == 2:
        G, Hbar = G.unsqueeze(1), Hbar.unsqueeze(1)
    if G.dim() != 3 or G.shape != Hbar.shape:
        raise ValueError("G and Hbar must have the same [B, T, d] shape")
    dt = _dtype_code(Hbar, G)               # one dtype, or Hbar e4m3 (an activation) with G e5m2
    Gc, Hc = G.contiguous(), Hbar.contiguous()
    _on_stream(stream, None if Gc is G else Gc, None if Hc is Hbar else Hc)
    G, Hbar = Gc, Hc
    B, T, d = G.shape
    if sqnorm is None:
        if accumulate:
            raise ValueError("accumulate needs an existing sqnorm tensor")
        sqnorm = torch.empty(B, dtype=torch.float32, device=G.device)
    gam = torch.empty((B, d), dtype=torch.float32, device=G.device)
    bet = torch.empty((B, d), dtype=torch.float32, device=G.device)
    st = lib.dp_layernorm_sqnorm(_ptr(G), _ptr(Hbar), B, T, d, dt, int(bool(accumulate)), _f32(sqnorm, (B,), "sqnorm"),
                                 _ptr(gam), _ptr(bet), _stream_ptr(stream))
    _check(st, "dp_layernorm_sqnorm")
    return sqnorm, gam, bet


def clipped_bias_grad(bias_rows: torch.Tensor, clip: torch.Tensor, grad_b: Optional[torch.Tensor] = None, *,
                      accumulate: bool = False, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """grad_b (+)= sum_i clip[i] bias_rows[i], float32 [d_out], via dp_clipped_bias_grad."""
    lib = load_library()
    if bias_rows.dtype != torch.float32 or bias_rows.dim() != 2 or not bias_rows.is_contiguous():
        raise TypeError("bias_rows must be a contiguous float32 [B, d_out] tensor")
    B, d_out = bias_rows.shape
    if grad_b is None:
        if accumulate:
            raise ValueError("accumulate needs an existing grad_b tensor")
        grad_b = torch.empty(d_out, dtype=torch.float32, device=bias_rows.device)
    st = lib.dp_clipped_bias_grad(_ptr(bias_rows), _f32(clip, (B,), "clip"), B, d_out, int(bool(accumulate)),
                                  _f32(grad_b, (d_out,), "grad_b"),
                                  _stream_ptr(stream))
    _check(st, "dp_clipped_bias_grad")
    return grad_b


def _conv_args(X: torch.Tensor, G: torch.Tensor, KH: int, KW: int, pad: int):
    if X.dim() != 4 or G.dim() != 3 or X.shape[0] != G.shape[0]:
        raise ValueError("X must be [B, H, W, C] (channels last) and G [B, H_out*W_out, d_out]")
    if not (X.is_contiguous() and G.is_contiguous()):
        raise ValueError("X and G must be contiguous (X channels last: [B, H, W, C] in memory)")
    B, H, W, C = X.shape
    T = (H + 2 * pad - KH + 1) * (W + 2 * pad - KW + 1)
    if G.shape[1] != T:
        raise ValueError("G does not match the convolution's output positions")
    _dtype_code(X, G)                       # one dtype, or the e4m3 / e5m2 pair
    return X, G, B, H, W, C, G.shape[2]


def conv_workspace_bytes(op: int, B: int, H: int, W: int, C: int, KH: int, KW: int, pad: int, d_out: int, dtype: int) -> int:
    return int(load_library().dp_conv_workspace_bytes(op, B, H, W, C, KH, KW, pad, d_out, dtype))


def conv_rows_resident(B: int, H: int, W: int, C: int, KH: int, KW: int, pad: int, d_out: int, dtype: int) -> bool:
    """Test hook: whether the convolution calls run this geometry on the kernel that keeps the image rows in LDS."""
    r = load_library().dp_conv_rows_resident(B, H, W, C, KH, KW, pad, d_out, dtype)
    if r < 0:
        raise ValueError("invalid or unsupported arguments")
    return bool(r)


def conv_sqnorm(X: torch.Tensor, G: torch.Tensor, KH: int, KW: int, pad: int, sqnorm: Optional[torch.Tensor] = None, *,
                accumulate: bool = False, workspace: Optional[torch.Tensor] = None,
                stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """sqnorm[i] (+)= squared norm of example i's kernel gradient, from the image X, via dp_conv_sqnorm."""
    lib = load_library()
    X, G, B, H, W, C, d_out = _conv_args(X, G, KH, KW, pad)
    dt = _dtype_code(X, G)
    if sqnorm is None:
        if accumulate:
            raise ValueError("accumulate needs an existing sqnorm tensor")
        sqnorm = torch.empty(B, dtype=torch.float32, device=X.device)
    ws = _workspace(lambda: conv_workspace_bytes(DP_OP_SQNORM, B, H, W, C, KH, KW, pad, d_out, dt), X.device, workspace)
    _on_stream(stream, None if workspace is not None else ws)
    st = lib.dp_conv_sqnorm(_ptr(X), _ptr(G), B, H, W, C, KH, KW, pad, d_out, dt, int(bool(accumulate)), _f32(sqnorm, (B,), "sqnorm"),
                            _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(), _stream_ptr(stream))
    _check(st, "dp_conv_sqnorm")
    return sqnorm


def conv_clipped_grad(X: torch.Tensor, G: torch.Tensor, clip: torch.Tensor, KH: int, KW: int, pad: int,
                      grad: Optional[torch.Tensor] = None, *, accumulate: bool = False,
                      workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """grad (+)= sum_i clip[i] * (kernel gradient of example i), float32 [KH*KW*C, d_out], via dp_conv_clipped_grad."""
    lib = load_library()
    X, G, B, H, W, C, d_out = _conv_args(X, G, KH, KW, pad)
    dt = _dtype_code(X, G)
    if grad is None:
        if accumulate:
            raise ValueError("accumulate needs an existing grad tensor")
        grad = torch.empty((KH * KW * C, d_out), dtype=torch.float32, device=X.device)
    ws = _workspace(lambda: conv_workspace_bytes(DP_OP_CLIPPED_GRAD, B, H, W, C, KH, KW, pad, d_out, dt), X.device, workspace)
    _on_stream(stream, None if workspace is not None else ws)
    st = lib.dp_conv_clipped_grad(_ptr(X), _ptr(G), _f32(clip, (B,), "clip"), B, H, W, C, KH, KW, pad, d_out, dt, int(bool(accumulate)),
                                  _f32(grad, (KH * KW * C, d_out), "grad"), _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                                  _stream_ptr(stream))
    _check(st, "dp_conv_clipped_grad")
    return grad


def add_noise(grad: torch.Tensor, stddev: float, seed: int, offset: int = 0, *,
              stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """grad += stddev * N(0,1)[seed, offset + j] in place via dp_add_noise."""
    lib = load_library()
    st = lib.dp_add_noise(_f32(grad, (grad.numel(),), "grad"), grad.numel(), float(stddev), int(seed) & (2 ** 64 - 1), int(offset),
                          _stream_ptr(stream))
    _check(st, "dp_add_noise")
    return grad


def clipped_grad_rounds_inputs(B: int, T: int, d_in: int, d_out: int, dtype: int) -> bool:
    """Test hook: whether clipped_grad folds the clip factors into re-rounded 16-bit rows of A for this shape."""
    r = load_library().dp_clipped_grad_rounds_inputs(B, T, d_in, d_out, dtype)
    if r < 0:
        raise ValueError("invalid arguments")
    return bool(r)


def probe_mfma(dtype: int, random_operands: bool, iters: int, sink: torch.Tensor, *,
               stream: Optional[torch.cuda.Stream] = None) -> float:
    """Launch the register-resident matrix-unit probe (dp_probe_mfma); returns the flops of the launch."""
    work = ctypes.c_double(0.0)
    st = load_library().dp_probe_mfma(dtype, int(bool(random_operands)), int(iters), _f32(sink, (PROBE_SINK_FLOATS,), "sink"),
                                      ctypes.byref(work), _stream_ptr(stream))
    _check(st, "dp_probe_mfma")
    return work.value


def probe_read(src: torch.Tensor, sink: torch.Tensor, *, stream: Optional[torch.cuda.Stream] = None) -> float:
    """Launch the streaming-read probe over all of src (dp_probe_read); returns the bytes read."""
    nbytes = src.numel() * src.element_size()
    st = load_library().dp_probe_read(_ptr(src), nbytes, _f32(sink, (PROBE_SINK_FLOATS,), "sink"), _stream_ptr(stream))
    _check(st, "dp_probe_read")
    return float(nbytes)


def probe_lds_read(kind: int, iters: int, sink: torch.Tensor, *, stream: Optional[torch.cuda.Stream] = None) -> float:
    """Launch the LDS read probe (dp_probe_lds_read; kind 0: ds_read_b128, 1: ds_read_b64_tr_b16); returns the bytes
    that the lanes of the launch received."""
    work = ctypes.c_double(0.0)
    st = load_library().dp_probe_lds_read(int(kind), int(iters), _f32(sink, (PROBE_SINK_FLOATS,), "sink"),
                                          ctypes.byref(work), _stream_ptr(stream))
    _check(st, "dp_probe_lds_read")
    return work.value


def philox_raw(n_counters: int, seed: int, first_counter: int, device="cuda") -> torch.Tensor:
    """Raw Philox4x32-10 words, int32 view of uint32 [n_counters, 4] (test hook)."""
    lib = load_library()
    out = torch.empty((n_counters, 4), dtype=torch.int32, device=device)
    st = lib.dp_philox_raw(_ptr(out), n_counters, int(seed) & (2 ** 64 - 1), int(first_counter), _stream_ptr(None))
    _check(st, "dp_philox_raw")
    return out
