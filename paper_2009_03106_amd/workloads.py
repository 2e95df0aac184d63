"""Seeded synthetic layer inputs (A, G) for the per-example clipping path.

This module only draws random tensors.  It holds none of the method's
arithmetic (no norms, no clip factors, no gradients): both the CPU oracle's
tests and the HIP path's tests/bench read their inputs from here so that the
two sides consume identical bits.

The paper measured on MNIST / FMNIST / CIFAR10 / IMDB / LSUN models
(Section 6).  None of that data is needed by the path, which consumes only a
layer's inputs X^(l) and the back-propagated dLoss/dZ^(l) (Section 5, last
paragraph before 5.1).  The generators below stand in for those datasets:
they reproduce layer *shapes* and value *distributions* (post-ReLU half-zero
activations, tanh activations, small Gaussian output gradients).

Layouts: A is [B, T, d_in], G is [B, T, d_out], row-major, example-major.
fp32 tensors are numpy float32.  bf16 tensors are numpy uint16 holding the
upper 16 bits of the float32 value after round-to-nearest-even.  fp16 tensors
(dtype "f16", an override of a configuration's own type) are numpy float16.
8-bit tensors (dtypes "f8e4m3", "f8e5m2", and "f8" = A e4m3 with G e5m2; also
overrides) are numpy uint8 holding the bit patterns of the OCP 8-bit formats.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

BASE_SEED = 20090310


@dataclass(frozen=True)
class LayerSpec:
    name: str
    T: int
    d_in: int
    d_out: int


@dataclass(frozen=True)
class Workload:
    """One benchmark configuration: a list of linear layers sharing a batch."""
    name: str
    index: int            # position in the configuration list (also the seed offset)
    B: int
    dtype: str            # "f32" or "bf16"
    C: float              # clipping threshold
    layers: Tuple[LayerSpec, ...]
    a_dist: str           # "normal" | "relu" | "tanh"
    g_std: float
    typical_norm: float   # rough size of one example's gradient norm (only used to centre the straddle variant)
    noise_std: float = 0.0
    noise_seed: int = 0x5EED2009


WORKLOADS = {
    "dense": Workload("dense", 0, 32, "f32", 1.0,
                      (LayerSpec("fc", 1, 64, 32),), "normal", 0.1, 4.5),
    "mlp": Workload("mlp", 1, 256, "f32", 1.0,
                    (LayerSpec("fc1", 1, 784, 512), LayerSpec("fc2", 1, 512, 256),
                     LayerSpec("fc3", 1, 256, 10)), "relu", 0.01, 5.2),
    "rnn": Workload("rnn", 2, 128, "bf16", 0.5,
                    (LayerSpec("shared_linear", 64, 256, 256),), "tanh", 0.01, 12.9),
    "conv": Workload("conv", 3, 128, "bf16", 1.0,
                     (LayerSpec("conv3x3_im2col", 1024, 576, 128),), "relu", 0.001, 6.1),
    "transformer": Workload("transformer", 4, 64, "bf16", 1.0,
                            (LayerSpec("qkv", 512, 768, 2304), LayerSpec("attn_out", 512, 768, 768),
                             LayerSpec("ffn_up", 512, 768, 3072), LayerSpec("ffn_down", 512, 3072, 768)),
                            "normal", 1e-3, 60.0, noise_std=1.0),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns.
    Inputs here are finite, so NaN handling is not needed."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float32."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _draw(rng: np.random.Generator, shape, dist: str, std: float = 1.0) -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if dist == "relu":
        np.maximum(x, 0.0, out=x)
    elif dist == "tanh":
        np.tanh(x, out=x)
    elif dist != "normal":
        raise ValueError(dist)
    if std != 1.0:
        x *= np.float32(std)
    return x


F8_MAX = {"e4m3": 448.0, "e5m2": 57344.0}   # largest finite values of the two OCP 8-bit formats


def f32_to_f8_bits(x: np.ndarray, fmt: str) -> np.ndarray:
    """Round float32 to an OCP 8-bit float ("e4m3": torch.float8_e4m3fn, "e5m2": torch.float8_e5m2; nearest, ties to
    even, magnitudes beyond the largest finite value saturate to it); returns the uint8 bit patterns."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).clamp(-F8_MAX[fmt], F8_MAX[fmt])
    t8 = t.to(torch.float8_e4m3fn if fmt == "e4m3" else torch.float8_e5m2)
    return t8.view(torch.uint8).numpy().copy()


def f8_formats(dtype: str) -> Tuple[str, str]:
    """Storage types of (A, G) for the 8-bit dtype names: "f8e4m3" and "f8e5m2" store both alike, "f8" stores the
    activations A as e4m3 and the backpropagated gradients G as e5m2."""
    if dtype == "f8":
        return "f8e4m3", "f8e5m2"
    if dtype in ("f8e4m3", "f8e5m2"):
        return dtype, dtype
    raise ValueError(dtype)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return x
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    if dtype == "f16":
        return x.astype(np.float16)           # numpy rounds to nearest even
    if dtype in ("f8e4m3", "f8e5m2"):
        return f32_to_f8_bits(x, dtype[2:])
    raise ValueError(dtype)


def make_layer(rng: np.random.Generator, B: int, spec: LayerSpec, dtype: str,
               a_dist: str, g_std: float, g_row_scale: np.ndarray | None = None):
    """Draw one layer's (A, G).  g_row_scale, if given, is a per-example factor on G."""
    A = _draw(rng, (B, spec.T, spec.d_in), a_dist)
    G = _draw(rng, (B, spec.T, spec.d_out), "normal", g_std)
    if g_row_scale is not None:
        G *= g_row_scale.astype(np.float32)[:, None, None]
    da, dg = f8_formats(dtype) if dtype.startswith("f8") else (dtype, dtype)
    return _store(A, da), _store(G, dg)


def generate(name: str, B: int | None = None, straddle: bool = False,
             layers: Tuple[int, ...] | None = None, dtype: str | None = None, g_scale: float = 1.0):
    """Return (workload, [(A, G), ...]) for the named configuration.

    B overrides the batch size (used for bounded CPU samples and scaled sweeps).
    straddle=True multiplies each example's G by (C / typical_norm) times a
    log-uniform factor in [0.1, 10] so that roughly half of the examples end up
    below the clipping threshold and both branches of the clip function are
    exercised.
    layers selects a subset of layer indices (all layers are still drawn so
    the random stream of the remaining ones does not change).
    dtype stores the same draws in another format; g_scale multiplies G (a loss
    scale, as mixed-precision training uses to keep fp16 gradients in range).
    """
    w = WORKLOADS[name]
    B = w.B if B is None else int(B)
    rng = np.random.default_rng(BASE_SEED + w.index + (1000 if straddle else 0))
    scale = None
    if straddle:
        scale = (w.C / w.typical_norm) * np.exp(rng.uniform(np.log(0.1), np.log(10.0), size=B))
    out = []
    for li, spec in enumerate(w.layers):
        pair = make_layer(rng, B, spec, dtype or w.dtype, w.a_dist, w.g_std * g_scale, scale)
        if layers is None or li in layers:
            out.append(pair)
        else:
            out.append(None)
    return w, out


def random_layer(seed: int, B: int, T: int, d_in: int, d_out: int, dtype: str,
                 a_dist: str = "normal", g_std: float = 0.05, g_row_scale=None):
    """Free-form shapes for edge-case tests (ragged tiles, tiny sizes)."""
    rng = np.random.default_rng(seed)
    return make_layer(rng, B, LayerSpec("adhoc", T, d_in, d_out), dtype, a_dist, g_std, g_row_scale)


# The convolution configuration as an image: the same layer (3 x 3 kernel, padding 1, 64 -> 128 channels on
# 32 x 32 inputs) given by its input X[B, H, W, C] (channels last) instead of the unfolded patch matrix.
CONV_IMAGE = {"B": 128, "H": 32, "W": 32, "C": 64, "KH": 3, "KW": 3, "pad": 1, "d_out": 128,
              "dtype": "bf16", "C_clip": 1.0, "g_std": 1e-3}


def generate_conv_image(B: int | None = None, H: int | None = None, W: int | None = None, C: int | None = None,
                        KH: int | None = None, KW: int | None = None, pad: int | None = None,
                        d_out: int | None = None, seed: int = BASE_SEED + 40, g_row_scale: np.ndarray | None = None,
                        dtype: str = "bf16"):
    """(spec, X, G): X[B,H,W,C] = max(0, N(0,1)), G[B, H_out*W_out, d_out] = N(0, g_std^2), both stored as `dtype`
    (bf16 bit patterns by default).  Any geometry argument overrides the configuration's value."""
    spec = dict(CONV_IMAGE)
    for k, v in (("B", B), ("H", H), ("W", W), ("C", C), ("KH", KH), ("KW", KW), ("pad", pad), ("d_out", d_out)):
        if v is not None:
            spec[k] = int(v)
    rng = np.random.default_rng(seed)
    ho, wo = spec["H"] + 2 * spec["pad"] - spec["KH"] + 1, spec["W"] + 2 * spec["pad"] - spec["KW"] + 1
    X = _draw(rng, (spec["B"], spec["H"], spec["W"], spec["C"]), "relu")
    G = _draw(rng, (spec["B"], ho * wo, spec["d_out"]), "normal", spec["g_std"])
    if g_row_scale is not None:
        G *= g_row_scale.astype(np.float32)[:, None, None]
    return spec, _store(X, dtype), _store(G, dtype)
