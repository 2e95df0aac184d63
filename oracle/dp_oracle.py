"""CPU oracle for per-example gradient clipping.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this file.  The product path (the HIP library and its binding) never does,
and this file imports nothing from the product.  It shares no code, table or
constant generator with the HIP kernels.

Everything is float64 and takes the slow, literal route: each example's
gradient matrix is materialised and then measured, clipped and summed, which
is numerically the "one example at a time" baseline the paper compares
against (Section 3.3, first baseline).  A numpy matmul is the only library
primitive used as a step.

Notation (Section 5): a layer has inputs X^(l) and pre-activation gradients
dLoss/dZ^(l).  Here A[B, T, d_in] holds the inputs (T = 1 for a dense layer,
the sequence length for a recurrent / attention projection, the number of
output positions for an unfolded convolution) and G[B, T, d_out] holds the
per-example pre-activation gradients.  Example i's weight gradient is
    g_i = sum_t outer(A[i,t,:], G[i,t,:]) = A_i^T G_i        (d_in x d_out)
(Eq. grad_linear_layer for T = 1; Eq. recurrent_gradient for a sum over time;
Algorithm 3's bmm of the unfolded patches with dZ for convolutions; the
attention result dL/dW^Q = (dL/dQ^(l))^T Q^(l-1) in Section 5.6).

Pins (tests/test_oracle_pins.py): Goodfellow's closed form for T = 1
(Section 4), hand-computed integer cases, brute-force scalar loops on tiny
inputs, Gram == direct, orthonormal-row and repeated-row closed forms,
scaling laws, additivity over a split of d_out and over layers, the clip
invariant of Section 3.2, reduction to a plain batch gradient when nothing
is clipped, and for the random stream an independent Philox4x32-10 engine
(ATen's header, compiled and called by the test) plus moment / KS checks of
the normals.  No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

_MASK32 = 0xFFFFFFFF


# --------------------------------------------------------------------------
# input widening
# --------------------------------------------------------------------------
def widen(x: np.ndarray) -> np.ndarray:
    """Stored bits -> float64, exactly.  uint16 arrays are bf16 bit patterns
    (upper half of a float32); float16 / float32 arrays are taken as they are."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if x.dtype == np.float16 or x.dtype == np.float32 or x.dtype == np.float64:
        return x.astype(np.float64)
    raise TypeError(f"unsupported storage dtype {x.dtype}")


def f8_to_f64(bits: np.ndarray, fmt: str) -> np.ndarray:
    """Bit patterns of an OCP 8-bit floating-point format -> float64, exactly,
    from the formats' definition (OCP 8-bit Floating Point Specification): a
    sign bit, E exponent bits with a bias and M mantissa bits;
        exponent field 0:      (-1)^s * 2^(1 - bias) * (m / 2^M)        (zero and subnormals)
        otherwise:             (-1)^s * 2^(e - bias) * (1 + m / 2^M)
    "e4m3": E = 4, M = 3, bias 7; no infinities, and only the code with every
            exponent and mantissa bit set is a NaN (so 1.75 * 2^8 = 448 is the largest value);
    "e5m2": E = 5, M = 2, bias 15; exponent field 31 is infinity (m = 0) or NaN.
    uint8 arrays carry no format of their own, so 8-bit inputs are widened with
    this function before they are handed to the functions below."""
    if fmt == "e4m3":
        E, M, bias = 4, 3, 7
    elif fmt == "e5m2":
        E, M, bias = 5, 2, 15
    else:
        raise ValueError(fmt)
    b = np.asarray(bits)
    if b.dtype != np.uint8:
        raise TypeError("8-bit patterns are uint8")
    b = b.astype(np.int64)
    s = b >> 7
    e = (b >> M) & ((1 << E) - 1)
    m = b & ((1 << M) - 1)
    frac = m.astype(np.float64) / float(1 << M)
    mag = np.where(e == 0, np.ldexp(frac, 1 - bias), np.ldexp(1.0 + frac, e - bias))
    if fmt == "e4m3":
        mag = np.where((e == 15) & (m == 7), np.nan, mag)
    else:
        mag = np.where(e == 31, np.where(m == 0, np.inf, np.nan), mag)
    return np.where(s == 1, -mag, mag)


def _as3d(x: np.ndarray) -> np.ndarray:
    x = widen(x)
    if x.ndim == 2:              # dense layer given as [B, d]
        x = x[:, None, :]
    if x.ndim != 3:
        raise ValueError("expected [B, T, d] or [B, d]")
    return x


# --------------------------------------------------------------------------
# per-example gradients and their squared norms
# --------------------------------------------------------------------------
def per_example_grad(A_i: np.ndarray, G_i: np.ndarray) -> np.ndarray:
    """g_i = sum_t outer(A_i[t], G_i[t]) for one example, [d_in, d_out].
    (Eq. grad_linear_layer / Eq. recurrent_gradient, stored input-major: the
    paper writes W as d_in x d_out in Algorithm 1's Z = XW + b.)"""
    return A_i.T @ G_i


def layer_sqnorm(A, G) -> np.ndarray:
    """s[i] = ||g_i||_F^2 by materialising g_i (the definition)."""
    A = _as3d(A)
    G = _as3d(G)
    B = A.shape[0]
    s = np.zeros(B, dtype=np.float64)
    for i in range(B):
        M = per_example_grad(A[i], G[i])
        s[i] = np.sum(M * M)
    return s


def layer_sqnorm_gram(A, G) -> np.ndarray:
    """The same squared norm through the two T x T Gram matrices:
    ||A_i^T G_i||_F^2 = trace(G_i^T A_i A_i^T G_i) = sum_{t,s} (A_i A_i^T)_{ts} (G_i G_i^T)_{ts}.
    Not in the paper; an algebraic identity of the Frobenius norm."""
    A = _as3d(A)
    G = _as3d(G)
    B = A.shape[0]
    s = np.zeros(B, dtype=np.float64)
    for i in range(B):
        s[i] = np.sum((A[i] @ A[i].T) * (G[i] @ G[i].T))
    return s


def layer_sqnorm_dense_closed_form(A, G) -> np.ndarray:
    """T = 1 only: ||dL/dW||_F^2 = ||dL/dz||^2 ||h||^2 (Section 4)."""
    A = _as3d(A)
    G = _as3d(G)
    if A.shape[1] != 1:
        raise ValueError("closed form holds for T = 1 only")
    return np.sum(A[:, 0, :] ** 2, axis=1) * np.sum(G[:, 0, :] ** 2, axis=1)


def total_sqnorm(layers) -> np.ndarray:
    """Squared norm of the whole parameter gradient: the sum of the layers'
    squared norms (Section 5, paragraph before 5.1; weights only)."""
    s = None
    for A, G in layers:
        sl = layer_sqnorm(A, G)
        s = sl if s is None else s + sl
    return s


# --------------------------------------------------------------------------
# clipping
# --------------------------------------------------------------------------
def clip_factors(sqnorm: np.ndarray, C: float) -> np.ndarray:
    """nu_i with clip_c(z) = z / max(1, ||z||_2 / c) (Section 3.2), i.e.
    nu_i = 1 / max(1, ||g_i|| / C) = min(1, C / ||g_i||) (Eq. per_example_weight);
    a zero norm gives 1 through the max form."""
    n = np.sqrt(np.asarray(sqnorm, dtype=np.float64))
    return 1.0 / np.maximum(1.0, n / float(C))


def clipped_grad(A, G, clip: np.ndarray) -> np.ndarray:
    """sum_i nu_i g_i, [d_in, d_out]: the gradient of the re-weighted loss
    (Eq. weighted_loss) without the 1/tau factor, formed example by example."""
    A = _as3d(A)
    G = _as3d(G)
    out = np.zeros((A.shape[2], G.shape[2]), dtype=np.float64)
    for i in range(A.shape[0]):
        out += float(clip[i]) * per_example_grad(A[i], G[i])
    return out


def clipped_grad_by_clip_function(A, G, C: float, other_sq: np.ndarray | None = None) -> np.ndarray:
    """sum_i clip_C(g_i) written with the clip function itself rather than
    through nu_i; single layer unless other_sq carries the other layers'
    squared norms.  Used to pin clipped_grad against Section 3.2."""
    A = _as3d(A)
    G = _as3d(G)
    out = np.zeros((A.shape[2], G.shape[2]), dtype=np.float64)
    for i in range(A.shape[0]):
        M = per_example_grad(A[i], G[i])
        sq = np.sum(M * M) + (0.0 if other_sq is None else float(other_sq[i]))
        out += M / max(1.0, np.sqrt(sq) / float(C))
    return out


# --------------------------------------------------------------------------
# bias parameters
# --------------------------------------------------------------------------
def bias_rows(G) -> np.ndarray:
    """Per-example gradient of the layer's bias vector, [B, d_out]: dL/db = dL/dz for a
    fully-connected layer (Section 5.1) and the sum over positions, sum_t dL/dz^(t), when the
    bias is shared by T positions (Section 5.3; likewise over the output positions of a
    convolution)."""
    G = _as3d(G)
    out = np.zeros((G.shape[0], G.shape[2]), dtype=np.float64)
    for i in range(G.shape[0]):
        for t in range(G.shape[1]):
            out[i] += G[i, t]
    return out


def bias_sqnorm(G) -> np.ndarray:
    """s[i] = ||dL_i/db||^2: the bias's share of the squared gradient norm (Section 5,
    paragraph before 5.1: the norm runs over the weight matrix and the bias of every layer)."""
    u = bias_rows(G)
    return np.sum(u * u, axis=1)


def clipped_bias_grad(G, clip: np.ndarray) -> np.ndarray:
    """sum_i nu_i dL_i/db, [d_out] (Eq. weighted_loss applied to the bias)."""
    u = bias_rows(G)
    out = np.zeros(u.shape[1], dtype=np.float64)
    for i in range(u.shape[0]):
        out += float(clip[i]) * u[i]
    return out


# --------------------------------------------------------------------------
# LayerNorm parameters
# --------------------------------------------------------------------------
def layernorm_rows(G, Hbar):
    """Per-example gradients of a LayerNorm layer's scale and shift (Section 5.5, Algorithm 5):
    dL/dgamma = dL/dh (*) hbar (elementwise) and dL/dbeta = dL/dh, each summed over the T positions
    that share the two vectors.  G = dL/dh and Hbar = the normalised input, both [B, T, d].
    Returns (gamma_rows, beta_rows), each [B, d]."""
    G = _as3d(G)
    Hbar = _as3d(Hbar)
    gam = np.zeros((G.shape[0], G.shape[2]), dtype=np.float64)
    bet = np.zeros_like(gam)
    for i in range(G.shape[0]):
        for t in range(G.shape[1]):
            gam[i] += G[i, t] * Hbar[i, t]
            bet[i] += G[i, t]
    return gam, bet


def layernorm_sqnorm(G, Hbar) -> np.ndarray:
    """The layer's share of the squared gradient norm: ||dL_i/dgamma||^2 + ||dL_i/dbeta||^2."""
    gam, bet = layernorm_rows(G, Hbar)
    return np.sum(gam * gam, axis=1) + np.sum(bet * bet, axis=1)


def clipped_rows_sum(rows: np.ndarray, clip: np.ndarray) -> np.ndarray:
    """sum_i nu_i rows[i] for per-example gradient rows [B, d] (Eq. weighted_loss)."""
    out = np.zeros(rows.shape[1], dtype=np.float64)
    for i in range(rows.shape[0]):
        out += float(clip[i]) * rows[i]
    return out


# --------------------------------------------------------------------------
# convolution layers given by their input image
# --------------------------------------------------------------------------
def conv_unfold(X, KH: int, KW: int, pad: int) -> np.ndarray:
    """Patch matrix of a stride-1 convolution (the unfolding step of Algorithm 3):
    X[B, H, W, C] (channels last, zero padding `pad` on every side) ->
    A[B, H_out*W_out, KH*KW*C] with A[b, y*W_out + x, (kh*KW + kw)*C + c] = Xpad[b, y+kh, x+kw, c].
    With it the layer is the sequence layer of Eq. recurrent_gradient over the output positions
    (Section 5.2); the column order only fixes how the [KH*KW*C, d_out] gradient is read."""
    X = widen(np.asarray(X))
    B, H, W, C = X.shape
    Xp = np.zeros((B, H + 2 * pad, W + 2 * pad, C), dtype=np.float64)
    Xp[:, pad:pad + H, pad:pad + W, :] = X
    ho, wo = H + 2 * pad - KH + 1, W + 2 * pad - KW + 1
    A = np.zeros((B, ho * wo, KH * KW * C), dtype=np.float64)
    for y in range(ho):
        for x in range(wo):
            for kh in range(KH):
                for kw in range(KW):
                    A[:, y * wo + x, (kh * KW + kw) * C:(kh * KW + kw + 1) * C] = Xp[:, y + kh, x + kw, :]
    return A


# --------------------------------------------------------------------------
# path choice (host logic twin for tests)
# --------------------------------------------------------------------------
def gram_flops(T: int, d_in: int, d_out: int) -> int:
    """Multiply-add count x2 of the two Gram products using their symmetry
    (t <= s only)."""
    return T * (T + 1) * (d_in + d_out)


def direct_flops(T: int, d_in: int, d_out: int) -> int:
    return 2 * T * d_in * d_out


def choose_path(T: int, d_in: int, d_out: int) -> str:
    """'gram' iff it costs strictly fewer flops than materialising g_i."""
    return "gram" if gram_flops(T, d_in, d_out) < direct_flops(T, d_in, d_out) else "direct"


# --------------------------------------------------------------------------
# Gaussian noise: Philox4x32-10 counter stream + Box-Muller
# --------------------------------------------------------------------------
_PHILOX_M0 = 0xD2511F53
_PHILOX_M1 = 0xCD9E8D57
_PHILOX_W0 = 0x9E3779B9   # golden ratio
_PHILOX_W1 = 0xBB67AE85   # sqrt(3) - 1


def philox4x32_10(counter, key):
    """Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11) on Python
    integers.  counter = (c0, c1, c2, c3), key = (k0, k1); returns 4 words."""
    c0, c1, c2, c3 = (int(c) & _MASK32 for c in counter)
    k0, k1 = (int(k) & _MASK32 for k in key)
    for _ in range(10):
        p0 = _PHILOX_M0 * c0
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> 32, p0 & _MASK32
        hi1, lo1 = p1 >> 32, p1 & _MASK32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0) & _MASK32, lo1, (hi0 ^ c3 ^ k1) & _MASK32, lo0
        k0 = (k0 + _PHILOX_W0) & _MASK32
        k1 = (k1 + _PHILOX_W1) & _MASK32
    return c0, c1, c2, c3


def philox_words(n_counters: int, seed: int, first_counter: int) -> np.ndarray:
    """Vectorised form of the same rounds: words[q, 0..3] for the counters
    first_counter + q, with (c0, c1) = (low, high) word of the 64-bit counter,
    (c2, c3) = (0, 0) and key = (low, high) word of the seed."""
    q = (np.arange(n_counters, dtype=np.uint64) + np.uint64(first_counter))
    c0 = q & np.uint64(_MASK32)
    c1 = q >> np.uint64(32)
    c2 = np.zeros_like(q)
    c3 = np.zeros_like(q)
    k0 = int(seed) & _MASK32
    k1 = (int(seed) >> 32) & _MASK32
    m32 = np.uint64(_MASK32)
    for _ in range(10):
        p0 = np.uint64(_PHILOX_M0) * c0
        p1 = np.uint64(_PHILOX_M1) * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & m32
        hi1, lo1 = p1 >> np.uint64(32), p1 & m32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0)), lo1, (hi0 ^ c3 ^ np.uint64(k1)), lo0
        k0 = (k0 + _PHILOX_W0) & _MASK32
        k1 = (k1 + _PHILOX_W1) & _MASK32
    return np.stack([c0, c1, c2, c3], axis=1).astype(np.uint32)


def _uniform23(w: np.ndarray) -> np.ndarray:
    """Top 23 bits of a word -> the open interval (0, 1): (k + 1/2) / 2^23.
    Every value is exactly representable in float32 as well."""
    return ((w >> np.uint32(9)).astype(np.float64) + 0.5) * (2.0 ** -23)


def standard_normals(n: int, seed: int, offset: int) -> np.ndarray:
    """z[j], j in [0, n): element e = offset + j takes counter e >> 2 and slot
    e & 3.  Slots (0, 1) come from words (w0, w1), slots (2, 3) from
    (w2, w3), by Box-Muller: r = sqrt(-2 ln u_a), z_even = r cos(2 pi u_b),
    z_odd = r sin(2 pi u_b)."""
    if n <= 0:
        return np.zeros(0, dtype=np.float64)
    first = offset >> 2
    last = (offset + n - 1) >> 2
    w = philox_words(last - first + 1, seed, first)
    z = np.empty((w.shape[0], 4), dtype=np.float64)
    for pair in (0, 1):
        ua = _uniform23(w[:, 2 * pair])
        ub = _uniform23(w[:, 2 * pair + 1])
        r = np.sqrt(-2.0 * np.log(ua))
        z[:, 2 * pair] = r * np.cos(2.0 * np.pi * ub)
        z[:, 2 * pair + 1] = r * np.sin(2.0 * np.pi * ub)
    z = z.reshape(-1)
    start = offset - 4 * first
    return z[start:start + n]


def add_noise(grad: np.ndarray, stddev: float, seed: int, offset: int) -> np.ndarray:
    """grad + stddev * N(0, I) (the Gaussian mechanism lemma of Section 2 applied to the
    clipped sum, Algorithm 1's update line); returns a new float64 array."""
    g = np.asarray(grad, dtype=np.float64)
    z = standard_normals(g.size, seed, offset).reshape(g.shape)
    return g + float(stddev) * z


# --------------------------------------------------------------------------
# whole pipeline for one configuration
# --------------------------------------------------------------------------
def run_pipeline(layers, C: float, noise_std: float = 0.0, seed: int = 0):
    """layers: list of (A, G).  Returns (sqnorm[B], clip[B], [grad_l])."""
    s = total_sqnorm(layers)
    c = clip_factors(s, C)
    grads = []
    off = 0
    for A, G in layers:
        g = clipped_grad(A, G, c)
        if noise_std > 0.0:
            g = add_noise(g, noise_std, seed, off)
        off += g.size
        grads.append(g)
    return s, c, grads
