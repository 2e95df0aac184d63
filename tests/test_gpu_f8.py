"""Parity of the 8-bit (OCP e4m3 / e5m2) inputs of the HIP path against the CPU oracle.  Needs a real MI355X.

The oracle works on the stored bytes widened exactly to float64 (oracle f8_to_f64).  A product of two 8-bit values
has at most 8 significant bits, so it enters the fp32 accumulation exactly; what remains is the fp32 summation
(order and rounding) of the matrix unit and of the partial sums:
  squared norms   rel 2e-4
  clipped grad    rel Frobenius 2e-4
"""
import numpy as np
import pytest
import torch

from oracle import dp_oracle as orc
from paper_2009_03106_amd import workloads as wl

pytestmark = pytest.mark.gpu

SQ_TOL8 = 2e-4
FRO_TOL8 = 2e-4
TORCH8 = {"f8e4m3": torch.float8_e4m3fn, "f8e5m2": torch.float8_e5m2}
# G is drawn with a standard deviation of 1e-3: in e4m3 that lies below the normal range (2^-6), so it gets a
# loss scale; e5m2 reaches down to 2^-14
G_SCALE = {"f8e4m3": 256.0, "f8e5m2": 1.0, "f8": 1.0}
DTYPES = ["f8e4m3", "f8e5m2", "f8"]


@pytest.fixture(scope="module")
def dp():
    assert torch.cuda.is_available(), "GPU tests need a device"
    from paper_2009_03106_amd import dpclip
    dpclip.load_library()
    return dpclip


def to_dev8(bits: np.ndarray, store: str) -> torch.Tensor:
    assert bits.dtype == np.uint8
    return torch.from_numpy(bits).cuda().view(TORCH8[store])


def wide(bits: np.ndarray, store: str) -> np.ndarray:
    return orc.f8_to_f64(bits, store[2:])


def rel_err(got, ref) -> float:
    return float(np.max(np.abs(got.astype(np.float64) - ref) / np.maximum(np.abs(ref), 1e-300)))


def fro_err(got, ref) -> float:
    return float(np.linalg.norm(got.astype(np.float64) - ref) / max(np.linalg.norm(ref), 1e-300))


def draw(seed, B, T, d_in, d_out, dtype, g_std=1e-3):
    """One layer: A half zeros (post-ReLU), G Gaussian with per-example scales; stored bits, widened copies, device tensors."""
    rng = np.random.default_rng(seed)
    A = np.maximum(rng.standard_normal((B, T, d_in), dtype=np.float32), 0)
    G = rng.standard_normal((B, T, d_out), dtype=np.float32) * np.float32(g_std * G_SCALE[dtype])
    G *= (0.25 + 2.0 * rng.random((B, 1, 1), dtype=np.float32))
    sa, sg = wl.f8_formats(dtype)
    Ab, Gb = wl.f32_to_f8_bits(A, sa[2:]), wl.f32_to_f8_bits(G, sg[2:])
    return (wide(Ab, sa), wide(Gb, sg)), (to_dev8(Ab, sa), to_dev8(Gb, sg))


GRAM_SHAPES = [(3, 256, 256, 384), (2, 200, 128, 256), (2, 512, 768, 768), (4, 65, 128, 128), (5, 129, 384, 128)]
DIRECT_SHAPES = [(3, 128, 256, 256), (2, 192, 128, 384), (2, 112, 256, 128), (3, 64, 512, 256), (2, 168, 240, 256),
                 (9, 64, 1024, 768), (2, 320, 240, 128)]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", GRAM_SHAPES)
def test_f8_gram_sqnorm(dp, dtype, shape):
    B, T, d_in, d_out = shape
    (A, G), (Ad, Gd) = draw(11, B, T, d_in, d_out, dtype)
    ref = orc.layer_sqnorm(A, G)
    s = dp.layer_sqnorm(Ad, Gd, path="gram").cpu().numpy()
    assert rel_err(s, ref) <= SQ_TOL8, rel_err(s, ref)
    # accumulate on top of an earlier value
    base = torch.full((B,), 3.0, device="cuda")
    dp.layer_sqnorm(Ad, Gd, base, path="gram", accumulate=True)
    assert rel_err(base.cpu().numpy(), ref + 3.0) <= SQ_TOL8


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", DIRECT_SHAPES)
def test_f8_direct_sqnorm(dp, dtype, shape):
    B, T, d_in, d_out = shape
    (A, G), (Ad, Gd) = draw(12, B, T, d_in, d_out, dtype)
    ref = orc.layer_sqnorm(A, G)
    s = dp.layer_sqnorm(Ad, Gd, path="direct").cpu().numpy()
    assert rel_err(s, ref) <= SQ_TOL8, rel_err(s, ref)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", DIRECT_SHAPES + [(40, 256, 256, 256), (70, 64, 128, 128)])
def test_f8_clipped_grad(dp, dtype, shape):
    B, T, d_in, d_out = shape
    (A, G), (Ad, Gd) = draw(13, B, T, d_in, d_out, dtype)
    rng = np.random.default_rng(5)
    clip = np.where(rng.random(B) < 0.4, 1.0, 0.05 + 0.9 * rng.random(B)).astype(np.float32)
    ref = orc.clipped_grad(A, G, clip.astype(np.float64))
    c = torch.from_numpy(clip).cuda()
    g = dp.clipped_grad(Ad, Gd, c)
    assert fro_err(g.cpu().numpy(), ref) <= FRO_TOL8, fro_err(g.cpu().numpy(), ref)
    h = torch.full_like(g, 2.0)
    dp.clipped_grad(Ad, Gd, c, h, accumulate=True)
    np.testing.assert_array_equal(h.cpu().numpy(), g.cpu().numpy() + np.float32(2.0))


@pytest.mark.parametrize("shape", [(9, 64, 512, 256), (9, 128, 256, 256), (7, 168, 240, 256), (9, 40, 136, 128)])
def test_f8_zero_and_tiny_clip_factors(dp, shape):
    """Zero factors (masked examples, overflowed norms) and factors far below their neighbours at the first, a middle
    and the last example of a K slice: finite, and the weighted sum of the oracle."""
    B, T, d_in, d_out = shape
    (A, G), (Ad, Gd) = draw(15, B, T, d_in, d_out, "f8")
    rng = np.random.default_rng(B + T)
    base = (0.1 + 0.9 * rng.random(B)).astype(np.float32)
    pats = []
    for val in (0.0, 1e-30, 1e-45):
        a = base.copy(); a[[0, B // 2, B - 1]] = val; pats.append(a)
        b = base.copy(); b[1:3] = val; b[B - 3:B - 1] = val; pats.append(b)
    pats.append(np.zeros(B, dtype=np.float32))
    z = base.copy(); z[::2] = 0.0; pats.append(z)
    for clip in pats:
        ref = orc.clipped_grad(A, G, clip.astype(np.float64))
        scale = orc.clipped_grad(np.abs(A), np.abs(G), clip.astype(np.float64))
        got = dp.clipped_grad(Ad, Gd, torch.from_numpy(clip).cuda()).cpu().numpy()
        assert np.all(np.isfinite(got)), clip
        # 8-bit shapes outside their own kernels run widened through the fp16 kernels, which may re-round c * a
        # (the 64-deep 8-bit matrix instruction adds its products more coarsely than the 16-bit one: 2e-5 of the sum
        # of the terms' magnitudes has been seen per element, against 1e-6 for 16-bit inputs)
        unit = 2.0 ** -11 * 1.01 if dp.clipped_grad_rounds_inputs(B, T, d_in, d_out, dp.DP_F8_E4M3_E5M2) else 6e-5
        assert np.all(np.abs(got - ref) <= unit * scale + 1e-300), (clip, float(np.max(np.abs(got - ref) / (scale + 1e-300))))
        if not clip.any():
            assert not got.any()


def test_f8_all_ones_clip_is_the_plain_sum(dp):
    """c_i = 1: the clipped sum is A^T G over all B T rows, whatever the example boundaries."""
    (A, G), (Ad, Gd) = draw(14, 6, 128, 256, 256, "f8")
    g = dp.clipped_grad(Ad, Gd, torch.ones(6, device="cuda")).cpu().numpy()
    ref = A.reshape(-1, 256).T @ G.reshape(-1, 256)
    assert fro_err(g, ref) <= FRO_TOL8


@pytest.mark.parametrize("dtype,B", [("f8e4m3", 6), ("f8e5m2", 6), ("f8", 6), ("f8", 64)])
def test_f8_transformer_pipeline(dp, dtype, B):
    """The transformer configuration's four layers with 8-bit inputs through the several-layers calls: norms, clip
    factors, clipped sums and noise against the oracle's pipeline on the widened bytes; B = 64 is the configuration's
    full size, in the launch shapes that bench.py times."""
    w, layers = wl.generate("transformer", B=B, straddle=True, dtype=dtype, g_scale=G_SCALE[dtype])
    C = w.C * G_SCALE[dtype]
    sa, sg = wl.f8_formats(dtype)
    layers64 = [(wide(A, sa), wide(G, sg)) for A, G in layers]
    s_ref, c_ref, g_ref = orc.run_pipeline(layers64, C, w.noise_std, w.noise_seed)
    dev = [(to_dev8(A, sa), to_dev8(G, sg)) for A, G in layers]
    c = torch.empty(B, device="cuda")
    s = dp.layers_sqnorm(dev, C=C, clip=c)
    assert rel_err(s.cpu().numpy(), s_ref) <= SQ_TOL8
    assert rel_err(c.cpu().numpy(), c_ref) <= SQ_TOL8
    assert (c == 1.0).any() and (c < 1.0).any()
    sizes = [A.shape[-1] * G.shape[-1] for A, G in dev]
    starts = np.concatenate([[0], np.cumsum(sizes)]).tolist()
    flat = torch.zeros(sum(sizes), device="cuda")
    grads = [flat[starts[i]:starts[i + 1]].view(A.shape[-1], G.shape[-1]) for i, (A, G) in enumerate(dev)]
    descs = dp.layer_descs(dev, grads, starts[:-1])
    dp.layers_clipped_grad(dev, c, descs=descs, noise_std=w.noise_std, seed=w.noise_seed)
    for g, gr in zip(grads, g_ref):
        assert fro_err(g.cpu().numpy(), gr) <= FRO_TOL8
    # the layer-by-layer calls give the same numbers
    s1 = None
    for li, (A, G) in enumerate(dev):
        s1 = dp.layer_sqnorm(A, G, s1, accumulate=li > 0)
    assert rel_err(s1.cpu().numpy(), s_ref) <= SQ_TOL8


def test_f8_auto_takes_the_path_whose_kernels_fit(dp):
    """T = 128, 240 x 256: the flop rule says Gram, whose 8-bit kernel needs widths that are multiples of 128; the
    direct kernel takes multiples of 16.  T = 256, 128 x 128: the rule says direct and both fit."""
    (A, G), (Ad, Gd) = draw(15, 3, 128, 240, 256, "f8")
    assert dp.choose_path(128, 240, 256) == "gram"
    s_auto = dp.layer_sqnorm(Ad, Gd).cpu().numpy()
    s_dir = dp.layer_sqnorm(Ad, Gd, path="direct").cpu().numpy()
    np.testing.assert_array_equal(s_auto, s_dir)
    assert rel_err(s_auto, orc.layer_sqnorm(A, G)) <= SQ_TOL8
    # an explicit request for the Gram path is honoured through the fp16 kernels
    s_gram = dp.layer_sqnorm(Ad, Gd, path="gram").cpu().numpy()
    assert rel_err(s_gram, orc.layer_sqnorm(A, G)) <= SQ_TOL8


def test_f8_extreme_values(dp):
    """Largest finite values, subnormals and signed zeros of both formats go through the matrix unit exactly."""
    B, T, d = 2, 128, 128
    rng = np.random.default_rng(3)
    # e4m3 activations from the whole finite code range (NaN codes 0x7f / 0xff left out), scaled-down e5m2 gradients
    # from the subnormal and lowest normal codes
    Ab = rng.integers(0, 0x7F, size=(B, T, d), dtype=np.uint8) | (rng.integers(0, 2, size=(B, T, d), dtype=np.uint8) << 7)
    Gb = rng.integers(0, 0x10, size=(B, T, d), dtype=np.uint8) | (rng.integers(0, 2, size=(B, T, d), dtype=np.uint8) << 7)
    A, G = wide(Ab, "f8e4m3"), wide(Gb, "f8e5m2")
    assert np.isfinite(A).all() and np.abs(A).max() == 448.0 and 0 < np.abs(G[G != 0]).min() == 2.0 ** -16
    Ad, Gd = to_dev8(Ab, "f8e4m3"), to_dev8(Gb, "f8e5m2")
    ref = orc.layer_sqnorm(A, G)
    for path in ("gram", "direct"):
        s = dp.layer_sqnorm(Ad, Gd, path=path).cpu().numpy()
        assert rel_err(s, ref) <= SQ_TOL8, (path, rel_err(s, ref))
    g = dp.clipped_grad(Ad, Gd, torch.ones(B, device="cuda")).cpu().numpy()
    assert fro_err(g, orc.clipped_grad(A, G, np.ones(B))) <= FRO_TOL8


# shapes outside the 8-bit kernels: dense layers, widths that are not multiples of 16, short or very ragged T
WIDENED_SHAPES = [(32, 1, 64, 32), (7, 1, 784, 512), (3, 128, 136, 128), (5, 32, 256, 256), (2, 70, 100, 60), (4, 20, 48, 33)]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", WIDENED_SHAPES)
def test_f8_other_shapes_run_widened(dp, dtype, shape):
    """Shapes that the 8-bit kernels do not take are widened to fp16 (exactly) inside the workspace and run through
    the fp16 kernels: same results against the oracle, a larger workspace."""
    B, T, d_in, d_out = shape
    (A, G), (Ad, Gd) = draw(21, B, T, d_in, d_out, dtype)
    code = dp._dtype_code(Ad, Gd)
    for path in ("auto", "gram", "direct"):
        s = dp.layer_sqnorm(Ad, Gd, path=path).cpu().numpy()
        assert rel_err(s, orc.layer_sqnorm(A, G)) <= SQ_TOL8, (path, rel_err(s, orc.layer_sqnorm(A, G)))
    need = dp.workspace_bytes(dp.DP_OP_SQNORM, B, T, d_in, d_out, code)
    assert need >= 2 * B * T * (d_in + d_out) + dp.workspace_bytes(dp.DP_OP_SQNORM, B, T, d_in, d_out, dp.DP_F16)
    rng = np.random.default_rng(6)
    clip = (0.1 + 0.9 * rng.random(B)).astype(np.float32)
    g = dp.clipped_grad(Ad, Gd, torch.from_numpy(clip).cuda()).cpu().numpy()
    # the fp16 kernels for these shapes re-round c_i * a to fp16: at most 2^-11 relative per element
    assert fro_err(g, orc.clipped_grad(A, G, clip.astype(np.float64))) <= 2e-3
    # bit for bit what the fp16 entry points give on the widened values
    A16 = torch.from_numpy(A.astype(np.float16)).cuda()
    G16 = torch.from_numpy(G.astype(np.float16)).cuda()
    assert np.array_equal(A16.cpu().numpy().astype(np.float64), A) and np.array_equal(G16.cpu().numpy().astype(np.float64), G)
    np.testing.assert_array_equal(dp.layer_sqnorm(Ad, Gd).cpu().numpy(), dp.layer_sqnorm(A16, G16).cpu().numpy())
    np.testing.assert_array_equal(g, dp.clipped_grad(A16, G16, torch.from_numpy(clip).cuda()).cpu().numpy())
    # too small a workspace is refused
    lib = dp.load_library()
    ws = torch.empty(max(16, need - 16), dtype=torch.uint8, device="cuda")
    sq = torch.zeros(B, device="cuda")
    assert lib.dp_layer_sqnorm(Ad.data_ptr(), Gd.data_ptr(), B, T, d_in, d_out, code, 0, 0, sq.data_ptr(), ws.data_ptr(),
                               need - 16, None) == dp.DP_ERR_WORKSPACE


@pytest.mark.parametrize("dtype", DTYPES)
def test_f8_mixed_layers_call(dp, dtype):
    """A model with dense layers, an aligned and an unaligned sequence layer in one several-layers call."""
    shapes = [(1, 784, 512), (256, 256, 384), (1, 512, 10), (100, 72, 40), (128, 512, 128)]
    B = 5
    wides, devs = [], []
    for k, (T, di, do) in enumerate(shapes):
        w, d = draw(30 + k, B, T, di, do, dtype)
        wides.append(w); devs.append(d)
    s_ref = orc.total_sqnorm(wides)
    C = float(np.sqrt(np.median(s_ref)))
    c = torch.empty(B, device="cuda")
    s = dp.layers_sqnorm(devs, C=C, clip=c)
    assert rel_err(s.cpu().numpy(), s_ref) <= SQ_TOL8
    c_ref = orc.clip_factors(s_ref, C)
    assert rel_err(c.cpu().numpy(), c_ref) <= SQ_TOL8
    grads = dp.layers_clipped_grad(devs, c)
    for (A, G), g in zip(wides, grads):
        assert fro_err(g.cpu().numpy(), orc.clipped_grad(A, G, c.cpu().numpy().astype(np.float64))) <= 2e-3


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", [(3, 256, 384), (2, 100, 136), (5, 1, 512), (4, 513, 48), (2, 37, 33)])
def test_f8_bias_and_layernorm_rows(dp, dtype, shape):
    """Bias rows sum_t G_i[t] and LayerNorm rows sum_t G_i[t] * Hbar_i[t] from 8-bit inputs (Hbar stored like A),
    their squared norms, and the clipped bias sum, for widths with and without whole 16-byte pieces."""
    B, T, d = shape
    (H, G), (Hd, Gd) = draw(41, B, T, d, d, dtype)
    u_ref = orc.bias_rows(G)
    rows = torch.empty((B, d), device="cuda")
    s, _ = dp.bias_sqnorm(Gd, None, rows)
    assert np.max(np.abs(rows.cpu().numpy() - u_ref)) <= 1e-6 * np.max(np.sum(np.abs(G), axis=1))
    assert rel_err(s.cpu().numpy(), orc.bias_sqnorm(G)) <= 1e-5 or np.all(np.abs(s.cpu().numpy() - orc.bias_sqnorm(G)) <= 1e-12)
    gam_ref, bet_ref = orc.layernorm_rows(G, H)
    out = dp.layernorm_sqnorm(Gd, Hd)
    s2, gam, bet = out
    scale = np.max(np.sum(np.abs(G * H), axis=1)) + 1e-300
    assert np.max(np.abs(gam.cpu().numpy() - gam_ref)) <= 1e-6 * scale
    assert np.max(np.abs(bet.cpu().numpy() - bet_ref)) <= 1e-6 * np.max(np.sum(np.abs(G), axis=1))
    ref2 = orc.layernorm_sqnorm(G, H)
    assert np.all(np.abs(s2.cpu().numpy() - ref2) <= 1e-5 * ref2 + 1e-12)
    clip = torch.rand(B, device="cuda")
    gb = dp.clipped_bias_grad(rows, clip).cpu().numpy()
    assert np.max(np.abs(gb - orc.clipped_bias_grad(G, clip.cpu().numpy().astype(np.float64)))) <= 1e-5 * np.max(np.abs(u_ref)) * B


@pytest.mark.parametrize("dtype", DTYPES)
def test_f8_layers_call_with_bias_rows(dp, dtype):
    """Weights and biases of several 8-bit layers clipped together in one norm call (the bias rows of 8-bit layers
    are taken in a pass of their own)."""
    shapes = [(256, 256, 384), (1, 512, 64), (100, 72, 40)]
    B = 4
    wides, devs = [], []
    for k, (T, di, do) in enumerate(shapes):
        w, d = draw(50 + k, B, T, di, do, dtype)
        wides.append(w); devs.append(d)
    rows = [torch.empty((B, do), device="cuda") for _, _, do in shapes]
    descs = dp.layer_descs(devs, bias_rows=rows)
    s = dp.layers_sqnorm(devs, descs=descs)
    ref = orc.total_sqnorm(wides) + sum(orc.bias_sqnorm(G) for _, G in wides)
    assert rel_err(s.cpu().numpy(), ref) <= SQ_TOL8
    for (_, G), u in zip(wides, rows):
        assert np.max(np.abs(u.cpu().numpy() - orc.bias_rows(G))) <= 1e-6 * np.max(np.sum(np.abs(G), axis=1))


@pytest.mark.parametrize("dtype", DTYPES)
def test_f8_conv_from_image_runs_widened(dp, dtype):
    """The convolution given by its image takes 8-bit inputs by widening them to fp16 in the workspace: results
    against the oracle's unfolding, and bit for bit the DP_F16 call on the widened values."""
    B, H, W, C, d_out, KH, KW, pad = 3, 16, 16, 64, 128, 3, 3, 1
    rng = np.random.default_rng(61)
    X = np.maximum(rng.standard_normal((B, H, W, C), dtype=np.float32), 0)
    G = rng.standard_normal((B, H * W, d_out), dtype=np.float32) * np.float32(1e-3 * G_SCALE[dtype])
    sa, sg = wl.f8_formats(dtype)
    Xb, Gb = wl.f32_to_f8_bits(X, sa[2:]), wl.f32_to_f8_bits(G, sg[2:])
    Xw, Gw = wide(Xb, sa), wide(Gb, sg)
    Xd, Gd = to_dev8(Xb, sa), to_dev8(Gb, sg)
    A = orc.conv_unfold(Xw, KH, KW, pad)
    s = dp.conv_sqnorm(Xd, Gd, KH, KW, pad)
    assert rel_err(s.cpu().numpy(), orc.layer_sqnorm(A, Gw)) <= SQ_TOL8
    clip = torch.tensor([1.0, 0.3, 0.7], device="cuda")
    g = dp.conv_clipped_grad(Xd, Gd, clip, KH, KW, pad)
    assert fro_err(g.cpu().numpy(), orc.clipped_grad(A, Gw, clip.cpu().numpy().astype(np.float64))) <= FRO_TOL8
    X16, G16 = torch.from_numpy(Xw.astype(np.float16)).cuda(), torch.from_numpy(Gw.astype(np.float16)).cuda()
    np.testing.assert_array_equal(s.cpu().numpy(), dp.conv_sqnorm(X16, G16, KH, KW, pad).cpu().numpy())
    np.testing.assert_array_equal(g.cpu().numpy(), dp.conv_clipped_grad(X16, G16, clip, KH, KW, pad).cpu().numpy())


def test_f8_unsupported_is_reported(dp):
    """A convolution geometry that the image kernels do not take stays DP_ERR_UNSUPPORTED for 8-bit inputs too
    (here 12 channels: whole 16-byte pieces must stay inside one pixel), before anything is launched."""
    X = torch.zeros((2, 16, 16, 12), dtype=torch.uint8, device="cuda").view(torch.float8_e4m3fn)
    Gc = torch.zeros((2, 256, 128), dtype=torch.uint8, device="cuda").view(torch.float8_e4m3fn)
    s = torch.full((2,), 7.0, device="cuda")
    with pytest.raises(dp.DpclipError) as ei:
        dp.conv_sqnorm(X, Gc, 3, 3, 1, s)
    assert ei.value.status == dp.DP_ERR_UNSUPPORTED
    with pytest.raises(dp.DpclipError) as ei:
        dp.conv_clipped_grad(X, Gc, torch.ones(2, device="cuda"), 3, 3, 1)
    assert ei.value.status == dp.DP_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert torch.all(s == 7.0)


def test_f8_empty_problems_and_argument_errors(dp):
    """Empty sizes are valid and zero-fill; misaligned inputs and a short workspace are refused before any launch."""
    lib = dp.load_library()
    code = dp.DP_F8_E4M3_E5M2
    e4, e5 = torch.float8_e4m3fn, torch.float8_e5m2
    z = lambda *shape: torch.zeros(shape, dtype=torch.uint8, device="cuda")
    # T = 0 and d_in = 0: zero norms, zero gradient
    s = dp.layer_sqnorm(z(3, 0, 128).view(e4), z(3, 0, 128).view(e5))
    assert torch.all(s == 0)
    s = torch.full((3,), 5.0, device="cuda")
    dp.layer_sqnorm(z(3, 128, 0).view(e4), z(3, 128, 128).view(e5), s)
    assert torch.all(s == 0)
    g = dp.clipped_grad(z(3, 0, 128).view(e4), z(3, 0, 256).view(e5), torch.ones(3, device="cuda"))
    assert g.shape == (128, 256) and torch.all(g == 0)
    # B = 0: nothing to do
    assert lib.dp_layer_sqnorm(None, None, 0, 128, 128, 128, code, 0, 0, None, None, 0, None) == dp.DP_OK
    # zeros in, zeros out through the 8-bit kernels (negative zeros included)
    A = torch.full((2, 128, 128), 0x80, dtype=torch.uint8, device="cuda").view(e4)
    G = z(2, 128, 128).view(e5)
    assert torch.all(dp.layer_sqnorm(A, G, path="gram") == 0) and torch.all(dp.layer_sqnorm(A, G, path="direct") == 0)
    assert torch.all(dp.clipped_grad(A, G, torch.ones(2, device="cuda")) == 0)
    # misaligned A
    buf = z(2 * 128 * 128 + 16)
    need = dp.workspace_bytes(dp.DP_OP_SQNORM, 2, 128, 128, 128, code)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    sq = torch.full((2,), 9.0, device="cuda")
    assert lib.dp_layer_sqnorm(buf.data_ptr() + 8, G.data_ptr(), 2, 128, 128, 128, code, 0, 0, sq.data_ptr(), ws.data_ptr(), ws.numel(),
                               None) == dp.DP_ERR_INVALID_ARG
    # the 8-bit kernels' own scratch: one float per example and tile pair, refused when short
    assert need == 2 * 1 * 4
    assert lib.dp_layer_sqnorm(A.data_ptr(), G.data_ptr(), 2, 128, 128, 128, code, 0, 0, sq.data_ptr(), ws.data_ptr(), need - 4,
                               None) == dp.DP_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert torch.all(sq == 9.0)


def test_f8_step_with_groups_and_biases_is_graph_capturable(dp):
    """A step on 8-bit inputs with per-layer clipping, bias rows (their own pass for 8-bit layers), a widened layer,
    clipped sums of weights and biases and fused noise, captured into a HIP graph: every replay (with eager work in
    between) reproduces the eager results bit for bit."""
    B = 4
    shapes = [(256, 256, 384), (128, 136, 128), (192, 128, 256)]           # the second one runs widened to fp16
    devs = [draw(70 + k, B, T, di, do, "f8")[1] for k, (T, di, do) in enumerate(shapes)]
    m = len(devs)
    sq = [torch.zeros(B, device="cuda") for _ in range(m)]
    cl = [torch.zeros(B, device="cuda") for _ in range(m)]
    rows = [torch.zeros((B, do), device="cuda") for _, _, do in shapes]
    sizes = [di * do + do for _, di, do in shapes]
    starts = np.concatenate([[0], np.cumsum(sizes)]).tolist()
    flat = torch.zeros(sum(sizes), device="cuda")
    grads = [flat[starts[i]:starts[i] + di * do].view(di, do) for i, (_, di, do) in enumerate(shapes)]
    gbs = [flat[starts[i] + di * do:starts[i + 1]] for i, (_, di, do) in enumerate(shapes)]
    groups = [(sq[l], cl[l], 0.05) for l in range(m)]
    d1 = dp.layer_descs(devs, bias_rows=rows, groups=groups)
    d2 = dp.layer_descs(devs, grads, starts[:-1], bias_rows=rows, groups=groups, grad_bs=gbs,
                        bias_noise_offsets=[starts[i] + di * do for i, (_, di, do) in enumerate(shapes)])
    ws1 = torch.empty(max(16, dp.layers_workspace_bytes(d1[0], B, d1[2])), dtype=torch.uint8, device="cuda")
    ws2 = torch.empty(max(16, dp.layers_clipped_workspace_bytes(d2[0], B, d2[2])), dtype=torch.uint8, device="cuda")
    unused = torch.zeros(B, device="cuda")

    def step():
        dp.layers_sqnorm(devs, unused, workspace=ws1, descs=d1)
        dp.layers_clipped_grad(devs, None, workspace=ws2, descs=d2, noise_std=0.25, seed=5)

    outs = sq + cl + rows + [flat]
    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in outs]
    assert all((c > 0).all() and (c <= 1).all() for c in cl) and any((c < 1).any() for c in cl)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in outs:
            t.fill_(-1.0)
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(outs, want):
            assert torch.equal(got, ref), rep
        _ = torch.randn(1 << 18, device="cuda").sum().item()        # eager work and a synchronisation between replays
