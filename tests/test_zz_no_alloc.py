"""dp_layer_sqnorm_static (the entry point for callers that cannot allocate) against dp_layer_sqnorm, through the
C-ABI: same kernels, so the results must be equal bit for bit; two calls in a row share the static scratch array, the
second one smaller than the first (stale partial sums of the first call must not leak into it).  Needs a real MI355X."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import dp_oracle as orc
from paper_2009_03106_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dp():
    assert torch.cuda.is_available(), "GPU tests need a device"
    from paper_2009_03106_amd import dpclip
    dpclip.load_library()
    return dpclip


def to_dev(x):
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(x).cuda()


def both(dp, lib, A, G, path, dtype_code, accumulate=False, start=0.0):
    """(result of dp_layer_sqnorm with a workspace of its own, result of dp_layer_sqnorm_static), raw C-ABI calls."""
    Ad, Gd = to_dev(A), to_dev(G)
    B, T, d_in = A.shape
    d_out = G.shape[-1]
    pc = {"auto": dp.DP_PATH_AUTO, "gram": dp.DP_PATH_GRAM, "direct": dp.DP_PATH_DIRECT}[path]
    need = lib.dp_workspace_bytes(dp.DP_OP_SQNORM, B, T, d_in, d_out, dtype_code, pc)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    want = torch.full((B,), start, dtype=torch.float32, device="cuda")
    got = torch.full((B,), start, dtype=torch.float32, device="cuda")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    st = lib.dp_layer_sqnorm(Ad.data_ptr(), Gd.data_ptr(), B, T, d_in, d_out, dtype_code, pc, int(accumulate),
                             want.data_ptr(), ws.data_ptr(), ws.numel(), stream)
    assert st == dp.DP_OK, dp.status_string(st)
    st = lib.dp_layer_sqnorm_static(Ad.data_ptr(), Gd.data_ptr(), B, T, d_in, d_out, dtype_code, pc, int(accumulate),
                                    got.data_ptr(), stream)
    assert st == dp.DP_OK, dp.status_string(st)
    torch.cuda.synchronize()
    return want.cpu().numpy(), got.cpu().numpy()


@pytest.mark.parametrize("dtype,code", [("bf16", 1), ("f32", 0)])
@pytest.mark.parametrize("path", ["gram", "direct"])
def test_static_scratch_two_calls_in_a_row(dp, dtype, code, path):
    lib = dp.load_library()
    # first call: several tile pairs / output tiles per example and a ragged tail; second call: fewer examples,
    # shorter sequences, narrower layer, so it uses a prefix of the scratch the first call filled
    for seed, (B, T, d_in, d_out) in enumerate([(6, 300, 256, 192), (3, 130, 128, 64)]):
        A, G = wl.random_layer(500 + seed, B, T, d_in, d_out, dtype)
        want, got = both(dp, lib, A, G, path, code)
        np.testing.assert_array_equal(got, want)
        ref = orc.layer_sqnorm(A, G)
        tol = 1e-5 if dtype == "f32" else 2e-4
        assert np.max(np.abs(got - ref) / ref) <= tol
    # accumulate on top of an earlier value, and a dense layer (needs no scratch at all)
    A, G = wl.random_layer(502, 4, 96, 72, 40, dtype)
    want, got = both(dp, lib, A, G, path, code, accumulate=True, start=2.5)
    np.testing.assert_array_equal(got, want)
    A, G = wl.random_layer(503, 5, 1, 130, 67, dtype)
    want, got = both(dp, lib, A, G, "auto", code)
    np.testing.assert_array_equal(got, want)


def test_static_scratch_limit_and_errors(dp):
    lib = dp.load_library()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    out = torch.full((4,), 7.0, device="cuda")
    # a problem whose partial sums exceed the static array is refused before anything is launched: made-up, aligned
    # input addresses are never touched.  B * npairs * 4 bytes with 128-row Gram tiles: T = 8192 -> 2080 pairs.
    B, T, d = 1024, 8192, 256
    assert lib.dp_workspace_bytes(dp.DP_OP_SQNORM, B, T, d, d, dp.DP_BF16, dp.DP_PATH_GRAM) > dp.STATIC_SCRATCH_BYTES
    big = torch.empty(B, device="cuda")
    st = lib.dp_layer_sqnorm_static(0x10000000, 0x20000000, B, T, d, d, dp.DP_BF16, dp.DP_PATH_GRAM, 0, big.data_ptr(), stream)
    assert st == dp.DP_ERR_WORKSPACE
    # argument errors as in dp_layer_sqnorm
    assert lib.dp_layer_sqnorm_static(None, None, 4, 64, 64, 64, dp.DP_BF16, dp.DP_PATH_GRAM, 0, out.data_ptr(), stream) == dp.DP_ERR_INVALID_ARG
    assert lib.dp_layer_sqnorm_static(None, None, -1, 64, 64, 64, dp.DP_BF16, dp.DP_PATH_GRAM, 0, out.data_ptr(), stream) == dp.DP_ERR_INVALID_ARG
    # an empty problem zero-fills
    assert lib.dp_layer_sqnorm_static(None, None, 4, 0, 64, 64, dp.DP_BF16, dp.DP_PATH_AUTO, 0, out.data_ptr(), stream) == dp.DP_OK
    torch.cuda.synchronize()
    assert not out.cpu().numpy().any()
