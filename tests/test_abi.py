"""The C-ABI library loads and exports every symbol the header declares; host-only
entry points (path choice, workspace sizes, status strings) behave as documented.
No kernel is launched here."""
import ctypes
import os
import re

import pytest

from oracle import dp_oracle as orc
from paper_2009_03106_amd import dpclip, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(dpclip.LIB_PATH):
        from paper_2009_03106_amd import build
        build.build_library()
    return dpclip.load_library()


def declared_symbols(header="dpclip.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dp_[a-z_]+)\s*\(", text)))


def test_exports_match_header(lib):
    syms = declared_symbols()
    assert set(syms) == set(dpclip.EXPORTS)
    for s in syms:
        assert getattr(lib, s) is not None
    probes = declared_symbols("dpclip_probes.h")
    assert set(probes) == set(dpclip.PROBE_EXPORTS)
    for s in probes:
        assert getattr(lib, s) is not None
    # every header under include/ is covered here
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["dpclip.h", "dpclip_probes.h"]


def test_status_strings(lib):
    seen = {dpclip.status_string(i) for i in range(5)}
    assert len(seen) == 5 and all(seen)
    assert dpclip.status_string(99)


def test_choose_path_matches_flop_model(lib):
    for w in wl.WORKLOADS.values():
        for spec in w.layers:
            if spec.T > 1:
                assert dpclip.choose_path(spec.T, spec.d_in, spec.d_out) == orc.choose_path(spec.T, spec.d_in, spec.d_out)
    for T in (2, 3, 8, 63, 64, 65, 500, 4096):
        for d_in in (1, 7, 64, 577, 4096):
            for d_out in (1, 10, 128, 3072):
                assert dpclip.choose_path(T, d_in, d_out) == orc.choose_path(T, d_in, d_out), (T, d_in, d_out)
    assert dpclip.choose_path(1024, 576, 128) == "direct"
    assert dpclip.choose_path(512, 768, 768) == "gram"


def test_workspace_sizes(lib):
    f = dpclip.workspace_bytes
    assert f(dpclip.DP_OP_SQNORM, 256, 1, 784, 512, dpclip.DP_F32) == 0          # T = 1 needs none
    assert f(dpclip.DP_OP_SQNORM, 0, 64, 256, 256, dpclip.DP_BF16) == 0
    assert f(dpclip.DP_OP_SQNORM, -1, 64, 256, 256, dpclip.DP_BF16) == 0
    g = f(dpclip.DP_OP_SQNORM, 64, 512, 768, 768, dpclip.DP_BF16, "gram")
    d = f(dpclip.DP_OP_SQNORM, 64, 512, 768, 768, dpclip.DP_BF16, "direct")
    assert g > 0 and d > 0 and g % 4 == 0 and d % 4 == 0
    assert f(dpclip.DP_OP_SQNORM, 64, 512, 768, 768, dpclip.DP_BF16, "auto") == g
    c = f(dpclip.DP_OP_CLIPPED_GRAD, 64, 512, 768, 2304, dpclip.DP_BF16)
    assert c % (768 * 2304 * 4) == 0 and c >= 768 * 2304 * 4
    assert f(dpclip.DP_OP_CLIPPED_GRAD, 1, 1, 8, 8, dpclip.DP_F32) == 0          # one K slice: no scratch


def test_workspace_sizes_over_many_shapes(lib):
    """Host logic only: the size queries answer for every shape class without crashing, are multiples of 4, hold at
    least one float per example for the norm scratch, and reject what the entry points reject."""
    f = dpclip.workspace_bytes
    shapes = [(1, 1, 1, 1), (3, 17, 72, 40), (64, 197, 768, 3072), (64, 200, 256, 256), (128, 64, 256, 256),
              (128, 1024, 576, 128), (2, 4096, 64, 128), (1, 100000, 64, 64), (1 << 16, 8, 8, 8), (7, 33, 129, 65),
              (4, 64, 4096, 4096), (2, 96, 192, 256), (5, 161, 192, 128)]
    for B, T, di, do in shapes:
        for dt in (dpclip.DP_F32, dpclip.DP_BF16):
            for path in ("auto", "gram", "direct"):
                n = f(dpclip.DP_OP_SQNORM, B, T, di, do, dt, path)
                assert n >= 0 and n % 4 == 0 and n < (1 << 40), (B, T, di, do, dt, path, n)
                if T > 1:
                    assert n >= 4 * B, (B, T, di, do, dt, path, n)
            n = f(dpclip.DP_OP_CLIPPED_GRAD, B, T, di, do, dt)
            assert n >= 0 and n % 4 == 0 and n < (1 << 40)
        # fp16 runs through the bf16 plans: the same scratch for every operation and path
        for path in ("auto", "gram", "direct"):
            assert f(dpclip.DP_OP_SQNORM, B, T, di, do, dpclip.DP_F16, path) == f(dpclip.DP_OP_SQNORM, B, T, di, do, dpclip.DP_BF16, path)
        assert f(dpclip.DP_OP_CLIPPED_GRAD, B, T, di, do, dpclip.DP_F16) == f(dpclip.DP_OP_CLIPPED_GRAD, B, T, di, do, dpclip.DP_BF16)
        # 8-bit inputs: either the 8-bit kernels' own scratch, or the fp16 scratch behind the two widened inputs
        r256 = lambda n: (n + 255) // 256 * 256
        for dt8 in (dpclip.DP_F8_E4M3, dpclip.DP_F8_E5M2, dpclip.DP_F8_E4M3_E5M2):
            widened = r256(2 * B * T * di) + r256(2 * B * T * do)
            for path in ("auto", "gram", "direct"):
                n = f(dpclip.DP_OP_SQNORM, B, T, di, do, dt8, path)
                assert n % 4 == 0 and (n >= 4 * B or T == 1)
                assert n <= widened or n == widened + f(dpclip.DP_OP_SQNORM, B, T, di, do, dpclip.DP_F16, path), (B, T, di, do, path)
            n = f(dpclip.DP_OP_CLIPPED_GRAD, B, T, di, do, dt8)
            assert n % 4 == 0 and (n <= widened or n == widened + f(dpclip.DP_OP_CLIPPED_GRAD, B, T, di, do, dpclip.DP_F16))
    assert f(dpclip.DP_OP_SQNORM, 64, 512, 768, 768, dpclip.DP_F8_E4M3_E5M2, "gram") == f(dpclip.DP_OP_SQNORM, 64, 512, 768, 768, dpclip.DP_BF16, "gram")
    assert f(dpclip.DP_OP_SQNORM, 3, 17, 72, 40, dpclip.DP_F8_E4M3) == 7424 + 4096 + f(dpclip.DP_OP_SQNORM, 3, 17, 72, 40, dpclip.DP_F16)
    assert f(dpclip.DP_OP_SQNORM, 4, 64, 64, 64, 6) == 0                                       # unknown dtype
    # a ragged sequence length on the copy-pipeline kernels sets aside a line of zeros even without K slices
    assert f(dpclip.DP_OP_CLIPPED_GRAD, 1, 197, 768, 768, dpclip.DP_BF16) >= 256
    # too large: B * T must stay below 2^31, layer widths below 2^24
    assert f(dpclip.DP_OP_SQNORM, 1 << 20, 1 << 12, 64, 64, dpclip.DP_BF16) == 0
    assert f(dpclip.DP_OP_CLIPPED_GRAD, 2, 64, 1 << 24, 64, dpclip.DP_BF16) == 0
    g = dpclip.conv_workspace_bytes
    assert g(dpclip.DP_OP_SQNORM, 128, 32, 32, 64, 3, 3, 1, 128, dpclip.DP_BF16) >= 256 + 4 * 128
    assert g(dpclip.DP_OP_CLIPPED_GRAD, 128, 32, 32, 64, 3, 3, 1, 128, dpclip.DP_BF16) >= 256
    assert g(dpclip.DP_OP_SQNORM, 128, 32, 32, 64, 3, 3, 1, 128, dpclip.DP_F16) == g(dpclip.DP_OP_SQNORM, 128, 32, 32, 64, 3, 3, 1, 128, dpclip.DP_BF16)
    assert g(dpclip.DP_OP_SQNORM, 128, 32, 32, 64, 3, 3, 1, 128, dpclip.DP_F32) == 0        # 16-bit inputs only
    assert g(dpclip.DP_OP_SQNORM, 128, 32, 32, 60, 3, 3, 1, 128, dpclip.DP_BF16) == 0       # C % 8 != 0
    assert g(dpclip.DP_OP_SQNORM, 128, 2, 2, 64, 3, 3, 0, 128, dpclip.DP_BF16) == 0         # kernel larger than the image
    assert g(dpclip.DP_OP_SQNORM, 128, 32, 32, 64, 0, 3, 1, 128, dpclip.DP_BF16) == 0


def test_layers_workspace_sizes(lib):
    """Host logic of the several-layers call: the copy-pipeline Gram layers of one launch (at most 16) have their partial
    sums side by side, the layers that run one by one each have what dp_layer_sqnorm needs, side by side too (one launch
    folds them at the end), and the two groups share the space."""
    import ctypes
    def descs(shapes):
        arr = (dpclip.LayerDesc * len(shapes))()
        for i, (T, di, do) in enumerate(shapes):
            arr[i] = dpclip.LayerDesc(None, None, T, di, do)
        return arr
    f = dpclip.layers_workspace_bytes
    tr = descs([(512, 768, 2304), (512, 768, 768), (512, 768, 3072), (512, 3072, 768)])
    assert f(tr, 64, dpclip.DP_BF16) == 4 * 64 * 10 * 4                  # 10 pairs of 128-row tiles per example and layer
    assert f(tr, 64, dpclip.DP_F16) == f(tr, 64, dpclip.DP_BF16)
    assert f(tr, 64, dpclip.DP_F32) == 4 * 64 * 36 * 4                    # fp32 Gram: 8 tiles of 64 rows, 36 pairs, four layers
    assert f(tr, 64, dpclip.DP_F32, "direct") == sum((dpclip.workspace_bytes(dpclip.DP_OP_SQNORM, 64, *sh, dpclip.DP_F32, "direct") + 15) // 16 * 16
                                            for sh in [(512, 768, 2304), (512, 768, 768), (512, 768, 3072), (512, 3072, 768)])
    assert f(tr, 64, dpclip.DP_F32, "gram") == 4 * 64 * 36 * 4
    assert f(descs([(512, 768, 2304)]), 64, dpclip.DP_F32) == 64 * 36 * 4
    # few positions, wide rows, small batch (16-bit): the shared column-split Gram launch keeps every layer's shares
    cols = descs([(16, 4608, 512), (16, 2304, 512), (64, 2304, 256)])
    one = [dpclip.workspace_bytes(dpclip.DP_OP_SQNORM, 32, *sh, dpclip.DP_BF16, "gram") for sh in [(16, 4608, 512), (16, 2304, 512), (64, 2304, 256)]]
    assert all(n > 32 * 4 for n in one)
    assert f(cols, 32, dpclip.DP_BF16, "gram") == max(one[0] + one[1], one[2])     # T <= 32 and T <= 64 in launches of their own
    wb = descs([(512, 768, 2304), (512, 768, 768)])
    wb[0].bias_rows = 16                    # any non-null value: only the sizes are looked at
    assert f(wb, 64, dpclip.DP_BF16) == 2 * 64 * 10 * 4 + 64 * 4 * 2304 * 4     # + column sums per 128-row tile
    many = descs([(128, 64, 64)] * 20)
    assert f(many, 8, dpclip.DP_BF16, "gram") == 16 * 8 * 1 * 4           # launches of 16 and 4 layers reuse the space
    mixed = descs([(1, 64, 32), (1024, 576, 128), (0, 8, 8)])
    assert f(mixed, 128, dpclip.DP_BF16) == (dpclip.workspace_bytes(dpclip.DP_OP_SQNORM, 128, 1024, 576, 128, dpclip.DP_BF16) + 15) // 16 * 16
    # at 16 examples the shared copy-pipeline launch of direct norms can take that layer: one sum per example and 128 x 128
    # tile (5 tiles), at least its own call's need (3 tiles of 192 x 128)
    assert f(mixed, 16, dpclip.DP_BF16) == 16 * 5 * 4 >= (dpclip.workspace_bytes(dpclip.DP_OP_SQNORM, 16, 1024, 576, 128, dpclip.DP_BF16) + 15) // 16 * 16
    assert f(descs([(512, 1 << 24, 64)]), 2, dpclip.DP_BF16) == 0         # width out of range
    # the clipped sums of several layers run one after the other and share the largest layer's scratch ...
    h = dpclip.layers_clipped_workspace_bytes
    shapes = [(512, 768, 2304), (512, 768, 768), (512, 768, 3072), (512, 3072, 768)]
    single = max((dpclip.workspace_bytes(dpclip.DP_OP_CLIPPED_GRAD, 64, *sh, dpclip.DP_BF16) + 15) // 16 * 16 for sh in shapes)
    assert h(descs(shapes[:1]), 64, dpclip.DP_BF16) == (dpclip.workspace_bytes(dpclip.DP_OP_CLIPPED_GRAD, 64, *shapes[0], dpclip.DP_BF16) + 15) // 16 * 16
    # (float32 too: 2048 stages of 16 rows per layer cut into 7 slices, 432 tiles of 128 x 128 x 7 = 5.9 rounds of 512 workgroups)
    assert h(tr, 64, dpclip.DP_F32) == 7 * sum(di * do for _, di, do in shapes) * 4
    assert h(descs(shapes[:1]), 64, dpclip.DP_F32) == (dpclip.workspace_bytes(dpclip.DP_OP_CLIPPED_GRAD, 64, *shapes[0], dpclip.DP_F32) + 15) // 16 * 16
    # ... except aligned 16-bit layers on 256 x 256 tiles, which share one launch and keep all their K slices at once:
    # 64 * 16 stages per layer cut into 7 slices (756 items = 3 rounds of the 256 compute units)
    assert h(tr, 64, dpclip.DP_BF16) == 7 * sum(di * do for _, di, do in shapes) * 4 > single
    assert h(tr, 64, dpclip.DP_F16) == h(tr, 64, dpclip.DP_BF16)
    assert h(descs([(1, 784, 512), (1, 512, 256), (1, 256, 10)]), 256, dpclip.DP_F32) == 0    # short contractions: no K slices


def test_layer_descriptor_layout_and_argument_checks(lib):
    """Host logic only: every field of dp_layer_desc is read where the header says (the checks below fail before any
    launch, so the pointers are never touched; they are made-up, 16-byte aligned addresses)."""
    B, T, di, do = 64, 64, 72, 40
    fake = lambda k: 0x10000000 + 0x100000 * k

    def descs(**over):
        arr = (dpclip.LayerDesc * 2)()
        for l in range(2):
            d = dict(A=fake(1 + l), G=fake(3 + l), T=T, d_in=di, d_out=do, grad=fake(5 + l), noise_offset=0, bias_rows=None,
                     sqnorm=None, clip=None, clip_C=0.0, grad_b=None, bias_noise_offset=0)
            d.update({k: (v[l] if isinstance(v, (list, tuple)) else v) for k, v in over.items()})
            arr[l] = dpclip.LayerDesc(**d)
        return arr

    dt, auto = dpclip.DP_BF16, 0
    sq = lib.dp_layers_sqnorm_clip
    assert dpclip.layers_workspace_bytes(descs(), B, dt) > 0       # every valid call below stops at the missing workspace
    # plain call: everything valid, so the first complaint is the missing workspace
    assert sq(descs(), 2, B, dt, auto, 0, fake(9), 0.0, None, None, 0, None) == dpclip.DP_ERR_WORKSPACE
    # sqnorm / clip / clip_C: one array with two thresholds is refused, with one threshold it gets as far as the workspace
    assert sq(descs(sqnorm=fake(10), clip=fake(11), clip_C=[1.0, 2.0]), 2, B, dt, auto, 0, None, 0.0, None, None, 0, None) == dpclip.DP_ERR_INVALID_ARG
    assert sq(descs(sqnorm=fake(10), clip=fake(11), clip_C=[1.5, 1.5]), 2, B, dt, auto, 0, None, 0.0, None, None, 0, None) == dpclip.DP_ERR_WORKSPACE
    assert sq(descs(sqnorm=fake(10), clip=fake(11), clip_C=[0.0, 0.0]), 2, B, dt, auto, 0, None, 0.0, None, None, 0, None) == dpclip.DP_ERR_INVALID_ARG
    # a layer without an array of its own needs the call's
    assert sq(descs(sqnorm=[fake(10), None]), 2, B, dt, auto, 0, None, 0.0, None, None, 0, None) == dpclip.DP_ERR_INVALID_ARG
    cg = lib.dp_layers_clipped_grad_noise
    need = dpclip.layers_clipped_workspace_bytes(descs(), B, dt)
    # clip: the layers' own factors stand in for the call's
    assert cg(descs(), 2, B, None, dt, 0, 0.0, 0, None, 0, None) == dpclip.DP_ERR_INVALID_ARG
    assert need > 0                                   # else the next call would go on to launch kernels on made-up pointers
    assert cg(descs(clip=fake(11)), 2, B, None, dt, 0, 0.0, 0, None, 0, None) == dpclip.DP_ERR_WORKSPACE
    # grad_b needs bias_rows; bias_noise_offset + d_out must not wrap
    assert cg(descs(grad_b=fake(12)), 2, B, fake(13), dt, 0, 0.0, 0, None, 0, None) == dpclip.DP_ERR_INVALID_ARG
    assert cg(descs(grad_b=fake(12), bias_rows=fake(14), bias_noise_offset=2 ** 64 - 8), 2, B, fake(13), dt, 0, 1.0, 0, None, 0, None) == dpclip.DP_ERR_INVALID_ARG
    assert cg(descs(noise_offset=2 ** 64 - 8), 2, B, fake(13), dt, 0, 1.0, 0, None, 0, None) == dpclip.DP_ERR_INVALID_ARG
    assert cg(descs(grad=[fake(5), None]), 2, B, fake(13), dt, 0, 0.0, 0, None, 0, None) == dpclip.DP_ERR_INVALID_ARG


def test_noise_layout_gives_every_gradient_its_own_stretch():
    """Host logic only: the default positions in the noise stream (weights back to back, then the biases) are pairwise
    disjoint, also next to weight offsets given by the caller; overlapping offsets are refused.  Independent noise
    per coordinate is what the Gaussian mechanism needs (Algorithm 1, the line that adds the noise)."""
    sizes = [(5, 3), (7, 2), (4, 4), (1, 9)]
    has_bias = [True, False, True, True]

    def stretches(w, b):
        return sorted([(o, di * do) for o, (di, do) in zip(w, sizes)] + [(o, do) for o, (_, do), h in zip(b, sizes, has_bias) if h])

    def disjoint(st):
        return all(a[0] + a[1] <= c[0] for a, c in zip(st, st[1:]))

    w, b = dpclip.noise_layout(sizes, has_bias)
    assert w == [0, 15, 29, 45] and b == [54, 0, 57, 61]
    assert disjoint(stretches(w, b))
    # weights placed by the caller (a flat parameter vector with gaps): the default biases start behind the last one
    w, b = dpclip.noise_layout(sizes, has_bias, noise_offsets=[100, 0, 40, 60])
    assert w == [100, 0, 40, 60] and b[0] == 115 and disjoint(stretches(w, b))
    # each layer's weights followed by its own bias, as a model's flat gradient lays them out
    w, b = dpclip.noise_layout(sizes, has_bias, noise_offsets=[0, 18, 32, 52], bias_noise_offsets=[15, 0, 48, 61])
    assert disjoint(stretches(w, b))
    # what the earlier default did (every bias at 0) shares draws with the first weight gradient: refused
    with pytest.raises(ValueError):
        dpclip.noise_layout(sizes, has_bias, bias_noise_offsets=[0, 0, 0, 0])
    with pytest.raises(ValueError):
        dpclip.noise_layout(sizes, [False] * 4, noise_offsets=[0, 14, 29, 45])      # weights overlapping by one element
    # layers without parameters take no room
    assert dpclip.noise_layout([(0, 3), (2, 2)], [False, False]) == ([0, 0], [0, 0])


def test_missing_library_raises(monkeypatch):
    monkeypatch.setattr(dpclip, "_lib", None)
    monkeypatch.setattr(dpclip, "LIB_PATH", "/nonexistent/libdpclip.so")
    with pytest.raises(RuntimeError):
        dpclip.load_library()


def test_conv_rows_resident_host_logic(lib):
    """Host logic only: which convolution geometries the image-rows-in-LDS kernel takes (3 x 3, C a multiple of 64,
    a padded row that fits its copy table), and that the workspace query follows the choice."""
    q = dpclip.conv_rows_resident
    bf = dpclip.DP_BF16
    assert q(128, 32, 32, 64, 3, 3, 1, 128, bf) is True             # the convolution configuration
    assert q(128, 32, 32, 64, 3, 3, 1, 128, dpclip.DP_F16) is True
    assert q(128, 32, 32, 64, 3, 3, 1, 128, dpclip.DP_F8_E4M3) is True      # widened to fp16 first
    assert q(2, 16, 98, 64, 3, 3, 1, 40, bf) is True                # 100-pixel padded row: the widest that fits
    assert q(3, 28, 28, 64, 3, 3, 1, 128, bf) is True               # 784 positions: 24.5 stages per example
    assert q(4, 7, 7, 128, 3, 3, 1, 64, bf) is True                 # 49 positions
    assert q(2, 8, 16, 64, 5, 5, 2, 120, bf) is False               # 5 x 5
    assert q(2, 9, 9, 32, 2, 2, 0, 128, bf) is False                # 32 channels
    assert q(2, 16, 128, 64, 3, 3, 1, 128, bf) is False             # 130-pixel padded row: general kernel
    for bad in ((2, 8, 8, 12, 3, 3, 1, 64, bf), (2, 6, 6, 64, 3, 3, 1, 128, bf), (2, 8, 8, 64, 3, 3, 1, 64, dpclip.DP_F32),
                (-1, 8, 8, 64, 3, 3, 1, 64, bf), (2, 1, 1, 64, 3, 3, 0, 64, bf)):
        with pytest.raises(ValueError):
            q(*bad)
    # workspace: a line of zeros + one float per (example, 576-row x 64-column tile) for the norm
    assert dpclip.conv_workspace_bytes(dpclip.DP_OP_SQNORM, 128, 32, 32, 64, 3, 3, 1, 128, bf) == 256 + 128 * 2 * 4
    assert dpclip.conv_workspace_bytes(dpclip.DP_OP_SQNORM, 5, 16, 16, 128, 3, 3, 1, 72, bf) == 256 + 5 * 4 * 4
    # clipped sum: whole float32 slices of the 576 x 128 gradient
    w = dpclip.conv_workspace_bytes(dpclip.DP_OP_CLIPPED_GRAD, 128, 32, 32, 64, 3, 3, 1, 128, bf)
    assert (w - 256) % (576 * 128 * 4) == 0 and w > 256


def test_conv_geometry_queries_over_many_shapes(lib):
    """Host logic only: the kernel choice and the workspace sizes of the convolution calls answer consistently over a
    sweep of image sizes, paddings, channel counts and batch sizes (the choice replays the copy schedule of the
    image-rows-in-LDS kernel on the host for every geometry it accepts)."""
    bf = dpclip.DP_BF16
    n_rows = n_general = n_none = 0
    for H in (1, 3, 4, 7, 8, 9, 14, 16, 17, 28, 32, 33, 56, 64, 98, 100, 112):
        for W in (4, 7, 8, 14, 16, 24, 28, 32, 56, 64, 98, 100, 130):
            for pad in (0, 1, 2):
                if H + 2 * pad < 3 or W + 2 * pad < 3:
                    continue
                for (C, N, B) in ((64, 64, 1), (64, 128, 128), (128, 72, 5), (192, 256, 1100), (256, 40, 33)):
                    geo = (B, H, W, C, 3, 3, pad, N, bf)
                    ws_s = dpclip.conv_workspace_bytes(dpclip.DP_OP_SQNORM, *geo)
                    ws_c = dpclip.conv_workspace_bytes(dpclip.DP_OP_CLIPPED_GRAD, *geo)
                    try:
                        rows = dpclip.conv_rows_resident(*geo)
                    except ValueError:
                        n_none += 1
                        assert ws_s == 0 and ws_c == 0, geo
                        continue
                    assert ws_s >= 256 + 4 * B and ws_c >= 256 and ws_s % 4 == 0 and ws_c % 4 == 0, geo
                    T = (H + 2 * pad - 2) * (W + 2 * pad - 2)
                    if rows:
                        n_rows += 1
                        assert W + 2 * pad <= 102 and 4 * T >= 3 * (-(-T // 32) * 32), geo
                        assert ws_s == 256 + 4 * B * (C // 64) * (-(-N // 64)), geo
                        assert (ws_c - 256) % (9 * C * N * 4) == 0, geo
                    else:
                        n_general += 1
                        # the general kernel: short examples, rows too wide for the other kernel's copy table, or so
                        # narrow that a 32-position stage consumes more image rows than a round of copies brings
                        assert T >= 64 and (T < 512 or W + 2 * pad > 102 or W + 2 * pad - 2 < 8), geo
    assert n_rows > 500 and n_general > 100 and n_none > 100, (n_rows, n_general, n_none)
