"""Pins for the oracle's stack runner (no GPU): the toy network of Figures 2/3,
the paper's invariant that depth-first order leaves the results unchanged
(Sections 1, 3 and 6), identity stacks, and an independent library pipeline."""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import breadth_first as bf
from oracle import depth_first as df
from paper_1804_08378_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden(name):
    rows = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, vals = line.split(":")
            rows[key.strip()] = np.array([float(v) for v in vals.split()], np.float32)
    return rows


def _toy_layers():
    one = np.ones(1, np.float32)
    return [{"kind": "bn", "gamma": 2 * one, "beta": 0.5 * one, "mean": one, "var": one, "eps": 0.0},
            wl.relu(), wl.maxpool((1, 4), (1, 4), 0, True)]


def test_fig2_fig3_toy_network_breadth_first():
    g = _golden("fig2_fig3_toy.txt")
    x = g["x"].reshape(1, 1, 1, 8)
    out, idx, inter = bf.run_stack(_toy_layers(), x, keep_intermediates=True)
    assert np.array_equal(inter[0].ravel(), g["a"])
    assert np.array_equal(inter[1].ravel(), g["b"])
    assert np.array_equal(out.ravel(), g["out"])
    assert np.array_equal(idx[0].ravel(), g["argmax"].astype(np.int32))


def test_fig2_fig3_toy_network_depth_first_is_the_same():
    g = _golden("fig2_fig3_toy.txt")
    x = g["x"].reshape(1, 1, 1, 8)
    out, idx = df.run_stack_tiled(_toy_layers(), x, tile=(1, 1))  # one "white box" per output
    assert np.array_equal(out.ravel(), g["out"])
    assert np.array_equal(idx[0].ravel(), g["argmax"].astype(np.int32))


def test_identity_stack():
    x = np.abs(wl.activation((2, 3, 6, 6), 1))
    one, zero = np.ones(3, np.float32), np.zeros(3, np.float32)
    ident = {"kind": "bn", "gamma": one, "beta": zero, "mean": zero, "var": one, "eps": 0.0}
    out, _, _ = bf.run_stack([ident, wl.relu(), ident, wl.relu()], x)
    assert np.array_equal(out, x)


def _tiny_stacks():
    c = 3
    return {
        "bn_relu_max2": [wl.bn_params(c, 1), wl.relu(), wl.maxpool(2, 2, 0, True)],
        "bn_relu_max3s2p1": [wl.bn_params(c, 2), wl.relu(), wl.maxpool(3, 2, 1, True)],
        "bn_add_relu": [wl.bn_params(c, 3), wl.add(), wl.relu()],
        "bn_relu_avg2": [wl.bn_params(c, 4), wl.relu(), wl.avgpool(2, 2)],
        "halo_stress": [wl.bn_params(c, 5), wl.relu(), wl.avgpool(3, 1, 1, True),
                        wl.maxpool(3, 2, 1, True), wl.bn_params(c, 6), wl.relu()],
        "max_bn_relu_x3": sum(([wl.maxpool(3, 1, 1, False), wl.bn_params(c, 7 + i), wl.relu()]
                               for i in range(3)), []),
        "avg_nopad_div": [wl.relu(), wl.avgpool(3, 2, 1, False), wl.add(), wl.maxpool(2, 1, 0, True)],
        "rect_windows": [wl.bn_params(c, 9), wl.maxpool((3, 2), (2, 1), (1, 0), True),
                         wl.avgpool((2, 3), (1, 2), (1, 1), True)],
    }


@pytest.mark.parametrize("name", list(_tiny_stacks()))
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_depth_first_equals_breadth_first_bit_for_bit(name, dtype):
    """The paper's invariant, for several tile sizes including 1x1 and ragged ones."""
    layers = _tiny_stacks()[name]
    shape = (2, 3, 13, 11)
    x = wl.activation(shape, 20, dtype)
    res = [wl.activation(s, 21 + i, dtype) for i, s in enumerate(wl.residual_shapes(layers, shape))]
    ref, ref_idx, _ = bf.run_stack(layers, x, res, dtype)
    assert ref.shape == wl.output_shape(layers, shape)
    for tile in [(1, 1), (2, 3), (3, 2), (5, 100), (100, 4), (100, 100)]:
        out, idx = df.run_stack_tiled(layers, x, res, dtype, tile)
        assert np.array_equal(out.view(np.uint32), ref.view(np.uint32)), (name, tile)
        assert len(idx) == len(ref_idx)
        for a, b in zip(idx, ref_idx):
            covered = a >= 0  # cells no output depends on are never computed depth-first
            assert np.array_equal(a[covered], b[covered]), (name, tile)
            if name != "avg_nopad_div":
                assert covered.all()


def _torch_pipeline(layers, x, residuals, double=False):
    t = torch.from_numpy(x)
    t = t.double() if double else t
    res = [torch.from_numpy(r).double() if double else torch.from_numpy(r) for r in residuals]
    idx = []
    for l in layers:
        k = l["kind"]
        if k == "bn":
            cv = (lambda a: torch.from_numpy(a).double()) if double else torch.from_numpy
            t = F.batch_norm(t, cv(l["mean"]), cv(l["var"]), cv(l["gamma"]), cv(l["beta"]),
                             False, 0.0, l["eps"])
        elif k == "relu":
            t = torch.relu(t)
        elif k == "add":
            t = t + res.pop(0)
        elif k == "maxpool":
            t, i = F.max_pool2d(t, l["k"], l["s"], l["p"], return_indices=True)
            if l["return_indices"]:
                idx.append(i.numpy())
        else:
            t = F.avg_pool2d(t, l["k"], l["s"], l["p"], False, l["count_include_pad"])
    return t.numpy(), idx


def test_activation_stack_depth_first_equals_breadth_first_and_torch():
    """Leaky ReLU and clamp inside a pooled stack, f32 and bf16: depth-first equals
    breadth-first bit for bit; f32 agrees with the framework's layers."""
    import torch
    import torch.nn.functional as F
    layers = [wl.leaky_relu(0.1), wl.maxpool(3, 2, 1, True), wl.relu6(), wl.avgpool(2, 2, 0), wl.clamp(-0.25, 0.75)]
    x = wl.activation((2, 3, 12, 16), 10) * 5
    for dtype in ("f32", "bf16", "f16"):
        xin = L_round(x, dtype)
        ref, ref_idx, _ = bf.run_stack(layers, xin, (), dtype)
        for tile in ((1, 1), (2, 3), (100, 100)):
            out, idx = df.run_stack_tiled(layers, xin, (), dtype, tile)
            assert np.array_equal(out.view(np.uint32), ref.view(np.uint32))
            assert np.array_equal(idx[0], ref_idx[0])
    ref, _, _ = bf.run_stack(layers, x)
    t = F.max_pool2d(F.leaky_relu(torch.from_numpy(x), 0.1), 3, 2, 1)
    t = F.hardtanh(F.avg_pool2d(F.relu6(t), 2, 2), -0.25, 0.75).numpy()
    assert np.abs(ref - t).max() <= 1e-6


def L_round(x, dtype):
    from oracle import layers as L
    return L.round_to(x, dtype)


def test_ceil_mode_stack_depth_first_equals_breadth_first_and_torch():
    """A stack with ceil-mode pools (overhanging last windows): tiled depth-first execution
    gives the breadth-first result bit for bit, which agrees with the framework's layers."""
    import torch
    import torch.nn.functional as F
    layers = [wl.bn_params(3, 5), wl.relu(), wl.maxpool(3, 2, 0, True, ceil_mode=True),
              wl.avgpool(3, 2, 1, True, ceil_mode=True), wl.relu(), wl.avgpool(2, 2, 0, False, ceil_mode=True)]
    x = wl.activation((2, 3, 18, 21), 9)
    ref, ref_idx, _ = bf.run_stack(layers, x)
    assert ref.shape == wl.output_shape(layers, x.shape)
    for tile in ((1, 1), (2, 3), (100, 100)):
        out, idx = df.run_stack_tiled(layers, x, (), "f32", tile)
        assert np.array_equal(out.view(np.uint32), ref.view(np.uint32))
        assert np.array_equal(idx[0], ref_idx[0])
    b = layers[0]
    t = F.batch_norm(torch.from_numpy(x).double(), torch.from_numpy(b["mean"]).double(), torch.from_numpy(b["var"]).double(),
                     torch.from_numpy(b["gamma"]).double(), torch.from_numpy(b["beta"]).double(), False, 0.0, b["eps"])
    t = F.max_pool2d(F.relu(t), 3, 2, 0, ceil_mode=True)
    t = F.relu(F.avg_pool2d(t, 3, 2, 1, ceil_mode=True, count_include_pad=True))
    t = F.avg_pool2d(t, 2, 2, 0, ceil_mode=True, count_include_pad=False).numpy()
    assert t.shape == ref.shape and np.abs(ref - t).max() <= 1e-5 * np.abs(t).max()


@pytest.mark.parametrize("name", wl.CONFIG_NAMES)
def test_named_configs_vs_library_pipeline_f64(name):
    """Every benchmark configuration (batch cut to 2, planes cut to keep it quick) against
    torch's CPU operators evaluated in float64: fp32 tolerance of the benchmark spec."""
    layers, shape, _ = wl.build(name, seed=0, batch=2, indices=True)
    c = min(shape[1], 8)
    for l in layers:
        if l["kind"] == "bn":
            for key in ("gamma", "beta", "mean", "var"):
                l[key] = l[key][:c]
    shape = (2, c, min(shape[2], 56), min(shape[3], 56))
    x = wl.activation(shape, 0)
    res = [wl.activation(s, 1 + i) for i, s in enumerate(wl.residual_shapes(layers, shape))]
    out, idx, _ = bf.run_stack(layers, x, res)
    ref, ref_idx = _torch_pipeline(layers, x, res, double=True)
    assert out.shape == ref.shape
    assert np.abs(out - ref).max() <= 1e-5 * np.abs(ref).max()
    # argmax: float64 and float32 may break near-ties differently; the picked cell must
    # hold the window maximum of the oracle's own pre-pool tensor (checked in layer pins),
    # and must agree with the library wherever the library's choice is not a near-tie.
    for a, b in zip(idx, ref_idx):
        assert (a == b).mean() > 0.6  # ReLU zeros tie exactly, same rule -> mostly equal


def test_config0_end_to_end_fp32_library_pipeline():
    """Config 0 (1x16x32x32 BN->ReLU->MaxPool 2/2) against the same operators of torch in
    float32: max values agree to tolerance, indices agree except at float near-ties."""
    layers, x, res = wl.inputs_for("tiny", 0, "f32", indices=True)
    out, idx, _ = bf.run_stack(layers, x, res)
    ref, ref_idx = _torch_pipeline(layers, x, res)
    assert out.shape == (1, 16, 16, 16)
    assert np.abs(out - ref).max() <= 1e-5 * np.abs(ref).max()
    assert (idx[0] == ref_idx[0]).mean() > 0.99


def test_bf16_stack_rounds_at_every_layer_boundary():
    layers, x, res = wl.inputs_for("resnet_tail", 0, "bf16", batch=1)
    for l in layers:
        if l["kind"] == "bn":
            for key in ("gamma", "beta", "mean", "var"):
                l[key] = l[key][:4]
    x, res = x[:, :4, :8, :8], [r[:, :4, :8, :8] for r in res]
    out, _, inter = bf.run_stack(layers, x, res, "bf16", keep_intermediates=True)
    for t in inter:
        assert np.array_equal(t, torch.from_numpy(t).to(torch.bfloat16).float().numpy())
    # same pipeline with torch bf16 tensors layer by layer (fp32 math inside each layer)
    p = layers[0]
    s = p["gamma"].astype(np.float64) / np.sqrt(p["var"].astype(np.float64) + p["eps"])
    sh = p["beta"].astype(np.float64) - p["mean"].astype(np.float64) * s
    a = (x.astype(np.float64) * s[None, :, None, None] + sh[None, :, None, None])
    a = torch.from_numpy(a).to(torch.bfloat16).double().numpy()  # fma == exact-then-round
    b = torch.from_numpy(a + res[0].astype(np.float64)).to(torch.bfloat16).float().numpy()
    ref = np.maximum(b, 0)
    # float64 -> bf16 vs float32-fma -> bf16 can differ only by double rounding at ties
    assert (out != ref).mean() < 1e-3
    assert np.abs(out - ref).max() <= 1e-2 * np.abs(ref).max()


def test_f16_stack_rounds_at_every_layer_boundary_like_the_framework():
    """binary16 storage: every intermediate is representable in float16, and the stack agrees
    with the framework's float16 tensors run layer by layer (float32 math inside a layer)."""
    import torch.nn.functional as F
    layers = [wl.bn_params(3, 7), wl.relu(), wl.maxpool(3, 2, 1), wl.avgpool(2, 2, 0)]
    x = wl.activation((2, 3, 12, 16), 8, "f16") * 3
    x = x.astype(np.float16).astype(np.float32)
    out, _, inter = bf.run_stack(layers, x, (), "f16", keep_intermediates=True)
    for t in inter:
        assert np.array_equal(t, t.astype(np.float16).astype(np.float32))
    b = layers[0]
    t = torch.from_numpy(x)
    t = F.batch_norm(t, *(torch.from_numpy(b[k]) for k in ("mean", "var", "gamma", "beta")), False, 0.0, b["eps"]).half().float()
    t = F.max_pool2d(F.relu(t), 3, 2, 1)
    t = F.avg_pool2d(t, 2, 2).half().float().numpy()
    assert (out != t).mean() < 0.02                       # double-rounding ties of the differently ordered BatchNorm
    assert np.abs(out - t).max() <= 2e-3 * np.abs(t).max()


def test_runner_argument_errors():
    x = wl.activation((1, 2, 4, 4), 0)
    with pytest.raises(ValueError):
        bf.run_stack([wl.add()], x, [])
    with pytest.raises(ValueError):
        bf.run_stack([wl.relu()], x, [x])
    with pytest.raises(ValueError):
        bf.run_stack([{"kind": "conv"}], x)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_max_pool_commutes_with_non_decreasing_lists_that_hold_a_relu(dtype):
    """The identity behind running a max pool before the element-wise list in front of it
    (when no argmax is wanted): for operations that never decrease -- BatchNorm with scales
    >= 0, ReLU, leaky ReLU with slope >= 0, clamp, the roundings to the storage type --
    max_i f(x_i) and f(max_i x_i) are the same number, and once a ReLU has made every zero +0
    the same bits.  Checked on the oracle alone: both layer orders, bit for bit, with zeros of
    both signs and a zero BatchNorm shift in the input; and the identity must fail to hold
    where it is not claimed (negative scales)."""
    c, shape = 6, (2, 6, 11, 13)
    x = wl.activation(shape, 77, dtype)
    x[:, :, ::3, ::2] = 0.0
    x[:, :, 1::3, 1::2] = -0.0
    bn = wl.bn_params(c, 78)
    zero = wl.bn_params(c, 79)
    zero["beta"] = np.zeros(c, np.float32)
    zero["mean"] = np.zeros(c, np.float32)
    for pool in (wl.maxpool(3, 2, 1), wl.maxpool(2, 2), wl.maxpool(3, 1, 1), wl.maxpool((2, 3), (1, 2), (1, 1))):
        for lst in ([bn, wl.relu()], [zero, wl.relu()], [wl.relu(), bn, wl.leaky_relu(0.1), wl.clamp(-0.5, 2.0)],
                    [wl.relu()], [wl.clamp(-1.0, 1.0), wl.relu(), zero]):
            a, _, _ = bf.run_stack(lst + [pool], x, [], dtype)
            b, _, _ = bf.run_stack([pool] + lst, x, [], dtype)
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    neg = wl.bn_params(c, 80)
    neg["gamma"] = -neg["gamma"]
    a, _, _ = bf.run_stack([neg, wl.relu(), wl.maxpool(3, 2, 1)], x, [], dtype)
    b, _, _ = bf.run_stack([wl.maxpool(3, 2, 1), neg, wl.relu()], x, [], dtype)
    assert not np.array_equal(a, b)
