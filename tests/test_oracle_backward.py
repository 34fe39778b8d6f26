"""Pins of the backward-pass oracle (oracle/backward.py) against things other than itself:
the framework's automatic differentiation in float64, finite differences of the (separately
pinned) forward oracle, closed forms and conservation laws."""
from __future__ import annotations

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import backward as bw
from oracle import breadth_first as bf
from paper_1804_08378_amd import workloads as wl


def _autograd(layers, x, residuals, dy):
    """d sum(out * dy) / d(x, residuals) by the framework's autograd over its own layers, float64."""
    t = torch.from_numpy(x).double().requires_grad_(True)
    res = [torch.from_numpy(r).double().requires_grad_(True) for r in residuals]
    pending = list(res)
    cur = t
    for l in layers:
        k = l["kind"]
        if k == "bn":
            cv = lambda a: torch.from_numpy(a).double()
            cur = F.batch_norm(cur, cv(l["mean"]), cv(l["var"]), cv(l["gamma"]), cv(l["beta"]), False, 0.0, l["eps"])
        elif k == "relu":
            cur = torch.relu(cur)
        elif k == "leaky_relu":
            cur = F.leaky_relu(cur, float(np.float32(l["slope"])))
        elif k == "clamp":
            cur = torch.clamp(cur, float(np.float32(l["lo"])), float(np.float32(l["hi"])))
        elif k == "add":
            cur = cur + pending.pop(0)
        elif k == "maxpool":
            cur = F.max_pool2d(cur, l["k"], l["s"], l["p"], ceil_mode=l.get("ceil_mode", False))
        else:
            cur = F.avg_pool2d(cur, l["k"], l["s"], l["p"], l.get("ceil_mode", False), l["count_include_pad"])
    grads = torch.autograd.grad((cur * torch.from_numpy(dy).double()).sum(), [t] + res)
    return grads[0].numpy(), [g.numpy() for g in grads[1:]]


def _stacks():
    c = 3
    return {
        "bn_relu_max2": [wl.bn_params(c, 1), wl.relu(), wl.maxpool(2, 2, 0)],
        "bn_relu_max3s2p1": [wl.bn_params(c, 2), wl.relu(), wl.maxpool(3, 2, 1)],
        "bn_add_relu": [wl.bn_params(c, 3), wl.add(), wl.relu()],
        "bn_relu_avg2": [wl.bn_params(c, 4), wl.relu(), wl.avgpool(2, 2)],
        "halo_stress": [wl.bn_params(c, 5), wl.relu(), wl.avgpool(3, 1, 1, True), wl.maxpool(3, 2, 1),
                        wl.bn_params(c, 6), wl.relu()],
        "max_bn_relu_x3": sum(([wl.maxpool(3, 1, 1), wl.bn_params(c, 7 + i), wl.relu()] for i in range(3)), []),
        "avg_nopad_div": [wl.relu(), wl.avgpool(3, 2, 1, False), wl.add(), wl.maxpool(2, 1, 0)],
        "rect_windows": [wl.bn_params(c, 9), wl.maxpool((3, 2), (2, 1), (1, 0)), wl.avgpool((2, 3), (1, 2), (1, 1), True)],
        "two_adds": [wl.add(), wl.bn_params(c, 10), wl.leaky_relu(0.1), wl.add(), wl.clamp(-0.5, 1.5)],
        "ceil_avg": [wl.bn_params(c, 11), wl.avgpool(3, 2, 1, True, ceil_mode=True), wl.relu()],
        "ceil_avg_nopad": [wl.avgpool(2, 2, 0, False, ceil_mode=True), wl.bn_params(c, 12)],
        "ceil_max": [wl.leaky_relu(0.2), wl.maxpool(3, 2, 0, ceil_mode=True), wl.add(), wl.relu()],
        "global_avg": [wl.bn_params(c, 13), wl.relu(), wl.avgpool((11, 13), (11, 13), 0)],
    }


def _inputs(layers, shape, seed, dtype="f32"):
    x = wl.activation(shape, seed, dtype)
    res = [wl.activation(s, seed + 1 + i, dtype) for i, s in enumerate(wl.residual_shapes(layers, shape))]
    dy = wl.activation(wl.output_shape(layers, shape), seed + 50, dtype)
    return x, res, dy


@pytest.mark.parametrize("name", list(_stacks()))
def test_backward_equals_the_frameworks_autograd_in_float64(name):
    layers = _stacks()[name]
    # ceil mode: sizes at which a last window overhangs the padded plane (its divisor is clipped)
    x, res, dy = _inputs(layers, (2, 3, 12, 14) if name.startswith("ceil") else (2, 3, 11, 13), 3)
    gx, gres = bw.backward_stack(layers, x, res, dy)
    tx, tres = _autograd(layers, x, res, dy)
    # the forward decisions are float32 here and float64 there: equal unless a value sits within
    # rounding of a kink, which these seeds avoid
    np.testing.assert_allclose(gx, tx, rtol=1e-6, atol=1e-7)
    assert len(gres) == len(tres) == wl.num_residuals(layers)
    for a, b in zip(gres, tres):
        np.testing.assert_allclose(a, b, rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("name", ["bn_relu_max3s2p1", "halo_stress", "avg_nopad_div", "two_adds", "ceil_avg"])
def test_backward_equals_finite_differences_of_the_forward_oracle(name):
    """The stack is piecewise linear: a central difference of the forward oracle is its exact
    directional derivative wherever the step crosses no kink."""
    layers = _stacks()[name]
    shape = (1, 3, 7, 6)
    x, res, dy = _inputs(layers, shape, 11)
    gx, gres = bw.backward_stack(layers, x, res, dy)
    eps = np.float32(2.0 ** -7)  # a power of two: x +- eps are exact

    def loss(xv, rv):
        out, _, _ = bf.run_stack(layers, xv, rv)
        return float((out.astype(np.float64) * dy.astype(np.float64)).sum())

    rng = np.random.default_rng(0)
    checked = 0
    for target, grad in [(-1, gx)] + list(enumerate(gres)):
        base = x if target < 0 else res[target]
        for flat in rng.choice(base.size, 25, replace=False):
            lo, hi = base.copy(), base.copy()
            lo.flat[flat] -= eps
            hi.flat[flat] += eps
            args = (lambda v: (v, res)) if target < 0 else (lambda v: (x, res[:target] + [v] + res[target + 1:]))
            fd = (loss(*args(hi)) - loss(*args(lo))) / (2.0 * float(eps))
            # a kink inside the step shows as a one-sided slope; such points are rare and skipped
            one = (loss(*args(hi)) - loss(x, res)) / float(eps)
            if abs(one - fd) > 1e-3 * max(1.0, abs(fd)):
                continue
            assert abs(fd - grad.flat[flat]) <= 2e-3 * max(1.0, abs(fd)), (name, target, flat)
            checked += 1
    assert checked >= 20 * (1 + len(gres)) // 2


def test_closed_forms():
    c = 4
    x = wl.activation((2, c, 6, 8), 0)
    dy = wl.activation((2, c, 6, 8), 1)
    bn = wl.bn_params(c, 5)
    # BatchNorm alone: dy times the folded scale
    gx, _ = bw.backward_stack([bn], x, [], dy)
    scale = (bn["gamma"].astype(np.float64) / np.sqrt(bn["var"].astype(np.float64) + bn["eps"])).astype(np.float32)
    np.testing.assert_array_equal(gx, dy.astype(np.float64) * scale.astype(np.float64)[None, :, None, None])
    # ReLU: where x > 0; zero at exactly 0
    x0 = x.copy()
    x0[0, 0, 0, :4] = 0.0
    gx, _ = bw.backward_stack([wl.relu()], x0, [], dy)
    np.testing.assert_array_equal(gx, np.where(x0 > 0, dy, 0).astype(np.float64))
    # leaky ReLU and clamp (bounds included)
    gx, _ = bw.backward_stack([wl.leaky_relu(0.25)], x, [], dy)
    np.testing.assert_array_equal(gx, np.where(x > 0, dy, dy * 0.25).astype(np.float64))
    xb = x.copy()
    xb[0, 0, 0, 0], xb[0, 0, 0, 1] = -0.5, 1.0
    gx, _ = bw.backward_stack([wl.clamp(-0.5, 1.0)], xb, [], dy)
    np.testing.assert_array_equal(gx, np.where((xb >= -0.5) & (xb <= 1.0), dy, 0).astype(np.float64))
    assert gx[0, 0, 0, 0] == dy[0, 0, 0, 0] and gx[0, 0, 0, 1] == dy[0, 0, 0, 1]
    # Add: the residual gets what flows on; ops after it apply to both, ops before it to x only
    r = wl.activation((2, c, 6, 8), 2)
    gx, (gr,) = bw.backward_stack([bn, wl.add(), wl.relu()], x, [r], dy)
    out, _, inter = bf.run_stack([bn, wl.add()], x, [r], keep_intermediates=True)
    np.testing.assert_array_equal(gr, np.where(out > 0, dy, 0).astype(np.float64))
    np.testing.assert_array_equal(gx, gr * scale.astype(np.float64)[None, :, None, None])


def test_average_pooling_closed_forms():
    x = wl.activation((1, 2, 6, 6), 0)
    ones = np.ones((1, 2, 3, 3), np.float32)
    # disjoint windows: every cell gets dy / (k * k)
    gx, _ = bw.backward_stack([wl.avgpool(2, 2)], x, [], ones)
    np.testing.assert_array_equal(gx, np.full(x.shape, 0.25))
    # whole-plane window: dy / (H * W) everywhere (float32 reciprocal)
    gx, _ = bw.backward_stack([wl.avgpool(6, 6)], x, [], 3 * np.ones((1, 2, 1, 1), np.float32))
    np.testing.assert_array_equal(gx, np.full(x.shape, 3.0 * float(np.float32(1) / np.float32(36))))
    # 3x3 / 1 / pad 1, padding counted: a cell's gradient is (number of windows over it) / 9
    gx, _ = bw.backward_stack([wl.avgpool(3, 1, 1, True)], x, [], np.ones((1, 2, 6, 6), np.float32))
    cover = np.full((6, 6), 9.0)
    cover[0, :] = cover[-1, :] = cover[:, 0] = cover[:, -1] = 6.0
    cover[0, 0] = cover[0, -1] = cover[-1, 0] = cover[-1, -1] = 4.0
    np.testing.assert_allclose(gx[0, 0], cover * float(np.float32(1) / np.float32(9)), rtol=1e-15)
    # padding not counted: the gradients of one window sum to its dy, so the whole tensor sums to sum(dy)
    dy = wl.activation((1, 2, 6, 6), 4)
    gx, _ = bw.backward_stack([wl.avgpool(3, 1, 1, False)], x, [], dy)
    np.testing.assert_allclose(gx.sum(), dy.astype(np.float64).sum(), rtol=1e-6)


def test_max_pooling_routes_to_the_forward_picks_and_conserves_the_gradient():
    x = wl.activation((2, 3, 9, 10), 7)
    layers = [wl.maxpool(3, 2, 1, True)]
    out, (idx,), _ = bf.run_stack(layers, x, [])
    dy = wl.activation(out.shape, 8)
    gx, _ = bw.backward_stack([wl.maxpool(3, 2, 1)], x, [], dy)
    np.testing.assert_allclose(gx.sum(axis=(2, 3)), dy.astype(np.float64).sum(axis=(2, 3)), rtol=1e-12)
    picked = np.zeros(x.shape, bool).reshape(6, -1)
    picked[np.repeat(np.arange(6), idx[0, 0].size), idx.reshape(-1)] = True
    assert not gx.reshape(6, -1)[~picked].any()
    # an all-equal plane: every window picks its first in-range cell (row-major)
    gx, _ = bw.backward_stack([wl.maxpool(2, 2)], np.zeros((1, 1, 4, 4), np.float32), [], np.ones((1, 1, 2, 2), np.float32))
    want = np.zeros((4, 4))
    want[::2, ::2] = 1.0
    np.testing.assert_array_equal(gx[0, 0], want)
    # overlapping windows that pick the same cell add up
    peak = np.zeros((1, 1, 5, 5), np.float32)
    peak[0, 0, 2, 2] = 1.0
    gx, _ = bw.backward_stack([wl.maxpool(3, 1, 1)], peak, [], np.ones((1, 1, 5, 5), np.float32))
    assert gx[0, 0, 2, 2] == 9.0


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_sixteen_bit_storage_takes_its_decisions_from_the_rounded_forward_pass(dtype):
    """With 16-bit storage the masks and picks come from the rounded layer outputs: the gradient
    equals autograd's over a forward pass that is fed those rounded values layer by layer."""
    layers = _stacks()["halo_stress"]
    x, res, dy = _inputs(layers, (2, 3, 11, 13), 5, dtype)
    gx, _ = bw.backward_stack(layers, x, res, dy, dtype)
    fwd = [dict(l, return_indices=True) if l["kind"] == "maxpool" else l for l in layers]
    _, _, inter = bf.run_stack(fwd, x, res, dtype, keep_intermediates=True)
    g = torch.from_numpy(dy).double()
    for i in range(len(layers) - 1, -1, -1):  # one layer at a time, each from its stored input
        xin = torch.from_numpy(x if i == 0 else inter[i - 1]).double().requires_grad_(True)
        (out,) = _autograd_forward([layers[i]], xin)
        (g,) = torch.autograd.grad((out * g).sum(), [xin])
    np.testing.assert_allclose(gx, g.numpy(), rtol=1e-6, atol=1e-7)


def _autograd_forward(layers, t):
    cur = t
    for l in layers:
        k = l["kind"]
        if k == "bn":
            cv = lambda a: torch.from_numpy(a).double()
            cur = F.batch_norm(cur, cv(l["mean"]), cv(l["var"]), cv(l["gamma"]), cv(l["beta"]), False, 0.0, l["eps"])
        elif k == "relu":
            cur = torch.relu(cur)
        elif k == "maxpool":
            cur = F.max_pool2d(cur, l["k"], l["s"], l["p"])
        else:
            cur = F.avg_pool2d(cur, l["k"], l["s"], l["p"], False, l["count_include_pad"])
    return (cur,)


def test_argument_errors():
    x = wl.activation((1, 2, 4, 4), 0)
    with pytest.raises(ValueError):
        bw.backward_stack([wl.maxpool(2, 2)], x, [], np.zeros((1, 2, 4, 4), np.float32))
