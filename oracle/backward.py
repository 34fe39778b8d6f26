"""Backward pass of a layer stack on the CPU -- TEST INFRASTRUCTURE.

The paper's outlook (Section 7) names training as the next step for the method; the forward
pass it defines (Sections 2 and 3) fixes what a backward pass has to compute: the product of
the upstream gradient with the Jacobian of the layer-by-layer forward pass, with respect to
the stack's input and to every residual operand.  This module writes that definition out,
layer by layer in reverse order, on whole tensors:

  * the forward pass is the breadth-first runner's (float32 arithmetic, every layer's output
    rounded to the storage type), so that every decision the gradient depends on -- the sign
    seen by a ReLU, the cell a max pooling window picked -- is the forward pass's own;
  * storage rounding counts as the identity (what automatic differentiation of a
    layer-by-layer run in 16-bit storage does);
  * BatchNorm is the inference-mode layer: y = x * scale[c] + shift[c] with constant folded
    parameters, so its Jacobian is scale[c]; no gradient for the parameters;
  * ReLU passes the gradient where its input is > 0; leaky ReLU multiplies by the slope
    elsewhere; clamp passes it where lo <= input <= hi (both bounds included);
  * Add passes the gradient on unchanged and hands a copy to the residual operand;
  * max pooling sends each output's gradient to the one cell the forward pass picked (first
    maximum in row-major window order) and sums where windows overlap;
  * average pooling sends each output's gradient, times the float32 reciprocal of the divisor
    the forward pass used for that window, to every in-range cell of the window.

Gradients are accumulated in float64 and returned unrounded; callers round to the storage type.
Nothing here is used by the HIP library or its binding.
"""
from __future__ import annotations

import numpy as np

from . import layers as L
from .breadth_first import run_stack


def _pool_geometry(layer, h, w):
    kh, kw = layer["k"]
    sh, sw = layer["s"]
    ph, pw = layer["p"]
    ceil_mode = layer.get("ceil_mode", False)
    ho, wo = L.pool_out(h, kh, sh, ph, ceil_mode), L.pool_out(w, kw, sw, pw, ceil_mode)
    return kh, kw, sh, sw, ph, pw, ho, wo


def _maxpool_backward(g, idx, h, w):
    n, c, ho, wo = g.shape
    gin = np.zeros((n * c, h * w), np.float64)
    planes = np.repeat(np.arange(n * c), ho * wo)
    np.add.at(gin, (planes, idx.reshape(-1).astype(np.int64)), g.reshape(-1))
    return gin.reshape(n, c, h, w)


def _avgpool_backward(g, layer, h, w):
    kh, kw, sh, sw, ph, pw, ho, wo = _pool_geometry(layer, h, w)
    include_pad = layer.get("count_include_pad", True)
    oh, ow = np.arange(ho), np.arange(wo)
    h0, w0 = oh * sh - ph, ow * sw - pw
    # divisor of each window, as the forward layer counts it
    if include_pad:  # cells inside the padded plane
        dh = np.minimum(h0 + kh, h + ph) - h0
        dw = np.minimum(w0 + kw, w + pw) - w0
    else:            # cells inside the plane
        dh = np.minimum(h0 + kh, h) - np.maximum(h0, 0)
        dw = np.minimum(w0 + kw, w) - np.maximum(w0, 0)
    inv = (np.float32(1.0) / np.outer(dh, dw).astype(np.float32)).astype(np.float64)
    gs = g * inv[None, None]
    gin = np.zeros(g.shape[:2] + (h, w), np.float64)
    for a in range(kh):
        ih = h0 + a
        vh = (ih >= 0) & (ih < h)
        for b in range(kw):
            iw = w0 + b
            vw = (iw >= 0) & (iw < w)
            # one window offset: distinct outputs hit distinct cells, so += on the fancy index is safe
            gin[:, :, ih[vh][:, None], iw[vw][None, :]] += gs[:, :, oh[vh][:, None], ow[vw][None, :]]
    return gin


def backward_stack(layers, x, residuals, grad_out, dtype: str = "f32"):
    """Gradient of sum(out * grad_out) with respect to `x` and to each residual operand.

    Returns (grad_x, [grad_residual_0, ...]) as float64 arrays, residuals in layer order.
    """
    # the forward pass, with every layer's input and every max pooling's picks kept
    fwd_layers = [dict(l, return_indices=True) if l["kind"] == "maxpool" else l for l in layers]
    out, indices, inter = run_stack(fwd_layers, x, residuals, dtype, keep_intermediates=True)
    g = np.ascontiguousarray(grad_out, dtype=np.float64)
    if g.shape != out.shape:
        raise ValueError("grad_out must have the shape of the stack's output")
    layer_in = [np.ascontiguousarray(x, dtype=np.float32)] + inter[:-1]
    indices = list(indices)
    grad_res = []
    for i in range(len(layers) - 1, -1, -1):
        layer, xin = layers[i], layer_in[i]
        kind = layer["kind"]
        if kind == "bn":
            scale, _ = L.bn_fold(layer["gamma"], layer["beta"], layer["mean"], layer["var"], layer["eps"])
            g = g * scale.astype(np.float64)[None, :, None, None]
        elif kind == "relu":
            g = np.where(xin > 0, g, 0.0)
        elif kind == "leaky_relu":
            g = np.where(xin > 0, g, g * np.float64(np.float32(layer["slope"])))
        elif kind == "clamp":
            lo, hi = np.float32(layer["lo"]), np.float32(layer["hi"])
            g = np.where((xin >= lo) & (xin <= hi), g, 0.0)
        elif kind == "add":
            grad_res.append(g.copy())
        elif kind == "maxpool":
            g = _maxpool_backward(g, indices.pop(), xin.shape[2], xin.shape[3])
        elif kind == "avgpool":
            g = _avgpool_backward(g, layer, xin.shape[2], xin.shape[3])
        else:
            raise ValueError(f"unknown layer kind {kind!r}")
    grad_res.reverse()
    return g, grad_res
