"""Breadth-first execution of a layer stack -- TEST INFRASTRUCTURE.

This is the order Figure 2 of the paper shows: every layer is applied to the
whole tensor, and its whole output is materialised, before the next layer
starts.  The paper's claim (Sections 1, 3, 6) is that depth-first execution
gives the same numbers; this runner is therefore what the fused GPU path is
compared against.

dtype "bf16" (not in the paper, which is float32 only): activations are stored
in bfloat16, so each layer computes in float32 from bf16-representable inputs
and its output is rounded to bfloat16 (round-to-nearest-even) before the next
layer sees it -- exactly what a layer-by-layer bf16 run would store.
"""
from __future__ import annotations

import numpy as np

from . import layers as L


def run_stack(layers, x, residuals=(), dtype: str = "f32", keep_intermediates: bool = False):
    """Apply `layers` (plain dicts, see the workloads module) to NCHW float32 `x`.

    Returns (out, indices, intermediates): `indices` holds one int32 array per
    max-pool layer with return_indices, in layer order; `intermediates` is the
    list of every layer's output when requested (else empty).
    """
    if dtype not in ("f32", "bf16", "f16"):
        raise ValueError("dtype")
    cur = np.ascontiguousarray(x, dtype=np.float32)
    res = list(residuals)
    indices = []
    inter = []
    for layer in layers:
        kind = layer["kind"]
        if kind == "bn":
            cur = L.batchnorm(cur, layer["gamma"], layer["beta"], layer["mean"], layer["var"],
                              layer["eps"])
        elif kind == "relu":
            cur = L.relu(cur)
        elif kind == "leaky_relu":
            cur = L.leaky_relu(cur, layer["slope"])
        elif kind == "clamp":
            cur = L.clamp(cur, layer["lo"], layer["hi"])
        elif kind == "add":
            if not res:
                raise ValueError("stack has more Add layers than residual tensors")
            cur = L.add(cur, res.pop(0))
        elif kind == "maxpool":
            if layer.get("return_indices"):
                cur, idx = L.maxpool(cur, layer["k"], layer["s"], layer["p"], True, layer.get("ceil_mode", False))
                indices.append(idx)
            else:
                cur = L.maxpool(cur, layer["k"], layer["s"], layer["p"], False, layer.get("ceil_mode", False))
        elif kind == "avgpool":
            cur = L.avgpool(cur, layer["k"], layer["s"], layer["p"],
                            layer.get("count_include_pad", True), layer.get("ceil_mode", False))
        else:
            raise ValueError(f"unknown layer kind {kind!r}")
        cur = L.round_to(cur, dtype)
        if keep_intermediates:
            inter.append(cur)
    if res:
        raise ValueError("more residual tensors than Add layers")
    return cur, indices, inter
