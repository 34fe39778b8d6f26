"""PyTorch front-end: aggregation detection and model rewriting (Sections 4 and 4.3, Figure 4).

`optimize(model)` scans the layers of every `torch.nn.Sequential` in the model in order, pushes
consecutive optimizable layers (inference BatchNorm2d, ReLU, LeakyReLU, ReLU6, Hardtanh, MaxPool2d,
AvgPool2d, adaptive pools whose output size divides their input, and the layers
that are the identity at inference time) on a stack, and when it meets a layer it cannot optimize
(a convolution, a linear layer, ...) collapses the stack: the first layer of the run is replaced
by a `BrainSlugStack` module that executes the whole run depth-first through the C ABI, the
others are replaced by `torch.nn.Identity` (the paper removes them; keeping the positions leaves
every index and name of the container valid).  One call, no change to the model's code -- the
paper's Listing 3.

Only `Sequential` containers are rewritten: they are the only modules whose children are known to
execute in order, one feeding the next.  Everything else (convolutions, the model's own `forward`)
keeps running in PyTorch.

A `BrainSlugStack` plans lazily, once per input shape and dtype (the scheduler of Section 4.2: it
computes the output size, asks the framework for the memory and launches the kernels on the
framework's stream), and identical stack signatures share their compiled kernels library-wide
(Section 4.3).  There is no fallback: an input the library cannot take (not on a GPU, not
float32/bfloat16 NCHW, a model in training mode) raises.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Tuple

import numpy as np
import torch
from torch import nn

from . import brainslug as bs
from . import workloads as wl

__all__ = ["optimize", "BrainSlugStack", "layer_desc", "find_runs", "resolve_layers"]


def _pair(v) -> Tuple[int, int]:
    return (int(v), int(v)) if isinstance(v, int) else (int(v[0]), int(v[1]))


def layer_desc(m: nn.Module) -> Optional[dict]:
    """The library's description of module `m`: a layer dict, {} for a layer that is the identity
    at inference time, or None when the module is not optimizable."""
    if isinstance(m, nn.BatchNorm2d):
        if not m.track_running_stats or m.running_mean is None:
            return None  # batch statistics even in eval mode: not the inference BatchNorm
        c = m.num_features
        ones, zeros = np.ones(c, np.float32), np.zeros(c, np.float32)
        f = lambda t, d: d if t is None else t.detach().float().cpu().numpy()
        return {"kind": "bn", "gamma": f(m.weight, ones), "beta": f(m.bias, zeros),
                "mean": f(m.running_mean, zeros), "var": f(m.running_var, ones), "eps": float(m.eps)}
    if isinstance(m, nn.ReLU):
        return {"kind": "relu"}
    if isinstance(m, nn.LeakyReLU):
        return {"kind": "leaky_relu", "slope": float(m.negative_slope)}
    if isinstance(m, nn.ReLU6):
        return {"kind": "clamp", "lo": 0.0, "hi": 6.0}
    if isinstance(m, nn.Hardtanh):
        return {"kind": "clamp", "lo": float(m.min_val), "hi": float(m.max_val)}
    if isinstance(m, nn.MaxPool2d):
        if _pair(m.dilation) != (1, 1) or m.return_indices:
            return None  # a Sequential cannot pass on the (values, indices) pair anyway
        k = _pair(m.kernel_size)
        return {"kind": "maxpool", "k": k, "s": _pair(m.stride if m.stride is not None else k),
                "p": _pair(m.padding), "return_indices": False, "ceil_mode": bool(m.ceil_mode)}
    if isinstance(m, nn.AvgPool2d):
        if m.divisor_override is not None:
            return None
        k = _pair(m.kernel_size)
        return {"kind": "avgpool", "k": k, "s": _pair(m.stride if m.stride is not None else k),
                "p": _pair(m.padding), "count_include_pad": bool(m.count_include_pad),
                "ceil_mode": bool(m.ceil_mode)}
    if isinstance(m, (nn.AdaptiveAvgPool2d, nn.AdaptiveMaxPool2d)):
        if getattr(m, "return_indices", False):
            return None
        out = m.output_size if isinstance(m.output_size, (tuple, list)) else (m.output_size, m.output_size)
        # resolved to a fixed pool when the input size is known (plan_for): an adaptive pool whose
        # input size is a multiple of its output size is a pool with k = s = in / out
        return {"kind": "adaptive_avg" if isinstance(m, nn.AdaptiveAvgPool2d) else "adaptive_max", "out": tuple(out)}
    if isinstance(m, (nn.Identity, nn.Dropout, nn.Dropout2d)):
        return {}  # identity at inference time
    return None


def find_runs(seq: nn.Sequential) -> List[Tuple[int, int]]:
    """Maximal runs [start, stop) of consecutive optimizable children of `seq` that contain at
    least one real layer (the aggregation detection of Figure 4)."""
    runs, start, real = [], None, 0
    mods = list(seq.children())
    for i, m in enumerate(mods + [None]):
        d = layer_desc(m) if m is not None and not isinstance(m, BrainSlugStack) else None
        if d is None:
            if start is not None and real > 0:
                runs.append((start, i))
            start, real = None, 0
        else:
            if start is None:
                start = i
            real += 1 if d else 0
    return runs


def resolve_layers(layers: List[dict], shape) -> List[dict]:
    """Concrete layer list for an input of `shape`: adaptive pools become fixed pools."""
    h, w = int(shape[2]), int(shape[3])
    out = []
    for l in layers:
        if l["kind"] in ("adaptive_avg", "adaptive_max"):
            oh = h if l["out"][0] is None else int(l["out"][0])
            ow = w if l["out"][1] is None else int(l["out"][1])
            if oh < 1 or ow < 1 or h % oh or w % ow:
                raise RuntimeError(f"adaptive pooling of a {h}x{w} plane to {oh}x{ow}: only sizes that divide "
                                   "the input are supported")
            k = (h // oh, w // ow)
            l = ({"kind": "avgpool", "k": k, "s": k, "p": (0, 0), "count_include_pad": True}
                 if l["kind"] == "adaptive_avg" else
                 {"kind": "maxpool", "k": k, "s": k, "p": (0, 0), "return_indices": False})
        if l["kind"] in ("maxpool", "avgpool"):
            h = wl.pool_out(h, l["k"][0], l["s"][0], l["p"][0], l.get("ceil_mode", False))
            w = wl.pool_out(w, l["k"][1], l["s"][1], l["p"][1], l.get("ceil_mode", False))
        out.append(l)
    return out


class BrainSlugStack(nn.Module):
    """A run of optimizable layers executed depth-first by the HIP library."""

    def __init__(self, modules: List[nn.Module], **plan_opts):
        super().__init__()
        self.replaced = [type(m).__name__ for m in modules]
        self.layers = [d for d in (layer_desc(m) for m in modules) if d]
        if any(d is None for d in (layer_desc(m) for m in modules)) or not self.layers:
            raise ValueError("BrainSlugStack needs a non-empty run of optimizable layers")
        self.channels = next((len(l["gamma"]) for l in self.layers if l["kind"] == "bn"), None)
        self.plan_opts = dict(plan_opts)
        self._plans: Dict[tuple, bs.Stack] = {}

    def extra_repr(self) -> str:
        return "replaces " + " -> ".join(self.replaced)

    def plan_for(self, shape, dtype: torch.dtype) -> bs.Stack:
        """The planned stack for this input shape and dtype (cached)."""
        key = (tuple(int(v) for v in shape), dtype)
        st = self._plans.get(key)
        if st is None:
            name = {torch.float32: "f32", torch.bfloat16: "bf16", torch.float16: "f16"}.get(dtype)
            if name is None:
                raise TypeError(f"BrainSlugStack supports float32, bfloat16 and float16 tensors, not {dtype}")
            st = bs.Stack(resolve_layers(self.layers, key[0]), key[0], name).plan(**self.plan_opts)
            self._plans[key] = st
        return st

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        if self.training:
            raise RuntimeError("BrainSlugStack implements the inference forward pass only: call model.eval()")
        if not x.is_cuda or x.dim() != 4:
            raise RuntimeError("BrainSlugStack needs a 4-D NCHW tensor on the GPU")
        if self.channels is not None and x.shape[1] != self.channels:
            raise RuntimeError(f"expected {self.channels} channels, got {x.shape[1]}")
        with torch.no_grad():
            st = self.plan_for(x.shape, x.dtype)
            # a channel slice of a concatenation buffer is read in place; other layouts are copied
            if bs.batch_stride(x) is None or (x.data_ptr() % 16) or (x.stride(0) * x.element_size()) % 16:
                x = x.contiguous()
            out, _ = st.run(x, indices=[])
        return out

    def close(self) -> None:
        for st in self._plans.values():
            st.close()
        self._plans.clear()


def optimize(model: nn.Module, min_layers: int = 1, **plan_opts) -> nn.Module:
    """Rewrite `model` in place (and return it): every run of at least `min_layers` consecutive
    optimizable layers inside a Sequential becomes one BrainSlugStack.  `plan_opts` are passed to
    `bs_stack_plan` (e.g. max_steps_per_sequence)."""
    model.optimized_stacks = []
    for parent in [m for m in model.modules() if isinstance(m, nn.Sequential)]:
        names = list(parent._modules.keys())
        mods = [parent._modules[n] for n in names]
        for start, stop in find_runs(parent):
            real = [m for m in mods[start:stop] if layer_desc(m)]
            if len(real) < min_layers:
                continue
            stack = BrainSlugStack(mods[start:stop], **plan_opts)
            stack.train(parent.training)
            parent._modules[names[start]] = stack
            for n in names[start + 1:stop]:
                parent._modules[n] = nn.Identity()
            model.optimized_stacks.append(stack)
    return model
