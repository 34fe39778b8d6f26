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

`optimize` rewrites `Sequential` containers only: they are the only modules whose children are
known to execute in order, one feeding the next.  Everything else (convolutions, the model's own
`forward`) keeps running in PyTorch.

`optimize_graph(model)` sees through hand-written `forward` methods as well: it records the model's
data flow with `torch.fx`, follows every chain of optimizable operations -- layer modules, their
functional forms (`F.relu`, `F.max_pool2d`, ...) and tensor additions written as `a + b`,
`a += b` or `torch.add(a, b)` -- and replaces each chain by one `BrainSlugStack` call whose extra
arguments are the residual operands.  This covers the residual blocks of a ResNet (BatchNorm ->
Add -> ReLU) and the pre-activation / transition layers of a DenseNet, whose layers are not
children of one `Sequential`.

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

__all__ = ["optimize", "optimize_graph", "capture", "CapturedModel", "find_chains", "BrainSlugStack", "PrefixConcat", "ConcatSink", "CaptureOnlyStack",
           "layer_desc", "find_runs", "resolve_layers"]


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
        # "module": where the parameters come from, so that a stack can notice when they change
        return {"kind": "bn", "gamma": f(m.weight, ones), "beta": f(m.bias, zeros),
                "mean": f(m.running_mean, zeros), "var": f(m.running_var, ones), "eps": float(m.eps), "module": m}
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


class _StackFunction(torch.autograd.Function):
    """A stack as one node of the autograd graph: the forward pass keeps only the stack's operands
    (no intermediate tensor exists to keep), the backward pass recomputes what it needs from them
    (`bs_stack_backward`).  BatchNorm is the inference-mode layer with its parameters folded in when the
    stack was built: they get no gradient (frozen BatchNorm; freeze them in the original model as well
    when comparing the two)."""

    @staticmethod
    def forward(ctx, module, nhwc, stride, x, *residuals):
        # x: dense in the plan's memory format, or (stride != 0) a channel slice that is read in place
        st = module.plan_for(x.shape, x.dtype, nhwc, keep_picks=True)
        mf = torch.channels_last if nhwc else torch.contiguous_format
        out = torch.empty(st.out_shape, dtype=x.dtype, device=x.device, memory_format=mf)
        # the last max pooling's picks, where the plan writes them, are kept for the backward pass
        # (saves recomputing them)
        picks = [torch.empty(sh, dtype=torch.int32, device=x.device, memory_format=mf) for sh in st.idx_shapes] or None
        st.run_unchecked(x, list(residuals), out, stride, 0, picks)
        ctx.save_for_backward(x, *residuals)
        ctx.stack, ctx.mf, ctx.picks, ctx.stride, ctx.nhwc = st, mf, picks, stride, nhwc
        return out

    @staticmethod
    def backward(ctx, grad_out):
        x, *residuals = ctx.saved_tensors
        need = ctx.needs_input_grad  # (module, nhwc, stride, x, *residuals)
        mf = ctx.mf
        gx = torch.empty(x.shape, dtype=x.dtype, device=x.device, memory_format=mf) if need[3] else None
        gres = [torch.empty_like(r, memory_format=mf) if wanted else None for r, wanted in zip(residuals, need[4:])]
        # operands validated in forward(); the upstream gradient has the output's shape and dtype and is
        # read in place when it is dense or a channel slice (a gradient buffer's channel range)
        gstride = BrainSlugStack._slice_stride(grad_out, ctx.stack.out_shape, x, ctx.nhwc)
        if gstride is None:
            grad_out, gstride = grad_out.contiguous(memory_format=mf), 0
        ctx.stack.backward_unchecked(x, residuals, grad_out, gx, gres, ctx.picks, ctx.stride, gstride, 0)
        return (None, None, None, gx, *gres)


class BrainSlugStack(nn.Module):
    """A run of optimizable layers executed depth-first by the HIP library.  Inference-mode layers
    (BatchNorm with its running statistics); gradients flow through it to its input and its residual
    operands when autograd records the call (fine-tuning with frozen BatchNorm layers)."""

    def __init__(self, modules: List[nn.Module], **plan_opts):
        descs = [layer_desc(m) for m in modules]
        if any(d is None for d in descs):
            raise ValueError("BrainSlugStack needs a non-empty run of optimizable layers")
        self._init([d for d in descs if d], [type(m).__name__ for m in modules], plan_opts)

    @classmethod
    def from_layers(cls, layers: List[dict], replaced: List[str], **plan_opts) -> "BrainSlugStack":
        """A stack from layer descriptions (see `layer_desc`); `replaced` names what it stands for."""
        self = cls.__new__(cls)
        self._init([dict(l) for l in layers if l], list(replaced), plan_opts)
        return self

    def _init(self, layers, replaced, plan_opts):
        nn.Module.__init__(self)
        if not layers:
            raise ValueError("BrainSlugStack needs a non-empty run of optimizable layers")
        self.replaced = replaced
        self.layers = layers
        self.n_residuals = sum(1 for l in layers if l["kind"] == "add")
        self.channels = next((len(l["gamma"]) for l in self.layers if l["kind"] == "bn"), None)
        self.plan_opts = dict(plan_opts)
        self._plans: Dict[tuple, bs.Stack] = {}
        # BatchNorm parameters are folded when a plan is made.  The stack keeps the modules they came
        # from (not as sub-modules: they stay where they are in the model) and looks at their tensors'
        # versions and addresses before every call: after load_state_dict, .half(), an in-place update
        # or a moving average the parameters are read again and the plans made anew (Section 4.2: the
        # front-end hands over the parameter tensors at run time).  Layer descriptions without a
        # source module (from_layers with plain arrays) are fixed.
        object.__setattr__(self, "_bn_modules", [l.get("module") for l in layers if l["kind"] == "bn"])
        self._bn_seen = self._bn_state()

    def _bn_state(self) -> tuple:
        st = []
        for m in self._bn_modules:
            if m is not None:
                for t in (m.weight, m.bias, m.running_mean, m.running_var):
                    st.append(None if t is None else (t.data_ptr(), t._version))
        return tuple(st)

    def sync_parameters(self) -> bool:
        """Re-read the BatchNorm parameters from their modules if any of their tensors changed
        since they were last read; the plans are then made anew at the next call.  Called by
        `forward`.  Returns whether anything changed."""
        state = self._bn_state()
        if state == self._bn_seen:
            return False
        for l in self.layers:
            if l["kind"] == "bn" and l.get("module") is not None:
                fresh = layer_desc(l["module"])
                if fresh is None or len(fresh["gamma"]) != len(l["gamma"]):
                    raise RuntimeError("a BatchNorm module of a BrainSlugStack no longer is an inference-mode "
                                       "BatchNorm of the same width")
                l.update(fresh)
        for st in self._plans.values():
            st.close()
        self._plans.clear()
        self._bn_seen = state
        return True

    def extra_repr(self) -> str:
        return "replaces " + " -> ".join(self.replaced)

    def plan_for(self, shape, dtype: torch.dtype, channels_last: bool = False, keep_picks: bool = False) -> bs.Stack:
        """The planned stack for this input shape, dtype and memory format (cached).  `keep_picks`
        (the plan autograd records): when the stack's last pooling layer is a max pooling whose
        picks the backward pass would have to recompute, the forward pass writes them out."""
        key = (tuple(int(v) for v in shape), dtype, bool(channels_last), bool(keep_picks))
        st = self._plans.get(key)
        if st is None:
            name = {torch.float32: "f32", torch.bfloat16: "bf16", torch.float16: "f16"}.get(dtype)
            if name is None:
                raise TypeError(f"BrainSlugStack supports float32, bfloat16 and float16 tensors, not {dtype}")
            layers = resolve_layers(self.layers, key[0])
            if keep_picks:
                layers = self._with_saved_picks(layers, key[0])
            opts = dict(self.plan_opts)
            if channels_last:
                # channels-last plans have their own kernels: options that pick or tune the
                # NCHW ones do not apply
                opts = {k: v for k, v in opts.items() if k in ("threads_per_group", "num_cus")}
                opts["layout"] = bs.BS_LAYOUT_NHWC
            st = bs.Stack(layers, key[0], name).plan(**opts)
            st.layers = layers
            st.res_shapes = [tuple(v) for v in wl.residual_shapes(layers, key[0])]
            self._plans[key] = st
        return st

    @staticmethod
    def _with_saved_picks(layers, shape):
        """`layers` with an index output on the last pooling layer, if that is a max pooling other than
        2 x 2 / 2 windows that tile the plane (those the backward kernel finds again by itself)."""
        pools = [i for i, l in enumerate(layers) if l["kind"] in ("maxpool", "avgpool")]
        if not pools or layers[pools[-1]]["kind"] != "maxpool":
            return layers
        i = pools[-1]
        l = layers[i]
        h, w = wl.output_shape(layers[:i], shape)[2:]
        if l["k"] == (2, 2) and l["s"] == (2, 2) and l["p"] == (0, 0) and h % 2 == 0 and w % 2 == 0:
            return layers
        return layers[:i] + [dict(l, return_indices=True)] + layers[i + 1:]

    def forward(self, x: torch.Tensor, *residuals: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """`residuals`: the second operand of every Add layer of the stack, in layer order.  `out`:
        where to write the result -- a tensor of the output's shape, dense in the input's memory
        format or a channel slice of such a tensor (a concatenation buffer); when it does not fit
        (shape, type, alignment) it is ignored and a new tensor is returned."""
        if self.training:
            raise RuntimeError("BrainSlugStack implements inference-mode layers only (BatchNorm with running "
                               "statistics): call model.eval(); gradients still flow in that mode")
        if not x.is_cuda:
            raise RuntimeError("BrainSlugStack needs a tensor on the GPU")
        if x.dim() != 4:
            # the activations between fully connected layers: element-wise layers without
            # per-channel parameters do not care about the shape, so the tensor runs as one row
            if any(l["kind"] not in ("relu", "leaky_relu", "clamp", "add") for l in self.layers):
                raise RuntimeError("BrainSlugStack needs a 4-D NCHW tensor for BatchNorm and pooling layers")
            if any(tuple(r.shape) != tuple(x.shape) for r in residuals):
                raise RuntimeError("residual operands must have the input's shape (no broadcasting)")
            flat = self.forward(x.contiguous().view(1, 1, 1, -1), *[r.contiguous().view(1, 1, 1, -1) for r in residuals])
            return flat.view(x.shape)
        if self._bn_seen:
            self.sync_parameters()
        if self.channels is not None and x.shape[1] != self.channels:
            raise RuntimeError(f"expected {self.channels} channels, got {x.shape[1]}")
        if torch.is_grad_enabled() and (x.requires_grad or any(r.requires_grad for r in residuals)):
            # recorded by autograd: the input dense in its memory format or a channel slice of a
            # concatenation buffer (read in place, forward and backward), dense residual operands, a
            # new output tensor (`out` is not used)
            if len(residuals) != self.n_residuals:
                raise RuntimeError(f"stack has {self.n_residuals} Add layers, got {len(residuals)} residual tensors")
            x, stride, nhwc = self._input_slice(x)
            mf = torch.channels_last if nhwc else torch.contiguous_format
            st = self.plan_for(x.shape, x.dtype, nhwc, keep_picks=True)
            for r, want in zip(residuals, st.res_shapes):
                if r.shape != want or r.dtype != x.dtype or r.device != x.device:
                    raise RuntimeError(f"residual operand of shape {tuple(r.shape)} / {r.dtype}: the Add layer "
                                       f"needs {tuple(want)} / {x.dtype} on the input's device (no broadcasting)")
            return _StackFunction.apply(self, nhwc, stride, x, *[r.contiguous(memory_format=mf) for r in residuals])
        with torch.no_grad():
            # a channels_last tensor stays channels_last: the stack is planned for that memory
            # order and its output is channels_last as well (what the convolutions around it use)
            # a channel slice of a concatenation buffer (of either memory format) is read in
            # place; other layouts are copied
            x, stride, nhwc = self._input_slice(x)
            st = self._plans.get((x.shape, x.dtype, nhwc, False)) or self.plan_for(x.shape, x.dtype, nhwc)
            mf = torch.channels_last if nhwc else torch.contiguous_format
            if len(residuals) != self.n_residuals:
                raise RuntimeError(f"stack has {self.n_residuals} Add layers, got {len(residuals)} residual tensors")
            res = []
            for r, want in zip(residuals, st.res_shapes):
                if r.shape != want or r.dtype != x.dtype or r.device != x.device:
                    raise RuntimeError(f"residual operand of shape {tuple(r.shape)} / {r.dtype}: the Add layer "
                                       f"needs {tuple(want)} / {x.dtype} on the input's device (no broadcasting)")
                res.append(r.contiguous(memory_format=mf))
            # dense tensors of the plan's layout, or validated channel slices as input / output
            ostride = 0
            if out is not None:
                ostride = self._slice_stride(out, st.out_shape, x, nhwc)
                if ostride is None:
                    out = None
            if out is None:
                out, ostride = torch.empty(st.out_shape, dtype=x.dtype, device=x.device, memory_format=mf), 0
            st.run_unchecked(x, res, out, stride, ostride)
        return out

    @staticmethod
    def _input_slice(x):
        """(tensor, batch stride, channels-last?) to run on: `x` itself when it is dense in either memory
        format (stride 0) or a channel slice of a dense tensor that can be read in place, else a dense copy."""
        stride, nhwc = 0, False
        if not x.is_contiguous():
            nhwc = x.is_contiguous(memory_format=torch.channels_last)
            if not nhwc:
                es = x.element_size()
                stride = bs.batch_stride(x)
                if stride is None or (x.data_ptr() % 16) or (stride * es) % 16:
                    stride = bs.batch_stride_nhwc(x)
                    hw = x.shape[2] * x.shape[3]
                    if stride is None or (x.data_ptr() % 16) or (stride // hw * es) % 16:
                        x, stride = x.contiguous(), 0
                    else:
                        nhwc = True
        return x, stride, nhwc

    @staticmethod
    def _slice_stride(t, shape, like, nhwc):
        """Batch stride to pass for `t` as an output of `shape` (0: dense), or None when `t` cannot be
        written in place."""
        if t.shape != shape or t.dtype != like.dtype or t.device != like.device or (t.data_ptr() % 16):
            return None
        if t.is_contiguous(memory_format=torch.channels_last if nhwc else torch.contiguous_format):
            return 0
        es = t.element_size()
        if nhwc:
            stride = bs.batch_stride_nhwc(t)
            return stride if stride is not None and (stride // (shape[2] * shape[3]) * es) % 16 == 0 else None
        stride = bs.batch_stride(t)
        return stride if stride is not None and (stride * es) % 16 == 0 else None

    def close(self) -> None:
        for st in self._plans.values():
            st.close()
        self._plans.clear()


def _lone_activation(layers: List[dict]) -> bool:
    """Is the run a single activation layer (plus identities)?  Nothing is fused then, and the
    framework's own in-place activation moves the same bytes with a cheaper call (measured:
    SqueezeNet, whose stacks are almost all lone ReLUs, ran 3..12 % slower with them replaced)."""
    real = [l for l in layers if l]
    return len(real) == 1 and real[0]["kind"] in ("relu", "leaky_relu", "clamp")


def optimize(model: nn.Module, min_layers: int = 1, lone_activations: bool = False, **plan_opts) -> nn.Module:
    """Rewrite `model` in place (and return it): every run of at least `min_layers` consecutive
    optimizable layers inside a Sequential becomes one BrainSlugStack.  A run that is a single
    activation layer stays in PyTorch unless `lone_activations` is set.  `plan_opts` are passed
    to `bs_stack_plan` (e.g. max_steps_per_sequence)."""
    model.optimized_stacks = []
    for parent in [m for m in model.modules() if isinstance(m, nn.Sequential)]:
        names = list(parent._modules.keys())
        mods = [parent._modules[n] for n in names]
        for start, stop in find_runs(parent):
            real = [m for m in mods[start:stop] if layer_desc(m)]
            if len(real) < min_layers or (not lone_activations and _lone_activation([layer_desc(m) for m in real])):
                continue
            stack = BrainSlugStack(mods[start:stop], **plan_opts)
            stack.train(parent.training)
            parent._modules[names[start]] = stack
            for n in names[start + 1:stop]:
                parent._modules[n] = nn.Identity()
            model.optimized_stacks.append(stack)
    return model


# ---------------------------------------------------------------------------- data-flow graphs
def _fn_args(node, names, defaults):
    """Positional / keyword arguments of a call node as a dict over `names`."""
    vals = dict(zip(names, node.args))
    vals.update(node.kwargs)
    if set(vals) - set(names):
        return None
    return {n: vals.get(n, defaults.get(n)) for n in names}


def _const(v) -> bool:
    """True when an argument is a plain Python value (not computed in the graph)."""
    from torch import fx
    if isinstance(v, fx.Node):
        return False
    if isinstance(v, (tuple, list)):
        return all(_const(e) for e in v)
    return v is None or isinstance(v, (int, float, bool))


def _node_desc(node, modules):
    """(layer dict or {} , main input node, residual node or None, display name) for an fx node
    the library can take, else None."""
    import operator

    import torch.nn.functional as F
    from torch import fx

    def unary(desc, name, a):
        return (desc, a, None, name) if isinstance(a, fx.Node) else None

    if node.op == "call_module":
        m = modules.get(node.target)
        if m is None or isinstance(m, BrainSlugStack) or len(node.args) != 1 or node.kwargs:
            return None
        d = layer_desc(m)
        return None if d is None else unary(d, type(m).__name__, node.args[0])

    if node.op == "call_function":
        t = node.target
        if t in (operator.add, operator.iadd, torch.add):
            if len(node.args) != 2 or (node.kwargs and node.kwargs.get("alpha", 1) != 1) or \
                    set(node.kwargs) - {"alpha"}:
                return None
            a, b = node.args
            if not (isinstance(a, fx.Node) and isinstance(b, fx.Node)) or a is b:
                return None  # a tensor plus a number, or x + x: not a residual Add
            return ({"kind": "add"}, a, b, "add")
        if t in (F.relu, torch.relu, torch.relu_, F.relu_):
            v = _fn_args(node, ["input", "inplace"], {"inplace": False})
            return None if v is None or not _const(v["inplace"]) else unary({"kind": "relu"}, "relu", v["input"])
        if t is F.leaky_relu:
            v = _fn_args(node, ["input", "negative_slope", "inplace"], {"negative_slope": 0.01, "inplace": False})
            if v is None or not _const(v["negative_slope"]):
                return None
            return unary({"kind": "leaky_relu", "slope": float(v["negative_slope"])}, "leaky_relu", v["input"])
        if t is F.relu6:
            v = _fn_args(node, ["input", "inplace"], {"inplace": False})
            return None if v is None else unary({"kind": "clamp", "lo": 0.0, "hi": 6.0}, "relu6", v["input"])
        if t is F.hardtanh:
            v = _fn_args(node, ["input", "min_val", "max_val", "inplace"], {"min_val": -1.0, "max_val": 1.0, "inplace": False})
            if v is None or not (_const(v["min_val"]) and _const(v["max_val"])):
                return None
            return unary({"kind": "clamp", "lo": float(v["min_val"]), "hi": float(v["max_val"])}, "hardtanh", v["input"])
        if t is F.max_pool2d:
            v = _fn_args(node, ["input", "kernel_size", "stride", "padding", "dilation", "ceil_mode", "return_indices"],
                         {"stride": None, "padding": 0, "dilation": 1, "ceil_mode": False, "return_indices": False})
            if v is None or not all(_const(v[k]) for k in v if k != "input") or v["return_indices"]:
                return None
            if _pair(v["dilation"]) != (1, 1):
                return None
            k = _pair(v["kernel_size"])
            d = {"kind": "maxpool", "k": k, "s": _pair(v["stride"] if v["stride"] not in (None, [], ()) else k),
                 "p": _pair(v["padding"]), "return_indices": False, "ceil_mode": bool(v["ceil_mode"])}
            return unary(d, "max_pool2d", v["input"])
        if t is F.avg_pool2d:
            v = _fn_args(node, ["input", "kernel_size", "stride", "padding", "ceil_mode", "count_include_pad",
                                "divisor_override"],
                         {"stride": None, "padding": 0, "ceil_mode": False, "count_include_pad": True,
                          "divisor_override": None})
            if v is None or not all(_const(v[k]) for k in v if k != "input") or v["divisor_override"] is not None:
                return None
            k = _pair(v["kernel_size"])
            d = {"kind": "avgpool", "k": k, "s": _pair(v["stride"] if v["stride"] not in (None, [], ()) else k),
                 "p": _pair(v["padding"]), "count_include_pad": bool(v["count_include_pad"]),
                 "ceil_mode": bool(v["ceil_mode"])}
            return unary(d, "avg_pool2d", v["input"])
        if t in (F.adaptive_avg_pool2d, F.adaptive_max_pool2d):
            v = _fn_args(node, ["input", "output_size", "return_indices"], {"return_indices": False})
            if v is None or not _const(v["output_size"]) or v["return_indices"]:
                return None
            o = v["output_size"]
            o = tuple(o) if isinstance(o, (tuple, list)) else (o, o)
            kind = "adaptive_avg" if t is F.adaptive_avg_pool2d else "adaptive_max"
            return unary({"kind": kind, "out": o}, t.__name__, v["input"])
        return None

    if node.op == "call_method":
        if node.target in ("add", "add_") and len(node.args) == 2 and not node.kwargs:
            a, b = node.args
            if isinstance(a, fx.Node) and isinstance(b, fx.Node) and a is not b:
                return ({"kind": "add"}, a, b, node.target)
            return None
        if node.target in ("relu", "relu_") and len(node.args) == 1 and not node.kwargs:
            return unary({"kind": "relu"}, node.target, node.args[0])
    return None


def _writes_in_place(node, modules) -> bool:
    """Does the operation overwrite its first operand (ReLU(inplace=True), `a += b`, `relu_`)?"""
    import operator

    if node.op == "call_module":
        return bool(getattr(modules.get(node.target), "inplace", False))
    if node.op == "call_method":
        return node.target.endswith("_")
    if node.op == "call_function":
        if node.target in (operator.iadd, operator.isub, operator.imul, operator.itruediv, torch.relu_,
                           torch.nn.functional.relu_) or node.kwargs.get("out") is not None:
            return True
        F = torch.nn.functional
        if node.target in (F.relu, F.leaky_relu, F.relu6, F.hardtanh):  # `inplace` is their last parameter
            last = node.args[-1] if len(node.args) > 1 and isinstance(node.args[-1], bool) else False
            return bool(node.kwargs.get("inplace", last))
    return False


class Chain:
    """One chain of optimizable graph nodes: `nodes[i + 1]` consumes `nodes[i]` and nothing else does."""

    def __init__(self, source):
        self.source = source      # node that produces the chain's input
        self.nodes = []           # graph nodes, in execution order
        self.layers = []          # their layer descriptions ({} for inference-time identities)
        self.names = []
        self.residuals = []       # second operand of every Add, in order

    def real_layers(self) -> int:
        return sum(1 for l in self.layers if l)


def find_chains(gm) -> List[Chain]:
    """Aggregation detection on a traced model (Figure 4 on a data-flow graph instead of a layer
    list): maximal chains of optimizable nodes in which every intermediate result has exactly one
    consumer, the next node of the chain.  For an addition the chain continues through the operand
    that ends a chain (the first one if both do); the other operand is a residual input."""
    modules = dict(gm.named_modules())
    tail_of: Dict[object, Chain] = {}   # node that currently ends an open chain -> chain
    chains: List[Chain] = []
    for node in gm.graph.nodes:
        d = _node_desc(node, modules)
        if d is None:
            continue
        desc, a, b, name = d
        if _writes_in_place(node, modules) and len(a.users) > 1:
            # the model overwrites a tensor that something else reads as well: what that reader
            # sees depends on execution order, which a fused chain would change.  Left to PyTorch.
            continue

        def extendable(n):
            return n is not None and n in tail_of and len(n.users) == 1

        if b is not None and not extendable(a) and extendable(b):
            a, b = b, a  # addition commutes bit for bit: continue the chain that ends in b
        if extendable(a):
            ch = tail_of.pop(a)
        else:
            ch = Chain(a)
            chains.append(ch)
        ch.nodes.append(node)
        ch.layers.append(desc)
        ch.names.append(name)
        if b is not None:
            ch.residuals.append(b)
        tail_of[node] = ch
    # A chain runs where its last node stood.  Should the model overwrite one of the chain's
    # inputs between the chain's first and last node, the chain would read the new contents
    # where the model read the old: such chains are left to PyTorch.
    order = {n: i for i, n in enumerate(gm.graph.nodes)}

    def overwritten(ch):
        lo, hi = order[ch.nodes[0]], order[ch.nodes[-1]]
        for v in [ch.source, *ch.residuals]:
            for u in v.users:
                if lo < order[u] < hi and u not in ch.nodes and u.args and u.args[0] is v and \
                        _writes_in_place(u, modules):
                    return True
        return False

    return [c for c in chains if c.real_layers() > 0 and not overwritten(c)]


class PrefixConcat(nn.Module):
    """The growing concatenations of a densely connected block -- cat([t0]), cat([t0, t1]),
    cat([t0, t1, t2]), ... along the channel axis, each feeding a stack -- without copying
    every earlier tensor again for every later concatenation: one buffer per forward pass holds
    the largest concatenation, every part is copied into its channel range once, and the result
    of the k-th concatenation is the view `buffer[:, :c_k]`, a channel slice that the stacks read
    in place (`bs_stack_run_strided`).  The copy traffic of a block with L layers drops from
    O(L^2) to O(L) tensors.

    The channel counts are learnt in the first forward pass (which concatenates the ordinary
    way); any call the bookkeeping cannot vouch for -- other shapes, parts that are not the
    tensors copied earlier in this pass, gradients being recorded -- concatenates the ordinary
    way as well.

    Measured on DenseNet-121 (batch 32): replayed from a HIP graph the shared buffer makes the
    forward pass 9 % faster; run eagerly, where that network is bound by the host's launch rate,
    the three tensor operations per call that replace one `torch.cat` make it 6 % slower.  Hence
    `when="capture"`: views while a graph is being captured, the ordinary concatenation
    otherwise; `when="always"` shares in both cases."""

    def __init__(self, positions: int, when: str = "always"):
        super().__init__()
        if when not in ("always", "capture"):
            raise ValueError("when must be 'always' or 'capture'")
        self.positions = positions   # concatenations in the family, smallest first
        self.when = when             # "capture": share the buffer only while a HIP graph is being captured
        self.known = None            # (N, H, W, dtype, device, total channels) of the last full pass
        self._buf = None
        self._parts = []             # data pointers of the parts already in the buffer
        self._channels = 0           # channels of the buffer filled so far
        self._format = torch.contiguous_format
        self.views_returned = 0      # concatenations answered with a view of the buffer

    def forward(self, position: int, *parts: torch.Tensor) -> torch.Tensor:
        first = parts[0]
        if position == 0:
            self._buf, self._parts, self._channels = None, [], 0
            k = self.known
            if self.when == "capture" and not (first.is_cuda and torch.cuda.is_current_stream_capturing()):
                k = None
            if k is not None and first.dim() == 4 and \
                    (first.shape[0], first.shape[2], first.shape[3], first.dtype, first.device) == k[:5]:
                # the buffer has the parts' memory format: NCHW, or channels_last
                self._format = torch.contiguous_format if first.is_contiguous() else torch.channels_last
                self._buf = torch.empty((k[0], k[5], k[1], k[2]), dtype=k[3], device=k[4], memory_format=self._format)
        buf, old = self._buf, self._parts
        if buf is not None and len(parts) >= len(old):
            # the parts copied earlier in this pass must be the same tensors (by address); the new
            # ones are checked in full
            good = not torch.is_grad_enabled() or not any(p.requires_grad for p in parts)
            for i in range(len(old)):
                good = good and parts[i].data_ptr() == old[i]
            new, c = parts[len(old):], self._channels
            plane = buf.shape[2:]
            for p in new:
                good = good and p.dim() == 4 and p.shape[2:] == plane and p.shape[0] == buf.shape[0] and \
                    p.dtype == buf.dtype and p.device == buf.device and p.is_contiguous(memory_format=self._format)
            if good and c + sum(p.shape[1] for p in new) <= buf.shape[1]:
                for p in new:
                    buf.narrow(1, c, p.shape[1]).copy_(p)
                    c += p.shape[1]
                    old.append(p.data_ptr())
                self._channels = c
                self.views_returned += 1
                return buf if c == buf.shape[1] else buf.narrow(1, 0, c)
        # the ordinary way; the largest concatenation of a pass teaches the buffer size
        self._buf = None
        out = torch.cat(parts, 1)
        if position == self.positions - 1 and first.dim() == 4 and not out.requires_grad:
            self.known = (first.shape[0], first.shape[2], first.shape[3], first.dtype, first.device, out.shape[1])
        return out


class CaptureOnlyStack(nn.Module):
    """A lone activation layer that runs as a stack only while a HIP graph is being captured and
    as the framework's own operation otherwise.  Alone it has nothing to fuse, and run eagerly the
    framework's call is cheaper; in a captured graph the call costs nothing and the stack can write
    its result straight into a concatenation (`ConcatSink`), which saves the copy (SqueezeNet
    replayed from a graph: 9..25 % faster with its lone ReLUs taken, 7..17 % slower when they are
    taken in eager mode)."""

    def __init__(self, stack: BrainSlugStack):
        super().__init__()
        self.stack = stack
        (layer,) = stack.layers
        if layer["kind"] == "relu":
            self.eager = torch.relu
        elif layer["kind"] == "leaky_relu":
            self.eager = lambda x, slope=layer["slope"]: torch.nn.functional.leaky_relu(x, slope)
        else:
            self.eager = lambda x, lo=layer["lo"], hi=layer["hi"]: torch.clamp(x, lo, hi)

    def forward(self, x: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        if x.is_cuda and torch.cuda.is_current_stream_capturing():
            return self.stack(x, out=out)
        return self.eager(x)


class ConcatSink(nn.Module):
    """A channel concatenation some of whose parts are produced by stacks: those stacks write
    their result straight into their channel range of the concatenated tensor (a channel slice
    as stack output, `bs_stack_run_strided`), the other parts are copied in as `torch.cat` would,
    and the concatenation itself disappears for the stack-made parts.

    Three small modules share this state and are called in graph order: `begin` before the first
    part is computed (it allocates the buffer), `slot(i)` before stack part i (it hands out the
    view to write into) and `finish` where the concatenation stood.  Shapes are learnt in the
    first forward pass, which concatenates the ordinary way; `when` as for `PrefixConcat`."""

    def __init__(self, n_parts: int, when: str = "capture"):
        super().__init__()
        self.n_parts, self.when = n_parts, when
        self.known = None    # (N, H, W, dtype, device, memory format, channels per part)
        self._buf, self._offsets = None, None
        self.in_place = 0    # parts that arrived already in place

    def begin(self, like: torch.Tensor) -> torch.Tensor:
        self._buf = None
        k = self.known
        if k is not None and like.is_cuda and (self.when == "always" or torch.cuda.is_current_stream_capturing()) and \
                not (torch.is_grad_enabled() and like.requires_grad) and like.dim() == 4 and \
                (like.shape[0], like.dtype, like.device) == (k[0], k[3], k[4]):
            self._buf = torch.empty((k[0], sum(k[6]), k[1], k[2]), dtype=k[3], device=k[4], memory_format=k[5])
        return like

    def slot(self, i: int) -> Optional[torch.Tensor]:
        if self._buf is None:
            return None
        c = self.known[6]
        return self._buf.narrow(1, sum(c[:i]), c[i])

    def finish(self, *parts: torch.Tensor) -> torch.Tensor:
        buf, k = self._buf, self.known
        self._buf = None
        first = parts[0]
        if buf is not None and len(parts) == len(k[6]) and \
                all(p.dim() == 4 and p.shape[1] == c and p.shape[0] == k[0] and p.shape[2:] == buf.shape[2:] and
                    p.dtype == buf.dtype and p.device == buf.device for p, c in zip(parts, k[6])):
            off = 0
            for p, c in zip(parts, k[6]):
                view = buf.narrow(1, off, c)
                if p.data_ptr() == view.data_ptr() and p.stride() == view.stride():
                    self.in_place += 1
                else:
                    view.copy_(p)
                off += c
            return buf
        out = torch.cat(parts, 1)
        if first.dim() == 4 and not out.requires_grad:
            mf = torch.contiguous_format if out.is_contiguous() else torch.channels_last
            if out.is_contiguous(memory_format=mf):
                self.known = (out.shape[0], out.shape[2], out.shape[3], out.dtype, out.device, mf,
                              tuple(p.shape[1] for p in parts))
        return out


class _SinkBegin(nn.Module):
    def __init__(self, sink):
        super().__init__()
        self.sink = sink

    def forward(self, like):
        return self.sink.begin(like)


class _SinkSlot(nn.Module):
    def __init__(self, sink, index):
        super().__init__()
        self.sink, self.index = sink, index

    def forward(self, token):  # `token`: the result of `begin`, so that the slot is taken after it
        return self.sink.slot(self.index)


class _SinkFinish(nn.Module):
    def __init__(self, sink):
        super().__init__()
        self.sink = sink

    def forward(self, *parts):
        return self.sink.finish(*parts)


def _sink_parts(node, stack_names):
    """(parts, indices of the parts a stack call produces for this node alone) of a channel
    concatenation that has at least one such part, else None."""
    from torch import fx

    if not (node.op == "call_function" and node.target in (torch.cat, torch.concat)):
        return None
    args = list(node.args) + [node.kwargs.get("dim", 0)] if len(node.args) == 1 else list(node.args)
    if not (len(args) == 2 and args[1] == 1 and isinstance(args[0], (list, tuple)) and len(args[0]) >= 2 and
            all(isinstance(a, fx.Node) for a in args[0]) and set(node.kwargs) <= {"dim"} and
            len(set(args[0])) == len(args[0])):
        return None
    parts = tuple(args[0])
    mine = [i for i, a in enumerate(parts)
            if a.op == "call_module" and a.target in stack_names and len(a.users) == 1 and "out" not in a.kwargs]
    return (parts, mine) if mine else None


def _concat_families(gm, stack_names):
    """Families of channel concatenations whose argument lists extend one another and whose
    results are read by stack calls only: [(cat nodes, smallest list first), ...]."""
    from torch import fx

    cats = {}
    for node in gm.graph.nodes:
        if node.op == "call_function" and node.target in (torch.cat, torch.concat):
            args = list(node.args) + [node.kwargs.get("dim", 0)] if len(node.args) == 1 else list(node.args)
            if len(args) == 2 and args[1] == 1 and isinstance(args[0], (list, tuple)) and args[0] and \
                    all(isinstance(a, fx.Node) for a in args[0]) and set(node.kwargs) <= {"dim"}:
                cats.setdefault(args[0][0], []).append((node, tuple(args[0])))
    families = []
    for members in cats.values():
        members.sort(key=lambda m: len(m[1]))
        ok = len(members) >= 2
        for (_, a), (_, b) in zip(members, members[1:]):
            ok = ok and len(b) > len(a) and b[:len(a)] == a
        for node, _ in members:
            ok = ok and all(u.op == "call_module" and u.target in stack_names and u.args and u.args[0] is node
                            and node not in u.args[1:] for u in node.users)
        if ok:
            families.append(members)
    return families


def optimize_graph(model: nn.Module, min_layers: int = 1, concrete_args=None, share_concat_buffers="capture",
                   lone_activations=False, **plan_opts):
    """Trace `model` with `torch.fx` and return a `GraphModule` in which every chain of at least
    `min_layers` optimizable operations (see `find_chains`) is one BrainSlugStack call.  The model
    itself is not modified; parameters and sub-modules that stay are shared with it.  Models whose
    `forward` depends on tensor values cannot be traced (a `torch.fx` restriction): use `optimize`
    on those.  `lone_activations`: what happens to a chain that is a single activation layer --
    False (default): it stays in PyTorch, where run eagerly it is cheapest; True: it becomes a stack
    like any other chain, which pays in a captured graph (`capture` rewrites with this setting);
    "capture": a stack while a HIP graph is being captured, PyTorch's own operation otherwise
    (`CaptureOnlyStack`).  `share_concat_buffers` ("capture", "always" or False): the growing channel
    concatenations of densely connected blocks, when only stacks read them, become views of one
    buffer per block (`PrefixConcat`) -- by default only while a HIP graph is being captured.
    `plan_opts` are passed to `bs_stack_plan`."""
    from torch import fx

    gm = model if isinstance(model, fx.GraphModule) else fx.symbolic_trace(model, concrete_args=concrete_args)
    stacks = []
    now: Dict[object, object] = {}  # last node of a replaced chain -> the call that stands for it
    for i, ch in enumerate(find_chains(gm)):
        lone = _lone_activation(ch.layers)
        if ch.real_layers() < min_layers or (lone and not lone_activations):
            continue
        stack = BrainSlugStack.from_layers(ch.layers, ch.names, **plan_opts)
        stack.train(model.training)
        name = f"brainslug_stack_{i}"
        gm.add_submodule(name, CaptureOnlyStack(stack) if lone and lone_activations == "capture" else stack)
        last = ch.nodes[-1]
        # every residual operand is computed before its Add and so before the chain's last node
        with gm.graph.inserting_after(last):
            call = gm.graph.call_module(name, args=tuple(now.get(n, n) for n in (ch.source, *ch.residuals)))
        last.replace_all_uses_with(call)
        now[last] = call
        for n in reversed(ch.nodes):
            gm.graph.erase_node(n)
        stacks.append(stack)
    gm.concat_buffers = []
    if share_concat_buffers:
        names = {n for n, m in gm.named_modules() if isinstance(m, (BrainSlugStack, CaptureOnlyStack)) and "." not in n}
        for f, members in enumerate(_concat_families(gm, names)):
            mod = PrefixConcat(len(members), "always" if share_concat_buffers in (True, "always") else "capture")
            name = f"brainslug_concat_{f}"
            gm.add_submodule(name, mod)
            for position, (node, parts) in enumerate(members):
                with gm.graph.inserting_after(node):
                    call = gm.graph.call_module(name, args=(position, *parts))
                node.replace_all_uses_with(call)
                gm.graph.erase_node(node)
            gm.concat_buffers.append(mod)
    gm.concat_sinks = []
    if share_concat_buffers:
        names = {n for n, m in gm.named_modules() if isinstance(m, (BrainSlugStack, CaptureOnlyStack)) and "." not in n}
        order = {n: i for i, n in enumerate(gm.graph.nodes)}
        for f, node in enumerate(list(gm.graph.nodes)):
            found = _sink_parts(node, names)  # read now: earlier rewrites have replaced some of its parts
            if found is None:
                continue
            parts, mine = found
            sink = ConcatSink(len(parts), "always" if share_concat_buffers in (True, "always") else "capture")
            gm.add_submodule(f"brainslug_sink_{f}", sink)
            gm.add_submodule(f"brainslug_sink_{f}_begin", _SinkBegin(sink))
            gm.add_submodule(f"brainslug_sink_{f}_finish", _SinkFinish(sink))
            first = min((parts[i] for i in mine), key=lambda n: order[n])
            with gm.graph.inserting_before(first):
                begin = gm.graph.call_module(f"brainslug_sink_{f}_begin", args=(first.args[0],))
            first.args = (begin, *first.args[1:])
            for i in mine:
                gm.add_submodule(f"brainslug_sink_{f}_slot_{i}", _SinkSlot(sink, i))
                with gm.graph.inserting_before(parts[i]):
                    slot = gm.graph.call_module(f"brainslug_sink_{f}_slot_{i}", args=(begin,))
                parts[i].kwargs = dict(parts[i].kwargs, out=slot)
            with gm.graph.inserting_after(node):
                call = gm.graph.call_module(f"brainslug_sink_{f}_finish", args=parts)
            node.replace_all_uses_with(call)
            gm.graph.erase_node(node)
            gm.concat_sinks.append(sink)
    gm.graph.lint()
    gm.recompile()
    gm.delete_all_unused_submodules()
    gm.optimized_stacks = stacks
    return gm


# ---------------------------------------------------------------------------- HIP graphs
class CapturedModel:
    """A model's forward pass for one input shape, recorded once in a HIP graph and replayed:
    one launch per pass instead of one per kernel, for serving loops that are bound by the host's
    launch rate.  `__call__` copies its argument into the recorded input buffer, replays the
    graph and returns the recorded output buffer: the result is overwritten by the next call
    (clone it to keep it).  `model` after construction is the model that was recorded.  Stack calls record nothing but their kernels (no memory is set or
    allocated outside torch's allocator), so a rewritten model can be captured like any other."""

    def __init__(self, model: nn.Module, example: torch.Tensor, warmup: int = 3, rewrite: bool = True):
        if not example.is_cuda:
            raise RuntimeError("capture needs an example input on the GPU")
        if rewrite and not hasattr(model, "optimized_stacks"):
            # not rewritten yet: with the settings that pay in a graph (lone activations write
            # straight into concatenations, dense blocks share their concatenation buffer)
            model = optimize_graph(model, lone_activations=True, share_concat_buffers="always")
        self.model = model
        self.input = example.clone(memory_format=torch.preserve_format)
        with torch.no_grad():
            side = torch.cuda.Stream(device=example.device)  # default priority
            side.wait_stream(torch.cuda.current_stream(example.device))
            with torch.cuda.stream(side):
                for _ in range(max(1, warmup)):  # plans, run-time builds, buffer sizes, library warm-up
                    model(self.input)
            torch.cuda.current_stream(example.device).wait_stream(side)
            torch.cuda.synchronize(example.device)
            self.graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(self.graph):
                self.output = model(self.input)

    def __call__(self, x: torch.Tensor):
        if x.shape != self.input.shape or x.dtype != self.input.dtype:
            raise RuntimeError(f"captured for an input of shape {tuple(self.input.shape)} / {self.input.dtype}, "
                               f"got {tuple(x.shape)} / {x.dtype}")
        self.input.copy_(x)
        self.graph.replay()
        return self.output


def capture(model: nn.Module, example: torch.Tensor, warmup: int = 3, rewrite: bool = True) -> CapturedModel:
    """Record `model(example)` (inference, no gradients) in a HIP graph; see `CapturedModel`.  A
    model that `optimize` / `optimize_graph` has not rewritten yet is rewritten first, with the
    settings that pay in a captured graph (`rewrite=False`: captured as it is)."""
    return CapturedModel(model, example, warmup, rewrite)
