"""Seeded synthetic inputs and the named stack configurations.

This module holds no arithmetic of the method (no BatchNorm, ReLU, pooling or
rounding logic): it only draws random tensors and lists layer descriptions as
plain data.  Both the CPU oracle's tests and the HIP path's tests / benchmark
take their inputs from here, so that both sides see the same bytes.

The tensors stand in for the post-convolution activations of the VGG-16-BN,
ResNet-50 and DenseNet-121 networks the paper evaluates (Section 5): same
NCHW shapes, N(0,1) values.  No network weights or images are used.

A layer is a plain dict:
    {"kind": "bn", "gamma": f32[C], "beta": f32[C], "mean": f32[C], "var": f32[C], "eps": float}
    {"kind": "relu"}
    {"kind": "add"}                      # adds the next residual tensor (same shape as its input)
    {"kind": "maxpool", "k": (kh, kw), "s": (sh, sw), "p": (ph, pw), "return_indices": bool}
    {"kind": "avgpool", "k": ..., "s": ..., "p": ..., "count_include_pad": bool}
"""
from __future__ import annotations

import numpy as np

DTYPES = ("f32", "bf16", "f16")


def _rng(seed: int) -> np.random.Generator:
    # Philox is a counter-based generator: the stream depends on the seed only.
    return np.random.Generator(np.random.Philox(int(seed)))


def activation(shape, seed: int, dtype: str = "f32") -> np.ndarray:
    """N(0,1) activation tensor, float32 storage.

    For dtype "bf16" / "f16" every value is made representable in that format (by a
    round-trip through torch's bfloat16 / numpy's float16 type), still stored as float32, so the
    same array can be handed to the oracle (float32 arrays) and, converted
    losslessly to bfloat16, to the GPU.
    """
    if dtype not in DTYPES:
        raise ValueError(f"dtype must be one of {DTYPES}")
    x = _rng(seed).standard_normal(size=tuple(int(s) for s in shape), dtype=np.float32)
    if dtype == "bf16":
        import torch

        x = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    elif dtype == "f16":
        x = x.astype(np.float16).astype(np.float32)
    return x


def bn_params(channels: int, seed: int, eps: float = 1e-5) -> dict:
    """BatchNorm inference parameters drawn as benchmark configuration 0 states:
    running_mean ~ N(0, sd 0.5), running_var ~ U(0.5, 2), gamma ~ U(0.5, 1.5),
    beta ~ N(0, sd 0.1)."""
    g = _rng(seed)
    c = int(channels)
    mean = (0.5 * g.standard_normal(c)).astype(np.float32)
    var = g.uniform(0.5, 2.0, c).astype(np.float32)
    gamma = g.uniform(0.5, 1.5, c).astype(np.float32)
    beta = (0.1 * g.standard_normal(c)).astype(np.float32)
    return {"kind": "bn", "gamma": gamma, "beta": beta, "mean": mean, "var": var, "eps": float(eps)}


def relu() -> dict:
    return {"kind": "relu"}


def leaky_relu(slope: float = 0.01) -> dict:
    return {"kind": "leaky_relu", "slope": float(slope)}


def clamp(lo: float, hi: float) -> dict:
    return {"kind": "clamp", "lo": float(lo), "hi": float(hi)}


def relu6() -> dict:
    return clamp(0.0, 6.0)


def add() -> dict:
    return {"kind": "add"}


def _pair(v):
    return (int(v), int(v)) if np.isscalar(v) else (int(v[0]), int(v[1]))


def maxpool(k, s=None, p=0, return_indices: bool = False, ceil_mode: bool = False) -> dict:
    s = k if s is None else s
    return {"kind": "maxpool", "k": _pair(k), "s": _pair(s), "p": _pair(p),
            "return_indices": bool(return_indices), "ceil_mode": bool(ceil_mode)}


def avgpool(k, s=None, p=0, count_include_pad: bool = True, ceil_mode: bool = False) -> dict:
    s = k if s is None else s
    return {"kind": "avgpool", "k": _pair(k), "s": _pair(s), "p": _pair(p),
            "count_include_pad": bool(count_include_pad), "ceil_mode": bool(ceil_mode)}


def pool_out(h: int, k: int, s: int, p: int, ceil_mode: bool = False) -> int:
    """Spatial output size of a pool (shape bookkeeping only)."""
    if not ceil_mode:
        return (h + 2 * p - k) // s + 1
    o = -((h + 2 * p - k) // -s) + 1
    return o - 1 if (o - 1) * s >= h + p else o


def output_shape(layers, shape):
    n, c, h, w = (int(v) for v in shape)
    for l in layers:
        if l["kind"] in ("maxpool", "avgpool"):
            h = pool_out(h, l["k"][0], l["s"][0], l["p"][0], l.get("ceil_mode", False))
            w = pool_out(w, l["k"][1], l["s"][1], l["p"][1], l.get("ceil_mode", False))
    return (n, c, h, w)


def num_residuals(layers) -> int:
    return sum(1 for l in layers if l["kind"] == "add")


# ---------------------------------------------------------------------------
# Named configurations (benchmark configurations 0-4).  Each entry: name -> builder
# returning (layers, shape, dtypes).  `seed` feeds: input = seed, residual i =
# seed + 1 + i, BN parameters of layer j = seed + 100 + j.
# ---------------------------------------------------------------------------

def _bn_relu_pool(c, seed, pool, want_idx):
    p = dict(pool)
    if p["kind"] == "maxpool":
        p["return_indices"] = bool(want_idx)
    return [bn_params(c, seed + 100), relu(), p]


def build(name: str, seed: int = 0, batch: int | None = None, indices: bool = False):
    """Return (layers, input_shape, dtypes) for a named configuration.

    `batch` overrides N (used to cut a bounded sample for CPU timing and for
    reduced-size parity runs); everything else is the configuration's own.
    """
    def nb(n):
        return int(batch) if batch is not None else n

    if name == "tiny":  # config 0
        return _bn_relu_pool(16, seed, maxpool(2, 2), indices), (nb(1), 16, 32, 32), ("f32",)
    if name == "vgg_a":  # config 1, 64x224x224
        return _bn_relu_pool(64, seed, maxpool(2, 2), indices), (nb(32), 64, 224, 224), ("f32",)
    if name == "vgg_b":
        return _bn_relu_pool(128, seed, maxpool(2, 2), indices), (nb(32), 128, 112, 112), ("f32",)
    if name == "vgg_c":
        return _bn_relu_pool(256, seed, maxpool(2, 2), indices), (nb(32), 256, 56, 56), ("f32",)
    if name == "resnet_stem":  # config 2
        return (_bn_relu_pool(64, seed, maxpool(3, 2, 1), indices), (nb(64), 64, 112, 112),
                ("f32", "bf16", "f16"))
    if name == "resnet_tail":
        return [bn_params(256, seed + 100), add(), relu()], (nb(64), 256, 56, 56), ("f32", "bf16", "f16")
    if name == "densenet_dense":  # config 3
        return [bn_params(256, seed + 100), relu()], (nb(64), 256, 56, 56), ("f32",)
    if name == "densenet_trans":
        return (_bn_relu_pool(512, seed, avgpool(2, 2), indices), (nb(64), 512, 28, 28), ("f32",))
    if name == "halo_stress":  # config 4
        layers = [bn_params(128, seed + 100), relu(), avgpool(3, 1, 1, True),
                  maxpool(3, 2, 1, indices), bn_params(128, seed + 104), relu()]
        return layers, (nb(128), 128, 56, 56), ("f32", "bf16", "f16")
    raise KeyError(name)


CONFIG_NAMES = ("tiny", "vgg_a", "vgg_b", "vgg_c", "resnet_stem", "resnet_tail",
                "densenet_dense", "densenet_trans", "halo_stress")
VGG_STACKS = ("vgg_a", "vgg_b", "vgg_c")


def inputs_for(name: str, seed: int = 0, dtype: str = "f32", batch: int | None = None,
               indices: bool = False):
    """(layers, x, residuals) for a named configuration."""
    layers, shape, _ = build(name, seed, batch, indices)
    x = activation(shape, seed, dtype)
    res = [activation(shape_at_add, seed + 1 + i, dtype)
           for i, shape_at_add in enumerate(residual_shapes(layers, shape))]
    return layers, x, res


def residual_shapes(layers, shape):
    """Shape each residual operand must have: that of the Add layer's input."""
    out = []
    cur = tuple(int(v) for v in shape)
    for l in layers:
        if l["kind"] == "add":
            out.append(cur)
        cur = output_shape([l], cur)
    return out


def algorithmic_bytes(layers, shape, dtype: str, indices: bool = False) -> int:
    """HBM bytes a perfectly fused stack must move: input + residuals + output
    (+ int32 indices when requested).  BatchNorm parameters are ignored."""
    es = 4 if dtype == "f32" else 2
    n_in = int(np.prod(shape))
    total = n_in * es
    for s in residual_shapes(layers, shape):
        total += int(np.prod(s)) * es
    total += int(np.prod(output_shape(layers, shape))) * es
    if indices:
        cur = tuple(shape)
        for l in layers:
            cur = output_shape([l], cur)
            if l["kind"] == "maxpool" and l.get("return_indices"):
                total += int(np.prod(cur)) * 4
    return total


def layer_by_layer_bytes(layers, shape, dtype: str) -> int:
    """HBM bytes of breadth-first execution: every layer reads its whole input
    (and residual) and writes its whole output."""
    es = 4 if dtype == "f32" else 2
    total = 0
    cur = tuple(shape)
    for l in layers:
        nxt = output_shape([l], cur)
        total += int(np.prod(cur)) * es + int(np.prod(nxt)) * es
        if l["kind"] == "add":
            total += int(np.prod(cur)) * es
        cur = nxt
    return total
