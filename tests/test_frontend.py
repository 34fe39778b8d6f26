"""Front-end tests: aggregation detection and model rewriting (Section 4.3, Figure 4).

The CPU part checks which runs of layers are found and replaced, and pins the layer
descriptions the front-end extracts from torch modules: the CPU oracle run on those
descriptions must agree with the unmodified torch model.  The GPU part runs rewritten models
through the HIP library and compares them with the original model and, stack by stack on the
tensors that actually reach each stack, with the oracle.
"""
import copy

import numpy as np
import pytest
import torch
from torch import nn

from oracle import breadth_first as bf
from paper_1804_08378_amd import brainslug as bs
from paper_1804_08378_amd import frontend as fe


def vgg_like(c_in=3, width=8, seed=0):
    torch.manual_seed(seed)
    m = nn.Sequential(
        nn.Conv2d(c_in, width, 3, padding=1), nn.BatchNorm2d(width), nn.ReLU(inplace=True), nn.MaxPool2d(2, 2),
        nn.Conv2d(width, 2 * width, 3, padding=1), nn.BatchNorm2d(2 * width), nn.ReLU(inplace=True), nn.Dropout(0.5),
        nn.AvgPool2d(3, 1, 1, count_include_pad=False), nn.MaxPool2d(3, 2, 1),
        nn.Conv2d(2 * width, 2 * width, 1), nn.ReLU(), nn.Flatten(), nn.LazyLinear(10))
    for mod in m.modules():  # non-trivial running statistics and affine parameters
        if isinstance(mod, nn.BatchNorm2d):
            c = mod.num_features
            mod.running_mean.copy_(torch.randn(c) * 0.5)
            mod.running_var.copy_(torch.rand(c) * 1.5 + 0.5)
            mod.weight.data.copy_(torch.rand(c) + 0.5)
            mod.bias.data.copy_(torch.randn(c) * 0.1)
    return m.eval()


class Wrapper(nn.Module):
    """A module with its own forward: its direct children are not known to run in order."""

    def __init__(self):
        super().__init__()
        self.bn = nn.BatchNorm2d(4)
        self.relu = nn.ReLU()
        self.body = nn.Sequential(nn.BatchNorm2d(4), nn.ReLU(), nn.MaxPool2d(2))

    def forward(self, x):
        return self.body(self.relu(self.bn(x)))


def test_aggregation_detection_finds_maximal_runs():
    m = vgg_like()
    assert fe.find_runs(m) == [(1, 4), (5, 10), (11, 12)]
    # layers the library does not take end a run
    seq = nn.Sequential(nn.ReLU(), nn.MaxPool2d(2, return_indices=True), nn.ReLU(), nn.MaxPool2d(2, ceil_mode=True),
                        nn.BatchNorm2d(4, track_running_stats=False),
                        nn.MaxPool2d(2, dilation=2), nn.AvgPool2d(2, divisor_override=3), nn.Dropout(), nn.Identity())
    assert fe.find_runs(seq) == [(0, 1), (2, 4)]  # the trailing Dropout/Identity run holds no real layer


def test_optimize_replaces_first_layer_and_blanks_the_rest():
    m = fe.optimize(vgg_like())
    kinds = [type(c).__name__ for c in m]
    assert kinds == ["Conv2d", "BrainSlugStack", "Identity", "Identity", "Conv2d", "BrainSlugStack", "Identity", "Identity",
                     "Identity", "Identity", "Conv2d", "BrainSlugStack", "Flatten", "LazyLinear"]
    assert len(m.optimized_stacks) == 3
    s0, s1, s2 = m.optimized_stacks
    assert [l["kind"] for l in s0.layers] == ["bn", "relu", "maxpool"]
    assert [l["kind"] for l in s1.layers] == ["bn", "relu", "avgpool", "maxpool"]  # Dropout is the identity
    assert s1.layers[2]["count_include_pad"] is False and s1.layers[3]["p"] == (1, 1)
    assert [l["kind"] for l in s2.layers] == ["relu"]
    assert s0.replaced == ["BatchNorm2d", "ReLU", "MaxPool2d"]
    # running it twice changes nothing more; min_layers keeps short runs in PyTorch
    again = fe.optimize(m)
    assert again.optimized_stacks == []
    m2 = fe.optimize(vgg_like(), min_layers=2)
    assert [type(c).__name__ for c in m2][11] == "ReLU" and len(m2.optimized_stacks) == 2


def test_only_sequential_containers_are_rewritten():
    m = fe.optimize(Wrapper().eval())
    assert isinstance(m.bn, nn.BatchNorm2d) and isinstance(m.relu, nn.ReLU)
    assert isinstance(m.body[0], fe.BrainSlugStack) and isinstance(m.body[1], nn.Identity)


def test_stack_refuses_what_the_library_cannot_run():
    m = fe.optimize(vgg_like())
    stack = m.optimized_stacks[0]
    with pytest.raises(RuntimeError, match="GPU"):
        stack(torch.zeros(1, 8, 8, 8))
    stack.train()
    with pytest.raises(RuntimeError, match="inference"):
        stack(torch.zeros(1, 8, 8, 8))


@pytest.mark.parametrize("shape", [(2, 3, 16, 16), (1, 3, 20, 12)])
def test_extracted_layer_descriptions_reproduce_the_torch_model(shape):
    """Pin of the parameter extraction: feeding each run's input to the oracle with the
    extracted descriptions gives what the torch layers give (float32, CPU)."""
    ref = vgg_like()
    opt = fe.optimize(copy.deepcopy(ref))
    x = torch.randn(*shape)
    with torch.no_grad():
        ref(x)  # materialise the lazy layer
        for (start, stop), stack in zip(fe.find_runs(ref), opt.optimized_stacks):
            xin = ref[:start](x)
            want = ref[start:stop](xin).numpy()
            got, _, _ = bf.run_stack(stack.layers, np.ascontiguousarray(xin.numpy()))
            assert got.shape == want.shape
            assert np.abs(got - want).max() <= 1e-5 * max(1.0, np.abs(want).max())
            # the library accepts the descriptions and plans them
            st = bs.Stack(stack.layers, tuple(xin.shape), "f32").plan(host_only=1)
            assert tuple(st.out_shape) == want.shape
            st.close()


def head_like(c=8, seed=1):
    """The tail of a DenseNet / ResNet style network written as modules."""
    torch.manual_seed(seed)
    m = nn.Sequential(nn.Conv2d(3, c, 3, padding=1), nn.BatchNorm2d(c), nn.LeakyReLU(0.1), nn.MaxPool2d(3, 2, ceil_mode=True),
                      nn.ReLU6(), nn.AdaptiveAvgPool2d(1), nn.Flatten(), nn.Linear(c, 5))
    bn = m[1]
    bn.running_mean.copy_(torch.randn(c) * 0.5)
    bn.running_var.copy_(torch.rand(c) + 0.5)
    return m.eval()


def test_adaptive_pools_ceil_mode_and_further_activations_are_taken():
    ref = head_like()
    assert fe.find_runs(ref) == [(1, 6)]
    opt = fe.optimize(copy.deepcopy(ref))
    stack = opt.optimized_stacks[0]
    assert [l["kind"] for l in stack.layers] == ["bn", "leaky_relu", "maxpool", "clamp", "adaptive_avg"]
    x = torch.randn(2, 3, 14, 18)
    with torch.no_grad():
        xin = ref[:1](x)
        want = ref[1:6](xin).numpy()
    layers = fe.resolve_layers(stack.layers, xin.shape)
    assert layers[-1] == {"kind": "avgpool", "k": (7, 9), "s": (7, 9), "p": (0, 0), "count_include_pad": True}
    got, _, _ = bf.run_stack(layers, np.ascontiguousarray(xin.numpy()))
    assert got.shape == want.shape == (2, 8, 1, 1)
    assert np.abs(got - want).max() <= 1e-5 * max(1.0, np.abs(want).max())
    with pytest.raises(RuntimeError, match="divide"):
        fe.resolve_layers([{"kind": "adaptive_avg", "out": (3, 3)}], (1, 1, 7, 7))


# ------------------------------------------------------------------ GPU
@pytest.mark.gpu
def test_head_like_model_on_the_gpu():
    ref = head_like(c=16).cuda()
    opt = fe.optimize(copy.deepcopy(ref))
    x = torch.randn(3, 3, 30, 34, device="cuda")
    with torch.no_grad():
        want, got = ref(x), opt(x)
        xin = ref[:1](x)
    assert (got - want).abs().max().item() <= 1e-4 * max(1.0, want.abs().max().item())
    stack = opt.optimized_stacks[0]
    expect, _, _ = bf.run_stack(fe.resolve_layers(stack.layers, xin.shape), xin.cpu().numpy())
    with torch.no_grad():
        out = stack(xin)
    assert np.array_equal(out.cpu().numpy().view(np.uint32), expect.view(np.uint32))
    stack.close()


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_rewritten_model_matches_the_original_and_the_oracle(dtype):
    ref = vgg_like(width=16).cuda()
    x = torch.randn(4, 3, 40, 48, device="cuda")
    with torch.no_grad():
        ref(x)
    ref = ref.to(dtype)
    x = x.to(dtype)
    opt = fe.optimize(copy.deepcopy(ref))
    seen = {}
    for i, stack in enumerate(opt.optimized_stacks):
        stack.register_forward_hook(lambda mod, inp, out, i=i: seen.__setitem__(i, (inp[0].detach().clone(), out.detach().clone())))
    with torch.no_grad():
        want = ref(x).float()
        got = opt(x).float()
    tol = 1e-4 if dtype == torch.float32 else 5e-2
    assert (got - want).abs().max().item() <= tol * max(1.0, want.abs().max().item())
    assert len(seen) == 3
    name = "f32" if dtype == torch.float32 else "bf16"
    for i, stack in enumerate(opt.optimized_stacks):
        xin, out = seen[i]
        expect, _, _ = bf.run_stack(stack.layers, xin.float().cpu().numpy(), [], name)
        assert np.array_equal(out.float().cpu().numpy().view(np.uint32), expect.view(np.uint32)), i
    # a second input shape plans again; the first plan is kept
    with torch.no_grad():
        opt[:12](x[:2, :, :32, :32].contiguous())  # the convolutional part only: the classifier is sized for x
    assert all(len(s._plans) == 2 for s in opt.optimized_stacks)
    for s in opt.optimized_stacks:
        s.close()
