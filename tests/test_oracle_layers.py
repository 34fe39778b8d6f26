"""Pins for the CPU oracle's single layers (no GPU).

Each layer is checked against something other than itself: closed forms and
invariants that follow from the definitions in Section 2 of the paper
(element-wise normalisation / ReLU, pooling over fixed windows), and the CPU
routines of an independent library (torch.nn.functional) as a second witness.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import layers as L
from paper_1804_08378_amd import workloads as wl


def _x(shape, seed=0):
    return wl.activation(shape, seed)


def _ulp_diff(a, b):
    a = np.ascontiguousarray(a, np.float32).view(np.int32).astype(np.int64)
    b = np.ascontiguousarray(b, np.float32).view(np.int32).astype(np.int64)
    a = np.where(a < 0, -(a & 0x7FFFFFFF), a)
    b = np.where(b < 0, -(b & 0x7FFFFFFF), b)
    return np.abs(a - b)


# ----------------------------------------------------------------- BatchNorm
def test_bn_identity_closed_form():
    x = _x((2, 3, 5, 7))
    c = 3
    one, zero = np.ones(c, np.float32), np.zeros(c, np.float32)
    y = L.batchnorm(x, one, zero, zero, one, 0.0)
    assert np.array_equal(y, x)


def test_bn_eps_closed_form():
    x = _x((1, 2, 4, 4), 1)
    one, zero = np.ones(2, np.float32), np.zeros(2, np.float32)
    y = L.batchnorm(x, one, zero, zero, one, 1e-5)
    ref = (x.astype(np.float64) / np.sqrt(1.0 + 1e-5)).astype(np.float32)
    assert _ulp_diff(y, ref).max() <= 1


def test_bn_gamma_zero_gives_beta():
    x = _x((2, 4, 3, 3), 2)
    beta = np.array([0.25, -1.5, 3.0, 0.0], np.float32)
    p = wl.bn_params(4, 5)
    y = L.batchnorm(x, np.zeros(4, np.float32), beta, p["mean"], p["var"], 1e-5)
    assert np.array_equal(y, np.broadcast_to(beta[None, :, None, None], x.shape))


def test_bn_exact_small_integers():
    # mean 1, var 1, eps 0, gamma 2, beta 0.5: y = (x-1)*2+0.5, exact in float32
    x = np.arange(-12, 12, dtype=np.float32).reshape(1, 2, 3, 4)
    c = 2
    y = L.batchnorm(x, np.full(c, 2, np.float32), np.full(c, 0.5, np.float32),
                    np.ones(c, np.float32), np.ones(c, np.float32), 0.0)
    assert np.array_equal(y, (x - 1) * 2 + 0.5)


def test_bn_channel_axis_and_params_not_swapped():
    # distinct parameters per channel; a transposed axis or swapped gamma/beta/mean/var fails
    x = _x((3, 5, 4, 6), 3)
    p = wl.bn_params(5, 7)
    y = L.batchnorm(x, p["gamma"], p["beta"], p["mean"], p["var"], p["eps"])
    for c in range(5):
        ref = ((x[:, c].astype(np.float64) - p["mean"][c]) / np.sqrt(p["var"][c] + 1e-5)
               * p["gamma"][c] + p["beta"][c])
        assert np.abs(y[:, c] - ref).max() <= 1e-6 * max(1.0, np.abs(ref).max())


def test_bn_folded_vs_textbook_f64_and_torch():
    x = _x((4, 16, 9, 11), 4)
    p = wl.bn_params(16, 8)
    y = L.batchnorm(x, p["gamma"], p["beta"], p["mean"], p["var"], p["eps"])
    t = L.batchnorm_textbook_f64(x, p["gamma"], p["beta"], p["mean"], p["var"], p["eps"])
    assert np.abs(y - t).max() <= 1e-5 * np.abs(t).max()
    tt = F.batch_norm(torch.from_numpy(x).double(), torch.from_numpy(p["mean"]).double(),
                      torch.from_numpy(p["var"]).double(), torch.from_numpy(p["gamma"]).double(),
                      torch.from_numpy(p["beta"]).double(), False, 0.0, p["eps"]).numpy()
    assert np.abs(t - tt).max() <= 1e-12 * np.abs(tt).max()
    assert np.abs(y - tt).max() <= 1e-5 * np.abs(tt).max()


def test_bn_fold_is_one_rounding_of_the_f64_value():
    p = wl.bn_params(64, 11)
    scale, shift = L.bn_fold(p["gamma"], p["beta"], p["mean"], p["var"], p["eps"])
    s64 = p["gamma"].astype(np.float64) / np.sqrt(p["var"].astype(np.float64) + p["eps"])
    assert np.array_equal(scale, s64.astype(np.float32))
    assert np.array_equal(shift, (p["beta"].astype(np.float64) - p["mean"].astype(np.float64) * s64)
                          .astype(np.float32))


def test_bn_uses_a_fused_multiply_add():
    # x*scale+shift with a separate rounding of the product differs from fma on this input:
    # scale = 1+2^-12, x = 1+2^-12 -> product needs 2^-24 which fma keeps, mul drops.
    x = np.full((1, 1, 1, 1), 1 + 2.0 ** -12, np.float32)
    gamma = np.array([1 + 2.0 ** -12], np.float32)
    beta = np.array([-1.0], np.float32)
    y = L.batchnorm(x, gamma, beta, np.zeros(1, np.float32), np.ones(1, np.float32), 0.0)
    exact = (1 + 2.0 ** -12) ** 2 - 1.0
    assert y[0, 0, 0, 0] == np.float32(exact)
    assert np.float32(np.float32(x[0, 0, 0, 0] * gamma[0]) - np.float32(1.0)) != np.float32(exact)


# ---------------------------------------------------------------------- ReLU
def test_relu_properties():
    x = _x((2, 3, 8, 8), 5)
    y = L.relu(x)
    assert (y >= 0).all()
    assert np.array_equal(y[x > 0], x[x > 0])
    assert (y[x <= 0] == 0).all()
    assert np.array_equal(L.relu(y).view(np.int32), y.view(np.int32))  # idempotent, bitwise
    assert np.array_equal(y, torch.relu(torch.from_numpy(x)).numpy())


def test_relu_negative_zero_and_nan_become_plus_zero():
    x = np.array([-0.0, np.nan, -np.inf, 0.0, np.inf, 1e-45], np.float32).reshape(1, 1, 1, 6)
    y = L.relu(x)
    assert np.array_equal(y.view(np.uint32).ravel()[:4], np.zeros(4, np.uint32))
    assert y.ravel()[4] == np.inf and y.ravel()[5] == np.float32(1e-45)


# ----------------------------------------------------------------------- Add
def test_add_properties():
    a, r = _x((2, 2, 5, 5), 6), _x((2, 2, 5, 5), 7)
    assert np.array_equal(L.add(a, np.zeros_like(a)), a)
    assert (L.add(a, -a) == 0).all()
    assert np.array_equal(L.add(a, r), L.add(r, a))
    assert np.array_equal(L.add(a, r), a + r)  # numpy float32 add, one rounding
    with pytest.raises(ValueError):
        L.add(a, r[:, :1])


# ------------------------------------------------------------------- MaxPool
POOL_CASES = [
    # (H, W, k, s, p)
    (8, 8, (2, 2), (2, 2), (0, 0)),
    (7, 9, (2, 2), (2, 2), (0, 0)),
    (9, 7, (3, 3), (2, 2), (1, 1)),
    (10, 10, (3, 3), (1, 1), (1, 1)),
    (11, 6, (3, 2), (2, 1), (1, 0)),
    (5, 13, (2, 3), (1, 2), (1, 1)),
    (6, 6, (3, 3), (3, 3), (0, 0)),
    (4, 4, (4, 4), (4, 4), (2, 2)),
    (5, 5, (1, 1), (1, 1), (0, 0)),
    (9, 9, (2, 2), (3, 3), (0, 0)),  # stride > kernel: cells skipped
]


@pytest.mark.parametrize("H,W,k,s,p", POOL_CASES)
def test_maxpool_vs_torch_and_invariants(H, W, k, s, p):
    x = _x((2, 3, H, W), H * 100 + W)
    x[0, 0] = np.maximum(x[0, 0], 0)  # ties at zero, as after ReLU
    x[1, 1] = 0.0                     # an all-tie plane
    y, idx = L.maxpool(x, k, s, p, True)
    ty, tidx = F.max_pool2d(torch.from_numpy(x), k, s, p, return_indices=True)
    assert y.shape == tuple(ty.shape)
    assert np.array_equal(y, ty.numpy())
    assert np.array_equal(idx, tidx.numpy().astype(np.int32))
    # in[idx] == out, idx inside the window
    flat = x.reshape(2, 3, -1)
    assert np.array_equal(np.take_along_axis(flat, idx.reshape(2, 3, -1).astype(np.int64), 2),
                          y.reshape(2, 3, -1))
    oh, ow = np.meshgrid(np.arange(y.shape[2]), np.arange(y.shape[3]), indexing="ij")
    ih, iw = idx // W, idx % W
    assert ((ih >= oh * s[0] - p[0]) & (ih < oh * s[0] - p[0] + k[0]) & (ih >= 0) & (ih < H)).all()
    assert ((iw >= ow * s[1] - p[1]) & (iw < ow * s[1] - p[1] + k[1]) & (iw >= 0) & (iw < W)).all()
    # all-tie plane: first in-range cell of the window
    first = np.maximum(oh * s[0] - p[0], 0) * W + np.maximum(ow * s[1] - p[1], 0)
    assert np.array_equal(idx[1, 1], first.astype(np.int32))
    # monotone under an exactly representable shift
    xs = (np.round(x * 8) / 8).astype(np.float32)
    assert np.array_equal(L.maxpool(xs + 4.0, k, s, p), L.maxpool(xs, k, s, p) + 4.0)


def test_maxpool_brute_force_definition():
    # window maximum through numpy's max/argmax on an explicit -inf padded copy
    rng = np.random.default_rng(3)
    for (H, W, k, s, p) in POOL_CASES:
        x = rng.integers(-3, 4, size=(1, 2, H, W)).astype(np.float32)  # many ties
        y, idx = L.maxpool(x, k, s, p, True)
        xp = np.full((1, 2, H + 2 * p[0], W + 2 * p[1]), -np.inf, np.float32)
        xp[:, :, p[0]:p[0] + H, p[1]:p[1] + W] = x
        for oh in range(y.shape[2]):
            for ow in range(y.shape[3]):
                win = xp[:, :, oh * s[0]:oh * s[0] + k[0], ow * s[1]:ow * s[1] + k[1]].reshape(1, 2, -1)
                assert np.array_equal(y[:, :, oh, ow], win.max(2))
                for c in range(2):
                    cand = [j for j in range(win.shape[2]) if win[0, c, j] == win[0, c].max()
                            and np.isfinite(win[0, c, j])]
                    j = cand[0]  # first maximum in row-major order among real cells
                    ih, iw = oh * s[0] - p[0] + j // k[1], ow * s[1] - p[1] + j % k[1]
                    assert idx[0, c, oh, ow] == ih * W + iw


def test_maxpool_constant_identity_and_ramps():
    c = np.full((1, 1, 6, 6), 2.5, np.float32)
    y, idx = L.maxpool(c, (3, 3), (2, 2), (1, 1), True)
    assert (y == 2.5).all()
    assert np.array_equal(idx[0, 0], np.array([[0, 1, 3], [6, 7, 9], [18, 19, 21]], np.int32))
    x = _x((1, 2, 5, 7), 9)
    y, idx = L.maxpool(x, (1, 1), (1, 1), (0, 0), True)
    assert np.array_equal(y, x)
    assert np.array_equal(idx[0, 0], np.arange(35, dtype=np.int32).reshape(5, 7))
    up = np.arange(64, dtype=np.float32).reshape(1, 1, 8, 8)
    _, iu = L.maxpool(up, (2, 2), (2, 2), (0, 0), True)   # increasing: last cell of each window
    _, idn = L.maxpool(-up, (2, 2), (2, 2), (0, 0), True)  # decreasing: first cell
    oh, ow = np.meshgrid(np.arange(4), np.arange(4), indexing="ij")
    assert np.array_equal(iu[0, 0], ((2 * oh + 1) * 8 + 2 * ow + 1).astype(np.int32))
    assert np.array_equal(idn[0, 0], ((2 * oh) * 8 + 2 * ow).astype(np.int32))


def test_maxpool_rejects_empty_output():
    with pytest.raises(ValueError):
        L.maxpool(np.zeros((1, 1, 2, 2), np.float32), (3, 3), (1, 1), (0, 0))


# ------------------------------------------------------------------- AvgPool
@pytest.mark.parametrize("H,W,k,s,p", POOL_CASES)
@pytest.mark.parametrize("cip", [True, False])
def test_avgpool_vs_torch(H, W, k, s, p, cip):
    x = _x((2, 3, H, W), H * 10 + W)
    y = L.avgpool(x, k, s, p, cip)
    ty = F.avg_pool2d(torch.from_numpy(x), k, s, p, ceil_mode=False, count_include_pad=cip).numpy()
    assert y.shape == ty.shape
    # the library divides, the definition here multiplies by the float32 reciprocal: <= 1 ulp,
    # and exact when the divisor is a power of two (and padding does not change it)
    assert _ulp_diff(y, ty).max() <= 2
    t64 = F.avg_pool2d(torch.from_numpy(x).double(), k, s, p, ceil_mode=False,
                       count_include_pad=cip).numpy()
    assert np.abs(y - t64).max() <= 4e-7 * max(1.0, np.abs(x).max()) * 2
    if k == (2, 2) and p == (0, 0):
        assert np.array_equal(y, ty)


def test_avgpool_closed_forms():
    c = np.full((1, 2, 6, 6), 3.0, np.float32)
    assert (L.avgpool(c, (2, 2), (2, 2), (0, 0)) == 3.0).all()
    y = L.avgpool(np.full((1, 1, 5, 5), 9.0, np.float32), (3, 3), (1, 1), (1, 1), True)
    ninth = np.float32(1.0) / np.float32(9.0)
    assert y[0, 0, 0, 0] == np.float32(36.0) * ninth       # corner: 4 cells of 9
    assert y[0, 0, 0, 2] == np.float32(54.0) * ninth       # edge: 6 cells
    assert y[0, 0, 2, 2] == np.float32(81.0) * ninth       # interior: 9 cells
    assert abs(y[0, 0, 0, 0] - 4.0) < 1e-6 and abs(y[0, 0, 0, 2] - 6.0) < 1e-6
    y2 = L.avgpool(np.full((1, 1, 5, 5), 9.0, np.float32), (3, 3), (1, 1), (1, 1), False)
    assert np.abs(y2 - 9.0).max() < 1e-6                   # padding excluded from the divisor
    x = _x((1, 2, 4, 5), 12)
    assert np.array_equal(L.avgpool(x, (1, 1), (1, 1), (0, 0)), x)
    ramp = np.arange(16, dtype=np.float32).reshape(1, 1, 4, 4)
    assert np.array_equal(L.avgpool(ramp, (2, 2), (2, 2), (0, 0))[0, 0],
                          np.array([[2.5, 4.5], [10.5, 12.5]], np.float32))


def test_avgpool_sum_order_is_row_major_sequential():
    # 1e8 + 1 + ... : the float32 result depends on the order; row-major sequential from +0
    x = np.array([[1e8, 1.0, 1.0], [1.0, 1.0, 1.0], [1.0, 1.0, -1e8]], np.float32).reshape(1, 1, 3, 3)
    y = L.avgpool(x, (3, 3), (1, 1), (0, 0))
    acc = np.float32(0)
    for v in x.ravel():
        acc = np.float32(acc + v)
    assert y.ravel()[0] == np.float32(acc * (np.float32(1) / np.float32(9)))
    assert acc == 0.0  # every +1 is absorbed by 1e8: shows the order matters (true sum is 7)


# ------------------------------------------------------------ bf16 rounding
def test_round_f16_vs_library_ties_subnormals_and_overflow():
    """binary16 rounding against numpy's float16 conversion (an independent implementation):
    every half value is a fixed point, midpoints between neighbours go to the even one, the
    subnormal grid has spacing 2^-24, and 65520 is the first value that overflows."""
    allh = np.arange(65536, dtype=np.uint16).view(np.float16)
    fin = allh[np.isfinite(allh)].astype(np.float32)
    assert np.array_equal(L.round_f16(fin).view(np.uint32), fin.view(np.uint32))
    pos = np.sort(fin[fin >= 0])
    mid = ((pos[:-1].astype(np.float64) + pos[1:].astype(np.float64)) / 2).astype(np.float32)  # exact in float32
    for x in (mid, -mid, np.nextafter(mid, np.float32(np.inf)), np.nextafter(mid, np.float32(-np.inf))):
        assert np.array_equal(L.round_f16(x).view(np.uint32), x.astype(np.float16).astype(np.float32).view(np.uint32))
    g = np.random.Generator(np.random.Philox(5))
    r = (g.standard_normal(200000) * np.exp(g.uniform(-20, 12, 200000))).astype(np.float32)
    with np.errstate(over="ignore"):
        assert np.array_equal(L.round_f16(r).view(np.uint32), r.astype(np.float16).astype(np.float32).view(np.uint32))
    sp = np.float32([65504, 65519.996, 65520, 70000, -65520, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -25, 2.0 ** -26, 0.0, -0.0])
    want = np.float32([65504, 65504, np.inf, np.inf, -np.inf, 2.0 ** -24, 0.0, 2.0 ** -24, 0.0, 0.0, -0.0])
    got = L.round_f16(sp)
    assert np.array_equal(got, want) and np.signbit(got[-1]) and not np.signbit(got[-2])
    assert np.isnan(L.round_f16(np.float32([np.nan]))[0])


# ------------------------------------------------------------------ further activations
def test_leaky_relu_closed_forms_and_library():
    x = np.array([-4.0, -1.0, -0.0, 0.0, 0.5, 3.0, -1e-30, np.inf, -np.inf], np.float32).reshape(1, 1, 3, 3)
    y = L.leaky_relu(x, 0.25)
    assert np.array_equal(y.ravel(), np.array([-1.0, -0.25, -0.0, 0.0, 0.5, 3.0, -2.5e-31, np.inf, -np.inf], np.float32))
    assert np.signbit(y.ravel()[2]) and not np.signbit(y.ravel()[3])       # -0 * slope = -0; +0 * slope = +0
    assert np.array_equal(L.leaky_relu(x, 1.0), x)                          # slope 1: identity
    fin = x[np.isfinite(x)]
    assert np.array_equal(L.leaky_relu(fin, 0.0), L.relu(fin))             # slope 0: ReLU up to the sign of zero
    r = wl.activation((2, 3, 9, 11), 21)
    for slope in (0.01, 0.2, 1.5):
        assert np.array_equal(L.leaky_relu(r, slope), F.leaky_relu(torch.from_numpy(r), slope).numpy())
    # one float32 rounding of the product
    assert L.leaky_relu(np.float32([-3.0]).reshape(1, 1, 1, 1), 0.1).ravel()[0] == np.float32(-3.0) * np.float32(0.1)


def test_clamp_closed_forms_and_library():
    x = np.array([-7.0, -1.0, -0.0, 0.0, 0.5, 6.0, 6.5, np.nan, np.inf], np.float32).reshape(1, 1, 3, 3)
    y = L.clamp(x, 0.0, 6.0).ravel()                                        # ReLU6
    assert np.array_equal(y, np.array([0.0, 0.0, 0.0, 0.0, 0.5, 6.0, 6.0, 0.0, 6.0], np.float32))
    assert not np.signbit(y[2])                                             # -0 is not above +0: becomes +0
    assert np.array_equal(L.clamp(x, -1.0, 1.0).ravel(), np.array([-1, -1, -0.0, 0, 0.5, 1, 1, -1, 1], np.float32))
    r = wl.activation((2, 3, 9, 11), 22) * 4
    assert np.array_equal(L.clamp(r, 0.0, 6.0), F.relu6(torch.from_numpy(r)).numpy())
    assert np.array_equal(L.clamp(r, -0.5, 2.0), F.hardtanh(torch.from_numpy(r), -0.5, 2.0).numpy())
    assert np.array_equal(L.clamp(r, 0.0, np.inf), L.relu(r))               # [0, inf) is ReLU
    # idempotent, and ordered bounds hold for every element
    c = L.clamp(r, -0.5, 2.0)
    assert np.array_equal(L.clamp(c, -0.5, 2.0), c) and c.min() >= -0.5 and c.max() <= 2.0


# ------------------------------------------------------------------ ceil mode
def test_ceil_mode_output_size_rule():
    """One more window when the floor-mode windows leave cells uncovered, dropped again if it
    would start beyond the input and its leading padding; checked against the framework's own
    shape rule for a sweep of sizes, and on hand-computed cases."""
    assert L.pool_out(5, 2, 2, 0, True) == 3 and L.pool_out(5, 2, 2, 0, False) == 2
    assert L.pool_out(6, 2, 2, 0, True) == 3                      # nothing uncovered: same as floor
    assert L.pool_out(3, 2, 2, 1, True) == 2                      # third window would start at 3 >= 3 + 1 - ... dropped
    assert L.pool_out(111, 3, 2, 0, True) == 55 and L.pool_out(112, 3, 2, 0, True) == 56
    for size in range(1, 24):
        for k in (1, 2, 3, 5):
            for s in (1, 2, 3):
                for p in range(0, k // 2 + 1):
                    if size + 2 * p < k:
                        continue
                    want = F.max_pool2d(torch.zeros(1, 1, size, size), k, s, p, ceil_mode=True).shape[-1]
                    assert L.pool_out(size, k, s, p, True) == want == wl.pool_out(size, k, s, p, True), (size, k, s, p)


@pytest.mark.parametrize("H,W,k,s,p", [(5, 5, 2, 2, 0), (7, 9, 3, 2, 0), (7, 9, 3, 2, 1), (10, 11, 3, 3, 1),
                                       (13, 13, (3, 2), (2, 3), (1, 0)), (6, 6, 2, 2, 0)])
def test_ceil_mode_pools_vs_torch(H, W, k, s, p):
    x = wl.activation((2, 3, H, W), 11)
    t = torch.from_numpy(x)
    y, idx = L.maxpool(x, wl._pair(k), wl._pair(s), wl._pair(p), True, True)
    ty, tidx = F.max_pool2d(t, k, s, p, ceil_mode=True, return_indices=True)
    assert y.shape == tuple(ty.shape)
    assert np.array_equal(y, ty.numpy()) and np.array_equal(idx, tidx.numpy().astype(np.int32))
    for cip in (True, False):
        a = L.avgpool(x, wl._pair(k), wl._pair(s), wl._pair(p), cip, True)
        ta = F.avg_pool2d(t.double(), k, s, p, ceil_mode=True, count_include_pad=cip).numpy()
        assert a.shape == ta.shape
        assert np.abs(a - ta).max() <= 1e-6 * max(1.0, np.abs(ta).max())


def test_ceil_mode_average_divisor_closed_form():
    """Constant input 1: an overhanging window averages (in-range cells) / (cells inside the
    padded input) with count_include_pad, and exactly 1 without."""
    x = np.ones((1, 1, 5, 5), np.float32)
    a = L.avgpool(x, (2, 2), (2, 2), (0, 0), True, True)      # 3x3 outputs; last row/col overhang by one
    assert a.shape == (1, 1, 3, 3)
    assert np.array_equal(a[0, 0], np.ones((3, 3), np.float32))   # overhang is outside the padded input: not counted
    b = L.avgpool(x, (3, 3), (2, 2), (1, 1), True, True)      # 5 + 2 - 3 = 4 -> 3 outputs, no overhang beyond padding
    assert b.shape == (1, 1, 3, 3)
    assert b[0, 0, 0, 0] == np.float32(4) * (np.float32(1) / np.float32(9))   # corner: 4 in-range of 9
    c = L.avgpool(x, (3, 3), (2, 2), (1, 1), False, True)
    assert np.array_equal(c[0, 0], np.ones((3, 3), np.float32))
    x6 = np.ones((1, 1, 6, 6), np.float32)
    d = L.avgpool(x6, (3, 3), (2, 2), (1, 1), True, True)     # 4 outputs; last window rows 5..7: 1 in range, 2 inside padded
    assert d.shape == (1, 1, 4, 4)
    assert d[0, 0, 3, 1] == np.float32(3) * (np.float32(1) / np.float32(6))   # 1 row x 3 cols in range / 2 x 3 counted


def test_round_bf16_vs_library_and_ties():
    x = _x((1, 1, 64, 64), 13) * 100
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(L.round_bf16(x), ref)
    t = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -20, -1 - 2.0 ** -8,
                  0.0, -0.0, np.inf, 3.4e38], np.float32)
    r = L.round_bf16(t)
    assert r[0] == 1.0 and r[1] == np.float32(1 + 2.0 ** -6) and r[2] == np.float32(1 + 2.0 ** -7)
    assert r[3] == -1.0 and r[6] == np.inf and r[7] == np.inf
    assert np.signbit(r[5]) and not np.signbit(r[4])
    assert np.isnan(L.round_bf16(np.array([np.nan], np.float32))[0])
