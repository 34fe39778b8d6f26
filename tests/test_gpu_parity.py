"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by
element, on the same seeded inputs.

Bars (the benchmark spec): max-pool argmax indices bit-exact; float32 values within
1e-5 * max|ref|; bfloat16 within 1e-2 * max|ref|.  Both sides use the same fixed
float32 operation order per layer, so values are in fact expected to be
bit-identical; the count of differing elements is printed as a diagnostic.
"""
import numpy as np
import pytest
import torch

from oracle import breadth_first as bf
from paper_1804_08378_amd import brainslug as bs
from paper_1804_08378_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 1e-2, "f16": 1e-3}
TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}


def _dev(a, dtype):
    t = torch.from_numpy(np.ascontiguousarray(a))
    return t.to(TORCH_DTYPE[dtype]).cuda()  # inputs are representable in the storage type: lossless


def run_gpu(layers, x, res, dtype, **opts):
    st = bs.Stack(layers, x.shape, dtype).plan(**opts)
    # a channels-last plan takes channels_last tensors; the values read back are the logical N, C, H, W ones
    mf = torch.channels_last if opts.get("layout") == bs.BS_LAYOUT_NHWC else torch.contiguous_format
    out, idx = st.run(_dev(x, dtype).contiguous(memory_format=mf), [_dev(r, dtype).contiguous(memory_format=mf) for r in res])
    torch.cuda.synchronize()
    info = st.info()
    o = np.ascontiguousarray(out.float().cpu().numpy())
    ii = [np.ascontiguousarray(t.cpu().numpy()) for t in idx]
    st.close()
    return o, ii, info


def check(layers, x, res, dtype, label, **opts):
    """One stack through the HIP path against the oracle.  When the plan uses kernels built at
    plan time for the stack's signature, the same stack is checked again with such builds
    switched off (the kernels that read shapes at run time), so both paths stay covered."""
    ref, ref_idx, _ = bf.run_stack(layers, x, res, dtype)
    info = _check_one(layers, x, res, dtype, label, ref, ref_idx, **opts)
    if "jit" not in opts and any(q["run_time_build"] for q in info["sequences"]):
        _check_one(layers, x, res, dtype, label + "/no-run-time-build", ref, ref_idx, jit=-1, **opts)
    return info


def _check_one(layers, x, res, dtype, label, ref, ref_idx, **opts):
    print(f"[parity] {label} shape={x.shape} dtype={dtype} opts={opts}", flush=True)
    out, idx, info = run_gpu(layers, x, res, dtype, **opts)
    assert out.shape == ref.shape
    scale = float(np.abs(ref).max()) or 1.0
    err = float(np.abs(out - ref).max())
    ndiff = int((out.view(np.uint32) != ref.view(np.uint32)).sum())
    print(f"         max|err|={err:.3e} (bar {TOL[dtype] * scale:.3e}) non-identical={ndiff} "
          f"variants={[q['variant_name'] + ('*' if q['run_time_build'] else '') for q in info['sequences']]}", flush=True)
    assert err <= TOL[dtype] * scale, label
    assert len(idx) == len(ref_idx)
    for k, (a, b) in enumerate(zip(idx, ref_idx)):
        assert a.shape == b.shape
        assert np.array_equal(a, b), f"{label}: argmax output {k} differs in {(a != b).sum()} cells"
    assert ndiff == 0, f"{label}: values within tolerance but not bit-identical ({ndiff})"
    return info


def _shrunk(name, dtype, batch=2, indices=True, seed=0):
    layers, x, res = wl.inputs_for(name, seed, dtype, batch=batch, indices=indices)
    return layers, x, res


# ------------------------------------------------------------------ named configs
CASES = [(n, d) for n in wl.CONFIG_NAMES for d in wl.build(n)[2]]


@pytest.mark.parametrize("name,dtype", CASES)
def test_config_reduced_batch(name, dtype):
    layers, x, res = _shrunk(name, dtype, batch=3)
    check(layers, x, res, dtype, f"{name}/auto")


@pytest.mark.parametrize("name,dtype", CASES)
def test_config_layer_by_layer_plan_is_identical(name, dtype):
    """Breadth-first plan (one kernel per layer, Figure 2) on the GPU: second witness."""
    layers, x, res = _shrunk(name, dtype, batch=2)
    info = check(layers, x, res, dtype, f"{name}/breadth_first", breadth_first=1)
    assert info["n_sequences"] == len(layers)


@pytest.mark.parametrize("name,dtype", [c for c in CASES if "pool" in
                                        " ".join(l["kind"] for l in wl.build(c[0])[0])])
@pytest.mark.parametrize("tile", [(3, 5, 1), (1, 1, 2), (7, 1000, 3)])
def test_config_forced_lds_tiles(name, dtype, tile):
    """Every pooling config through the LDS kernel with small, ragged tiles: halo
    recompute, padding at tile edges, several planes per work-group."""
    layers, x, res = _shrunk(name, dtype, batch=1)
    c = min(x.shape[1], 5)
    for l in layers:
        if l["kind"] == "bn":
            for key in ("gamma", "beta", "mean", "var"):
                l[key] = l[key][:c]
    x = np.ascontiguousarray(x[:, :c, :40, :36])
    res = [np.ascontiguousarray(r[:, :c, :40, :36]) for r in res]
    info = check(layers, x, res, dtype, f"{name}/lds{tile}", force_variant=bs.BS_VARIANT_LDS_TILE,
                 tile_rows=tile[0], tile_cols=tile[1], planes_per_group=tile[2])
    assert all(q["variant_name"] == "lds_tile" for q in info["sequences"])


# ------------------------------------------------------------------ ragged shapes
def _stacks(c):
    return {
        "bn_relu_max2": [wl.bn_params(c, 1), wl.relu(), wl.maxpool(2, 2, 0, True)],
        "bn_relu_max3s2p1": [wl.bn_params(c, 2), wl.relu(), wl.maxpool(3, 2, 1, True)],
        "bn_add_relu": [wl.bn_params(c, 3), wl.add(), wl.relu()],
        "bn_relu_avg2": [wl.bn_params(c, 4), wl.relu(), wl.avgpool(2, 2)],
        "halo_stress": [wl.bn_params(c, 5), wl.relu(), wl.avgpool(3, 1, 1, True),
                        wl.maxpool(3, 2, 1, True), wl.bn_params(c, 6), wl.relu()],
        "max_bn_relu_x3": sum(([wl.maxpool(3, 1, 1, True), wl.bn_params(c, 7 + i), wl.relu()]
                               for i in range(3)), []),
        "avg_nopad_div": [wl.relu(), wl.avgpool(3, 2, 1, False), wl.add(), wl.maxpool(2, 1, 0, True)],
        "rect_windows": [wl.bn_params(c, 9), wl.maxpool((3, 2), (2, 1), (1, 0), True),
                         wl.avgpool((2, 3), (1, 2), (1, 1), True)],
        "add_after_pool": [wl.maxpool(2, 2, 0, True), wl.add(), wl.bn_params(c, 10), wl.relu(), wl.add()],
        "max4_direct": [wl.bn_params(c, 11), wl.maxpool(4, 4, 0, True), wl.relu()],
        "avg_1x2_direct": [wl.avgpool((1, 2), (1, 2), 0), wl.bn_params(c, 12)],
        "stride_gt_kernel": [wl.bn_params(c, 13), wl.maxpool(2, 3, 0, True), wl.relu()],
        "mid_idx_then_gap": [wl.maxpool(3, 1, 1, True), wl.relu(), wl.maxpool(2, 3, 0, True)],
    }


SHAPES = [(2, 3, 13, 11), (1, 1, 1, 1), (1, 2, 9, 16), (3, 5, 32, 24), (1, 7, 57, 61), (2, 4, 64, 64)]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_ragged_shapes_all_stacks(shape, dtype):
    for name, layers in _stacks(shape[1]).items():
        if wl.output_shape(layers, shape)[2] < 1 or wl.output_shape(layers, shape)[3] < 1:
            continue
        try:
            ok = all(v >= 1 for v in wl.output_shape(layers, shape))
            # intermediate pools must not produce empty planes either
            cur = shape
            for l in layers:
                cur = wl.output_shape([l], cur)
                ok = ok and cur[2] >= 1 and cur[3] >= 1
        except Exception:
            ok = False
        if not ok:
            continue
        x = wl.activation(shape, 30, dtype)
        res = [wl.activation(s, 31 + i, dtype) for i, s in enumerate(wl.residual_shapes(layers, shape))]
        check(layers, x, res, dtype, f"{name}{shape}/auto")
        check(layers, x, res, dtype, f"{name}{shape}/steps1", max_steps_per_sequence=1)
        if any(l["kind"] in ("maxpool", "avgpool") for l in layers):
            check(layers, x, res, dtype, f"{name}{shape}/lds-small", force_variant=bs.BS_VARIANT_LDS_TILE,
                  tile_rows=2, tile_cols=3, planes_per_group=2, max_lds_bytes=4096)


def test_deep_synthetic_blocks_split_into_sequences():
    """Section 5.1's block <MaxPool 3/1/1, BatchNorm, ReLU> repeated: with a small on-chip
    budget the halo growth forces several sequences; results stay identical."""
    c, blocks = 4, 12
    layers = sum(([wl.maxpool(3, 1, 1, i % 5 == 0), wl.bn_params(c, 40 + i), wl.relu()]
                  for i in range(blocks)), [])
    x = wl.activation((2, c, 33, 29), 50)
    for opts in ({}, {"max_steps_per_sequence": 1}, {"max_steps_per_sequence": 5},
                 {"max_lds_bytes": 8192}, {"max_lds_bytes": 2048, "threads_per_group": 64}):
        info = check(layers, x, [], "f32", f"blocks{blocks}/{opts}", **opts)
        if opts.get("max_steps_per_sequence") == 1:
            assert info["n_sequences"] == blocks
        if opts.get("max_lds_bytes") == 8192:
            assert info["n_sequences"] > 1


@pytest.mark.parametrize("blocks", [5, 12])
def test_deep_synthetic_blocks_at_the_benchmarked_size(blocks):
    """The stacked-blocks experiment of Section 5.1 at the size `bench.py --deep` times
    (64 x 64 x 56 x 56, float32), with the plans it times: whole tensor against the oracle."""
    c = 64
    layers = sum(([wl.maxpool(3, 1, 1), wl.bn_params(c, 100 + i), wl.relu()] for i in range(blocks)), [])
    x = wl.activation((64, c, 56, 56), 0)
    ref, _, _ = bf.run_stack(layers, x, [], "f32")
    for opts in (dict(), dict(max_steps_per_sequence=5), dict(max_steps_per_sequence=1)):
        print(f"[parity] deep{blocks} full size opts={opts}", flush=True)
        out, _, info = run_gpu(layers, x, [], "f32", **opts)
        assert np.array_equal(out.view(np.uint32), ref.view(np.uint32)), opts
        if opts.get("max_steps_per_sequence") == 1:
            assert info["n_sequences"] == blocks


def test_in_place_elementwise_and_stream_argument():
    layers, x, res = _shrunk("resnet_tail", "f32", batch=1)
    ref, _, _ = bf.run_stack(layers, x, res)
    st = bs.Stack(layers, x.shape, "f32").plan()
    xd, rd = _dev(x, "f32"), [_dev(r, "f32") for r in res]
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        st.run(xd, rd, out=xd, indices=[])  # out == in
    s.synchronize()
    assert np.array_equal(xd.cpu().numpy(), ref)


def test_run_argument_errors():
    layers, x, res = _shrunk("resnet_tail", "f32", batch=1)
    st = bs.Stack(layers, x.shape, "f32")
    xd, rd = _dev(x, "f32"), _dev(res[0], "f32")
    out = torch.empty_like(xd)
    h = st.handle
    with pytest.raises(bs.BrainSlugError) as e:
        bs.bs_stack_run(h, xd.data_ptr(), [rd.data_ptr()], out.data_ptr(), None, 0, 0, 0)
    assert e.value.status == 5  # not planned
    st.plan()
    for args, status in [
        ((0, [rd.data_ptr()], out.data_ptr()), 1),
        ((xd.data_ptr(), None, out.data_ptr()), 1),
        ((xd.data_ptr(), [0], out.data_ptr()), 1),
        ((xd.data_ptr() + 4, [rd.data_ptr()], out.data_ptr()), 7),
        ((xd.data_ptr(), [rd.data_ptr()], rd.data_ptr()), 12),
    ]:
        with pytest.raises(bs.BrainSlugError) as e:
            bs.bs_stack_run(h, args[0], args[1], args[2], None, 0, 0, 0)
        assert e.value.status == status, args
    # pooled stack may not run in place; multi-sequence stack needs its workspace
    layers2, x2, _ = _shrunk("halo_stress", "f32", batch=1)
    st2 = bs.Stack(layers2, x2.shape, "f32").plan(max_steps_per_sequence=1)
    x2d = _dev(x2, "f32")
    o2, _ = st2.alloc_outputs()
    assert bs.bs_stack_workspace_bytes(st2.handle) > 0
    with pytest.raises(bs.BrainSlugError) as e:
        bs.bs_stack_run(st2.handle, x2d.data_ptr(), None, o2.data_ptr(), None, 0, 0, 0)
    assert e.value.status == 8
    ws = st2.workspace()
    with pytest.raises(bs.BrainSlugError) as e:
        bs.bs_stack_run(st2.handle, x2d.data_ptr(), None, x2d.data_ptr(), None, ws.data_ptr(),
                        ws.numel(), 0)
    assert e.value.status == 12
    torch.cuda.synchronize()


def test_indices_can_be_skipped():
    layers, x, res = _shrunk("resnet_stem", "f32", batch=1, indices=True)
    ref, _, _ = bf.run_stack(layers, x, res)
    st = bs.Stack(layers, x.shape, "f32").plan()
    out, _ = st.run(_dev(x, "f32"), [], indices=[])
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), ref)


# ------------------------------------------------------------------ full benchmark sizes
@pytest.mark.parametrize("name,dtype", [c for c in CASES if c[0] != "tiny"])
def test_config_full_size(name, dtype):
    """Whole tensors at the benchmark sizes, in the launch configuration the benchmark
    times (automatic plan, indices off as in the bandwidth runs, then on)."""
    layers, x, res = wl.inputs_for(name, 0, dtype, indices=False)
    check(layers, x, res, dtype, f"{name}/full")
    if any(l["kind"] == "maxpool" for l in layers):
        layers, x, res = wl.inputs_for(name, 0, dtype, indices=True)
        check(layers, x, res, dtype, f"{name}/full+indices")


# ------------------------------------------------------------------ rows kernel (no LDS)
def _rows_stacks(c):
    return {
        "stem": [wl.bn_params(c, 60), wl.relu(), wl.maxpool(3, 2, 1, True)],
        "max3s2p1": [wl.maxpool(3, 2, 1, True)],
        "stem_nopad": [wl.bn_params(c, 61), wl.relu(), wl.maxpool(3, 2, 0, True)],
        "max3s2p0": [wl.maxpool(3, 2, 0, False)],
        "relu_max3s2p0": [wl.relu(), wl.maxpool(3, 2, 0, True)],
        "relu_max3s2p1": [wl.relu(), wl.maxpool(3, 2, 1, False)],
        "block": [wl.maxpool(3, 1, 1, True), wl.bn_params(c, 62), wl.relu()],
        "bn_relu_max3s1": [wl.bn_params(c, 63), wl.relu(), wl.maxpool(3, 1, 1, False)],
        "max3s1p1": [wl.maxpool(3, 1, 1, True)],
        "bn_relu_avg3s1": [wl.bn_params(c, 64), wl.relu(), wl.avgpool(3, 1, 1, True)],
        "avg3s1p1": [wl.avgpool(3, 1, 1, True)],
    }


# rows of 8 ... 64 column blocks of four float32 values, one more than a wave holds (the lanes
# of such a plane load their edge columns instead of exchanging them), a wave with 31 idle lanes
ROWS_SHAPES = [(2, 3, 12, 16), (1, 2, 9, 8), (3, 5, 33, 24), (1, 4, 64, 64), (1, 1, 3, 8), (2, 3, 57, 56),
               (1, 2, 10, 256), (1, 1, 7, 264), (2, 3, 20, 136)]


@pytest.mark.parametrize("shape", ROWS_SHAPES)
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_pool_rows_kernel(shape, dtype):
    """Single pooling step with overlapping / padded windows through the register-sliding
    rows kernels -- lanes exchanging their edge columns, and lanes loading them -- for several
    chunk lengths (1 row per lane, ragged, whole plane)."""
    for name, layers in _rows_stacks(shape[1]).items():
        x = wl.activation(shape, 70, dtype)
        for rc in (0, 1, 3, 1000):
            for exchange in (0, -1):
                info = check(layers, x, [], dtype, f"rows/{name}{shape}/rc{rc}/x{exchange}", tile_rows=rc,
                             lane_exchange=exchange)
                assert info["sequences"][0]["variant_name"] == "pool_rows", name
        # work-groups of one and of three waves (the kernels have no barrier: any number of whole waves)
        for threads in (64, 192):
            info = check(layers, x, [], dtype, f"rows/{name}{shape}/threads{threads}", threads_per_group=threads)
            assert info["sequences"][0]["threads_per_group"] == threads, name
        # the same stack through the LDS kernels agrees as well
        info = check(layers, x, [], dtype, f"rows/{name}{shape}/lds", force_variant=bs.BS_VARIANT_LDS_TILE)
        assert info["sequences"][0]["variant_name"] == "lds_tile"


def _rows2_stacks(c):
    return {
        "halo": [wl.bn_params(c, 65), wl.relu(), wl.avgpool(3, 1, 1, True), wl.maxpool(3, 2, 1, True),
                 wl.bn_params(c, 66), wl.relu()],
        "halo_in_range_count": [wl.bn_params(c, 65), wl.relu(), wl.avgpool(3, 1, 1, False), wl.maxpool(3, 2, 1, False),
                                wl.bn_params(c, 66), wl.relu()],
        "blocks2": [wl.maxpool(3, 1, 1, False), wl.bn_params(c, 67), wl.relu(),
                    wl.maxpool(3, 1, 1, True), wl.bn_params(c, 68), wl.relu()],
        "listing2": [wl.maxpool(3, 1, 1, False), wl.bn_params(c, 69), wl.relu(), wl.avgpool(3, 1, 1, True)],
    }


@pytest.mark.parametrize("shape", ROWS_SHAPES + [(1, 2, 1, 8), (2, 2, 2, 16)])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_pool_rows2_kernel(shape, dtype):
    """Two pooling steps in one sequence through the two-level register-sliding kernels (lanes
    exchanging their edge columns, and lanes recomputing them), for several chunk lengths (1 row
    per lane, ragged, whole plane), and the same stacks through the LDS kernels."""
    for name, layers in _rows2_stacks(shape[1]).items():
        x = wl.activation(shape, 71, dtype)
        for rc in (0, 1, 3, 1000):
            for exchange in (0, -1):
                info = check(layers, x, [], dtype, f"rows2/{name}{shape}/rc{rc}/x{exchange}", tile_rows=rc,
                             force_variant=bs.BS_VARIANT_POOL_ROWS, lane_exchange=exchange)
                assert info["n_sequences"] == 1, name
                assert info["sequences"][0]["variant_name"] == "pool_rows", name
        for threads in (64, 192):
            info = check(layers, x, [], dtype, f"rows2/{name}{shape}/threads{threads}", threads_per_group=threads,
                         force_variant=bs.BS_VARIANT_POOL_ROWS)
            assert info["sequences"][0]["threads_per_group"] == threads, name
        info = check(layers, x, [], dtype, f"rows2/{name}{shape}/lds", force_variant=bs.BS_VARIANT_LDS_TILE)
        assert [q["variant_name"] for q in info["sequences"]] == ["lds_tile"] * info["n_sequences"]


@pytest.mark.parametrize("shape", [(2, 3, 56, 56), (1, 2, 33, 24), (2, 2, 7, 8), (1, 1, 1, 8), (1, 2, 5, 256), (1, 1, 70, 16)])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_chains_of_identical_pooling_blocks_in_registers(shape, dtype):
    """Two to eight blocks <MaxPool 3/1/1, BatchNorm, ReLU> (Section 5.1) in one sequence: the kernel in which a
    new input row ripples through all levels in registers, for several chunk lengths (one row per lane, ragged, a
    quarter of the plane, the whole plane); the same stacks through the LDS kernels; what the chain kernel does not
    take (binary16 storage, lanes that must not exchange columns, an index output inside, other lists)."""
    c = shape[1]
    vec = 4 if dtype == "f32" else 8
    chain = shape[3] % vec == 0 and shape[3] // vec <= 64  # binary16: a run-time build of the same kernel
    for blocks in (2, 3, 4, 5, 8):
        layers = sum(([wl.maxpool(3, 1, 1), wl.bn_params(c, 300 + i), wl.relu()] for i in range(blocks)), [])
        x = wl.activation(shape, 72, dtype)
        x[:, :, ::2, 1::3] = 0.5  # equal values inside windows
        for rc in (0, 1, 3, 1000):
            info = check(layers, x, [], dtype, f"chain/{blocks}{shape}/rc{rc}", tile_rows=rc, max_steps_per_sequence=blocks)
            assert info["n_sequences"] == 1
            other = ("lds_tile", "pool_rows") if blocks == 2 else ("lds_tile",)  # two blocks: also the two-level kernel
            assert info["sequences"][0]["variant_name"] in (("rows_chain",) if chain else other), (blocks, rc)
        for opts in (dict(lane_exchange=-1), dict(force_variant=bs.BS_VARIANT_LDS_TILE)):
            info = check(layers, x, [], dtype, f"chain/{blocks}{shape}/{opts}", max_steps_per_sequence=blocks, **opts)
            other = ("lds_tile", "pool_rows") if blocks == 2 and "lane_exchange" in opts else ("lds_tile",)
            assert all(q["variant_name"] in other for q in info["sequences"]), (blocks, opts)
    # other lists and windows: run-time builds of the chain kernel
    for layers in (sum(([wl.maxpool(3, 1, 1), wl.bn_params(c, 316 + i), wl.leaky_relu(0.1)] for i in range(3)), []),
                   sum(([wl.maxpool(5, 1, 2), wl.clamp(-0.5, 1.0), wl.bn_params(c, 320 + i)] for i in range(4)), []),
                   sum(([wl.maxpool((3, 1), 1, (1, 0))] for i in range(5)), [])):
        info = check(layers, wl.activation(shape, 74, dtype), [], dtype, f"chain/built{shape}", max_steps_per_sequence=8)
        assert [q["variant_name"] for q in info["sequences"]] == (["rows_chain"] if chain else ["lds_tile"] * info["n_sequences"])
    # an index output inside the chain, a list in front of the first pooling: the LDS tiles
    for layers in ([wl.maxpool(3, 1, 1), wl.bn_params(c, 310), wl.relu(), wl.maxpool(3, 1, 1, True), wl.bn_params(c, 311), wl.relu(),
                    wl.maxpool(3, 1, 1), wl.bn_params(c, 312), wl.relu()],
                   [wl.relu()] + sum(([wl.maxpool(3, 1, 1), wl.bn_params(c, 313 + i), wl.relu()] for i in range(3)), [])):
        info = check(layers, wl.activation(shape, 73, dtype), [], dtype, f"chain/not taken{shape}", max_steps_per_sequence=3)
        assert all(q["variant_name"] != "rows_chain" for q in info["sequences"])


# ------------------------------------------------------------------ run-time builds
def _built_stacks(c):
    """Signatures with no instance compiled into the library."""
    return {
        "max5s1p2": ([wl.maxpool(5, 1, 2, True), wl.bn_params(c, 80), wl.relu()], 0),
        "avg2s1p0": ([wl.relu(), wl.avgpool(2, 1, 0)], 0),
        "max3x2": ([wl.bn_params(c, 81), wl.maxpool((3, 2), (1, 2), (1, 0), True)], 0),
        "three_levels": ([wl.maxpool(3, 2, 1), wl.bn_params(c, 82), wl.relu(), wl.avgpool(2, 2, 0),
                          wl.maxpool(3, 1, 1, True)], 0),
        "listing2": ([wl.maxpool(3, 1, 1), wl.bn_params(c, 83), wl.relu(), wl.avgpool(2, 2, 0)], 0),
        "residual": ([wl.bn_params(c, 84), wl.add(), wl.relu(), wl.maxpool(3, 2, 1, True), wl.bn_params(c, 85),
                      wl.relu(), wl.avgpool(3, 1, 1, False)], 1),
        "two_max": ([wl.maxpool(3, 1, 1, True), wl.relu(), wl.maxpool(3, 2, 0, True)], 0),
    }


@pytest.mark.parametrize("shape", [(2, 3, 24, 32), (1, 2, 31, 30), (2, 4, 17, 16)])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_run_time_builds(shape, dtype):
    """Stacks whose signature has no pre-compiled kernel get one built at plan time (required
    here: a failed build fails the plan); the result matches the oracle, and so does the same
    stack on the kernels that read shapes at run time."""
    for name, (layers, n_res) in _built_stacks(shape[1]).items():
        x = wl.activation(shape, 72, dtype)
        res = [wl.activation(shape, 73 + i, dtype) for i in range(n_res)]
        info = check(layers, x, res, dtype, f"built/{name}{shape}", jit=1)
        assert any(q["run_time_build"] for q in info["sequences"]), name
        check(layers, x, res, dtype, f"built/{name}{shape}/off", jit=-1)


# ------------------------------------------------------------------ random stacks
def _random_stack(rng, c, h, w, small=False):
    """A random valid stack: 1..8 layers, every pooling output at least 1 x 1.  `small`: short
    stacks with windows up to 3 x 3 and strides up to 2 and no residuals -- the shapes the
    register kernels take when the width is a multiple of the vector width."""
    layers, res_shapes, n_idx, ew_run = [], [], 0, 0
    kinds = ["bn", "relu", "leaky", "clamp", "add", "max", "max", "avg", "avg"]
    if small:
        kinds.remove("add")
    for _ in range(int(rng.integers(1, 5 if small else 9))):
        kind = rng.choice(kinds)
        if kind in ("max", "avg"):
            k = (int(rng.integers(1, 4 if small else 6)), int(rng.integers(1, 4 if small else 6)))
            st = (int(rng.integers(1, 3 if small else 4)), int(rng.integers(1, 3 if small else 4)))
            p = (int(rng.integers(0, k[0] // 2 + 1)), int(rng.integers(0, k[1] // 2 + 1)))
            ceil = bool(rng.integers(0, 3) == 0)
            ho, wo = wl.pool_out(h, k[0], st[0], p[0], ceil), wl.pool_out(w, k[1], st[1], p[1], ceil)
            if h + 2 * p[0] < k[0] or w + 2 * p[1] < k[1] or ho < 1 or wo < 1:
                continue
            if kind == "max":
                want_idx = bool(rng.integers(0, 2)) and n_idx < 4
                n_idx += want_idx
                layers.append(wl.maxpool(k, st, p, want_idx, ceil_mode=ceil))
            else:
                layers.append(wl.avgpool(k, st, p, bool(rng.integers(0, 2)), ceil_mode=ceil))
            h, w, ew_run = ho, wo, 0
            continue
        if ew_run >= 5:
            continue
        ew_run += 1
        if kind == "bn":
            layers.append(wl.bn_params(c, int(rng.integers(0, 1000))))
        elif kind == "relu":
            layers.append(wl.relu())
        elif kind == "leaky":
            layers.append(wl.leaky_relu(float(rng.choice([0.01, 0.1, 0.3]))))
        elif kind == "clamp":
            layers.append(wl.clamp(float(rng.choice([-1.0, 0.0, -0.25])), float(rng.choice([0.5, 1.0, 6.0]))))
        elif len(res_shapes) < 4:
            layers.append(wl.add())
            res_shapes.append((h, w))
    return layers or [wl.relu()], res_shapes


@pytest.mark.parametrize("seed", range(12))
def test_random_stacks_match_the_oracle(seed):
    """Seeded random stacks (all layer kinds, odd window shapes, ceil mode, residuals, index
    outputs) on random small shapes, through the automatic plan and the other plan modes."""
    rng = np.random.default_rng(1000 + seed)
    done = 0
    for case in range(10):
        n, c = int(rng.integers(1, 4)), int(rng.integers(1, 6))
        h = int(rng.choice([5, 7, 8, 12, 16, 20, 24, 31, 40]))
        w = int(rng.choice([5, 8, 9, 12, 16, 24, 32, 40]))
        small = seed >= 6
        if small:
            w = int(rng.choice([8, 16, 24, 32, 40, 48]))
        dtype = ("f32", "bf16", "f16")[(seed + case) % 3]
        layers, res_shapes = _random_stack(rng, c, h, w, small)
        x = wl.activation((n, c, h, w), 2000 + 10 * seed + case, dtype)
        res = [wl.activation((n, c) + rs, 3000 + i, dtype) for i, rs in enumerate(res_shapes)]
        opts = [dict(), dict(jit=-1), dict(force_variant=bs.BS_VARIANT_LDS_TILE), dict(breadth_first=1),
                dict(layout=bs.BS_LAYOUT_NHWC),
                dict(max_steps_per_sequence=1)][int(rng.integers(0, 6))]
        label = f"random/{seed}.{case} {[l['kind'] for l in layers]}"
        try:
            check(layers, x, res, dtype, label, **opts)
            done += 1
        except bs.BrainSlugError as e:
            # a combination the planner declines (too many element-wise operations on one level,
            # an index output the tiles cannot cover, ...) is reported, not hidden
            assert e.status in (4, 6), label
            print(f"         declined with {e}", flush=True)
    assert done >= 7


# ------------------------------------------------------------------ tracing
def test_tracing_ranges_do_not_change_results():
    """BS_TRACE=1 wraps every sequence launch in a rocTX range (looked up at run time); a traced
    run in a fresh process gives the oracle's result."""
    import os
    import subprocess
    import sys
    code = (
        "import numpy as np, torch\n"
        "from oracle import breadth_first as bf\n"
        "from paper_1804_08378_amd import brainslug as bs, workloads as wl\n"
        "layers = [wl.bn_params(4, 1), wl.relu(), wl.maxpool(3, 2, 1, True), wl.maxpool(3, 1, 1), wl.bn_params(4, 2),\n"
        "          wl.relu(), wl.avgpool(5, 1, 2), wl.relu()]\n"
        "x = wl.activation((2, 4, 24, 32), 3)\n"
        "st = bs.Stack(layers, x.shape, 'f32').plan(max_steps_per_sequence=1)\n"
        "assert st.info()['n_sequences'] == 3\n"
        "out, idx = st.run(torch.from_numpy(x).cuda())\n"
        "torch.cuda.synchronize()\n"
        "ref, ridx, _ = bf.run_stack(layers, x)\n"
        "assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32))\n"
        "assert np.array_equal(idx[0].cpu().numpy(), ridx[0])\n"
        "print('traced run ok')\n")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    env = dict(os.environ, BS_TRACE="1", PYTHONPATH=root)
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=env, cwd=root, timeout=300)
    assert r.returncode == 0 and "traced run ok" in r.stdout, r.stdout[-2000:] + r.stderr[-4000:]


# ------------------------------------------------------------------ 64-bit column blocks
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_sixteen_bit_rows_of_four_mod_eight_use_the_disjoint_window_kernel(dtype):
    """16-bit storage, rows that are a multiple of 4 but not of 8 elements (the 28 x 28 planes of VGG and
    DenseNet): the disjoint-window kernel with one 64-bit vector per lane and row, not the tile kernel."""
    c = 6
    for layers, shape in (([wl.bn_params(c, 1), wl.relu(), wl.maxpool(2, 2, 0, True)], (3, c, 28, 28)),
                          ([wl.bn_params(c, 2), wl.relu(), wl.avgpool(2, 2), wl.bn_params(c, 3), wl.add()], (2, c, 28, 28)),
                          ([wl.add(), wl.leaky_relu(0.1), wl.maxpool((3, 4), (3, 4), 0, True), wl.relu()], (2, c, 9, 12)),
                          ([wl.avgpool((2, 1), (2, 1)), wl.clamp(-0.5, 0.5)], (2, c, 10, 20))):
        x = wl.activation(shape, 7, dtype)
        res = [wl.activation(s, 8 + i, dtype) for i, s in enumerate(wl.residual_shapes(layers, shape))]
        info = check(layers, x, res, dtype, f"64-bit column blocks {shape}")
        q = info["sequences"][0]
        assert [v["variant_name"] for v in info["sequences"]] == ["pool_direct"]
        # one lane per output row and block of four input columns
        ho = wl.output_shape([l for l in layers if l["kind"] in ("maxpool", "avgpool")], shape)[2]
        lanes = shape[0] * shape[1] * ho * (shape[3] // 4)
        assert 0 <= q["grid"] * q["threads_per_group"] - lanes < q["threads_per_group"]


# ------------------------------------------------------------------ HIP graph capture
def test_run_can_be_captured_in_a_hip_graph_and_replayed():
    """bs_stack_run only enqueues kernels on the caller's stream (no allocation, no
    synchronisation, no memset), so a whole multi-sequence stack -- pre-compiled kernels and one
    built at plan time -- can be captured once and replayed; every replay, with new input
    contents and eager work in between, matches the oracle."""
    c = 6
    layers = ([wl.bn_params(c, 40), wl.relu(), wl.maxpool(2, 2, 0, True)] +
              sum(([wl.maxpool(3, 1, 1), wl.bn_params(c, 41 + i), wl.relu()] for i in range(7)), []) +
              [wl.maxpool(5, 1, 2), wl.leaky_relu(0.1), wl.add(), wl.avgpool(2, 2, 0)])
    shape = (2, c, 32, 48)
    st = bs.Stack(layers, shape, "f32").plan()
    info = st.info()
    assert info["n_sequences"] >= 2 and info["workspace_bytes"] > 0
    assert any(q["run_time_build"] for q in info["sequences"])
    rshape = (2, c, 16, 24)
    x_static = torch.zeros(shape, device="cuda")
    r_static = torch.zeros(rshape, device="cuda")
    out, idx = st.alloc_outputs("cuda", True)
    st.workspace("cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        st.run(x_static, [r_static], out=out, indices=idx)  # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        st.run(x_static, [r_static], out=out, indices=idx)
    for rep in range(3):
        x = wl.activation(shape, 50 + rep)
        r = wl.activation(rshape, 60 + rep)
        x_static.copy_(torch.from_numpy(x))
        r_static.copy_(torch.from_numpy(r))
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        ref, ref_idx, _ = bf.run_stack(layers, x, [r])
        assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32)), rep
        assert np.array_equal(idx[0].cpu().numpy(), ref_idx[0]), rep
        # eager launch of the same stack between replays
        o2, _ = st.run(x_static, [r_static])
        torch.cuda.synchronize()
        assert torch.equal(o2, out)
    del graph
    st.close()


# ------------------------------------------------------------------ global pooling
@pytest.mark.parametrize("shape", [(3, 5, 7, 7), (2, 4, 1, 1), (1, 300, 6, 5), (2, 3, 13, 9)])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_global_pooling_one_lane_per_plane(shape, dtype):
    """Pools whose window is the whole plane (the head of a network): average and maximum with
    indices, element-wise layers (a residual Add among them) before and after."""
    h, w = shape[2], shape[3]
    x = wl.activation(shape, 77, dtype)
    out_shape = shape[:2] + (1, 1)
    stacks = {
        "avg_head": ([wl.bn_params(shape[1], 98), wl.relu(), wl.avgpool((h, w), (h, w), 0)], []),
        "max_head": ([wl.leaky_relu(0.1), wl.maxpool((h, w), (1, 1), 0, True), wl.bn_params(shape[1], 99)], []),
        "residuals": ([wl.add(), wl.relu(), wl.avgpool((h, w), (h, w), 0, False), wl.add(), wl.relu6()],
                      [wl.activation(shape, 78, dtype), wl.activation(out_shape, 79, dtype)]),
    }
    for name, (layers, res) in stacks.items():
        info = check(layers, x, res, dtype, f"global/{name}{shape}")
        if h * w > 4:
            assert info["sequences"][0]["variant_name"] in ("plane_pool", "pool_rows"), name
        check(layers, x, res, dtype, f"global/{name}{shape}/lds", force_variant=bs.BS_VARIANT_LDS_TILE)


# ------------------------------------------------------------------ maximum sizes
def _slice_bn(layers, lo, hi):
    out = []
    for l in layers:
        if l["kind"] == "bn":
            l = dict(l, **{key: l[key][lo:hi] for key in ("gamma", "beta", "mean", "var")})
        out.append(l)
    return out


@pytest.mark.parametrize("layout", [bs.BS_LAYOUT_NCHW, bs.BS_LAYOUT_NHWC])
@pytest.mark.parametrize("dtype,stack", [("bf16", "bn_relu"), ("f16", "bn_relu_max2"), ("bf16", "relu_max3s2p1"),
                                         ("f32", "bn_add_relu_small")])
def test_tensors_close_to_the_largest_supported_size(layout, dtype, stack):
    """Tensors of just under 2^31 elements (the library's limit; all index arithmetic is 32-bit).
    The input is drawn on the device (seeded); the planes of a few channels from both ends and the
    middle of the tensor are copied back and checked against the oracle run on those planes alone
    (every plane is independent of the others in all supported layers)."""
    c = 2040
    shape = (1, c, 1024, 1024) if stack != "bn_add_relu_small" else (1, 680, 1024, 1024)  # 2.14e9 / 0.71e9 elements
    c = shape[1]
    layers = {"bn_relu": [wl.bn_params(c, 170), wl.relu()],
              "bn_relu_max2": [wl.bn_params(c, 171), wl.relu(), wl.maxpool(2, 2, 0, True)],
              "relu_max3s2p1": [wl.relu(), wl.maxpool(3, 2, 1, True)],
              "bn_add_relu_small": [wl.bn_params(c, 172), wl.add(), wl.relu()]}[stack]
    td = TORCH_DTYPE[dtype]
    mf = torch.channels_last if layout == bs.BS_LAYOUT_NHWC else torch.contiguous_format
    gen = torch.Generator(device="cuda").manual_seed(173)
    x = torch.empty(shape, dtype=td, device="cuda", memory_format=mf).normal_(generator=gen)
    res = [torch.empty(shape, dtype=td, device="cuda", memory_format=mf).normal_(generator=gen)
           for _ in range(wl.num_residuals(layers))]
    print(f"[parity] max-size {stack} {shape} {dtype} layout={layout}", flush=True)
    st = bs.Stack(layers, shape, dtype).plan(layout=layout)
    out, idx = st.run(x, res)
    torch.cuda.synchronize()
    info = st.info()
    st.close()
    print(f"         variants={[q['variant_name'] for q in info['sequences']]}", flush=True)
    for p0 in (0, 1, c // 2, c - 2, c - 1):
        xs = x[:, p0:p0 + 1].float().contiguous().cpu().numpy()
        rs = [r[:, p0:p0 + 1].float().contiguous().cpu().numpy() for r in res]
        ref, ref_idx, _ = bf.run_stack(_slice_bn(layers, p0, p0 + 1), xs, rs, dtype)
        got = out[:, p0:p0 + 1].float().contiguous().cpu().numpy()
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), (stack, p0)
        for a, b in zip(idx, ref_idx):
            assert np.array_equal(a[:, p0:p0 + 1].contiguous().cpu().numpy(), b), (stack, p0)
    del x, res, out, idx
    torch.cuda.empty_cache()


# ------------------------------------------------------------------ odd planes
@pytest.mark.parametrize("shape", [(4, 8, 5, 7), (2, 4, 3, 3), (8, 2, 7, 7), (3, 8, 35, 35), (8, 8, 1, 3), (2, 16, 17, 17)])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_elementwise_stacks_on_planes_that_are_no_multiple_of_the_vector_width(shape, dtype):
    """Element-wise sequences whose plane size is odd but whose tensor is a whole number of
    128-bit vectors run with vectors that straddle plane (and image) boundaries; BatchNorm then
    takes each element's parameters from the right one of two channels.  Also as channel slices,
    where the scalar kernel takes over."""
    c = shape[1]
    stacks = {
        "bn_relu": [wl.bn_params(c, 150), wl.relu()],
        "bn_add_relu": [wl.bn_params(c, 151), wl.add(), wl.relu()],
        "two_bn": [wl.relu(), wl.bn_params(c, 152), wl.leaky_relu(0.1), wl.bn_params(c, 153), wl.clamp(-1.0, 1.0), wl.add()],
        "relu": [wl.relu()],
    }
    for name, layers in stacks.items():
        x = wl.activation(shape, 154, dtype)
        res = [wl.activation(shape, 155 + i, dtype) for i in range(wl.num_residuals(layers))]
        info = check(layers, x, res, dtype, f"odd/{name}{shape}")
        assert [q["variant_name"] for q in info["sequences"]] == ["stream"]
        if shape[1] == 8:
            _check_sliced(layers, x, res, dtype, f"odd/{name}{shape}")


# ------------------------------------------------------------------ channel slices
def _run_sliced(layers, x, res, dtype, lead, trail, **opts):
    """Run with the input and the output as channel slices [lead, lead + C) of tensors with
    lead + C + trail channels, read and written in place.  Returns (out, indices, info); checks
    that no byte of the output tensor outside the slice was written."""
    n, c, h, w = x.shape
    st = bs.Stack(layers, x.shape, dtype).plan(**opts)
    td = TORCH_DTYPE[dtype]
    big_in = torch.full((n, lead + c + trail, h, w), float("nan"), dtype=td, device="cuda")
    big_in[:, lead:lead + c] = _dev(x, dtype)
    oshape = st.out_shape
    guard = 12345.0
    big_out = torch.full((n, lead + c + trail) + tuple(oshape[2:]), guard, dtype=td, device="cuda")
    xs, outs = big_in[:, lead:lead + c], big_out[:, lead:lead + c]
    assert not xs.is_contiguous() or n == 1
    out, idx = st.run(xs, [_dev(r, dtype) for r in res], out=outs)
    torch.cuda.synchronize()
    assert out.data_ptr() == outs.data_ptr()
    assert bool((big_out[:, :lead] == guard).all()) and bool((big_out[:, lead + c:] == guard).all()), \
        "wrote outside the output slice"
    assert bool(torch.isnan(big_in[:, :lead]).all()) and bool(torch.isnan(big_in[:, lead + c:]).all())
    info = st.info()
    o = outs.float().cpu().numpy()
    ii = [t.cpu().numpy() for t in idx]
    st.close()
    return o, ii, info


def _check_sliced(layers, x, res, dtype, label, **opts):
    print(f"[parity] sliced/{label} shape={x.shape} dtype={dtype} opts={opts}", flush=True)
    ref, ref_idx, _ = bf.run_stack(layers, x, res, dtype)
    out, idx, info = _run_sliced(layers, x, res, dtype, 8, 8, **opts)
    ndiff = int((out.view(np.uint32) != ref.view(np.uint32)).sum())
    print(f"         non-identical={ndiff} "
          f"variants={[q['variant_name'] + ('*' if q['run_time_build'] else '') for q in info['sequences']]}", flush=True)
    assert out.shape == ref.shape and ndiff == 0, label
    assert len(idx) == len(ref_idx)
    for a, b in zip(idx, ref_idx):
        assert np.array_equal(a, b), label
    return info


@pytest.mark.parametrize("shape", [(2, 8, 12, 16), (3, 8, 9, 8), (2, 8, 33, 24), (3, 8, 13, 11)])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_channel_slices_are_read_and_written_in_place(shape, dtype):
    """Input and output as channel slices of larger tensors (a concatenation buffer), through
    every kernel family and through several sequences: results identical to the dense run's
    oracle, nothing outside the slices touched.  Eight channels on either side of an
    eight-channel slice keep every image start on a 16-byte boundary for any plane size."""
    c = shape[1]
    stacks = {}
    stacks.update({"s/" + k: (v, None) for k, v in _stacks(c).items()})
    stacks.update({"r/" + k: (v, None) for k, v in list(_rows_stacks(c).items())[:4]})
    stacks.update({"r2/" + k: (v, bs.BS_VARIANT_POOL_ROWS) for k, v in _rows2_stacks(c).items()})
    stacks.update({"b/" + k: (v[0], None) for k, v in _built_stacks(c).items()})
    h, w = shape[2], shape[3]
    stacks["g/avg_head"] = ([wl.bn_params(c, 98), wl.relu(), wl.avgpool((h, w), (h, w), 0)], None)
    stacks["g/max_head"] = ([wl.maxpool((h, w), (1, 1), 0, True), wl.relu()], None)
    seen = set()
    for name, (layers, force) in stacks.items():
        cur, ok = shape, True
        for l in layers:
            cur = wl.output_shape([l], cur)
            ok = ok and cur[2] >= 1 and cur[3] >= 1
        if not ok:
            continue
        x = wl.activation(shape, 90, dtype)
        res = [wl.activation(sh, 91 + i, dtype) for i, sh in enumerate(wl.residual_shapes(layers, shape))]
        plans = [dict(), dict(max_steps_per_sequence=1), dict(jit=-1)]
        if force:
            plans = [dict(force_variant=force)]
        if any(l["kind"] in ("maxpool", "avgpool") for l in layers) and not force:
            plans.append(dict(force_variant=bs.BS_VARIANT_LDS_TILE, tile_rows=3, tile_cols=5, planes_per_group=3))
        for opts in plans:
            info = _check_sliced(layers, x, res, dtype, f"{name}{shape}", **opts)
            seen.update(q["variant_name"] for q in info["sequences"])
    assert {"stream", "lds_tile", "plane_pool"} <= seen
    if shape[3] % 8 == 0:
        assert {"pool_direct", "pool_rows"} <= seen


def test_channel_slice_in_place_and_argument_errors():
    layers = [wl.bn_params(8, 3), wl.relu()]
    x = wl.activation((3, 8, 6, 8), 95)
    ref, _, _ = bf.run_stack(layers, x, [])
    st = bs.Stack(layers, x.shape, "f32").plan()
    big = torch.zeros((3, 24, 6, 8), device="cuda")
    big[:, 8:16] = _dev(x, "f32")
    before = big.clone()
    view = big[:, 8:16]
    st.run(view, out=view, indices=[])  # in place on a slice
    torch.cuda.synchronize()
    assert np.array_equal(view.cpu().numpy(), ref)
    assert torch.equal(big[:, :8], before[:, :8]) and torch.equal(big[:, 16:], before[:, 16:])
    # slices of one buffer that interleave without sharing a byte are fine ...
    big[:, 8:16] = _dev(x, "f32")
    st.run(big[:, 8:16], out=big[:, 16:24], indices=[])
    torch.cuda.synchronize()
    assert np.array_equal(big[:, 16:24].cpu().numpy(), ref)
    # ... overlapping ones are refused, and so are layouts that are not channel slices
    with pytest.raises(bs.BrainSlugError) as e:
        st.run(big[:, 8:16], out=big[:, 12:20], indices=[])
    assert e.value.status == 12
    with pytest.raises(ValueError):
        st.run(torch.zeros((3, 8, 6, 16), device="cuda")[:, :, :, :8], indices=[])
    with pytest.raises(bs.BrainSlugError) as e:
        bs.bs_stack_run_strided(st.handle, big.data_ptr(), 8 * 6 * 8 - 4, None, view.data_ptr(), 0, None, 0, 0, 0)
    assert e.value.status == 2
    st.close()


# ------------------------------------------------------------------ channels last
def _check_nhwc(layers, x, res, dtype, label, **opts):
    """The same stack on channels-last tensors: the oracle's numbers, in another memory order."""
    print(f"[parity] nhwc/{label} shape={x.shape} dtype={dtype} opts={opts}", flush=True)
    ref, ref_idx, _ = bf.run_stack(layers, x, res, dtype)
    cl = torch.channels_last
    st = bs.Stack(layers, x.shape, dtype).plan(layout=bs.BS_LAYOUT_NHWC, **opts)
    out, idx = st.run(_dev(x, dtype).contiguous(memory_format=cl),
                      [_dev(r, dtype).contiguous(memory_format=cl) for r in res])
    torch.cuda.synchronize()
    info = st.info()
    st.close()
    assert out.is_contiguous(memory_format=cl) and all(t.is_contiguous(memory_format=cl) for t in idx)
    o = out.float().cpu().numpy()  # logical N, C, H, W values
    ndiff = int((np.ascontiguousarray(o).view(np.uint32) != ref.view(np.uint32)).sum())
    print(f"         non-identical={ndiff} variants={[q['variant_name'] for q in info['sequences']]}", flush=True)
    assert o.shape == ref.shape and ndiff == 0, label
    assert len(idx) == len(ref_idx)
    for a, b in zip(idx, ref_idx):
        assert np.array_equal(a.cpu().numpy(), b), label
    names = [q["variant_name"] for q in info["sequences"]]
    assert all(v in ("nhwc_stream", "nhwc_pool", "nhwc_tile", "nhwc_rows") for v in names)
    assert sum(2 if v in ("nhwc_tile", "nhwc_rows") else 1 for v in names) == info["n_steps"]
    if opts.get("max_steps_per_sequence") == 1 or opts.get("breadth_first"):
        assert "nhwc_tile" not in names and "nhwc_rows" not in names
    if opts.get("lane_exchange") == -1:
        assert "nhwc_rows" not in names
    return info


NHWC_SHAPES = [(2, 8, 13, 11), (1, 16, 9, 16), (2, 12, 12, 10), (3, 5, 7, 9), (1, 24, 1, 1), (2, 8, 57, 31),
               (1, 1, 6, 5)]


@pytest.mark.parametrize("shape", NHWC_SHAPES)
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_channels_last_plans_match_the_oracle(shape, dtype):
    """Every stack family on channels-last tensors: channel counts that give 128-bit vectors
    for both element sizes (8, 16, 24), for float32 only (12) and for neither (5, 1)."""
    c = shape[1]
    stacks = {}
    for fam, d in (("s", _stacks(c)), ("r", _rows_stacks(c)), ("r2", _rows2_stacks(c)), ("c", _ceil_stacks(c))):
        stacks.update({f"{fam}/{k}": v for k, v in d.items()})
    stacks.update({"b/" + k: v[0] for k, v in _built_stacks(c).items()})
    stacks.update({"a/" + k: v[0] for k, v in _activation_stacks(c).items()})
    h, w = shape[2], shape[3]
    stacks["g/avg_head"] = [wl.bn_params(c, 98), wl.relu(), wl.avgpool((h, w), (h, w), 0)]
    stacks["g/max_head"] = [wl.leaky_relu(0.1), wl.maxpool((h, w), (1, 1), 0, True), wl.bn_params(c, 99)]
    ran = 0
    for name, layers in stacks.items():
        cur, ok = shape, True
        for l in layers:
            if l["kind"] in ("maxpool", "avgpool") and (cur[2] + 2 * l["p"][0] < l["k"][0] or cur[3] + 2 * l["p"][1] < l["k"][1]):
                ok = False
                break
            cur = wl.output_shape([l], cur)
            ok = ok and cur[2] >= 1 and cur[3] >= 1
        if not ok:
            continue
        x = wl.activation(shape, 110, dtype)
        res = [wl.activation(sh, 111 + i, dtype) for i, sh in enumerate(wl.residual_shapes(layers, shape))]
        _check_nhwc(layers, x, res, dtype, f"{name}{shape}")
        ran += 1
    assert ran >= 6


@pytest.mark.parametrize("name,dtype", [("vgg_a", "f32"), ("resnet_stem", "bf16"), ("resnet_tail", "f16"),
                                        ("densenet_trans", "f32"), ("halo_stress", "f32")])
def test_channels_last_configs_reduced_batch(name, dtype):
    layers, x, res = _shrunk(name, dtype, batch=2)
    _check_nhwc(layers, x, res, dtype, name)
    _check_nhwc(layers, x, res, dtype, name + "/step-by-step", max_steps_per_sequence=1)


def _tile_stacks(c):
    """Two pooling steps the channels-last tile kernel exists for: every pair of its windows
    (3 x 3 stride 1 and 2, 2 x 2 stride 2), both pooling kinds on either level, lists in front,
    between and behind (residual operands at each plane size), every divisor rule, ceil mode."""
    win = {"3s1": (3, 1, 1), "3s2": (3, 2, 1), "2s2": (2, 2, 0)}
    stacks = {}
    for a, (k1, s1, p1) in win.items():
        for b, (k2, s2, p2) in win.items():
            stacks[f"avg{a}_max{b}_idx"] = [wl.bn_params(c, 170), wl.relu(), wl.avgpool(k1, s1, p1, True),
                                            wl.maxpool(k2, s2, p2, True), wl.bn_params(c, 171), wl.relu()]
            stacks[f"max{a}_avg{b}"] = [wl.maxpool(k1, s1, p1), wl.bn_params(c, 172), wl.add(), wl.relu(),
                                        wl.avgpool(k2, s2, p2, False), wl.add()]
    # the stacked pooling with its activations and no index output: the instances with the lists (and, 16-bit, the kinds) compiled in
    stacks["halo_stress"] = [wl.bn_params(c, 168), wl.relu(), wl.avgpool(3, 1, 1, True), wl.maxpool(3, 2, 1), wl.bn_params(c, 169), wl.relu()]
    stacks["halo_stress_in_range_count"] = [wl.bn_params(c, 168), wl.relu(), wl.avgpool(3, 1, 1, False), wl.maxpool(3, 2, 1),
                                            wl.bn_params(c, 169), wl.relu()]
    stacks["max_max_lists_move"] = [wl.bn_params(c, 173), wl.relu(), wl.maxpool(3, 2, 1), wl.relu(), wl.bn_params(c, 174),
                                    wl.maxpool(3, 1, 1), wl.leaky_relu(0.2)]
    stacks["add_first"] = [wl.add(), wl.bn_params(c, 175), wl.maxpool(3, 1, 1), wl.clamp(-0.5, 0.75), wl.maxpool(2, 2, 0, True)]
    stacks["avg_avg_ceil"] = [wl.avgpool(3, 2, 1, True, True), wl.bn_params(c, 176), wl.avgpool(2, 2, 0, False, True)]
    stacks["max_ceil_max_ceil"] = [wl.relu(), wl.maxpool(3, 2, 0, False, True), wl.maxpool(3, 2, 1, True, True)]
    stacks["no_padding"] = [wl.bn_params(c, 177), wl.avgpool(3, 1, 0), wl.relu(), wl.maxpool(3, 2, 0, True)]
    return stacks


@pytest.mark.parametrize("shape", [(2, 8, 13, 11), (1, 16, 9, 16), (2, 24, 12, 10), (1, 8, 57, 31), (3, 32, 7, 7), (1, 128, 6, 5)])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_channels_last_two_pools_in_one_kernel(shape, dtype):
    """The tile kernel against the oracle: the planner's own tile, one output per work-group,
    ragged tiles with one channel vector per work-group, and a tile larger than the plane."""
    vec = 4 if dtype == "f32" else 8
    ran = 0
    for name, layers in _tile_stacks(shape[1]).items():
        cur, ok = shape, True
        for l in layers:
            if l["kind"] in ("maxpool", "avgpool") and (cur[2] + 2 * l["p"][0] < l["k"][0] or cur[3] + 2 * l["p"][1] < l["k"][1]):
                ok = False
                break
            cur = wl.output_shape([l], cur)
            ok = ok and cur[2] >= 1 and cur[3] >= 1
        if not ok:
            continue
        x = wl.activation(shape, 178, dtype)
        x[:, :, ::3, ::2] = 0.0  # ties for the maximum and for its index
        res = [wl.activation(sh, 179 + i, dtype) for i, sh in enumerate(wl.residual_shapes(layers, shape))]
        # lane_exchange = -1: the tile kernel also where the register kernel (below) would take the pair
        for opts in ({}, dict(tile_rows=1, tile_cols=1), dict(tile_rows=3, tile_cols=2, planes_per_group=vec),
                     dict(tile_rows=16, tile_cols=16, planes_per_group=vec)):
            info = _check_nhwc(layers, x, res, dtype, f"tile/{name}{shape}", lane_exchange=-1, **opts)
            assert [q["variant_name"] for q in info["sequences"]] == ["nhwc_tile"], name
        ran += 1
    assert ran >= 10


def _nhwc_rows_stacks(c):
    """Pairs of pooling steps the channels-last register kernel is compiled for (3 x 3 windows with padding 1, the
    first with stride 1, the second a maximum with stride 1 or 2, no index output, lists of BatchNorm and ReLU
    in the places the planner leaves them), and pairs it must leave to the tile kernel."""
    mine = {
        "halo_stress": [wl.bn_params(c, 180), wl.relu(), wl.avgpool(3, 1, 1, True), wl.maxpool(3, 2, 1), wl.bn_params(c, 181), wl.relu()],
        "avg_max_s1": [wl.bn_params(c, 182), wl.relu(), wl.avgpool(3, 1, 1, True), wl.maxpool(3, 1, 1), wl.bn_params(c, 183), wl.relu()],
        "avg_max_no_lists": [wl.avgpool(3, 1, 1, True), wl.maxpool(3, 2, 1)],
        "avg_max_front_only": [wl.bn_params(c, 184), wl.relu(), wl.avgpool(3, 1, 1, True), wl.maxpool(3, 2, 1)],
        "avg_max_behind_only": [wl.avgpool(3, 1, 1, True), wl.maxpool(3, 1, 1), wl.bn_params(c, 185), wl.relu()],
        # lists in front of a maximum that never decrease run behind it: both end up behind the second pooling
        "blocks2": [wl.maxpool(3, 1, 1), wl.bn_params(c, 186), wl.relu(), wl.maxpool(3, 1, 1), wl.bn_params(c, 187), wl.relu()],
        "max_max_s2": [wl.maxpool(3, 1, 1), wl.maxpool(3, 2, 1), wl.bn_params(c, 188), wl.relu()],
        "max_max_no_lists": [wl.maxpool(3, 1, 1), wl.maxpool(3, 2, 1)],
    }
    other = {
        "in_range_count": [wl.bn_params(c, 180), wl.relu(), wl.avgpool(3, 1, 1, False), wl.maxpool(3, 2, 1)],
        "with_indices": [wl.avgpool(3, 1, 1, True), wl.maxpool(3, 2, 1, True)],
        "first_stride_2": [wl.avgpool(3, 2, 1, True), wl.maxpool(3, 1, 1)],
        "average_last": [wl.maxpool(3, 1, 1), wl.avgpool(3, 2, 1, True)],
        "other_list": [wl.leaky_relu(0.1), wl.avgpool(3, 1, 1, True), wl.maxpool(3, 2, 1)],
        "add_in_front": [wl.add(), wl.avgpool(3, 1, 1, True), wl.maxpool(3, 2, 1)],
    }
    return mine, other


@pytest.mark.parametrize("shape", [(2, 8, 13, 11), (1, 16, 9, 16), (2, 24, 12, 10), (1, 8, 57, 31), (3, 32, 7, 7), (1, 128, 6, 5),
                                   (2, 64, 56, 56), (1, 8, 3, 64), (1, 8, 1, 1), (1, 16, 70, 2),
                                   (8, 16, 9, 10), (16, 40, 17, 6), (24, 8, 5, 33)])  # batches of 8 k: work-groups ordered by XCD
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_channels_last_two_pools_in_registers(shape, dtype):
    """The channels-last kernel whose lanes are the pixel columns of an image row (neighbouring columns by lane
    shifts, no LDS; 16-bit storage) against the oracle: the planner's chunk length, one output row per chunk, a ragged last chunk,
    the whole image as one chunk; images wider than a wave and the pairs it is not compiled for take the tile kernel."""
    mine, other = _nhwc_rows_stacks(shape[1])
    vec = 4 if dtype == "f32" else 8
    for name, layers in mine.items():
        x = wl.activation(shape, 189, dtype)
        x[:, :, ::3, ::2] = 0.0
        for rc in (0, 1, 3, 5, 1000):
            info = _check_nhwc(layers, x, [], dtype, f"rows/{name}{shape}/rc{rc}", tile_rows=rc)
            names = [q["variant_name"] for q in info["sequences"]]
            if shape[1] % vec == 0 and dtype != "f32":  # compiled for 16-bit storage (float32 is faster through the tile kernel)
                assert names == ["nhwc_rows"], name
                q = info["sequences"][0]
                cvn = shape[1] // vec
                assert q["lds_bytes"] == 0 and q["threads_per_group"] == 64 * max(d for d in (1, 2, 3, 4) if cvn % d == 0)
            else:
                assert "nhwc_rows" not in names
    for name, layers in other.items():
        x = wl.activation(shape, 190, dtype)
        res = [wl.activation(sh, 191 + i, dtype) for i, sh in enumerate(wl.residual_shapes(layers, shape))]
        info = _check_nhwc(layers, x, res, dtype, f"rows-not/{name}{shape}")
        assert "nhwc_rows" not in [q["variant_name"] for q in info["sequences"]], name


def test_channels_last_register_kernel_needs_rows_that_fit_a_wave():
    layers = [wl.avgpool(3, 1, 1, True), wl.maxpool(3, 2, 1)]
    for w, want in ((64, True), (65, False)):
        shape = (1, 8, 5, w)
        info = _check_nhwc(layers, wl.activation(shape, 192, "bf16"), [], "bf16", f"rows/width{w}")
        assert ("nhwc_rows" in [q["variant_name"] for q in info["sequences"]]) == want


def _premax_stacks(c):
    """Max pools without an index output behind lists that never decrease (the pool may then
    run first), and lists that do not qualify (a negative scale or slope, no ReLU, an Add)."""
    neg = wl.bn_params(c, 131)
    neg["gamma"] = neg["gamma"].copy()
    neg["gamma"][::2] *= -1.0
    zero = wl.bn_params(c, 132)
    zero["beta"] = np.zeros(c, np.float32)
    zero["mean"] = np.zeros(c, np.float32)
    return {
        "bn_relu_max3s2": [wl.bn_params(c, 130), wl.relu(), wl.maxpool(3, 2, 1)],
        "bn_relu_max2": [wl.bn_params(c, 130), wl.relu(), wl.maxpool(2, 2)],
        "negative_scales": [neg, wl.relu(), wl.maxpool(3, 2, 1)],
        "zero_shift": [zero, wl.relu(), wl.maxpool(3, 1, 1), wl.bn_params(c, 133)],
        "long_list": [wl.relu(), wl.bn_params(c, 134), wl.leaky_relu(0.1), wl.clamp(-0.5, 2.0), wl.maxpool(2, 2),
                      wl.bn_params(c, 135), wl.relu()],
        "negative_slope": [wl.relu(), wl.bn_params(c, 136), wl.leaky_relu(-0.1), wl.maxpool(2, 2)],
        "no_relu": [wl.bn_params(c, 137), wl.maxpool(3, 2, 1)],
        "add_before": [wl.bn_params(c, 138), wl.add(), wl.relu(), wl.maxpool(2, 2)],
        "any_window": [wl.bn_params(c, 139), wl.relu(), wl.maxpool((2, 3), (1, 2), (1, 1))],
    }


@pytest.mark.parametrize("shape", [(2, 8, 13, 11), (1, 16, 12, 16), (2, 5, 9, 10)])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_channels_last_max_pool_before_monotone_lists(shape, dtype):
    """The planner lets a max pool without index output run before a list of element-wise
    operations that never decrease; the values must stay those of the layer order, bit for
    bit, zeros of both signs in the input included."""
    for name, layers in _premax_stacks(shape[1]).items():
        x = wl.activation(shape, 140, dtype)
        x[:, :, ::3, ::2] = 0.0
        x[:, :, 1::3, 1::2] = -0.0
        res = [wl.activation(sh, 141 + i, dtype) for i, sh in enumerate(wl.residual_shapes(layers, shape))]
        _check_nhwc(layers, x, res, dtype, f"premax/{name}{shape}")


@pytest.mark.parametrize("shape", [(2, 8, 13, 11), (3, 16, 9, 16), (2, 8, 7, 7), (2, 24, 6, 8)])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_channels_last_channel_slices(shape, dtype):
    """Input and output as channel slices of larger channels-last tensors (every pixel holds the
    slice's channels and skips the others): all channels-last kernels, nothing outside the slices
    touched.  Eight channels on either side keep every pixel's slice on a 16-byte boundary."""
    n, c, h, w = shape
    td, cl = TORCH_DTYPE[dtype], torch.channels_last
    stacks = {"bn_relu": [wl.bn_params(c, 160), wl.relu()], "bn_add_relu": [wl.bn_params(c, 161), wl.add(), wl.relu()],
              "stem": [wl.bn_params(c, 162), wl.relu(), wl.maxpool(3, 2, 1, True)],
              "max2": [wl.relu(), wl.maxpool(2, 2, 0, True), wl.bn_params(c, 163)],
              "avg3s1": [wl.bn_params(c, 164), wl.relu(), wl.avgpool(3, 1, 1)],
              "any": [wl.relu(), wl.maxpool((2, 3), (1, 2), (1, 1), True)],
              "head": [wl.bn_params(c, 165), wl.relu(), wl.avgpool((h, w), (h, w), 0)],
              "two_pools": [wl.bn_params(c, 166), wl.relu(), wl.avgpool(3, 1, 1), wl.maxpool(3, 2, 1, True), wl.relu()],
              # without the index output: the register kernel with 16-bit storage
              "two_pools_in_registers": [wl.bn_params(c, 166), wl.relu(), wl.avgpool(3, 1, 1, True), wl.maxpool(3, 2, 1),
                                         wl.bn_params(c, 159), wl.relu()]}
    for name, layers in stacks.items():
        print(f"[parity] nhwc-slice/{name}{shape} {dtype}", flush=True)
        x = wl.activation(shape, 167, dtype)
        res = [wl.activation(sh, 168 + i, dtype) for i, sh in enumerate(wl.residual_shapes(layers, shape))]
        ref, ref_idx, _ = bf.run_stack(layers, x, res, dtype)
        st = bs.Stack(layers, shape, dtype).plan(layout=bs.BS_LAYOUT_NHWC)
        if name == "two_pools_in_registers" and dtype != "f32":
            assert [q["variant_name"] for q in st.info()["sequences"]] == ["nhwc_rows"]
        big_in = torch.full((n, c + 16, h, w), float("nan"), dtype=td, device="cuda").contiguous(memory_format=cl)
        big_in[:, 8:8 + c] = _dev(x, dtype)
        guard = 4321.0
        big_out = torch.full((n, c + 16) + tuple(st.out_shape[2:]), guard, dtype=td, device="cuda").contiguous(memory_format=cl)
        xs, outs = big_in[:, 8:8 + c], big_out[:, 8:8 + c]
        idx = [torch.empty(bs.bs_stack_index_shape(st.handle, i), dtype=torch.int32, device="cuda").contiguous(memory_format=cl)
               for i in range(st.n_idx)]
        resd = [_dev(r, dtype).contiguous(memory_format=cl) for r in res]
        ws = st.workspace("cuda")
        bs.bs_stack_run_strided(st.handle, xs.data_ptr(), bs.batch_stride_nhwc(xs), [r.data_ptr() for r in resd],
                                outs.data_ptr(), bs.batch_stride_nhwc(outs), [t.data_ptr() for t in idx] or None,
                                ws.data_ptr() if ws is not None else 0, ws.numel() if ws is not None else 0,
                                torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        out = outs.float().cpu().numpy()
        assert np.array_equal(np.ascontiguousarray(out).view(np.uint32), ref.view(np.uint32)), name
        for a, b in zip(idx, ref_idx):
            assert np.array_equal(a.cpu().numpy(), b), name
        assert bool((big_out[:, :8] == guard).all()) and bool((big_out[:, 8 + c:] == guard).all()), name
        st.close()


@pytest.mark.parametrize("name,dtype", [("vgg_a", "f32"), ("resnet_stem", "bf16"), ("resnet_tail", "f16"),
                                        ("densenet_trans", "f32"), ("halo_stress", "f16"), ("halo_stress", "f32"),
                                        ("halo_stress", "bf16")])
def test_channels_last_configs_full_size(name, dtype):
    """Whole tensors at the benchmark sizes with channels-last plans, as `bench.py --nhwc` times them."""
    layers, x, res = wl.inputs_for(name, 0, dtype, indices=False)
    _check_nhwc(layers, x, res, dtype, f"{name}/full")


def test_channels_last_argument_checks():
    layers = [wl.bn_params(8, 3), wl.relu(), wl.maxpool(2, 2, 0, True)]
    x = wl.activation((2, 8, 6, 8), 120)
    st = bs.Stack(layers, x.shape, "f32").plan(layout=bs.BS_LAYOUT_NHWC)
    xd = _dev(x, "f32")
    with pytest.raises(ValueError, match="channels_last"):
        st.run(xd)  # an NCHW tensor given to a channels-last plan
    with pytest.raises(bs.BrainSlugError) as e:  # a batch stride that is no whole number of pixels
        bs.bs_stack_run_strided(st.handle, xd.data_ptr(), 8 * 6 * 8 + 64 - 8, None, xd.data_ptr() + (1 << 20), 0, None, 0, 0, 0)
    assert e.value.status == 2
    st.close()
    with pytest.raises(bs.BrainSlugError) as e:
        bs.Stack(layers, x.shape, "f32").plan(layout=bs.BS_LAYOUT_NHWC, force_variant=bs.BS_VARIANT_LDS_TILE)
    assert e.value.status == 3


# ------------------------------------------------------------------ further activations
def _activation_stacks(c):
    return {
        "stream": ([wl.bn_params(c, 93), wl.leaky_relu(0.1), wl.add(), wl.relu6()], 1),
        "direct": ([wl.bn_params(c, 94), wl.relu6(), wl.maxpool(2, 2, 0, True), wl.leaky_relu(0.2)], 0),
        "rows": ([wl.bn_params(c, 95), wl.leaky_relu(0.01), wl.maxpool(3, 2, 1, True), wl.clamp(-0.5, 1.5)], 0),
        "rows2": ([wl.clamp(-1.0, 1.0), wl.avgpool(3, 1, 1), wl.leaky_relu(0.3), wl.maxpool(3, 2, 1, True),
                   wl.bn_params(c, 96), wl.relu6()], 0),
        "lds": ([wl.leaky_relu(0.1), wl.maxpool(3, 1, 1, True), wl.bn_params(c, 97), wl.add(), wl.relu6(),
                 wl.avgpool(2, 2, 0), wl.clamp(0.25, 0.75), wl.maxpool(3, 1, 1)], 1),
    }


@pytest.mark.parametrize("shape", [(2, 3, 24, 32), (1, 2, 31, 30)])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_leaky_relu_and_clamp_in_every_kernel_family(shape, dtype):
    for name, (layers, n_res) in _activation_stacks(shape[1]).items():
        x = wl.activation(shape, 75, dtype) * 3
        res = []
        if n_res:
            rshape = wl.output_shape(layers[:[l["kind"] for l in layers].index("add")], shape)
            res = [wl.activation(rshape, 76, dtype)]
        x = np.ascontiguousarray(x.astype(np.float32))
        from oracle import layers as OL
        x = OL.round_to(x, dtype)
        check(layers, x, res, dtype, f"act/{name}{shape}")
        check(layers, x, res, dtype, f"act/{name}{shape}/layer-by-layer", breadth_first=1)
        check(layers, x, res, dtype, f"act/{name}{shape}/lds", force_variant=bs.BS_VARIANT_LDS_TILE)


# ------------------------------------------------------------------ ceil mode
def _ceil_stacks(c):
    return {
        "squeeze": [wl.relu(), wl.maxpool(3, 2, 0, True, ceil_mode=True)],
        "googlenet": [wl.maxpool(3, 2, 0, False, ceil_mode=True), wl.bn_params(c, 90), wl.relu()],
        "max2s2": [wl.bn_params(c, 91), wl.relu(), wl.maxpool(2, 2, 0, True, ceil_mode=True)],
        "avg_padded_count": [wl.avgpool(3, 2, 1, True, ceil_mode=True), wl.relu()],
        "avg_in_range_count": [wl.avgpool(3, 2, 1, False, ceil_mode=True)],
        "avg2s2": [wl.relu(), wl.avgpool(2, 2, 0, True, ceil_mode=True)],
        "two_pools": [wl.bn_params(c, 92), wl.relu(), wl.maxpool(3, 2, 0, True, ceil_mode=True),
                      wl.avgpool(3, 2, 1, True, ceil_mode=True), wl.relu()],
        "three_pools": [wl.maxpool(3, 2, 1, False, ceil_mode=True), wl.relu(), wl.avgpool(2, 2, 0, False, ceil_mode=True),
                        wl.maxpool(3, 1, 1, True, ceil_mode=True)],
    }


@pytest.mark.parametrize("shape", [(2, 3, 18, 24), (1, 2, 21, 21), (2, 2, 13, 16), (1, 4, 8, 8)])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_ceil_mode_pools(shape, dtype):
    """Ceil-mode pools: one more, overhanging, window per dimension where the floor-mode windows
    leave cells uncovered; its cells outside the plane count like padding."""
    for name, layers in _ceil_stacks(shape[1]).items():
        x = wl.activation(shape, 74, dtype)
        check(layers, x, [], dtype, f"ceil/{name}{shape}")
        check(layers, x, [], dtype, f"ceil/{name}{shape}/lds", force_variant=bs.BS_VARIANT_LDS_TILE)
        check(layers, x, [], dtype, f"ceil/{name}{shape}/layer-by-layer", breadth_first=1)


# ------------------------------------------------------------------ special values
def test_signed_zero_and_subnormals_follow_the_oracle():
    """ReLU maps -0 to +0, subnormal values pass through unchanged, and max pooling of windows
    that mix +0 and -0 returns a zero (sign not compared) with the oracle's argmax."""
    vals = np.array([-0.0, 0.0, -1.0, 1e-40, -1e-40, 2.5, 1e-38, -3.0], np.float32)
    x = np.tile(vals, 64 * 4).reshape(1, 4, 16, 32).copy()
    ref, _, _ = bf.run_stack([wl.relu()], x)
    out, _, _ = run_gpu([wl.relu()], x, [], "f32")
    assert np.array_equal(out.view(np.uint32), ref.view(np.uint32))
    for layers in ([wl.relu(), wl.maxpool(2, 2, 0, True)], [wl.relu(), wl.maxpool(3, 2, 1, True)],
                   [wl.relu(), wl.maxpool(3, 2, 1, False)], [wl.relu(), wl.avgpool(3, 1, 1)]):
        ref, ridx, _ = bf.run_stack(layers, x)
        out, idx, _ = run_gpu(layers, x, [], "f32")
        assert np.array_equal(out.view(np.uint32), ref.view(np.uint32)), layers
        for a, b in zip(idx, ridx):
            assert np.array_equal(a, b)
    # windows holding only zeros of both signs: values compare equal; indices follow the
    # first-maximum rule of the oracle when they are requested
    z = np.zeros((1, 2, 8, 8), np.float32)
    z[:, :, ::2, ::2] = -0.0
    for want in (True, False):
        layers = [wl.maxpool(2, 2, 0, want)]
        ref, ridx, _ = bf.run_stack(layers, z)
        out, idx, _ = run_gpu(layers, z, [], "f32")
        assert np.array_equal(out, ref)
        if want:
            assert np.array_equal(out.view(np.uint32), ref.view(np.uint32))
            assert np.array_equal(idx[0], ridx[0])


def test_one_planned_handle_runs_on_two_streams_at_once():
    """bs_stack_run does not modify the handle: two streams may run one planned stack at the same
    time on different buffers -- each with a workspace of its own, since the stack here is
    several sequences.  Many launches are queued on both streams before anything is waited for,
    so the kernels of the two streams do overlap; every result must be the oracle's."""
    c = 8
    layers = sum(([wl.maxpool(3, 1, 1, i == 1), wl.bn_params(c, 500 + i), wl.relu()] for i in range(4)), [])
    shape = (16, c, 56, 56)
    xs = [wl.activation(shape, 60 + i) for i in range(2)]
    refs = [bf.run_stack(layers, x, [], "f32") for x in xs]
    st = bs.Stack(layers, shape, "f32").plan(max_steps_per_sequence=1)
    assert st.info()["n_sequences"] == 4 and st.info()["workspace_bytes"] > 0
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    xd = [_dev(x, "f32") for x in xs]
    rounds = 6
    outs = [[st.alloc_outputs("cuda") for _ in range(rounds)] for _ in streams]
    torch.cuda.synchronize()
    for r in range(rounds):
        for i, s in enumerate(streams):
            o, idx = outs[i][r]
            st.run(xd[i], [], out=o, indices=idx, stream=s.cuda_stream)
    torch.cuda.synchronize()
    assert len(st._workspace) == 2, "one workspace per stream"
    for i in range(2):
        ref, ref_idx, _ = refs[i]
        for r in range(rounds):
            o, idx = outs[i][r]
            assert np.array_equal(o.cpu().numpy().view(np.uint32), ref.view(np.uint32)), (i, r)
            assert np.array_equal(idx[0].cpu().numpy(), ref_idx[0]), (i, r)
    st.close()


def test_streaming_probe_moves_what_it_says():
    """bs_probe_stream (the no-arithmetic kernel the roofline notes are priced against): the copy
    pattern copies, R reads per write give the exclusive-or of the R streams, a read-only launch
    writes nothing."""
    n = 3 * 1024 * 256 + 40  # vectors: whole work-groups and a ragged tail
    g = torch.Generator(device="cuda").manual_seed(3)
    stream = torch.cuda.current_stream().cuda_stream
    for r in (1, 2, 4):
        src = torch.randint(-2 ** 31, 2 ** 31 - 1, (r, n, 4), dtype=torch.int32, device="cuda", generator=g)
        dst = torch.full((n, 4), 77, dtype=torch.int32, device="cuda")
        bs.bs_probe_stream(r, False, src.data_ptr(), src.numel() * 4, dst.data_ptr(), dst.numel() * 4, stream)
        torch.cuda.synchronize()
        want = src[0].clone()
        for j in range(1, r):
            want ^= src[j]
        assert torch.equal(dst, want)
        dst.fill_(77)
        bs.bs_probe_stream(r, True, src.data_ptr(), src.numel() * 4, dst.data_ptr(), dst.numel() * 4, stream)
        torch.cuda.synchronize()
        assert bool((dst == 77).all())

