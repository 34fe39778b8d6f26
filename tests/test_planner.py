"""Planner tests (host-only plans, no GPU): the collapse process of Section 4.1 --
operations, steps, sequences -- and the tile geometry the LDS kernels rely on."""
import numpy as np
import pytest

from oracle import breadth_first as bf
from paper_1804_08378_amd import brainslug as bs
from paper_1804_08378_amd import workloads as wl


def plan(layers, shape, dtype="f32", **opts):
    st = bs.Stack(layers, shape, dtype).plan(host_only=1, **opts)
    info = st.info()
    st.close()
    return info


def steps_of(info):
    return [(s["first_operation"], s["n_operations"]) for s in info["steps"]]


def test_listing2_example_partition():
    """Listing 2: <MaxPooling, BatchNorm, ReLU> | <AvgPooling, AvgNormalization>."""
    layers = [wl.maxpool(3, 1, 1), wl.bn_params(4, 0), wl.relu(), wl.avgpool(2, 2)]
    info = plan(layers, (1, 4, 16, 16))
    assert info["operations"] == ["MaxPooling", "BatchNorm", "ReLU", "AvgPooling", "AvgNormalization"]
    assert steps_of(info) == [(0, 3), (3, 2)]
    assert [s["pool_operation"] for s in info["steps"]] == [0, 3]
    # both steps fit one sequence (Listing 2's sequence_0), whose kernel is built for this
    # signature when the stack is planned ...
    assert info["n_sequences"] == 1 and info["workspace_bytes"] == 0
    assert info["sequences"][0]["run_time_build"] == 1 and info["sequences"][0]["variant_name"] == "pool_rows"
    one = plan(layers, (1, 4, 16, 16), force_variant=bs.BS_VARIANT_LDS_TILE)
    assert one["n_sequences"] == 1 and one["workspace_bytes"] == 0
    assert steps_of(one) == [(0, 3), (3, 2)]
    # ... and without run-time builds the plan keeps the steps apart, because each step alone
    # has a pre-compiled fast kernel and the pair would run the slow run-time-shape kernel
    two = plan(layers, (1, 4, 16, 16), jit=-1)
    assert two["n_sequences"] == 2 and two["workspace_bytes"] > 0
    assert [q["run_time_build"] for q in two["sequences"]] == [0, 0]


def test_run_time_builds_compile_without_a_device():
    """Signatures with no pre-compiled kernel are marked for a run-time build by a host-only
    plan, and those builds compile for gfx950 on a machine without a GPU."""
    cases = [
        ([wl.bn_params(4, 0), wl.relu(), wl.maxpool((3, 2), (1, 2), (1, 0), True)], (2, 4, 32, 32), ["pool_rows"], 2),
        # 5x5 windows: lanes that exchange their edge columns serve them in registers ...
        ([wl.maxpool(5, 1, 2, True), wl.bn_params(4, 0), wl.relu()], (2, 4, 32, 32), ["pool_rows"], 2),
        ([wl.maxpool(3, 2, 1), wl.bn_params(4, 1), wl.relu(), wl.avgpool(2, 2), wl.maxpool(3, 1, 1)],
         (2, 4, 64, 64), ["lds_tile"], 1),
        ([wl.bn_params(4, 2), wl.add(), wl.relu(), wl.maxpool(3, 2, 1)], (1, 4, 30, 30), ["lds_tile"], 1),
        # chains of identical blocks with a list or a window that has no compiled instance
        (sum(([wl.maxpool(3, 1, 1), wl.bn_params(4, 3 + i), wl.leaky_relu(0.1)] for i in range(4)), []), (2, 4, 32, 32), ["rows_chain"], 1),
        (sum(([wl.maxpool(5, 1, 2), wl.clamp(-1.0, 1.0)] for i in range(3)), []), (2, 4, 32, 32), ["rows_chain"], 1),
    ]
    # ... without the exchange a lane of the rows kernel would compute 8 columns for 4 owned (float32)
    # or 12 for 8 (16-bit types); LDS shares them between lanes and wins in the first case
    cases.append(([wl.maxpool(5, 1, 2, True), wl.bn_params(4, 0), wl.relu()], (2, 4, 32, 32),
                  {"f32": ["lds_tile"], "bf16": ["pool_rows"], "f16": ["pool_rows"]}, 2, {"lane_exchange": -1}))
    for dt in ("f32", "bf16", "f16"):
        for layers, shape, variants, n_kernels, *more in cases:
            st = bs.Stack(layers, shape, dt).plan(host_only=1, num_cus=256, **(more[0] if more else {}))
            info = st.info()
            want = variants[dt] if isinstance(variants, dict) else variants
            assert [q["variant_name"] for q in info["sequences"]] == want
            assert all(q["run_time_build"] == 1 for q in info["sequences"])
            assert bs.bs_stack_jit_check(st.handle) == n_kernels  # with and without index outputs
            st.close()
    # the benchmark stacks need none in float32 / bfloat16; in binary16, which has no signature
    # tables compiled in, the ResNet stem's sliding-window kernel is a run-time build
    layers, shape, _ = wl.build("vgg_a")
    st = bs.Stack(layers, shape, "f32").plan(host_only=1, num_cus=256)
    assert bs.bs_stack_jit_check(st.handle) == 0
    st.close()
    layers, shape, _ = wl.build("resnet_stem")
    for dt, n in (("bf16", 0), ("f16", 1)):
        st = bs.Stack(layers, shape, dt).plan(host_only=1, num_cus=256)
        assert st.info()["sequences"][0]["variant_name"] == "pool_rows"
        assert bs.bs_stack_jit_check(st.handle) == n
        st.close()


def test_step_rule_elementwise_always_joins_second_pool_opens_a_step():
    layers = [wl.bn_params(4, 0), wl.relu(), wl.maxpool(2, 2), wl.relu(), wl.add(), wl.avgpool(2, 2),
              wl.maxpool(2, 1), wl.relu()]
    info = plan(layers, (1, 4, 32, 32))
    # BN ReLU Max ReLU Add | AvgSum AvgNorm | Max ReLU
    assert steps_of(info) == [(0, 5), (5, 2), (7, 2)]
    # a stack without pooling is one step, one streaming sequence
    info = plan([wl.bn_params(4, 0), wl.add(), wl.relu()], (1, 4, 8, 8))
    assert steps_of(info) == [(0, 3)]
    assert info["sequences"][0]["variant_name"] == "stream"


@pytest.mark.parametrize("name,steps,variant", [
    ("tiny", 1, "pool_direct"), ("vgg_a", 1, "pool_direct"), ("vgg_b", 1, "pool_direct"),
    ("vgg_c", 1, "pool_direct"), ("resnet_stem", 1, "pool_rows"), ("resnet_tail", 1, "stream"),
    ("densenet_dense", 1, "stream"), ("densenet_trans", 1, "pool_direct"), ("halo_stress", 2, "pool_rows"),
])
def test_baseline_configs_are_one_fused_sequence(name, steps, variant):
    layers, shape, dtypes = wl.build(name)
    for dt in dtypes:
        info = plan(layers, shape, dt, num_cus=256)
        assert info["n_steps"] == steps and info["n_sequences"] == 1
        q = info["sequences"][0]
        assert q["variant_name"] == variant
        assert tuple(q["in_shape"]) == shape and tuple(q["out_shape"]) == wl.output_shape(layers, shape)
        assert info["algorithmic_bytes"] == wl.algorithmic_bytes(layers, shape, dt)
        assert q["lds_bytes"] <= 64 * 1024
        assert q["grid"] >= 1
        if name == "halo_stress":
            # rc output rows per lane (2 for float32, 4 for the 16-bit types): 2 rc + 3 input rows of every
            # 2 rc are loaded; only rows shared with the chunk above are read twice, never columns
            assert 1.0 <= q["redundancy"] < (1.75 if dt == "f32" else 1.45)
            lds = plan(layers, shape, dt, num_cus=256, force_variant=bs.BS_VARIANT_LDS_TILE)["sequences"]
            assert len(lds) == 1 and lds[0]["variant_name"] == "lds_tile" and 1.0 <= lds[0]["redundancy"] < 1.1
    if name == "halo_stress":
        assert info["operations"] == ["BatchNorm", "ReLU", "AvgPooling", "AvgNormalization", "MaxPooling",
                                      "BatchNorm", "ReLU"]
        assert steps_of(info) == [(0, 4), (4, 3)]


def _blocks(n, c=4):
    return sum(([wl.maxpool(3, 1, 1), wl.bn_params(c, i), wl.relu()] for i in range(n)), [])


def test_steps_per_sequence_strategies():
    """Section 5.1: 1 step per sequence, at most 5, unrestricted."""
    layers = _blocks(12)
    shape = (2, 4, 56, 56)
    one = plan(layers, shape, max_steps_per_sequence=1)
    five = plan(layers, shape, max_steps_per_sequence=5, max_lds_bytes=65536)
    free = plan(layers, shape, max_lds_bytes=65536)
    assert one["n_steps"] == five["n_steps"] == free["n_steps"] == 12
    assert one["n_sequences"] == 12
    assert all(q["n_steps"] <= 5 for q in five["sequences"]) and five["n_sequences"] >= 3
    assert free["n_sequences"] <= five["n_sequences"]
    assert one["workspace_bytes"] == 2 * 256 * ((2 * 4 * 56 * 56 * 4 + 255) // 256)
    for info in (one, five, free):
        assert sum(q["n_steps"] for q in info["sequences"]) == 12
        assert [q["first_step"] for q in info["sequences"]] == list(
            np.cumsum([0] + [q["n_steps"] for q in info["sequences"]][:-1]))


def test_breadth_first_plan_is_one_sequence_per_layer():
    layers, shape, _ = wl.build("halo_stress")
    info = plan(layers, shape, breadth_first=1)
    assert info["n_sequences"] == len(layers)
    assert [q["n_layers"] for q in info["sequences"]] == [1] * len(layers)
    assert info["workspace_bytes"] > 0


def test_halo_grows_with_every_block_and_forces_a_new_sequence():
    """Section 5.1: every padded block adds overlap; at a fixed on-chip budget an additional
    sequence becomes necessary at some depth."""
    shape = (1, 4, 64, 64)
    lds, halos, seqs = [], [], []
    for n in range(1, 9):
        info = plan(_blocks(n), shape, max_lds_bytes=65536, tile_rows=8, tile_cols=16,
                    force_variant=bs.BS_VARIANT_LDS_TILE)
        q = info["sequences"][0]
        if info["n_sequences"] == 1:
            lds.append(q["lds_bytes"])
            halos.append((q["halo_rows"], q["halo_cols"]))
        seqs.append(plan(_blocks(n), shape, max_lds_bytes=8192, force_variant=bs.BS_VARIANT_LDS_TILE)["n_sequences"])
    assert all(b > a for a, b in zip(lds, lds[1:]))
    assert [h[0] for h in halos] == [2 * (i + 1) for i in range(len(halos))]  # k=3, s=1: +2 rows per block
    assert seqs[0] == 1 and seqs[-1] > 1 and all(b >= a for a, b in zip(seqs, seqs[1:]))


def test_chains_of_identical_blocks_take_the_register_kernel():
    """Two to eight blocks <MaxPool 3/1/1, BatchNorm, ReLU> on rows that fit a wave: one sequence without LDS
    whatever the on-chip budget, as many levels as the kernel is compiled for, chunks of half the plane; longer
    stacks are cut into sequences of even length."""
    shape = (2, 4, 56, 56)
    for n in (3, 5, 8):
        info = plan(_blocks(n), shape, max_lds_bytes=8192)
        q = info["sequences"][0]
        assert info["n_sequences"] == 1 and q["variant"] == bs.BS_VARIANT_ROWS_CHAIN and q["lds_bytes"] == 0
        assert q["n_steps"] == n and q["tile_rows"] == 28 and q["halo_rows"] == 2 * n
    assert [q["n_steps"] for q in plan(_blocks(12), shape)["sequences"]] == [6, 6]
    assert [q["n_steps"] for q in plan(_blocks(20), shape)["sequences"]] == [7, 7, 6]
    # one block: the one-level kernel; two: the chain; rows too wide for a wave or no lane exchange: the LDS tiles
    assert plan(_blocks(1), shape)["sequences"][0]["variant"] == bs.BS_VARIANT_POOL_ROWS
    assert plan(_blocks(2), shape)["sequences"][0]["variant"] == bs.BS_VARIANT_ROWS_CHAIN
    f16 = plan(_blocks(4), shape, "f16")["sequences"][0]   # binary16: no compiled tables, a run-time build of the same kernel
    assert f16["variant"] == bs.BS_VARIANT_ROWS_CHAIN and f16["run_time_build"] == 1
    assert plan(_blocks(4), shape, "f16", jit=-1)["sequences"][0]["variant"] == bs.BS_VARIANT_LDS_TILE
    assert plan(_blocks(4), (1, 4, 8, 512))["sequences"][0]["variant"] == bs.BS_VARIANT_LDS_TILE
    assert plan(_blocks(4), shape, lane_exchange=-1)["sequences"][0]["variant"] == bs.BS_VARIANT_LDS_TILE


def test_lds_budget_is_respected_and_no_fit_is_reported():
    layers, shape, _ = wl.build("halo_stress")
    for budget in (4096, 8192, 16384, 32768, 65536):
        info = plan(layers, shape, max_lds_bytes=budget)
        assert all(q["lds_bytes"] <= budget for q in info["sequences"])
    with pytest.raises(bs.BrainSlugError) as e:
        plan([wl.maxpool(31, 1, 15)], (1, 1, 64, 64), max_lds_bytes=1024)
    assert e.value.status == 6


def test_resource_example_ratio_is_k_squared():
    """Section 4.1's example: a non-overlapping 3x3 pooling needs 3*3 times the output's data
    as input."""
    info = plan([wl.maxpool(3, 3)], (1, 4, 96, 96), force_variant=bs.BS_VARIANT_LDS_TILE,
                tile_rows=8, tile_cols=16, max_lds_bytes=65536)
    q = info["sequences"][0]
    assert (q["halo_rows"], q["halo_cols"]) == (0, 0)
    ratio = (q["lds_bytes"] / 4) / (8 * 16)
    assert 9.0 <= ratio < 9.0 * 1.12  # row pitch slack only


def test_tile_region_covers_the_true_dependency_cone():
    """Brute force: perturb one input row / column at a time in the oracle and record which
    output rows / columns move; the rectangle the planner reserves for an interior tile must be
    exactly as tall as the set of input rows that tile depends on, and as wide up to strip
    rounding."""
    c = 2
    layers = [wl.bn_params(c, 0), wl.relu(), wl.avgpool(3, 1, 1), wl.maxpool(3, 2, 1), wl.relu()]
    shape = (1, c, 40, 36)
    x = np.abs(wl.activation(shape, 5)) + 1.0  # positive: BN/ReLU/avg/max all pass a bump through
    for l in layers:
        if l["kind"] == "bn":
            l["gamma"] = np.abs(l["gamma"]) + 0.5
            l["mean"][:] = 0
            l["beta"][:] = 0
    ref, _, _ = bf.run_stack(layers, x)
    th, tw = 4, 8
    info = plan(layers, shape, force_variant=bs.BS_VARIANT_LDS_TILE, tile_rows=th, tile_cols=tw,
                max_lds_bytes=65536)
    q = info["sequences"][0]
    for axis, tile, halo, size in ((2, th, q["halo_rows"], 40), (3, tw, q["halo_cols"], 36)):
        dep = []
        for i in range(size):
            xp = x.copy()
            sl = [slice(None)] * 4
            sl[axis] = i
            xp[tuple(sl)] += 100.0
            out, _, _ = bf.run_stack(layers, xp)
            moved = np.nonzero((out != ref).any(axis=tuple(a for a in range(4) if a != axis)))[0]
            dep.append(set(moved.tolist()))
        t = 1  # an interior tile
        outs = set(range(t * tile, (t + 1) * tile))
        needed = [i for i in range(size) if dep[i] & outs]
        assert needed == list(range(needed[0], needed[-1] + 1))
        reserved = tile * 2 + halo
        if axis == 2:
            assert reserved == len(needed), (len(needed), reserved)
        else:  # column extents are rounded up to the four-output strips of the pooling phases
            assert len(needed) <= reserved <= len(needed) + 3, (len(needed), reserved)


def test_index_output_in_mid_sequence_needs_full_coverage():
    """A max pool whose indices are wanted may stay inside a sequence only if the windows of
    the later pooling operations cover its whole output; otherwise the sequence ends there."""
    covered = [wl.maxpool(3, 1, 1, True), wl.relu(), wl.maxpool(3, 2, 1)]
    gaps = [wl.maxpool(3, 1, 1, True), wl.relu(), wl.maxpool(2, 3, 0)]
    assert plan(covered, (1, 2, 32, 32))["n_sequences"] == 1
    assert plan(gaps, (1, 2, 32, 32))["n_sequences"] == 2


def test_capacity_splits_keep_every_operation():
    layers = [wl.relu()] * 40 + [wl.maxpool(2, 2)] + [wl.add()] * 9
    info = plan(layers, (1, 2, 16, 16))
    assert info["n_operations"] == 50
    assert sum(s["n_operations"] for s in info["steps"]) == 50
    assert sum(q["n_layers"] for q in info["sequences"]) == 50


def test_channels_last_plans_take_one_or_two_steps_per_sequence():
    """Host-only channels-last plans: a sequence per step (or per pair of steps the tile kernel
    exists for), the channels-last kernel families, workspace between the sequences; options
    that belong to the NCHW kernels are refused."""
    for name in ("vgg_a", "resnet_stem", "resnet_tail", "densenet_trans", "halo_stress"):
        layers, shape, dtypes = wl.build(name)
        for dtype in dtypes:
            pools = sum(1 for l in layers if l["kind"] in ("maxpool", "avgpool"))
            st = bs.Stack(layers, shape, dtype).plan(host_only=1, layout=bs.BS_LAYOUT_NHWC, max_steps_per_sequence=1)
            info = st.info()
            assert info["n_sequences"] == info["n_steps"]
            names = [q["variant_name"] for q in info["sequences"]]
            assert names == (["nhwc_pool"] * pools if pools else ["nhwc_stream"])
            assert (info["workspace_bytes"] > 0) == (pools > 1)
            for q in info["sequences"]:
                assert q["run_time_build"] == 0 and q["lds_bytes"] == 0 and q["grid"] >= 1
            st.close()
            st = bs.Stack(layers, shape, dtype).plan(host_only=1, layout=bs.BS_LAYOUT_NHWC)
            info = st.info()
            names = [q["variant_name"] for q in info["sequences"]]
            # halo_stress (3 x 3 / 1 average, 3 x 3 / 2 maximum, 56 pixels per row) takes the register kernel with 16-bit storage
            two = "nhwc_tile" if dtype == "f32" else "nhwc_rows"
            assert names == ([two] if pools == 2 else ["nhwc_pool"] * pools if pools else ["nhwc_stream"])
            assert info["workspace_bytes"] == 0
            for q in info["sequences"]:
                if q["variant_name"] == "nhwc_rows":
                    assert q["lds_bytes"] == 0 and q["threads_per_group"] == 64 * 4 and q["tile_rows"] == 7
                    assert q["grid"] == shape[0] * (28 // 7) * (shape[1] // 8 // 4)
            if pools == 2:  # without lane exchange: the tile kernel
                st.close()
                st = bs.Stack(layers, shape, dtype).plan(host_only=1, layout=bs.BS_LAYOUT_NHWC, lane_exchange=-1)
                info = st.info()
                names = [q["variant_name"] for q in info["sequences"]]
                assert names == ["nhwc_tile"]
            for q in info["sequences"]:
                if q["variant_name"] != "nhwc_tile":
                    continue
                # both rectangles of the tile (each followed by spare rows for blocks that hang over its edge), one
                # 16-byte vector per cell and channel vector, and the two BatchNorm operations' scale and shift
                # vectors; a lane holds at most four input cells and one block per pooling level
                vec = 4 if dtype == "f32" else 8
                th, tw, cv = q["tile_rows"], q["tile_cols"], q["planes_per_group"] // vec
                r1 = ((th - 1) * 2 + 3, (tw - 1) * 2 + 3)   # max pool 3 x 3 stride 2 on top
                r0 = (r1[0] + 2, r1[1] + 2)                 # average pool 3 x 3 stride 1 under it (2 x 2 blocks)
                cells = (r0[0] + 2) * r0[1] + (r1[0] + 1) * r1[1]
                assert q["lds_bytes"] == cells * cv * 16 + 2 * 2 * cv * vec * 4 <= 64 * 1024
                lanes = 256 // cv
                assert r0[0] * r0[1] <= 4 * lanes and -(-r1[0] // 2) * -(-r1[1] // 2) <= lanes and th * tw <= lanes
                assert q["n_steps"] == 2 and q["n_levels"] == 2 and q["threads_per_group"] == 256
                # work-groups walk runs of tiles: no more groups than 256 compute units hold at once by LDS
                tiles = shape[0] * -(-28 // th) * -(-28 // tw) * (shape[1] // vec // cv)
                assert q["grid"] == min(tiles, 256 * min(8, 160 * 1024 // q["lds_bytes"]))
                assert 1.0 < q["redundancy"] < 2.0
            st.close()
    # pairs are taken from the front; windows outside the tile kernel's table, first pools with
    # an index output and channel counts that give no 128-bit vectors stay one step per sequence
    three = [wl.maxpool(3, 2, 1), wl.relu(), wl.avgpool(2, 2, 0), wl.maxpool(3, 1, 1, True)]
    for layers, shape, want in ((three, (1, 8, 32, 32), ["nhwc_tile", "nhwc_pool"]),
                                ([wl.maxpool(5, 1, 2), wl.avgpool(3, 1, 1)], (1, 8, 16, 16), ["nhwc_pool"] * 2),
                                ([wl.maxpool(3, 1, 1, True), wl.avgpool(3, 1, 1)], (1, 8, 16, 16), ["nhwc_pool"] * 2),
                                ([wl.maxpool(3, 1, 1), wl.avgpool(3, 1, 1)], (1, 6, 16, 16), ["nhwc_pool"] * 2),
                                ([wl.maxpool(3, 1, 1), wl.maxpool(3, 1, 1, True)], (1, 8, 16, 16), ["nhwc_tile"])):
        st = bs.Stack(layers, shape, "f32").plan(host_only=1, layout=bs.BS_LAYOUT_NHWC)
        assert [q["variant_name"] for q in st.info()["sequences"]] == want
        st.close()
    h = bs.bs_stack_create([wl.relu()], (1, 4, 8, 8), "f32")
    try:
        for bad in (dict(layout=2), dict(layout=-1), dict(layout=1, force_variant=bs.BS_VARIANT_STREAM)):
            with pytest.raises(bs.BrainSlugError) as e:
                bs.bs_stack_plan(h, host_only=1, **bad)
            assert e.value.status == 3
        bs.bs_stack_plan(h, host_only=1, layout=1)
        # a channel slice of a channels-last tensor: the batch stride is H * W times the larger
        # tensor's channel count, and that count times the element size a multiple of 16 bytes
        assert bs.bs_stack_check_buffers(h, 4096, 0, None, 1 << 20, 0, None, 0, 0) == 0
        assert bs.bs_stack_check_buffers(h, 4096, 8 * 8 * 8, None, 1 << 20, 0, None, 0, 0) == 0       # 8 channels
        assert bs.bs_stack_check_buffers(h, 4096, 0, None, 1 << 20, 8 * 8 * 12, None, 0, 0) == 0      # 12 channels
        assert bs.bs_stack_check_buffers(h, 4096, 8 * 8 * 8 + 4, None, 1 << 20, 0, None, 0, 0) == 2   # no whole pixels
        assert bs.bs_stack_check_buffers(h, 4096, 8 * 8 * 5, None, 1 << 20, 0, None, 0, 0) == 7       # 20-byte pixels
        assert bs.bs_stack_check_buffers(h, 4096, 8 * 8 * 3, None, 1 << 20, 0, None, 0, 0) == 2       # below the image
        # slices of one channels-last buffer interleave pixel by pixel: refused (not provably disjoint)
        assert bs.bs_stack_check_buffers(h, 4096, 8 * 8 * 8, None, 4096 + 16, 8 * 8 * 8, None, 0, 0) == 12
    finally:
        bs.bs_stack_destroy(h)


def test_threads_per_group_is_honoured_by_the_register_kernels():
    """The sliding-row kernels have no barrier, so a work-group may be any number of whole waves:
    the plan option changes the work-group size and the grid, not the work per wave."""
    for name, dtype in (("halo_stress", "f32"), ("halo_stress", "bf16"), ("resnet_stem", "f16")):
        layers, shape = wl.build(name)[:2]
        base = plan(layers, shape, dtype)["sequences"][0]
        assert base["variant_name"] == "pool_rows" and base["threads_per_group"] == 256
        for threads in (64, 128, 192):
            q = plan(layers, shape, dtype, threads_per_group=threads)["sequences"][0]
            assert q["variant_name"] == "pool_rows" and q["threads_per_group"] == threads
            assert q["tile_rows"] == base["tile_rows"]
            waves = base["grid"] * 4
            assert -(-waves // (threads // 64)) - 1 <= q["grid"] <= -(-waves // (threads // 64))
        q = plan(layers, shape, dtype, threads_per_group=512)["sequences"][0]
        assert q["threads_per_group"] == 256 and q["grid"] == base["grid"]
