"""Host-only checks of the C-ABI library (no GPU, no compute calls): it loads, exports
every symbol include/brainslug.h declares, validates its arguments, folds BatchNorm
as the header says, and reports shapes."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_1804_08378_amd import brainslug as bs
from paper_1804_08378_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "brainslug.h")).read()
    declared = set(re.findall(r"BS_API\s+[\w\s\*]+?\b(bs_\w+)\s*\(", hdr))
    assert declared, "no BS_API declarations found"
    lib = C.CDLL(bs.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} declared in brainslug.h but not exported"
    assert declared == set(bs.EXPORTS), declared ^ set(bs.EXPORTS)
    assert bs.bs_version().startswith("brainslug-hip")
    assert bs.bs_status_string(0) == "ok" and bs.bs_status_string(6)


def _status(fn, *a, **k):
    with pytest.raises(bs.BrainSlugError) as e:
        fn(*a, **k)
    return e.value.status


def test_create_rejects_bad_arguments():
    ok_bn = wl.bn_params(4, 0)
    assert _status(bs.bs_stack_create, [wl.relu()], (0, 4, 8, 8), "f32") == 2      # shape
    assert _status(bs.bs_stack_create, [wl.relu()], (1, 4, 8, -1), "f32") == 2
    assert _status(bs.bs_stack_create, [], (1, 4, 8, 8), "f32") == 4                # no layers
    assert _status(bs.bs_stack_create, [wl.relu()] * 257, (1, 4, 8, 8), "f32") == 4
    assert _status(bs.bs_stack_create, [wl.relu()], (1, 4, 8, 8), 7) == 4            # dtype
    assert _status(bs.bs_stack_create, [wl.maxpool(3, 1, 0)], (1, 4, 2, 2), "f32") == 2  # empty output
    assert _status(bs.bs_stack_create, [wl.maxpool(2, 2, 2)], (1, 4, 8, 8), "f32") == 3  # p > k/2
    assert _status(bs.bs_stack_create, [wl.maxpool(0, 1, 0)], (1, 4, 8, 8), "f32") == 3
    assert _status(bs.bs_stack_create, [wl.avgpool(2, 0, 0)], (1, 4, 8, 8), "f32") == 3
    assert _status(bs.bs_stack_create, [wl.clamp(1.0, 0.0)], (1, 4, 8, 8), "f32") == 3       # lo > hi
    assert _status(bs.bs_stack_create, [wl.leaky_relu(float("nan"))], (1, 4, 8, 8), "f32") == 3
    h = bs.bs_stack_create([wl.maxpool(2, 2, ceil_mode=True)], (1, 4, 9, 9), "f32")  # ceil mode: 5 x 5 outputs
    assert bs.bs_stack_output_shape(h) == (1, 4, 5, 5)
    bs.bs_stack_destroy(h)
    dil = dict(wl.maxpool(2, 2), dilation=(2, 2))
    assert _status(bs.bs_stack_create, [dil], (1, 4, 8, 8), "f32") == 4
    bad = dict(ok_bn, var=np.array([1, 1, -1, 1], np.float32))
    assert _status(bs.bs_stack_create, [bad], (1, 4, 8, 8), "f32") == 3             # var + eps <= 0
    nan = dict(ok_bn, gamma=np.array([1, np.nan, 1, 1], np.float32))
    assert _status(bs.bs_stack_create, [nan], (1, 4, 8, 8), "f32") == 3
    assert _status(bs.bs_stack_create, [wl.add()] * 17, (1, 4, 8, 8), "f32") == 4
    too_big = (4, 1024, 1024, 1024)
    assert _status(bs.bs_stack_create, [wl.relu()], too_big, "f32") == 4
    # NULL handling straight at the ABI
    lib = bs.load()
    h = C.c_void_p()
    shape = (C.c_int64 * 4)(1, 4, 8, 8)
    assert lib.bs_stack_create(None, 1, shape, 0, C.byref(h)) == 1
    d = (bs.bs_layer_desc * 1)()
    d[0].kind = bs.BS_BATCHNORM  # parameter pointers left NULL
    assert lib.bs_stack_create(d, 1, shape, 0, C.byref(h)) == 1
    lib.bs_stack_destroy(None)  # allowed
    assert lib.bs_stack_num_residuals(None) == -1 and lib.bs_stack_num_index_outputs(None) == -1
    assert lib.bs_stack_output_shape(None, shape) == 1


def test_shapes_residuals_indices():
    layers = [wl.bn_params(6, 1), wl.add(), wl.maxpool(3, 2, 1, True), wl.relu(), wl.add(),
              wl.avgpool((2, 3), (2, 1), (1, 1)), wl.maxpool(2, 1, 0, True)]
    shape = (2, 6, 17, 23)
    h = bs.bs_stack_create(layers, shape, "bf16")
    try:
        assert bs.bs_stack_output_shape(h) == wl.output_shape(layers, shape) == (2, 6, 4, 11)
        assert bs.bs_stack_num_residuals(h) == 2
        assert [bs.bs_stack_residual_shape(h, i) for i in range(2)] == wl.residual_shapes(layers, shape)
        assert bs.bs_stack_num_index_outputs(h) == 2
        assert bs.bs_stack_index_shape(h, 0) == (2, 6, 9, 12)
        assert bs.bs_stack_index_shape(h, 1) == (2, 6, 4, 11)
        assert _status(bs.bs_stack_index_shape, h, 2) == 11
        assert _status(bs.bs_stack_residual_shape, h, -1) == 11
        # not planned yet
        assert _status(bs.bs_stack_plan_info, h) == 5
        assert bs.bs_stack_workspace_bytes(h) == 0
        assert _status(bs.bs_stack_run, h, 16, [16, 32], 64, None, 0, 0, 0) == 5
    finally:
        bs.bs_stack_destroy(h)


def test_folded_batchnorm_matches_float64_definition():
    p = wl.bn_params(32, 3)
    h = bs.bs_stack_create([wl.relu(), p], (1, 32, 4, 4), "f32")
    try:
        scale, shift = bs.bs_stack_folded_bn(h, 1, 32)
        s64 = p["gamma"].astype(np.float64) / np.sqrt(p["var"].astype(np.float64) + p["eps"])
        assert np.array_equal(scale, s64.astype(np.float32))
        assert np.array_equal(shift, (p["beta"].astype(np.float64) - p["mean"].astype(np.float64) * s64)
                              .astype(np.float32))
        assert _status(bs.bs_stack_folded_bn, h, 0, 32) == 11  # layer 0 is not a BatchNorm
    finally:
        bs.bs_stack_destroy(h)


def test_parameters_are_copied_at_create():
    p = wl.bn_params(8, 4)
    h = bs.bs_stack_create([p], (1, 8, 4, 4), "f32")
    before = bs.bs_stack_folded_bn(h, 0, 8)
    for k in ("gamma", "beta", "mean", "var"):
        p[k][:] = 123.0
    after = bs.bs_stack_folded_bn(h, 0, 8)
    bs.bs_stack_destroy(h)
    assert np.array_equal(before[0], after[0]) and np.array_equal(before[1], after[1])


def test_plan_option_validation():
    h = bs.bs_stack_create([wl.relu()], (1, 4, 8, 8), "f32")
    try:
        assert _status(bs.bs_stack_plan, h, host_only=1, threads_per_group=100) == 3
        assert _status(bs.bs_stack_plan, h, host_only=1, threads_per_group=1024) == 3
        assert _status(bs.bs_stack_plan, h, host_only=1, force_variant=9) == 3
        assert _status(bs.bs_stack_plan, h, host_only=1, max_lds_bytes=1 << 20) == 3
        assert _status(bs.bs_stack_plan, h, host_only=1, max_steps_per_sequence=-1) == 3
        bs.bs_stack_plan(h, host_only=1, threads_per_group=128)
        info = bs.bs_stack_plan_info(h)
        assert info["device_planned"] == 0 and info["n_sequences"] == 1
        assert _status(bs.bs_stack_run, h, 16, None, 32, None, 0, 0, 0) == 5  # host-only plan cannot run
        assert _status(bs.bs_stack_step_info, h, 5) == 11
        assert _status(bs.bs_stack_sequence_info, h, 1) == 11
        assert bs.bs_stack_operation_name(h, 0) == "ReLU" and bs.bs_stack_operation_name(h, 1) is None
    finally:
        bs.bs_stack_destroy(h)


def test_backward_entry_points_without_a_device_plan():
    """The backward pass needs the device plan (its parameter table and kernels): without one the
    entry points say so and report no plan."""
    h = bs.bs_stack_create([wl.bn_params(4, 0), wl.relu(), wl.maxpool(2, 2)], (1, 4, 8, 8), "f32")
    try:
        assert bs.bs_stack_backward_num_stages(h) == -1 and bs.bs_stack_backward_workspace_bytes(h) == 0
        assert _status(bs.bs_stack_plan_backward, h) == 5           # not planned at all
        bs.bs_stack_plan(h, host_only=1)
        assert _status(bs.bs_stack_backward, h, 16, None, None, 32, 48, None, 0, 0, 0) == 5
        bs.bs_stack_plan_backward(h)                                # host-only: stages and sizes, nothing that runs
        assert bs.bs_stack_backward_num_stages(h) == 1
        assert _status(bs.bs_stack_backward, h, 16, None, None, 32, 48, None, 0, 0, 0) == 5
        bs.bs_stack_plan(h, host_only=1)                            # a new plan drops the backward plan
        assert bs.bs_stack_backward_num_stages(h) == -1
        assert _status(bs.bs_stack_plan_backward, None) == 1
    finally:
        bs.bs_stack_destroy(h)


def _backward_plan(layers, shape, dtype="f32", **opts):
    h = bs.bs_stack_create(layers, shape, dtype)
    try:
        bs.bs_stack_plan(h, host_only=1, **opts)
        bs.bs_stack_plan_backward(h)
        return bs.bs_stack_backward_num_stages(h), bs.bs_stack_backward_workspace_bytes(h)
    finally:
        bs.bs_stack_destroy(h)


def test_backward_stages_and_workspace():
    """A stage is a run of element-wise operations with at most one pooling operation at its end.  The
    workspace holds, 256-byte aligned: input and input gradient of every stage after the first, the picks
    of every max pooling that does not find them itself, the unused output of a last stage that is run
    forward for its picks, and the forward stage plans' own workspace."""
    c, shape = 8, (2, 8, 16, 16)
    al = lambda n: (n + 255) // 256 * 256
    bn = lambda i: wl.bn_params(c, i)
    # one stage, nothing to recompute
    assert _backward_plan([bn(0), wl.add(), wl.relu()], shape) == (1, 0)
    assert _backward_plan([bn(0), wl.relu(), wl.avgpool(3, 2, 1)], shape) == (1, 0)
    # 2 x 2 windows that tile the plane find their picks themselves, in both layouts
    assert _backward_plan([bn(0), wl.relu(), wl.maxpool(2, 2)], shape) == (1, 0)
    assert _backward_plan([bn(0), wl.relu(), wl.maxpool(2, 2)], shape, layout=bs.BS_LAYOUT_NHWC) == (1, 0)
    # ... unless the rows are no whole vectors (float32: 4 per vector) or the plane is odd
    n_out = 2 * 8 * 7 * 7
    assert _backward_plan([bn(0), wl.relu(), wl.maxpool(2, 2)], (2, 8, 14, 14)) == (1, al(n_out * 4) + al(n_out * 4))
    # overlapping 3 x 3 windows (padding 1, stride 1 or 2) on rows of whole vectors: the lanes of a row find the picks
    n_out = 2 * 8 * 8 * 8
    assert _backward_plan([bn(0), wl.relu(), wl.maxpool(3, 2, 1)], shape) == (1, 0)
    assert _backward_plan([bn(0), wl.relu(), wl.maxpool(3, 1, 1)], shape, "f16") == (1, 0)
    # other overlapping windows, or that kernel switched off: picks (int32) and the forward run's output
    assert _backward_plan([bn(0), wl.relu(), wl.maxpool(3, 2, 1)], shape, lane_exchange=-1) == (1, al(n_out * 4) + al(n_out * 4))
    assert _backward_plan([bn(0), wl.relu(), wl.maxpool(3, 2, 1)], shape, "f16", lane_exchange=-1) == (1, al(n_out * 4) + al(n_out * 2))
    assert _backward_plan([bn(0), wl.relu(), wl.maxpool(5, 2, 2)], shape) == (1, al(n_out * 4) + al(n_out * 4))
    # pool, then element-wise operations: two stages; the second one's input and input gradient
    stages, ws = _backward_plan([bn(0), wl.relu(), wl.avgpool(2, 2), bn(1), wl.relu()], shape)
    assert (stages, ws) == (2, 2 * al(n_out * 4))
    # the halo stress stack is three stages: BatchNorm, ReLU, average pooling | max pooling | BatchNorm, ReLU.  The last one
    # joins the max pooling's stage, and the kernel that walks both pooling levels takes the first two: one stage, no workspace
    n_in = 2 * 8 * 16 * 16
    halo = [bn(0), wl.relu(), wl.avgpool(3, 1, 1), wl.maxpool(3, 2, 1), bn(1), wl.relu()]
    assert _backward_plan(halo, shape) == (1, 0)
    assert _backward_plan(halo, shape, "bf16") == (1, 0)
    # ... not with an Add in front of the average pooling, or with anything between the two poolings: two stages
    stages, ws = _backward_plan([bn(0), wl.add(), wl.avgpool(3, 1, 1), wl.maxpool(3, 2, 1), bn(1), wl.relu()], shape)
    assert stages == 2 and ws >= 2 * al(n_in * 4)
    stages, ws = _backward_plan([bn(0), wl.relu(), wl.avgpool(3, 1, 1), wl.relu(), wl.maxpool(3, 2, 1), bn(1), wl.relu()], shape)
    assert stages == 2 and ws >= 2 * al(n_in * 4)
    stages, ws = _backward_plan([bn(0), wl.relu(), wl.avgpool(3, 1, 1), wl.maxpool(3, 2, 1), bn(1), wl.relu()], shape, lane_exchange=-1)
    assert stages == 3 and ws >= 2 * al(n_in * 4) + al(n_out * 4) + 2 * al(n_out * 4)
    # capacity: 16 element-wise operations and 4 residual operands per stage
    assert _backward_plan([wl.relu()] * 16, shape)[0] == 1
    assert _backward_plan([wl.relu()] * 17, shape)[0] == 2
    assert _backward_plan([wl.add()] * 4, shape)[0] == 1
    assert _backward_plan([wl.add()] * 5, shape)[0] == 2


def test_index_outputs_may_share_bytes_with_nothing():
    """Index outputs are written by the kernels like the output itself: one that overlaps the
    input, the output, a residual operand, the workspace or another index output is refused
    (host only, fake addresses; the expectation comes from explicit byte ranges)."""
    n, c, h, w = 2, 2, 8, 8
    layers = [wl.maxpool(2, 2, 0, True), wl.add(), wl.maxpool(2, 2, 0, True)]
    hd = bs.bs_stack_create(layers, (n, c, h, w), "f32")
    try:
        bs.bs_stack_plan(hd, host_only=1, max_steps_per_sequence=1)
        wsn = bs.bs_stack_workspace_bytes(hd)
        assert wsn > 0
        sizes = {"in": n * c * h * w * 4, "res": n * c * 16 * 4, "out": n * c * 4 * 4, "ws": wsn,
                 "i0": n * c * 16 * 4, "i1": n * c * 4 * 4}
        base = {"in": 1 << 20, "res": 2 << 20, "out": 3 << 20, "ws": 4 << 20, "i0": 5 << 20, "i1": 6 << 20}

        def status(**moved):
            p = dict(base, **moved)
            return bs.bs_stack_check_buffers(hd, p["in"], 0, [p["res"]], p["out"], 0, [p["i0"], p["i1"]], p["ws"], wsn)

        def overlap(p, a, b):
            return p[a] < p[b] + sizes[b] and p[b] < p[a] + sizes[a]

        assert status() == 0
        rng = np.random.default_rng(11)
        hits = 0
        for which in ("i0", "i1"):
            for other in ("in", "res", "out", "ws", "i1" if which == "i0" else "i0"):
                for _ in range(20):
                    off = 16 * int(rng.integers(-(sizes[which] // 16) - 2, sizes[other] // 16 + 3))
                    moved = {which: base[other] + off}
                    p = dict(base, **moved)
                    truth = any(overlap(p, which, o) for o in p if o != which)
                    assert status(**moved) == (12 if truth else 0), (which, other, off)
                    hits += truth
        assert hits > 40
        # a skipped index output (NULL) takes part in nothing
        assert bs.bs_stack_check_buffers(hd, base["in"], 0, [base["res"]], base["out"], 0, [0, base["in"]], base["ws"], wsn) == 12
        assert bs.bs_stack_check_buffers(hd, base["in"], 0, [base["res"]], base["out"], 0, [0, base["i1"]], base["ws"], wsn) == 0
    finally:
        bs.bs_stack_destroy(hd)


def test_size_limit_is_two_to_the_31_elements():
    """All index arithmetic is 32-bit: a tensor (input, output or intermediate) of 2^31 elements
    or more is refused at create, one just below is accepted and plans (host only)."""
    ok = bs.bs_stack_create([wl.relu(), wl.maxpool(2, 2)], (1, 2047, 1024, 1024), "bf16")
    try:
        bs.bs_stack_plan(ok, host_only=1)
        assert bs.bs_stack_plan_info(ok)["n_sequences"] == 1
        bs.bs_stack_plan(ok, host_only=1, layout=bs.BS_LAYOUT_NHWC)
    finally:
        bs.bs_stack_destroy(ok)
    for shape in ((1, 2048, 1024, 1024), (2, 1024, 1024, 1024), (65536, 1, 256, 128)):
        assert _status(bs.bs_stack_create, [wl.relu()], shape, "f32") in (2, 4)


def test_buffer_checks_against_brute_force_byte_sets():
    """The argument checks of the strided run (host only, fake addresses): an overlap of the
    output with an input is never let through, slices of one buffer that interleave without
    sharing a byte are accepted, and stride / alignment errors have their own codes.  The
    expected answers come from explicit byte sets, not from the library's interval logic."""
    n, c, h, w = 3, 2, 8, 8
    layers = [wl.relu(), wl.maxpool(2, 2), wl.add(), wl.avgpool(2, 2)]
    hd = bs.bs_stack_create(layers, (n, c, h, w), "f32")
    try:
        bs.bs_stack_plan(hd, host_only=1, max_steps_per_sequence=1)  # several sequences: needs a workspace
        wsn = bs.bs_stack_workspace_bytes(hd)
        assert wsn > 0
        in_img, out_img = c * h * w * 4, c * (h // 4) * (w // 4) * 4
        res_bytes = n * c * (h // 2) * (w // 2) * 4

        def bytes_of(p, img, stride_b):
            return {p + i * stride_b + b for i in range(n) for b in range(img)}

        far_res, far_ws = 1 << 30, 1 << 31
        rng = np.random.default_rng(5)
        seen = {0: 0, 12: 0}
        for _ in range(400):
            s_in = int(rng.choice([0, 128, 132, 136, 160, 256]))   # elements
            s_out = int(rng.choice([0, 8, 12, 128, 136, 160, 256]))
            p_in = 4096
            p_out = 4096 + 16 * int(rng.integers(-40, 120))
            st = bs.bs_stack_check_buffers(hd, p_in, s_in, [far_res], p_out, s_out, None, far_ws, wsn)
            truth = bool(bytes_of(p_in, in_img, (s_in or 128) * 4) & bytes_of(p_out, out_img, (s_out or 8) * 4))
            assert st in (0, 12), (st, s_in, s_out, p_out)
            if truth:
                assert st == 12, (s_in, s_out, p_out)
            if st == 0:
                assert not truth
            # equal strides and disjoint images of one buffer: must be accepted
            if not truth and (s_in or 128) == (s_out or 8):
                assert st == 0, (s_in, s_out, p_out)
            seen[st] += 1
        assert seen[0] > 20 and seen[12] > 20
        # interleaved slices of one concatenation buffer (channels [0,2) in, [2,..) out)
        assert bs.bs_stack_check_buffers(hd, 4096, 256, [far_res], 4096 + in_img, 256, None, far_ws, wsn) == 0
        # residual or workspace under the output
        assert bs.bs_stack_check_buffers(hd, 4096, 0, [1 << 20], (1 << 20) + res_bytes - 16, 0, None, far_ws, wsn) == 12
        assert bs.bs_stack_check_buffers(hd, 4096, 0, [far_res], far_ws + 16, 0, None, far_ws, wsn) == 12
        assert bs.bs_stack_check_buffers(hd, far_ws + wsn - 16, 0, [far_res], 1 << 20, 0, None, far_ws, wsn) == 12
        # strides: below the image, not a multiple of 16 bytes, beyond 2^31 - 1 elements
        assert bs.bs_stack_check_buffers(hd, 4096, 127, [far_res], 1 << 20, 0, None, far_ws, wsn) == 2
        assert bs.bs_stack_check_buffers(hd, 4096, 0, [far_res], 1 << 20, 7, None, far_ws, wsn) == 2
        assert bs.bs_stack_check_buffers(hd, 4096, 129, [far_res], 1 << 20, 0, None, far_ws, wsn) == 7
        assert bs.bs_stack_check_buffers(hd, 4096, 0, [far_res], 1 << 20, 10, None, far_ws, wsn) == 7
        assert bs.bs_stack_check_buffers(hd, 4096, 1 << 31, [far_res], 1 << 20, 0, None, far_ws, wsn) == 2
        # pointers: misaligned, missing, workspace too small
        assert bs.bs_stack_check_buffers(hd, 4100, 0, [far_res], 1 << 20, 0, None, far_ws, wsn) == 7
        assert bs.bs_stack_check_buffers(hd, 4096, 0, None, 1 << 20, 0, None, far_ws, wsn) == 1
        assert bs.bs_stack_check_buffers(hd, 4096, 0, [far_res], 1 << 20, 0, None, far_ws, wsn - 1) == 8
        assert bs.bs_stack_check_buffers(hd, 4096, 0, [far_res], 1 << 20, 0, None, 0, 0) == 8
    finally:
        bs.bs_stack_destroy(hd)
    # in place: allowed without pooling and with equal strides only
    hd = bs.bs_stack_create([wl.relu()], (n, c, h, w), "f32")
    try:
        bs.bs_stack_plan(hd, host_only=1)
        assert bs.bs_stack_check_buffers(hd, 4096, 0, None, 4096, 0, None, 0, 0) == 0
        assert bs.bs_stack_check_buffers(hd, 4096, 256, None, 4096, 256, None, 0, 0) == 0
        assert bs.bs_stack_check_buffers(hd, 4096, 256, None, 4096, 0, None, 0, 0) == 12
        assert bs.bs_stack_check_buffers(hd, 4096, 0, None, 4096 + 16, 0, None, 0, 0) == 12
    finally:
        bs.bs_stack_destroy(hd)
    hd = bs.bs_stack_create([wl.relu()], (n, c, h, w), "f32")
    try:
        assert bs.bs_stack_check_buffers(hd, 4096, 0, None, 1 << 20, 0, None, 0, 0) == 5  # no plan yet
    finally:
        bs.bs_stack_destroy(hd)


def test_probe_arguments_are_checked_before_anything_is_launched():
    """The measurement aids refuse bad arguments on the host (fake addresses, no device needed)."""
    def status(call):
        with pytest.raises(bs.BrainSlugError) as e:
            call()
        return bs.STATUS_NAMES[e.value.status]

    a, b = 1 << 20, 2 << 20
    assert status(lambda: bs.bs_probe_stream(4, False, 0, 64, b, 16, 0)) == "BS_ERR_NULL"
    assert status(lambda: bs.bs_probe_stream(3, False, a, 64, b, 16, 0)) == "BS_ERR_PARAM"      # 1, 2 or 4 reads per write
    assert status(lambda: bs.bs_probe_stream(4, False, a, 64, b, 24, 0)) == "BS_ERR_PARAM"      # whole 128-bit vectors
    assert status(lambda: bs.bs_probe_stream(4, False, a, 63, b, 16, 0)) == "BS_ERR_WORKSPACE"  # the input holds 4 x the output
    assert status(lambda: bs.bs_probe_stream(1, True, a + 8, 64, b, 16, 0)) == "BS_ERR_ALIGN"
    assert status(lambda: bs.bs_probe_issue_rate(0, 1, 10, 0, 1 << 20, 0)) == "BS_ERR_NULL"
    assert status(lambda: bs.bs_probe_issue_rate(0, 9, 10, a, 1 << 20, 0)) == "BS_ERR_PARAM"


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(bs, "_lib", None)
    monkeypatch.setattr(bs, "LIB_PATH", "/nonexistent/libbrainslug_hip.so")
    with pytest.raises(RuntimeError):
        bs.load()
