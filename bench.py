#!/usr/bin/env python3
"""Benchmark of the fused (depth-first) stack path on one MI355X.

Workload (benchmark configuration 1): the three VGG-16-BN shaped post-convolution stacks
BN -> ReLU -> MaxPool 2x2/2 on fp32 tensors 32x64x224x224, 32x128x112x112 and
32x256x56x56 (seeded synthetic N(0,1) activations; no network, weights or images).
One "step" runs all three stacks once.  Inputs are resident in HBM before timing;
every launch reads a buffer set that has not been touched for >= 1 GB of traffic
(rotation), so the 256 MB last-level cache cannot serve it.

Prints ONE JSON line on stdout: whole-step effective GB/s (algorithmic bytes /
wall time), the roofline entry of the dominant kernel (the 64x224x224 stack),
the speed-up over the layer-by-layer HIP plan, and the CPU oracle timed on a
bounded sample.  The line also carries `all_configs`: every benchmark configuration and
storage type timed back to back over rotating buffers (kernel family, microseconds, GB/s,
fraction of the HBM peak).  `--all` adds the long per-configuration table (stderr) with the
layer-by-layer plan and single-launch event timings; `--batch-fit` times the pooling
configurations at several batch sizes and fits time = fixed cost + bytes / rate.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak
PAPER_CONTEXT = ("paper (GTX 1080 Ti / Xeon E5-2690v4, fp32, whole networks vs PyTorch 0.3): up to "
                 "35.7% GPU and 41.1% CPU speed-up; VGG16-BN optimizable layers +146.7% (GPU)")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class StackBench:
    """One stack with `sets` rotating buffer sets on the GPU."""

    def __init__(self, name, dtype, indices=False, min_rotation_bytes=1 << 30, seed=0, **plan_opts):
        import torch
        from paper_1804_08378_amd import brainslug as bs
        from paper_1804_08378_amd import workloads as wl

        self.name, self.dtype = name, dtype
        layers, x, res = wl.inputs_for(name, seed, dtype, indices=indices)
        self.layers, self.shape = layers, x.shape
        self.bytes = wl.algorithmic_bytes(layers, x.shape, dtype, indices)
        self.lbl_bytes = wl.layer_by_layer_bytes(layers, x.shape, dtype)
        self.images = x.shape[0]
        tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[dtype]
        self.fused = bs.Stack(layers, x.shape, dtype).plan(**plan_opts)
        nhwc = plan_opts.get("layout", 0) == bs.BS_LAYOUT_NHWC
        self.lbl = bs.Stack(layers, x.shape, dtype).plan(breadth_first=1, layout=int(nhwc))
        self.sets = min(64, max(2, -(-min_rotation_bytes // self.bytes)))
        mf = torch.channels_last if nhwc else torch.contiguous_format
        x0 = torch.from_numpy(x).to(tdt).cuda().contiguous(memory_format=mf)
        r0 = [torch.from_numpy(r).to(tdt).cuda().contiguous(memory_format=mf) for r in res]
        self.x = [x0] + [x0.clone() for _ in range(self.sets - 1)]
        self.res = [r0] + [[r.clone() for r in r0] for _ in range(self.sets - 1)]
        self.out, self.idx = [], []
        for _ in range(self.sets):
            o, i = self.fused.alloc_outputs("cuda", indices)
            self.out.append(o)
            self.idx.append(i)
        self.fused.workspace("cuda")
        self.lbl.workspace("cuda")
        self.cursor = 0
        self.info = self.fused.info()

    def launch(self, which="fused", stream=None, hot=False):
        s = 0 if hot else self.cursor  # hot: always the same buffers (served by the last-level cache)
        self.cursor = (self.cursor + 1) % self.sets
        st = self.fused if which == "fused" else self.lbl
        st.run(self.x[s], self.res[s], out=self.out[s], indices=self.idx[s],
               stream=None if stream is None else stream.cuda_stream)


def time_steps(stacks, which, steps, warmup, streams=None):
    """K steps (each: every stack once, rotating buffers).  With `streams` (one HIP stream of
    default priority per stack) the stacks of a step, which are independent of each other, are
    enqueued on their own streams, so the tail of one kernel overlaps the start of the next.

    Returns (wall ms per step, {name: mean ms}, {name: min ms}).  The wall time brackets exactly
    `steps` steps with a device synchronisation on both sides and nothing else in between; the
    per-stack figures come from a second pass with one HIP event pair around every launch (on
    torch's current stream, the stream the kernels are launched on).
    """
    import torch

    streams = streams or [None] * len(stacks)
    for _ in range(warmup):
        for sb, st in zip(stacks, streams):
            sb.launch(which, st)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        for sb, st in zip(stacks, streams):
            sb.launch(which, st)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ev = {sb.name: [] for sb in stacks}
    for _ in range(steps):
        for sb in stacks:
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            sb.launch(which)
            b.record()
            ev[sb.name].append((a, b))
    torch.cuda.synchronize()
    per = {k: sum(a.elapsed_time(b) for a, b in v) / len(v) for k, v in ev.items()}
    mins = {k: min(a.elapsed_time(b) for a, b in v) for k, v in ev.items()}
    return (t1 - t0) * 1e3 / steps, per, mins


def time_back_to_back(sb, which, launches, hot=False):
    """Average duration of one launch of `sb` when `launches` of them run back to back between
    one HIP event pair: the kernel's own duration plus the gap to the next launch.  `hot`: every
    launch on the same buffers instead of rotating ones."""
    import torch

    for _ in range(3):
        sb.launch(which, hot=hot)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(launches):
        sb.launch(which, hot=hot)
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / launches


def all_configs_summary(launches=60):
    """Every benchmark configuration and storage type, index outputs off: `launches` launches of
    the fused plan back to back over rotating buffer sets between one HIP event pair."""
    import torch
    from paper_1804_08378_amd import workloads as wl

    rows = []
    for name in wl.CONFIG_NAMES:
        for dt in wl.build(name)[2]:
            sb = StackBench(name, dt)
            us = time_back_to_back(sb, "fused", launches) * 1e3
            g = sb.bytes / us * 1e-3
            rows.append({"config": name, "dtype": dt, "kernels": [q["variant_name"] for q in sb.info["sequences"]],
                         "work_groups": [q["grid"] for q in sb.info["sequences"]], "MB": round(sb.bytes / 1e6, 2),
                         "us": round(us, 2), "GBps": round(g, 1), "frac": round(g / HBM_PEAK_GBPS, 4)})
            log(f"all_configs {name:<16}{dt:<6}{'+'.join(rows[-1]['kernels']):<14}{rows[-1]['MB']:>8.1f} MB"
                f"{us:>8.1f} us{g:>8.0f} GB/s{100 * g / HBM_PEAK_GBPS:>6.1f} %")
            del sb
            torch.cuda.empty_cache()
    return rows


def batch_fit(configs=(("vgg_c", "f32"), ("densenet_trans", "f32"), ("resnet_stem", "f32"), ("resnet_stem", "bf16"),
                       ("halo_stress", "f32"), ("halo_stress", "bf16")), factors=(0.25, 0.5, 1, 2, 4), launches=60):
    """Time = fixed cost per launch + bytes / streaming rate?  Each configuration at several
    multiples of its batch size (same planes, same kernel), least-squares line through
    (bytes, microseconds).  The intercept is what a launch costs however little it moves
    (dispatch, the first memory round trip, the last waves draining); the slope is the rate the
    kernel streams at once the chip is full."""
    import torch
    from paper_1804_08378_amd import brainslug as bs
    from paper_1804_08378_amd import workloads as wl

    rows = []
    for name, dt in configs:
        layers, shape, _ = wl.build(name)
        tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[dt]
        pts = []
        for f in factors:
            n = max(1, int(round(shape[0] * f)))
            shp = (n,) + tuple(shape[1:])
            byts = wl.algorithmic_bytes(layers, shp, dt, False)
            sets = max(2, min(32, (1 << 30) // byts + 1))
            xs = [torch.randn(shp, device="cuda").to(tdt) for _ in range(sets)]
            st = bs.Stack(layers, shp, dt).plan()
            outs = [st.alloc_outputs("cuda", False)[0] for _ in range(sets)]
            for i in range(3):
                st.run(xs[i % sets], out=outs[i % sets], indices=[])
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for i in range(launches):
                st.run(xs[i % sets], out=outs[i % sets], indices=[])
            b.record()
            torch.cuda.synchronize()
            us = a.elapsed_time(b) / launches * 1e3
            pts.append((byts, us, n))
            st.close()
            del xs, outs
            torch.cuda.empty_cache()
        # least squares through the three largest sizes (the smallest do not fill the chip)
        use = pts[-3:]
        mx = sum(p[0] for p in use) / len(use)
        my = sum(p[1] for p in use) / len(use)
        slope = sum((p[0] - mx) * (p[1] - my) for p in use) / sum((p[0] - mx) ** 2 for p in use)
        icpt = my - slope * mx
        row = {"config": name, "dtype": dt, "points": [{"batch": n, "MB": round(b / 1e6, 1), "us": round(u, 2),
                                                         "GBps": round(b / u * 1e-3, 1)} for b, u, n in pts],
               "fixed_us": round(icpt, 2), "streaming_GBps": round(1e-3 / slope, 1)}
        rows.append(row)
        log(f"batch_fit {name:<16}{dt:<6} fixed {icpt:5.1f} us, streaming {1e-3 / slope:6.0f} GB/s   " +
            "  ".join(f"n={n}: {u:.1f} us" for _, u, n in pts))
    return rows


def issue_rates(iterations=20000, clock_ghz=2.4):
    """Cycles per instruction group per SIMD (and per wave) for the kinds of bs_probe_issue_rate,
    with 1, 2, 4 and 8 waves per SIMD: the issue limits that bound the kernels which are not
    bound by HBM.  Cycles are at the nominal 2.4 GHz engine clock."""
    import torch
    from paper_1804_08378_amd import brainslug as bs

    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.empty(cus * 8 * 256, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    rows = []
    for name, kind in bs.PROBE_KINDS.items():
        row = {"kind": name}
        for wps in (1, 2, 4, 8):
            bs.bs_probe_issue_rate(kind, wps, 200, sink.data_ptr(), sink.numel(), stream)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            bs.bs_probe_issue_rate(kind, wps, iterations, sink.data_ptr(), sink.numel(), stream)
            b.record()
            torch.cuda.synchronize()
            ns = a.elapsed_time(b) * 1e6
            row[f"cycles_per_simd_{wps}w"] = round(ns * clock_ghz / (8.0 * iterations * wps), 2)
            row[f"cycles_per_wave_{wps}w"] = round(ns * clock_ghz / (8.0 * iterations), 2)
        rows.append(row)
        log(f"issue_rates {name:<14}" + "".join(f"  {w} waves/SIMD: {row[f'cycles_per_simd_{w}w']:6.2f} per SIMD, "
                                                f"{row[f'cycles_per_wave_{w}w']:6.1f} per wave;" for w in (1, 2, 4, 8)))
    return rows


def hbm_patterns(out_mb=(26, 103), launches=40):
    """What the chip's memory system delivers for streaming access patterns with no arithmetic
    (bs_probe_stream): pure reads, a copy, and four bytes read per byte written (the pattern of a
    2 x 2 pooling step), at the output sizes of vgg_c and vgg_a, over rotating buffers (>= 1 GB
    touched between two uses of a buffer).  Back-to-back launches between two events."""
    import torch
    from paper_1804_08378_amd import brainslug as bs

    stream = torch.cuda.current_stream().cuda_stream
    rows = []
    g = torch.Generator(device="cuda").manual_seed(0)
    for mb in out_mb:
        out_bytes = mb * 1000 * 1000 // 16 * 16
        for rpw, read_only, label in ((4, True, "read only"), (1, False, "copy 1:1"), (2, False, "read 2 : write 1"), (4, False, "read 4 : write 1")):
            in_bytes = out_bytes * rpw
            moved = in_bytes + (0 if read_only else out_bytes)
            sets = max(2, min(16, (1 << 30) // moved + 1))
            ins = [torch.randint(0, 2 ** 31 - 1, (in_bytes // 4,), dtype=torch.int32, device="cuda", generator=g) for _ in range(sets)]
            outs = [torch.empty(out_bytes // 4, dtype=torch.int32, device="cuda") for _ in range(sets)]
            for i in range(3):
                bs.bs_probe_stream(rpw, read_only, ins[i % sets].data_ptr(), in_bytes, outs[i % sets].data_ptr(), out_bytes, stream)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for i in range(launches):
                bs.bs_probe_stream(rpw, read_only, ins[i % sets].data_ptr(), in_bytes, outs[i % sets].data_ptr(), out_bytes, stream)
            b.record()
            torch.cuda.synchronize()
            us = a.elapsed_time(b) * 1e3 / launches
            row = {"pattern": label, "MB_moved": moved / 1e6, "us_per_launch": us, "GBps": moved / (us * 1e-6) / 1e9,
                   "pct_peak": 100 * moved / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS}
            rows.append(row)
            log(f"hbm_pattern {label:<18}{row['MB_moved']:>8.1f} MB{us:>8.1f} us{row['GBps']:>8.0f} GB/s{row['pct_peak']:>6.1f} % of peak")
            del ins, outs
            torch.cuda.empty_cache()
    return rows


def launch_only(spec, launches):
    """`launches` launches of one configuration and nothing else (no timing): the leg for
    rocprofv3 counter and kernel-trace runs.  spec = NAME:DTYPE[:key=value,...]; NAME is a
    benchmark configuration or deepN (N blocks of MaxPool 3/1/1 -> BatchNorm -> ReLU on
    64 x 64 x 56 x 56); the keys are plan options (layout=1, lane_exchange=-1, force_variant=3,
    max_steps_per_sequence=5 ...), indices=1 and backward=1 (the backward pass of the configuration)."""
    import torch
    from paper_1804_08378_amd import brainslug as bs
    from paper_1804_08378_amd import workloads as wl

    parts = spec.split(":")
    name, dt = parts[0], parts[1]
    opts = dict(kv.split("=") for kv in parts[2].split(",")) if len(parts) > 2 and parts[2] else {}
    opts = {k: int(v) for k, v in opts.items()}
    indices = bool(opts.pop("indices", 0))
    backward = bool(opts.pop("backward", 0))
    if backward:
        layers, shape, _ = wl.build(name, 0, None, False)
        tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[dt]
        mf = torch.channels_last if opts.get("layout", 0) else torch.contiguous_format
        rnd = lambda sh: torch.randn(sh, device="cuda").to(tdt).contiguous(memory_format=mf)
        st = bs.Stack(layers, shape, dt).plan(**opts).plan_backward()
        sets = [(rnd(shape), [rnd(sh) for sh in wl.residual_shapes(layers, shape)], rnd(wl.output_shape(layers, shape))) for _ in range(3)]
        for i in range(launches):
            x, res, dy = sets[i % 3]
            st.backward(x, res, dy)
        info = st.info()
    elif name.startswith("deep"):
        c, n = 64, int(name[4:])
        layers = sum(([wl.maxpool(3, 1, 1), wl.bn_params(c, 100 + i), wl.relu()] for i in range(n)), [])
        tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[dt]
        st = bs.Stack(layers, (64, c, 56, 56), dt).plan(**opts)
        xs = [torch.randn(64, c, 56, 56, device="cuda").to(tdt) for _ in range(4)]
        outs = [st.alloc_outputs("cuda", False)[0] for _ in range(4)]
        for i in range(launches):
            st.run(xs[i % 4], out=outs[i % 4], indices=[])
        info = st.info()
    else:
        sb = StackBench(name, dt, indices=indices, **opts)
        for _ in range(launches):
            sb.launch("fused")
        info = sb.info
    torch.cuda.synchronize()
    log("launched", spec, "x", launches, "sequences:",
        [(q["variant_name"], q["grid"], q["threads_per_group"], q["tile_rows"]) for q in info["sequences"]])


def cpu_baseline(names, dtype, batch, passes):
    """Time the breadth-first CPU oracle, as it stands, on the same stacks: `passes` passes over
    the workload at `batch` images with all host threads, plus one single-thread pass."""
    from oracle import breadth_first as bf
    from oracle import layers as OL
    from paper_1804_08378_amd import workloads as wl

    threads = OL.max_threads()
    data = [wl.inputs_for(n, 0, dtype, batch=batch) for n in names]
    nbytes = sum(wl.algorithmic_bytes(l, x.shape, dtype) for l, x, _ in data)
    for layers, x, res in data:  # warm the pages
        bf.run_stack(layers, x, res, dtype)
    t0 = time.perf_counter()
    for _ in range(passes):
        for layers, x, res in data:
            bf.run_stack(layers, x, res, dtype)
    t_all = (time.perf_counter() - t0) / passes
    OL.set_threads(1)
    t0 = time.perf_counter()
    for layers, x, res in data:
        bf.run_stack(layers, x, res, dtype)
    t_one = time.perf_counter() - t0
    OL.set_threads(threads)
    return {"value": round(nbytes / t_all / 1e9, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "seconds_per_pass": round(t_all, 4), "single_thread_GBps": round(nbytes / t_one / 1e9, 3),
            "sample": f"stacks {'+'.join(names)} at batch {batch} (the full workload), {passes} passes with "
                      f"{threads} OpenMP threads (~{t_all * passes * threads:.0f} core-seconds) and one "
                      "single-thread pass; same algorithmic-bytes metric"}


def backward_configs(steps=30, warmup=3, min_rotation_bytes=1 << 30, channels_last=False):
    """Backward pass of every benchmark configuration: `bs_stack_backward` (recompute from the stack
    input, one gather kernel per stage) against the framework's autograd over the same layers run one by
    one (its backward alone, on a retained graph; and forward + backward together on both sides).
    GB/s counts the bytes a backward pass must move: input, residual operands and upstream gradient in,
    gradients out."""
    import numpy as np
    import torch
    import torch.nn.functional as F
    from paper_1804_08378_amd import brainslug as bs
    from paper_1804_08378_amd import workloads as wl

    def torch_forward(layers, x, res):
        cur, pending = x, list(res)
        for l in layers:
            k = l["kind"]
            if k == "bn":
                cur = F.batch_norm(cur, l["_mean"], l["_var"], l["_gamma"], l["_beta"], False, 0.0, l["eps"])
            elif k == "relu":
                cur = torch.relu(cur)
            elif k == "add":
                cur = cur + pending.pop(0)
            elif k == "maxpool":
                cur = F.max_pool2d(cur, l["k"], l["s"], l["p"])
            else:
                cur = F.avg_pool2d(cur, l["k"], l["s"], l["p"], False, l["count_include_pad"])
        return cur

    def timed(fn, n):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        ev = []
        for _ in range(n):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            ev.append((a, b))
        torch.cuda.synchronize()
        t = [a.elapsed_time(b) for a, b in ev]
        return sum(t) / len(t), min(t)

    mf = torch.channels_last if channels_last else torch.contiguous_format
    log("backward pass%s: bs_stack_backward vs the framework's autograd over the same layers" %
        (", channels-last tensors" if channels_last else ""))
    log(f"{'config':<16}{'dtype':<6}{'stages':>7}{'MB':>8}{'us mean':>9}{'us min':>8}{'GB/s':>8}{'%peak':>7}"
        f"{'autograd us':>12}{'speedup':>8}{'f+b us':>9}{'torch f+b':>10}{'speedup':>8}")
    rows = []
    for name in wl.CONFIG_NAMES:
        for dt in wl.build(name)[2]:
            layers, shape, _ = wl.build(name, 0, None, False)
            tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[dt]
            es = 4 if dt == "f32" else 2
            out_shape = wl.output_shape(layers, shape)
            res_shapes = wl.residual_shapes(layers, shape)
            numel = lambda sh: int(np.prod(sh))
            nbytes = (2 * numel(shape) + 2 * sum(numel(r) for r in res_shapes) + numel(out_shape)) * es
            sets = min(16, max(2, -(-min_rotation_bytes // nbytes)))
            g = torch.Generator(device="cuda").manual_seed(0)
            rnd = lambda sh: torch.randn(sh, device="cuda", generator=g).to(tdt).contiguous(memory_format=mf)
            xs = [rnd(shape) for _ in range(sets)]
            rs = [[rnd(r) for r in res_shapes] for _ in range(sets)]
            dys = [rnd(out_shape) for _ in range(sets)]
            st = bs.Stack(layers, shape, dt).plan(layout=1 if channels_last else 0).plan_backward()
            stages = bs.bs_stack_backward_num_stages(st.handle)
            gx = [torch.empty_like(xs[0], memory_format=mf) for _ in range(sets)]
            gr = [[torch.empty_like(r, memory_format=mf) for r in rs[0]] for _ in range(sets)]
            wsn = bs.bs_stack_backward_workspace_bytes(st.handle)
            ws = torch.empty(max(wsn, 16), dtype=torch.uint8, device="cuda")
            stream = torch.cuda.current_stream().cuda_stream
            cur = [0]

            def ours():
                i = cur[0] = (cur[0] + 1) % sets
                bs.bs_stack_backward(st.handle, xs[i].data_ptr(), [r.data_ptr() for r in rs[i]], None, dys[i].data_ptr(),
                                     gx[i].data_ptr(), [t.data_ptr() for t in gr[i]], ws.data_ptr(), wsn, stream)

            outs = [st.alloc_outputs("cuda", False)[0] for _ in range(sets)]

            def ours_fb():
                i = cur[0] = (cur[0] + 1) % sets
                st.run(xs[i], rs[i], out=outs[i], indices=[])
                bs.bs_stack_backward(st.handle, xs[i].data_ptr(), [r.data_ptr() for r in rs[i]], None, dys[i].data_ptr(),
                                     gx[i].data_ptr(), [t.data_ptr() for t in gr[i]], ws.data_ptr(), wsn, stream)

            ms, mn = timed(ours, steps)
            ms_fb, _ = timed(ours_fb, steps)
            # with the picks kept from the forward pass (index outputs of bs_stack_run) instead of recomputed
            ms_kept = None
            layers_idx = wl.build(name, 0, None, True)[0]
            if any(l.get("return_indices") for l in layers_idx):
                st2 = bs.Stack(layers_idx, shape, dt).plan(layout=1 if channels_last else 0).plan_backward()
                kept = [st2.run(xs[i], rs[i])[1] for i in range(sets)]

                def ours_kept():
                    i = cur[0] = (cur[0] + 1) % sets
                    bs.bs_stack_backward(st2.handle, xs[i].data_ptr(), [r.data_ptr() for r in rs[i]], [t.data_ptr() for t in kept[i]],
                                         dys[i].data_ptr(), gx[i].data_ptr(), [t.data_ptr() for t in gr[i]], ws.data_ptr(), wsn, stream)

                if bs.bs_stack_backward_workspace_bytes(st2.handle) <= max(wsn, 16):
                    ms_kept, _ = timed(ours_kept, steps)
                st2.close()
                del kept
            # the framework: parameters on the device, one retained graph per buffer set
            tl = []
            for l in layers:
                l = dict(l)
                if l["kind"] == "bn":
                    for k in ("mean", "var", "gamma", "beta"):
                        l["_" + k] = torch.from_numpy(l[k]).cuda().to(tdt)
                tl.append(l)
            tsets = min(sets, 3)  # a retained graph holds every layer's output
            graphs = []
            for i in range(tsets):
                leaves = [xs[i].detach().requires_grad_(True)] + [r.detach().requires_grad_(True) for r in rs[i]]
                graphs.append((torch_forward(tl, leaves[0], leaves[1:]), leaves))

            def torch_bwd():
                i = cur[0] = (cur[0] + 1) % tsets
                y, leaves = graphs[i]
                torch.autograd.grad(y, leaves, dys[i], retain_graph=True)

            ms_t, _ = timed(torch_bwd, max(5, steps // 3))
            del graphs

            def torch_fb():
                i = cur[0] = (cur[0] + 1) % tsets
                leaves = [xs[i].detach().requires_grad_(True)] + [r.detach().requires_grad_(True) for r in rs[i]]
                torch.autograd.grad(torch_forward(tl, leaves[0], leaves[1:]), leaves, dys[i])

            ms_tfb, _ = timed(torch_fb, max(5, steps // 3))
            gbps = nbytes / (ms * 1e-3) / 1e9
            row = {"config": name, "dtype": dt, "stages": stages, "MB": nbytes / 1e6, "us_mean": ms * 1e3, "us_min": mn * 1e3,
                   "GBps": gbps, "pct_peak": 100 * gbps / HBM_PEAK_GBPS, "autograd_backward_us": ms_t * 1e3,
                   "speedup_backward": ms_t / ms, "forward_backward_us": ms_fb * 1e3,
                   "autograd_forward_backward_us": ms_tfb * 1e3, "speedup_forward_backward": ms_tfb / ms_fb,
                   "us_mean_with_saved_picks": None if ms_kept is None else ms_kept * 1e3}
            rows.append(row)
            log(f"{name:<16}{dt:<6}{stages:>7}{row['MB']:>8.1f}{row['us_mean']:>9.1f}{row['us_min']:>8.1f}{gbps:>8.0f}"
                f"{row['pct_peak']:>7.1f}{row['autograd_backward_us']:>12.1f}{row['speedup_backward']:>8.2f}"
                f"{row['forward_backward_us']:>9.1f}{row['autograd_forward_backward_us']:>10.1f}"
                f"{row['speedup_forward_backward']:>8.2f}" + ("" if ms_kept is None else f"   with saved picks {ms_kept * 1e3:.1f} us"))
            st.close()
            del xs, rs, dys, gx, gr, outs, ws
            torch.cuda.empty_cache()
    return rows


def deep_stacks(shape=(64, 64, 56, 56), counts=(1, 2, 3, 4, 5, 6, 8, 10, 12, 16, 20, 24, 32, 40)):
    """Section 5.1: networks of n blocks <MaxPool k3 s1 p1, BatchNorm, ReLU>, executed layer by
    layer and fused with at most 1 step, at most 5 steps, and unrestricted steps per sequence.
    The paper does not state its tensor shape; 64x64x56x56 fp32 is this benchmark's choice.
    Times are the minimum of 10 launches (the paper's protocol) over rotating inputs."""
    import torch
    from paper_1804_08378_amd import brainslug as bs
    from paper_1804_08378_amd import workloads as wl

    xs = [torch.from_numpy(wl.activation(shape, 0)).cuda()]
    xs += [xs[0].clone() for _ in range(9)]
    strategies = (("layer_by_layer", dict(breadth_first=1)), ("steps1", dict(max_steps_per_sequence=1)),
                  ("steps5", dict(max_steps_per_sequence=5)), ("unrestricted", dict()))
    rows = []
    log(f"{'blocks':>6}" + "".join(f"{n + ' us (seq)':>24}" for n, _ in strategies) + f"{'best speed-up':>15}")
    for n in counts:
        layers = sum(([wl.maxpool(3, 1, 1), wl.bn_params(shape[1], 100 + i), wl.relu()] for i in range(n)), [])
        row = {"blocks": n}
        for name, opts in strategies:
            st = bs.Stack(layers, shape, "f32").plan(**opts)
            outs = [st.alloc_outputs("cuda", False)[0] for _ in range(10)]
            st.workspace("cuda")
            for i in range(3):
                st.run(xs[i], out=outs[i], indices=[])
            torch.cuda.synchronize()
            times = []
            for i in range(10):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                st.run(xs[i], out=outs[i], indices=[])
                b.record()
                torch.cuda.synchronize()
                times.append(a.elapsed_time(b) * 1e3)
            row[name] = {"us_min": round(min(times), 1), "sequences": st.info()["n_sequences"]}
            st.close()
            del outs
        row["speedup_best_fused_vs_layer_by_layer"] = round(
            row["layer_by_layer"]["us_min"] / min(row[k]["us_min"] for k in ("steps1", "steps5", "unrestricted")), 2)
        rows.append(row)
        log(f"{n:>6}" + "".join(f"{row[k]['us_min']:>17.1f} ({row[k]['sequences']:>3})" for k, _ in strategies)
            + f"{row['speedup_best_fused_vs_layer_by_layer']:>15.2f}")
    return {"shape": list(shape), "dtype": "f32", "protocol": "min of 10 launches", "rows": rows}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--all", action="store_true", help="also report every benchmark configuration (stderr)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--cpu-batch", type=int, default=32)
    ap.add_argument("--cpu-passes", type=int, default=25,
                    help="passes of the CPU oracle over the workload (25: about 17 core-seconds on 16 threads)")
    ap.add_argument("--no-baseline", action="store_true",
                    help="skip the layer-by-layer HIP plan (its pooling layer runs the same kernel symbol "
                         "as the fused stack, which would mix the two in a rocprofv3 --stats summary)")
    ap.add_argument("--deep", action="store_true",
                    help="also run the stacked-layers experiment of Section 5.1: 1..40 blocks of "
                         "<MaxPool 3/1/1, BatchNorm, ReLU> under the three sequence strategies")
    ap.add_argument("--streams", action="store_true",
                    help="enqueue the three independent stacks of a step on one HIP stream each (default priority) "
                         "instead of all on one stream: kernels then overlap at their edges")
    ap.add_argument("--backward", action="store_true",
                    help="also time the backward pass of every benchmark configuration against the framework's autograd (stderr)")
    ap.add_argument("--nhwc", action="store_true",
                    help="also time every configuration with channels-last (NHWC) tensors and plans")
    ap.add_argument("--no-all-configs", action="store_true", help="leave the all_configs summary out of the JSON line")
    ap.add_argument("--batch-fit", action="store_true",
                    help="also time the pooling configurations at 1/4 .. 4 times their batch size and fit "
                         "time = fixed cost + bytes / rate")
    ap.add_argument("--issue-rates", action="store_true",
                    help="also measure the device's instruction issue rates (bs_probe_issue_rate)")
    ap.add_argument("--hbm-patterns", action="store_true",
                    help="also measure what streaming access patterns without arithmetic reach (bs_probe_stream)")
    ap.add_argument("--launch", nargs=2, metavar=("SPEC", "N"),
                    help="only launch one configuration N times (for rocprofv3): SPEC = NAME:DTYPE[:key=value,...]")
    ap.add_argument("--time", nargs=2, metavar=("SPEC", "N"), dest="time_one",
                    help="time the fused plan of one configuration: N single launches between event pairs over rotating "
                         "inputs; SPEC as for --launch (forward plans; plan options and indices=1).  One JSON line.")
    ap.add_argument("--probe", type=int, default=0, metavar="N",
                    help="counter probe for rocprofv3 --pmc: N launches of a plain copy of known size, "
                         "then N launches of each VGG stack; no timing, no JSON")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build measures one GPU only (the path shards over the batch with no "
            "exchange; multi-GPU figures are not produced). Use --gpus 1.")
        sys.exit(2)

    import torch
    from paper_1804_08378_amd import brainslug as bs
    from paper_1804_08378_amd import workloads as wl

    if not torch.cuda.is_available():
        log("bench.py needs a GPU")
        sys.exit(2)
    bs.load()
    log(bs.bs_version(), "|", torch.cuda.get_device_name(0))

    if args.launch:
        launch_only(args.launch[0], int(args.launch[1]))
        return

    if args.time_one:
        parts = args.time_one[0].split(":")
        opts = {k: int(v) for k, v in (kv.split("=") for kv in parts[2].split(","))} if len(parts) > 2 and parts[2] else {}
        sb = StackBench(parts[0], parts[1], indices=bool(opts.pop("indices", 0)), **opts)
        _, per, mins = time_steps([sb], "fused", int(args.time_one[1]), 3)
        q = sb.info["sequences"]
        print(json.dumps({"config": parts[0], "dtype": parts[1], "options": opts, "launches": int(args.time_one[1]),
                          "us_mean": round(per[parts[0]] * 1e3, 1), "us_min": round(mins[parts[0]] * 1e3, 1),
                          "GBps": round(sb.bytes / (per[parts[0]] * 1e-3) / 1e9), "variants": [x["variant_name"] for x in q],
                          "tile_rows": [x["tile_rows"] for x in q], "work_groups": [x["grid"] for x in q]}))
        return

    if args.probe:
        # a copy of exactly 256 MiB in and 256 MiB out calibrates the byte counters
        n = (256 << 20) // 4
        src, dst = torch.ones(n, device="cuda"), torch.empty(n, device="cuda")
        for _ in range(args.probe):
            torch.mul(src, 1.0, out=dst)  # an element-wise kernel: reads n floats, writes n floats
        torch.cuda.synchronize()
        for name in wl.VGG_STACKS:
            sb = StackBench(name, "f32")
            for _ in range(args.probe):
                sb.launch("fused")
            torch.cuda.synchronize()
            log("probe", name, "algorithmic bytes per launch", sb.bytes)
            # the backward pass of the same stack (input and upstream gradient in, input gradient out)
            dy, gx = torch.randn_like(sb.out[0]), torch.empty_like(sb.x[0])
            sb.fused.plan_backward()
            for _ in range(args.probe):
                sb.fused.backward_unchecked(sb.x[0], sb.res[0], dy, gx, [])
            torch.cuda.synchronize()
            log("probe", name, "backward: algorithmic bytes per launch", 2 * sb.x[0].numel() * 4 + dy.numel() * 4)
        return

    stacks = [StackBench(n, "f32") for n in wl.VGG_STACKS]
    step_bytes = sum(sb.bytes for sb in stacks)
    streams = [torch.cuda.Stream() for _ in stacks] if args.streams else None
    ms, per, mins = time_steps(stacks, "fused", args.steps, args.warmup, streams)
    if args.no_baseline:
        ms_lbl = float("nan")
    else:
        ms_lbl, per_lbl, _ = time_steps(stacks, "lbl", max(10, args.steps // 4), max(2, args.warmup // 2), streams)
    value = step_bytes / (ms * 1e-3) / 1e9
    dom = stacks[0]
    b2b = {sb.name: time_back_to_back(sb, "fused", max(20, args.steps // 2)) for sb in stacks}
    dom_ms = b2b[dom.name]
    achieved = dom.bytes / (dom_ms * 1e-3) / 1e9
    out = {
        "metric": "fused-stack effective HBM GB/s (algorithmic bytes / time), 1 GPU",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "BASELINE config 1: VGG-16-BN stacks BN->ReLU->MaxPool2x2/2, fp32, "
                               "batch 32, 64x224x224 + 128x112x112 + 256x56x56, indices off",
                   "rotation_sets": [sb.sets for sb in stacks],
                   "streams": len(stacks) if args.streams else 1},
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBPS, 2),
        "images_per_s": round(dom.images / (ms * 1e-3), 1),
        "speedup_vs_layer_by_layer": None if args.no_baseline else round(ms_lbl / ms, 3),
        "layer_by_layer": None if args.no_baseline else {
            "ms_per_step": round(ms_lbl, 4),
            "GBps_of_its_own_traffic": round(sum(sb.lbl_bytes for sb in stacks) / (ms_lbl * 1e-3) / 1e9, 1)},
        # ms_back_to_back: launches of this stack alone, back to back between one HIP event pair (what the
        # roofline entry uses; it agrees with the kernel trace).  ms_mean / ms_min: one event pair per launch
        # inside the step loop, which adds the events' own 2 .. 3 us to every launch.
        "per_stack": {sb.name: {"ms_back_to_back": round(b2b[sb.name], 4),
                                "GBps": round(sb.bytes / (b2b[sb.name] * 1e-3) / 1e9, 1),
                                "ms_mean": round(per[sb.name], 4), "ms_min": round(mins[sb.name], 4),
                                "GBps_single_event_pair": round(sb.bytes / (per[sb.name] * 1e-3) / 1e9, 1),
                                "variant": [q["variant_name"] for q in sb.info["sequences"]]}
                      for sb in stacks},
        "roofline": {"bound": "hbm", "kernel": "pool_direct_kernel<f32,4,2,2> on 32x64x224x224",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None,
                     "bytes_per_launch": dom.bytes, "avg_launch_ms": round(dom_ms, 4),
                     "avg_launch_ms_single_event_pair": round(per[dom.name], 4)},
        "context": PAPER_CONTEXT,
    }
    # HBM bytes per launch from hardware counters are not measured by this run: they are the figure
    # recorded in profiles/traffic.json (from two rocprofv3 --pmc runs of `bench.py --probe`, see
    # profiles/pool_direct_vgg_hbm_traffic.md), and `traffic_source` says so
    traffic_file = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(traffic_file):
        try:
            with open(traffic_file) as f:
                tj = json.load(f)
            out["roofline"]["traffic"] = tj.get("vgg_a_f32_bytes_per_launch")
            out["roofline"]["traffic_source"] = ("stored: profiles/traffic.json (" + str(tj.get("measured", "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE")) +
                                                 "), not measured by this run")
        except Exception:
            pass
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(wl.VGG_STACKS, "f32", args.cpu_batch, args.cpu_passes)
    else:
        out["cpu_baseline"] = None

    if not args.no_all_configs and not args.all:
        del stacks
        stacks = None
        torch.cuda.empty_cache()
        out["all_configs"] = all_configs_summary()
    if args.issue_rates:
        out["issue_rates"] = issue_rates()
    if args.hbm_patterns:
        stacks = None
        torch.cuda.empty_cache()
        out["hbm_patterns"] = hbm_patterns()
    if args.batch_fit:
        stacks = None
        torch.cuda.empty_cache()
        out["batch_fit"] = batch_fit()
    if args.deep:
        out["deep_stacks"] = deep_stacks()

    if args.all:
        del stacks
        torch.cuda.empty_cache()
        # context: a plain device-to-device copy (read N + write N bytes) of the largest input
        src = [torch.empty(411041792 // 4, dtype=torch.float32, device="cuda").normal_() for _ in range(3)]
        dst = [torch.empty_like(t) for t in src]
        for i in range(6):
            dst[i % 3].copy_(src[i % 3])
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(30):
            dst[i % 3].copy_(src[i % 3])
        b.record()
        torch.cuda.synchronize()
        out["copy_GBps_context"] = round(2 * 411041792 * 30 / (a.elapsed_time(b) * 1e-3) / 1e9, 1)
        log("plain copy (torch copy_, 411 MB read + 411 MB write):", out["copy_GBps_context"], "GB/s")
        del src, dst
        torch.cuda.empty_cache()
        log(f"{'config':<16}{'dtype':<6}{'variant':<13}{'MB':>8}{'us mean':>9}{'us min':>8}{'GB/s':>8}"
            f"{'%peak':>7}{'img/s':>10}{'lbl us':>9}{'speedup':>8}{'b2b us':>8}{'hot us':>8}")
        rows = []
        for name in wl.CONFIG_NAMES:
            for dt in wl.build(name)[2]:
                for idx in ([False, True] if any(l["kind"] == "maxpool" for l in wl.build(name)[0]) else [False]):
                    sb = StackBench(name, dt, indices=idx)
                    m, p, mn = time_steps([sb], "fused", args.steps, args.warmup)
                    pl = {name: float("nan")}
                    if not args.no_baseline:
                        ml, pl, _ = time_steps([sb], "lbl", max(10, args.steps // 4), 2)
                    g = sb.bytes / (p[name] * 1e-3) / 1e9
                    row = {"config": name + ("+idx" if idx else ""), "dtype": dt,
                           "variant": sb.info["sequences"][0]["variant_name"], "MB": sb.bytes / 1e6,
                           "us_mean": p[name] * 1e3, "us_min": mn[name] * 1e3, "GBps": g,
                           "pct_peak": 100 * g / HBM_PEAK_GBPS, "img_s": sb.images / (p[name] * 1e-3),
                           "lbl_us": pl[name] * 1e3, "speedup": pl[name] / p[name],
                           # back-to-back launches over rotating buffers, and on one buffer set: the
                           # latter is served by the 256 MB last-level cache where the tensors fit
                           # and is no HBM figure
                           "us_back_to_back": time_back_to_back(sb, "fused", args.steps) * 1e3,
                           "us_hot_single_buffer": time_back_to_back(sb, "fused", args.steps, hot=True) * 1e3,
                           # work-items per launch of every sequence: what a kernel trace lists as grid size
                           "work_items": [q["grid"] * q["threads_per_group"] for q in sb.info["sequences"]]}
                    # the same fraction from the back-to-back time (no event pair per launch: what a network's
                    # stream of kernels sees); pct_peak above is the single-launch figure
                    row["pct_peak_back_to_back"] = 100 * sb.bytes / (row["us_back_to_back"] * 1e-6) / 1e9 / HBM_PEAK_GBPS
                    rows.append(row)
                    log(f"{row['config']:<16}{dt:<6}{row['variant']:<13}{row['MB']:>8.1f}{row['us_mean']:>9.1f}"
                        f"{row['us_min']:>8.1f}{g:>8.0f}{row['pct_peak']:>7.1f}{row['img_s']:>10.0f}"
                        f"{row['lbl_us']:>9.1f}{row['speedup']:>8.2f}{row['us_back_to_back']:>8.1f}"
                        f"{row['us_hot_single_buffer']:>8.1f}")
                    del sb
                    torch.cuda.empty_cache()
        out["all_configs"] = rows

    if args.backward:
        stacks = None
        torch.cuda.empty_cache()
        out["backward_configs"] = backward_configs(steps=min(args.steps, 30))
        out["backward_configs_channels_last"] = backward_configs(steps=min(args.steps, 30), channels_last=True)

    if args.nhwc:
        stacks = None
        torch.cuda.empty_cache()
        log("channels-last (NHWC) plans: one step per sequence, or two pooling steps in one tile kernel")
        log(f"{'config':<16}{'dtype':<6}{'sequences':<24}{'MB':>8}{'us mean':>9}{'us min':>8}{'GB/s':>8}{'%peak':>7}"
            f"{'lbl us':>9}{'speedup':>8}")
        rows = []
        for name in wl.CONFIG_NAMES:
            for dt in wl.build(name)[2]:
                sb = StackBench(name, dt, layout=1)
                m, p, mn = time_steps([sb], "fused", args.steps, args.warmup)
                ml, pl, _ = time_steps([sb], "lbl", max(10, args.steps // 4), 2)
                g = sb.bytes / (p[name] * 1e-3) / 1e9
                seqs = "+".join(q["variant_name"] for q in sb.info["sequences"])
                row = {"config": name, "dtype": dt, "sequences": seqs, "MB": sb.bytes / 1e6,
                       "us_mean": p[name] * 1e3, "us_min": mn[name] * 1e3, "GBps": g,
                       "pct_peak": 100 * g / HBM_PEAK_GBPS, "lbl_us": pl[name] * 1e3, "speedup": pl[name] / p[name]}
                rows.append(row)
                log(f"{name:<16}{dt:<6}{seqs:<24}{row['MB']:>8.1f}{row['us_mean']:>9.1f}{row['us_min']:>8.1f}{g:>8.0f}"
                    f"{row['pct_peak']:>7.1f}{row['lbl_us']:>9.1f}{row['speedup']:>8.2f}")
                del sb
                torch.cuda.empty_cache()
        out["nhwc_configs"] = rows
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
