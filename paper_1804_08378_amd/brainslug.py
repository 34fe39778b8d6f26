"""ctypes binding of libbrainslug_hip.so -- argument marshalling only.

Every function here has the name of the C entry point it forwards to
(include/brainslug.h).  `Stack` is a small convenience wrapper around a
handle that takes torch tensors and passes their device pointers and the
current HIP stream.  No step of the method runs in Python, and there is no
fallback: if the library has not been built, loading it raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libbrainslug_hip.so")

BS_OK = 0
BS_F32, BS_BF16, BS_F16 = 0, 1, 2
BS_BATCHNORM, BS_RELU, BS_ADD, BS_MAXPOOL, BS_AVGPOOL, BS_LEAKY_RELU, BS_CLAMP = 1, 2, 3, 4, 5, 6, 7
BS_VARIANT_AUTO, BS_VARIANT_STREAM, BS_VARIANT_POOL_DIRECT, BS_VARIANT_LDS_TILE = 0, 1, 2, 3
BS_VARIANT_POOL_ROWS, BS_VARIANT_PLANE_POOL = 4, 5
BS_VARIANT_NHWC_STREAM, BS_VARIANT_NHWC_POOL, BS_VARIANT_NHWC_TILE, BS_VARIANT_ROWS_CHAIN, BS_VARIANT_NHWC_ROWS = 6, 7, 8, 9, 10
VARIANT_NAMES = {1: "stream", 2: "pool_direct", 3: "lds_tile", 4: "pool_rows", 5: "plane_pool", 6: "nhwc_stream",
                 7: "nhwc_pool", 8: "nhwc_tile", 9: "rows_chain", 10: "nhwc_rows"}
BS_LAYOUT_NCHW, BS_LAYOUT_NHWC = 0, 1
STATUS_NAMES = {
    0: "BS_OK", 1: "BS_ERR_NULL", 2: "BS_ERR_SHAPE", 3: "BS_ERR_PARAM", 4: "BS_ERR_UNSUPPORTED",
    5: "BS_ERR_NOT_PLANNED", 6: "BS_ERR_NO_FIT", 7: "BS_ERR_ALIGN", 8: "BS_ERR_WORKSPACE",
    9: "BS_ERR_HIP", 10: "BS_ERR_ALLOC", 11: "BS_ERR_RANGE", 12: "BS_ERR_ALIAS", 13: "BS_ERR_JIT", 14: "BS_ERR_DEVICE",
}

STATUS_BY_NAME = {v: k for k, v in STATUS_NAMES.items()}

_f32p = C.POINTER(C.c_float)


class bs_layer_desc(C.Structure):
    _fields_ = [("kind", C.c_int32),
                ("kh", C.c_int32), ("kw", C.c_int32), ("sh", C.c_int32), ("sw", C.c_int32),
                ("ph", C.c_int32), ("pw", C.c_int32),
                ("count_include_pad", C.c_int32), ("return_indices", C.c_int32),
                ("ceil_mode", C.c_int32), ("dilation_h", C.c_int32), ("dilation_w", C.c_int32),
                ("eps", C.c_double),
                ("gamma", _f32p), ("beta", _f32p), ("running_mean", _f32p), ("running_var", _f32p),
                ("negative_slope", C.c_float), ("clamp_min", C.c_float), ("clamp_max", C.c_float),
                ("reserved", C.c_float)]


class bs_plan_options(C.Structure):
    _fields_ = [("max_lds_bytes", C.c_uint64),
                ("max_steps_per_sequence", C.c_int32), ("threads_per_group", C.c_int32),
                ("num_cus", C.c_int32), ("breadth_first", C.c_int32), ("force_variant", C.c_int32),
                ("tile_rows", C.c_int32), ("tile_cols", C.c_int32), ("planes_per_group", C.c_int32),
                ("host_only", C.c_int32), ("jit", C.c_int32), ("layout", C.c_int32),
                ("lane_exchange", C.c_int32), ("reserved", C.c_int32 * 2)]


class bs_plan_info(C.Structure):
    _fields_ = [("n_operations", C.c_int32), ("n_steps", C.c_int32), ("n_sequences", C.c_int32),
                ("device_planned", C.c_int32), ("workspace_bytes", C.c_uint64),
                ("algorithmic_bytes", C.c_uint64)]


class bs_step_info(C.Structure):
    _fields_ = [("first_operation", C.c_int32), ("n_operations", C.c_int32),
                ("pool_operation", C.c_int32), ("sequence", C.c_int32)]


class bs_sequence_info(C.Structure):
    _fields_ = [("first_step", C.c_int32), ("n_steps", C.c_int32),
                ("first_layer", C.c_int32), ("n_layers", C.c_int32),
                ("variant", C.c_int32), ("n_levels", C.c_int32),
                ("tile_rows", C.c_int32), ("tile_cols", C.c_int32), ("planes_per_group", C.c_int32),
                ("halo_rows", C.c_int32), ("halo_cols", C.c_int32), ("threads_per_group", C.c_int32),
                ("grid", C.c_int64), ("lds_bytes", C.c_uint64),
                ("in_shape", C.c_int64 * 4), ("out_shape", C.c_int64 * 4), ("redundancy", C.c_double),
                ("run_time_build", C.c_int32), ("reserved", C.c_int32)]


_lib = None

_SIGNATURES = {
    "bs_stack_create": (C.c_int, [C.POINTER(bs_layer_desc), C.c_int32, C.POINTER(C.c_int64), C.c_int,
                                  C.POINTER(C.c_void_p)]),
    "bs_stack_destroy": (None, [C.c_void_p]),
    "bs_stack_output_shape": (C.c_int, [C.c_void_p, C.POINTER(C.c_int64)]),
    "bs_stack_num_residuals": (C.c_int32, [C.c_void_p]),
    "bs_stack_residual_shape": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_int64)]),
    "bs_stack_num_index_outputs": (C.c_int32, [C.c_void_p]),
    "bs_stack_index_shape": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_int64)]),
    "bs_stack_folded_bn": (C.c_int, [C.c_void_p, C.c_int32, _f32p, _f32p]),
    "bs_stack_plan": (C.c_int, [C.c_void_p, C.POINTER(bs_plan_options)]),
    "bs_stack_plan_info": (C.c_int, [C.c_void_p, C.POINTER(bs_plan_info)]),
    "bs_stack_step_info": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(bs_step_info)]),
    "bs_stack_sequence_info": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(bs_sequence_info)]),
    "bs_stack_operation_name": (C.c_char_p, [C.c_void_p, C.c_int32]),
    "bs_stack_workspace_bytes": (C.c_uint64, [C.c_void_p]),
    "bs_stack_run": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p), C.c_void_p,
                               C.POINTER(C.c_void_p), C.c_void_p, C.c_uint64, C.c_void_p]),
    "bs_stack_run_static": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p), C.c_void_p,
                                      C.POINTER(C.c_void_p), C.c_void_p]),
    "bs_static_workspace_capacity": (C.c_uint64, []),
    "bs_stack_run_strided": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.POINTER(C.c_void_p), C.c_void_p,
                                       C.c_int64, C.POINTER(C.c_void_p), C.c_void_p, C.c_uint64, C.c_void_p]),
    "bs_stack_check_buffers": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.POINTER(C.c_void_p), C.c_void_p,
                                         C.c_int64, C.POINTER(C.c_void_p), C.c_void_p, C.c_uint64]),
    "bs_stack_plan_backward": (C.c_int, [C.c_void_p]),
    "bs_stack_backward_workspace_bytes": (C.c_uint64, [C.c_void_p]),
    "bs_stack_backward_num_stages": (C.c_int32, [C.c_void_p]),
    "bs_stack_backward": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_void_p,
                                    C.c_void_p, C.POINTER(C.c_void_p), C.c_void_p, C.c_uint64, C.c_void_p]),
    "bs_stack_backward_strided": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                            C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.POINTER(C.c_void_p), C.c_void_p,
                                            C.c_uint64, C.c_void_p]),
    "bs_probe_issue_rate": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_uint64, C.c_void_p]),
    "bs_probe_stream": (C.c_int, [C.c_int32, C.c_int32, C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64, C.c_void_p]),
    "bs_stack_jit_check": (C.c_int, [C.c_void_p, C.c_char_p, C.POINTER(C.c_int32)]),
    "bs_jit_log": (C.c_char_p, []),
    "bs_status_string": (C.c_char_p, [C.c_int]),
    "bs_version": (C.c_char_p, []),
    "bs_last_hip_error": (C.c_int32, []),
}
EXPORTS = tuple(_SIGNATURES)


def load():
    """Load the built library; raises (never falls back) when it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
                "or `python paper_1804_08378_amd/build.py`")
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


class BrainSlugError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        msg = load().bs_status_string(self.status).decode()
        extra = ""
        if self.status == 9:
            extra = f" (hipError_t {load().bs_last_hip_error()})"
        if self.status == 13:
            extra = "\n" + load().bs_jit_log().decode(errors="replace")[-4000:]
        super().__init__(f"{where}: {STATUS_NAMES.get(self.status, self.status)}: {msg}{extra}")


def _check(status: int, where: str):
    if status != BS_OK:
        raise BrainSlugError(status, where)


# ---- same-name forwarding functions ---------------------------------------------------
def bs_version() -> str:
    return load().bs_version().decode()


def bs_status_string(status: int) -> str:
    return load().bs_status_string(int(status)).decode()


def bs_last_hip_error() -> int:
    return int(load().bs_last_hip_error())


def bs_jit_log() -> str:
    return load().bs_jit_log().decode(errors="replace")


def bs_stack_jit_check(handle, arch: str = "gfx950") -> int:
    """Compile (only) the plan's run-time builds for `arch`; returns how many were compiled."""
    n = C.c_int32(0)
    _check(load().bs_stack_jit_check(C.c_void_p(handle), arch.encode(), C.byref(n)), "bs_stack_jit_check")
    return int(n.value)


def _shape4(shape):
    if len(shape) != 4:
        raise ValueError("expected an NCHW shape")
    return (C.c_int64 * 4)(*[int(v) for v in shape])


def _marshal_layers(layers, channels):
    """layer dicts (see workloads) -> (ctypes array, keep-alive list)."""
    arr = (bs_layer_desc * max(1, len(layers)))()
    keep = []
    for i, l in enumerate(layers):
        d = arr[i]
        kind = l["kind"]
        if kind == "bn":
            d.kind = BS_BATCHNORM
            d.eps = float(l["eps"])
            for field, key in (("gamma", "gamma"), ("beta", "beta"), ("running_mean", "mean"),
                               ("running_var", "var")):
                a = np.ascontiguousarray(l[key], dtype=np.float32)
                if a.size != channels:
                    raise ValueError("BatchNorm parameter length must equal C")
                keep.append(a)
                setattr(d, field, a.ctypes.data_as(_f32p))
        elif kind == "relu":
            d.kind = BS_RELU
        elif kind == "add":
            d.kind = BS_ADD
        elif kind == "leaky_relu":
            d.kind = BS_LEAKY_RELU
            d.negative_slope = float(l["slope"])
        elif kind == "clamp":
            d.kind = BS_CLAMP
            d.clamp_min, d.clamp_max = float(l["lo"]), float(l["hi"])
        elif kind in ("maxpool", "avgpool"):
            d.kind = BS_MAXPOOL if kind == "maxpool" else BS_AVGPOOL
            d.kh, d.kw = l["k"]
            d.sh, d.sw = l["s"]
            d.ph, d.pw = l["p"]
            d.count_include_pad = 1 if l.get("count_include_pad", True) else 0
            d.return_indices = 1 if l.get("return_indices", False) else 0
            d.ceil_mode = 1 if l.get("ceil_mode", False) else 0
            dil = l.get("dilation", (1, 1))
            d.dilation_h, d.dilation_w = dil
        else:
            raise ValueError(f"unknown layer kind {kind!r}")
    return arr, keep


def bs_stack_create(layers, in_shape, dtype) -> int:
    """Returns the opaque handle (an int).  `dtype` is BS_F32/BS_BF16 or "f32"/"bf16"."""
    dt = {"f32": BS_F32, "bf16": BS_BF16, "f16": BS_F16}.get(dtype, dtype)
    arr, keep = _marshal_layers(layers, int(in_shape[1]))
    h = C.c_void_p()
    _check(load().bs_stack_create(arr, len(layers), _shape4(in_shape), int(dt), C.byref(h)),
           "bs_stack_create")
    del keep
    return h.value


def bs_stack_destroy(handle) -> None:
    load().bs_stack_destroy(C.c_void_p(handle))


def bs_stack_output_shape(handle):
    out = (C.c_int64 * 4)()
    _check(load().bs_stack_output_shape(C.c_void_p(handle), out), "bs_stack_output_shape")
    return tuple(out)


def bs_stack_num_residuals(handle) -> int:
    return int(load().bs_stack_num_residuals(C.c_void_p(handle)))


def bs_stack_residual_shape(handle, i):
    out = (C.c_int64 * 4)()
    _check(load().bs_stack_residual_shape(C.c_void_p(handle), int(i), out), "bs_stack_residual_shape")
    return tuple(out)


def bs_stack_num_index_outputs(handle) -> int:
    return int(load().bs_stack_num_index_outputs(C.c_void_p(handle)))


def bs_stack_index_shape(handle, i):
    out = (C.c_int64 * 4)()
    _check(load().bs_stack_index_shape(C.c_void_p(handle), int(i), out), "bs_stack_index_shape")
    return tuple(out)


def bs_stack_folded_bn(handle, layer, channels):
    scale = np.empty(channels, np.float32)
    shift = np.empty(channels, np.float32)
    _check(load().bs_stack_folded_bn(C.c_void_p(handle), int(layer), scale.ctypes.data_as(_f32p),
                                     shift.ctypes.data_as(_f32p)), "bs_stack_folded_bn")
    return scale, shift


def bs_stack_plan(handle, **opts) -> None:
    o = bs_plan_options()
    for k, v in opts.items():
        if not hasattr(o, k) or k == "reserved":
            raise TypeError(f"unknown plan option {k!r}")
        setattr(o, k, int(v))
    _check(load().bs_stack_plan(C.c_void_p(handle), C.byref(o) if opts else None), "bs_stack_plan")


def _struct_dict(s):
    out = {}
    for name, _ in s._fields_:
        v = getattr(s, name)
        out[name] = tuple(v) if hasattr(v, "__len__") else v
    return out


def bs_stack_plan_info(handle) -> dict:
    info = bs_plan_info()
    _check(load().bs_stack_plan_info(C.c_void_p(handle), C.byref(info)), "bs_stack_plan_info")
    return _struct_dict(info)


def bs_stack_step_info(handle, step) -> dict:
    info = bs_step_info()
    _check(load().bs_stack_step_info(C.c_void_p(handle), int(step), C.byref(info)), "bs_stack_step_info")
    return _struct_dict(info)


def bs_stack_sequence_info(handle, seq) -> dict:
    info = bs_sequence_info()
    _check(load().bs_stack_sequence_info(C.c_void_p(handle), int(seq), C.byref(info)),
           "bs_stack_sequence_info")
    d = _struct_dict(info)
    d["variant_name"] = VARIANT_NAMES.get(d["variant"], "?")
    return d


def bs_stack_operation_name(handle, op):
    r = load().bs_stack_operation_name(C.c_void_p(handle), int(op))
    return r.decode() if r else None


def bs_stack_workspace_bytes(handle) -> int:
    return int(load().bs_stack_workspace_bytes(C.c_void_p(handle)))


def bs_stack_run(handle, in_ptr, residual_ptrs, out_ptr, index_ptrs, workspace_ptr, workspace_bytes,
                 stream) -> None:
    """All *_ptr arguments are integer device addresses (0 / None = NULL)."""
    res = None
    if residual_ptrs:
        res = (C.c_void_p * len(residual_ptrs))(*[C.c_void_p(p or None) for p in residual_ptrs])
    idx = None
    if index_ptrs:
        idx = (C.c_void_p * len(index_ptrs))(*[C.c_void_p(p or None) for p in index_ptrs])
    _check(load().bs_stack_run(C.c_void_p(handle), C.c_void_p(in_ptr or None), res,
                               C.c_void_p(out_ptr or None), idx, C.c_void_p(workspace_ptr or None),
                               int(workspace_bytes), C.c_void_p(stream or None)), "bs_stack_run")


def bs_stack_run_static(handle, in_ptr, residual_ptrs, out_ptr, index_ptrs, stream) -> None:
    """bs_stack_run on the library's own static workspace; *_ptr are integer device addresses."""
    res = None
    if residual_ptrs:
        res = (C.c_void_p * len(residual_ptrs))(*[C.c_void_p(p or None) for p in residual_ptrs])
    idx = None
    if index_ptrs:
        idx = (C.c_void_p * len(index_ptrs))(*[C.c_void_p(p or None) for p in index_ptrs])
    _check(load().bs_stack_run_static(C.c_void_p(handle), C.c_void_p(in_ptr or None), res,
                                      C.c_void_p(out_ptr or None), idx, C.c_void_p(stream or None)),
           "bs_stack_run_static")


def bs_static_workspace_capacity() -> int:
    return int(load().bs_static_workspace_capacity())


PROBE_KINDS = {"add": 0, "fma": 1, "max3": 2, "select_vcc": 3, "select_sgpr": 4, "lane_shift": 5, "add_scalar": 6,
               "add_branch": 7, "dependent_add": 8}


def bs_probe_stream(reads_per_write: int, read_only: bool, in_ptr: int, in_bytes: int, out_ptr: int, out_bytes: int, stream) -> None:
    """Enqueue the streaming probe (no arithmetic); *_ptr are integer device addresses."""
    _check(load().bs_probe_stream(int(reads_per_write), int(bool(read_only)), C.c_void_p(in_ptr or None), int(in_bytes),
                                  C.c_void_p(out_ptr or None), int(out_bytes), C.c_void_p(stream or None)), "bs_probe_stream")


def bs_probe_issue_rate(kind: int, waves_per_simd: int, iterations: int, sink_ptr: int, sink_floats: int, stream) -> None:
    _check(load().bs_probe_issue_rate(int(kind), int(waves_per_simd), int(iterations), C.c_void_p(sink_ptr or None),
                                      int(sink_floats), C.c_void_p(stream or None)), "bs_probe_issue_rate")


def bs_stack_plan_backward(handle) -> None:
    _check(load().bs_stack_plan_backward(C.c_void_p(handle)), "bs_stack_plan_backward")


def bs_stack_backward_workspace_bytes(handle) -> int:
    return int(load().bs_stack_backward_workspace_bytes(C.c_void_p(handle)))


def bs_stack_backward_num_stages(handle) -> int:
    return int(load().bs_stack_backward_num_stages(C.c_void_p(handle)))


def bs_stack_backward(handle, in_ptr, residual_ptrs, index_ptrs, grad_out_ptr, grad_in_ptr, grad_residual_ptrs,
                      workspace_ptr, workspace_bytes, stream) -> None:
    """All *_ptr arguments are integer device addresses (0 / None = NULL: that gradient is not wanted, those
    saved indices are not there)."""
    res = gres = idx = None
    if residual_ptrs:
        res = (C.c_void_p * len(residual_ptrs))(*[C.c_void_p(p or None) for p in residual_ptrs])
    if index_ptrs:
        idx = (C.c_void_p * len(index_ptrs))(*[C.c_void_p(p or None) for p in index_ptrs])
    if grad_residual_ptrs:
        gres = (C.c_void_p * len(grad_residual_ptrs))(*[C.c_void_p(p or None) for p in grad_residual_ptrs])
    _check(load().bs_stack_backward(C.c_void_p(handle), C.c_void_p(in_ptr or None), res, idx,
                                    C.c_void_p(grad_out_ptr or None), C.c_void_p(grad_in_ptr or None), gres,
                                    C.c_void_p(workspace_ptr or None), int(workspace_bytes), C.c_void_p(stream or None)),
           "bs_stack_backward")


def bs_stack_backward_strided(handle, in_ptr, in_batch_stride, residual_ptrs, index_ptrs, grad_out_ptr, grad_out_batch_stride,
                              grad_in_ptr, grad_in_batch_stride, grad_residual_ptrs, workspace_ptr, workspace_bytes, stream) -> None:
    """bs_stack_backward on channel slices: batch strides in elements (0 = dense)."""
    res = gres = idx = None
    if residual_ptrs:
        res = (C.c_void_p * len(residual_ptrs))(*[C.c_void_p(p or None) for p in residual_ptrs])
    if index_ptrs:
        idx = (C.c_void_p * len(index_ptrs))(*[C.c_void_p(p or None) for p in index_ptrs])
    if grad_residual_ptrs:
        gres = (C.c_void_p * len(grad_residual_ptrs))(*[C.c_void_p(p or None) for p in grad_residual_ptrs])
    _check(load().bs_stack_backward_strided(C.c_void_p(handle), C.c_void_p(in_ptr or None), int(in_batch_stride), res, idx,
                                            C.c_void_p(grad_out_ptr or None), int(grad_out_batch_stride),
                                            C.c_void_p(grad_in_ptr or None), int(grad_in_batch_stride), gres,
                                            C.c_void_p(workspace_ptr or None), int(workspace_bytes), C.c_void_p(stream or None)),
           "bs_stack_backward_strided")


def bs_stack_run_strided(handle, in_ptr, in_batch_stride, residual_ptrs, out_ptr, out_batch_stride,
                         index_ptrs, workspace_ptr, workspace_bytes, stream) -> None:
    """bs_stack_run on channel slices: batch strides in elements (0 = dense)."""
    res = None
    if residual_ptrs:
        res = (C.c_void_p * len(residual_ptrs))(*[C.c_void_p(p or None) for p in residual_ptrs])
    idx = None
    if index_ptrs:
        idx = (C.c_void_p * len(index_ptrs))(*[C.c_void_p(p or None) for p in index_ptrs])
    _check(load().bs_stack_run_strided(C.c_void_p(handle), C.c_void_p(in_ptr or None), int(in_batch_stride),
                                       res, C.c_void_p(out_ptr or None), int(out_batch_stride), idx,
                                       C.c_void_p(workspace_ptr or None), int(workspace_bytes),
                                       C.c_void_p(stream or None)), "bs_stack_run_strided")


def bs_stack_check_buffers(handle, in_ptr, in_batch_stride, residual_ptrs, out_ptr, out_batch_stride,
                           index_ptrs, workspace_ptr, workspace_bytes) -> int:
    """The bs_status bs_stack_run_strided's argument checks give (no launch, no device); returned,
    not raised."""
    res = None
    if residual_ptrs:
        res = (C.c_void_p * len(residual_ptrs))(*[C.c_void_p(p or None) for p in residual_ptrs])
    idx = None
    if index_ptrs:
        idx = (C.c_void_p * len(index_ptrs))(*[C.c_void_p(p or None) for p in index_ptrs])
    return int(load().bs_stack_check_buffers(C.c_void_p(handle), C.c_void_p(in_ptr or None), int(in_batch_stride),
                                             res, C.c_void_p(out_ptr or None), int(out_batch_stride), idx,
                                             C.c_void_p(workspace_ptr or None), int(workspace_bytes)))


def batch_stride(t):
    """Batch stride (elements) of a 4-D tensor that is dense in C, H, W -- a contiguous tensor
    or a slice of one along the channel axis -- else None."""
    n, c, h, w = t.shape
    sn, sc, sh, sw = t.stride()
    if (w == 1 or sw == 1) and (h == 1 or sh == w) and (c == 1 or sc == h * w) and (n == 1 or sn >= c * h * w):
        return int(sn) if n > 1 else c * h * w
    return None


def batch_stride_nhwc(t):
    """Batch stride (elements) of a 4-D channels-last tensor that holds its channels contiguously
    in every pixel of a tensor with at least as many channels -- a channels_last tensor or a
    slice of one along the channel axis -- else None."""
    n, c, h, w = t.shape
    sn, sc, sh, sw = t.stride()
    ct = sw if w > 1 else (sh if h > 1 else (sn if n > 1 else c))  # channels of the larger tensor
    if ct >= c and (c == 1 or sc == 1) and (w == 1 or sw == ct) and (h == 1 or sh == w * ct) and \
            (n == 1 or sn == h * w * ct):
        return int(h * w * ct)
    return None


# ---- convenience wrapper -----------------------------------------------------------------
class Stack:
    """A planned stack bound to torch tensors (device memory and streams only)."""

    def __init__(self, layers, in_shape, dtype="f32"):
        self.dtype = dtype
        self.in_shape = tuple(int(v) for v in in_shape)
        self.handle = bs_stack_create(layers, self.in_shape, dtype)
        self.out_shape = bs_stack_output_shape(self.handle)
        self.n_res = bs_stack_num_residuals(self.handle)
        self.n_idx = bs_stack_num_index_outputs(self.handle)
        self.res_shapes = [bs_stack_residual_shape(self.handle, i) for i in range(self.n_res)]
        self.idx_shapes = [bs_stack_index_shape(self.handle, i) for i in range(self.n_idx)]
        self._workspace = None
        self._workspace_bytes = 0
        self._fast = None
        self._bwd_workspace = None
        self._bwd_planned = False
        self.layout = BS_LAYOUT_NCHW

    def close(self):
        # also runs as __del__, possibly while the interpreter shuts down and module globals are gone
        if getattr(self, "handle", None) and bs_stack_destroy is not None:
            bs_stack_destroy(self.handle)
            self.handle = None

    __del__ = close

    def plan(self, **opts):
        bs_stack_plan(self.handle, **opts)
        self.layout = int(opts.get("layout", BS_LAYOUT_NCHW))
        self._workspace = None
        self._fast = None
        self._workspace_bytes = bs_stack_workspace_bytes(self.handle)
        self._bwd_workspace = None
        self._bwd_planned = False
        return self

    def plan_backward(self):
        """Plan the backward pass (after `plan`; for the plan's memory layout)."""
        bs_stack_plan_backward(self.handle)
        self._bwd_planned = True
        self._bwd_workspace = None
        self._bwd_workspace_bytes = bs_stack_backward_workspace_bytes(self.handle)
        return self

    def backward(self, x, residuals, grad_out, need_input_grad=True, need_residual_grads=None, stream=None, indices=None):
        """Enqueue the backward pass; returns (grad_x or None, [grad_residual or None, ...]).
        `indices`: the index outputs `run` wrote for this `x` (entries may be None), which save
        recomputing the last pooling layer's picks.
        `x` and `residuals` are the forward pass's operands, `grad_out` the gradient with respect
        to its output; all dense tensors of the stack's dtype in the plan's memory layout (the
        gradients come back in that layout)."""
        import torch
        if not getattr(self, "_bwd_planned", False):
            self.plan_backward()
        dt = self.torch_dtype()
        mf = torch.channels_last if self.layout == BS_LAYOUT_NHWC else torch.contiguous_format
        if tuple(x.shape) != self.in_shape or x.dtype != dt or not x.is_contiguous(memory_format=mf):
            raise ValueError("x must be a dense tensor of the stack's input shape, dtype and memory layout")
        if tuple(grad_out.shape) != self.out_shape or grad_out.dtype != dt or not grad_out.is_contiguous(memory_format=mf):
            raise ValueError("grad_out must be a dense tensor of the stack's output shape, dtype and memory layout")
        if len(residuals) != self.n_res:
            raise ValueError(f"the stack has {self.n_res} residual operands")
        for i, r in enumerate(residuals):
            if tuple(r.shape) != self.res_shapes[i] or r.dtype != dt or not r.is_contiguous(memory_format=mf):
                raise ValueError("residuals must be dense tensors of their Add layer's shape, the stack's dtype and memory layout")
        need_res = [True] * self.n_res if need_residual_grads is None else list(need_residual_grads)
        gx = torch.empty_like(x, memory_format=mf) if need_input_grad else None
        gres = [torch.empty_like(r, memory_format=mf) if need else None for r, need in zip(residuals, need_res)]
        n = self._bwd_workspace_bytes
        st = stream if stream is not None else torch.cuda.current_stream(x.device).cuda_stream
        ws = self.workspace(x.device, st, backward=True)
        if indices is not None:
            if len(indices) != self.n_idx:
                raise ValueError(f"the stack has {self.n_idx} index outputs")
            for i, t in enumerate(indices):
                if t is not None and (tuple(t.shape) != self.idx_shapes[i] or t.dtype != torch.int32 or
                                      not t.is_contiguous(memory_format=mf)):
                    raise ValueError("saved indices must be the int32 index outputs of run()")
        idx = [t.data_ptr() if t is not None else 0 for t in indices] if indices else None
        bs_stack_backward(self.handle, x.data_ptr(), [r.data_ptr() for r in residuals], idx, grad_out.data_ptr(),
                          gx.data_ptr() if gx is not None else 0, [g.data_ptr() if g is not None else 0 for g in gres],
                          ws.data_ptr() if ws is not None else 0, n, st)
        return gx, gres

    def info(self) -> dict:
        p = bs_stack_plan_info(self.handle)
        p["operations"] = [bs_stack_operation_name(self.handle, i) for i in range(p["n_operations"])]
        p["steps"] = [bs_stack_step_info(self.handle, i) for i in range(p["n_steps"])]
        p["sequences"] = [bs_stack_sequence_info(self.handle, i) for i in range(p["n_sequences"])]
        return p

    def torch_dtype(self):
        import torch
        if self.dtype in ("f32", BS_F32):
            return torch.float32
        return torch.bfloat16 if self.dtype in ("bf16", BS_BF16) else torch.float16

    def alloc_outputs(self, device="cuda", indices=True):
        import torch
        mf = torch.channels_last if self.layout == BS_LAYOUT_NHWC else torch.contiguous_format
        out = torch.empty(self.out_shape, dtype=self.torch_dtype(), device=device, memory_format=mf)
        idx = [torch.empty(self.idx_shapes[i], dtype=torch.int32, device=device, memory_format=mf)
               for i in range(self.n_idx)] if indices else []
        return out, idx

    def workspace(self, device="cuda", stream=None, backward=False):
        """The workspace for launches on `stream` (a raw stream handle; None: torch's current
        stream): one buffer per stream, because the library's promise that runs on different
        streams may overlap holds only when they do not share the buffer the sequences hand
        their intermediate tensors through."""
        import torch
        n = self._bwd_workspace_bytes if backward else self._workspace_bytes
        if not n:
            return None
        dev = torch.device(device)
        if stream is None:
            stream = torch.cuda.current_stream(dev).cuda_stream
        cache = self._bwd_workspace if backward else self._workspace
        if cache is None:
            cache = {}
            if backward:
                self._bwd_workspace = cache
            else:
                self._workspace = cache
        key = (dev.index if dev.index is not None else torch.cuda.current_device(), int(stream or 0))
        ws = cache.get(key)
        if ws is None or ws.numel() < n:
            ws = cache[key] = torch.empty(n, dtype=torch.uint8, device=dev)
        return ws

    def run(self, x, residuals=(), out=None, indices=None, stream=None):
        """Enqueue on `stream` (default: torch's current stream); returns (out, indices).
        `x` and `out` may be channel slices (t[:, a:b]) of larger contiguous tensors: they are
        read and written in place."""
        import torch
        if self.layout == BS_LAYOUT_NHWC:
            return self._run_nhwc(x, residuals, out, indices, stream)
        if tuple(x.shape) != self.in_shape or x.dtype != self.torch_dtype() or batch_stride(x) is None:
            raise ValueError("input must be a tensor of the stack's shape and dtype, contiguous or a "
                             "channel slice of a contiguous tensor")
        for r in residuals:
            if r.dtype != self.torch_dtype() or not r.is_contiguous():
                raise ValueError("residuals must be contiguous tensors of the stack's dtype")
        if out is None or indices is None:
            o2, i2 = self.alloc_outputs(x.device, indices is None)
            out = o2 if out is None else out
            indices = i2 if indices is None else indices
        if tuple(out.shape) != self.out_shape or out.dtype != self.torch_dtype() or batch_stride(out) is None:
            raise ValueError("out must be a tensor of the stack's output shape and dtype, contiguous or a "
                             "channel slice of a contiguous tensor")
        st = stream if stream is not None else torch.cuda.current_stream(x.device).cuda_stream
        ws = self.workspace(x.device, st)
        res = [r.data_ptr() for r in residuals]
        idx = [t.data_ptr() if t is not None else 0 for t in indices] if indices else None
        wsp, wsn = (ws.data_ptr(), ws.numel()) if ws is not None else (0, 0)
        if x.is_contiguous() and out.is_contiguous():
            bs_stack_run(self.handle, x.data_ptr(), res, out.data_ptr(), idx, wsp, wsn, st)
        else:
            bs_stack_run_strided(self.handle, x.data_ptr(), batch_stride(x), res, out.data_ptr(),
                                 batch_stride(out), idx, wsp, wsn, st)
        return out, indices

    def run_unchecked(self, x, residuals, out, in_batch_stride=0, out_batch_stride=0, indices=None):
        """`bs_stack_run_strided` with as little Python in the way as possible (`indices`: None, or one
        int32 tensor of the plan's layout per index output;
        the residuals dense tensors of the plan's layout; `x` / `out` dense, or channel slices with
        `in_batch_stride` / `out_batch_stride` elements between their images): for callers that have validated
        shapes, dtypes and layouts themselves -- the front-end does, once per call.  The library
        still checks alignment, aliasing and the workspace."""
        import torch
        fast = self._fast
        if fast is None:
            lib = load()
            fast = self._fast = (lib.bs_stack_run_strided, C.c_void_p(self.handle),
                                 C.c_void_p * max(1, self.n_res), self._workspace_bytes,
                                 getattr(torch._C, "_cuda_getCurrentRawStream", None), x.device.index)
        fn, h, res_type, wsn, raw_stream, dev = fast
        # a fresh pointer array per call: the library reads it while the interpreter lock is released
        res = res_type(*[r.data_ptr() for r in residuals]) if residuals else None
        st = raw_stream(dev) if raw_stream is not None else torch.cuda.current_stream(x.device).cuda_stream
        wsp = self.workspace(x.device, st).data_ptr() if wsn else None  # one buffer per stream
        idx = (C.c_void_p * len(indices))(*[t.data_ptr() for t in indices]) if indices else None
        rc = fn(h, x.data_ptr(), in_batch_stride, res, out.data_ptr(), out_batch_stride, idx, wsp, wsn, st)
        if rc != 0:
            _check(rc, "bs_stack_run_strided")
        return out

    def backward_unchecked(self, x, residuals, grad_out, grad_x, grad_residuals, indices=None, in_batch_stride=0,
                           grad_out_batch_stride=0, grad_in_batch_stride=0):
        """`bs_stack_backward_strided` with as little Python in the way as possible: tensors of the plan's
        layout and the stack's dtype that the caller has validated and allocated (`grad_x` and entries
        of `grad_residuals` may be None: not wanted; `indices`: the forward pass's index outputs or
        None; batch strides in elements for `x`, `grad_out`, `grad_x` that are channel slices, 0 = dense).
        The library still checks strides, alignment, aliasing and the workspace."""
        import torch
        if not self._bwd_planned:
            self.plan_backward()
        n = self._bwd_workspace_bytes
        ptr = C.c_void_p * max(1, self.n_res)
        res = ptr(*[r.data_ptr() for r in residuals]) if residuals else None
        gres = ptr(*[g.data_ptr() if g is not None else None for g in grad_residuals]) if grad_residuals else None
        idx = (C.c_void_p * len(indices))(*[t.data_ptr() if t is not None else None for t in indices]) if indices else None
        raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)
        st = raw_stream(x.device.index) if raw_stream is not None else torch.cuda.current_stream(x.device).cuda_stream
        rc = load().bs_stack_backward_strided(self.handle, x.data_ptr(), in_batch_stride, res, idx, grad_out.data_ptr(),
                                              grad_out_batch_stride, grad_x.data_ptr() if grad_x is not None else None,
                                              grad_in_batch_stride, gres,
                                              self.workspace(x.device, st, backward=True).data_ptr() if n else None, n, st)
        if rc != 0:
            _check(rc, "bs_stack_backward_strided")

    def _run_nhwc(self, x, residuals, out, indices, stream):
        """A channels-last plan: every tensor is in torch's channels_last memory format."""
        import torch
        cl = torch.channels_last
        if tuple(x.shape) != self.in_shape or x.dtype != self.torch_dtype() or not x.is_contiguous(memory_format=cl):
            raise ValueError("input must be a channels_last tensor of the stack's shape and dtype")
        for r in residuals:
            if r.dtype != self.torch_dtype() or not r.is_contiguous(memory_format=cl):
                raise ValueError("residuals must be channels_last tensors of the stack's dtype")
        if out is None or indices is None:
            o2, i2 = self.alloc_outputs(x.device, indices is None)
            out = o2 if out is None else out
            indices = i2 if indices is None else indices
        if tuple(out.shape) != self.out_shape or out.dtype != self.torch_dtype() or \
                not out.is_contiguous(memory_format=cl):
            raise ValueError("out must be a channels_last tensor of the stack's output shape and dtype")
        for t in indices or []:
            if t is not None and not t.is_contiguous(memory_format=cl):
                raise ValueError("index outputs must be channels_last tensors")
        st = stream if stream is not None else torch.cuda.current_stream(x.device).cuda_stream
        ws = self.workspace(x.device, st)
        idx = [t.data_ptr() if t is not None else 0 for t in indices] if indices else None
        wsp, wsn = (ws.data_ptr(), ws.numel()) if ws is not None else (0, 0)
        bs_stack_run(self.handle, x.data_ptr(), [r.data_ptr() for r in residuals], out.data_ptr(), idx, wsp, wsn, st)
        return out, indices
