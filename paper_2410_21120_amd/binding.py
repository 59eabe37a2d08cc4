"""ctypes binding of include/fusedinf.h: argument marshalling only.

The fi_* functions below take and return exactly what the C entry points do.
`Dag` is a small convenience owner (keeps the borrowed spec memory alive, turns
a non-zero fi_status into an exception carrying fi_last_error()).  PyTorch is
used for device memory and streams only: `torch_allocators()` hands the
library torch-backed dev_alloc / pin_alloc callbacks.
"""
from __future__ import annotations

import ctypes as C
import os

from . import build as _build

FI_OK, FI_EINVAL, FI_EUNSUPPORTED, FI_ESTATE, FI_ENOMEM_HOST, FI_ENOMEM_DEVICE, FI_EBUDGET, FI_EHIP = range(8)
FI_F32, FI_BF16 = 0, 1
FI_CONV2D, FI_DWCONV2D, FI_MAXPOOL2D, FI_GLOBAL_AVGPOOL, FI_FC, FI_SOFTMAX, FI_CONCAT, FI_AVGPOOL2D, FI_MUL, FI_SLICE, FI_SHUFFLE = range(11)
FI_ACT_NONE, FI_ACT_RELU, FI_ACT_RELU6, FI_ACT_HARDSWISH, FI_ACT_HARDSIGMOID, FI_ACT_SILU, FI_ACT_SIGMOID = range(7)
FI_INPUT, FI_NO_RESIDUAL = -1, -2
FI_LOAD_ONE_COPY, FI_LOAD_PER_MODEL, FI_LOAD_AUTO = 0, 1, 2
FI_MAX_GROUP = 16
STATUS_NAMES = ["FI_OK", "FI_EINVAL", "FI_EUNSUPPORTED", "FI_ESTATE", "FI_ENOMEM_HOST", "FI_ENOMEM_DEVICE",
                "FI_EBUDGET", "FI_EHIP"]


class fi_layer_spec(C.Structure):
    _fields_ = [("op", C.c_int32), ("input", C.c_int32), ("residual", C.c_int32), ("cin", C.c_int32),
                ("cout", C.c_int32), ("kh", C.c_int32), ("kw", C.c_int32), ("stride", C.c_int32),
                ("pad", C.c_int32), ("act", C.c_int32), ("ceil_mode", C.c_int32), ("groups", C.c_int32),
                ("c_first", C.c_int32), ("reserved", C.c_int32), ("w_off", C.c_uint64), ("b_off", C.c_uint64)]


class fi_model_spec(C.Structure):
    _fields_ = [("name", C.c_char_p), ("dtype", C.c_int32), ("act_dtype", C.c_int32), ("in_c", C.c_int32),
                ("in_h", C.c_int32), ("in_w", C.c_int32), ("n_layers", C.c_int32),
                ("layers", C.POINTER(fi_layer_spec)), ("output_node", C.c_int32), ("weights_packed", C.c_int32),
                ("weights", C.c_void_p), ("weight_bytes", C.c_uint64)]


ALLOC_FN = C.CFUNCTYPE(C.c_void_p, C.c_size_t, C.c_void_p)
FREE_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p)


class fi_build_opts(C.Structure):
    _fields_ = [("max_batch", C.c_int32), ("group_levels", C.c_int32), ("load_mode", C.c_int32),
                ("use_graph", C.c_int32), ("serial_lanes", C.c_int32), ("per_member_inputs", C.c_int32),
                ("max_device_bytes", C.c_uint64), ("dev_alloc", ALLOC_FN),
                ("dev_free", FREE_FN), ("pin_alloc", ALLOC_FN), ("pin_free", FREE_FN), ("user", C.c_void_p),
                ("swap_headroom_bytes", C.c_uint64), ("copy_concats", C.c_int32), ("separate_affine", C.c_int32),
                ("separate_chains", C.c_int32), ("member_chunks", C.c_int32), ("separate_stem", C.c_int32),
                ("reserved0", C.c_int32)]


class fi_dag_info(C.Structure):
    _fields_ = [("arena_bytes", C.c_uint64), ("act_bytes", C.c_uint64), ("workspace_bytes", C.c_uint64),
                ("device_bytes", C.c_uint64), ("macs_per_image", C.c_uint64), ("n_models", C.c_int32),
                ("n_nodes", C.c_int32), ("n_levels", C.c_int32), ("n_launches", C.c_int32),
                ("n_device_allocs", C.c_int32), ("n_h2d_copies", C.c_int32), ("state", C.c_int32),
                ("n_lanes", C.c_int32), ("device_capacity", C.c_uint64), ("last_h2d_bytes", C.c_uint64),
                ("last_h2d_copies", C.c_int32), ("reserved", C.c_int32), ("input_image_bytes", C.c_uint64)]


class fi_sched_opts(C.Structure):
    _fields_ = [("iterations", C.c_int32), ("rounds", C.c_int32), ("overlap_load", C.c_int32), ("reserved", C.c_int32)]


class fi_sched_stats(C.Structure):
    _fields_ = [("build_ms", C.c_double), ("total_ms", C.c_double), ("run_ms", C.c_double), ("swap_ms", C.c_double),
                ("peak_device_bytes", C.c_uint64), ("n_loads", C.c_int32), ("n_runs", C.c_int32),
                ("n_groups", C.c_int32), ("reserved", C.c_int32)]


class fi_server_opts(C.Structure):
    _fields_ = [("max_wait_us", C.c_int32), ("reserved", C.c_int32)]


class fi_server_stats(C.Structure):
    _fields_ = [("requests", C.c_uint64), ("passes", C.c_uint64), ("max_images_per_pass", C.c_uint64),
                ("mean_images_per_pass", C.c_double), ("mean_latency_ms", C.c_double), ("max_latency_ms", C.c_double),
                ("busy_ms", C.c_double)]


class fi_member_info(C.Structure):
    _fields_ = [("arena_off", C.c_uint64), ("packed_bytes", C.c_uint64), ("lane", C.c_int32),
                ("first_node", C.c_int32), ("n_nodes", C.c_int32), ("reserved", C.c_int32), ("output_row_bytes", C.c_uint64)]


class fi_node_info(C.Structure):
    _fields_ = [("model", C.c_int32), ("index", C.c_int32), ("op", C.c_int32), ("level", C.c_int32),
                ("launch", C.c_int32), ("out_c", C.c_int32), ("out_h", C.c_int32), ("out_w", C.c_int32),
                ("out_cp", C.c_int32), ("out_dtype", C.c_int32), ("is_output", C.c_int32),
                ("first_level", C.c_int32), ("last_level", C.c_int32), ("out_off", C.c_uint64),
                ("out_bytes", C.c_uint64), ("w_off", C.c_uint64), ("b_off", C.c_uint64), ("macs", C.c_uint64)]


class fi_launch_info(C.Structure):
    _fields_ = [("level", C.c_int32), ("kind", C.c_int32), ("n_problems", C.c_int32), ("first_node", C.c_int32),
                ("lane", C.c_int32), ("reserved", C.c_int32), ("macs_per_image", C.c_uint64), ("bytes_per_image", C.c_uint64), ("weight_bytes", C.c_uint64),
                ("name", C.c_char * 32)]


LIB_PATH = _build.OUT
EXPORTS = ["fi_model_packed_size", "fi_model_pack", "fi_build_dag", "fi_footprint", "fi_partition", "fi_round_robin", "fi_query", "fi_node", "fi_launch", "fi_member", "fi_load",
           "fi_run", "fi_run_static", "fi_run_inputs", "fi_run_batches", "fi_run_lane", "fi_profile", "fi_timeline", "fi_swap_model", "fi_server_start", "fi_server_submit", "fi_server_wait", "fi_server_query", "fi_server_swap", "fi_server_stop",
           "fi_unload", "fi_destroy", "fi_last_error", "fi_version"]
_lib = None


def lib():
    """Loads the built library; builds it first only when no build exists.  Raises if it cannot be loaded."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            _build.build()
        # One HIP runtime per process: PyTorch (which owns the device memory and the streams we are
        # handed) ships its own libamdhip64; import it first so the library binds to that same runtime
        # instead of pulling a second copy in from the system ROCm.
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp, i32, u64 = C.c_void_p, C.c_int32, C.c_uint64
        L.fi_model_packed_size.argtypes = [C.POINTER(fi_model_spec), C.POINTER(u64)]
        L.fi_model_pack.argtypes = [C.POINTER(fi_model_spec), vp, u64]
        L.fi_build_dag.argtypes = [C.POINTER(fi_model_spec), i32, C.POINTER(fi_build_opts), C.POINTER(vp)]
        L.fi_query.argtypes = [vp, C.POINTER(fi_dag_info)]
        L.fi_node.argtypes = [vp, i32, C.POINTER(fi_node_info)]
        L.fi_launch.argtypes = [vp, i32, C.POINTER(fi_launch_info)]
        L.fi_load.argtypes = [vp, vp]
        L.fi_run.argtypes = [vp, vp, i32, C.POINTER(vp), vp]
        L.fi_run_static.argtypes = [vp, vp, i32, C.POINTER(vp), vp]
        L.fi_run_inputs.argtypes = [vp, C.POINTER(vp), i32, C.POINTER(vp), vp]
        L.fi_run_batches.argtypes = [vp, C.POINTER(vp), C.POINTER(i32), C.POINTER(vp), vp]
        L.fi_run_lane.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(i32), C.POINTER(vp), vp]
        L.fi_profile.argtypes = [vp, vp, i32, C.POINTER(vp), vp, C.POINTER(C.c_float), i32]
        L.fi_timeline.argtypes = [vp, vp, i32, C.POINTER(vp), vp, C.POINTER(C.c_float), C.POINTER(C.c_float), i32]
        L.fi_footprint.argtypes = [C.POINTER(fi_model_spec), i32, C.POINTER(fi_build_opts), C.POINTER(fi_dag_info)]
        L.fi_partition.argtypes = [C.POINTER(fi_model_spec), i32, C.POINTER(fi_build_opts), C.c_uint64, C.POINTER(i32), C.POINTER(i32)]
        L.fi_round_robin.argtypes = [C.POINTER(fi_model_spec), i32, C.POINTER(fi_build_opts), C.POINTER(i32), i32,
                                     C.POINTER(fi_sched_opts), vp, i32, C.POINTER(vp), vp, C.POINTER(fi_sched_stats)]
        L.fi_swap_model.argtypes = [vp, i32, C.POINTER(fi_model_spec), vp]
        L.fi_member.argtypes = [vp, i32, C.POINTER(fi_member_info)]
        L.fi_server_start.argtypes = [vp, C.POINTER(fi_server_opts), C.POINTER(vp)]
        L.fi_server_submit.argtypes = [vp, i32, vp, vp, C.POINTER(u64)]
        L.fi_server_wait.argtypes = [vp, u64]
        L.fi_server_query.argtypes = [vp, C.POINTER(fi_server_stats)]
        L.fi_server_stop.argtypes = [vp]
        L.fi_server_swap.argtypes = [vp, i32, C.POINTER(fi_model_spec)]
        L.fi_unload.argtypes = [vp]
        L.fi_destroy.argtypes = [vp]
        L.fi_destroy.restype = None
        L.fi_last_error.restype = C.c_char_p
        L.fi_version.restype = C.c_char_p
        for name in EXPORTS:
            getattr(L, name)
        _lib = L
    return _lib


class FiError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().fi_last_error().decode(errors="replace")
        super().__init__(f"{where}: {STATUS_NAMES[status] if 0 <= status < 8 else status}: {msg}")


def _check(st, where):
    if st != FI_OK:
        raise FiError(st, where)


# ---- the entry points, same names as the header --------------------------------------------
def fi_last_error() -> str:
    return lib().fi_last_error().decode(errors="replace")


def fi_version() -> str:
    return lib().fi_version().decode()


def fi_model_packed_size(spec: fi_model_spec) -> int:
    n = C.c_uint64(0)
    _check(lib().fi_model_packed_size(C.byref(spec), C.byref(n)), "fi_model_packed_size")
    return n.value


def fi_model_pack(spec: fi_model_spec, dst_ptr: int, dst_bytes: int) -> None:
    _check(lib().fi_model_pack(C.byref(spec), C.c_void_p(dst_ptr), dst_bytes), "fi_model_pack")


def fi_build_dag(specs, opts: fi_build_opts) -> int:
    arr = (fi_model_spec * len(specs))(*specs)
    h = C.c_void_p(0)
    _check(lib().fi_build_dag(arr, len(specs), C.byref(opts), C.byref(h)), "fi_build_dag")
    return h.value


def fi_footprint(specs, opts: fi_build_opts) -> fi_dag_info:
    arr = (fi_model_spec * len(specs))(*specs)
    info = fi_dag_info()
    _check(lib().fi_footprint(arr, len(specs), C.byref(opts), C.byref(info)), "fi_footprint")
    return info


def fi_partition(specs, opts: fi_build_opts, budget_bytes):
    arr = (fi_model_spec * len(specs))(*specs)
    group_of = (C.c_int32 * len(specs))()
    n_groups = C.c_int32(0)
    _check(lib().fi_partition(arr, len(specs), C.byref(opts), budget_bytes, group_of, C.byref(n_groups)), "fi_partition")
    return list(group_of), n_groups.value


def fi_round_robin(specs, opts: fi_build_opts, group_of, n_groups, iterations, rounds, overlap_load,
                   d_input_ptr, batch, d_output_ptrs, stream_ptr=0) -> fi_sched_stats:
    arr = (fi_model_spec * len(specs))(*specs)
    grp = (C.c_int32 * len(specs))(*group_of)
    outs = (C.c_void_p * len(d_output_ptrs))(*d_output_ptrs)
    sched = fi_sched_opts(iterations, rounds, int(overlap_load), 0)
    stats = fi_sched_stats()
    _check(lib().fi_round_robin(arr, len(specs), C.byref(opts), grp, n_groups, C.byref(sched), C.c_void_p(d_input_ptr),
                                batch, outs, C.c_void_p(stream_ptr), C.byref(stats)), "fi_round_robin")
    return stats


def make_opts(max_batch, allocators=None, group_levels=True, load_mode=FI_LOAD_ONE_COPY, max_device_bytes=0,
              use_graph=False, serial_lanes=False, swap_headroom_bytes=0, per_member_inputs=False,
              copy_concats=False, separate_affine=False, separate_chains=False, member_chunks=0, separate_stem=False) -> fi_build_opts:
    opts = fi_build_opts()
    opts.max_batch, opts.group_levels, opts.load_mode, opts.max_device_bytes = max_batch, int(group_levels), load_mode, max_device_bytes
    opts.use_graph = int(use_graph)
    opts.serial_lanes = int(serial_lanes)
    opts.swap_headroom_bytes = int(swap_headroom_bytes)
    opts.per_member_inputs = int(per_member_inputs)
    opts.copy_concats = int(copy_concats)
    opts.separate_affine = int(separate_affine)
    opts.separate_chains = int(separate_chains)
    opts.member_chunks = int(member_chunks)
    opts.separate_stem = int(separate_stem)
    if allocators is not None:
        allocators.apply(opts)
    return opts


def fi_query(h) -> fi_dag_info:
    info = fi_dag_info()
    _check(lib().fi_query(h, C.byref(info)), "fi_query")
    return info


def fi_node(h, i) -> fi_node_info:
    info = fi_node_info()
    _check(lib().fi_node(h, i, C.byref(info)), "fi_node")
    return info


def fi_launch(h, i) -> fi_launch_info:
    info = fi_launch_info()
    _check(lib().fi_launch(h, i, C.byref(info)), "fi_launch")
    return info


def fi_load(h, stream_ptr=0) -> None:
    _check(lib().fi_load(h, C.c_void_p(stream_ptr)), "fi_load")


def fi_run(h, d_input_ptr, batch, d_output_ptrs, stream_ptr=0) -> None:
    outs = (C.c_void_p * len(d_output_ptrs))(*d_output_ptrs)
    _check(lib().fi_run(h, C.c_void_p(d_input_ptr), batch, outs, C.c_void_p(stream_ptr)), "fi_run")


def fi_run_static(h, d_input_ptr, batch, d_output_ptrs, stream_ptr=0) -> None:
    outs = (C.c_void_p * len(d_output_ptrs))(*d_output_ptrs)
    _check(lib().fi_run_static(h, C.c_void_p(d_input_ptr), batch, outs, C.c_void_p(stream_ptr)), "fi_run_static")


def fi_run_inputs(h, d_input_ptrs, batch, d_output_ptrs, stream_ptr=0) -> None:
    ins = (C.c_void_p * len(d_input_ptrs))(*d_input_ptrs)
    outs = (C.c_void_p * len(d_output_ptrs))(*d_output_ptrs)
    _check(lib().fi_run_inputs(h, ins, batch, outs, C.c_void_p(stream_ptr)), "fi_run_inputs")


def fi_run_batches(h, d_input_ptrs, batches, d_output_ptrs, stream_ptr=0) -> None:
    ins = (C.c_void_p * len(d_input_ptrs))(*d_input_ptrs)
    outs = (C.c_void_p * len(d_output_ptrs))(*d_output_ptrs)
    nb = (C.c_int32 * len(batches))(*batches)
    _check(lib().fi_run_batches(h, ins, nb, outs, C.c_void_p(stream_ptr)), "fi_run_batches")


def fi_run_lane(h, lane, d_input_ptrs, batches, d_output_ptrs, stream_ptr=0) -> None:
    ins = (C.c_void_p * len(d_input_ptrs))(*d_input_ptrs)
    outs = (C.c_void_p * len(d_output_ptrs))(*d_output_ptrs)
    nb = (C.c_int32 * len(batches))(*batches)
    _check(lib().fi_run_lane(h, lane, ins, nb, outs, C.c_void_p(stream_ptr)), "fi_run_lane")


def fi_profile(h, d_input_ptr, batch, d_output_ptrs, stream_ptr, n_launches):
    outs = (C.c_void_p * len(d_output_ptrs))(*d_output_ptrs)
    ms = (C.c_float * n_launches)()
    _check(lib().fi_profile(h, C.c_void_p(d_input_ptr), batch, outs, C.c_void_p(stream_ptr), ms, n_launches), "fi_profile")
    return list(ms)


def fi_timeline(h, d_input_ptr, batch, d_output_ptrs, stream_ptr, n_launches):
    outs = (C.c_void_p * len(d_output_ptrs))(*d_output_ptrs)
    b = (C.c_float * n_launches)()
    e = (C.c_float * n_launches)()
    _check(lib().fi_timeline(h, C.c_void_p(d_input_ptr), batch, outs, C.c_void_p(stream_ptr), b, e, n_launches), "fi_timeline")
    return list(b), list(e)


def fi_swap_model(h, slot, spec, stream_ptr=0) -> None:
    _check(lib().fi_swap_model(h, slot, C.byref(spec), C.c_void_p(stream_ptr)), "fi_swap_model")


def fi_member(h, m):
    info = fi_member_info()
    _check(lib().fi_member(h, m, C.byref(info)), "fi_member")
    return info


def fi_unload(h) -> None:
    _check(lib().fi_unload(h), "fi_unload")


def fi_destroy(h) -> None:
    lib().fi_destroy(h)


# ---- marshalling helpers ---------------------------------------------------------------------
_OPS = {"conv": FI_CONV2D, "dwconv": FI_DWCONV2D, "maxpool": FI_MAXPOOL2D, "gap": FI_GLOBAL_AVGPOOL,
        "fc": FI_FC, "softmax": FI_SOFTMAX, "concat": FI_CONCAT, "avgpool": FI_AVGPOOL2D, "mul": FI_MUL, "slice": FI_SLICE, "shuffle": FI_SHUFFLE}
_ACTS = {"none": FI_ACT_NONE, "relu": FI_ACT_RELU, "relu6": FI_ACT_RELU6, "hardswish": FI_ACT_HARDSWISH,
         "hardsigmoid": FI_ACT_HARDSIGMOID, "silu": FI_ACT_SILU, "sigmoid": FI_ACT_SIGMOID}
_DT = {"f32": FI_F32, "bf16": FI_BF16}


def make_spec(model, weights_ptr: int, weight_bytes: int, act_dtype=None, packed=False):
    """fi_model_spec from a model description (any object with name/dtype/in_c/in_h/in_w/layers whose
    layers carry op/input/residual/cin/cout/k/stride/pad/act/w_off/b_off).  Returns (spec, keepalive)."""
    layers = (fi_layer_spec * len(model.layers))()
    for i, L in enumerate(model.layers):
        layers[i] = fi_layer_spec(_OPS[L.op], L.input, L.residual, L.cin, L.cout, L.k, getattr(L, "kw", 0) or L.k, L.stride, L.pad,
                                  _ACTS[L.act], int(getattr(L, "ceil", False)), int(getattr(L, "groups", 1)), int(getattr(L, "first", 0)), 0, L.w_off, L.b_off)
    name = model.name.encode()
    dt = _DT[model.dtype]
    spec = fi_model_spec(name, dt, dt if act_dtype is None else _DT.get(act_dtype, act_dtype), model.in_c, model.in_h,
                         model.in_w, len(model.layers), layers, len(model.layers) - 1, 1 if packed else 0,
                         C.c_void_p(weights_ptr), weight_bytes)
    return spec, (layers, name)


class HostAllocators:
    """malloc-backed callbacks (CPU-only tests of the planner; pin_alloc need not be pinned there)."""

    def __init__(self, fail_device=False):
        self.live = {}
        self.fail_device = fail_device
        self.n_dev = self.n_pin = 0

        def pin_alloc(n, _u):
            buf = C.create_string_buffer(max(1, n))
            self.live[C.addressof(buf)] = buf
            self.n_pin += 1
            return C.addressof(buf)

        def free(p, _u):
            self.live.pop(p, None)

        def dev_alloc(n, _u):
            self.n_dev += 1
            return None

        self.cb = (ALLOC_FN(dev_alloc), FREE_FN(free), ALLOC_FN(pin_alloc), FREE_FN(free))

    def apply(self, opts: fi_build_opts):
        opts.dev_alloc, opts.dev_free, opts.pin_alloc, opts.pin_free = self.cb
        return opts


class TorchAllocators:
    """Device and pinned memory from PyTorch's allocators (memory plumbing only)."""

    def __init__(self, device="cuda:0"):
        import torch
        self.torch = torch
        self.device = device
        self.live = {}
        self.n_dev = self.n_pin = 0
        self.dev_bytes_peak = 0

        def dev_alloc(n, _u):
            try:
                t = torch.empty(max(1, n), dtype=torch.uint8, device=self.device)
            except Exception:
                return None
            self.live[t.data_ptr()] = t
            self.n_dev += 1
            self.dev_bytes_peak = max(self.dev_bytes_peak, sum(v.numel() for v in self.live.values() if v.is_cuda))
            return t.data_ptr()

        def pin_alloc(n, _u):
            try:
                t = torch.empty(max(1, n), dtype=torch.uint8, pin_memory=True)
            except Exception:
                return None
            self.live[t.data_ptr()] = t
            self.n_pin += 1
            return t.data_ptr()

        def free(p, _u):
            self.live.pop(p, None)

        self.cb = (ALLOC_FN(dev_alloc), FREE_FN(free), ALLOC_FN(pin_alloc), FREE_FN(free))

    def apply(self, opts: fi_build_opts):
        opts.dev_alloc, opts.dev_free, opts.pin_alloc, opts.pin_free = self.cb
        return opts


class Server:
    """Request aggregator in front of a loaded Dag built with per_member_inputs (argument marshalling only)."""

    def __init__(self, dag, max_wait_us=0):
        h = C.c_void_p()
        opts = fi_server_opts(max_wait_us, 0)
        _check(lib().fi_server_start(dag.h, C.byref(opts), C.byref(h)), "fi_server_start")
        self.h = h
        self.dag = dag   # the DAG must outlive the server

    def submit(self, member, d_image_ptr, d_output_ptr) -> int:
        t = C.c_uint64()
        _check(lib().fi_server_submit(self.h, member, C.c_void_p(d_image_ptr), C.c_void_p(d_output_ptr), C.byref(t)), "fi_server_submit")
        return t.value

    def wait(self, ticket) -> None:
        _check(lib().fi_server_wait(self.h, ticket), "fi_server_wait")

    def stats(self) -> fi_server_stats:
        st = fi_server_stats()
        _check(lib().fi_server_query(self.h, C.byref(st)), "fi_server_query")
        return st

    def swap(self, slot, spec, keepalive=None) -> None:
        self.dag.keepalive.append((spec, keepalive))   # borrowed by the DAG until it is destroyed
        _check(lib().fi_server_swap(self.h, slot, C.byref(spec)), "fi_server_swap")

    def stop(self) -> None:
        if self.h:
            h, self.h = self.h, None
            _check(lib().fi_server_stop(h), "fi_server_stop")

    def __del__(self):
        try:
            if getattr(self, "h", None):   # a forgotten server still has worker threads: stop them before the DAG goes
                h, self.h = self.h, None
                lib().fi_server_stop(h)
        except Exception:
            pass


class Dag:
    """Owner of one fi_dag handle."""

    def __init__(self, specs, max_batch, allocators=None, group_levels=True, load_mode=FI_LOAD_ONE_COPY,
                 max_device_bytes=0, keepalive=None, use_graph=False, serial_lanes=False, swap_headroom_bytes=0,
                 per_member_inputs=False, copy_concats=False, separate_affine=False, separate_chains=False, member_chunks=0,
                 separate_stem=False):
        self.keepalive = [specs, keepalive, allocators]
        opts = make_opts(max_batch, allocators, group_levels, load_mode, max_device_bytes, use_graph, serial_lanes,
                         swap_headroom_bytes, per_member_inputs, copy_concats, separate_affine, separate_chains, member_chunks, separate_stem)
        self.opts = opts
        self.h = fi_build_dag(specs, opts)
        self.n_models = len(specs)

    def query(self):
        return fi_query(self.h)

    def nodes(self):
        return [fi_node(self.h, i) for i in range(self.query().n_nodes)]

    def launches(self):
        return [fi_launch(self.h, i) for i in range(self.query().n_launches)]

    def members(self):
        return [fi_member(self.h, m) for m in range(self.n_models)]

    def load(self, stream_ptr=0):
        fi_load(self.h, stream_ptr)

    def swap_model(self, slot, spec, stream_ptr=0, keepalive=None):
        """Replaces member `slot`; `keepalive` holds whatever backs the spec's borrowed pointers."""
        fi_swap_model(self.h, slot, spec, stream_ptr)
        self.keepalive.append((spec, keepalive))

    def run(self, d_input_ptr, batch, d_output_ptrs, stream_ptr=0):
        fi_run(self.h, d_input_ptr, batch, d_output_ptrs, stream_ptr)

    def run_static(self, d_input_ptr, batch, d_output_ptrs, stream_ptr=0):
        fi_run_static(self.h, d_input_ptr, batch, d_output_ptrs, stream_ptr)

    def run_inputs(self, d_input_ptrs, batch, d_output_ptrs, stream_ptr=0):
        fi_run_inputs(self.h, d_input_ptrs, batch, d_output_ptrs, stream_ptr)

    def run_batches(self, d_input_ptrs, batches, d_output_ptrs, stream_ptr=0):
        fi_run_batches(self.h, d_input_ptrs, batches, d_output_ptrs, stream_ptr)

    def run_lane(self, lane, d_input_ptrs, batches, d_output_ptrs, stream_ptr=0):
        fi_run_lane(self.h, lane, d_input_ptrs, batches, d_output_ptrs, stream_ptr)

    def profile(self, d_input_ptr, batch, d_output_ptrs, stream_ptr=0):
        return fi_profile(self.h, d_input_ptr, batch, d_output_ptrs, stream_ptr, self.query().n_launches)

    def timeline(self, d_input_ptr, batch, d_output_ptrs, stream_ptr=0):
        return fi_timeline(self.h, d_input_ptr, batch, d_output_ptrs, stream_ptr, self.query().n_launches)

    def unload(self):
        fi_unload(self.h)

    def destroy(self):
        if self.h:
            fi_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
