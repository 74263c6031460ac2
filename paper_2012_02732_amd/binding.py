"""ctypes binding with the same names as the C ABI (include/nimble_graph.h).

Marshalling only. The shared library must have been built (``python -m
paper_2012_02732_amd.build``); there is no fallback of any kind: if it cannot be
loaded, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch  # noqa: F401  (loads the process-wide HIP runtime before the library binds to it)

NG_MAX_PREDS = 8
NG_OK, NG_EINVAL, NG_ESHAPE, NG_ESTATE, NG_ENOMEM, NG_EHIP = 0, -1, -2, -3, -4, -5
(NG_OP_INPUT, NG_OP_CONV1X1, NG_OP_DWCONV, NG_OP_CONV3X3, NG_OP_BN_ACT, NG_OP_RELU, NG_OP_ADD_N,
 NG_OP_CONCAT, NG_OP_POOL, NG_OP_GLOBAL_AVGPOOL, NG_OP_FC,
 NG_OP_CONV1X1_DGRAD, NG_OP_CONV1X1_WGRAD, NG_OP_CONV3X3_DGRAD, NG_OP_CONV3X3_WGRAD, NG_OP_DWCONV_DGRAD, NG_OP_DWCONV_WGRAD,
 NG_OP_BN_ACT_DGRAD, NG_OP_BN_ACT_WGRAD, NG_OP_RELU_DGRAD, NG_OP_POOL_DGRAD, NG_OP_GAP_DGRAD, NG_OP_CHANNEL_SUM,
 NG_OP_SLICE_PAD, NG_OP_SGD_UPDATE) = range(25)
NG_MODE_GRAPH_MULTI, NG_MODE_GRAPH_SINGLE, NG_MODE_EAGER_SINGLE, NG_MODE_EAGER_MULTI, NG_MODE_DEVICE_RESIDENT, NG_MODE_AUTO = range(6)
NG_ASSIGN_ALGORITHM1, NG_ASSIGN_EXACT = 0, 1

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libnimble_graph.so")

# every symbol include/nimble_graph.h declares
SYMBOLS = ("ng_create", "ng_destroy", "ng_add_input", "ng_add_node", "ng_mark_output", "ng_num_nodes",
           "ng_node_shape", "ng_schedule", "ng_set_assignment", "ng_schedule_sizes", "ng_get_schedule", "ng_get_scaffold",
           "ng_plan_memory", "ng_set_memory_reuse", "ng_set_launch_fusion", "ng_get_graph_edges", "ng_get_offsets",
           "ng_graph_multi_check", "ng_graph_multi_recheck", "ng_graph_multi_distrust", "ng_critical_path", "ng_bind", "ng_capture",
           "ng_tensor_ptr", "ng_replay_mode", "ng_replay", "ng_replay_static", "ng_sync", "ng_resident_config",
           "ng_auto_mode", "ng_resident_dry_plan", "ng_resident_dry_plan_setting", "ng_resident_xcd_mapping", "ng_resident_fusion", "ng_resident_plan_trials", "ng_resident_plan_kept", "ng_resident_sizes", "ng_resident_trace", "ng_time_replay", "ng_time_chain", "ng_time_task",
           "ng_time_task_device", "ng_task_kernel_executed", "ng_time_launch_floor", "ng_launch_task_solo",
           "ng_task_kernel", "ng_planned_task_kernel", "ng_task_work", "ng_last_error", "ng_version")


class ng_op_params(C.Structure):
    _fields_ = [("cout", C.c_int32), ("k", C.c_int32), ("stride", C.c_int32), ("pad", C.c_int32),
                ("relu", C.c_int32), ("pool_mode", C.c_int32), ("eps", C.c_float),
                ("slice_lo", C.c_int32 * NG_MAX_PREDS), ("slice_hi", C.c_int32 * NG_MAX_PREDS), ("lr", C.c_float)]


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2012_02732_amd.build`")
lib = C.CDLL(LIB_PATH)

_P, _I, _IP = C.c_void_p, C.c_int, C.POINTER(C.c_int)
_SZP, _FP, _DP = C.POINTER(C.c_size_t), C.POINTER(C.c_float), C.POINTER(C.c_double)
_sig = {
    "ng_create": (_I, [C.POINTER(_P)]),
    "ng_destroy": (None, [_P]),
    "ng_add_input": (_I, [_P, C.POINTER(C.c_int64), _IP]),
    "ng_add_node": (_I, [_P, _I, C.POINTER(ng_op_params), _IP, _I, C.POINTER(_P), _I, _IP]),
    "ng_mark_output": (_I, [_P, _I]),
    "ng_num_nodes": (_I, [_P]),
    "ng_node_shape": (_I, [_P, _I, C.POINTER(C.c_int64)]),
    "ng_schedule": (_I, [_P]),
    "ng_set_assignment": (_I, [_P, _I]),
    "ng_schedule_sizes": (_I, [_P, _IP, _IP, _IP, _IP, _IP, _IP, _IP]),
    "ng_get_schedule": (_I, [_P, _IP, _IP, _IP, _IP, _IP, _IP, _IP, _IP]),
    "ng_get_scaffold": (_I, [_P, _IP, _IP, _IP, _IP]),
    "ng_plan_memory": (_I, [_P, _SZP]),
    "ng_set_memory_reuse": (_I, [_P, _I]),
    "ng_get_offsets": (_I, [_P, _SZP, _SZP]),
    "ng_set_launch_fusion": (_I, [_P, _I]),
    "ng_get_graph_edges": (_I, [_P, _I, _IP, _IP, _IP, _IP, _I]),
    "ng_graph_multi_check": (_I, [_P, _IP, _IP]),
    "ng_graph_multi_recheck": (_I, [_P, _I]),
    "ng_graph_multi_distrust": (_I, [_P]),
    "ng_critical_path": (_I, [_P, _FP, _FP, _IP, _IP]),
    "ng_bind": (_I, [_P, _P, C.c_size_t, C.POINTER(_P), _I]),
    "ng_capture": (_I, [_P]),
    "ng_tensor_ptr": (_P, [_P, _I]),
    "ng_replay_mode": (_I, [_P, _I]),
    "ng_replay": (_I, [_P]),
    "ng_replay_static": (_I, [_P]),
    "ng_sync": (_I, [_P]),
    "ng_resident_config": (_I, [_P, _I, _I, C.c_uint, _I]),
    "ng_auto_mode": (_I, [_P, _IP, C.POINTER(C.c_float)]),
    "ng_resident_dry_plan": (_I, [_P, _I, _I, _DP, _IP, _IP, _IP]),
    "ng_resident_dry_plan_setting": (_I, [_P, _I, _I, _I, _DP, _IP, _IP, _IP]),
    "ng_resident_xcd_mapping": (_I, [_P, _IP]),
    "ng_resident_fusion": (_I, [_P, _IP]),
    "ng_resident_plan_trials": (_I, [_P, _I]),
    "ng_resident_plan_kept": (_I, [_P, _IP]),
    "ng_resident_sizes": (_I, [_P, _IP, _IP, _IP, _DP]),
    "ng_resident_trace": (_I, [_P, _I, C.POINTER(C.c_ulonglong)]),
    "ng_time_replay": (_I, [_P, _I, _FP]),
    "ng_time_chain": (_I, [_P, _I, _I, _FP]),
    "ng_time_task": (_I, [_P, _I, _I, _FP]),
    "ng_time_task_device": (_I, [_P, _I, _I, _I, _FP, _FP]),
    "ng_task_kernel_executed": (C.c_char_p, [_P, _I]),
    "ng_launch_task_solo": (_I, [_P, _I, _I]),
    "ng_time_launch_floor": (_I, [_P, _I, _FP]),
    "ng_task_kernel": (C.c_char_p, [_P, _I]),
    "ng_planned_task_kernel": (C.c_char_p, [_P, _I]),
    "ng_task_work": (_I, [_P, _I, _DP, _DP]),
    "ng_last_error": (C.c_char_p, [_P]),
    "ng_version": (C.c_char_p, []),
}
for _name, (_res, _args) in _sig.items():
    _fn = getattr(lib, _name)
    _fn.restype, _fn.argtypes = _res, _args


class NgError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"[{code}] {msg}")
        self.code = code


def check(g, rc):
    if rc != NG_OK:
        raise NgError(rc, lib.ng_last_error(g).decode() if g else "null graph")


def _ints(n):
    return (C.c_int * max(n, 1))()


# ---- same names as the C functions ------------------------------------------------
def ng_version() -> str:
    return lib.ng_version().decode()


def ng_create():
    g = _P()
    check(None, lib.ng_create(C.byref(g)))
    return g


def ng_destroy(g):
    lib.ng_destroy(g)


def ng_add_input(g, nchw) -> int:
    arr, out = (C.c_int64 * 4)(*nchw), C.c_int()
    check(g, lib.ng_add_input(g, arr, C.byref(out)))
    return out.value


def ng_add_node(g, op_kind, params: ng_op_params, preds, dev_weights) -> int:
    """dev_weights: device addresses as ints (0 allowed while no GPU work is requested)."""
    p = (C.c_int * max(len(preds), 1))(*preds)
    w = (_P * max(len(dev_weights), 1))(*[_P(a) for a in dev_weights])
    out = C.c_int()
    check(g, lib.ng_add_node(g, op_kind, C.byref(params), p, len(preds), w, len(dev_weights), C.byref(out)))
    return out.value


def ng_mark_output(g, node_id):
    check(g, lib.ng_mark_output(g, node_id))


def ng_num_nodes(g) -> int:
    return lib.ng_num_nodes(g)


def ng_node_shape(g, node_id):
    arr = (C.c_int64 * 4)()
    rc = lib.ng_node_shape(g, node_id, arr)
    if rc != NG_OK:
        raise NgError(rc, "ng_node_shape: bad id")
    return tuple(arr)


def ng_schedule(g):
    check(g, lib.ng_schedule(g))


def ng_set_memory_reuse(g, on: bool):
    check(g, lib.ng_set_memory_reuse(g, int(bool(on))))


def ng_set_assignment(g, assignment: int):
    check(g, lib.ng_set_assignment(g, assignment))


def ng_schedule_sizes(g) -> dict:
    v = [C.c_int() for _ in range(7)]
    check(g, lib.ng_schedule_sizes(g, *[C.byref(x) for x in v]))
    keys = ("n_nodes", "n_streams", "n_chains", "n_meg_edges", "n_matching", "n_sync", "n_events")
    return dict(zip(keys, (x.value for x in v)))


def ng_get_schedule(g) -> dict:
    sz = ng_schedule_sizes(g)
    n, ne, ns = sz["n_nodes"], sz["n_meg_edges"], sz["n_sync"]
    order, stream_of, chain_of, event_of = _ints(n), _ints(n), _ints(n), _ints(n)
    ms, md, ss, sd = _ints(ne), _ints(ne), _ints(ns), _ints(ns)
    check(g, lib.ng_get_schedule(g, order, stream_of, chain_of, event_of, ms, md, ss, sd))
    return dict(sz, order=list(order[:n]), stream_of=list(stream_of[:n]), chain_of=list(chain_of[:n]),
                event_of=list(event_of[:n]), meg=list(zip(ms[:ne], md[:ne])), sync=list(zip(ss[:ns], sd[:ns])))


def ng_get_scaffold(g):
    ns = ng_schedule_sizes(g)["n_streams"]
    fork, join, nf, nj = _ints(ns), _ints(ns), C.c_int(), C.c_int()
    check(g, lib.ng_get_scaffold(g, fork, C.byref(nf), join, C.byref(nj)))
    return list(fork[:nf.value]), list(join[:nj.value])


def ng_plan_memory(g) -> int:
    out = C.c_size_t()
    check(g, lib.ng_plan_memory(g, C.byref(out)))
    return out.value


def ng_get_offsets(g):
    n = ng_num_nodes(g)
    off, nbytes = (C.c_size_t * n)(), (C.c_size_t * n)()
    check(g, lib.ng_get_offsets(g, off, nbytes))
    return list(off), list(nbytes)


def ng_set_launch_fusion(g, on: bool):
    check(g, lib.ng_set_launch_fusion(g, int(bool(on))))


def ng_get_graph_edges(g, fuse=True):
    """(launched_by[n_nodes], [(src task, dst task)]) of the multi-stream HIP graph; fuse=2: of the single-stream modes."""
    n, ne = ng_num_nodes(g), C.c_int()
    fuse = 2 if fuse == 2 else int(bool(fuse))
    check(g, lib.ng_get_graph_edges(g, fuse, None, C.byref(ne), None, None, 0))
    by, src, dst = _ints(n), _ints(ne.value), _ints(ne.value)
    check(g, lib.ng_get_graph_edges(g, fuse, by, C.byref(ne), src, dst, ne.value))
    return list(by[:n]), list(zip(src[:ne.value], dst[:ne.value]))


def ng_graph_multi_check(g):
    """(state, replays compared): 1 reproduced the single-stream result, -1 did not, 0 not checked."""
    st, k = C.c_int(), C.c_int()
    check(g, lib.ng_graph_multi_check(g, C.byref(st), C.byref(k)))
    return st.value, k.value


def ng_graph_multi_recheck(g, replays: int):
    check(g, lib.ng_graph_multi_recheck(g, replays))


def ng_graph_multi_distrust(g):
    check(g, lib.ng_graph_multi_distrust(g))


def ng_critical_path(g, t):
    n = ng_num_nodes(g)
    arr, total, path, npath = (C.c_float * n)(*t), C.c_float(), _ints(n), C.c_int()
    check(g, lib.ng_critical_path(g, arr, C.byref(total), path, C.byref(npath)))
    return total.value, list(path[:npath.value])


def ng_bind(g, arena_ptr: int, arena_bytes: int, stream_handles):
    s = (_P * max(len(stream_handles), 1))(*[_P(h) for h in stream_handles])
    check(g, lib.ng_bind(g, _P(arena_ptr), arena_bytes, s, len(stream_handles)))


def ng_capture(g):
    check(g, lib.ng_capture(g))


def ng_tensor_ptr(g, node_id) -> int:
    return lib.ng_tensor_ptr(g, node_id) or 0


def ng_replay_mode(g, mode):
    check(g, lib.ng_replay_mode(g, mode))


def ng_replay(g):
    check(g, lib.ng_replay(g))


def ng_replay_static(g):
    check(g, lib.ng_replay_static(g))


def ng_sync(g):
    check(g, lib.ng_sync(g))


def ng_resident_config(g, workgroups_per_cu=0, xcds=0, spin_limit=0, device_scope_everywhere=0):
    check(g, lib.ng_resident_config(g, workgroups_per_cu, xcds, spin_limit, device_scope_everywhere))


def ng_auto_mode(g):
    """(mode NG_MODE_AUTO resolves to, {mode: trial median in microseconds})"""
    m, t = C.c_int(), (C.c_float * 3)()
    check(g, lib.ng_auto_mode(g, C.byref(m), t))
    return m.value, {NG_MODE_GRAPH_MULTI: t[0], NG_MODE_GRAPH_SINGLE: t[1], NG_MODE_DEVICE_RESIDENT: t[2]}


def ng_resident_dry_plan(g, n_workgroups=256, xcds=0) -> dict:
    e, n, f, ok = C.c_double(), C.c_int(), C.c_int(), C.c_int()
    check(g, lib.ng_resident_dry_plan(g, n_workgroups, xcds, C.byref(e), C.byref(n), C.byref(f), C.byref(ok)))
    return {"expected_us": e.value, "n_entries": n.value, "n_far_edges": f.value, "ok": bool(ok.value)}


def ng_resident_dry_plan_setting(g, setting, n_workgroups=256, xcds=0) -> dict:
    e, n, f, ok = C.c_double(), C.c_int(), C.c_int(), C.c_int()
    check(g, lib.ng_resident_dry_plan_setting(g, setting, n_workgroups, xcds, C.byref(e), C.byref(n), C.byref(f), C.byref(ok)))
    return {"expected_us": e.value, "n_entries": n.value, "n_far_edges": f.value, "ok": bool(ok.value)}


def ng_resident_xcd_mapping(g) -> bool:
    v = C.c_int()
    check(g, lib.ng_resident_xcd_mapping(g, C.byref(v)))
    return bool(v.value)


def ng_resident_fusion(g):
    """Per node: the convolution whose tiles also apply it in the device-resident replay, or -1."""
    host_of = _ints(lib.ng_num_nodes(g))
    check(g, lib.ng_resident_fusion(g, host_of))
    return list(host_of)[:lib.ng_num_nodes(g)]


def ng_resident_plan_trials(g, trials: int):
    check(g, lib.ng_resident_plan_trials(g, trials))


def ng_resident_plan_kept(g) -> int:
    v = C.c_int()
    check(g, lib.ng_resident_plan_kept(g, C.byref(v)))
    return v.value


def ng_resident_sizes(g):
    a, b, x, e = C.c_int(), C.c_int(), C.c_int(), C.c_double()
    check(g, lib.ng_resident_sizes(g, C.byref(a), C.byref(b), C.byref(x), C.byref(e)))
    return a.value, b.value, x.value, e.value


def ng_resident_trace(g, enable, fetch=False):
    """Switch the per-task timeline on/off (switching on clears it); with fetch=True return
    [(first wait, last ready, first done, last done)] in microseconds relative to the earliest
    reading, None for nodes that did not run."""
    if not fetch:
        check(g, lib.ng_resident_trace(g, int(enable), None))
        return None
    n = ng_num_nodes(g)
    buf = (C.c_ulonglong * (4 * n))()
    check(g, lib.ng_resident_trace(g, int(enable), buf))
    top = 2 ** 64 - 1
    ran = {i for i in range(n) if buf[4 * i + 3] != 0 and buf[4 * i] != top}
    base = min((buf[4 * i] for i in ran), default=0)
    return [tuple((buf[4 * i + j] - base) / 100.0 for j in range(4)) if i in ran else None for i in range(n)]


def ng_time_replay(g, reps) -> float:
    out = C.c_float()
    check(g, lib.ng_time_replay(g, reps, C.byref(out)))
    return out.value


def ng_time_chain(g, node_id, reps) -> float:
    out = C.c_float()
    check(g, lib.ng_time_chain(g, node_id, reps, C.byref(out)))
    return out.value


def ng_time_task(g, node_id, reps) -> float:
    out = C.c_float()
    check(g, lib.ng_time_task(g, node_id, reps, C.byref(out)))
    return out.value


def ng_time_task_device(g, node_id, as_executed, reps):
    """(median, minimum) of the kernel's begin-to-end time by device timestamps, microseconds."""
    med, lo = C.c_float(), C.c_float()
    check(g, lib.ng_time_task_device(g, node_id, int(bool(as_executed)), reps, C.byref(med), C.byref(lo)))
    return med.value, lo.value


def ng_launch_task_solo(g, node_id, as_executed=False):
    check(g, lib.ng_launch_task_solo(g, node_id, int(bool(as_executed))))


def ng_task_kernel_executed(g, node_id) -> str:
    return lib.ng_task_kernel_executed(g, node_id).decode()


def ng_time_launch_floor(g, reps) -> float:
    out = C.c_float()
    check(g, lib.ng_time_launch_floor(g, reps, C.byref(out)))
    return out.value


def ng_task_kernel(g, node_id) -> str:
    return lib.ng_task_kernel(g, node_id).decode()


def ng_planned_task_kernel(g, node_id) -> str:
    """The kernel the node will be bound to, from the shapes alone (no GPU)."""
    name = lib.ng_planned_task_kernel(g, node_id)
    if name is None:
        raise NgError(NG_EINVAL, lib.ng_last_error(g).decode() if g else "null graph")
    return name.decode()


def ng_task_work(g, node_id):
    b, f = C.c_double(), C.c_double()
    rc = lib.ng_task_work(g, node_id, C.byref(b), C.byref(f))
    if rc != NG_OK:
        raise NgError(rc, "ng_task_work: bad id")
    return b.value, f.value


def ng_last_error(g) -> str:
    return lib.ng_last_error(g).decode()
