"""Registers a workload description with the library and owns the torch plumbing.

PyTorch is used for exactly three things: device memory (weights, the arena),
stream handles, and host<->device copies of inputs/outputs. Every step of the
method itself - shape inference, Algorithm 1, the memory plan, the task table,
capture, replay and all kernels - runs inside libnimble_graph.so.
"""
from __future__ import annotations

import ctypes as C

import numpy as np
import torch

from . import binding as B

# torch hands out streams from a pool of 32 per device, so asking it for more returns the
# same handle twice; wide DAGs need more distinct streams than that. Streams are therefore
# created straight from the HIP runtime torch has already loaded.
def _loaded_hip_runtime():
    """The libamdhip64 this process has mapped already (torch brought it in): its path as the
    loader recorded it, so that no second copy and no guessed version suffix is involved."""
    try:
        with open("/proc/self/maps") as maps:
            for line in maps:
                path = line.rsplit(" ", 1)[-1].strip()
                if "libamdhip64.so" in path.rsplit("/", 1)[-1]:
                    return path
    except OSError:
        pass
    raise ImportError("libamdhip64 is not loaded in this process (PyTorch-ROCm should have loaded it)")


_hip = C.CDLL(_loaded_hip_runtime())
_hip.hipStreamCreateWithFlags.argtypes = [C.POINTER(C.c_void_p), C.c_uint]
_hip.hipStreamDestroy.argtypes = [C.c_void_p]
_HIP_STREAM_NON_BLOCKING = 1


def _new_streams(n):
    out = []
    for _ in range(n):
        h = C.c_void_p()
        rc = _hip.hipStreamCreateWithFlags(C.byref(h), _HIP_STREAM_NON_BLOCKING)
        if rc != 0 or not h.value:
            raise RuntimeError(f"hipStreamCreateWithFlags failed with {rc}")
        out.append(h.value)
    return out

_OPS = {"conv1x1": B.NG_OP_CONV1X1, "dwconv": B.NG_OP_DWCONV, "conv3x3": B.NG_OP_CONV3X3,
        "bn_act": B.NG_OP_BN_ACT, "relu": B.NG_OP_RELU, "add_n": B.NG_OP_ADD_N,
        "concat": B.NG_OP_CONCAT, "pool": B.NG_OP_POOL, "global_avgpool": B.NG_OP_GLOBAL_AVGPOOL,
        "fc": B.NG_OP_FC,
        "conv1x1_dgrad": B.NG_OP_CONV1X1_DGRAD, "conv1x1_wgrad": B.NG_OP_CONV1X1_WGRAD,
        "conv3x3_dgrad": B.NG_OP_CONV3X3_DGRAD, "conv3x3_wgrad": B.NG_OP_CONV3X3_WGRAD,
        "dwconv_dgrad": B.NG_OP_DWCONV_DGRAD, "dwconv_wgrad": B.NG_OP_DWCONV_WGRAD,
        "bn_act_dgrad": B.NG_OP_BN_ACT_DGRAD, "bn_act_wgrad": B.NG_OP_BN_ACT_WGRAD, "relu_dgrad": B.NG_OP_RELU_DGRAD,
        "pool_dgrad": B.NG_OP_POOL_DGRAD, "global_avgpool_dgrad": B.NG_OP_GAP_DGRAD, "channel_sum": B.NG_OP_CHANNEL_SUM,
        "slice_pad": B.NG_OP_SLICE_PAD, "sgd_update": B.NG_OP_SGD_UPDATE}


def _params(nd) -> B.ng_op_params:
    p, q = B.ng_op_params(), nd.params
    p.cout = int(q.get("cout", 0))
    p.k = int(q.get("k", 0))
    p.stride = int(q.get("stride", 1))
    p.pad = int(q.get("pad", 0))
    p.relu = int(q.get("relu", 0))
    p.pool_mode = 1 if q.get("mode") == "avg" else 0
    p.eps = float(q.get("eps", 0.0))
    for j, (lo, hi) in enumerate(zip(q.get("lo", []), q.get("hi", []))):
        p.slice_lo[j], p.slice_hi[j] = int(lo), int(hi)
    if nd.op == "slice_pad":
        p.slice_lo[0], p.slice_hi[0], p.slice_lo[1] = int(q["src_lo"]), int(q["src_hi"]), int(q["dst_lo"])
    if nd.op == "sgd_update":
        p.lr, p.slice_lo[0], p.cout = float(q["lr"]), int(q["offset"]), int(q["numel"])
    return p


class GraphRunner:
    """One registered DAG. ``device=None`` keeps everything on the host (scheduling
    and planning only; weights are registered as null pointers)."""

    def __init__(self, workload, device=None):
        self.workload = workload
        self.device = device
        self.g = B.ng_create()
        self._weights = {}                       # (node id, weight index) -> device tensor (kept alive; shared by backward nodes)
        self.arena = None
        self.streams = []
        for v, nd in enumerate(workload.nodes):
            if nd.op == "input":
                q = nd.params
                vid = B.ng_add_input(self.g, (q["n"], q["c"], q["h"], q["w"]))
            else:
                ptrs = []
                for j, w in enumerate(nd.weights):
                    if device is None:
                        ptrs.append(0)
                    else:
                        t = torch.from_numpy(np.ascontiguousarray(w, dtype=np.float32)).to(device)
                        self._weights[(v, j)] = t
                        ptrs.append(t.data_ptr())
                for ref in getattr(nd, "shared_weights", []):       # the same buffers as an earlier node's
                    ptrs.append(0 if device is None else self._weights[tuple(ref)].data_ptr())
                vid = B.ng_add_node(self.g, _OPS[nd.op], _params(nd), nd.preds, ptrs)
            assert vid == v
        for o in workload.outputs:
            B.ng_mark_output(self.g, o)

    def close(self):
        if self.g is not None:
            if self.device is not None:
                torch.cuda.synchronize(self.device)
            B.ng_destroy(self.g)
            self.g = None
            for h in self.streams:
                _hip.hipStreamDestroy(h)
            self.streams = []

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- host-only part of the AoT pass ------------------------------------------
    def schedule(self) -> dict:
        B.ng_schedule(self.g)
        return B.ng_get_schedule(self.g)

    def plan(self) -> int:
        return B.ng_plan_memory(self.g)

    # -- GPU part ----------------------------------------------------------------
    def prepare(self, resident_wg_per_cu=0, resident_xcds=0, resident_device_scope=0, plan_trials=None, launch_fusion=True):
        """schedule -> plan -> bind -> capture, allocating arena and streams with torch."""
        assert self.device is not None, "GraphRunner was created without a device"
        if plan_trials is not None:
            B.ng_resident_plan_trials(self.g, plan_trials)
        if not launch_fusion:
            B.ng_set_launch_fusion(self.g, False)
        if resident_wg_per_cu or resident_xcds or resident_device_scope:
            B.ng_resident_config(self.g, resident_wg_per_cu, resident_xcds, 0, resident_device_scope)
        sched = self.schedule()
        nbytes = self.plan()
        self.arena = torch.zeros(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = (self.arena.data_ptr() + 255) // 256 * 256
        with torch.cuda.device(self.device):
            self.streams = _new_streams(sched["n_streams"])
        torch.cuda.synchronize(self.device)
        B.ng_bind(self.g, base, nbytes, self.streams)
        self.set_input(self.workload.input)
        for node_id, value in getattr(self.workload, "inputs", {}).items():
            self.set_input(value, node_id)
        B.ng_capture(self.g)
        return sched

    def _view(self, node_id) -> torch.Tensor:
        shape = B.ng_node_shape(self.g, node_id)
        off = B.ng_tensor_ptr(self.g, node_id) - self.arena.data_ptr()
        n = int(np.prod(shape))
        return self.arena[off:off + 4 * n].view(torch.float32).view(*shape)

    def set_input(self, x: np.ndarray, node_id: int = 0):
        t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
        self._view(node_id).copy_(t.to(self.device))
        torch.cuda.synchronize(self.device)

    def weight(self, node_id, j) -> np.ndarray:
        """Current value of weight j of a node (a training graph updates it in place)."""
        torch.cuda.synchronize(self.device)
        return self._weights[(node_id, j)].cpu().numpy()

    def set_weight(self, node_id, j, value: np.ndarray):
        self._weights[(node_id, j)].copy_(torch.from_numpy(np.ascontiguousarray(value, dtype=np.float32)).to(self.device))
        torch.cuda.synchronize(self.device)

    def replay(self, mode=None):
        if mode is not None:
            B.ng_replay_mode(self.g, mode)
        B.ng_replay(self.g)

    def sync(self):
        B.ng_sync(self.g)

    def output(self, node_id) -> np.ndarray:
        self.sync()
        torch.cuda.synchronize(self.device)
        return self._view(node_id).cpu().numpy()

    def output_images(self, node_id, lo, hi) -> np.ndarray:
        """Images [lo, hi) of a node's tensor (only that slice crosses to the host)."""
        self.sync()
        torch.cuda.synchronize(self.device)
        return self._view(node_id)[lo:hi].cpu().numpy()

    def run(self, x=None, mode=None) -> dict:
        if x is not None:
            self.set_input(x)
        self.replay(mode)
        return {o: self.output(o) for o in self.workload.outputs}
