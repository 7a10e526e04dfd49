"""Thin ctypes binding of libmgwfbp.so (see include/mgwfbp.h for the contract of each call).

Only argument marshalling happens here: every step of the path (planning, table building,
pack, reduce, unpack, update) runs inside the library.  PyTorch tensors are accepted as
sources of device pointers and streams; nothing is computed with them.  There is no CPU or
PyTorch fallback: if the library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
import weakref
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmgwfbp.so")

OK, EINVAL, ENOMEM, EHIP, ESTATE = 0, -1, -2, -3, -4
MODE_OPTIMAL, MODE_PAPER_GREEDY, MODE_WFBP, MODE_SINGLE = 0, 1, 2, 3
OPT_TILE_ELEMS, OPT_SMALL_ELEMS, OPT_NONTEMPORAL, OPT_PACE, OPT_LONG_TILES, OPT_PAD_ELEMS = 1, 2, 3, 4, 5, 6
OPT_UPDATE_WGS_PER_CU = 7
OPT_GATED_WGS_PER_CU = 8
OPT_GATED_CUS = 9
STATIC_WORKSPACE_BYTES = 64 * 1024 * 1024

EXPORTS = [
    "mgwfbp_plan", "mgwfbp_plan_explicit", "mgwfbp_plan_info", "mgwfbp_plan_timeline",
    "mgwfbp_plan_set_option", "mgwfbp_plan_layout", "mgwfbp_bind", "mgwfbp_tune", "mgwfbp_workspace_bytes",
    "mgwfbp_pack_reduce_unpack", "mgwfbp_step", "mgwfbp_pack", "mgwfbp_reduce", "mgwfbp_unpack",
    "mgwfbp_pack_reduce", "mgwfbp_unpack_update", "mgwfbp_pack_reduce_unpack_static",
    "mgwfbp_run_iteration", "mgwfbp_run_iteration_streams", "mgwfbp_run_iteration_gated",
    "mgwfbp_gated_launch", "mgwfbp_gated_signal", "mgwfbp_gated_gave_up", "mgwfbp_gated_workgroups",
    "mgwfbp_streams_side_by_side", "mgwfbp_confined_stream_create", "mgwfbp_confined_stream_destroy",
    "mgwfbp_iteration_capture", "mgwfbp_iteration_replay",
    "mgwfbp_iteration_destroy", "mgwfbp_fit_cost", "mgwfbp_table2_cost", "mgwfbp_scaling_curve", "mgwfbp_plan_destroy",
    "mgwfbp_last_error",
]
# include/mgwfbp_probe.h: bandwidth probes for the benchmark, not part of the method
PROBE_EXPORTS = ["mgwfbp_probe_copy", "mgwfbp_probe_read", "mgwfbp_probe_fill", "mgwfbp_probe_streams"]


class MgwfbpError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"mgwfbp error {code}: {msg}")
        self.code = code


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_1811_11141_amd.build` "
            "(there is no fallback path)")
    # PyTorch owns the device memory and streams this library works on, and ships its own
    # HIP runtime.  Import it first so that libmgwfbp.so resolves libamdhip64 to that same
    # already-loaded runtime: two HIP runtimes in one process do not share a device.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, u64, f64, f32, sz = (C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_double,
                                       C.c_float, C.c_size_t)
    P = C.POINTER
    lib.mgwfbp_plan.argtypes = [i32, P(u64), P(f64), f64, f64, f64, i32, i32, P(vp)]
    lib.mgwfbp_plan_explicit.argtypes = [i32, P(u64), P(f64), f64, f64, f64, i32, P(C.c_uint8), P(vp)]
    lib.mgwfbp_plan_info.argtypes = [vp, P(i32), P(i32), P(u64), P(u64), P(f64), P(f64)]
    lib.mgwfbp_plan_timeline.argtypes = [vp, P(f64), P(f64), P(f64)]
    lib.mgwfbp_plan_set_option.argtypes = [vp, i32, i64]
    lib.mgwfbp_plan_layout.argtypes = [vp, vp, vp, sz, vp, vp, sz]
    lib.mgwfbp_bind.argtypes = [vp, P(vp), P(vp), P(vp), P(vp)]
    lib.mgwfbp_workspace_bytes.argtypes = [vp, i32, P(sz)]
    lib.mgwfbp_tune.argtypes = [vp, vp, P(i32), P(f64)]
    lib.mgwfbp_pack_reduce_unpack.argtypes = [vp, i32, vp, sz, vp]
    lib.mgwfbp_pack_reduce_unpack_static.argtypes = [vp, i32, vp]
    lib.mgwfbp_step.argtypes = [vp, i32, f32, f32, vp, sz, vp]
    for name in ("mgwfbp_pack", "mgwfbp_reduce", "mgwfbp_unpack"):
        getattr(lib, name).argtypes = [vp, i32, vp, sz, vp]
    lib.mgwfbp_run_iteration.argtypes = [vp, P(f64), i32, f32, f32, vp, vp, P(f64), P(f64), P(f64), P(f64)]
    lib.mgwfbp_iteration_capture.argtypes = [vp, P(f64), i32, f32, f32, vp, vp, P(vp)]
    lib.mgwfbp_iteration_replay.argtypes = [vp, vp, P(f64)]
    lib.mgwfbp_iteration_destroy.argtypes = [vp]
    lib.mgwfbp_iteration_destroy.restype = None
    lib.mgwfbp_pack_reduce.argtypes = [vp, i32, vp, sz, vp]
    lib.mgwfbp_unpack_update.argtypes = [vp, i32, vp, sz, i32, f32, f32, vp]
    lib.mgwfbp_fit_cost.argtypes = [i32, P(f64), P(f64), P(f64), P(f64)]
    lib.mgwfbp_table2_cost.argtypes = [i32, i32, f64, f64, f64, P(f64), P(f64)]
    lib.mgwfbp_scaling_curve.argtypes = [i32, P(u64), P(f64), f64, i32, f64, f64, f64, i32, P(i32), i32,
                                         P(f64), P(f64)]
    lib.mgwfbp_run_iteration_streams.argtypes = [vp, P(f64), i32, f32, f32, vp, P(vp), i32, P(f64), P(f64), P(f64), P(f64)]
    lib.mgwfbp_run_iteration_gated.argtypes = [vp, P(f64), i32, f32, f32, vp, vp, f64, P(f64)]
    lib.mgwfbp_gated_launch.argtypes = [vp, i32, f32, f32, C.c_uint32, f64, vp]
    lib.mgwfbp_gated_signal.argtypes = [vp, i32, C.c_uint32, vp]
    lib.mgwfbp_gated_gave_up.argtypes = [vp, P(i32)]
    lib.mgwfbp_gated_workgroups.argtypes = [vp, i32, P(C.c_uint32), P(C.c_uint32)]
    lib.mgwfbp_confined_stream_create.argtypes = [C.c_uint32, P(vp)]
    lib.mgwfbp_confined_stream_destroy.argtypes = [vp]
    lib.mgwfbp_streams_side_by_side.argtypes = [vp, vp, vp, P(i32)]
    lib.mgwfbp_probe_copy.argtypes = [vp, vp, u64, vp]
    lib.mgwfbp_probe_read.argtypes = [vp, u64, vp, vp]
    lib.mgwfbp_probe_fill.argtypes = [vp, f32, u64, vp]
    lib.mgwfbp_probe_streams.argtypes = [vp, i32, u64, u64, vp, vp]
    lib.mgwfbp_plan_destroy.argtypes = [vp]
    lib.mgwfbp_plan_destroy.restype = None
    lib.mgwfbp_last_error.argtypes = []
    lib.mgwfbp_last_error.restype = C.c_char_p
    for name in EXPORTS + PROBE_EXPORTS:
        if name not in ("mgwfbp_plan_destroy", "mgwfbp_iteration_destroy", "mgwfbp_last_error"):
            getattr(lib, name).restype = i32
    return lib


_lib = _load()


def last_error() -> str:
    return _lib.mgwfbp_last_error().decode()


def _check(rc: int) -> None:
    if rc != OK:
        raise MgwfbpError(rc, last_error())


def _ptr(x) -> int:
    """Device address of a torch tensor, or the integer itself."""
    if x is None:
        return 0
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _stream(stream) -> int:
    """hipStream_t handle: int, torch.cuda.Stream, or None for torch's current stream."""
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return stream
    return int(stream.cuda_stream)


def _ptr_array(items: Optional[Sequence]) -> Optional[C.Array]:
    if items is None:
        return None
    return (C.c_void_p * len(items))(*[_ptr(t) for t in items])


class Plan:
    """Owner of one mgwfbp_plan_t handle."""

    def __init__(self, handle: int, L: int, N: int, p: np.ndarray):
        self._h = C.c_void_p(handle)
        self.L, self.N = L, N
        self.p = p
        self._keep = None
        self._graphs = []          # weak references to the iteration graphs captured from this plan

    # ---- read back -------------------------------------------------------------------
    def info(self) -> dict:
        ng = C.c_int32()
        _check(_lib.mgwfbp_plan_info(self._h, C.byref(ng), None, None, None, None, None))
        gol = np.zeros(self.L, dtype=np.int32)
        off = np.zeros(self.L, dtype=np.uint64)
        ge = np.zeros(ng.value, dtype=np.uint64)
        t, tw = C.c_double(), C.c_double()
        _check(_lib.mgwfbp_plan_info(self._h, C.byref(ng), gol.ctypes.data_as(C.POINTER(C.c_int32)),
                                     off.ctypes.data_as(C.POINTER(C.c_uint64)),
                                     ge.ctypes.data_as(C.POINTER(C.c_uint64)), C.byref(t), C.byref(tw)))
        return {"n_groups": ng.value, "group_of_layer": gol, "offset_in_group": off,
                "group_elems": ge, "t_iter_ms": t.value, "t_iter_wfbp_ms": tw.value}

    def timeline(self) -> dict:
        ng = self.info()["n_groups"]
        mu = np.zeros(self.L)
        gs, gf = np.zeros(ng), np.zeros(ng)
        dp = lambda a: a.ctypes.data_as(C.POINTER(C.c_double))
        _check(_lib.mgwfbp_plan_timeline(self._h, dp(mu), dp(gs), dp(gf)))
        return {"mu_b": mu, "group_start": gs, "group_finish": gf}

    def groups(self) -> List[List[int]]:
        """0-based layers of each group in arrival order (highest first)."""
        inf = self.info()
        out: List[List[int]] = [[] for _ in range(inf["n_groups"])]
        for l in range(self.L - 1, -1, -1):
            out[int(inf["group_of_layer"][l])].append(l)
        return out

    def merged_layers(self) -> List[int]:
        """The set M in the paper's 1-based numbering, descending."""
        gol = self.info()["group_of_layer"]
        return [l + 1 for l in range(self.L - 1, 0, -1) if gol[l] == gol[l - 1]]

    # ---- set-up ----------------------------------------------------------------------
    def set_option(self, key: int, value: int) -> None:
        _check(_lib.mgwfbp_plan_set_option(self._h, key, value))

    def layout(self) -> dict:
        """Segment and tile tables as the kernels would see them (host only, no device needed):
        segments [n][layer, elements, plan offset, group], tiles [n][first segment, segment
        count, start, elements, list, tile length, padding]."""
        ns, nt = C.c_uint64(0), C.c_uint64(0)
        _check(_lib.mgwfbp_plan_layout(self._h, C.byref(ns), None, 0, C.byref(nt), None, 0))
        segs = np.zeros((ns.value, 4), dtype=np.uint64)
        tiles = np.zeros((nt.value, 7), dtype=np.uint64)
        _check(_lib.mgwfbp_plan_layout(self._h, None, segs.ctypes.data, ns.value, None, tiles.ctypes.data, nt.value))
        return {"segments": segs, "tiles": tiles}

    def bind(self, grads: Sequence[Sequence], out: Optional[Sequence] = None,
             w: Optional[Sequence] = None, v: Optional[Sequence] = None) -> None:
        """grads[g][l], out[l], w[l], v[l]: torch CUDA fp32 tensors (or raw device addresses)."""
        if len(grads) != self.N or any(len(r) != self.L for r in grads):
            raise ValueError("grads must be N lists of L tensors")
        for name, lst in (("out", out), ("w", w), ("v", v)):
            if lst is not None and len(lst) != self.L:
                raise ValueError(f"{name} must hold L tensors")
        for lst in list(grads) + [x for x in (out, w, v) if x is not None]:
            for l, t in enumerate(lst):
                if isinstance(t, int):
                    continue
                if not t.is_cuda or str(t.dtype) != "torch.float32" or not t.is_contiguous() \
                        or t.numel() != int(self.p[l]):
                    raise ValueError(f"layer {l}: need a contiguous CUDA fp32 tensor of {int(self.p[l])} elements")
        flat = [t for rep in grads for t in rep]
        _check(_lib.mgwfbp_bind(self._h, _ptr_array(flat), _ptr_array(out), _ptr_array(w),
                                _ptr_array(v)))
        self._keep = (grads, out, w, v)

    def tune(self, stream=None) -> dict:
        """Pick the launch shape of the whole-plan fused reduce pass by timing (see mgwfbp_tune)."""
        idx, ms = C.c_int32(), C.c_double()
        _check(_lib.mgwfbp_tune(self._h, C.c_void_p(_stream(stream)), C.byref(idx), C.byref(ms)))
        return {"candidate": idx.value, "ms_per_launch": ms.value}

    def workspace_bytes(self, group: int = -1) -> int:
        n = C.c_size_t()
        _check(_lib.mgwfbp_workspace_bytes(self._h, group, C.byref(n)))
        return int(n.value)

    # ---- device calls ----------------------------------------------------------------
    @staticmethod
    def _ws(workspace):
        if workspace is None:
            return None, 0
        if isinstance(workspace, tuple):
            return C.c_void_p(workspace[0]), workspace[1]
        return C.c_void_p(int(workspace.data_ptr())), workspace.numel() * workspace.element_size()

    def pack_reduce_unpack(self, group: int = -1, workspace=None, stream=None) -> None:
        ws, nb = self._ws(workspace)
        _check(_lib.mgwfbp_pack_reduce_unpack(self._h, group, ws, nb, C.c_void_p(_stream(stream))))

    def pack_reduce_unpack_static(self, group: int = -1, stream=None) -> None:
        """The materialised path with the library's own static workspace (no allocation)."""
        _check(_lib.mgwfbp_pack_reduce_unpack_static(self._h, group, C.c_void_p(_stream(stream))))

    def step(self, lr: float, momentum: float, group: int = -1, workspace=None, stream=None) -> None:
        ws, nb = self._ws(workspace)
        _check(_lib.mgwfbp_step(self._h, group, lr, momentum, ws, nb, C.c_void_p(_stream(stream))))

    def pack(self, workspace, group: int = -1, stream=None) -> None:
        ws, nb = self._ws(workspace)
        _check(_lib.mgwfbp_pack(self._h, group, ws, nb, C.c_void_p(_stream(stream))))

    def reduce(self, workspace, group: int = -1, stream=None) -> None:
        ws, nb = self._ws(workspace)
        _check(_lib.mgwfbp_reduce(self._h, group, ws, nb, C.c_void_p(_stream(stream))))

    def unpack(self, workspace, group: int = -1, stream=None) -> None:
        ws, nb = self._ws(workspace)
        _check(_lib.mgwfbp_unpack(self._h, group, ws, nb, C.c_void_p(_stream(stream))))

    def pack_reduce(self, merged, group: int = -1, stream=None) -> None:
        ws, nb = self._ws(merged)
        _check(_lib.mgwfbp_pack_reduce(self._h, group, ws, nb, C.c_void_p(_stream(stream))))

    def unpack_update(self, merged, group: int = -1, update: bool = False, lr: float = 0.0,
                      momentum: float = 0.0, stream=None) -> None:
        ws, nb = self._ws(merged)
        _check(_lib.mgwfbp_unpack_update(self._h, group, ws, nb, int(update), lr, momentum,
                                         C.c_void_p(_stream(stream))))

    def run_iteration(self, compute_stream, comm_stream, tb_ms=None, update: bool = False,
                      lr: float = 0.0, momentum: float = 0.0, timeline: bool = True) -> dict:
        """One event-driven iteration (see mgwfbp_run_iteration); returns the measured timeline,
        or only t_iter_ms with timeline=False (no per-group timestamps are taken then).
        comm_stream may be a list of streams (see mgwfbp_run_iteration_streams)."""
        ng = self.info()["n_groups"]
        ready, gs, gf = np.zeros(ng), np.zeros(ng), np.zeros(ng)
        t_iter = C.c_double()
        dp = lambda a: a.ctypes.data_as(C.POINTER(C.c_double))
        tb = None if tb_ms is None else np.ascontiguousarray(tb_ms, dtype=np.float64)
        if tb is not None and tb.shape != (self.L,):
            raise ValueError("tb_ms must have L entries")
        outs = (dp(ready) if timeline else None, dp(gs) if timeline else None,
                dp(gf) if timeline else None, C.byref(t_iter))
        if isinstance(comm_stream, (list, tuple)):
            arr = (C.c_void_p * len(comm_stream))(*[_stream(s) for s in comm_stream])
            _check(_lib.mgwfbp_run_iteration_streams(self._h, None if tb is None else dp(tb), int(update), lr,
                                                     momentum, C.c_void_p(_stream(compute_stream)), arr,
                                                     len(comm_stream), *outs))
        else:
            _check(_lib.mgwfbp_run_iteration(self._h, None if tb is None else dp(tb), int(update), lr, momentum,
                                             C.c_void_p(_stream(compute_stream)), C.c_void_p(_stream(comm_stream)),
                                             *outs))
        if not timeline:
            return {"t_iter_ms": t_iter.value}
        return {"group_ready_ms": ready, "group_start_ms": gs, "group_finish_ms": gf,
                "t_iter_ms": t_iter.value}

    def run_iteration_gated(self, compute_stream, comm_stream, tb_ms=None, update: bool = False,
                            lr: float = 0.0, momentum: float = 0.0, give_up_ms: float = 2000.0) -> float:
        """One iteration with the communication side as a single gated launch; returns t_iter in ms."""
        tb = None if tb_ms is None else np.ascontiguousarray(tb_ms, dtype=np.float64)
        if tb is not None and tb.shape != (self.L,):
            raise ValueError("tb_ms must have L entries")
        t = C.c_double()
        _check(_lib.mgwfbp_run_iteration_gated(
            self._h, None if tb is None else tb.ctypes.data_as(C.POINTER(C.c_double)), int(update), lr, momentum,
            C.c_void_p(_stream(compute_stream)), C.c_void_p(_stream(comm_stream)), give_up_ms, C.byref(t)))
        return t.value

    def streams_side_by_side(self, stream_a, stream_b) -> bool:
        """Does the device run stream_a's kernels while one of stream_b's is still running?"""
        y = C.c_int32()
        _check(_lib.mgwfbp_streams_side_by_side(self._h, C.c_void_p(_stream(stream_a)),
                                                C.c_void_p(_stream(stream_b)), C.byref(y)))
        return bool(y.value)

    def gated_launch(self, arrival: int, update: bool = False, lr: float = 0.0, momentum: float = 0.0,
                     give_up_ms: float = 2000.0, stream=None) -> None:
        _check(_lib.mgwfbp_gated_launch(self._h, int(update), lr, momentum, arrival, give_up_ms,
                                        C.c_void_p(_stream(stream))))

    def gated_signal(self, group: int, arrival: int, stream=None) -> None:
        _check(_lib.mgwfbp_gated_signal(self._h, group, arrival, C.c_void_p(_stream(stream))))

    def gated_gave_up(self) -> bool:
        g = C.c_int32()
        _check(_lib.mgwfbp_gated_gave_up(self._h, C.byref(g)))
        return bool(g.value)

    def gated_workgroups(self, update: bool = False):
        """(workgroups of the gated launch, at most that many per compute unit)"""
        g, per = C.c_uint32(), C.c_uint32()
        _check(_lib.mgwfbp_gated_workgroups(self._h, int(update), C.byref(g), C.byref(per)))
        return g.value, per.value

    def capture_iteration(self, compute_stream, comm_stream, tb_ms=None, update: bool = False,
                          lr: float = 0.0, momentum: float = 0.0) -> "IterationGraph":
        """The iteration of run_iteration captured into a HIP graph (see mgwfbp_iteration_capture)."""
        tb = None if tb_ms is None else np.ascontiguousarray(tb_ms, dtype=np.float64)
        if tb is not None and tb.shape != (self.L,):
            raise ValueError("tb_ms must have L entries")
        h = C.c_void_p()
        _check(_lib.mgwfbp_iteration_capture(
            self._h, None if tb is None else tb.ctypes.data_as(C.POINTER(C.c_double)), int(update), lr,
            momentum, C.c_void_p(_stream(compute_stream)), C.c_void_p(_stream(comm_stream)), C.byref(h)))
        it = IterationGraph(h.value, self)
        self._graphs.append(weakref.ref(it))
        return it

    def destroy(self) -> None:
        for ref in self._graphs:      # a graph must not outlive the tables it points into
            it = ref()
            if it is not None:
                it.destroy()
        self._graphs = []
        if self._h:
            _lib.mgwfbp_plan_destroy(self._h)
            self._h = C.c_void_p(0)
            self._keep = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


class IterationGraph:
    """Owner of one mgwfbp_iteration_t handle; keeps its plan alive."""

    def __init__(self, handle: int, plan: Plan):
        self._h = C.c_void_p(handle)
        self._plan = plan

    def replay(self, stream=None, measure: bool = True):
        """Launch the graph; with measure=True wait and return t_iter in ms, else return None."""
        t = C.c_double()
        _check(_lib.mgwfbp_iteration_replay(self._h, C.c_void_p(_stream(stream)),
                                            C.byref(t) if measure else None))
        return t.value if measure else None

    def destroy(self) -> None:
        if self._h:
            _lib.mgwfbp_iteration_destroy(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def _plan_args(p, tb_ms):
    p_arr = np.ascontiguousarray(p, dtype=np.uint64)
    tb = np.ascontiguousarray(tb_ms, dtype=np.float64)
    if p_arr.ndim != 1 or tb.shape != p_arr.shape:
        raise ValueError("p and tb_ms must be 1-D arrays of the same length")
    return p_arr, tb


def mgwfbp_plan(p, tb_ms, tf_ms: float, a_ms: float, b_ms_per_byte: float, N: int,
                mode: int = MODE_OPTIMAL) -> Plan:
    p_arr, tb = _plan_args(p, tb_ms)
    h = C.c_void_p()
    _check(_lib.mgwfbp_plan(len(p_arr), p_arr.ctypes.data_as(C.POINTER(C.c_uint64)),
                            tb.ctypes.data_as(C.POINTER(C.c_double)), tf_ms, a_ms, b_ms_per_byte,
                            N, mode, C.byref(h)))
    return Plan(h.value, len(p_arr), N, p_arr)


def mgwfbp_plan_explicit(p, tb_ms, tf_ms: float, a_ms: float, b_ms_per_byte: float, N: int,
                         merged_layers: Sequence[int]) -> Plan:
    """merged_layers: the set M in the paper's 1-based numbering (subset of {2..L})."""
    p_arr, tb = _plan_args(p, tb_ms)
    flags = np.zeros(len(p_arr), dtype=np.uint8)
    for l in merged_layers:
        flags[l - 1] = 1
    h = C.c_void_p()
    _check(_lib.mgwfbp_plan_explicit(len(p_arr), p_arr.ctypes.data_as(C.POINTER(C.c_uint64)),
                                     tb.ctypes.data_as(C.POINTER(C.c_double)), tf_ms, a_ms,
                                     b_ms_per_byte, N, flags.ctypes.data_as(C.POINTER(C.c_uint8)),
                                     C.byref(h)))
    return Plan(h.value, len(p_arr), N, p_arr)


def mgwfbp_pack_reduce_unpack(plan: Plan, group: int = -1, workspace=None, stream=None) -> None:
    plan.pack_reduce_unpack(group, workspace, stream)


def mgwfbp_step(plan: Plan, lr: float, momentum: float, group: int = -1, workspace=None,
                stream=None) -> None:
    plan.step(lr, momentum, group, workspace, stream)


TABLE2 = {"binary_tree": 0, "recursive_doubling": 1, "recursive_halving_doubling": 2, "ring": 3}


class ConfinedStream:
    """A HIP stream whose kernels run on the first n_compute_units of the current device only
    (mgwfbp_confined_stream_create), wrapped for torch as `.stream`."""

    def __init__(self, n_compute_units: int):
        import torch

        h = C.c_void_p()
        _check(_lib.mgwfbp_confined_stream_create(n_compute_units, C.byref(h)))
        self._h = h
        self.n_compute_units = n_compute_units
        self.stream = torch.cuda.ExternalStream(h.value)

    def destroy(self) -> None:
        if self._h is not None:
            self.stream.synchronize()
            _check(_lib.mgwfbp_confined_stream_destroy(self._h))
            self._h = None


def mgwfbp_fit_cost(nbytes, ms):
    """Least-squares (a_ms, b_ms_per_byte) of T_ar(M) = a + b*M."""
    x = np.ascontiguousarray(nbytes, dtype=np.float64)
    y = np.ascontiguousarray(ms, dtype=np.float64)
    if x.shape != y.shape or x.ndim != 1:
        raise ValueError("nbytes and ms must be 1-D arrays of the same length")
    a, b = C.c_double(), C.c_double()
    dp = lambda v: v.ctypes.data_as(C.POINTER(C.c_double))
    _check(_lib.mgwfbp_fit_cost(len(x), dp(x), dp(y), C.byref(a), C.byref(b)))
    return a.value, b.value


def mgwfbp_table2_cost(algorithm: str, N: int, alpha_ms: float, beta: float, gamma: float):
    a, b = C.c_double(), C.c_double()
    _check(_lib.mgwfbp_table2_cost(TABLE2[algorithm], N, alpha_ms, beta, gamma, C.byref(a), C.byref(b)))
    return a.value, b.value


def mgwfbp_scaling_curve(p, tb_ms, tf_ms: float, algorithm: str, alpha_ms: float, beta: float,
                         gamma: float, n_workers: Sequence[int], mode: int = MODE_OPTIMAL):
    """(t_iter_ms[], speedup[]) predicted for each worker count."""
    p_arr, tb = _plan_args(p, tb_ms)
    nw = np.ascontiguousarray(n_workers, dtype=np.int32)
    t, s = np.zeros(len(nw)), np.zeros(len(nw))
    dp = lambda v: v.ctypes.data_as(C.POINTER(C.c_double))
    _check(_lib.mgwfbp_scaling_curve(len(p_arr), p_arr.ctypes.data_as(C.POINTER(C.c_uint64)), dp(tb), tf_ms,
                                     TABLE2[algorithm], alpha_ms, beta, gamma, len(nw),
                                     nw.ctypes.data_as(C.POINTER(C.c_int32)), mode, dp(t), dp(s)))
    return t, s


def mgwfbp_probe_copy(src, dst, n_elems: int, stream=None) -> None:
    _check(_lib.mgwfbp_probe_copy(C.c_void_p(_ptr(src)), C.c_void_p(_ptr(dst)), n_elems,
                                  C.c_void_p(_stream(stream))))


def mgwfbp_probe_read(src, n_elems: int, sink, stream=None) -> None:
    _check(_lib.mgwfbp_probe_read(C.c_void_p(_ptr(src)), n_elems, C.c_void_p(_ptr(sink)),
                                  C.c_void_p(_stream(stream))))


def mgwfbp_probe_fill(dst, value: float, n_elems: int, stream=None) -> None:
    _check(_lib.mgwfbp_probe_fill(C.c_void_p(_ptr(dst)), value, n_elems, C.c_void_p(_stream(stream))))


def mgwfbp_probe_streams(src, n_streams: int, stride_elems: int, n_elems: int, dst,
                         stream=None) -> None:
    _check(_lib.mgwfbp_probe_streams(C.c_void_p(_ptr(src)), n_streams, stride_elems, n_elems,
                                     C.c_void_p(_ptr(dst)), C.c_void_p(_stream(stream))))


def raw():
    """The ctypes library object (for tests of the error paths)."""
    return _lib
