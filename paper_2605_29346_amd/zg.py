"""Thin ctypes binding over libzg.so (the C-ABI of include/zg.h): argument marshalling only.

PyTorch is used for device memory and streams; every step of the path runs in the library's HIP
kernels.  There is no fallback: if the library is missing, importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

MAX_HOPS = 8
MAX_FANOUT = 64
LOG_STRIDE = 32

OK, EINVAL, ENOMEM, EHIP, ESTATE = 0, -1, -2, -3, -4
I32, I64 = 0, 1
GRAPH_VALIDATE = 1
PLAN_EAGER, PLAN_REPLACE, PLAN_SAFE_TWIN, PLAN_FUSED_INPUT, PLAN_AUTO_FALLBACK = 1, 2, 4, 8, 16
PLAN_X_ONE_PASS, PLAN_X_TWO_PASS = 32, 64
ENV_MAX, ENV_MODEL, ENV_EXPLICIT, ENV_GRAPH = 0, 1, 2, 3
FLAG_SEED_RANGE, FLAG_SEED_DUP, FLAG_INTERNAL = 1 << 16, 1 << 17, 1 << 18


def FLAG_HOP_OVERFLOW(h: int) -> int:
    return 1 << h


_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libzg.so")

EXPORTS = ["zg_strerror", "zg_last_error", "zg_graph_create", "zg_graph_create_stats", "zg_graph_destroy",
           "zg_graph_degree_histogram", "zg_normal_quantile", "zg_envelope_model", "zg_plan_query", "zg_plan",
           "zg_plan_destroy", "zg_plan_bind_features", "zg_plan_outputs", "zg_step", "zg_gather",
           "zg_aggregate_mean", "zg_overflow_flag", "zg_overflow_clear", "zg_step_safe", "zg_plan_outputs_safe",
           "zg_step_status", "zg_envelope_model_graph", "zg_envelope_from_pilot", "zg_pilot_update", "zg_build_id",
           "zg_calibration_copy", "zg_envelope_model_graph_static", "zg_plan_replay_features", "zg_step_timed"]


class Envelope(C.Structure):
    _fields_ = [("mode", C.c_int32), ("flags", C.c_uint32), ("margin", C.c_double), ("confidence", C.c_double),
                ("iterations", C.c_int64), ("node_caps", C.c_int64 * (MAX_HOPS + 1)),
                ("model_mean", C.c_double * (MAX_HOPS + 1)), ("model_sigma", C.c_double * (MAX_HOPS + 1)),
                ("max_tickets", C.c_int32), ("reserved", C.c_int32)]


class PlanInfo(C.Structure):
    _fields_ = [("num_hops", C.c_int32), ("feat_dim", C.c_int32),
                ("node_cap", C.c_int64 * (MAX_HOPS + 1)), ("edge_cap", C.c_int64 * MAX_HOPS),
                ("maxsg_nodes", C.c_int64 * (MAX_HOPS + 1)),
                ("model_mean", C.c_double * (MAX_HOPS + 1)), ("model_sigma", C.c_double * (MAX_HOPS + 1)),
                ("z", C.c_double),
                ("envelope_bytes", C.c_int64), ("scratch_bytes", C.c_int64), ("workspace_bytes", C.c_int64),
                ("maxsg_envelope_bytes", C.c_int64),
                ("grid_sample", C.c_int32 * MAX_HOPS), ("grid_compact", C.c_int32),
                ("grid_relabel", C.c_int32 * MAX_HOPS), ("grid_gather", C.c_int32), ("grid_aggregate", C.c_int32),
                ("safe_envelope_bytes", C.c_int64)]


class Outputs(C.Structure):
    _fields_ = [("num_hops", C.c_int32), ("feat_dim", C.c_int32),
                ("d_n", C.c_void_p), ("d_E", C.c_void_p), ("d_n_exact", C.c_void_p), ("d_flags", C.c_void_p),
                ("d_S", C.c_void_p),
                ("d_row_ptr", C.c_void_p * MAX_HOPS), ("d_nbr_gid", C.c_void_p * MAX_HOPS),
                ("d_col", C.c_void_p * MAX_HOPS),
                ("node_cap", C.c_int64 * (MAX_HOPS + 1)), ("edge_cap", C.c_int64 * MAX_HOPS),
                ("d_X", C.c_void_p), ("ldx", C.c_int64), ("d_agg", C.c_void_p), ("ld_agg", C.c_int64),
                ("d_log", C.c_void_p), ("log_capacity", C.c_int32), ("d_epoch", C.c_void_p), ("x_row_cap", C.c_int64),
                ("d_active", C.c_void_p), ("x_one_pass", C.c_int32), ("reserved", C.c_int32)]


_lib = None


def lib() -> C.CDLL:
    """The loaded C-ABI library.  A library that is missing, or was built from other sources than the ones beside it,
    is (re)built when hipcc is there; otherwise this raises: there is no fallback path."""
    global _lib
    if _lib is None:
        import torch  # noqa: F401  (first: the library must bind to the HIP runtime PyTorch brings, not load a second one)
        from . import build as _build
        _build.ensure_current()
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it first (__graft_entry__.build()); "
                               "there is no fallback path")
        L = C.CDLL(_LIB_PATH)
        L.zg_build_id.restype = C.c_char_p
        L.zg_build_id.argtypes = []
        want = _build.source_id()
        if want is not None and L.zg_build_id().decode() != want:
            raise RuntimeError(f"{_LIB_PATH} was built from other sources ({L.zg_build_id().decode()} != {want}) and "
                               "hipcc is not available to rebuild it")
        vp, i32, i64, u32, u64, dbl = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_uint64, C.c_double
        P = C.POINTER
        L.zg_strerror.restype = C.c_char_p
        L.zg_strerror.argtypes = [C.c_int]
        L.zg_last_error.restype = C.c_char_p
        L.zg_last_error.argtypes = []
        L.zg_graph_create.argtypes = [P(vp), i64, i64, vp, i32, vp, u32]
        L.zg_graph_create_stats.argtypes = [P(vp), i64, i64, P(i64), P(i64), i64]
        L.zg_graph_destroy.argtypes = [vp]
        L.zg_graph_degree_histogram.argtypes = [vp, P(i64), P(P(i64)), P(P(i64))]
        L.zg_normal_quantile.restype = dbl
        L.zg_normal_quantile.argtypes = [dbl]
        L.zg_envelope_model.argtypes = [P(i64), P(i64), i64, P(i32), i32, i32, i32, P(dbl), P(dbl)]
        L.zg_plan_query.argtypes = [vp, P(i32), i32, i32, P(Envelope), i32, P(PlanInfo)]
        L.zg_plan.argtypes = [P(vp), vp, P(i32), i32, i32, P(Envelope), i32, vp, C.c_size_t, vp]
        L.zg_plan_destroy.argtypes = [vp]
        L.zg_plan_bind_features.argtypes = [vp, vp, i64]
        L.zg_plan_outputs.argtypes = [vp, P(Outputs)]
        L.zg_step.argtypes = [vp, vp, u64, vp]
        L.zg_gather.argtypes = [vp, vp, i64, i32, vp, i64, vp]
        L.zg_aggregate_mean.argtypes = [vp, i32, vp, i64, i32, vp, i64, vp]
        L.zg_overflow_flag.argtypes = [vp, P(vp)]
        L.zg_overflow_clear.argtypes = [vp, vp]
        L.zg_step_safe.argtypes = [vp, vp, u64, vp]
        L.zg_plan_outputs_safe.argtypes = [vp, P(Outputs)]
        L.zg_step_status.argtypes = [vp, P(u32), P(u32)]
        L.zg_envelope_model_graph.argtypes = [vp, P(i32), i32, i32, i32, vp, vp, C.c_size_t, vp, P(dbl), P(dbl)]
        L.zg_envelope_model_graph_static.argtypes = [vp, P(i32), i32, i32, i32, vp, vp, vp]
        L.zg_envelope_from_pilot.argtypes = [P(i64), i32, dbl, u32, P(Envelope)]
        L.zg_pilot_update.argtypes = [vp, P(i64), vp]
        L.zg_calibration_copy.argtypes = [vp, vp, C.c_size_t, vp]
        L.zg_plan_replay_features.argtypes = [vp, i32, vp]
        L.zg_step_timed.argtypes = [vp, vp, u64, vp, vp, vp]
        for name in EXPORTS:
            if name not in ("zg_strerror", "zg_last_error", "zg_normal_quantile", "zg_build_id"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


class ZgError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        L = lib()
        super().__init__(f"{L.zg_strerror(status).decode()} ({status}): {L.zg_last_error().decode()}")


def _check(status: int) -> None:
    if status != OK:
        raise ZgError(status)


def normal_quantile(p: float) -> float:
    return float(lib().zg_normal_quantile(p))


def envelope_model(degrees: Sequence[int], counts: Sequence[int], fanouts: Sequence[int], batch: int,
                   with_replacement: bool = False):
    """Lemma 1 mean and sigma of n_h for h = 0..H from a degree histogram (host only)."""
    n = len(degrees)
    H = len(fanouts)
    d = (C.c_int64 * n)(*degrees)
    c = (C.c_int64 * n)(*counts)
    f = (C.c_int32 * H)(*fanouts)
    mean = (C.c_double * (MAX_HOPS + 1))()
    sigma = (C.c_double * (MAX_HOPS + 1))()
    _check(lib().zg_envelope_model(d, c, n, f, H, batch, int(with_replacement), mean, sigma))
    return list(mean[: H + 1]), list(sigma[: H + 1])


def make_envelope(mode: int = ENV_MAX, *, flags: int = 0, margin: float = -1.0, confidence: float = 0.0,
                  iterations: int = 0, node_caps: Optional[Sequence[int]] = None, model_mean: Optional[Sequence[float]] = None,
                  model_sigma: Optional[Sequence[float]] = None, max_tickets: int = 0) -> Envelope:
    e = Envelope()
    e.mode, e.flags, e.margin, e.confidence, e.iterations = mode, flags, margin, confidence, iterations
    e.max_tickets = max_tickets
    if node_caps is not None:
        for h, c in enumerate(node_caps):
            e.node_caps[h] = int(c)
    for dst, src in ((e.model_mean, model_mean), (e.model_sigma, model_sigma)):
        if src is not None:
            for h, x in enumerate(src):
                dst[h] = float(x)
    return e


_hip = None


def new_stream() -> int:
    """A fresh non-blocking hipStream_t (default priority) as an integer handle.  Streams made this way land on
    distinct hardware queues, so steps of different plans issued on them overlap."""
    global _hip
    if _hip is None:
        _hip = C.CDLL("libamdhip64.so")
        _hip.hipStreamCreateWithFlags.argtypes = [C.POINTER(C.c_void_p), C.c_uint]
        _hip.hipStreamSynchronize.argtypes = [C.c_void_p]
        _hip.hipStreamDestroy.argtypes = [C.c_void_p]
    s = C.c_void_p()
    rc = _hip.hipStreamCreateWithFlags(C.byref(s), 1)  # hipStreamNonBlocking
    if rc != 0:
        raise RuntimeError(f"hipStreamCreateWithFlags failed with {rc}")
    return s.value


def _stream_ptr(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def graph_model(graph: "Graph", fanouts: Sequence[int], batch: int, *, with_replacement: bool = False, seed_prob=None,
                stream=None):
    """Mean and sigma of n_h from the graph-aware size model (computed on the device, synchronises)."""
    import torch
    H = len(fanouts)
    f = (C.c_int32 * H)(*fanouts)
    mean = (C.c_double * (MAX_HOPS + 1))()
    sigma = (C.c_double * (MAX_HOPS + 1))()
    nbytes = 12 * graph.num_nodes + 576
    temp = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
    base = (temp.data_ptr() + 255) // 256 * 256
    sp = None
    if seed_prob is not None:
        assert seed_prob.is_cuda and seed_prob.dtype == torch.float32 and seed_prob.numel() == graph.num_nodes
        sp = seed_prob.contiguous()
    _check(lib().zg_envelope_model_graph(graph._h, f, H, batch, int(with_replacement), sp.data_ptr() if sp is not None else None,
                                         base, nbytes, _stream_ptr(stream), mean, sigma))
    return list(mean[: H + 1]), list(sigma[: H + 1])


def graph_model_static(graph: "Graph", fanouts: Sequence[int], batch: int, out, *, with_replacement: bool = False,
                       seed_prob=None, stream=None) -> None:
    """The graph-aware size model on the library's static scratch: allocates nothing, does not synchronise; `out` (float64
    CUDA tensor, 2 * (H + 1) elements) receives mean[0..H] then sigma[0..H] once the stream gets there."""
    H = len(fanouts)
    f = (C.c_int32 * H)(*fanouts)
    assert out.is_cuda and out.element_size() == 8 and out.numel() >= 2 * (H + 1) and out.is_contiguous()
    _check(lib().zg_envelope_model_graph_static(graph._h, f, H, batch, int(with_replacement),
                                                seed_prob.data_ptr() if seed_prob is not None else None, _stream_ptr(stream),
                                                out.data_ptr()))


def graph_envelope(graph: "Graph", fanouts: Sequence[int], batch: int, *, margin: float = 0.20, confidence: float = 0.999,
                   iterations: int = 100_000, flags: int = 0, seed_prob=None) -> Envelope:
    """A ZG_ENV_GRAPH request: mean and sigma from the graph-aware size model; the library's planner turns them into
    caps (the lemma's margin / z-sigma formula)."""
    mean, sigma = graph_model(graph, fanouts, batch, with_replacement=bool(flags & PLAN_REPLACE), seed_prob=seed_prob)
    return make_envelope(ENV_GRAPH, flags=flags, margin=margin, confidence=confidence, iterations=iterations,
                         model_mean=mean, model_sigma=sigma)


def pilot_envelope(graph: "Graph", fanouts: Sequence[int], batch: int, seed_batches, keys, *, margin: float = 0.20,
                   flags: int = 0) -> Envelope:
    """Plan-time pilot (the paper's warm-up iterations): run the given mini-batches once on a worst-case plan; the
    library tracks the largest realised n_h per hop (zg_pilot_update) and turns it into an explicit envelope with
    `margin` head-room (zg_envelope_from_pilot)."""
    H = len(fanouts)
    plan = Plan(graph, fanouts, batch, make_envelope(ENV_MAX, flags=flags & PLAN_REPLACE))
    largest = (C.c_int64 * (MAX_HOPS + 1))()
    try:
        for seeds, key in zip(seed_batches, keys):
            plan.step(seeds, key)
            _check(lib().zg_pilot_update(plan._h, largest, _stream_ptr(None)))
    finally:
        plan.close()
    env = Envelope()
    _check(lib().zg_envelope_from_pilot(largest, H, margin, flags, C.byref(env)))
    return env


def calibration_copy(src, dst, stream=None) -> None:
    """dst = src as one plain streaming kernel of the library (reads and writes src.numel() * itemsize bytes)."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(lib().zg_calibration_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream_ptr(stream)))


class Graph:
    """CSR graph on the device (torch tensors: int32/int64 offsets, int32 indices), borrowed by the library."""

    def __init__(self, offsets=None, indices=None, *, validate: bool = False, _handle=None, num_nodes=None):
        import torch
        self._h = C.c_void_p()
        if _handle is not None:
            self._h = _handle
            self.num_nodes = num_nodes
            self.offsets = self.indices = None
            return
        assert offsets.is_cuda and indices.is_cuda and offsets.is_contiguous() and indices.is_contiguous()
        assert offsets.dtype in (torch.int32, torch.int64) and indices.dtype == torch.int32
        self.offsets, self.indices = offsets, indices  # keep alive
        self.num_nodes = offsets.numel() - 1
        _check(lib().zg_graph_create(C.byref(self._h), self.num_nodes, indices.numel(), offsets.data_ptr(),
                                     I64 if offsets.dtype == torch.int64 else I32, indices.data_ptr(),
                                     GRAPH_VALIDATE if validate else 0))

    @classmethod
    def from_degree_histogram(cls, degrees: Sequence[int], counts: Sequence[int]) -> "Graph":
        """Statistics-only handle (no device arrays): good for plan_query on a machine without a GPU."""
        n = len(degrees)
        d = (C.c_int64 * n)(*degrees)
        c = (C.c_int64 * n)(*counts)
        h = C.c_void_p()
        nn = sum(counts)
        ne = sum(int(a) * int(b) for a, b in zip(degrees, counts))
        _check(lib().zg_graph_create_stats(C.byref(h), nn, ne, d, c, n))
        return cls(_handle=h, num_nodes=nn)

    def degree_histogram(self):
        n = C.c_int64()
        d = C.POINTER(C.c_int64)()
        c = C.POINTER(C.c_int64)()
        _check(lib().zg_graph_degree_histogram(self._h, C.byref(n), C.byref(d), C.byref(c)))
        return [d[i] for i in range(n.value)], [c[i] for i in range(n.value)]

    def plan_query(self, fanouts: Sequence[int], batch: int, env: Optional[Envelope] = None, feat_dim: int = 0) -> PlanInfo:
        env = env or make_envelope()
        H = len(fanouts)
        f = (C.c_int32 * H)(*fanouts)
        info = PlanInfo()
        _check(lib().zg_plan_query(self._h, f, H, batch, C.byref(env), feat_dim, C.byref(info)))
        return info

    def close(self):
        if self._h:
            lib().zg_graph_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


@dataclass
class StepResult:
    """Host copies of one step's outputs (for checks; the hot path never makes them)."""
    n: List[int]
    E: List[int]
    n_exact: List[int]
    flags: int
    S: "object"
    row_ptr: List["object"]
    nbr_gid: List["object"]
    col: List["object"]
    X: Optional["object"]
    agg: Optional["object"]


class Plan:
    """A provisioned execution envelope + captured step for (graph, fanouts, batch)."""

    def __init__(self, graph: Graph, fanouts: Sequence[int], batch: int, env: Optional[Envelope] = None,
                 feat_dim: int = 0, stream=None, workspace_slack: int = 0):
        import torch
        self.graph = graph
        self.fanouts = tuple(int(f) for f in fanouts)
        self.batch = batch
        self.env = env or make_envelope()
        self.feat_dim = feat_dim
        self.info = graph.plan_query(self.fanouts, batch, self.env, feat_dim)
        self.workspace = torch.empty(self.info.workspace_bytes + workspace_slack, dtype=torch.uint8, device="cuda")
        assert self.workspace.data_ptr() % 256 == 0
        H = len(self.fanouts)
        f = (C.c_int32 * H)(*self.fanouts)
        self._h = C.c_void_p()
        _check(lib().zg_plan(C.byref(self._h), graph._h, f, H, batch, C.byref(self.env), feat_dim,
                             self.workspace.data_ptr(), self.info.workspace_bytes, _stream_ptr(stream)))
        self.out = Outputs()
        _check(lib().zg_plan_outputs(self._h, C.byref(self.out)))
        self.features = None

    @property
    def num_hops(self) -> int:
        return len(self.fanouts)

    def bind_features(self, feat) -> None:
        import torch
        assert feat.is_cuda and feat.dtype == torch.float32 and feat.dim() == 2 and feat.stride(1) == 1
        self.features = feat
        _check(lib().zg_plan_bind_features(self._h, feat.data_ptr(), feat.stride(0)))
        _check(lib().zg_plan_outputs(self._h, C.byref(self.out)))  # (which kernel writes X depends on the table)

    def step(self, seeds, rng_key: int, stream=None) -> None:
        """Enqueue one mini-batch (seeds: int32 CUDA tensor of `batch` distinct ids); returns at once."""
        _check(lib().zg_step(self._h, seeds.data_ptr(), C.c_uint64(rng_key & 0xFFFFFFFFFFFFFFFF), _stream_ptr(stream)))

    def step_timed(self, seeds, rng_key: int, event_before, event_after, stream=None) -> None:
        """One step enqueued kernel by kernel, the two events (torch.cuda.Event with timing, already recorded once so
        that their handles exist) recorded right before and after its aggregation launch."""
        _check(lib().zg_step_timed(self._h, seeds.data_ptr(), C.c_uint64(rng_key & 0xFFFFFFFFFFFFFFFF), _stream_ptr(stream),
                                   C.c_void_p(event_before.cuda_event), C.c_void_p(event_after.cuda_event)))

    def step_safe(self, seeds, rng_key: int, stream=None) -> None:
        """Replay the same mini-batch on the worst-case twin (plan made with PLAN_SAFE_TWIN)."""
        _check(lib().zg_step_safe(self._h, seeds.data_ptr(), C.c_uint64(rng_key & 0xFFFFFFFFFFFFFFFF), _stream_ptr(stream)))

    def step_status(self):
        """(steps finished, flags of the last finished step) read from pinned host memory: no device call."""
        done, flags = C.c_uint32(), C.c_uint32()
        _check(lib().zg_step_status(self._h, C.byref(done), C.byref(flags)))
        return done.value, flags.value

    def safe_view(self) -> "Plan":
        """A Plan-like object whose views/read_step address the twin's outputs."""
        import copy
        twin = copy.copy(self)
        twin.out = Outputs()
        _check(lib().zg_plan_outputs_safe(self._h, C.byref(twin.out)))
        twin._h = C.c_void_p()  # the view owns nothing
        return twin

    def gather(self, feat, out, stream=None) -> None:
        _check(lib().zg_gather(self._h, feat.data_ptr(), feat.stride(0), feat.shape[1], out.data_ptr(), out.stride(0),
                               _stream_ptr(stream)))

    def aggregate_mean(self, hop: int, x, out, stream=None) -> None:
        _check(lib().zg_aggregate_mean(self._h, hop, x.data_ptr(), x.stride(0), x.shape[1], out.data_ptr(),
                                       out.stride(0), _stream_ptr(stream)))

    def replay_features(self, which: int, stream=None) -> None:
        """Re-enqueue the step's gather (0) or aggregation (1) launch on the last step's state (for timing)."""
        _check(lib().zg_plan_replay_features(self._h, which, _stream_ptr(stream)))

    def overflow_flag_ptr(self) -> int:
        p = C.c_void_p()
        _check(lib().zg_overflow_flag(self._h, C.byref(p)))
        return p.value

    def overflow_clear(self, stream=None) -> None:
        _check(lib().zg_overflow_clear(self._h, _stream_ptr(stream)))

    # ---- views into the workspace (no copies) ----
    def _view(self, ptr: int, count: int, dtype):
        import torch
        off = ptr - self.workspace.data_ptr()
        nbytes = count * torch.empty(0, dtype=dtype).element_size()
        assert 0 <= off and off + nbytes <= self.workspace.numel()
        return self.workspace[off: off + nbytes].view(dtype)

    def view_counts(self):
        import torch
        H = self.num_hops
        return (self._view(self.out.d_n, H + 1, torch.int32), self._view(self.out.d_E, H, torch.int32),
                self._view(self.out.d_n_exact, H + 1, torch.int32), self._view(self.out.d_flags, 1, torch.int32))

    def view_S(self):
        import torch
        return self._view(self.out.d_S, self.out.node_cap[self.num_hops], torch.int32)

    def view_block(self, h: int):
        import torch
        return (self._view(self.out.d_row_ptr[h], self.out.node_cap[h] + 1, torch.int32),
                self._view(self.out.d_nbr_gid[h], self.out.edge_cap[h], torch.int32),
                self._view(self.out.d_col[h], self.out.edge_cap[h], torch.int32))

    def _rows_view(self, ptr: int, rows: int, ld: int):
        """[rows, ld] strided fp32 view starting at a device address inside the workspace (the last row may end
        before a full stride when two matrices interleave)."""
        import torch
        off = (ptr - self.workspace.data_ptr()) // 4
        flat = self.workspace.view(torch.float32)
        width = min(ld, flat.numel() - off - (rows - 1) * ld) if rows > 0 else ld
        return torch.as_strided(flat, (rows, width), (ld, 1), off)

    def view_X(self):
        return self._rows_view(self.out.d_X, self.out.x_row_cap, self.out.ldx)

    def view_agg(self):
        return self._rows_view(self.out.d_agg, self.out.node_cap[self.num_hops - 1], self.out.ld_agg)

    def view_log(self):
        import torch
        return self._view(self.out.d_log, self.out.log_capacity * LOG_STRIDE, torch.int32).view(-1, LOG_STRIDE)

    def epoch(self) -> int:
        import torch
        return int(self._view(self.out.d_epoch, 1, torch.int32).item())

    def view_active(self):
        """Device word of a PLAN_AUTO_FALLBACK plan: 1 if the last step's valid outputs are the twin's."""
        import torch
        return self._view(self.out.d_active, 1, torch.int32)

    def read_step(self, with_features: bool = True) -> StepResult:
        """Synchronise and copy the last step's outputs to the host (numpy)."""
        import torch
        torch.cuda.synchronize()
        H = self.num_hops
        n_t, E_t, nx_t, fl_t = self.view_counts()
        n = [int(x) for x in n_t.cpu().tolist()]
        E = [int(x) for x in E_t.cpu().tolist()]
        nx = [int(x) for x in nx_t.cpu().tolist()]
        flags = int(fl_t.cpu().item()) & 0xFFFFFFFF
        S = self.view_S()[: n[H]].cpu().numpy()
        rp, nb, col = [], [], []
        for h in range(H):
            r, b, c = self.view_block(h)
            rp.append(r[: n[h] + 1].cpu().numpy())
            nb.append(b[: E[h]].cpu().numpy())
            col.append(c[: E[h]].cpu().numpy())
        X = agg = None
        if with_features and self.feat_dim > 0 and self.features is not None:
            x_rows = n[H - 1] if (self.env.flags & PLAN_FUSED_INPUT) else n[H]
            X = self.view_X()[: x_rows, : self.feat_dim].cpu().numpy()
            agg = self.view_agg()[: n[H - 1], : self.feat_dim].cpu().numpy()
        return StepResult(n, E, nx, flags, S, rp, nb, col, X, agg)

    def close(self):
        if self._h:
            lib().zg_plan_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
