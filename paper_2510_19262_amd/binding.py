"""ctypes marshalling for the railsched C ABI (include/railsched.h).

PyTorch is used for device memory and streams only: tensors are allocated with
torch, their data pointers and the current HIP stream are handed to the library.
There is no fallback: if librailsched.so cannot be loaded, importing a symbol
works but the first call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "librailsched.so")
_lib = None

EXPORTS = (
    "railsched_version", "railsched_strerror", "railsched_check_capacity", "railsched_route_topk",
    "railsched_traffic_matrix_workspace_bytes", "railsched_traffic_matrix",
    "railsched_route_traffic_workspace_bytes", "railsched_route_traffic",
    "railsched_chunk_sort_workspace_bytes", "railsched_chunk_sort", "railsched_lpt_spray_workspace_bytes", "railsched_lpt_spray",
    "railsched_lpt_spray_chunkwise",
    "railsched_eval_workspace_bytes", "railsched_eval", "railsched_schedule_workspace_bytes", "railsched_schedule", "railsched_schedule_static", "railsched_transpose_matrix", "railsched_assign_policy",
    "railsched_port_round_robin_workspace_bytes", "railsched_port_round_robin",
)


class RailschedError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


class _TopoStruct(C.Structure):
    _fields_ = [("nodes", C.c_int32), ("rails", C.c_int32), ("chunk_bytes", C.c_int64),
                ("rail_bw_Bps", C.c_int64), ("include_intra_node", C.c_int32), ("reserved", C.c_int32)]


@dataclass(frozen=True)
class Topo:
    """M nodes x N rails, chunk size C, rail rate R2 (Section 4.1 of the paper)."""
    nodes: int
    rails: int
    chunk_bytes: int
    rail_bw_Bps: int = 50_000_000_000
    include_intra_node: int = 0

    @property
    def G(self) -> int:
        return self.nodes * self.rails

    def c(self) -> _TopoStruct:
        return _TopoStruct(self.nodes, self.rails, self.chunk_bytes, self.rail_bw_Bps, self.include_intra_node, 0)


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Load librailsched.so (building it first only if it is absent)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build as _build
        _build.build(force=True)
    lib = C.CDLL(_LIB_PATH)           # torch is imported above, so its HIP runtime is the one resolved
    lib.railsched_version.restype = C.c_char_p
    lib.railsched_strerror.restype = C.c_char_p
    lib.railsched_strerror.argtypes = [C.c_int]
    P, I32, I64, SZ = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    TP = C.POINTER(_TopoStruct)
    lib.railsched_route_topk.argtypes = [P, I64, I32, I32, P, P]
    lib.railsched_check_capacity.argtypes = [P, I32, TP, I64, C.POINTER(C.c_int64), P]
    lib.railsched_traffic_matrix_workspace_bytes.argtypes = [I32, I64, I32, TP]
    lib.railsched_traffic_matrix_workspace_bytes.restype = SZ
    lib.railsched_traffic_matrix.argtypes = [P, I32, I64, I32, P, I32, I32, I64, TP, P, P, SZ, P]
    lib.railsched_route_traffic_workspace_bytes.argtypes = [I32, I64, I32, I32, TP]
    lib.railsched_route_traffic_workspace_bytes.restype = SZ
    lib.railsched_route_traffic.argtypes = [P, I32, I64, I32, I32, P, I32, I64, TP, P, P, P, SZ, P]
    lib.railsched_chunk_sort_workspace_bytes.argtypes = [I32, TP]
    lib.railsched_chunk_sort_workspace_bytes.restype = SZ
    lib.railsched_chunk_sort.argtypes = [P, I32, TP, P, P, P, P, I64, P, SZ, P]
    lib.railsched_lpt_spray_workspace_bytes.argtypes = [I32, TP]
    lib.railsched_lpt_spray_workspace_bytes.restype = SZ
    lib.railsched_lpt_spray.argtypes = [P, P, I32, TP, I64, P, P, P, SZ, P]
    lib.railsched_lpt_spray_chunkwise.argtypes = [P, P, I32, TP, I64, P, P, P, SZ, P]
    lib.railsched_eval_workspace_bytes.argtypes = [I32, TP]
    lib.railsched_eval_workspace_bytes.restype = SZ
    lib.railsched_eval.argtypes = [P, P, P, P, P, I32, TP, I64, P, P, P, SZ, P]
    lib.railsched_schedule_workspace_bytes.argtypes = [I32, TP]
    lib.railsched_schedule_workspace_bytes.restype = SZ
    lib.railsched_schedule.argtypes = [P, I32, TP, P, P, P, P, I64, P, P, P, P, P, SZ, P]
    lib.railsched_schedule_static.argtypes = [P, I32, TP, P, P, P, P, I64, P, P, P, P, P]
    lib.railsched_schedule_static.restype = C.c_int
    lib.railsched_transpose_matrix.argtypes = [P, I32, TP, P, P]
    lib.railsched_assign_policy.argtypes = [I32, C.c_uint64, P, P, P, I32, TP, I64, P, P, P]
    lib.railsched_port_round_robin_workspace_bytes.argtypes = [I32, TP, I64]
    lib.railsched_port_round_robin_workspace_bytes.restype = SZ
    lib.railsched_port_round_robin.argtypes = [P, P, I32, TP, I32, I64, P, P, SZ, P]
    lib.railsched_port_round_robin.restype = C.c_int
    lib.railsched_transpose_matrix.restype = C.c_int
    lib.railsched_assign_policy.restype = C.c_int
    for fn in ("railsched_check_capacity", "railsched_route_topk", "railsched_traffic_matrix", "railsched_route_traffic",
               "railsched_chunk_sort", "railsched_lpt_spray", "railsched_lpt_spray_chunkwise", "railsched_eval",
               "railsched_schedule"):
        getattr(lib, fn).restype = C.c_int
    _lib = lib
    return lib


def version() -> str:
    return load().railsched_version().decode()


def strerror(status: int) -> str:
    return load().railsched_strerror(int(status)).decode()


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t


def _check(status: int, where: str):
    if status != 0:
        raise RailschedError(status, where)


def _ws(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def check_capacity(chunk_off: torch.Tensor, batch: int, topo: Topo, capacity: int) -> int:
    """Waits for the current stream, returns the chunk count; raises RailschedError(RAILSCHED_ERR_CAPACITY) if it
    exceeds `capacity` (the one synchronising call of the library)."""
    _dev(chunk_off, torch.int64, "chunk_off")
    total = C.c_int64(0)
    t = topo.c()
    rc = load().railsched_check_capacity(_ptr(chunk_off), batch, C.byref(t), capacity, C.byref(total), _stream())
    if rc != 0:
        err = RailschedError(rc, "railsched_check_capacity")
        err.total = int(total.value)
        raise err
    return int(total.value)


# ---------------------------------------------------------------------------------- stage 1
def route_topk(logits: torch.Tensor, k: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """[rows][E] fp32 -> [rows][k] int32 indices of the k largest logits, lowest index on ties."""
    _dev(logits, torch.float32, "logits")
    rows, E = logits.shape
    if out is None:
        out = torch.empty((rows, k), dtype=torch.int32, device=logits.device)
    _dev(out, torch.int32, "out")
    _check(load().railsched_route_topk(_ptr(logits), rows, E, k, _ptr(out), _stream()), "railsched_route_topk")
    return out


# ---------------------------------------------------------------------------------- stage 2
def traffic_matrix_workspace_bytes(batch: int, tokens_per_gpu: int, k: int, topo: Topo) -> int:
    t = topo.c()
    return int(load().railsched_traffic_matrix_workspace_bytes(batch, tokens_per_gpu, k, C.byref(t)))


def traffic_matrix(topk_idx: torch.Tensor, batch: int, tokens_per_gpu: int, expert_gpu: torch.Tensor,
                   payload_bytes: int, topo: Topo, out: Optional[torch.Tensor] = None,
                   ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """top-k indices + expert placement -> D1 [batch][G][G] int64 bytes."""
    _dev(topk_idx, torch.int32, "topk_idx")
    _dev(expert_gpu, torch.int32, "expert_gpu")
    k = topk_idx.shape[1]
    E, R = expert_gpu.shape
    G = topo.G
    if topk_idx.shape[0] != batch * G * tokens_per_gpu:
        raise ValueError("topk_idx must hold batch*G*tokens_per_gpu rows")
    if out is None:
        out = torch.empty((batch, G, G), dtype=torch.int64, device=topk_idx.device)
    _dev(out, torch.int64, "out")
    if ws is None:
        ws = _ws(traffic_matrix_workspace_bytes(batch, tokens_per_gpu, k, topo), topk_idx.device)
    t = topo.c()
    _check(load().railsched_traffic_matrix(_ptr(topk_idx), batch, tokens_per_gpu, k, _ptr(expert_gpu), E, R,
                                           payload_bytes, C.byref(t), _ptr(out), _ptr(ws), ws.numel(), _stream()),
           "railsched_traffic_matrix")
    return out


def route_traffic_workspace_bytes(batch: int, tokens_per_gpu: int, E: int, k: int, topo: Topo) -> int:
    t = topo.c()
    return int(load().railsched_route_traffic_workspace_bytes(batch, tokens_per_gpu, E, k, C.byref(t)))


def route_traffic(logits: torch.Tensor, k: int, batch: int, tokens_per_gpu: int, expert_gpu: torch.Tensor,
                  payload_bytes: int, topo: Topo, want_idx: bool = True,
                  out: Optional[Tuple[Optional[torch.Tensor], torch.Tensor]] = None, ws: Optional[torch.Tensor] = None):
    """Stages 1 and 2 in one call: (topk_idx or None, D1)."""
    _dev(logits, torch.float32, "logits")
    _dev(expert_gpu, torch.int32, "expert_gpu")
    rows, E = logits.shape
    E2, R = expert_gpu.shape
    G = topo.G
    if E2 != E:
        raise ValueError("expert_gpu must have one row per expert")
    if rows != batch * G * tokens_per_gpu:
        raise ValueError("logits must hold batch*G*tokens_per_gpu rows")
    if out is None:
        idx = torch.empty((rows, k), dtype=torch.int32, device=logits.device) if want_idx else None
        D1 = torch.empty((batch, G, G), dtype=torch.int64, device=logits.device)
    else:
        idx, D1 = out
    if idx is not None:
        _dev(idx, torch.int32, "topk_idx")
    _dev(D1, torch.int64, "D1")
    if ws is None:
        ws = _ws(route_traffic_workspace_bytes(batch, tokens_per_gpu, E, k, topo), logits.device)
    t = topo.c()
    _check(load().railsched_route_traffic(_ptr(logits), batch, tokens_per_gpu, E, k, _ptr(expert_gpu), R, payload_bytes,
                                          C.byref(t), None if idx is None else _ptr(idx), _ptr(D1), _ptr(ws), ws.numel(),
                                          _stream()),
           "railsched_route_traffic")
    return idx, D1


# ---------------------------------------------------------------------------------- stage 3
def chunk_sort_workspace_bytes(batch: int, topo: Topo) -> int:
    t = topo.c()
    return int(load().railsched_chunk_sort_workspace_bytes(batch, C.byref(t)))


def eval_workspace_bytes(batch: int, topo: Topo) -> int:
    t = topo.c()
    return int(load().railsched_eval_workspace_bytes(batch, C.byref(t)))


def chunk_count(D1: torch.Tensor, topo: Topo, ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Count query: chunk_off [batch*M+1] int64 only."""
    _dev(D1, torch.int64, "D1")
    batch = D1.shape[0]
    off = torch.empty(batch * topo.nodes + 1, dtype=torch.int64, device=D1.device)
    if ws is None:
        ws = _ws(chunk_sort_workspace_bytes(batch, topo), D1.device)
    t = topo.c()
    _check(load().railsched_chunk_sort(_ptr(D1), batch, C.byref(t), _ptr(off), None, None, None, 0,
                                       _ptr(ws), ws.numel(), _stream()), "railsched_chunk_sort(count)")
    return off


def chunk_total(D1: torch.Tensor, topo: Topo, ws: Optional[torch.Tensor] = None) -> int:
    """Count query followed by the one synchronising call: the number of chunks stage 3 will produce for D1."""
    off = chunk_count(D1, topo, ws)
    return check_capacity(off, D1.shape[0], topo, (1 << 62))


def chunk_sort(D1: torch.Tensor, topo: Topo, want_perm: bool = True, capacity: Optional[int] = None,
               out=None, ws: Optional[torch.Tensor] = None):
    """D1 -> (chunk_off, chunk_w, chunk_flow, perm|None), every instance sorted by descending weight.

    Without `capacity` a count query runs first and the host waits for the total (one
    synchronisation) to size the record arrays.  With `capacity` (and optionally preallocated
    `out` = (chunk_off, chunk_w, chunk_flow, perm)) the call is fully asynchronous; the record
    arrays are left untouched if the total exceeds the capacity.
    """
    _dev(D1, torch.int64, "D1")
    batch = D1.shape[0]
    dev = D1.device
    if ws is None:
        ws = _ws(chunk_sort_workspace_bytes(batch, topo), dev)
    if capacity is None:
        capacity = chunk_total(D1, topo, ws)
    if out is None:
        off = torch.empty(batch * topo.nodes + 1, dtype=torch.int64, device=dev)
        w = torch.empty(max(capacity, 1), dtype=torch.int32, device=dev)
        flow = torch.empty(max(capacity, 1), dtype=torch.int32, device=dev)
        perm = torch.empty(max(capacity, 1), dtype=torch.int32, device=dev) if want_perm else None
    else:
        off, w, flow, perm = out
    t = topo.c()
    _check(load().railsched_chunk_sort(_ptr(D1), batch, C.byref(t), _ptr(off), _ptr(w), _ptr(flow), _ptr(perm),
                                       capacity, _ptr(ws), ws.numel(), _stream()), "railsched_chunk_sort")
    return off, w, flow, perm


# ---------------------------------------------------------------------------------- stage 4
def lpt_spray_workspace_bytes(batch: int, topo: Topo) -> int:
    t = topo.c()
    return int(load().railsched_lpt_spray_workspace_bytes(batch, C.byref(t)))


def lpt_spray(chunk_off: torch.Tensor, chunk_w: torch.Tensor, batch: int, topo: Topo, out=None, chunkwise: bool = False,
              capacity: Optional[int] = None, ws="auto"):
    """Greedy least-loaded-rail assignment per instance -> (rail uint8 [capacity], S int64 [batch][M][N]).
    chunkwise=True calls railsched_lpt_spray_chunkwise (same result, no closed-form periods).
    capacity = records chunk_w and rail hold (default: the length of chunk_w).
    ws: workspace tensor, None for none, "auto" to allocate one here (instances are then taken longest first)."""
    _dev(chunk_off, torch.int64, "chunk_off")
    if chunk_w.dtype not in (torch.int32, torch.uint32):
        raise ValueError("chunk_w must be a 32-bit integer tensor")
    if capacity is None:
        capacity = chunk_w.numel()
    if out is None:
        rail = torch.empty(max(capacity, 1), dtype=torch.uint8, device=chunk_off.device)
        S = torch.empty((batch, topo.nodes, topo.rails), dtype=torch.int64, device=chunk_off.device)
    else:
        rail, S = out
    if min(chunk_w.numel(), rail.numel()) < capacity:
        raise ValueError("chunk_w and rail must hold `capacity` records")
    t = topo.c()
    if isinstance(ws, str):
        ws = _ws(lpt_spray_workspace_bytes(batch, topo), chunk_off.device)
    fn = load().railsched_lpt_spray_chunkwise if chunkwise else load().railsched_lpt_spray
    _check(fn(_ptr(chunk_off), _ptr(chunk_w), batch, C.byref(t), capacity, _ptr(rail), _ptr(S), _ptr(ws),
              0 if ws is None else ws.numel(), _stream()), "railsched_lpt_spray")
    return rail, S


# ---------------------------------------------------------------------------------- stage 5
def eval(chunk_off, chunk_w, chunk_flow, rail, S, batch: int, topo: Topo, out=None,  # noqa: A001
         ws: Optional[torch.Tensor] = None, capacity: Optional[int] = None):
    """Receive loads R [batch][M][N] and stats [batch][8] (see include/railsched.h).
    capacity = records the per-chunk arrays hold (default: the shortest of them)."""
    dev = chunk_off.device
    if capacity is None:
        capacity = min(chunk_w.numel(), chunk_flow.numel(), rail.numel())
    if out is None:
        R = torch.empty((batch, topo.nodes, topo.rails), dtype=torch.int64, device=dev)
        stats = torch.empty((batch, 8), dtype=torch.int64, device=dev)
    else:
        R, stats = out
    if ws is None:
        ws = _ws(eval_workspace_bytes(batch, topo), dev)
    t = topo.c()
    _check(load().railsched_eval(_ptr(chunk_off), _ptr(chunk_w), _ptr(chunk_flow), _ptr(rail), _ptr(S), batch,
                                 C.byref(t), capacity, _ptr(R), _ptr(stats), _ptr(ws), ws.numel(), _stream()), "railsched_eval")
    return R, stats


evaluate = eval

POLICIES = {"nic_direct": 0, "flow_hash": 1, "random_spray": 2, "round_robin": 3}


def transpose_matrix(D1: torch.Tensor, topo: Topo, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Traffic of the second all-to-all: D1T[b][d][s] = D1[b][s][d]."""
    _dev(D1, torch.int64, "D1")
    if out is None:
        out = torch.empty_like(D1)
    t = topo.c()
    _check(load().railsched_transpose_matrix(_ptr(D1), D1.shape[0], C.byref(t), _ptr(out), _stream()),
           "railsched_transpose_matrix")
    return out


def assign_policy(policy, seed: int, chunk_off, chunk_w, chunk_flow, batch: int, topo: Topo, out=None,
                  capacity: Optional[int] = None):
    """Rails under a comparison scheme ("nic_direct", "flow_hash", "random_spray", "round_robin") -> (rail, S)."""
    if capacity is None:
        capacity = min(chunk_w.numel(), chunk_flow.numel())
    if out is None:
        rail = torch.empty(max(capacity, 1), dtype=torch.uint8, device=chunk_off.device)
        S = torch.empty((batch, topo.nodes, topo.rails), dtype=torch.int64, device=chunk_off.device)
    else:
        rail, S = out
    t = topo.c()
    pol = POLICIES[policy] if isinstance(policy, str) else int(policy)
    if rail.numel() < capacity:
        raise ValueError("rail must hold `capacity` records")
    _check(load().railsched_assign_policy(pol, seed, _ptr(chunk_off), _ptr(chunk_w), _ptr(chunk_flow), batch, C.byref(t),
                                          capacity, _ptr(rail), _ptr(S), _stream()), "railsched_assign_policy")
    return rail, S


# ---------------------------------------------------------------------------------- whole path
def schedule_workspace_bytes(batch: int, topo: Topo) -> int:
    t = topo.c()
    return int(load().railsched_schedule_workspace_bytes(batch, C.byref(t)))


def schedule(D1: torch.Tensor, topo: Topo, capacity: int, want_perm: bool = True, out=None, ws: Optional[torch.Tensor] = None):
    """Stages 3-5 in one call: (chunk_off, chunk_w, chunk_flow, perm, rail, S, R, stats)."""
    _dev(D1, torch.int64, "D1")
    batch = D1.shape[0]
    M, N = topo.nodes, topo.rails
    dev = D1.device
    if out is None:
        n = max(capacity, 1)
        out = (torch.empty(batch * M + 1, dtype=torch.int64, device=dev), torch.empty(n, dtype=torch.int32, device=dev),
               torch.empty(n, dtype=torch.int32, device=dev), torch.empty(n, dtype=torch.int32, device=dev) if want_perm else None,
               torch.empty(n, dtype=torch.uint8, device=dev), torch.empty((batch, M, N), dtype=torch.int64, device=dev),
               torch.empty((batch, M, N), dtype=torch.int64, device=dev), torch.empty((batch, 8), dtype=torch.int64, device=dev))
    off, w, flow, perm, rail, S, R, stats = out
    if ws is None:
        ws = _ws(schedule_workspace_bytes(batch, topo), dev)
    t = topo.c()
    _check(load().railsched_schedule(_ptr(D1), batch, C.byref(t), _ptr(off), _ptr(w), _ptr(flow), _ptr(perm), capacity, _ptr(rail),
                                     _ptr(S), _ptr(R), _ptr(stats), _ptr(ws), ws.numel(), _stream()), "railsched_schedule")
    return out


STATIC_SCRATCH_BYTES = 4 << 20


def schedule_static(D1: torch.Tensor, topo: Topo, capacity: int, out):
    """railsched_schedule_static: stages 3-5 with the library's own static scratch buffer instead of a workspace.
    `out` = (chunk_off, chunk_w, chunk_flow, perm or None, rail, S, R, stats), preallocated: nothing is allocated here."""
    _dev(D1, torch.int64, "D1")
    off, w, flow, perm, rail, S, R, stats = out
    t = topo.c()
    _check(load().railsched_schedule_static(_ptr(D1), D1.shape[0], C.byref(t), _ptr(off), _ptr(w), _ptr(flow), _ptr(perm), capacity,
                                            _ptr(rail), _ptr(S), _ptr(R), _ptr(stats), _stream()), "railsched_schedule_static")
    return out


class Plan:
    """Preallocated buffers for repeated passes of the whole path over same-shaped batches
    (no allocation and no host synchronisation inside step())."""

    def __init__(self, topo: Topo, batch: int, capacity: int, device, rows: int = 0, k: int = 0, want_perm: bool = True):
        self.topo, self.batch, self.capacity = topo, batch, capacity
        M, N, G = topo.nodes, topo.rails, topo.G
        i32, i64 = torch.int32, torch.int64
        self.topk_idx = torch.empty((rows, k), dtype=i32, device=device) if rows else None
        self.D1 = torch.empty((batch, G, G), dtype=i64, device=device)
        self.chunk_off = torch.empty(batch * M + 1, dtype=i64, device=device)
        self.chunk_w = torch.empty(max(capacity, 1), dtype=i32, device=device)
        self.chunk_flow = torch.empty(max(capacity, 1), dtype=i32, device=device)
        self.perm = torch.empty(max(capacity, 1), dtype=i32, device=device) if want_perm else None
        self.rail = torch.empty(max(capacity, 1), dtype=torch.uint8, device=device)
        self.S = torch.empty((batch, M, N), dtype=i64, device=device)
        self.R = torch.empty((batch, M, N), dtype=i64, device=device)
        self.stats = torch.empty((batch, 8), dtype=i64, device=device)
        self.ws_sort = _ws(chunk_sort_workspace_bytes(batch, topo), device)
        self.ws_eval = _ws(eval_workspace_bytes(batch, topo), device)
        self.ws_sched = _ws(schedule_workspace_bytes(batch, topo), device)
        self.ws_lpt = _ws(lpt_spray_workspace_bytes(batch, topo), device)
        self.ws_tm = None

    def route(self, logits, tokens_per_gpu, expert_gpu, payload_bytes):
        k = self.topk_idx.shape[1]
        if self.ws_tm is None:
            self.ws_tm = _ws(traffic_matrix_workspace_bytes(self.batch, tokens_per_gpu, k, self.topo), logits.device)
        route_topk(logits, k, out=self.topk_idx)
        traffic_matrix(self.topk_idx, self.batch, tokens_per_gpu, expert_gpu, payload_bytes, self.topo, out=self.D1, ws=self.ws_tm)
        return self.D1

    def schedule_one_call(self, D1=None):
        """Stages 3-5 through railsched_schedule (same outputs as schedule())."""
        D1 = self.D1 if D1 is None else D1
        schedule(D1, self.topo, self.capacity, out=(self.chunk_off, self.chunk_w, self.chunk_flow, self.perm, self.rail, self.S,
                                                   self.R, self.stats), ws=self.ws_sched)
        return self.stats

    def schedule(self, D1=None):
        """Stages 3-5 through the three calls; like schedule_one_call, fills S, R and stats with -1 (and touches no
        per-chunk array) if the batch yields more chunks than the plan's capacity."""
        D1 = self.D1 if D1 is None else D1
        chunk_sort(D1, self.topo, capacity=self.capacity,
                   out=(self.chunk_off, self.chunk_w, self.chunk_flow, self.perm), ws=self.ws_sort)
        lpt_spray(self.chunk_off, self.chunk_w, self.batch, self.topo, out=(self.rail, self.S), capacity=self.capacity, ws=self.ws_lpt)
        eval(self.chunk_off, self.chunk_w, self.chunk_flow, self.rail, self.S, self.batch, self.topo,
             out=(self.R, self.stats), ws=self.ws_eval, capacity=self.capacity)
        return self.stats


def port_round_robin(chunk_off, rail, batch: int, topo: Topo, ports: int, capacity: Optional[int] = None, out=None, ws=None):
    """Port (queue pair) of every chunk: round robin per rail inside each instance -> uint8 [chunks]."""
    if capacity is None:
        capacity = rail.numel()
    t = topo.c()
    if ws is None:
        ws = _ws(load().railsched_port_round_robin_workspace_bytes(batch, C.byref(t), capacity), chunk_off.device)
    port = torch.empty(max(capacity, 1), dtype=torch.uint8, device=chunk_off.device) if out is None else out
    _check(load().railsched_port_round_robin(_ptr(chunk_off), _ptr(rail), batch, C.byref(t), ports, capacity, _ptr(port),
                                             _ptr(ws), ws.numel(), _stream()), "railsched_port_round_robin")
    return port
