"""ctypes face of the CPU oracle (oracle/railsched_oracle.c).

TEST INFRASTRUCTURE ONLY: the test-suite, the smoke check and the CPU-baseline
leg of the benchmark call this; the GPU library never does and shares no code
with it.  Arrays are numpy, host memory; every function restates one step of
the pipeline as the paper defines it (citations are in the C file).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from fractions import Fraction

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "railsched_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (about a second)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fopenmp", "-fPIC",
                               "-shared", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_chunk_split.restype = C.c_int64
        _lib.oracle_opt_makespan.restype = C.c_int64
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def num_threads() -> int:
    return lib().oracle_num_threads()


def set_threads(n: int) -> int:
    """Threads of the oracle's parallel loops from now on (n < 1: all the runtime offers); returns the count in force."""
    return lib().oracle_set_threads(int(n))


def route_topk(logits: np.ndarray, k: int) -> np.ndarray:
    logits = _chk(logits, np.float32)
    rows, E = logits.shape
    out = np.empty((rows, k), dtype=np.int32)
    rc = lib().oracle_route_topk(_p(logits), C.c_int64(rows), E, k, _p(out))
    if rc:
        raise ValueError(f"oracle_route_topk rc={rc}")
    return out


def traffic_matrix(topk_idx, batch, tokens_per_gpu, expert_gpu, payload_bytes, M, N) -> np.ndarray:
    topk_idx = _chk(topk_idx, np.int32)
    expert_gpu = _chk(expert_gpu, np.int32)
    E, R = expert_gpu.shape
    k = topk_idx.shape[1]
    G = M * N
    assert topk_idx.shape[0] == batch * G * tokens_per_gpu
    D1 = np.empty((batch, G, G), dtype=np.int64)
    rc = lib().oracle_traffic_matrix(_p(topk_idx), batch, C.c_int64(tokens_per_gpu), k, _p(expert_gpu),
                                     E, R, C.c_int64(payload_bytes), M, N, _p(D1))
    if rc:
        raise ValueError(f"oracle_traffic_matrix rc={rc}")
    return D1


def domain_matrix(D1mat, M, N) -> np.ndarray:
    D1mat = _chk(D1mat, np.int64)
    D2 = np.empty((M, M), dtype=np.int64)
    lib().oracle_domain_matrix(_p(D1mat), M, N, _p(D2))
    return D2


def chunk_split(D1mat, M, N, chunk_bytes, node, include_intra=0):
    """Canonical (unsorted) chunk list of one (matrix, node) instance: (w, flow)."""
    D1mat = _chk(D1mat, np.int64)
    n = lib().oracle_chunk_split(_p(D1mat), M, N, C.c_int64(chunk_bytes), include_intra, node, None, None)
    w = np.empty(n, dtype=np.uint32)
    flow = np.empty(n, dtype=np.uint32)
    lib().oracle_chunk_split(_p(D1mat), M, N, C.c_int64(chunk_bytes), include_intra, node, _p(w), _p(flow))
    return w, flow


def sort_desc(w, flow):
    """Stable descending sort; returns (w, flow, perm) as new arrays."""
    w = np.array(w, dtype=np.uint32, copy=True)
    flow = np.array(flow, dtype=np.uint32, copy=True)
    perm = np.empty(w.shape[0], dtype=np.uint32)
    rc = lib().oracle_sort_desc(C.c_int64(w.shape[0]), _p(w), _p(flow), _p(perm))
    if rc:
        raise MemoryError
    return w, flow, perm


def lpt(w, N, heap: bool = False):
    """Greedy least-loaded-rail assignment of the weights in the given order: (rail, L)."""
    w = _chk(w, np.uint32)
    rail = np.empty(w.shape[0], dtype=np.uint8)
    L = np.empty(N, dtype=np.int64)
    fn = lib().oracle_lpt_heap if heap else lib().oracle_lpt
    fn(C.c_int64(w.shape[0]), _p(w), N, _p(rail), _p(L))
    return rail, L


def opt_makespan(w, N) -> int:
    w = _chk(w, np.uint32)
    assert N ** len(w) <= 20_000_000, "brute force is for tiny inputs"
    return int(lib().oracle_opt_makespan(len(w), _p(w), N))


def eval_matrix(chunk_off, w, flow, rail, M, N):
    """One matrix: (Ssum, R, stats[8]).  chunk_off holds the matrix's M+1 offsets."""
    chunk_off = _chk(chunk_off, np.int64)
    Ssum = np.empty((M, N), dtype=np.int64)
    R = np.empty((M, N), dtype=np.int64)
    stats = np.empty(8, dtype=np.int64)
    lib().oracle_eval(_p(chunk_off), _p(_chk(w, np.uint32)), _p(_chk(flow, np.uint32)),
                      _p(_chk(rail, np.uint8)), M, N, _p(Ssum), _p(R), _p(stats))
    return Ssum, R, stats


def schedule_matrix_by_node(D1mat, M, N, chunk_bytes, include_intra=0):
    """One whole matrix, one source node at a time (records of a node are dropped once its loads are added):
    (chunk_off [M+1], S [M][N], R [M][N], stats [8])."""
    D1mat = _chk(D1mat, np.int64)
    off = np.empty(M + 1, dtype=np.int64)
    S = np.empty((M, N), dtype=np.int64)
    R = np.empty((M, N), dtype=np.int64)
    stats = np.empty(8, dtype=np.int64)
    rc = lib().oracle_schedule_matrix_by_node(_p(D1mat), M, N, C.c_int64(chunk_bytes), include_intra, _p(off), _p(S), _p(R), _p(stats))
    if rc:
        raise MemoryError("oracle_schedule_matrix_by_node")
    return off, S, R, stats


# ---------------------------------------------------------------- batched
def chunk_count_batch(D1, M, N, chunk_bytes, include_intra=0) -> np.ndarray:
    D1 = _chk(D1, np.int64)
    batch = D1.shape[0]
    off = np.empty(batch * M + 1, dtype=np.int64)
    lib().oracle_chunk_count_batch(_p(D1), batch, M, N, C.c_int64(chunk_bytes), include_intra, _p(off))
    return off


def chunk_sort_batch(D1, M, N, chunk_bytes, include_intra=0, want_perm=True):
    """(chunk_off, w, flow, perm) for every (matrix, node) instance of the batch."""
    D1 = _chk(D1, np.int64)
    batch = D1.shape[0]
    off = chunk_count_batch(D1, M, N, chunk_bytes, include_intra)
    total = int(off[-1])
    w = np.empty(total, dtype=np.uint32)
    flow = np.empty(total, dtype=np.uint32)
    perm = np.empty(total, dtype=np.uint32) if want_perm else None
    rc = lib().oracle_chunk_sort_batch(_p(D1), batch, M, N, C.c_int64(chunk_bytes), include_intra,
                                       _p(off), _p(w), _p(flow), _p(perm))
    if rc:
        raise RuntimeError(f"oracle_chunk_sort_batch rc={rc}")
    return off, w, flow, perm


def lpt_batch(chunk_off, w, batch, M, N):
    chunk_off = _chk(chunk_off, np.int64)
    w = _chk(w, np.uint32)
    rail = np.empty(w.shape[0], dtype=np.uint8)
    S = np.empty((batch, M, N), dtype=np.int64)
    lib().oracle_lpt_batch(_p(chunk_off), _p(w), batch, M, N, _p(rail), _p(S))
    return rail, S


def eval_batch(chunk_off, w, flow, rail, batch, M, N):
    chunk_off = _chk(chunk_off, np.int64)
    Ssum = np.empty((batch, M, N), dtype=np.int64)
    R = np.empty((batch, M, N), dtype=np.int64)
    stats = np.empty((batch, 8), dtype=np.int64)
    lib().oracle_eval_batch(_p(chunk_off), _p(_chk(w, np.uint32)), _p(_chk(flow, np.uint32)),
                            _p(_chk(rail, np.uint8)), batch, M, N, _p(Ssum), _p(R), _p(stats))
    return Ssum, R, stats


def transpose_batch(D1) -> np.ndarray:
    """Traffic of the second all-to-all: every matrix transposed."""
    D1 = _chk(D1, np.int64)
    out = np.empty_like(D1)
    lib().oracle_transpose_batch(_p(D1), D1.shape[0], C.c_int64(D1.shape[1]), _p(out))
    return out


POLICIES = {"nic_direct": 0, "flow_hash": 1, "random_spray": 2, "round_robin": 3}


def assign_policy(policy, seed, chunk_off, w, flow, batch, M, N):
    """Rail of every chunk under one of the comparison schemes: (rail, S)."""
    chunk_off = _chk(chunk_off, np.int64)
    w = _chk(w, np.uint32)
    rail = np.empty(w.shape[0], dtype=np.uint8)
    S = np.empty((batch, M, N), dtype=np.int64)
    rc = lib().oracle_assign_policy(POLICIES[policy] if isinstance(policy, str) else int(policy), C.c_uint64(seed),
                                    _p(chunk_off), _p(w), _p(_chk(flow, np.uint32)), batch, M, N, _p(rail), _p(S))
    if rc:
        raise ValueError(f"oracle_assign_policy rc={rc}")
    return rail, S


def port_round_robin(chunk_off, rail, batch, M, N, P) -> np.ndarray:
    """Port (queue pair) of every chunk: round robin per rail inside each instance."""
    chunk_off = _chk(chunk_off, np.int64)
    rail = _chk(rail, np.uint8)
    port = np.empty(rail.shape[0], dtype=np.uint8)
    lib().oracle_port_round_robin(_p(chunk_off), _p(rail), batch, M, N, P, _p(port))
    return port


# ---------------------------------------------------------------- derived, exact
def load_mse(L, normalized: bool = False) -> Fraction:
    """Algorithm 2 step 6: mu = mean load, MSE = (1/N) sum (L_j - mu)^2, as an exact
    rational.  normalized=True divides by (N-1)*mu^2, the MSE of "all load on one
    rail", giving a 0-1 scale; the paper prints no formula for its normalisation."""
    L = [int(x) for x in L]
    N = len(L)
    mu = Fraction(sum(L), N)
    mse = sum((Fraction(x) - mu) ** 2 for x in L) / N
    if normalized:
        return mse / ((N - 1) * mu * mu) if N > 1 and mu != 0 else Fraction(0)
    return mse
