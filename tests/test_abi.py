"""Host-side checks of the C ABI that need no GPU: the shared library loads, exports every
symbol the header declares, and rejects bad arguments before anything is launched."""
import ctypes as C
import os
import re

import pytest

import paper_2510_19262_amd as rs
from paper_2510_19262_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "railsched.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(railsched_[a-z_0-9]+)\s*\(", text)))


def test_header_and_library_agree():
    lib = rs.load()
    names = _declared()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n
    assert "gfx950" in rs.version()
    assert rs.strerror(0) == "ok" and "workspace" in rs.strerror(-5)


def _topo(M=4, N=4, Cb=4096, intra=0, reserved=0):
    t = binding._TopoStruct(M, N, Cb, 1, intra, reserved)
    return t


P = C.c_void_p
FAKE = P(0x1000)      # never dereferenced: validation fails first


def test_route_topk_validation():
    lib = rs.load()
    assert lib.railsched_route_topk(FAKE, -1, 8, 2, FAKE, None) == -1
    assert lib.railsched_route_topk(FAKE, 10, 0, 1, FAKE, None) == -1
    assert lib.railsched_route_topk(FAKE, 10, 8, 9, FAKE, None) == -1
    assert lib.railsched_route_topk(FAKE, 10, 8, 0, FAKE, None) == -1
    assert lib.railsched_route_topk(FAKE, 10, 2048, 2, FAKE, None) == -3
    assert lib.railsched_route_topk(None, 10, 8, 2, FAKE, None) == -2
    assert lib.railsched_route_topk(FAKE, 10, 8, 2, None, None) == -2
    assert lib.railsched_route_topk(None, 0, 8, 2, None, None) == 0      # nothing to do


def test_topology_validation():
    lib = rs.load()
    for t, want in ((_topo(M=0), -1), (_topo(N=0), -1), (_topo(Cb=0), -1), (_topo(reserved=1), -1), (_topo(intra=2), -1),
                    (_topo(N=65), -3), (_topo(M=4096, N=8), -3), (_topo(Cb=1 << 32), -3)):
        assert lib.railsched_lpt_spray(FAKE, FAKE, 1, C.byref(t), 10, FAKE, FAKE, None, 0, None) == want
        assert lib.railsched_chunk_sort_workspace_bytes(1, C.byref(t)) == 0
        assert lib.railsched_eval_workspace_bytes(1, C.byref(t)) == 0
    assert lib.railsched_lpt_spray(FAKE, FAKE, 1, None, 10, FAKE, FAKE, None, 0, None) == -2


def test_traffic_matrix_validation():
    lib = rs.load()
    t = _topo()
    need = lib.railsched_traffic_matrix_workspace_bytes(1, 100_000, 2, C.byref(t))
    assert need >= 4 * 16 * 16 * (200_000 // 8192) and need % 256 == 0                 # several slices per pair
    assert lib.railsched_traffic_matrix_workspace_bytes(1, 10, 2, C.byref(t)) == 256     # one slice per pair: nothing needed
    assert lib.railsched_traffic_matrix_workspace_bytes(-1, 10, 2, C.byref(t)) == 0
    assert lib.railsched_traffic_matrix_workspace_bytes(1, 10, 0, C.byref(t)) == 0
    f = lib.railsched_traffic_matrix   # (idx, batch, tokens_per_gpu, k, expert_gpu, E, R, payload, topo, D1, ws, ws_bytes, stream)
    assert f(FAKE, -1, 10, 2, FAKE, 8, 2, 1024, C.byref(t), FAKE, FAKE, 256, None) == -1
    assert f(FAKE, 1, 10, 0, FAKE, 8, 2, 1024, C.byref(t), FAKE, FAKE, 256, None) == -1
    assert f(FAKE, 1, 10, 2, FAKE, 8, 0, 1024, C.byref(t), FAKE, FAKE, 256, None) == -1
    assert f(FAKE, 1, 10, 2, FAKE, 8, 2, -5, C.byref(t), FAKE, FAKE, 256, None) == -1
    assert f(FAKE, 1, 1 << 31, 2, FAKE, 8, 2, 1024, C.byref(t), FAKE, FAKE, 256, None) == -3
    assert f(FAKE, 1, 10, 2, None, 8, 2, 1024, C.byref(t), FAKE, FAKE, 256, None) == -2
    assert f(FAKE, 1, 10, 2, FAKE, 8, 2, 1024, C.byref(t), None, FAKE, 256, None) == -2
    assert f(FAKE, 1, 100_000, 2, FAKE, 8, 2, 1024, C.byref(t), FAKE, None, need, None) == -5
    assert f(FAKE, 1, 100_000, 2, FAKE, 8, 2, 1024, C.byref(t), FAKE, FAKE, need - 256, None) == -5
    assert f(FAKE, 1, 100_000, 2, FAKE, 8, 2, 1024, C.byref(t), FAKE, P(0x1001), need, None) == -5
    assert f(FAKE, 0, 10, 2, FAKE, 8, 2, 1024, C.byref(t), FAKE, FAKE, 256, None) == 0


def test_check_capacity_validation():
    lib = rs.load()
    t = _topo()
    total = C.c_int64(-7)
    f = lib.railsched_check_capacity   # (chunk_off, batch, topo, capacity, h_total, stream)
    assert f(None, 1, C.byref(t), 10, C.byref(total), None) == -2
    assert f(FAKE, -1, C.byref(t), 10, C.byref(total), None) == -1
    assert f(FAKE, 1, C.byref(t), -1, C.byref(total), None) == -1
    assert f(FAKE, 1, None, 10, C.byref(total), None) == -2
    assert total.value == -7                                              # untouched on an argument error
    assert "chunks" in rs.strerror(-4)


def test_route_traffic_validation():
    lib = rs.load()
    t = _topo()
    need = lib.railsched_route_traffic_workspace_bytes(1, 10_000, 8, 2, C.byref(t))
    assert need >= 4 * 16 * 16 * (10_000 // 4096) and need % 256 == 0
    assert lib.railsched_route_traffic_workspace_bytes(1, 10, 8, 2, C.byref(t)) == 256     # one slice per pair: nothing needed
    assert lib.railsched_route_traffic_workspace_bytes(1, 1_000, 16, 2, C.byref(t)) == 256
    assert lib.railsched_route_traffic_workspace_bytes(-1, 10, 8, 2, C.byref(t)) == 0
    assert lib.railsched_route_traffic_workspace_bytes(1, 10, 8, 0, C.byref(t)) == 0
    f = lib.railsched_route_traffic   # (logits, batch, tokens_per_gpu, E, k, expert_gpu, R, payload, topo, idx, D1, ws, ws_bytes, stream)
    assert f(FAKE, -1, 10, 8, 2, FAKE, 2, 1024, C.byref(t), FAKE, FAKE, FAKE, need, None) == -1
    assert f(FAKE, 1, 10, 8, 9, FAKE, 2, 1024, C.byref(t), FAKE, FAKE, FAKE, need, None) == -1
    assert f(FAKE, 1, 10, 8, 2, FAKE, 0, 1024, C.byref(t), FAKE, FAKE, FAKE, need, None) == -1
    assert f(FAKE, 1, 10, 8, 2, FAKE, 2, -1, C.byref(t), FAKE, FAKE, FAKE, need, None) == -1
    assert f(FAKE, 1, 10, 2048, 2, FAKE, 2, 1024, C.byref(t), FAKE, FAKE, FAKE, need, None) == -3
    assert f(FAKE, 1, 1 << 31, 8, 2, FAKE, 2, 1024, C.byref(t), FAKE, FAKE, FAKE, need, None) == -3
    assert f(None, 1, 10, 8, 2, FAKE, 2, 1024, C.byref(t), FAKE, FAKE, FAKE, need, None) == -2
    assert f(FAKE, 1, 10, 8, 2, None, 2, 1024, C.byref(t), FAKE, FAKE, FAKE, need, None) == -2
    assert f(FAKE, 1, 10, 8, 2, FAKE, 2, 1024, C.byref(t), FAKE, None, FAKE, need, None) == -2
    assert f(FAKE, 1, 10, 16, 2, FAKE, 2, 1024, C.byref(t), None, FAKE, FAKE, need, None) == -2   # wide rows need the index array
    assert f(FAKE, 1, 10, 8, 2, FAKE, 2, 1024, None, FAKE, FAKE, FAKE, need, None) == -2
    assert f(FAKE, 1, 10_000, 8, 2, FAKE, 2, 1024, C.byref(t), FAKE, FAKE, None, need, None) == -5
    assert f(FAKE, 1, 10_000, 8, 2, FAKE, 2, 1024, C.byref(t), FAKE, FAKE, FAKE, need - 256, None) == -5
    assert f(FAKE, 1, 10_000, 8, 2, FAKE, 2, 1024, C.byref(t), FAKE, FAKE, P(0x1001), need, None) == -5
    assert f(FAKE, 0, 10, 8, 2, FAKE, 2, 1024, C.byref(t), FAKE, FAKE, FAKE, need, None) == 0


def test_chunk_sort_and_eval_validation():
    lib = rs.load()
    t = _topo()
    need = lib.railsched_chunk_sort_workspace_bytes(2, C.byref(t))
    assert need > 0 and need % 256 == 0
    cs = lib.railsched_chunk_sort
    assert cs(FAKE, -1, C.byref(t), FAKE, FAKE, FAKE, FAKE, 10, FAKE, need, None) == -1
    assert cs(FAKE, 2, C.byref(t), FAKE, FAKE, FAKE, FAKE, -1, FAKE, need, None) == -1
    assert cs(FAKE, 2, C.byref(t), None, FAKE, FAKE, FAKE, 10, FAKE, need, None) == -2
    assert cs(None, 2, C.byref(t), FAKE, FAKE, FAKE, FAKE, 10, FAKE, need, None) == -2
    assert cs(FAKE, 2, C.byref(t), FAKE, FAKE, None, FAKE, 10, FAKE, need, None) == -2
    assert cs(FAKE, 2, C.byref(t), FAKE, FAKE, FAKE, FAKE, 10, None, need, None) == -5
    assert cs(FAKE, 2, C.byref(t), FAKE, FAKE, FAKE, FAKE, 10, FAKE, need - 1, None) == -5
    assert cs(FAKE, 2, C.byref(t), FAKE, FAKE, FAKE, FAKE, 10, P(0x1001), need, None) == -5
    big = _topo(M=64, N=32)                                              # N*G = 65536 flows per instance
    assert cs(FAKE, 1, C.byref(big), FAKE, FAKE, FAKE, FAKE, 10, FAKE, 1 << 40, None) == -3
    ev = lib.railsched_eval
    need = lib.railsched_eval_workspace_bytes(2, C.byref(t))
    assert need > 0
    assert ev(FAKE, FAKE, FAKE, FAKE, FAKE, -1, C.byref(t), 10, FAKE, FAKE, FAKE, need, None) == -1
    assert ev(FAKE, FAKE, FAKE, FAKE, FAKE, 2, C.byref(t), -1, FAKE, FAKE, FAKE, need, None) == -1
    assert ev(FAKE, FAKE, FAKE, FAKE, None, 2, C.byref(t), 10, FAKE, FAKE, FAKE, need, None) == -2
    assert ev(FAKE, FAKE, FAKE, FAKE, FAKE, 2, C.byref(t), 10, None, FAKE, FAKE, need, None) == -2
    assert ev(FAKE, FAKE, None, FAKE, FAKE, 2, C.byref(t), 10, FAKE, FAKE, FAKE, need, None) == -2
    assert ev(FAKE, FAKE, FAKE, FAKE, FAKE, 2, C.byref(t), 10, FAKE, FAKE, FAKE, need - 1, None) == -5
    assert ev(FAKE, FAKE, FAKE, FAKE, FAKE, 0, C.byref(t), 10, FAKE, FAKE, FAKE, need, None) == 0
    lp = lib.railsched_lpt_spray   # (chunk_off, chunk_w, batch, topo, capacity, rail, S, ws, ws_bytes, stream)
    assert lp(FAKE, FAKE, 0, C.byref(t), 10, FAKE, FAKE, None, 0, None) == 0
    assert lp(None, FAKE, 1, C.byref(t), 10, FAKE, FAKE, None, 0, None) == -2
    assert lp(FAKE, FAKE, 1, C.byref(t), -1, FAKE, FAKE, None, 0, None) == -1
    assert lp(FAKE, None, 1, C.byref(t), 10, FAKE, FAKE, None, 0, None) == -2     # records without arrays
    assert lib.railsched_lpt_spray_chunkwise(FAKE, FAKE, 1, C.byref(t), 10, None, FAKE, None, 0, None) == -2
    need_l = lib.railsched_lpt_spray_workspace_bytes(2, C.byref(t))
    assert need_l >= 4 * 2 * 4 + 4 and need_l % 256 == 0 and lib.railsched_lpt_spray_workspace_bytes(-1, C.byref(t)) == 0
    assert lp(FAKE, FAKE, 2, C.byref(t), 10, FAKE, FAKE, FAKE, need_l - 1, None) == -5      # a workspace is optional, but not a short one
    assert lp(FAKE, FAKE, 2, C.byref(t), 10, FAKE, FAKE, P(0x1001), need_l, None) == -5


def test_extras_validation():
    lib = rs.load()
    t = _topo()
    tr = lib.railsched_transpose_matrix
    assert tr(FAKE, -1, C.byref(t), P(0x2000), None) == -1
    assert tr(None, 1, C.byref(t), P(0x2000), None) == -2
    assert tr(FAKE, 1, C.byref(t), FAKE, None) == -1           # in place is refused
    assert tr(FAKE, 0, C.byref(t), FAKE, None) == 0
    ap = lib.railsched_assign_policy
    assert ap(4, 0, FAKE, FAKE, FAKE, 1, C.byref(t), 10, FAKE, FAKE, None) == -1
    assert ap(-1, 0, FAKE, FAKE, FAKE, 1, C.byref(t), 10, FAKE, FAKE, None) == -1
    assert ap(0, 0, FAKE, FAKE, FAKE, 1, C.byref(t), -1, FAKE, FAKE, None) == -1
    assert ap(0, 0, None, FAKE, FAKE, 1, C.byref(t), 10, FAKE, FAKE, None) == -2
    assert ap(0, 0, FAKE, FAKE, FAKE, 1, C.byref(t), 10, FAKE, None, None) == -2
    assert ap(0, 0, FAKE, FAKE, FAKE, 0, C.byref(t), 10, FAKE, FAKE, None) == 0


def test_port_round_robin_validation():
    lib = rs.load()
    t = _topo()
    need = lib.railsched_port_round_robin_workspace_bytes(2, C.byref(t), 100000)
    assert need > 0 and need % 256 == 0
    f = lib.railsched_port_round_robin
    assert f(FAKE, FAKE, 2, C.byref(t), 0, 10, FAKE, FAKE, need, None) == -1
    assert f(FAKE, FAKE, 2, C.byref(t), 257, 10, FAKE, FAKE, need, None) == -3
    assert f(FAKE, FAKE, 2, C.byref(t), 4, -1, FAKE, FAKE, need, None) == -1
    assert f(None, FAKE, 2, C.byref(t), 4, 10, FAKE, FAKE, need, None) == -2
    assert f(FAKE, FAKE, 2, C.byref(t), 4, 10, None, FAKE, need, None) == -2
    assert f(FAKE, FAKE, 2, C.byref(t), 4, 100000, FAKE, FAKE, need - 1, None) == -5
    assert f(FAKE, FAKE, 0, C.byref(t), 4, 10, FAKE, FAKE, need, None) == 0


def test_binding_rejects_host_tensors():
    import torch
    with pytest.raises(ValueError):
        rs.route_topk(torch.zeros((4, 8)), 2)


def test_schedule_validation():
    lib = rs.load()
    t = _topo()
    need = lib.railsched_schedule_workspace_bytes(2, C.byref(t))
    assert need >= lib.railsched_chunk_sort_workspace_bytes(2, C.byref(t)) + lib.railsched_eval_workspace_bytes(2, C.byref(t))
    assert need % 256 == 0
    assert lib.railsched_schedule_workspace_bytes(-1, C.byref(t)) == 0
    f = lib.railsched_schedule   # (D1, batch, topo, off, w, flow, perm, capacity, rail, S, R, stats, ws, ws_bytes, stream)
    assert f(FAKE, -1, C.byref(t), FAKE, FAKE, FAKE, FAKE, 10, FAKE, FAKE, FAKE, FAKE, FAKE, need, None) == -1
    assert f(FAKE, 2, C.byref(t), FAKE, FAKE, FAKE, FAKE, -1, FAKE, FAKE, FAKE, FAKE, FAKE, need, None) == -1
    assert f(None, 2, C.byref(t), FAKE, FAKE, FAKE, FAKE, 10, FAKE, FAKE, FAKE, FAKE, FAKE, need, None) == -2
    assert f(FAKE, 2, C.byref(t), FAKE, FAKE, FAKE, FAKE, 10, None, FAKE, FAKE, FAKE, FAKE, need, None) == -2
    assert f(FAKE, 2, C.byref(t), FAKE, FAKE, FAKE, FAKE, 10, FAKE, FAKE, FAKE, None, FAKE, need, None) == -2
    assert f(FAKE, 2, None, FAKE, FAKE, FAKE, FAKE, 10, FAKE, FAKE, FAKE, FAKE, FAKE, need, None) == -2
    assert f(FAKE, 2, C.byref(t), FAKE, FAKE, FAKE, FAKE, 10, FAKE, FAKE, FAKE, FAKE, None, need, None) == -5
    assert f(FAKE, 2, C.byref(t), FAKE, FAKE, FAKE, FAKE, 10, FAKE, FAKE, FAKE, FAKE, FAKE, need - 1, None) == -5
    assert f(FAKE, 2, C.byref(t), FAKE, FAKE, FAKE, FAKE, 10, FAKE, FAKE, FAKE, FAKE, P(0x1001), need, None) == -5
    assert f(FAKE, 0, C.byref(t), FAKE, FAKE, FAKE, FAKE, 10, FAKE, FAKE, FAKE, FAKE, FAKE, need, None) == 0
    big = _topo(M=64, N=32)
    assert f(FAKE, 1, C.byref(big), FAKE, FAKE, FAKE, FAKE, 10, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 40, None) == -3


def test_schedule_static_validation():
    lib = rs.load()
    t = _topo()
    f = lib.railsched_schedule_static   # railsched_schedule without (ws, ws_bytes)
    assert f(FAKE, -1, C.byref(t), FAKE, FAKE, FAKE, FAKE, 10, FAKE, FAKE, FAKE, FAKE, None) == -1
    assert f(None, 2, C.byref(t), FAKE, FAKE, FAKE, FAKE, 10, FAKE, FAKE, FAKE, FAKE, None) == -2
    assert f(FAKE, 2, None, FAKE, FAKE, FAKE, FAKE, 10, FAKE, FAKE, FAKE, FAKE, None) == -2
    assert f(FAKE, 0, C.byref(t), FAKE, FAKE, FAKE, FAKE, 10, FAKE, FAKE, FAKE, FAKE, None) == 0
    big = _topo(M=32, N=8, Cb=65536)                                   # 64 matrices of 256 x 256: far more scratch than 4 MiB
    assert lib.railsched_schedule_workspace_bytes(64, C.byref(big)) > rs.STATIC_SCRATCH_BYTES
    assert f(FAKE, 64, C.byref(big), FAKE, FAKE, FAKE, FAKE, 10, FAKE, FAKE, FAKE, FAKE, None) == -7
    assert "static" in rs.strerror(-7)
    header = open(os.path.join(ROOT, "include", "railsched.h")).read()
    assert re.search(r"#define\s+RAILSCHED_STATIC_SCRATCH_BYTES\s+\(4u\s*<<\s*20\)", header) and rs.STATIC_SCRATCH_BYTES == 4 << 20
