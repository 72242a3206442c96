"""railsched_schedule_static (stages 3-5 with the library's static scratch buffer, for callers that cannot allocate)
against railsched_schedule with a caller-provided workspace: every output equal, on two calls in a row, the second
on a smaller batch that leaves most of the buffer holding the first call's contents."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu

rs = pytest.importorskip("paper_2510_19262_amd")
from paper_2510_19262_amd import binding  # noqa: E402

DEV = "cuda:0"
NAMES = ("chunk_off", "chunk_w", "chunk_flow", "perm", "rail", "S", "R", "stats")


def _stack(rng, B, G, C):
    m = rng.integers(0, 6 * C, size=(B, G, G)).astype(np.int64)
    m[rng.random((B, G, G)) < 0.3] = 0
    m[rng.random((B, G, G)) < 0.2] = 3 * C
    return m


def _buffers(B, M, N, cap):
    i32, i64 = torch.int32, torch.int64
    return (torch.full((B * M + 1,), -3, dtype=i64, device=DEV), torch.full((cap,), -3, dtype=i32, device=DEV),
            torch.full((cap,), -3, dtype=i32, device=DEV), torch.full((cap,), -3, dtype=i32, device=DEV),
            torch.full((cap,), 77, dtype=torch.uint8, device=DEV), torch.full((B, M, N), -3, dtype=i64, device=DEV),
            torch.full((B, M, N), -3, dtype=i64, device=DEV), torch.full((B, 8), -3, dtype=i64, device=DEV))


def _one(D1n, M, N, Cb):
    B = D1n.shape[0]
    topo = rs.Topo(M, N, Cb)
    assert rs.schedule_workspace_bytes(B, topo) <= rs.STATIC_SCRATCH_BYTES
    D1 = torch.from_numpy(D1n).to(DEV)
    off_c, w_c, flow_c, perm_c = oracle.chunk_sort_batch(D1n, M, N, Cb)
    total = int(off_c[-1])
    cap = total + 5
    want = _buffers(B, M, N, cap)
    rs.schedule(D1, topo, cap, out=want)                               # the existing entry point, workspace from torch
    got = _buffers(B, M, N, cap)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    rs.schedule_static(D1, topo, cap, out=got)                         # the new one: no workspace argument
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for name, a, b in zip(NAMES, got, want):
        assert torch.equal(a, b), name                                  # untouched tails of the record arrays included
    rail_c, S_c = oracle.lpt_batch(off_c, w_c, B, M, N)
    _, R_c, stats_c = oracle.eval_batch(off_c, w_c, flow_c, rail_c, B, M, N)
    assert np.array_equal(got[0].cpu().numpy(), off_c) and np.array_equal(got[4].cpu().numpy()[:total], rail_c)
    assert np.array_equal(got[1].cpu().numpy().view(np.uint32)[:total], w_c)
    assert np.array_equal(got[5].cpu().numpy(), S_c) and np.array_equal(got[6].cpu().numpy(), R_c)
    assert np.array_equal(got[7].cpu().numpy(), stats_c)


def test_schedule_static_matches_schedule_on_two_calls_in_a_row():
    rng = np.random.default_rng(2024)
    _one(_stack(rng, 32, 64, 262144), 8, 8, 262144)                     # 256 instances, one workgroup each; ~2 MiB of scratch
    _one(_stack(rng, 3, 16, 4096), 4, 4, 4096)                          # a much smaller batch right behind it
    _one(_stack(rng, 300, 16, 512), 4, 4, 512)                          # and the three-stage shape (more than 1024 instances)
    _one(_stack(rng, 2, 6, 100), 3, 2, 100)


def test_schedule_static_overflow_and_limits():
    rng = np.random.default_rng(7)
    M, N, Cb, B = 4, 4, 4096, 2
    D1n = _stack(rng, B, M * N, Cb)
    total = int(oracle.chunk_count_batch(D1n, M, N, Cb)[-1])
    out = _buffers(B, M, N, total - 1)
    rs.schedule_static(torch.from_numpy(D1n).to(DEV), rs.Topo(M, N, Cb), total - 1, out=out)
    torch.cuda.synchronize()
    assert int(out[0][-1].item()) == total
    assert bool((out[1] == -3).all()) and bool((out[4] == 77).all())    # records untouched
    assert all(bool((t == -1).all()) for t in out[5:])                  # S, R, stats flag the overflow
    # a batch whose workspace exceeds the static buffer is refused before anything runs
    lib = rs.load()
    big = binding._TopoStruct(32, 8, 65536, 1, 0, 0)
    assert lib.railsched_schedule_workspace_bytes(64, C.byref(big)) > rs.STATIC_SCRATCH_BYTES
    fake = C.c_void_p(0x1000)
    rc = lib.railsched_schedule_static(fake, 64, C.byref(big), fake, fake, fake, fake, 10, fake, fake, fake, fake, None)
    assert rc == -7 and "scratch" in rs.strerror(rc)
