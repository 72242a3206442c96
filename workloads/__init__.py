"""Seeded synthetic inputs for the rail-spraying pipeline.

This module only *draws inputs*: router logits, expert placement tables and
GPU-to-GPU byte matrices.  It contains none of the method's arithmetic (no
top-k, no histogram, no chunking, no scheduling) and is the single thing the
CPU oracle's tests and the GPU path's tests are allowed to share, so both
sides see identical bytes.

All randomness is counter based: every element is a pure function of
(seed, stream, index), so generation is order-, thread- and device-independent.

  * Logits use integer arithmetic up to one exact int->fp32 conversion, one fp32
    multiply and one fp32 add (each a separately rounded IEEE operation), so a
    CPU tensor and a GPU tensor produced by the same call are bit-identical.
  * Flow matrices need exp/log/cos in double and are always produced on the
    host with numpy; both consumers receive copies of the same array.

The shapes follow the five MoE/all-to-all workload classes of the paper's
evaluation (Section 6.1, workload table: uniform / Top-K sparse / Zipf-skewed
token and gating distributions); the paper's own traces are not available, so
these stand in for them.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Optional

import numpy as np
import torch

__all__ = [
    "Config", "CONFIGS", "get_config", "expert_gpu_table", "expert_bias",
    "gen_logits", "gen_flow_matrices", "gen_flow_matrices_device", "mix64_np", "symmetric_matrix",
]


@dataclass(frozen=True)
class Config:
    """One workload: topology (M domains x N rails), routing shape, chunking."""
    name: str
    M: int                      # domains (nodes)
    N: int                      # GPUs = NICs = rails per domain
    chunk_bytes: int            # C
    batch: int                  # number of traffic matrices (MoE layers)
    kind: str                   # "moe" (logits -> routing) or "flows" (D1 drawn directly)
    # --- moe ---
    E: int = 0                  # routed experts
    k: int = 0                  # top-k
    tokens_per_gpu: int = 0
    payload_bytes: int = 0      # bytes per routed token copy
    experts_per_gpu: int = 1    # epg
    zipf_s: float = 0.0         # exponent of the per-expert popularity bias
    # --- flows ---
    p_zero: float = 0.0
    mu_bytes: float = 0.0       # median of the non-zero flow size
    sigma: float = 0.0
    round_bytes: int = 4096
    # ---
    seed: int = 0
    rail_bw_Bps: int = 50_000_000_000   # 400 Gb/s-class NIC; the paper gives no rate

    @property
    def G(self) -> int:
        return self.M * self.N

    @property
    def rows_per_layer(self) -> int:
        return self.G * self.tokens_per_gpu

    @property
    def replicas(self) -> int:
        return self.G // (self.E // self.experts_per_gpu)

    def scaled(self, **kw) -> "Config":
        return replace(self, **kw)


KiB = 1024
MiB = 1024 * 1024

CONFIGS = {
    # Tiny: 4 nodes x 4 GPUs, 8 experts top-2, 2048 tokens/GPU, 2 KiB tokens, 64 KiB chunks.
    "c1": Config("c1", M=4, N=4, chunk_bytes=64 * KiB, batch=1, kind="moe", E=8, k=2,
                 tokens_per_gpu=2048, payload_bytes=2 * KiB, experts_per_gpu=1, zipf_s=1.0),
    # Mixtral-8x7B-shaped: 8x8 GPUs, 8 experts top-2 replicated per node, 16384 tokens/GPU,
    # hidden 4096 bf16, 256 KiB chunks, 32 layers.
    "c2": Config("c2", M=8, N=8, chunk_bytes=256 * KiB, batch=32, kind="moe", E=8, k=2,
                 tokens_per_gpu=16384, payload_bytes=8 * KiB, experts_per_gpu=1, zipf_s=1.2),
    # Synthetic sparse all-to-all: 32x8 GPUs, lognormal flows, 1024 matrices.
    "c3": Config("c3", M=32, N=8, chunk_bytes=64 * KiB, batch=1024, kind="flows",
                 p_zero=0.7, mu_bytes=4 * MiB, sigma=1.5),
    # DeepSeek-V3-shaped: 64x8 GPUs, 256 experts top-8, 2 experts/GPU over 128 GPUs (x4 replicas),
    # 8192 tokens/GPU, hidden 7168 bf16, 128 KiB chunks, 61 layers.
    "c4": Config("c4", M=64, N=8, chunk_bytes=128 * KiB, batch=61, kind="moe", E=256, k=8,
                 tokens_per_gpu=8192, payload_bytes=14 * KiB, experts_per_gpu=2, zipf_s=1.1),
    # Stress: 128x8 GPUs, heavier lognormal flows, 16 KiB chunks, 256 matrices.
    "c5": Config("c5", M=128, N=8, chunk_bytes=16 * KiB, batch=256, kind="flows",
                 p_zero=0.5, mu_bytes=16 * MiB, sigma=2.0),
}


def get_config(name: str) -> Config:
    return CONFIGS[name.lower()]


# --------------------------------------------------------------------------
# counter-based 64-bit mixer (splitmix64 finaliser), numpy and torch flavours
# --------------------------------------------------------------------------
_GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_MASK64 = (1 << 64) - 1


def _mix64_int(z: int) -> int:
    z &= _MASK64
    z ^= z >> 30
    z = (z * _M1) & _MASK64
    z ^= z >> 27
    z = (z * _M2) & _MASK64
    z ^= z >> 31
    return z


def mix64_np(z: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on a uint64 array (wrapping arithmetic)."""
    z = z.astype(np.uint64, copy=True)
    with np.errstate(over="ignore"):
        z ^= z >> np.uint64(30)
        z *= np.uint64(_M1)
        z ^= z >> np.uint64(27)
        z *= np.uint64(_M2)
        z ^= z >> np.uint64(31)
    return z


def _s64(v: int) -> int:
    """Reinterpret an unsigned 64-bit constant as the signed value torch.int64 holds."""
    v &= _MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of the 64-bit pattern held in an int64 tensor."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix64_torch(z: torch.Tensor) -> torch.Tensor:
    z = z ^ _lsr(z, 30)
    z = z * _s64(_M1)
    z = z ^ _lsr(z, 27)
    z = z * _s64(_M2)
    z = z ^ _lsr(z, 31)
    return z


def _stream_key(seed: int, stream: int, salt: int) -> int:
    return _mix64_int(_mix64_int(seed * _GOLDEN + salt) ^ ((stream + 1) * _M2))


# --------------------------------------------------------------------------
# MoE routing inputs
# --------------------------------------------------------------------------
def expert_gpu_table(cfg: Config) -> np.ndarray:
    """int32 [E][R]: GPU that hosts replica rho of expert e.

    epg experts per GPU fill an expert-parallel group of Gep = E/epg GPUs; the
    G GPUs hold R = G/Gep such groups: expert_gpu[e][rho] = rho*Gep + e//epg.
    """
    gep = cfg.E // cfg.experts_per_gpu
    assert gep * cfg.experts_per_gpu == cfg.E and cfg.G % gep == 0
    R = cfg.G // gep
    e = np.arange(cfg.E, dtype=np.int64)[:, None]
    rho = np.arange(R, dtype=np.int64)[None, :]
    return (rho * gep + e // cfg.experts_per_gpu).astype(np.int32)


def expert_bias(cfg: Config) -> np.ndarray:
    """fp32 [E]: -s*ln(e+1), so softmax of the bias alone is Zipf(s) (expert 0 hottest)."""
    e = np.arange(cfg.E, dtype=np.float64)
    return (-cfg.zipf_s * np.log(e + 1.0)).astype(np.float32)


# sum of four 16-bit uniforms, centred: variance 4*(65536^2-1)/12
_Z_STD = math.sqrt(4.0 * (65536.0 ** 2 - 1.0) / 12.0)
_Z_SCALE = np.float32(1.0 / _Z_STD)


def gen_logits(cfg: Config, layer: int, device="cpu", row_start: int = 0,
               rows: Optional[int] = None) -> torch.Tensor:
    """fp32 [rows][E] router logits of one MoE layer (rows of source GPU s are contiguous).

    logit = fp32(z) * scale + bias[e], z an integer approximate normal.  The
    coarse z lattice makes exact ties occur, which exercises the tie-break.
    """
    assert cfg.kind == "moe"
    if rows is None:
        rows = cfg.rows_per_layer - row_start
    E = cfg.E
    key = _stream_key(cfg.seed, layer, 0x10617)
    idx = torch.arange(row_start * E, (row_start + rows) * E, dtype=torch.int64, device=device)
    h = _mix64_torch(idx * _s64(_GOLDEN) + _s64(key))
    z = ((h & 0xFFFF) + (_lsr(h, 16) & 0xFFFF) + (_lsr(h, 32) & 0xFFFF) + _lsr(h, 48)) - 2 * 65535
    zf = z.to(torch.float32) * torch.tensor(_Z_SCALE, dtype=torch.float32, device=device)
    bias = torch.from_numpy(expert_bias(cfg)).to(device)
    out = zf.view(rows, E) + bias[None, :]
    return out.contiguous()


# --------------------------------------------------------------------------
# direct flow matrices (no routing stage)
# --------------------------------------------------------------------------
def _uniform01(h: np.ndarray) -> np.ndarray:
    return ((h >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def gen_flow_matrices(cfg: Config, first: int = 0, count: Optional[int] = None) -> np.ndarray:
    """int64 [count][G][G]: entry = 0 w.p. p_zero, else lognormal(ln mu_bytes, sigma)
    rounded to round_bytes; zero diagonal.  Matrix b uses stream b."""
    assert cfg.kind == "flows"
    if count is None:
        count = cfg.batch - first
    G = cfg.G
    out = np.empty((count, G, G), dtype=np.int64)
    idx = np.arange(G * G, dtype=np.uint64)
    mu = math.log(cfg.mu_bytes)
    for i in range(count):
        b = first + i
        with np.errstate(over="ignore"):
            u1 = _uniform01(mix64_np(idx * np.uint64(_GOLDEN) + np.uint64(_stream_key(cfg.seed, b, 0xF10A1))))
            u2 = _uniform01(mix64_np(idx * np.uint64(_GOLDEN) + np.uint64(_stream_key(cfg.seed, b, 0xF10A2))))
            u3 = _uniform01(mix64_np(idx * np.uint64(_GOLDEN) + np.uint64(_stream_key(cfg.seed, b, 0xF10A3))))
        z = np.sqrt(-2.0 * np.log(u2)) * np.cos(2.0 * math.pi * u3)
        size = np.floor(np.exp(mu + cfg.sigma * z) / cfg.round_bytes + 0.5) * cfg.round_bytes
        m = np.where(u1 < cfg.p_zero, 0.0, size).astype(np.int64).reshape(G, G)
        np.fill_diagonal(m, 0)
        out[i] = m
    return out


def gen_flow_matrices_device(cfg: Config, device, first: int = 0, count: Optional[int] = None) -> torch.Tensor:
    """Same recipe as gen_flow_matrices, evaluated with torch on `device` (int64 [count][G][G]).

    exp/log/cos come from the device's math library, so the values can differ from the numpy ones in
    rare rounding cases: whoever uses this must hand copies of the SAME tensor to every consumer."""
    assert cfg.kind == "flows"
    if count is None:
        count = cfg.batch - first
    G = cfg.G
    idx = torch.arange(G * G, dtype=torch.int64, device=device)
    mu = math.log(cfg.mu_bytes)
    out = torch.empty((count, G, G), dtype=torch.int64, device=device)

    def uni(b, salt):
        h = _mix64_torch(idx * _s64(_GOLDEN) + _s64(_stream_key(cfg.seed, b, salt)))
        return (_lsr(h, 11).to(torch.float64) + 0.5) * (1.0 / 9007199254740992.0)

    for i in range(count):
        b = first + i
        u1, u2, u3 = uni(b, 0xF10A1), uni(b, 0xF10A2), uni(b, 0xF10A3)
        z = torch.sqrt(-2.0 * torch.log(u2)) * torch.cos(2.0 * math.pi * u3)
        size = torch.floor(torch.exp(mu + cfg.sigma * z) / cfg.round_bytes + 0.5) * cfg.round_bytes
        m = torch.where(u1 < cfg.p_zero, torch.zeros_like(size), size).to(torch.int64).view(G, G)
        m.fill_diagonal_(0)
        out[i] = m
    return out


def symmetric_matrix(M: int, N: int, q: int, chunk_bytes: int) -> np.ndarray:
    """int64 [G][G] with every entry q*C: the all-equal ("uniform workload") input on
    which an even per-rail split exists exactly (discrete instance of Theorem 3)."""
    G = M * N
    return np.full((G, G), q * chunk_bytes, dtype=np.int64)
