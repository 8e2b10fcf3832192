"""Seeded generators for the five benchmark shapes plus free-form small cases.

Recipe (one batch element, one KV head ``g`` with its ``G`` query heads):
  u_g   unit vector from a standard normal draw of length d
  K_g   N(0,1)^{n x d};  V_g ~ N(0,1)^{n x d}
  S_g   the spike set (config dependent); K_g[j] += s * u_g for j in S_g
  Q_h   N(0,1)^{n x d} + gamma * sqrt(d) * u_g     for every h in the group
then everything is rounded to the storage dtype (bf16 round-to-nearest-even,
or kept fp32).  The shared query component is what lets a spiked key collect
attention mass (a spiked key gains a mean logit of gamma * s).

Draw order: for each batch, for each KV head: u, K, V, spike set, then the Q
of each query head of the group.  RNG: numpy Generator(PCG64(seed)).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np

GAMMA_DEFAULT = 1.75
M_PROBE = 64


def base_seed(cfg: int, layer: int = 0) -> int:
    return 241008584 + 1000 * cfg + layer


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 array -> fp32 array whose values are exactly representable in bf16
    (round to nearest, ties to even on the 16 dropped mantissa bits)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 array holding bf16-representable values -> their 16-bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


@dataclass(frozen=True)
class WorkloadSpec:
    name: str
    B: int
    Hq: int
    Hkv: int
    n: int
    d: int
    dtype: str            # "f32" | "bf16"
    spike: float          # s
    taus: Tuple[float, ...]
    n_visual: int
    layers: int = 1
    note: str = ""


CONFIGS: Dict[int, WorkloadSpec] = {
    1: WorkloadSpec("cfg1-llava15-576-f32", 1, 4, 4, 576, 64, "f32", 3.0, (0.975,), 512,
                    note="n=576 total: [0,512) visual, [512,576) text/probe span; 58 spiked positions"),
    2: WorkloadSpec("cfg2-llavanext7b-3072-bf16", 1, 32, 32, 3072, 128, "bf16", 2.5, (0.975,), 2880,
                    note="144 spiked visual positions plus the first 4 tokens (sinks)"),
    3: WorkloadSpec("cfg3-llavanext13b-4096-bf16", 1, 40, 40, 4096, 128, "bf16", 2.5,
                    (0.95, 0.975, 0.99), 3840,
                    note="per-head spike fraction uniform in [2%,20%] of the visual span"),
    4: WorkloadSpec("cfg4-longvideo-gqa-18432-bf16", 1, 28, 4, 18432, 128, "bf16", 2.5, (0.975,), 18432,
                    note="128 frames x 144; 553 spikes inside 4 of the 16 aligned 8-frame runs per KV head"),
    5: WorkloadSpec("cfg5-7b-stack-8192-bf16", 4, 32, 32, 8192, 128, "bf16", 2.5, (0.975,), 8192,
                    layers=32, note="spike fraction ramps 30% (layer 0) -> 2% (layer 31)"),
}


@dataclass
class Workload:
    spec: WorkloadSpec
    seed: int
    layer: int
    gamma: float
    Q: np.ndarray          # [B,Hq,n,d] fp32 (values representable in spec.dtype)
    K: np.ndarray          # [B,Hkv,n,d]
    V: np.ndarray          # [B,Hkv,n,d]
    probe_pos: np.ndarray  # [m] int32, ascending
    scale: float
    spikes: list = field(default_factory=list)   # per (b,g): int64 array of spiked positions

    @property
    def tau(self) -> float:
        return self.spec.taus[len(self.spec.taus) // 2]


def _spike_set(cfg: int, spec: WorkloadSpec, rng: np.random.Generator, layer: int) -> np.ndarray:
    n = spec.n
    if cfg == 1:
        return np.sort(rng.choice(n, size=int(round(0.10 * n)), replace=False))
    if cfg == 2:
        vis = rng.choice(spec.n_visual, size=int(round(0.05 * spec.n_visual)), replace=False)
        return np.unique(np.concatenate([vis, np.arange(4)]))
    if cfg == 3:
        f = rng.uniform(0.02, 0.20)
        return np.sort(rng.choice(spec.n_visual, size=int(round(f * spec.n_visual)), replace=False))
    if cfg == 4:
        run = 8 * 144
        runs = np.sort(rng.choice(n // run, size=4, replace=False))
        pool = np.concatenate([np.arange(r * run, (r + 1) * run) for r in runs])
        return np.sort(rng.choice(pool, size=int(round(0.03 * n)), replace=False))
    if cfg == 5:
        f = 0.30 - 0.28 * layer / 31.0
        return np.sort(rng.choice(n, size=int(round(f * n)), replace=False))
    raise ValueError(cfg)


def _draw(spec: WorkloadSpec, rng: np.random.Generator, gamma: float, spike_fn,
          batch: Optional[int] = None):
    B = spec.B if batch is None else batch
    G = spec.Hq // spec.Hkv
    n, d = spec.n, spec.d
    Q = np.empty((B, spec.Hq, n, d), dtype=np.float32)
    K = np.empty((B, spec.Hkv, n, d), dtype=np.float32)
    V = np.empty((B, spec.Hkv, n, d), dtype=np.float32)
    spikes = []
    for b in range(B):
        for g in range(spec.Hkv):
            u = rng.standard_normal(d)
            u = (u / np.linalg.norm(u)).astype(np.float32)
            K[b, g] = rng.standard_normal((n, d), dtype=np.float32)
            V[b, g] = rng.standard_normal((n, d), dtype=np.float32)
            S = np.asarray(spike_fn(rng), dtype=np.int64)
            if S.size:
                K[b, g, S] += np.float32(spec.spike) * u
            spikes.append(S)
            shift = np.float32(gamma * np.sqrt(d)) * u
            for h in range(g * G, (g + 1) * G):
                Q[b, h] = rng.standard_normal((n, d), dtype=np.float32)
                Q[b, h] += shift
    if spec.dtype == "bf16":
        Q, K, V = round_to_bf16(Q), round_to_bf16(K), round_to_bf16(V)
    return Q, K, V, spikes


def hybrid_probes(n: int, seed: int, recent: int = 64, random: int = 64) -> np.ndarray:
    """The probe recipe of the paper's supplementary Section A: the `recent` last positions plus
    `random` distinct positions drawn uniformly from the rest, ascending."""
    recent = min(recent, n)
    rng = np.random.Generator(np.random.PCG64(seed))
    rest = n - recent
    rnd = rng.choice(rest, size=min(random, rest), replace=False) if rest > 0 else np.zeros(0, np.int64)
    return np.sort(np.concatenate([rnd, np.arange(rest, n)])).astype(np.int32)


def make_workload(cfg: int, layer: int = 0, gamma: float = GAMMA_DEFAULT,
                  seed: Optional[int] = None, batch: Optional[int] = None) -> Workload:
    """One layer of benchmark shape ``cfg`` (1..5).  ``batch`` overrides B
    (used to draw a bounded slice of the 32-layer stack)."""
    spec = CONFIGS[cfg]
    seed = base_seed(cfg, layer) if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed))
    Q, K, V, spikes = _draw(spec, rng, gamma, lambda r: _spike_set(cfg, spec, r, layer), batch)
    m = min(M_PROBE, spec.n)
    probe = np.arange(spec.n - m, spec.n, dtype=np.int32)
    return Workload(spec, seed, layer, gamma, Q, K, V, probe, 1.0 / float(np.sqrt(spec.d)), spikes)


def make_custom(B: int, Hq: int, Hkv: int, n: int, d: int, dtype: str = "f32", *,
                seed: int = 0, spike: float = 3.0, spike_frac: float = 0.1,
                gamma: float = GAMMA_DEFAULT, m: int = M_PROBE, tau: float = 0.975,
                probe_pos: Optional[np.ndarray] = None) -> Workload:
    """Free-form small case with the same recipe (for parity tests and smoke)."""
    spec = WorkloadSpec(f"custom-B{B}-Hq{Hq}-Hkv{Hkv}-n{n}-d{d}-{dtype}", B, Hq, Hkv, n, d,
                        dtype, spike, (tau,), n)
    rng = np.random.Generator(np.random.PCG64(seed))
    cnt = int(round(spike_frac * n))
    Q, K, V, spikes = _draw(spec, rng, gamma,
                            lambda r: np.sort(r.choice(n, size=cnt, replace=False)) if cnt else np.zeros(0, np.int64))
    if probe_pos is None:
        mm = min(m, n)
        probe_pos = np.arange(n - mm, n, dtype=np.int32)
    probe_pos = np.ascontiguousarray(probe_pos, dtype=np.int32)
    return Workload(spec, seed, 0, gamma, Q, K, V, probe_pos, 1.0 / float(np.sqrt(d)), spikes)


def make_stack_layer_device(layer: int, device: str = "cuda:0", gamma: float = GAMMA_DEFAULT,
                            batch: Optional[int] = None):
    """One layer of the 32-layer stack (shape 5) drawn on the GPU with torch's seeded generator
    (the host generator needs ~5 s per layer; 32 layers are 25.8 GB).  Same recipe as `_draw`;
    the spike set of a (batch, head) unit is the `cnt` positions with the largest of n uniform
    draws.  Returns bf16 tensors Q, K, V [B,H,n,d] and the probe positions."""
    import torch
    spec = CONFIGS[5]
    B = spec.B if batch is None else batch
    H, n, d = spec.Hq, spec.n, spec.d
    gen = torch.Generator(device=device)
    gen.manual_seed(base_seed(5, layer))
    u = torch.randn((B, H, 1, d), generator=gen, device=device, dtype=torch.float32)
    u = u / u.norm(dim=-1, keepdim=True)
    K = torch.randn((B, H, n, d), generator=gen, device=device, dtype=torch.float32)
    V = torch.randn((B, H, n, d), generator=gen, device=device, dtype=torch.float32)
    cnt = int(round((0.30 - 0.28 * layer / 31.0) * n))
    pos = torch.rand((B, H, n), generator=gen, device=device).topk(cnt, dim=-1).indices
    spike = torch.zeros((B, H, n, 1), device=device, dtype=torch.float32)
    spike.scatter_(2, pos.unsqueeze(-1), float(spec.spike))
    K += spike * u
    Q = torch.randn((B, H, n, d), generator=gen, device=device, dtype=torch.float32)
    Q += float(gamma * np.sqrt(d)) * u
    m = min(M_PROBE, n)
    probe = np.arange(n - m, n, dtype=np.int32)
    return (Q.to(torch.bfloat16), K.to(torch.bfloat16), V.to(torch.bfloat16), probe, 1.0 / float(np.sqrt(d)))
