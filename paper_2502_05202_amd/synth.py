"""Seeded synthetic inputs for the TLI draft-and-verify path.

This module only draws numbers: vocabulary maps, logits and uniforms with the shapes, sizes and value
distributions of the five workloads (vocabulary sizes and overlaps follow the paper's appendix tables
of vocabulary sizes and vocabulary overlaps; no dataset item, prompt or model weight is involved).
It holds none of the method's arithmetic and is the one module that both the GPU tests/benchmark and
the CPU oracle's callers use, so that both sides see the identical stored values.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import numpy as np
import torch

BASE_SEED = 20250205


@dataclass(frozen=True)
class Workload:
    name: str
    cfg: int          # index used for the per-workload seed
    B: int            # sequences
    K: int            # draft positions per sequence (the paper's lookahead i)
    Vt: int           # |T|
    Vd: int           # |D|
    S: int            # |T ∩ D|
    dtype: str        # "f32" | "bf16" (storage type of the logits)
    tau_t: float
    tau_d: float
    kind: str         # "noise" | "corr" | "zipf"
    sigma: float = 0.0
    noise: float = 0.0      # kind=noise: std of the N(0, noise^2) added on shared ids
    only_mu: float = 0.0    # kind=noise, corr: mean of target-only logits (corr: of the bonus row too)
    rho: float = 0.0        # kind=corr: drafter/target correlation on shared ids

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS = {
    1: Workload("tiny", 1, 1, 3, 64, 48, 32, "f32", 1.0, 1.0, "noise", sigma=2.0, noise=1.0, only_mu=0.0),
    2: Workload("single_stream", 2, 1, 5, 128256, 32000, 24000, "f32", 1.0, 1.0, "noise", sigma=3.0, noise=1.5,
                only_mu=-2.0),
    3: Workload("batched", 3, 64, 5, 151936, 49152, 40000, "bf16", 0.8, 0.8, "corr", sigma=3.0, rho=0.8),
    4: Workload("large_vocab", 4, 256, 8, 256000, 128256, 90000, "bf16", 0.7, 0.7, "corr", sigma=4.0, rho=0.7),
    5: Workload("mismatch", 5, 128, 10, 202048, 128256, 60000, "bf16", 1.2, 0.3, "zipf"),
}


def make_d2t(Vd: int, Vt: int, S: int, seed: int) -> np.ndarray:
    """Partial injection drafter id -> target id (int32, -1 = not shared): S seeded random pairs."""
    rng = np.random.Generator(np.random.Philox(seed))
    d_ids = rng.permutation(Vd)[:S]
    t_ids = rng.permutation(Vt)[:S]
    d2t = np.full(Vd, -1, np.int32)
    d2t[d_ids] = t_ids.astype(np.int32)
    return d2t


def _uniform24(n: int, gen: torch.Generator, device) -> torch.Tensor:
    """fp32 uniforms k * 2^-24, k in [0, 2^24): exactly representable, always < 1."""
    k = torch.randint(0, 1 << 24, (n,), generator=gen, device=device, dtype=torch.int32)
    return k.to(torch.float32) * (2.0 ** -24)


def make_inputs(w: Workload, device="cpu", seed: int | None = None) -> dict:
    """Draw one batch for workload `w` on `device`.

    Returns torch tensors on `device`: logits_t [B,K+1,Vt], logits_d [B,K,Vd] (fp32 or bf16),
    u_draft [B,K], u_acc [B,K], u_fin [B] (fp32), plus d2t (numpy int32 [Vd]) and the temperatures.
    """
    seed = BASE_SEED + w.cfg if seed is None else seed
    device = torch.device(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    d2t = make_d2t(w.Vd, w.Vt, w.S, seed)
    d_idx_np = np.nonzero(d2t >= 0)[0]
    d_idx = torch.from_numpy(d_idx_np).to(device)
    t_idx = torch.from_numpy(d2t[d_idx_np].astype(np.int64)).to(device)
    store = torch.float32 if w.dtype == "f32" else torch.bfloat16
    B, K, Vt, Vd = w.B, w.K, w.Vt, w.Vd
    lt = torch.empty((B, K + 1, Vt), dtype=store, device=device)
    ld = torch.empty((B, K, Vd), dtype=store, device=device)

    def randn(*shape):
        return torch.randn(*shape, generator=gen, device=device, dtype=torch.float32)

    for b in range(B):
        if w.kind == "noise":
            d = randn(K, Vd) * w.sigma
            t = randn(K + 1, Vt) * w.sigma + w.only_mu
            t[K] = randn(Vt) * w.sigma
            t[:K, t_idx] = d[:, d_idx] + randn(K, d_idx.numel()) * w.noise
        elif w.kind == "corr":
            d = randn(K, Vd) * w.sigma
            t = randn(K + 1, Vt) * w.sigma + w.only_mu
            t[:K, t_idx] = w.rho * d[:, d_idx] + math.sqrt(1.0 - w.rho ** 2) * w.sigma * randn(K, d_idx.numel())
        elif w.kind == "zipf":
            rank = torch.rand(K + 1, Vd, generator=gen, device=device).argsort(dim=1)
            dz = -1.1 * torch.log(rank.to(torch.float32) + 1.0)
            d = dz[:K]
            r = torch.randint(1, Vt + 1, (K + 1, Vt), generator=gen, device=device)
            t = -1.1 * torch.log(r.to(torch.float32))
            t[:K, t_idx] = d[:, d_idx] + randn(K, d_idx.numel())
            t[K, t_idx] = dz[K, d_idx] + randn(d_idx.numel())
        else:
            raise ValueError(w.kind)
        lt[b] = t.to(store)
        ld[b] = d.to(store)
    u_draft = _uniform24(B * K, gen, device).reshape(B, K)
    u_acc = _uniform24(B * K, gen, device).reshape(B, K)
    u_fin = _uniform24(B, gen, device)
    return dict(workload=w, d2t=d2t, logits_t=lt, logits_d=ld, u_draft=u_draft, u_acc=u_acc, u_fin=u_fin,
                tau_t=w.tau_t, tau_d=w.tau_d)


def logits_to_numpy(t: torch.Tensor) -> np.ndarray:
    """Host copy of a logits tensor as the oracle reads it: float32, or uint16 = the bf16 bits."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float32:
        return t.numpy()
    raise TypeError(t.dtype)
