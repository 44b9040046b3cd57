"""Seeded synthetic inputs for the verify-and-recover block.

This module holds input recipes only: Gaussian / Zipf logit constructions,
draft tokens drawn from the specialist-with-context rows (the drafting phase,
Eq. 5, which sits before the block and is not part of it), lengths and
uniforms.  It contains none of the block's own arithmetic (no acceptance
rule, no recovery logits) and is the one module both the HIP path's tests and
the CPU oracle's tests take their inputs from.

The logits stand in for the generalist / specialist model outputs of the
paper's experiments, which need weights and datasets that are not available:
vocabulary sizes 151936 and 128256 match the model families the paper pairs,
and the mixing coefficients set how often the ratio test accepts.
"""
from __future__ import annotations

import dataclasses
import hashlib
from typing import Optional

import torch


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    k_max: int
    vocab: int
    dtype: str            # "f32" | "bf16"
    sigma: float          # std of the iid Gaussian components z0..z3
    c_g: float            # G       = z0 + c_g * z1 (+ prior)
    c_ctx: float          # S_ctx   = z0 + c_ctx * z2 (+ prior)
    c_noctx: float        # S_noctx = z0 + c_noctx * z3 (+ prior)
    zipf: float           # 0 => none; s => prior -s*ln(rank) over one seeded vocab permutation
    temperature: float
    beta: float           # steering-recovery strength (the configs call it "steering weight alpha")
    lam: float            # verification threshold; the configs do not set it: paper default 0.5
    ragged: bool          # K_b ~ Uniform{1..k_max} with a length array, else K_b = k_max
    index: int            # position in the config list; offsets the seeds


WORKLOADS = {
    "c1": Workload("c1", 1, 4, 32000, "f32", 3.0, 0.5, 0.5, 0.5, 0.0, 1.0, 1.0, 0.5, False, 1),
    "c2": Workload("c2", 8, 8, 151936, "bf16", 3.0, 0.5, 0.5, 0.5, 0.0, 1.0, 0.5, 0.5, False, 2),
    "c3": Workload("c3", 64, 8, 151936, "bf16", 2.0, 0.5, 0.5, 0.5, 1.1, 1.0, 1.0, 0.5, False, 3),
    "c4": Workload("c4", 256, 16, 128256, "bf16", 3.0, 0.3, 0.3, 0.3, 0.0, 0.7, 0.8, 0.5, True, 4),
    # the config text gives no generalist coefficient for c5; 0.5 as in c1..c3
    "c5": Workload("c5", 512, 8, 256000, "bf16", 8.0, 0.5, 1.0, 0.2, 0.0, 1.0, 1.5, 0.5, False, 5),
}

_SEED_LOGITS = 16219000
_SEED_PERM = 16219100
_SEED_DRAFT = 16219200
_SEED_UNIF = 16219300
_SEED_LEN = 16219400


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def scaled(w: Workload, *, batch: Optional[int] = None, vocab: Optional[int] = None,
           k_max: Optional[int] = None, name: Optional[str] = None) -> Workload:
    """Same recipe at another size (parity tests run reduced shapes through the oracle)."""
    return dataclasses.replace(
        w, batch=w.batch if batch is None else batch, vocab=w.vocab if vocab is None else vocab,
        k_max=w.k_max if k_max is None else k_max, name=name or w.name)


def generate(w: Workload, device="cpu", seed_shift: int = 0, seq_chunk: int = 4) -> dict:
    """Build every input of one block for workload ``w`` on ``device``.

    Returns dict(G, S_ctx, S_noctx [B,k_max+1,V]; draft [B,k_max] int32;
    draft_len [B] int32 or None; uniforms [B,k_max+1] fp32).  Generators are
    per-device, so CPU and GPU streams differ; a test generates once and hands
    the same tensors to both sides.
    """
    dev = torch.device(device)
    B, K1, V = w.batch, w.k_max + 1, w.vocab
    dt = torch_dtype(w.dtype)

    def gen(seed):
        g = torch.Generator(device=dev)
        g.manual_seed(seed + w.index + 1000 * seed_shift)
        return g

    g_log, g_draft, g_unif = gen(_SEED_LOGITS), gen(_SEED_DRAFT), gen(_SEED_UNIF)
    prior = None
    if w.zipf:
        perm = torch.randperm(V, generator=gen(_SEED_PERM), device=dev)
        prior = -w.zipf * torch.log((perm + 1).to(torch.float32))

    G = torch.empty(B, K1, V, dtype=dt, device=dev)
    Sp = torch.empty_like(G)
    Sm = torch.empty_like(G)
    draft = torch.empty(B, w.k_max, dtype=torch.int32, device=dev)
    for b0 in range(0, B, seq_chunk):
        b1 = min(B, b0 + seq_chunk)
        z = torch.randn(4, b1 - b0, K1, V, generator=g_log, device=dev, dtype=torch.float32) * w.sigma
        parts = (z[0] + w.c_g * z[1], z[0] + w.c_ctx * z[2], z[0] + w.c_noctx * z[3])
        if prior is not None:
            parts = tuple(p + prior for p in parts)
        G[b0:b1], Sp[b0:b1], Sm[b0:b1] = (p.to(dt) for p in parts)
        del z, parts
        if w.k_max:
            # drafting phase: y_t ~ softmax(S_ctx[b,t,:]/T), inverse CDF in float64
            rows = Sp[b0:b1, : w.k_max].to(torch.float64) / w.temperature
            cdf = torch.cumsum(torch.softmax(rows, dim=-1), dim=-1)
            ud = torch.rand(b1 - b0, w.k_max, 1, generator=g_draft, device=dev, dtype=torch.float64)
            idx = torch.searchsorted(cdf, ud * cdf[..., -1:]).squeeze(-1).clamp_(max=V - 1)
            draft[b0:b1] = idx.to(torch.int32)
            del rows, cdf
    uniforms = torch.rand(B, K1, generator=g_unif, device=dev, dtype=torch.float32)
    draft_len = None
    if w.ragged and w.k_max == 0:
        draft_len = torch.zeros(B, dtype=torch.int32, device=dev)
    elif w.ragged:
        draft_len = torch.randint(1, w.k_max + 1, (B,), generator=gen(_SEED_LEN), device=dev,
                                  dtype=torch.int32)
    return {"G": G, "S_ctx": Sp, "S_noctx": Sm, "draft": draft, "draft_len": draft_len,
            "uniforms": uniforms}


def tensor_sha256(t: torch.Tensor) -> str:
    """Content hash of a tensor's bytes (logged so a run can be tied to its inputs)."""
    raw = t.detach().contiguous().cpu()
    if raw.dtype == torch.bfloat16:
        raw = raw.view(torch.int16)
    return hashlib.sha256(raw.numpy().tobytes()).hexdigest()
