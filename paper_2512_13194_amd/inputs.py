"""Seeded synthetic inputs for the EARS verification step.

This module only draws logits, draft tokens and per-sequence parameters with torch's seeded
generators; it contains none of the method's arithmetic and imports neither the GPU binding nor
the CPU oracle, so both can be fed from it.

The paper evaluates on a Qwen3-32B target with an Eagle3 draft (Section 4.1); those models and
their prompts are not available here, so the verification step is driven with random logits that
have the shapes of real vocabularies (32000, 128256, 151936 entries) and a controllable
target/draft mismatch:

* target row  = sigma * N(0, 1), one sigma per row;
* draft row   = target row (before rounding) + noise_std * N(0, 1);
* both are then rounded to the storage type independently;
* draft token ~ softmax(draft_row / T), so that P_d(x) is the probability the token was actually
  drawn with (the losslessness of the beta = 0 rule depends on that).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch


@dataclass
class Batch:
    """One verification problem.  Rectangular batches have row_offsets None and K set; ragged
    batches have K None, packed rows, and per-sequence temperature/beta tensors."""
    target: torch.Tensor            # [B, K+1, V]  or packed [R + B, V]
    draft: torch.Tensor             # [B, K, V]    or packed [R, V]
    tokens: torch.Tensor            # [B, K] int32 or packed [R]
    B: int
    V: int
    K: Optional[int] = None
    row_offsets: Optional[torch.Tensor] = None   # [B+1] int64 over packed draft rows
    temperature: Optional[torch.Tensor] = None   # [B] float32 (ragged only)
    beta: Optional[torch.Tensor] = None          # [B] float32 (ragged only)

    @property
    def total_draft_rows(self) -> int:
        return int(self.draft.numel() // self.V)


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _sample_tokens(draft_rows: torch.Tensor, T_rows: torch.Tensor, g: torch.Generator,
                   chunk: int = 256) -> torch.Tensor:
    """draft_rows [R, V] (storage dtype), T_rows [R] -> tokens [R] int32, x ~ softmax(row / T)."""
    R = draft_rows.shape[0]
    out = torch.empty(R, dtype=torch.int32, device=draft_rows.device)
    for r0 in range(0, R, chunk):
        rows = draft_rows[r0:r0 + chunk].to(torch.float32) / T_rows[r0:r0 + chunk, None]
        probs = torch.softmax(rows, dim=-1)
        out[r0:r0 + chunk] = torch.multinomial(probs, 1, generator=g)[:, 0].to(torch.int32)
    return out


def _rows(n_rows: int, V: int, sigma: torch.Tensor, g: torch.Generator, device) -> torch.Tensor:
    return torch.randn(n_rows, V, generator=g, device=device, dtype=torch.float32) * sigma[:, None]


def make_rect(B: int, K: int, V: int, dtype: torch.dtype, *, T: float, data_seed: int,
              sigma_lo: float = 0.5, sigma_hi: float = 4.0, draft_noise: float = 0.5,
              peaked_frac: float = 0.0, peaked_sigma: float = 12.0,
              device="cpu") -> Batch:
    """Rectangular batch: every sequence has K draft positions and K+1 target rows.

    sigma ~ U[sigma_lo, sigma_hi] per target row; with probability peaked_frac a row instead gets
    sigma = peaked_sigma (a near one-hot distribution).
    """
    g = _gen(device, data_seed)
    n_t = B * (K + 1)
    sigma = sigma_lo + (sigma_hi - sigma_lo) * torch.rand(n_t, generator=g, device=device)
    if peaked_frac > 0.0:
        peaked = torch.rand(n_t, generator=g, device=device) < peaked_frac
        sigma = torch.where(peaked, torch.full_like(sigma, peaked_sigma), sigma)
    tgt32 = _rows(n_t, V, sigma, g, device).view(B, K + 1, V)
    noise = torch.randn(B, K, V, generator=g, device=device, dtype=torch.float32)
    drf32 = tgt32[:, :K, :] + draft_noise * noise
    del noise
    target = tgt32.to(dtype).contiguous()
    draft = drf32.to(dtype).contiguous()
    del tgt32, drf32
    T_rows = torch.full((B * K,), float(T), device=device)
    tokens = _sample_tokens(draft.view(B * K, V), T_rows, g).view(B, K)
    return Batch(target=target, draft=draft, tokens=tokens, B=B, V=V, K=K)


def make_ragged(B: int, V: int, dtype: torch.dtype, *, data_seed: int, K_lo: int = 1,
                K_hi: int = 8, sigma_lo: float = 0.5, sigma_hi: float = 4.0,
                noise_lo: float = 0.2, noise_hi: float = 1.5, T_lo: float = 0.5,
                T_hi: float = 1.5, beta_lo: float = 0.0, beta_hi: float = 1.0,
                device="cpu") -> Batch:
    """Ragged batch: K_b ~ U{K_lo..K_hi}; rows packed, CSR offsets over the draft rows; sequence b
    owns draft rows off[b]..off[b+1) and target rows off[b]+b .. off[b+1]+b (one more)."""
    g = _gen(device, data_seed)
    Ks = torch.randint(K_lo, K_hi + 1, (B,), generator=g, device=device)
    off = torch.zeros(B + 1, dtype=torch.int64, device=device)
    off[1:] = torch.cumsum(Ks, 0)
    R = int(off[-1].item())
    T = (T_lo + (T_hi - T_lo) * torch.rand(B, generator=g, device=device)).to(torch.float32)
    beta = (beta_lo + (beta_hi - beta_lo) * torch.rand(B, generator=g, device=device)).to(torch.float32)
    nstd = noise_lo + (noise_hi - noise_lo) * torch.rand(B, generator=g, device=device)
    target = torch.empty(R + B, V, dtype=dtype, device=device)
    draft = torch.empty(R, V, dtype=dtype, device=device)
    tokens = torch.empty(R, dtype=torch.int32, device=device)
    off_h = off.cpu().tolist()
    for b in range(B):
        r0, r1 = off_h[b], off_h[b + 1]
        Kb = r1 - r0
        sigma = sigma_lo + (sigma_hi - sigma_lo) * torch.rand(Kb + 1, generator=g, device=device)
        t32 = _rows(Kb + 1, V, sigma, g, device)
        d32 = t32[:Kb] + nstd[b] * torch.randn(Kb, V, generator=g, device=device)
        target[r0 + b:r1 + b + 1] = t32.to(dtype)
        draft[r0:r1] = d32.to(dtype)
        T_rows = T[b].expand(Kb).contiguous()
        tokens[r0:r1] = _sample_tokens(draft[r0:r1], T_rows, g)
    return Batch(target=target, draft=draft, tokens=tokens, B=B, V=V, row_offsets=off,
                 temperature=T, beta=beta)


# The five workloads, restated as synthetic inputs (data_seed = 1000 + index).  "betas" and
# "temperatures" are the sweeps each workload is checked on; "seed" is the verification RNG seed.
CONFIGS = [
    dict(name="c0_B1_K4_V32000_f32", kind="rect", B=1, K=4, V=32000, dtype="f32",
         gen=dict(draft_noise=0.5), temperatures=[1.0], betas=[0.5], seed=0, data_seed=1000),
    dict(name="c1_B64_K5_V32000_bf16", kind="rect", B=64, K=5, V=32000, dtype="bf16",
         gen=dict(draft_noise=0.5), temperatures=[0.8], betas=[0.0, 0.5], seed=1, data_seed=1001),
    dict(name="c2_B256_K8_V128256_bf16", kind="rect", B=256, K=8, V=128256, dtype="bf16",
         gen=dict(draft_noise=1.0), temperatures=[1.0], betas=[0.0, 0.25, 0.5, 1.0], seed=2,
         data_seed=1002),
    dict(name="c3_B512_K4_V151936_bf16", kind="rect", B=512, K=4, V=151936, dtype="bf16",
         gen=dict(draft_noise=0.5, sigma_lo=0.3, sigma_hi=1.5, peaked_frac=0.1, peaked_sigma=12.0),
         temperatures=[0.6, 1.0, 1.5], betas=[0.5], seed=3, data_seed=1003),
    dict(name="c4_ragged_B1024_V128256_bf16", kind="ragged", B=1024, V=128256, dtype="bf16",
         gen=dict(), temperatures=[None], betas=[None], seed=4, data_seed=1004),
]

_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def make_config(index: int, *, T: Optional[float] = None, device="cpu", scale_B: Optional[int] = None,
                scale_V: Optional[int] = None) -> Batch:
    """Inputs of workload `index`.  Draft tokens depend on the temperature, so a temperature
    sweep regenerates them (T defaults to the first temperature of the workload).  scale_B /
    scale_V shrink the batch or vocabulary for CPU-sized test cases; the recipe is unchanged."""
    cfg = CONFIGS[index]
    B = scale_B or cfg["B"]
    V = scale_V or cfg["V"]
    dtype = _TORCH_DTYPE[cfg["dtype"]]
    if cfg["kind"] == "rect":
        T = cfg["temperatures"][0] if T is None else T
        return make_rect(B, cfg["K"], V, dtype, T=T, data_seed=cfg["data_seed"], device=device,
                         **cfg["gen"])
    return make_ragged(B, V, dtype, data_seed=cfg["data_seed"], device=device, **cfg["gen"])


def logits_to_numpy(t: torch.Tensor) -> np.ndarray:
    """Host copy of a logits tensor in the layout the CPU oracle reads: float32 as is, bfloat16 as
    its uint16 bit pattern."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float32:
        return t.numpy()
    raise TypeError(t.dtype)
