"""A drop-in verifier object for a speculative-decoding loop (paper Section 3.3 item 4: EARS as a
pluggable "sampler" that receives the target model's logits and the draft information and returns
accept / reject decisions), plus acceptance telemetry (the three branches of Section 3.2 step 5).

Everything here is tensor bookkeeping around the C ABI: buffers are allocated once and reused, the
decode step is folded into the RNG seed, and sequences keep their noise streams under continuous
batching through `seq_ids` (the gather of "all active sequences" of Section 3.3 item 3).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import torch

from . import binding

_GOLDEN = 0x9E3779B97F4A7C15
_MASK64 = (1 << 64) - 1


@dataclass
class VerifyResult:
    accept_len: torch.Tensor            # [B] int32
    tokens: torch.Tensor                # [B, K+1] int32 (ragged: packed like the target rows)
    path: Optional[torch.Tensor] = None  # per position: 0 reject, 1 primary accept, 2 pardon
    stats: Optional[torch.Tensor] = None  # [rows, 10] float64, columns binding.STAT_NAMES


class EarsVerifier:
    """Verifies draft tokens step after step.

    temperature / beta are the sampling temperature and the base tolerance of the paper
    (Section 3.2; its experiments use T = 0.9, beta = 0.1).  beta = 0 is standard speculative
    sampling.  `seed` fixes the whole noise stream: step t of sequence id s always sees the same
    random numbers, whatever slot of the batch the sequence occupies.  `uncertainty` selects what
    scales the tolerance: "maxprob" (the paper's 1 - max P_target), or one of the refinements its
    Section 5 names: "entropy" (normalised Shannon entropy) or "variance" (1 - sum P_target^2).
    temperature = 0 selects greedy verification (accept while the draft token is the target
    arg-max): no draft logits, no noise.
    """

    UNCERTAINTY = {"maxprob": binding.EARS_UNCERTAINTY_MAXPROB,
                   "entropy": binding.EARS_UNCERTAINTY_ENTROPY,
                   "variance": binding.EARS_UNCERTAINTY_VARIANCE}

    def __init__(self, temperature: float = 0.9, beta: float = 0.1, seed: int = 0,
                 telemetry: bool = False, uncertainty: str = "maxprob"):
        binding.lib()  # fail now, loudly, if the HIP library has not been built
        if uncertainty not in self.UNCERTAINTY:
            raise ValueError("uncertainty must be one of %s" % sorted(self.UNCERTAINTY))
        self.uncertainty = self.UNCERTAINTY[uncertainty]
        self.temperature = float(temperature)
        self.beta = float(beta)
        self.seed = int(seed) & _MASK64
        self.telemetry = bool(telemetry)
        self.step = 0
        self._workspace: Optional[torch.Tensor] = None
        self._acc: Optional[torch.Tensor] = None
        self._tok: Optional[torch.Tensor] = None
        self._path: Optional[torch.Tensor] = None
        self.counts = {"positions": 0, "primary": 0, "pardon": 0, "rejected": 0, "accepted_tokens": 0,
                       "sequences": 0}

    def step_seed(self, step: int) -> int:
        """Seed of decode step `step`: the base seed advanced by a Weyl sequence."""
        return (self.seed + (step + 1) * _GOLDEN) & _MASK64

    def _buffers(self, rows: int, B: int, need: int, device) -> None:
        if self._workspace is None or self._workspace.numel() < need or self._workspace.device != device:
            self._workspace = torch.empty(need, dtype=torch.uint8, device=device)
        if self._acc is None or self._acc.numel() != B or self._acc.device != device:
            self._acc = torch.empty(B, dtype=torch.int32, device=device)
        if self._tok is None or self._tok.numel() != rows + B or self._tok.device != device:
            self._tok = torch.empty(rows + B, dtype=torch.int32, device=device)
        if self.telemetry and (self._path is None or self._path.numel() != rows or self._path.device != device):
            self._path = torch.empty(rows, dtype=torch.int32, device=device)

    def verify(self, target_logits: torch.Tensor, draft_logits: torch.Tensor,
               draft_tokens: torch.Tensor, *, seq_ids: Optional[torch.Tensor] = None,
               row_offsets: Optional[torch.Tensor] = None,
               temperature_per_seq: Optional[torch.Tensor] = None,
               beta_per_seq: Optional[torch.Tensor] = None, step: Optional[int] = None,
               want_stats: bool = False) -> VerifyResult:
        """One verification step.  Rectangular: target [B,K+1,V], draft [B,K,V], tokens [B,K].
        Ragged: packed 2-D tensors plus row_offsets [B+1].  The returned tensors are reused by
        the next call."""
        if self.temperature == 0.0:
            return self._verify_greedy(target_logits, draft_tokens, row_offsets, step)
        t = self.step if step is None else int(step)
        V = target_logits.shape[-1]
        if row_offsets is None:
            B, K1, _ = target_logits.shape
            rows = B * (K1 - 1)
        else:
            B = row_offsets.shape[0] - 1
            rows = draft_logits.shape[0]
        self._buffers(rows, B, binding.ears_workspace_bytes(rows, B, V), target_logits.device)
        out = binding.ears_verify_ex(
            target_logits, draft_logits, draft_tokens, row_offsets=row_offsets,
            temperature=self.temperature, beta=self.beta, temperature_per_seq=temperature_per_seq,
            beta_per_seq=beta_per_seq, uncertainty=self.uncertainty, seed=self.step_seed(t),
            seq_ids=seq_ids,
            workspace=self._workspace, out_accept_len=self._acc, out_tokens=self._tok,
            want_stats=want_stats, want_path=self._path if self.telemetry else False)
        if step is None:
            self.step += 1
        tokens = out["tokens"] if row_offsets is not None else out["tokens"].view(B, -1)
        res = VerifyResult(out["accept_len"], tokens, out["path"], out["stats"])
        if self.telemetry:
            self._count(res, rows, B)
        return res

    def _verify_greedy(self, target_logits, draft_tokens, row_offsets, step) -> VerifyResult:
        if row_offsets is None:
            B = target_logits.shape[0]
            rows = B * (target_logits.shape[1] - 1)
        else:
            B = row_offsets.shape[0] - 1
            rows = draft_tokens.shape[0]
        self._buffers(rows, B, binding.ears_greedy_workspace_bytes(rows, B), target_logits.device)
        acc, tok = binding.ears_verify_greedy(target_logits, draft_tokens, row_offsets=row_offsets,
                                              workspace=self._workspace, out_accept_len=self._acc,
                                              out_tokens=self._tok)
        if step is None:
            self.step += 1
        if self.telemetry:
            self.counts["positions"] += rows
            self.counts["sequences"] += B
            n = int(acc.sum().item())
            self.counts["accepted_tokens"] += n
            self.counts["primary"] += n
        return VerifyResult(acc, tok if row_offsets is not None else tok.view(B, -1))

    def _count(self, res: VerifyResult, rows: int, B: int) -> None:
        # one small device-to-host copy per step; telemetry is opt-in
        hist = torch.bincount(res.path.clamp(0, 2), minlength=3).tolist()
        self.counts["positions"] += rows
        self.counts["rejected"] += hist[0]
        self.counts["primary"] += hist[1]
        self.counts["pardon"] += hist[2]
        self.counts["accepted_tokens"] += int(res.accept_len.sum().item())
        self.counts["sequences"] += B

    def summary(self) -> dict:
        """Per-position branch rates (evaluated independently of the prefix) and the mean accepted
        length per sequence and step."""
        c = self.counts
        n = max(c["positions"], 1)
        return {"primary_rate": c["primary"] / n, "pardon_rate": c["pardon"] / n,
                "reject_rate": c["rejected"] / n,
                "mean_accept_len": c["accepted_tokens"] / max(c["sequences"], 1)}


def acceptance_sweep(batch, betas, temperature: float, seed: int = 0,
                     uncertainty: str = "maxprob") -> list:
    """Branch rates and mean accepted length of one rectangular batch for each beta (the
    efficiency / quality trade-off of Section 4.3)."""
    rows = []
    for beta in betas:
        v = EarsVerifier(temperature=temperature, beta=beta, seed=seed, telemetry=True,
                         uncertainty=uncertainty)
        v.verify(batch.target, batch.draft, batch.tokens, step=0)
        rows.append(dict(beta=float(beta), temperature=float(temperature), **v.summary()))
    return rows
