"""Element-by-element comparison of the GPU library's outputs with the CPU oracle's.

The bar: accept lengths and token indices bit-exact, except where the oracle itself says the
decision is numerically undecidable: |R - threshold| < 1e-6 (or |R - U| < 1e-6 for the branch id)
at the first position where the two decisions differ, or a Gumbel top-2 score gap below 1e-6 for
the sampled token, and then only when the differing token is the oracle's runner-up (the one other
entry that is a valid outcome inside the band).  After an exempt decision difference the rest of
that sequence is not compared.
Softmax statistics: relative 1e-5 (fp32 logits) / 2e-3 (bf16 logits) on Z, p_t(x), p_d(x), R and
max p = 1/Z, the row maximum exact, and absolute 1e-6 on the uncertainty and the threshold.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BAND = 1e-6


@dataclass
class ParityReport:
    sequences: int = 0
    positions: int = 0
    exempt_decisions: int = 0
    exempt_tokens: int = 0
    max_rel_Z: float = 0.0
    max_rel_P: float = 0.0
    max_abs_unc: float = 0.0
    notes: list = field(default_factory=list)

    def line(self) -> str:
        return ("seqs=%d pos=%d exempt_decisions=%d exempt_tokens=%d max_rel_Z=%.2e max_rel_P=%.2e "
                "max_abs_unc=%.2e" % (self.sequences, self.positions, self.exempt_decisions,
                                      self.exempt_tokens, self.max_rel_Z, self.max_rel_P,
                                      self.max_abs_unc))


def _relerr(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.maximum(np.abs(b), 1e-300)
    e = np.abs(a - b) / den
    e[(a == b)] = 0.0
    return e


def compare(ora, g_accept, g_tokens, g_stats, g_path, row_offsets, K, stats_rtol, draft_tokens, V,
            rep: ParityReport | None = None, unc_is_maxprob: bool = True) -> ParityReport:
    """ora: OracleResult.  g_*: numpy arrays from the GPU (stats [R,10], path [R], tokens packed
    [R+B] or [B,K+1], accept [B]).  row_offsets None for rectangular batches."""
    rep = rep or ParityReport()
    B = ora.accept_len.shape[0]
    o_diag = ora.diag.reshape(-1, ora.diag.shape[-1])
    o_path = ora.path.reshape(-1)
    o_tok = ora.tokens.reshape(-1)
    g_tok = np.asarray(g_tokens).reshape(-1)
    if row_offsets is None:
        off = np.arange(B + 1, dtype=np.int64) * K
    else:
        off = np.asarray(row_offsets, dtype=np.int64)

    if g_stats is not None:
        g = np.asarray(g_stats)
        assert g.shape == o_diag.shape
        assert np.array_equal(g[:, 0], o_diag[:, 0]), "row maximum m_t must be exact"
        assert np.array_equal(g[:, 3], o_diag[:, 3]), "row maximum m_d must be exact"
        assert np.array_equal(g[:, 8], o_diag[:, 8]), "acceptance uniforms must be identical"
        for col in (1, 4):
            e = _relerr(g[:, col], o_diag[:, col])
            rep.max_rel_Z = max(rep.max_rel_Z, float(e.max()))
            assert e.max() <= stats_rtol, ("Z", col, e.max())
        for col in (2, 5, 7):
            e = _relerr(g[:, col], o_diag[:, col])
            rep.max_rel_P = max(rep.max_rel_P, float(e.max()))
            assert e.max() <= 2 * stats_rtol, ("P/R", col, e.max())
        for col in (6, 9):
            e = np.abs(g[:, col] - o_diag[:, col])
            rep.max_abs_unc = max(rep.max_abs_unc, float(e.max()))
            assert e.max() <= 1e-6, ("unc/thr", col, e.max())
        # max p = 1/Z shortcut against the oracle's explicit maximum
        if unc_is_maxprob:
            e = _relerr(1.0 / g[:, 1], 1.0 - o_diag[:, 6])
            ok = (1.0 - o_diag[:, 6]) > 1e-3
            assert (e[ok] <= stats_rtol + 1e-9).all()

    for b in range(B):
        r0, r1 = int(off[b]), int(off[b + 1])
        Kb = r1 - r0
        rep.sequences += 1
        rep.positions += Kb
        n_o = int(ora.accept_len[b])
        n_g = int(g_accept[b])
        t0 = r0 + b
        exempt = False
        if g_path is not None:
            gp = np.asarray(g_path)[r0:r1]
            op = o_path[r0:r1]
            for i in range(Kb):
                if gp[i] == op[i]:
                    continue
                R, U, thr = o_diag[r0 + i, 7], o_diag[r0 + i, 8], o_diag[r0 + i, 9]
                near = min(abs(R - thr), abs(R - U))
                assert near < BAND, ("decision differs outside the band", b, i, gp[i], op[i], R, U, thr)
                if i <= n_o and (gp[i] != 0) != (op[i] != 0) and not exempt:
                    exempt = True
                    rep.exempt_decisions += 1
                    rep.notes.append(("decision", b, i, float(R - thr)))
        if n_g != n_o and not exempt:
            i = min(n_g, n_o)
            R, thr = o_diag[r0 + i, 7], o_diag[r0 + i, 9]
            assert abs(R - thr) < BAND, ("accept length differs outside the band", b, n_g, n_o, R, thr)
            exempt = True
            rep.exempt_decisions += 1
            rep.notes.append(("accept_len", b, i, float(R - thr)))
        if exempt:
            # still valid: a prefix of the draft, then a token, then -1
            d_tok = np.asarray(draft_tokens).reshape(-1)
            assert 0 <= n_g <= Kb
            assert np.array_equal(g_tok[t0:t0 + n_g], d_tok[r0:r0 + n_g])
            assert 0 <= g_tok[t0 + n_g] < V
            assert np.all(g_tok[t0 + n_g + 1:t0 + Kb + 1] == -1)
            continue
        assert n_g == n_o
        assert np.array_equal(g_tok[t0:t0 + n_o], o_tok[t0:t0 + n_o]), ("prefix", b)
        assert np.all(g_tok[t0 + n_o + 1:t0 + Kb + 1] == -1), ("tail", b)
        if g_tok[t0 + n_o] != o_tok[t0 + n_o]:
            gap, runner_up = ora.samp[b, 2], int(ora.samp[b, 4])
            assert gap < BAND, ("sampled token differs outside the band", b, n_o,
                                int(g_tok[t0 + n_o]), int(o_tok[t0 + n_o]), float(gap))
            assert int(g_tok[t0 + n_o]) == runner_up, (
                "inside the band only the oracle's runner-up is a valid other outcome", b, n_o,
                int(g_tok[t0 + n_o]), runner_up)
            rep.exempt_tokens += 1
            rep.notes.append(("token", b, n_o, float(gap)))
    return rep
