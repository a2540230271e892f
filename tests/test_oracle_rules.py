"""Pins for the oracle's decision rule and sampling law, taken from what the paper and the
mathematics fix (no expected value here comes from the GPU path):

* softmax statistics against torch / scipy fp64 routines;
* hand-worked cases with power-of-two probabilities: R, uncertainty, tolerance and the three
  decision branches of Section 3.2;
* beta = 0 against an independently written standard speculative-sampling loop (Section 3.1);
* identical target and draft accept everything; range and prefix properties; monotone in beta;
  the threshold clamp of Section 3.3 never changes a decision; tolerance grows with temperature
  (Section 4.3);
* per-position acceptance probability min(1, R + Tol) (acceptance region [0, R + Tol]);
* the closed-form output law on a tiny vocabulary (equal to P_target for beta = 0) and the
  categorical law of the bonus token, by chi-square.
"""
import math

import numpy as np
import pytest
import torch
from scipy import special, stats

EPS = 1e-10


def logits_from_probs(p, T):
    """fp32 logits whose softmax at temperature T is p (up to fp32 rounding of the logits)."""
    return (T * np.log(np.asarray(p, dtype=np.float64))).astype(np.float32)


def softmax64(row, T):
    return torch.softmax(torch.from_numpy(np.asarray(row, dtype=np.float64)) / T, dim=-1).numpy()


def bf16_bits(a32):
    t = torch.from_numpy(np.asarray(a32, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def bf16_to_f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# ---------------------------------------------------------------------------------- softmax
@pytest.mark.parametrize("T", [0.6, 1.0, 1.7])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_softmax_against_library(oracle, T, dtype):
    rng = np.random.default_rng(3)
    row32 = (rng.standard_normal(5000) * 3.0).astype(np.float32)
    row32[17] = -np.inf                      # a masked vocabulary entry has probability 0
    if dtype == "bf16":
        row = bf16_bits(row32)
        ref_in = bf16_to_f64(row)
    else:
        row = row32
        ref_in = row32.astype(np.float64)
    p, m, Z, pmax = oracle.softmax(row, T)
    want = softmax64(ref_in, T)
    np.testing.assert_allclose(p, want, rtol=1e-12, atol=0)
    assert p[17] == 0.0
    assert m == ref_in.max()
    lse = special.logsumexp(ref_in / T)
    assert math.log(Z) + m / T == pytest.approx(lse, rel=1e-13)
    assert pmax == pytest.approx(want.max(), rel=1e-12)
    assert pmax == pytest.approx(1.0 / Z, rel=1e-12)     # max P = 1/Z: the shortcut the GPU uses
    assert abs(p.sum() - 1.0) < 1e-12


def test_tolerance_grows_with_temperature(oracle):
    # flatter P_t at higher temperature -> lower max P_t -> larger uncertainty (Section 4.3)
    rng = np.random.default_rng(4)
    row = (rng.standard_normal(2000) * 2.0).astype(np.float32)
    unc = [1.0 - oracle.softmax(row, T)[3] for T in (0.3, 0.6, 1.0, 1.5, 3.0)]
    assert all(a < b for a, b in zip(unc, unc[1:]))


# ---------------------------------------------------------------------- hand-worked decisions
def _find_seq(oracle, seed, pos, lo, hi, start=0):
    """A sequence id whose acceptance uniform at `pos` falls in [lo, hi)."""
    for s in range(start, start + 100000):
        if lo <= oracle.accept_uniform(seed, s, pos) < hi:
            return s
    raise AssertionError("no such uniform")


@pytest.mark.parametrize("T", [1.0, 0.5])
def test_hand_worked_three_branches(oracle, T):
    # P_t = (1/2, 1/4, 1/8, 1/8), P_d = (1/4, 1/4, 1/4, 1/4), draft token x = 2:
    #   R = (1/8)/(1/4) = 1/2, uncertainty = 1 - 1/2 = 1/2, beta = 0.4 -> tolerance = 0.2
    #   U <= 0.5 primary accept; 0.5 < U <= 0.7 accepted only through the tolerance; else reject.
    pt, pd = [0.5, 0.25, 0.125, 0.125], [0.25] * 4
    lt, ld = logits_from_probs(pt, T), logits_from_probs(pd, T)
    target = np.stack([lt, lt])[None]       # [1, K+1=2, 4]
    draft = ld[None, None]                  # [1, 1, 4]
    tokens = np.array([[2]], dtype=np.int32)
    seed, beta = 77, 0.4
    for lo, hi, want_path, want_n in [(0.0, 0.45, 1, 1), (0.55, 0.65, 2, 1), (0.75, 1.0, 0, 0)]:
        s = _find_seq(oracle, seed, 0, lo, hi)
        r = oracle.verify(target, draft, tokens, T, beta, seed, seq_ids=np.array([s]))
        assert r.d("R")[0, 0] == pytest.approx(0.5, rel=1e-6)
        assert r.d("unc")[0, 0] == pytest.approx(0.5, rel=1e-6)
        assert r.d("P_t_x")[0, 0] == pytest.approx(0.125, rel=1e-6)
        assert r.d("P_d_x")[0, 0] == pytest.approx(0.25, rel=1e-6)
        U = oracle.accept_uniform(seed, s, 0)
        assert r.d("U")[0, 0] == U
        assert r.d("thr")[0, 0] == pytest.approx(max(U - 0.2, 0.0), abs=1e-6)
        assert r.path[0, 0] == want_path
        assert r.accept_len[0] == want_n
        if want_n == 1:
            assert r.tokens[0, 0] == 2 and 0 <= r.tokens[0, 1] < 4
        else:
            # residual max(0, P_t - P_d) = (1/4, 0, 0, 0): the replacement can only be token 0
            assert r.tokens[0, 0] == 0 and r.tokens[0, 1] == -1
    # with beta = 0 the middle case is rejected: the tolerance is what pardons it
    s = _find_seq(oracle, seed, 0, 0.55, 0.65)
    r0 = oracle.verify(target, draft, tokens, T, 0.0, seed, seq_ids=np.array([s]))
    assert r0.path[0, 0] == 0 and r0.accept_len[0] == 0


def test_hand_worked_uncertainty_uses_target_at_same_position(oracle):
    # target confident (max 7/8), draft flat: uncertainty must be 1/8 (from the TARGET row of
    # the position being verified), not 3/4 (draft) and not that of the next position.
    T, beta = 1.0, 1.0
    pt0 = [0.875, 0.0625, 0.03125, 0.03125]
    pt1 = [0.25, 0.25, 0.25, 0.25]
    pd0 = [0.25, 0.25, 0.25, 0.25]
    target = np.stack([logits_from_probs(pt0, T), logits_from_probs(pt1, T)])[None]
    draft = logits_from_probs(pd0, T)[None, None]
    r = oracle.verify(target, draft, np.array([[1]], dtype=np.int32), T, beta, 5)
    assert r.d("unc")[0, 0] == pytest.approx(0.125, rel=1e-6)
    assert r.d("R")[0, 0] == pytest.approx(0.25, rel=1e-6)
    U = r.d("U")[0, 0]
    assert r.d("thr")[0, 0] == pytest.approx(max(U - 0.125, 0.0), abs=1e-6)


def test_division_guard(oracle):
    # P_d(x) below 1e-10 is replaced by 1e-10 (Section 3.3 item 2): R = P_t(x) / 1e-10
    T = 1.0
    pd = np.array([1e-14, 0.5, 0.25, 0.25 - 1e-14])
    pt = np.array([1e-12, 0.5, 0.25, 0.25 - 1e-12])
    target = np.stack([logits_from_probs(pt, T)] * 2)[None]
    draft = logits_from_probs(pd, T)[None, None]
    r = oracle.verify(target, draft, np.array([[0]], dtype=np.int32), T, 0.0, 1)
    ptx = softmax64(target[0, 0], T)[0]
    assert r.d("R")[0, 0] == pytest.approx(ptx / EPS, rel=1e-9)      # ~0.01, not ~100
    assert r.d("R")[0, 0] < 0.02


def test_comparison_is_not_strict(oracle):
    # Section 3.2 step 5 compares with >=.  With beta = 2 and a target that is uniform over two
    # entries (uncertainty 1/2) the tolerance is 1, so the clamped threshold is exactly 0 for every
    # U, and a draft token the target gives probability 0 (R = 0) is still accepted: 0 >= 0.
    T = 1.0
    lt = np.array([0.0, 0.0, -np.inf, -np.inf], dtype=np.float32)
    ld = logits_from_probs([0.25] * 4, T)
    target = np.stack([lt] * 2)[None]
    draft = ld[None, None]
    for seed in range(5):
        r = oracle.verify(target, draft, np.array([[2]], dtype=np.int32), T, 2.0, seed)
        assert r.d("R")[0, 0] == 0.0 and r.d("thr")[0, 0] == 0.0
        assert r.path[0, 0] == 2 and r.accept_len[0] == 1


def test_out_of_range_token_is_rejected(oracle):
    T = 1.0
    lt = logits_from_probs([0.25] * 4, T)
    target = np.stack([lt] * 3)[None]
    draft = np.stack([lt] * 2)[None]
    r = oracle.verify(target, draft, np.array([[1, 9]], dtype=np.int32), T, 0.5, 3)
    assert r.status == 1 and r.accept_len[0] == 1 and r.path[0, 1] == 0
    assert r.tokens[0, 0] == 1 and 0 <= r.tokens[0, 1] < 4 and r.tokens[0, 2] == -1


# ------------------------------------------------------- beta = 0 == standard rejection sampling
def _standard_speculative_sampling(oracle, target, draft, tokens, T, seed, seq):
    """Textbook loop of the baseline scheme (Section 3.1): accept x_i iff P_t/P_d >= U_i; on the
    first rejection draw from norm(max(0, P_t - P_d)); if nothing is rejected draw from the next
    target row.  numpy/torch fp64, the same noise streams."""
    K, V = draft.shape
    out = []
    for i in range(K):
        pt, pd = softmax64(target[i], T), softmax64(draft[i], T)
        x = int(tokens[i])
        U = oracle.accept_uniform(seed, seq, i)
        if pt[x] / max(pd[x], EPS) >= U:
            out.append(x)
            continue
        g = np.array([oracle.gumbel(seed, seq, i, v) for v in range(V)])
        q = np.maximum(pt - pd, 0.0)
        with np.errstate(divide="ignore"):
            out.append(int(np.argmax(np.log(q) + g)))
        return i, out
    g = np.array([oracle.gumbel(seed, seq, K, v) for v in range(V)])
    out.append(int(np.argmax(target[K].astype(np.float64) / T + g)))
    return K, out


@pytest.mark.parametrize("T", [1.0, 0.7])
def test_beta_zero_is_standard_rejection_sampling(oracle, T):
    rng = np.random.default_rng(10)
    B, K, V = 40, 4, 64
    target = (rng.standard_normal((B, K + 1, V)) * 2.0).astype(np.float32)
    draft = (target[:, :K] + 0.8 * rng.standard_normal((B, K, V))).astype(np.float32)
    tokens = np.stack([[rng.choice(V, p=softmax64(draft[b, i], T)) for i in range(K)]
                       for b in range(B)]).astype(np.int32)
    seed = 1234
    r = oracle.verify(target, draft, tokens, T, 0.0, seed)
    lens = set()
    for b in range(B):
        n, out = _standard_speculative_sampling(oracle, target[b], draft[b], tokens[b], T, seed, b)
        assert r.accept_len[b] == n
        assert list(r.tokens[b, :n + 1]) == out
        assert np.all(r.tokens[b, n + 1:] == -1)
        assert np.all(r.path[b][r.path[b] != 0] == 1)       # no pardon path at beta = 0
        lens.add(n)
    assert len(lens) >= 3        # the case mix covers early, middle and no rejection


# ------------------------------------------------------------------------------- invariants
def _random_problem(rng, B, K, V, noise, T, dtype="f32"):
    target = (rng.standard_normal((B, K + 1, V)) * rng.uniform(0.5, 4.0, (B, K + 1, 1))).astype(np.float32)
    draft = (target[:, :K] + noise * rng.standard_normal((B, K, V))).astype(np.float32)
    if dtype == "bf16":
        target, draft = bf16_bits(target), bf16_bits(draft)
        d64 = bf16_to_f64(draft)
    else:
        d64 = draft.astype(np.float64)
    tokens = np.stack([[rng.choice(V, p=softmax64(d64[b, i], T)) for i in range(K)]
                       for b in range(B)]).astype(np.int32)
    return target, draft, tokens


def test_identical_distributions_accept_everything(oracle):
    rng = np.random.default_rng(20)
    B, K, V = 30, 5, 100
    target, _, _ = _random_problem(rng, B, K, V, 1.0, 1.0)
    draft = target[:, :K].copy()
    tokens = rng.integers(0, V, (B, K)).astype(np.int32)
    for beta in (0.0, 0.3, 1.0):
        r = oracle.verify(target, draft, tokens, 0.9, beta, 99)
        assert np.all(r.accept_len == K)
        assert np.all(r.path == 1)
        np.testing.assert_allclose(r.d("R"), 1.0, rtol=1e-12)
        assert np.all(r.tokens[:, :K] == tokens)
        assert np.all((r.tokens[:, K] >= 0) & (r.tokens[:, K] < V))
        assert np.all(r.samp[:, 3] == 1.0)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_range_prefix_monotone_clamp(oracle, dtype):
    rng = np.random.default_rng(21)
    B, K, V = 60, 6, 200
    T = 0.8
    target, draft, tokens = _random_problem(rng, B, K, V, 1.2, T, dtype)
    prev = None
    for beta in (0.0, 0.1, 0.25, 0.5, 1.0, 3.0):
        r = oracle.verify(target, draft, tokens, T, beta, 7)
        n = r.accept_len
        assert np.all((n >= 0) & (n <= K))
        for b in range(B):
            assert np.all(r.tokens[b, :n[b]] == tokens[b, :n[b]])
            assert 0 <= r.tokens[b, n[b]] < V
            assert np.all(r.tokens[b, n[b] + 1:] == -1)
            # accept length is the index of the first per-position rejection
            rej = np.nonzero(r.path[b] == 0)[0]
            assert n[b] == (rej[0] if len(rej) else K)
        R, U, unc, thr = r.d("R"), r.d("U"), r.d("unc"), r.d("thr")
        # threshold clamp never changes a decision because R >= 0
        assert np.array_equal(r.path != 0, R >= U - beta * unc)
        assert np.array_equal(r.path == 1, R >= U)
        np.testing.assert_allclose(thr, np.maximum(U - beta * unc, 0.0), rtol=0, atol=1e-15)
        assert np.all(thr >= 0.0) and np.all((unc >= 0) & (unc < 1))
        if prev is not None:
            # same seed -> same U; a larger beta only lowers thresholds
            assert np.all((r.path != 0) >= (prev.path != 0))
            assert np.all(n >= prev.accept_len)
            assert np.array_equal(U, prev.d("U"))
        prev = r
    assert prev.accept_len.mean() > oracle.verify(target, draft, tokens, T, 0.0, 7).accept_len.mean()


def test_seq_ids_select_the_noise_stream(oracle):
    # results depend on (seed, sequence id), not on the slot in the batch
    rng = np.random.default_rng(22)
    B, K, V = 12, 3, 50
    target, draft, tokens = _random_problem(rng, B, K, V, 1.0, 1.0)
    ids = rng.permutation(1000)[:B].astype(np.int64) + (1 << 40)
    r = oracle.verify(target, draft, tokens, 1.0, 0.2, 5, seq_ids=ids)
    perm = rng.permutation(B)
    rp = oracle.verify(target[perm], draft[perm], tokens[perm], 1.0, 0.2, 5, seq_ids=ids[perm])
    assert np.array_equal(r.accept_len[perm], rp.accept_len)
    assert np.array_equal(r.tokens[perm], rp.tokens)
    assert not np.array_equal(r.d("U"), oracle.verify(target, draft, tokens, 1.0, 0.2, 6, seq_ids=ids).d("U"))


def test_ragged_matches_rectangular(oracle):
    rng = np.random.default_rng(23)
    V = 80
    Ks = [1, 4, 2, 8, 3]
    B = len(Ks)
    off = np.concatenate([[0], np.cumsum(Ks)]).astype(np.int64)
    T = rng.uniform(0.5, 1.5, B).astype(np.float32)
    beta = rng.uniform(0.0, 1.0, B).astype(np.float32)
    seqs = []
    for b, K in enumerate(Ks):
        seqs.append(_random_problem(rng, 1, K, V, 1.0, float(T[b])))
    target = np.concatenate([s[0][0] for s in seqs])
    draft = np.concatenate([s[1][0] for s in seqs])
    tokens = np.concatenate([s[2][0] for s in seqs])
    r = oracle.verify_ragged(target, draft, tokens, off, T, beta, 31, nthreads=2)
    for b, K in enumerate(Ks):
        one = oracle.verify(seqs[b][0], seqs[b][1], seqs[b][2], float(T[b]), float(beta[b]), 31,
                            seq_ids=np.array([b]))
        assert r.accept_len[b] == one.accept_len[0]
        assert np.array_equal(r.tokens[off[b] + b: off[b + 1] + b + 1], one.tokens[0])
        assert np.array_equal(r.diag[off[b]:off[b + 1]], one.diag[0])
        assert np.array_equal(r.path[off[b]:off[b + 1]], one.path[0])


# -------------------------------------------------------------------------- statistical pins
def _tiled(row, n, extra_dims=1):
    return np.ascontiguousarray(np.broadcast_to(row, (n,) + (1,) * (extra_dims - 1) + row.shape[-1:]))


@pytest.mark.parametrize("beta", [0.0, 0.3, 1.0])
def test_acceptance_probability_closed_form(oracle, beta):
    # P(accept | x) = min(1, R_x + Tol): the acceptance region is [0, R + Tol] (Section 3.2)
    T = 1.0
    pt = np.array([0.40, 0.05, 0.20, 0.10, 0.05, 0.05, 0.10, 0.05])
    pd = np.array([0.10, 0.30, 0.20, 0.05, 0.15, 0.05, 0.05, 0.10])
    lt, ld = logits_from_probs(pt, T), logits_from_probs(pd, T)
    pt64, pd64 = softmax64(lt, T), softmax64(ld, T)
    N, V = 20000, 8
    tol = beta * (1.0 - pt64.max())
    target = np.ascontiguousarray(np.broadcast_to(lt, (N, 2, V)))
    draft = np.ascontiguousarray(np.broadcast_to(ld, (N, 1, V)))
    for x in (1, 4, 7, 0):
        tokens = np.full((N, 1), x, dtype=np.int32)
        r = oracle.verify(target, draft, tokens, T, beta, 1000 + x, nthreads=4)
        want = min(1.0, pt64[x] / pd64[x] + tol)
        k = int((r.accept_len == 1).sum())
        if want >= 1.0:
            assert k == N
        else:
            assert stats.binomtest(k, N, want).pvalue > 1e-4, (x, k / N, want)


def _output_law(pt, pd, tol):
    a = np.minimum(pd, pt + tol * pd)              # accepted mass per token
    q = np.maximum(pt - pd, 0.0)
    return a + (1.0 - a.sum()) * q / q.sum()


@pytest.mark.parametrize("beta,T", [(0.0, 1.0), (0.0, 0.6), (0.5, 1.0), (1.0, 1.4)])
def test_output_law_tiny_vocabulary(oracle, beta, T):
    # V = 8, K = 1, x ~ P_d.  For beta = 0 the emitted token follows P_target exactly (the
    # losslessness of standard speculative sampling); for beta > 0 it follows the closed form
    # a(v) + (1 - sum a) q(v) / sum q with a(v) = min(P_d, P_t + Tol P_d).
    rng = np.random.default_rng(40)
    V, N = 8, 200000
    lt = (rng.standard_normal(V) * 1.5).astype(np.float32)
    ld = (lt + 0.9 * rng.standard_normal(V)).astype(np.float32)
    pt, pd = softmax64(lt, T), softmax64(ld, T)
    tokens = rng.choice(V, size=(N, 1), p=pd).astype(np.int32)
    target = np.ascontiguousarray(np.broadcast_to(lt, (N, 2, V)))
    draft = np.ascontiguousarray(np.broadcast_to(ld, (N, 1, V)))
    r = oracle.verify(target, draft, tokens, T, beta, 4242, nthreads=4)
    obs = np.bincount(r.tokens[:, 0], minlength=V)
    law = _output_law(pt, pd, beta * (1.0 - pt.max()))
    if beta == 0.0:
        np.testing.assert_allclose(law, pt, rtol=1e-12)
    assert stats.chisquare(obs, law * N).pvalue > 1e-4
    # acceptance rate: sum_x min(P_d, P_t + Tol P_d); for beta = 0 this is 1 - TV(P_t, P_d)
    acc = np.minimum(pd, pt + beta * (1.0 - pt.max()) * pd).sum()
    if beta == 0.0:
        assert acc == pytest.approx(1.0 - 0.5 * np.abs(pt - pd).sum(), rel=1e-12)
    assert stats.binomtest(int((r.accept_len == 1).sum()), N, acc).pvalue > 1e-4
    # a deliberately wrong law (plain resampling from P_t on rejection) must be told apart
    wrong = np.minimum(pd, pt) + (1.0 - np.minimum(pd, pt).sum()) * pt
    if beta == 0.0:
        assert stats.chisquare(obs, wrong / wrong.sum() * N).pvalue < 1e-6


def test_bonus_token_follows_target_row(oracle):
    # all accepted (identical rows) -> token K ~ softmax(target row K / T): Gumbel-max = categorical
    rng = np.random.default_rng(41)
    V, N, T = 8, 100000, 0.7
    l0 = (rng.standard_normal(V)).astype(np.float32)
    lK = (rng.standard_normal(V) * 2.0).astype(np.float32)
    target = np.ascontiguousarray(np.broadcast_to(np.stack([l0, lK]), (N, 2, V)))
    draft = np.ascontiguousarray(np.broadcast_to(l0, (N, 1, V)))
    tokens = rng.integers(0, V, (N, 1)).astype(np.int32)
    r = oracle.verify(target, draft, tokens, T, 0.1, 777, nthreads=4)
    assert np.all(r.accept_len == 1)
    obs = np.bincount(r.tokens[:, 1], minlength=V)
    assert stats.chisquare(obs, softmax64(lK, T) * N).pvalue > 1e-4
    assert stats.chisquare(obs, softmax64(l0, T) * N).pvalue < 1e-6     # not the wrong row
    assert stats.chisquare(obs, softmax64(lK, 1.0) * N).pvalue < 1e-6   # temperature applied


def test_residual_law_and_empty_residual_fallback(oracle):
    # forced rejection (U-independent: R = 0 because P_t(x) = 0 exactly): the replacement follows
    # norm(max(0, P_t - P_d)) and never returns a token with P_t <= P_d
    rng = np.random.default_rng(42)
    V, N, T = 8, 100000, 1.0
    lt = (rng.standard_normal(V)).astype(np.float32)
    ld = (lt + rng.standard_normal(V)).astype(np.float32)
    lt[3] = -np.inf
    pt, pd = softmax64(lt, T), softmax64(ld, T)
    target = np.ascontiguousarray(np.broadcast_to(lt, (N, 2, V)))
    draft = np.ascontiguousarray(np.broadcast_to(ld, (N, 1, V)))
    tokens = np.full((N, 1), 3, dtype=np.int32)
    r = oracle.verify(target, draft, tokens, T, 0.0, 99, nthreads=4)
    # U = 0 would accept even R = 0 (non-strict comparison): allow for those few
    rej = r.accept_len == 0
    assert rej.sum() >= N - 3
    q = np.maximum(pt - pd, 0.0)
    obs = np.bincount(r.tokens[rej, 0], minlength=V)
    keep = q > 0
    assert np.all(obs[~keep] == 0)
    assert stats.chisquare(obs[keep], q[keep] / q.sum() * rej.sum()).pvalue > 1e-4
    # identical rows + a token with P_d below the guard: rejection with an empty residual
    ld2 = lt.copy()
    draft2 = np.ascontiguousarray(np.broadcast_to(ld2, (N, 1, V)))
    r2 = oracle.verify(target, draft2, tokens, T, 0.0, 99, nthreads=4)
    rej2 = r2.accept_len == 0
    assert rej2.sum() >= N - 3 and np.all(r2.samp[rej2, 3] == 2.0)
    obs2 = np.bincount(r2.tokens[rej2, 0], minlength=V)
    assert obs2[3] == 0
    assert stats.chisquare(np.delete(obs2, 3), np.delete(pt, 3) * rej2.sum()).pvalue > 1e-4


# ------------------------------------------ the Gumbel arg-max, its runner-up and their gap
LN2 = math.log(2.0)


def _pow2_logits(exponents):
    """fp32 logits k (small integers): at temperature 1/ln 2 their softmax weights are 2^k."""
    return np.asarray(exponents, dtype=np.float32)


def _numpy_top2(scores):
    """(winner, runner-up) of a score vector by a stable sort: highest score first, lowest index
    first among equals; -inf entries are not candidates."""
    scores = np.asarray(scores, dtype=np.float64)
    cand = [v for v in np.argsort(-scores, kind="stable") if scores[v] > -np.inf]
    return (cand[0] if cand else -1), (cand[1] if len(cand) > 1 else -1)


def test_top2_bookkeeping_against_sort(oracle):
    # exact ties (which the verification's own noise never produces) and every ordering of three
    # distinct values, against numpy's stable sort
    cases = [[1.0, 2.0, 3.0], [3.0, 2.0, 1.0], [2.0, 3.0, 1.0], [1.0, 3.0, 2.0], [3.0, 1.0, 2.0],
             [2.0, 1.0, 3.0],
             [5.0, 5.0], [1.0, 5.0, 5.0], [5.0, 1.0, 5.0], [5.0, 5.0, 5.0], [7.0, 5.0, 5.0],
             [5.0, 5.0, 7.0], [-np.inf, 4.0], [4.0], [-np.inf, -np.inf], [0.5, -np.inf, 0.5, 0.25]]
    rng = np.random.default_rng(8)
    cases += [list(rng.integers(0, 4, n).astype(np.float64)) for n in range(1, 9) for _ in range(20)]
    for sc in cases:
        arg, samp = oracle.top2(np.array(sc))
        w, r = _numpy_top2(sc)
        assert arg == w, sc
        assert int(samp[4]) == r, sc
        if w >= 0:
            assert samp[0] == sc[w]
        if r >= 0:
            assert samp[1] == sc[r] and samp[2] == sc[w] - sc[r], sc
        elif w >= 0:
            assert samp[1] == -np.inf and samp[2] == np.inf, sc


def test_replacement_scores_runner_up_and_gap(oracle):
    # P_t = (1/2, 1/4, 1/8, 1/8), P_d = (1/8, 1/8, 1/4, 1/2) as exact powers of two (T = 1/ln 2),
    # draft token 3: R = 1/4; the sequences picked have U >= 1/2, so with beta = 0 they reject.
    # Residual max(0, P_t - P_d) = (3/8, 1/8, 0, 0): two candidates with scores
    # log(3/8) + g(0) and log(1/8) + g(1), written out here with numpy.
    T = 1.0 / LN2
    lt, ld = _pow2_logits([-1, -2, -3, -3]), _pow2_logits([-3, -3, -2, -1])
    target = np.stack([lt, lt])[None]
    draft = ld[None, None]
    tokens = np.array([[3]], dtype=np.int32)
    seed = 2024
    first_wins = 0
    s = 0
    for _ in range(60):
        s = _find_seq(oracle, seed, 0, 0.5, 1.0, start=s + 1)
        r = oracle.verify(target, draft, tokens, T, 0.0, seed, seq_ids=np.array([s]))
        assert r.accept_len[0] == 0 and r.samp[0, 3] == 0.0
        pt, pd = softmax64(lt, T), softmax64(ld, T)
        q = pt - pd
        sc = np.array([math.log(q[0]) + oracle.gumbel(seed, s, 0, 0),
                       math.log(q[1]) + oracle.gumbel(seed, s, 0, 1)])
        w = 0 if sc[0] >= sc[1] else 1
        first_wins += (w == 0)
        assert r.tokens[0, 0] == w
        assert r.samp[0, 0] == pytest.approx(sc[w], abs=1e-12)
        assert r.samp[0, 1] == pytest.approx(sc[1 - w], abs=1e-12)
        assert r.samp[0, 2] == pytest.approx(sc[w] - sc[1 - w], abs=1e-12)
        assert r.samp[0, 2] > 0.0
        assert int(r.samp[0, 4]) == 1 - w
    assert 30 <= first_wins < 60          # both orders of arrival were exercised (3:1 odds)


def test_single_candidate_has_no_runner_up(oracle):
    # P_t = (3/4, 1/4), P_d = (1/4, 3/4), draft token 1: R = 1/3; residual (1/2, 0): one candidate
    T = 1.0
    target = np.stack([logits_from_probs([0.75, 0.25], T)] * 2)[None]
    draft = logits_from_probs([0.25, 0.75], T)[None, None]
    s = _find_seq(oracle, 9, 0, 0.5, 1.0)
    r = oracle.verify(target, draft, np.array([[1]], dtype=np.int32), T, 0.0, 9, seq_ids=np.array([s]))
    assert r.accept_len[0] == 0 and r.tokens[0, 0] == 0
    assert r.samp[0, 0] == pytest.approx(math.log(0.5) + oracle.gumbel(9, s, 0, 0), abs=1e-7)
    assert r.samp[0, 1] == -np.inf and r.samp[0, 2] == np.inf and int(r.samp[0, 4]) == -1


def test_bonus_scores_runner_up_and_gap(oracle):
    # identical rows accept everything; the bonus token is arg-max of l/T + g over target row K
    T = 0.7
    l0 = np.array([0.5, -1.0, 2.0], dtype=np.float32)
    lK = np.array([1.0, 0.25, -0.5], dtype=np.float32)
    target = np.stack([l0, lK])[None]
    draft = l0[None, None]
    for s in range(40):
        r = oracle.verify(target, draft, np.array([[1]], dtype=np.int32), T, 0.3, 5, seq_ids=np.array([s]))
        assert r.accept_len[0] == 1 and r.samp[0, 3] == 1.0
        sc = np.array([float(lK[v]) / T + oracle.gumbel(5, s, 1, v) for v in range(3)])
        w, ru = _numpy_top2(sc)
        assert r.tokens[0, 1] == w and int(r.samp[0, 4]) == ru
        assert r.samp[0, 0] == pytest.approx(sc[w], abs=1e-12)
        assert r.samp[0, 1] == pytest.approx(sc[ru], abs=1e-12)
        assert r.samp[0, 2] == pytest.approx(sc[w] - sc[ru], abs=1e-12)


# ----------------------------------------------- alternative uncertainty measure (Section 5)
def test_residual_support_ignores_rounding_noise(oracle):
    """Target and draft put 1 - 3.5e-13 on entry 0 and differ only far down the tail, so that
    p_t(0) - p_d(0) is about +2e-15, i.e. a few units in the last place of two numbers near 1.  That
    is the softmax's own rounding noise, not residual mass: the replacement token has to come from
    the entries where the target really is more likely (here only entry 1, with q ~ 4e-15)."""
    T = 1.0
    target = np.array([30.0, 1.0, 0.0, -1.0, -2.0, -3.0], dtype=np.float32)
    draft = np.array([30.0, 1.0 - 2.0 ** -6, 2.0 ** -4, -1.0, -2.0, -3.0], dtype=np.float32)
    pt, pd = softmax64(target, T), softmax64(draft, T)
    rel = (pt - pd) / (pt + pd)
    # the premise: entry 1 carries real residual mass, entry 2 none, and entries 0, 3, 4, 5 (equal
    # logits in both rows) differ only through the two normalisers, by ~1e-15 relative
    assert rel[1] > 1e-3 and rel[2] < 0 and ((rel[[0, 3, 4, 5]] > 0) & (rel[[0, 3, 4, 5]] < 1e-14)).all()
    assert pt[0] - pd[0] > 0.3 * (pt[1] - pd[1])       # unfloored, entry 0 would win often
    B = 3000
    r = oracle.verify(np.stack([target] * 2)[None].repeat(B, 0), draft[None, None].repeat(B, 0),
                      np.full((B, 1), 2, dtype=np.int32), T, 0.0, 11, nthreads=4)
    rejected = r.accept_len == 0
    assert rejected.sum() > 2900          # P_d(x) is below the division guard: R = P_t(x) / 1e-10 ~ 1e-3
    assert (r.tokens[rejected, 0] == 1).all()


def test_entropy_against_library(oracle):
    rng = np.random.default_rng(50)
    for V in (2, 17, 5000):
        p = rng.dirichlet(np.ones(V) * 0.3)
        p[rng.integers(0, V)] = 0.0
        p /= p.sum()
        assert oracle.entropy(p) == pytest.approx(stats.entropy(p), rel=1e-12)
    assert oracle.entropy(np.full(64, 1 / 64)) == pytest.approx(math.log(64), rel=1e-14)
    assert oracle.entropy(np.array([0.0, 1.0, 0.0])) == 0.0


def test_entropy_uncertainty_hand_worked(oracle):
    # P_t = (1/2, 1/4, 1/8, 1/8): H = 1.75 log 2, log V = 2 log 2 -> uncertainty 7/8 (1 - max P_t
    # would be 1/2).  P_d uniform, x = 2: R = 1/2.  With beta = 0.4 the tolerance is 0.35:
    # U <= 0.5 primary, 0.5 < U <= 0.85 pardon, else reject; the max-prob measure would stop at 0.7.
    T, beta, seed = 1.0, 0.4, 123
    lt = logits_from_probs([0.5, 0.25, 0.125, 0.125], T)
    ld = logits_from_probs([0.25] * 4, T)
    target, draft = np.stack([lt, lt])[None], ld[None, None]
    tokens = np.array([[2]], dtype=np.int32)
    for lo, hi, want in [(0.0, 0.45, 1), (0.55, 0.65, 2), (0.72, 0.83, 2), (0.87, 1.0, 0)]:
        s = _find_seq(oracle, seed, 0, lo, hi)
        r = oracle.verify(target, draft, tokens, T, beta, seed, seq_ids=np.array([s]),
                          uncertainty=oracle.UNC_ENTROPY)
        assert r.d("unc")[0, 0] == pytest.approx(0.875, rel=1e-6)
        U = r.d("U")[0, 0]
        assert r.d("thr")[0, 0] == pytest.approx(max(U - 0.35, 0.0), abs=1e-6)
        assert r.path[0, 0] == want
    s = _find_seq(oracle, seed, 0, 0.72, 0.83)
    r = oracle.verify(target, draft, tokens, T, beta, seed, seq_ids=np.array([s]))
    assert r.path[0, 0] == 0 and r.d("unc")[0, 0] == pytest.approx(0.5, rel=1e-6)


def test_entropy_uncertainty_limits_and_acceptance_rate(oracle):
    rng = np.random.default_rng(51)
    V, N, T, beta = 8, 20000, 0.8, 0.6
    # uniform target: uncertainty exactly 1; near one-hot target: close to 0
    flat = np.zeros(V, dtype=np.float32)
    peaked = np.array([40.0] + [0.0] * (V - 1), dtype=np.float32)
    for row, want in ((flat, 1.0), (peaked, 0.0)):
        r = oracle.verify(np.stack([row, row])[None], row[None, None], np.array([[1]], dtype=np.int32),
                          T, beta, 1, uncertainty=oracle.UNC_ENTROPY)
        assert r.d("unc")[0, 0] == pytest.approx(want, abs=1e-12)
    # acceptance probability min(1, R + beta H / log V) for a fixed token
    lt = (rng.standard_normal(V) * 1.5).astype(np.float32)
    ld = (lt + rng.standard_normal(V)).astype(np.float32)
    pt, pd = softmax64(lt, T), softmax64(ld, T)
    tol = beta * stats.entropy(pt) / math.log(V)
    target = np.ascontiguousarray(np.broadcast_to(lt, (N, 2, V)))
    draft = np.ascontiguousarray(np.broadcast_to(ld, (N, 1, V)))
    x = int(np.argmin(pt / pd))
    r = oracle.verify(target, draft, np.full((N, 1), x, dtype=np.int32), T, beta, 77, nthreads=4,
                      uncertainty=oracle.UNC_ENTROPY)
    want = min(1.0, pt[x] / pd[x] + tol)
    assert want < 1.0
    assert stats.binomtest(int((r.accept_len == 1).sum()), N, want).pvalue > 1e-4
    # and it differs from the max-prob tolerance
    want_mp = min(1.0, pt[x] / pd[x] + beta * (1.0 - pt.max()))
    assert stats.binomtest(int((r.accept_len == 1).sum()), N, want_mp).pvalue < 1e-6


def test_variance_against_its_definition(oracle):
    # closed forms: uniform 1 - 1/V, a point mass 0, two points 2 p (1 - p)
    assert oracle.variance(np.full(64, 1 / 64)) == pytest.approx(1 - 1 / 64, rel=1e-14)
    assert oracle.variance(np.array([0.0, 1.0, 0.0])) == 0.0
    assert oracle.variance(np.array([0.3, 0.7])) == pytest.approx(2 * 0.3 * 0.7, rel=1e-14)
    rng = np.random.default_rng(60)
    for V in (2, 17, 5000):
        p = rng.dirichlet(np.ones(V) * 0.3)
        assert oracle.variance(p) == pytest.approx(1.0 - float(np.dot(p, p)), rel=1e-11, abs=1e-15)
    # the name: trace of the covariance matrix of one-hot draws from p
    p = np.array([0.5, 0.2, 0.15, 0.1, 0.05])
    onehot = rng.multinomial(1, p, size=400000).astype(np.float64)
    assert float(np.trace(np.cov(onehot.T))) == pytest.approx(oracle.variance(p), rel=5e-3)


def test_variance_uncertainty_hand_worked(oracle):
    # P_t = (1/2, 1/4, 1/8, 1/8): sum of squares 11/32, uncertainty 21/32 = 0.65625 (1 - max P_t is
    # 1/2, the entropy measure 7/8).  P_d uniform, x = 2: R = 1/2.  beta = 0.4: tolerance 0.2625,
    # so U <= 0.5 primary, 0.5 < U <= 0.7625 pardon, else reject.
    T, beta, seed = 1.0, 0.4, 321
    lt = logits_from_probs([0.5, 0.25, 0.125, 0.125], T)
    ld = logits_from_probs([0.25] * 4, T)
    target, draft = np.stack([lt, lt])[None], ld[None, None]
    tokens = np.array([[2]], dtype=np.int32)
    for lo, hi, want in [(0.0, 0.45, 1), (0.55, 0.65, 2), (0.71, 0.75, 2), (0.78, 0.84, 0), (0.87, 1.0, 0)]:
        s = _find_seq(oracle, seed, 0, lo, hi)
        r = oracle.verify(target, draft, tokens, T, beta, seed, seq_ids=np.array([s]),
                          uncertainty=oracle.UNC_VARIANCE)
        assert r.d("unc")[0, 0] == pytest.approx(0.65625, rel=1e-6)
        U = r.d("U")[0, 0]
        assert r.d("thr")[0, 0] == pytest.approx(max(U - 0.2625, 0.0), abs=1e-6)
        assert r.path[0, 0] == want
    # the same uniforms under the other two measures: 0.71..0.75 is beyond 1 - max P_t's reach,
    # 0.78..0.84 within the entropy measure's
    s = _find_seq(oracle, seed, 0, 0.71, 0.75)
    assert oracle.verify(target, draft, tokens, T, beta, seed, seq_ids=np.array([s])).path[0, 0] == 0
    s = _find_seq(oracle, seed, 0, 0.78, 0.84)
    assert oracle.verify(target, draft, tokens, T, beta, seed, seq_ids=np.array([s]),
                         uncertainty=oracle.UNC_ENTROPY).path[0, 0] == 2


def test_variance_uncertainty_limits_order_and_acceptance_rate(oracle):
    rng = np.random.default_rng(61)
    V, N, T, beta = 8, 20000, 0.8, 0.6
    flat = np.zeros(V, dtype=np.float32)
    peaked = np.array([40.0] + [0.0] * (V - 1), dtype=np.float32)
    for row, want in ((flat, 1.0 - 1.0 / V), (peaked, 0.0)):
        r = oracle.verify(np.stack([row, row])[None], row[None, None], np.array([[1]], dtype=np.int32),
                          T, beta, 1, uncertainty=oracle.UNC_VARIANCE)
        assert r.d("unc")[0, 0] == pytest.approx(want, abs=1e-12)
    # sum p^2 <= max p: never below the paper's measure, never above 1 - 1/V
    rows = (rng.standard_normal((50, 2, 33)) * rng.uniform(0.2, 6.0, (50, 1, 1))).astype(np.float32)
    tok = rng.integers(0, 33, (50, 1)).astype(np.int32)
    r_var = oracle.verify(rows, rows[:, :1], tok, T, beta, 5, uncertainty=oracle.UNC_VARIANCE)
    r_max = oracle.verify(rows, rows[:, :1], tok, T, beta, 5)
    assert (r_var.d("unc") >= r_max.d("unc") - 1e-15).all()
    assert (r_var.d("unc") <= 1.0 - 1.0 / 33 + 1e-15).all()
    assert (r_var.d("unc") > r_max.d("unc") + 1e-3).any()
    # acceptance probability min(1, R + beta (1 - sum p_t^2)) for a fixed token
    lt = (rng.standard_normal(V) * 1.5).astype(np.float32)
    ld = (lt + rng.standard_normal(V)).astype(np.float32)
    pt, pd = softmax64(lt, T), softmax64(ld, T)
    tol = beta * (1.0 - float(np.dot(pt, pt)))
    target = np.ascontiguousarray(np.broadcast_to(lt, (N, 2, V)))
    draft = np.ascontiguousarray(np.broadcast_to(ld, (N, 1, V)))
    x = int(np.argmin(pt / pd))
    r = oracle.verify(target, draft, np.full((N, 1), x, dtype=np.int32), T, beta, 78, nthreads=4,
                      uncertainty=oracle.UNC_VARIANCE)
    want = min(1.0, pt[x] / pd[x] + tol)
    assert want < 1.0
    assert stats.binomtest(int((r.accept_len == 1).sum()), N, want).pvalue > 1e-4
    want_mp = min(1.0, pt[x] / pd[x] + beta * (1.0 - pt.max()))
    assert stats.binomtest(int((r.accept_len == 1).sum()), N, want_mp).pvalue < 1e-6


def test_sequence_without_draft_tokens(oracle):
    """K_b = 0 in a ragged batch: accept length 0 and the token is the Gumbel-max draw from the
    sequence's only target row with the noise of position 0 (written out here with numpy)."""
    rng = np.random.default_rng(70)
    V, seed = 300, 12
    off = np.array([0, 2, 2, 3, 3, 3, 5], dtype=np.int64)          # K_b = 2, 0, 1, 0, 0, 2
    B, R = 6, 5
    target = (rng.standard_normal((R + B, V)) * 2).astype(np.float32)
    draft = (target[[0, 1, 3, 6, 7]] + rng.standard_normal((R, V))).astype(np.float32)
    tokens = rng.integers(0, V, R).astype(np.int32)
    T = np.array([1.0, 0.7, 1.3, 0.5, 2.0, 1.0], dtype=np.float32)
    beta = np.full(B, 0.2, dtype=np.float32)
    ids = np.array([5, 900, 7, 2 ** 40 + 3, 11, 13], dtype=np.int64)
    r = oracle.verify_ragged(target, draft, tokens, off, T, beta, seed, seq_ids=ids)
    for b in (1, 3, 4):
        row = target[off[b] + b].astype(np.float64)
        g = np.array([oracle.gumbel(seed, int(ids[b]), 0, v) for v in range(V)])
        assert r.accept_len[b] == 0
        assert r.tokens[off[b] + b] == int(np.argmax(row / float(T[b]) + g))
    # the other sequences are what they are without the empty ones around them
    keep = np.array([0, 2, 5])
    t2 = np.concatenate([target[off[b] + b: off[b + 1] + b + 1] for b in keep])
    d2 = np.concatenate([draft[off[b]: off[b + 1]] for b in keep])
    k2 = np.concatenate([tokens[off[b]: off[b + 1]] for b in keep])
    off2 = np.array([0, 2, 3, 5], dtype=np.int64)
    r2 = oracle.verify_ragged(t2, d2, k2, off2, T[keep], beta[keep], seed, seq_ids=ids[keep])
    assert np.array_equal(r2.accept_len, r.accept_len[keep])
    for i, b in enumerate(keep):
        assert np.array_equal(r2.tokens[off2[i] + i: off2[i + 1] + i + 1], r.tokens[off[b] + b: off[b + 1] + b + 1])
