"""Producer-side fusion on the GPU: the vocabulary projection with the statistics epilogue, against
the CPU oracle (fp64 dot products, explicit bf16 rounding, three-pass softmax on the emitted rows),
and the verification step started from the imported statistics."""
import os

import numpy as np
import pytest
import torch

from parity_util import compare

pytestmark = pytest.mark.gpu

NTHREADS = min(16, os.cpu_count() or 1)


@pytest.fixture(scope="module")
def ears():
    import paper_2512_13194_amd as p
    p.lib()
    assert torch.cuda.is_available()
    return p


def _log(msg):
    print(msg, flush=True)


def _bits(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def _val(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _operands(N, D, V, seed, sigma=2.5):
    g = torch.Generator(device="cuda").manual_seed(seed)
    hidden = torch.randn(N, D, generator=g, device="cuda").to(torch.bfloat16)
    weight = (torch.randn(V, D, generator=g, device="cuda") * (sigma / D ** 0.5)).to(torch.bfloat16)
    return hidden, weight


def _check_logits(got_bits, exact, want_bits):
    """Every emitted logit is a bf16 neighbour of the exact sum (fp32 accumulation moves a sum by far
    less than one bf16 step), and nearly all are the nearest one."""
    got = _val(got_bits)
    step = np.maximum(np.abs(exact), 2.0 ** -126) * 2.0 ** -7      # one bf16 step at that magnitude
    assert (np.abs(got - exact) <= 0.51 * step + 1e-5).all()
    assert (got_bits == want_bits).mean() > 0.995


def _check_stats(oracle, logits_bits, row_max, row_sum, T, rows):
    for n in rows:
        Tn = float(T[n]) if isinstance(T, np.ndarray) else float(np.float32(T))
        _, m, Z, _ = oracle.softmax(logits_bits[n], Tn)
        assert row_max[n] == m, (n, row_max[n], m)
        assert abs(row_sum[n] - Z) <= 1e-5 * Z, (n, row_sum[n], Z)


@pytest.mark.parametrize("N,D,V", [(1, 64, 1), (70, 128, 1000), (300, 192, 513), (257, 64, 255),
                                   (33, 256, 2049), (512, 64, 768)])
def test_projection_and_statistics_small(ears, oracle, N, D, V):
    _log("lm_head N=%d D=%d V=%d" % (N, D, V))
    hidden, weight = _operands(N, D, V, seed=N + V)
    T = 0.8
    logits, row_max, row_sum = ears.ears_lm_head_bf16(hidden, weight, temperature=T)
    torch.cuda.synchronize()
    exact, want = oracle.lm_head(_bits(hidden), _bits(weight), nthreads=NTHREADS)
    got = _bits(logits)
    _check_logits(got, exact, want)
    _check_stats(oracle, got, row_max.cpu().numpy(), row_sum.cpu().numpy(), T, range(N))


def test_statistics_keep_small_terms_beside_a_dominant_logit(ears, oracle):
    """Rows whose softmax is dominated by one entry (weight row n is a multiple of hidden row n):
    Z = 1 + ~4e-4 from thousands of terms near 1e-8.  The slice that holds the dominant entry sums
    its terms in short fp32 runs combined in fp64, so they are not rounded away at ulp(1)."""
    _log("lm_head: dominant logit")
    N, D, V = 64, 128, 8192
    hidden, weight = _operands(N, D, V, 9)
    h = hidden.float()
    weight[:N] = (h * (20.0 / (h * h).sum(1, keepdim=True))).to(torch.bfloat16)
    logits, rm, rs = ears.ears_lm_head_bf16(hidden, weight, temperature=1.0)
    torch.cuda.synchronize()
    bits, rs = _bits(logits), rs.cpu().numpy()
    worst = 0.0
    for n in range(N):
        _, m, Z, _ = oracle.softmax(bits[n], 1.0)
        assert 1.0 < Z < 1.01
        worst = max(worst, abs(rs[n] / Z - 1.0))
    _log("  worst relative error of Z: %.2e" % worst)
    assert worst < 2e-7


def test_per_row_temperature(ears, oracle):
    _log("lm_head per-row temperature")
    N, D, V = 40, 128, 3000
    hidden, weight = _operands(N, D, V, seed=5)
    T = (torch.rand(N, device="cuda") + 0.5).float()
    logits, row_max, row_sum = ears.ears_lm_head_bf16(hidden, weight, row_temperature=T)
    torch.cuda.synchronize()
    _check_stats(oracle, _bits(logits), row_max.cpu().numpy(), row_sum.cpu().numpy(),
                 T.cpu().numpy(), range(N))


def test_verification_from_imported_statistics(ears, oracle):
    """Target and draft logits come from two projections; their statistics are imported and the
    step runs DECIDE | SAMPLE only.  Oracle: the whole verification on the emitted logits."""
    _log("lm_head -> import -> verify")
    B, K, V, D, T, beta, seed = 12, 3, 5000, 128, 0.9, 0.3, 17
    ht, wt = _operands(B * (K + 1), D, V, seed=21)
    g = torch.Generator(device="cuda").manual_seed(22)
    wd = (wt.float() + 0.08 * torch.randn(V, D, generator=g, device="cuda")).to(torch.bfloat16)
    hd = ht.view(B, K + 1, D)[:, :K].reshape(B * K, D).contiguous()
    tl, tm, tz = ears.ears_lm_head_bf16(ht, wt, temperature=T)
    dl, dm, dz = ears.ears_lm_head_bf16(hd, wd, temperature=T)
    target, draft = tl.view(B, K + 1, V), dl.view(B, K, V)
    tokens = torch.multinomial(torch.softmax(draft.float().view(B * K, V) / T, -1), 1,
                               generator=g).view(B, K).to(torch.int32)
    ws = torch.empty(ears.ears_workspace_bytes(B * K, B, V), dtype=torch.uint8, device="cuda")
    ears.ears_import_stats(target, draft, tokens, tm, tz, dm, dz, ws)
    out = ears.ears_verify_ex(target, draft, tokens, temperature=T, beta=beta, seed=seed, workspace=ws,
                              stages=ears.EARS_STAGE_DECIDE | ears.EARS_STAGE_SAMPLE,
                              want_stats=True, want_path=True)
    torch.cuda.synchronize()
    ora = oracle.verify(_bits(target), _bits(draft), tokens.cpu().numpy(), float(np.float32(T)),
                        float(np.float32(beta)), seed, nthreads=NTHREADS)
    rep = compare(ora, out["accept_len"].cpu().numpy(), out["tokens"].cpu().numpy(),
                  out["stats"].cpu().numpy(), out["path"].cpu().numpy(), None, K, 2e-3,
                  tokens.cpu().numpy(), V)
    assert rep.exempt_decisions == 0 and rep.exempt_tokens == 0
    assert 0 < ora.accept_len.sum() < B * K
    # and it is what the unfused call gives on the same logits
    full = ears.ears_verify_ex(target, draft, tokens, temperature=T, beta=beta, seed=seed)
    torch.cuda.synchronize()
    assert torch.equal(full["accept_len"], out["accept_len"]) and torch.equal(full["tokens"], out["tokens"])


def test_headline_shape_sampled(ears, oracle):
    """N = 256 * 9 rows, D = 4096, V = 128256: sampled logits against single fp64 dot products and
    sampled rows' statistics against the oracle's softmax of the emitted row."""
    _log("lm_head headline shape")
    N, D, V, T = 2304, 4096, 128256, 1.0
    hidden, weight = _operands(N, D, V, seed=1)
    logits, row_max, row_sum = ears.ears_lm_head_bf16(hidden, weight, temperature=T)
    torch.cuda.synchronize()
    rng = np.random.default_rng(3)
    ns = np.concatenate([rng.integers(0, N, 1500), [0, N - 1, 255, 256, 2303]])
    vs = np.concatenate([rng.integers(0, V, 1500), [0, V - 1, 255, 256, 128255]])
    hb, wb = _bits(hidden), _bits(weight)
    got = _val(_bits(logits[torch.as_tensor(ns, device="cuda"), torch.as_tensor(vs, device="cuda")]))
    exact = np.array([oracle.lm_head_dot(hb, wb, int(n), int(v)) for n, v in zip(ns, vs)])
    step = np.maximum(np.abs(exact), 2.0 ** -126) * 2.0 ** -7
    assert (np.abs(got - exact) <= 0.51 * step + 1e-4).all()
    rows = [0, 1, 255, 256, 1000, 2303]
    lb = _bits(logits[torch.as_tensor(rows, device="cuda")])
    rm, rs = row_max.cpu().numpy(), row_sum.cpu().numpy()
    for i, n in enumerate(rows):
        _, m, Z, _ = oracle.softmax(lb[i], T)
        assert rm[n] == m and abs(rs[n] - Z) <= 1e-5 * Z


def test_weight_matrix_larger_than_4_gib(ears, oracle):
    """D = 16384, V = 131072 + 700: the weight matrix is 4.3 GB, so its last 700 rows lie beyond
    what a 32-bit byte offset from the matrix base reaches; every tile addresses its rows from its
    own base.  Sampled logits (many of them in those rows) against single fp64 dot products, and
    sampled rows' statistics against the oracle's softmax of the emitted row."""
    _log("lm_head weight > 4 GiB")
    N, D, V, T = 300, 16384, 131072 + 700, 1.0
    g = torch.Generator(device="cuda").manual_seed(17)
    hidden = torch.randn(N, D, generator=g, device="cuda").to(torch.bfloat16)
    weight = torch.empty(V, D, dtype=torch.bfloat16, device="cuda")
    for r0 in range(0, V, 16384):          # generated in slices: no fp32 copy of the whole matrix
        r1 = min(V, r0 + 16384)
        weight[r0:r1] = (torch.randn(r1 - r0, D, generator=g, device="cuda") * (2.5 / D ** 0.5)).to(torch.bfloat16)
    logits, row_max, row_sum = ears.ears_lm_head_bf16(hidden, weight, temperature=T)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    ns = np.concatenate([rng.integers(0, N, 400), [0, N - 1, 255, 256]])
    vs = np.concatenate([rng.integers(0, V, 200), rng.integers(131072, V, 200), [0, 131071, 131072, V - 1]])
    hb = _bits(hidden)
    wb = _bits(weight[torch.as_tensor(vs, device="cuda")])          # only the sampled weight rows
    got = _val(_bits(logits[torch.as_tensor(ns, device="cuda"), torch.as_tensor(vs, device="cuda")]))
    exact = np.array([oracle.lm_head_dot(hb, wb, int(n), i) for i, n in enumerate(ns)])
    step = np.maximum(np.abs(exact), 2.0 ** -126) * 2.0 ** -7
    assert (np.abs(got - exact) <= 0.51 * step + 1e-4).all()
    rows = [0, 255, 256, N - 1]
    lb = _bits(logits[torch.as_tensor(rows, device="cuda")])
    rm, rs = row_max.cpu().numpy(), row_sum.cpu().numpy()
    for i, n in enumerate(rows):
        _, m, Z, _ = oracle.softmax(lb[i], T)
        assert rm[n] == m and abs(rs[n] - Z) <= 1e-5 * Z


@pytest.mark.parametrize("dtype,V", [(torch.bfloat16, 32000), (torch.float32, 4099), (torch.bfloat16, 13)])
def test_precomputed_row_statistics_feed_the_verification(ears, oracle, dtype, V):
    """ears_row_stats on the draft and the target logits separately (as a pipeline would run it
    after each model), imported, then DECIDE | SAMPLE: identical to the one-call path."""
    from paper_2512_13194_amd import inputs
    _log("row_stats -> import -> verify %s V=%d" % (dtype, V))
    B, K, T, beta, seed = 10, 4, 0.7, 0.4, 5
    batch = inputs.make_rect(B, K, V, dtype, T=T, data_seed=95, draft_noise=1.0, device="cuda")
    dm, dz = ears.ears_row_stats(batch.draft, temperature=T)
    tm, tz = ears.ears_row_stats(batch.target, temperature=T)
    torch.cuda.synchronize()
    tb = inputs.logits_to_numpy(batch.target).reshape(B * (K + 1), V)
    for n in (0, 7, B * (K + 1) - 1):
        _, m, Z, _ = oracle.softmax(tb[n], float(np.float32(T)))
        assert tm.view(-1)[n].item() == m and abs(tz.view(-1)[n].item() - Z) <= 1e-5 * Z
    ws = torch.empty(ears.ears_workspace_bytes(B * K, B, V), dtype=torch.uint8, device="cuda")
    ears.ears_import_stats(batch.target, batch.draft, batch.tokens, tm.view(-1), tz.view(-1),
                           dm.view(-1), dz.view(-1), ws)
    out = ears.ears_verify_ex(batch.target, batch.draft, batch.tokens, temperature=T, beta=beta, seed=seed,
                              workspace=ws, stages=ears.EARS_STAGE_DECIDE | ears.EARS_STAGE_SAMPLE,
                              want_stats=True, want_path=True)
    full = ears.ears_verify_ex(batch.target, batch.draft, batch.tokens, temperature=T, beta=beta, seed=seed,
                               want_stats=True, want_path=True)
    torch.cuda.synchronize()
    assert torch.equal(out["accept_len"], full["accept_len"]) and torch.equal(out["tokens"], full["tokens"])
    assert torch.equal(out["stats"], full["stats"]) and torch.equal(out["path"], full["path"])
    ora = oracle.verify(inputs.logits_to_numpy(batch.target), inputs.logits_to_numpy(batch.draft),
                        batch.tokens.cpu().numpy(), float(np.float32(T)), float(np.float32(beta)), seed,
                        nthreads=NTHREADS)
    rep = compare(ora, out["accept_len"].cpu().numpy(), out["tokens"].cpu().numpy(),
                  out["stats"].cpu().numpy(), out["path"].cpu().numpy(), None, K,
                  1e-5 if dtype == torch.float32 else 2e-3, batch.tokens.cpu().numpy(), V)
    assert rep.exempt_decisions == 0 and rep.exempt_tokens == 0


def test_entropy_measure_from_producer_side_statistics(ears, oracle):
    """Entropy of the emitted rows from the projection's epilogue and from ears_row_stats, against
    the oracle; imported, the DECIDE stage with the entropy measure gives the oracle's decisions."""
    _log("entropy through lm_head / row_stats / import")
    B, K, V, D, T, beta, seed = 10, 3, 3000, 128, 0.8, 0.6, 23
    ht, wt = _operands(B * (K + 1), D, V, seed=31)
    g = torch.Generator(device="cuda").manual_seed(32)
    wd = (wt.float() + 0.08 * torch.randn(V, D, generator=g, device="cuda")).to(torch.bfloat16)
    hd = ht.view(B, K + 1, D)[:, :K].reshape(B * K, D).contiguous()
    th = torch.empty(B * (K + 1), dtype=torch.float64, device="cuda")
    tl, tm, tz = ears.ears_lm_head_bf16(ht, wt, temperature=T, out_row_entropy=th)
    dl, dm, dz = ears.ears_lm_head_bf16(hd, wd, temperature=T)
    th2 = torch.empty_like(th)
    tm2, tz2 = ears.ears_row_stats(tl, temperature=T, out_row_entropy=th2)
    torch.cuda.synchronize()
    bits = _bits(tl)
    for n in range(B * (K + 1)):
        p, m, Z, _ = oracle.softmax(bits[n], float(np.float32(T)))
        H = oracle.entropy(p)
        assert abs(th[n].item() - H) <= 2e-6 and abs(th2[n].item() - H) <= 2e-6, (n, th[n].item(), th2[n].item(), H)
    assert torch.equal(tm, tm2)
    target, draft = tl.view(B, K + 1, V), dl.view(B, K, V)
    tokens = torch.multinomial(torch.softmax(draft.float().view(B * K, V) / T, -1), 1,
                               generator=g).view(B, K).to(torch.int32)
    ws = torch.empty(ears.ears_workspace_bytes(B * K, B, V), dtype=torch.uint8, device="cuda")
    ears.ears_import_stats(target, draft, tokens, tm, tz, dm, dz, ws, target_row_entropy=th)
    out = ears.ears_verify_ex(target, draft, tokens, temperature=T, beta=beta, seed=seed, workspace=ws,
                              uncertainty=ears.EARS_UNCERTAINTY_ENTROPY,
                              stages=ears.EARS_STAGE_DECIDE | ears.EARS_STAGE_SAMPLE,
                              want_stats=True, want_path=True)
    torch.cuda.synchronize()
    ora = oracle.verify(_bits(target), _bits(draft), tokens.cpu().numpy(), float(np.float32(T)),
                        float(np.float32(beta)), seed, nthreads=NTHREADS, uncertainty=oracle.UNC_ENTROPY)
    rep = compare(ora, out["accept_len"].cpu().numpy(), out["tokens"].cpu().numpy(),
                  out["stats"].cpu().numpy(), out["path"].cpu().numpy(), None, K, 2e-3,
                  tokens.cpu().numpy(), V, unc_is_maxprob=False)
    assert rep.exempt_decisions == 0 and rep.exempt_tokens == 0
    assert (ora.path == 2).any()                  # the tolerance did decide some positions
