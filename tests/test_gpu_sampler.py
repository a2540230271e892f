"""The verifier object and its telemetry on the GPU, against the CPU oracle."""
import os

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

NTHREADS = min(16, os.cpu_count() or 1)


@pytest.fixture(scope="module")
def pkg():
    import paper_2512_13194_amd as p
    p.lib()
    assert torch.cuda.is_available()
    return p


def test_multi_step_loop_with_continuous_batching(pkg, oracle):
    """Three decode steps; between steps sequences leave and the rest are compacted.  Every
    (sequence id, step) must give what the oracle gives for that id and that step's seed."""
    from paper_2512_13194_amd import inputs
    from paper_2512_13194_amd.sampler import EarsVerifier
    print("sampler: multi-step", flush=True)
    B, K, V, T, beta = 24, 4, 6000, 0.9, 0.1
    ver = EarsVerifier(temperature=T, beta=beta, seed=2024)
    ids = torch.arange(B, dtype=torch.int64, device="cuda") + 1000
    alive = torch.ones(B, dtype=torch.bool)
    for step in range(3):
        batch = inputs.make_rect(int(alive.sum()), K, V, torch.bfloat16, T=T, data_seed=300 + step,
                                 draft_noise=1.0, device="cuda")
        cur = ids[alive.cuda()]
        res = ver.verify(batch.target, batch.draft, batch.tokens, seq_ids=cur)
        torch.cuda.synchronize()
        ora = oracle.verify(inputs.logits_to_numpy(batch.target), inputs.logits_to_numpy(batch.draft),
                            batch.tokens.cpu().numpy(), float(np.float32(T)), float(np.float32(beta)),
                            ver.step_seed(step), seq_ids=cur.cpu().numpy(), nthreads=NTHREADS)
        assert np.array_equal(res.accept_len.cpu().numpy(), ora.accept_len)
        assert np.array_equal(res.tokens.cpu().numpy(), ora.tokens)
        # sequences that accepted nothing "finish" and leave the batch
        keep = torch.from_numpy(ora.accept_len > 0)
        idx = torch.nonzero(alive)[:, 0]
        alive[idx[~keep]] = False
        if alive.sum() == 0:
            break
    assert ver.step == step + 1


def test_telemetry_matches_oracle_and_trade_off_direction(pkg, oracle):
    """Branch counts equal the oracle's; a larger beta pardons more and accepts longer prefixes
    (Section 4.3), and beta = 0 never pardons."""
    from paper_2512_13194_amd import inputs
    from paper_2512_13194_amd.sampler import EarsVerifier, acceptance_sweep
    print("sampler: telemetry", flush=True)
    T = 0.9
    batch = inputs.make_rect(64, 5, 32000, torch.bfloat16, T=T, data_seed=41, draft_noise=1.0,
                             device="cuda")
    betas = [0.0, 0.05, 0.1, 0.2, 0.5]
    rows = acceptance_sweep(batch, betas, T, seed=9)
    ver = EarsVerifier(temperature=T, beta=0.0, seed=9)
    tgt, drf = inputs.logits_to_numpy(batch.target), inputs.logits_to_numpy(batch.draft)
    tok = batch.tokens.cpu().numpy()
    for beta, row in zip(betas, rows):
        ora = oracle.verify(tgt, drf, tok, float(np.float32(T)), float(np.float32(beta)),
                            ver.step_seed(0), nthreads=NTHREADS)
        n = ora.path.size
        assert row["primary_rate"] == pytest.approx((ora.path == 1).sum() / n, abs=1.5 / n)
        assert row["pardon_rate"] == pytest.approx((ora.path == 2).sum() / n, abs=1.5 / n)
        assert row["mean_accept_len"] == pytest.approx(ora.accept_len.mean(), abs=1.5 / 64)
    assert rows[0]["pardon_rate"] == 0.0
    assert all(a["pardon_rate"] <= b["pardon_rate"] for a, b in zip(rows, rows[1:]))
    assert all(a["mean_accept_len"] <= b["mean_accept_len"] for a, b in zip(rows, rows[1:]))
    assert rows[-1]["mean_accept_len"] > rows[0]["mean_accept_len"]
    # the primary path is the traditional rule: its rate does not depend on beta
    assert all(r["primary_rate"] == rows[0]["primary_rate"] for r in rows)


def test_uncertainty_rises_with_temperature(pkg):
    """Higher temperature flattens P_t, lowers max P_t and so raises the tolerance (Section 4.3)."""
    from paper_2512_13194_amd import inputs
    from paper_2512_13194_amd.sampler import EarsVerifier
    print("sampler: temperature", flush=True)
    batch = inputs.make_rect(32, 4, 20000, torch.float32, T=1.0, data_seed=42, device="cuda")
    means = []
    for T in (0.5, 0.8, 1.0, 1.5):
        res = EarsVerifier(temperature=T, beta=0.1, seed=1).verify(
            batch.target, batch.draft, batch.tokens, want_stats=True)
        torch.cuda.synchronize()
        means.append(res.stats[:, 6].mean().item())
    assert all(a < b for a, b in zip(means, means[1:]))


@pytest.mark.parametrize("measure", ["entropy", "variance"])
def test_alternative_measures_through_the_verifier(pkg, oracle, measure):
    """The verifier's entropy / variance option gives the oracle's decisions and tokens for that
    tolerance, its telemetry counts the oracle's branches, and it rises with temperature too."""
    from paper_2512_13194_amd import inputs
    from paper_2512_13194_amd.sampler import EarsVerifier, acceptance_sweep
    print("sampler: %s measure" % measure, flush=True)
    ora_measure = {"entropy": oracle.UNC_ENTROPY, "variance": oracle.UNC_VARIANCE}[measure]
    T, beta = 0.9, 0.3
    batch = inputs.make_rect(48, 5, 32000, torch.bfloat16, T=T, data_seed=43, draft_noise=1.0,
                             device="cuda")
    ver = EarsVerifier(temperature=T, beta=beta, seed=5, telemetry=True, uncertainty=measure)
    res = ver.verify(batch.target, batch.draft, batch.tokens)
    torch.cuda.synchronize()
    ora = oracle.verify(inputs.logits_to_numpy(batch.target), inputs.logits_to_numpy(batch.draft),
                        batch.tokens.cpu().numpy(), float(np.float32(T)), float(np.float32(beta)),
                        ver.step_seed(0), nthreads=NTHREADS, uncertainty=ora_measure)
    assert np.array_equal(res.accept_len.cpu().numpy(), ora.accept_len)
    assert np.array_equal(res.tokens.cpu().numpy(), ora.tokens)
    assert np.array_equal(res.path.cpu().numpy().reshape(ora.path.shape), ora.path)
    assert ver.counts["pardon"] == int((ora.path == 2).sum())
    rows = acceptance_sweep(batch, [0.0, 0.2, 0.6], T, seed=5, uncertainty=measure)
    assert rows[0]["pardon_rate"] == 0.0
    assert rows[0]["mean_accept_len"] <= rows[1]["mean_accept_len"] <= rows[2]["mean_accept_len"]
    means = []
    for temp in (0.5, 1.0, 1.5):
        r = EarsVerifier(temperature=temp, beta=0.1, seed=1, uncertainty=measure).verify(
            batch.target, batch.draft, batch.tokens, want_stats=True)
        torch.cuda.synchronize()
        means.append(r.stats[:, 6].mean().item())
    assert means[0] < means[1] < means[2]
    with pytest.raises(ValueError):
        EarsVerifier(uncertainty="kurtosis")
