"""The entry point that allocates nothing (fixed device scratch inside the library), through the C
ABI, against ears_verify_ex with a caller-owned workspace: identical outputs, on two calls in a row
of which the second is smaller, then a ragged batch, then the size limit."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ears():
    import paper_2512_13194_amd as pkg
    pkg.lib()           # raises if libears.so has not been built: there is no fallback
    assert torch.cuda.is_available()
    return pkg


def _both(ears, batch, T, beta, seed, uncertainty=0, ragged=False):
    dev = batch.target.device
    R, B = batch.total_draft_rows, batch.B
    kw = dict(seed=seed, uncertainty=uncertainty)
    if ragged:
        kw.update(row_offsets=batch.row_offsets, temperature_per_seq=batch.temperature,
                  beta_per_seq=batch.beta)
    else:
        kw.update(temperature=T, beta=beta)
    ref = ears.ears_verify_ex(batch.target, batch.draft, batch.tokens, want_stats=True, want_path=True, **kw)
    acc = torch.full((B,), -7, dtype=torch.int32, device=dev)
    tok = torch.full((R + B,), -7, dtype=torch.int32, device=dev)
    stats = torch.zeros(R, ears.EARS_NSTATS, dtype=torch.float64, device=dev)
    path = torch.full((R,), -7, dtype=torch.int32, device=dev)
    before = torch.cuda.memory_allocated()
    ears.ears_verify_noalloc(batch.target, batch.draft, batch.tokens, acc, tok, out_stats=stats,
                             out_path=path, **kw)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(acc, ref["accept_len"]) and torch.equal(tok, ref["tokens"])
    assert torch.equal(path, ref["path"]) and torch.equal(stats, ref["stats"])
    return acc, tok


def test_no_alloc_matches_workspace_entry_point(ears):
    from paper_2512_13194_amd import inputs
    print("no-alloc: B=96 K=6 V=65536, then B=5 K=2 V=1003, then ragged", flush=True)
    # long rows, 576 draft positions: this call is a single launch, the small one after it two
    big = inputs.make_rect(96, 6, 65536, torch.bfloat16, T=0.9, data_seed=501, draft_noise=1.0, device="cuda")
    small = inputs.make_rect(5, 2, 1003, torch.float32, T=1.1, data_seed=502, device="cuda")
    acc_big, _ = _both(ears, big, 0.9, 0.3, 41)
    acc_small, _ = _both(ears, small, 1.1, 0.6, 42, uncertainty=ears.EARS_UNCERTAINTY_ENTROPY)
    assert 0 < int((acc_big < 6).sum()) and acc_small.numel() == 5
    # the larger problem again: nothing of the smaller call is left behind
    _both(ears, big, 0.9, 0.3, 43)
    rag = inputs.make_ragged(33, 4099, torch.bfloat16, data_seed=503, K_lo=0, K_hi=5, device="cuda")
    _both(ears, rag, None, None, 44, ragged=True)


def test_no_alloc_rejects_what_does_not_fit(ears):
    from paper_2512_13194_amd import binding
    # B = 4096 sequences of K = 64: the statistics alone need more than the fixed scratch
    B, K, V = 4096, 64, 8
    assert ears.ears_workspace_bytes(B * K, B, V) > ears.EARS_NOALLOC_SCRATCH_BYTES
    t = torch.zeros(B, K + 1, V, dtype=torch.float32, device="cuda")
    d = torch.zeros(B, K, V, dtype=torch.float32, device="cuda")
    x = torch.zeros(B, K, dtype=torch.int32, device="cuda")
    acc = torch.empty(B, dtype=torch.int32, device="cuda")
    tok = torch.empty(B * (K + 1), dtype=torch.int32, device="cuda")
    with pytest.raises(ears.EarsError) as e:
        ears.ears_verify_noalloc(t, d, x, acc, tok, temperature=1.0, beta=0.1)
    assert e.value.status == binding.EARS_ERR_WORKSPACE
