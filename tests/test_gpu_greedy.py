"""The temperature -> 0 entry point on the GPU against the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ears():
    import paper_2512_13194_amd as p
    p.lib()
    assert torch.cuda.is_available()
    return p


def _log(msg):
    print(msg, flush=True)


def _plant_prefixes(target, tokens, gen):
    """Draft tokens that agree with the target arg-max on a random prefix of every sequence."""
    B, K = tokens.shape
    top = target[:, :K].float().argmax(-1).to(torch.int32)
    keep = torch.rand(B, K, generator=gen, device=target.device) < 0.8
    return torch.where(keep, top, tokens)


def _check_rect(ears, oracle, target, tokens):
    from paper_2512_13194_amd import inputs
    acc, out = ears.ears_verify_greedy(target, tokens)
    torch.cuda.synchronize()
    o_acc, o_out, _ = oracle.verify_greedy(inputs.logits_to_numpy(target), tokens.cpu().numpy())
    assert np.array_equal(acc.cpu().numpy(), o_acc)
    assert np.array_equal(out.cpu().numpy(), o_out)
    return o_acc


@pytest.mark.parametrize("B,K,V,dtype", [
    (1, 1, 1, torch.float32), (3, 2, 8, torch.float32), (5, 3, 13, torch.bfloat16),
    (4, 1, 1003, torch.bfloat16), (2, 4, 4099, torch.float32), (7, 8, 8192, torch.bfloat16),
    (3, 2, 8200, torch.bfloat16), (2, 3, 65537, torch.bfloat16), (33, 5, 2048, torch.float32),
    (300, 2, 520, torch.bfloat16), (64, 5, 32000, torch.bfloat16), (2000, 1, 50, torch.float32),
    (3, 70, 300, torch.bfloat16), (2, 130, 64, torch.float32), (2, 2, 300001, torch.bfloat16),
])
def test_greedy_shapes(ears, oracle, B, K, V, dtype):
    from paper_2512_13194_amd import inputs
    _log("greedy B=%d K=%d V=%d %s" % (B, K, V, dtype))
    batch = inputs.make_rect(B, K, V, dtype, T=1.0, data_seed=B * 1000 + V + 2, device="cuda")
    gen = torch.Generator(device="cuda").manual_seed(V)
    tokens = _plant_prefixes(batch.target, batch.tokens, gen)
    acc = _check_rect(ears, oracle, batch.target, tokens)
    if B * K >= 64:
        assert 0 < acc.sum() < B * K      # both outcomes occur


def test_greedy_target_buffer_larger_than_4_gib(ears, oracle):
    """B = 2500, K = 8, V = 128256, bf16: 5.8 GB of target logits (22500 rows)."""
    from paper_2512_13194_amd import inputs
    _log("greedy target buffer > 4 GiB")
    g = torch.Generator(device="cuda").manual_seed(94)
    B, K, V = 2500, 8, 128256
    target = torch.empty(B, K + 1, V, dtype=torch.bfloat16, device="cuda")
    for b0 in range(0, B, 250):   # generated in slices: no fp32 copy of the whole buffer
        target[b0:b0 + 250] = (torch.randn(250, K + 1, V, generator=g, device="cuda") * 2.0).to(torch.bfloat16)
    assert target.numel() * 2 > 2 ** 32
    tokens = torch.randint(0, V, (B, K), generator=g, device="cuda", dtype=torch.int32)
    tokens = _plant_prefixes(target, tokens, g)
    acc = _check_rect(ears, oracle, target, tokens)
    assert 0 < acc.sum() < B * K


def test_greedy_ragged_with_sequences_without_draft_tokens(ears, oracle):
    from paper_2512_13194_amd import inputs
    _log("greedy ragged with empty sequences")
    batch = inputs.make_ragged(50, 2500, torch.bfloat16, data_seed=88, K_lo=0, K_hi=2, device="cuda")
    off = batch.row_offsets.cpu().numpy()
    assert (np.diff(off) == 0).sum() > 8
    tokens = batch.tokens.clone()
    top = batch.target.float().argmax(-1).to(torch.int32)
    for b in range(50):
        r0, r1 = int(off[b]), int(off[b + 1])
        if r1 > r0 and b % 2 == 0:
            tokens[r0:r1] = top[r0 + b:r1 + b]
    acc, out = ears.ears_verify_greedy(batch.target, tokens, row_offsets=batch.row_offsets)
    torch.cuda.synchronize()
    o_acc, o_out, _ = oracle.verify_greedy(inputs.logits_to_numpy(batch.target), tokens.cpu().numpy(), off)
    assert np.array_equal(acc.cpu().numpy(), o_acc) and np.array_equal(out.cpu().numpy(), o_out)
    assert (o_acc[np.diff(off) == 0] == 0).all()


def test_greedy_ties_masked_rows_and_bad_tokens(ears, oracle):
    _log("greedy ties / masked")
    V, B, K = 5000, 6, 3
    gen = torch.Generator(device="cuda").manual_seed(3)
    # bf16 values drawn from a handful of levels: every row has many equal maxima
    levels = torch.tensor([-2.0, -1.0, 0.0, 0.5, 1.0], device="cuda")
    target = levels[torch.randint(0, 5, (B, K + 1, V), generator=gen, device="cuda")].to(torch.bfloat16)
    target[0, 0, :] = float("-inf")                 # a row with no finite entry: arg-max is index 0
    target[1, 1, :] = float("-inf")
    target[1, 1, 4321] = -3.0                       # a single finite entry
    target[2, 0, :] = 1.0                           # all equal
    tokens = target[:, :K].float().argmax(-1).to(torch.int32)
    tokens[3, 1] = -5                               # out of range: never matches
    tokens[4, 2] = V
    acc = _check_rect(ears, oracle, target, tokens)
    assert acc.tolist() == [3, 3, 3, 1, 2, 3]
    # the same with an unaligned row length and fp32
    target32 = target.float()[:, :, :4999].contiguous()
    tokens32 = target32[:, :K].argmax(-1).to(torch.int32)
    _check_rect(ears, oracle, target32, tokens32)


def test_greedy_ragged_and_caller_workspace(ears, oracle):
    from paper_2512_13194_amd import inputs
    _log("greedy ragged")
    batch = inputs.make_ragged(37, 3001, torch.bfloat16, data_seed=84, device="cuda")
    off = batch.row_offsets.cpu().numpy()
    R, B = batch.total_draft_rows, off.shape[0] - 1
    tokens = batch.tokens.clone()
    top = batch.target.float().argmax(-1).to(torch.int32)
    gen = torch.Generator(device="cuda").manual_seed(5)
    keep = torch.rand(R, generator=gen, device="cuda") < 0.8
    for b in range(B):                               # target row of draft row r is r + b
        r0, r1 = int(off[b]), int(off[b + 1])
        tokens[r0:r1] = torch.where(keep[r0:r1], top[r0 + b:r1 + b], tokens[r0:r1])
    ws = torch.empty(ears.ears_greedy_workspace_bytes(R, B), dtype=torch.uint8, device="cuda")
    acc, out = ears.ears_verify_greedy(batch.target, tokens, row_offsets=batch.row_offsets, workspace=ws)
    torch.cuda.synchronize()
    o_acc, o_out, o_amax = oracle.verify_greedy(inputs.logits_to_numpy(batch.target),
                                                tokens.cpu().numpy(), off)
    assert np.array_equal(acc.cpu().numpy(), o_acc) and np.array_equal(out.cpu().numpy(), o_out)
    # the scratch holds the arg-max of every target row
    assert np.array_equal(ws.view(torch.int32)[:R + B].cpu().numpy(), o_amax)
    acc2, out2 = ears.ears_verify_greedy(batch.target, tokens, row_offsets=batch.row_offsets)
    torch.cuda.synchronize()
    assert torch.equal(acc, acc2) and torch.equal(out, out2)


def test_greedy_headline_shape_and_small_temperature_limit(ears, oracle):
    """Full headline shape against the oracle; and the stochastic entry point at a small temperature
    takes the same decisions when the draft proposes its own arg-max (the limit the corner is)."""
    from paper_2512_13194_amd import inputs
    _log("greedy headline shape")
    batch = inputs.make_config(2, device="cuda")
    gen = torch.Generator(device="cuda").manual_seed(11)
    tokens = _plant_prefixes(batch.target, batch.tokens, gen)
    acc = _check_rect(ears, oracle, batch.target, tokens)
    assert 0 < acc.sum() < batch.B * batch.K
    del batch
    torch.cuda.empty_cache()

    _log("greedy limit")
    # logits are permutations of 0..V-1 and T = 0.05: gaps of 20 nats, |l|/T below 1000
    B, K, V = 32, 4, 48
    g = torch.Generator(device="cuda").manual_seed(12)
    target = torch.stack([torch.randperm(V, generator=g, device="cuda") for _ in range(B * (K + 1))])
    target = target.view(B, K + 1, V).float()
    draft = torch.stack([torch.randperm(V, generator=g, device="cuda") for _ in range(B * K)])
    draft = draft.view(B, K, V).float()
    agree = torch.rand(B, K, generator=g, device="cuda") < 0.7
    draft = torch.where(agree[:, :, None], target[:, :K], draft).contiguous()
    tokens = draft.argmax(-1).to(torch.int32)
    acc, out = ears.ears_verify_greedy(target, tokens)
    a2, o2 = ears.ears_verify_f32(target, draft, tokens, 0.05, 0.5, 99)
    torch.cuda.synchronize()
    assert torch.equal(acc, a2) and torch.equal(out, o2)


def test_verifier_object_at_temperature_zero(ears, oracle):
    from paper_2512_13194_amd import inputs
    _log("greedy verifier")
    batch = inputs.make_rect(20, 4, 9000, torch.bfloat16, T=1.0, data_seed=90, device="cuda")
    gen = torch.Generator(device="cuda").manual_seed(6)
    tokens = _plant_prefixes(batch.target, batch.tokens, gen)
    ver = ears.EarsVerifier(temperature=0.0, telemetry=True)
    res = ver.verify(batch.target, None, tokens)
    torch.cuda.synchronize()
    o_acc, o_out, _ = oracle.verify_greedy(inputs.logits_to_numpy(batch.target), tokens.cpu().numpy())
    assert np.array_equal(res.accept_len.cpu().numpy(), o_acc)
    assert np.array_equal(res.tokens.cpu().numpy(), o_out)
    assert ver.summary()["mean_accept_len"] == pytest.approx(o_acc.mean())
    assert ver.step == 1
