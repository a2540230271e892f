"""A verification call captured in a HIP graph (through torch.cuda.CUDAGraph) and replayed: the
library launches kernels only (no allocation, no memset, no synchronisation) once its buffers
exist, so a serving loop can replay it.  The seed is a by-value argument and is frozen in the
graph; fresh noise per step comes from the device-side `seq_ids` buffer."""
import os
import time

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

NTHREADS = min(16, os.cpu_count() or 1)


@pytest.mark.parametrize("B,K,V", [
    (64, 5, 32000),    # two launches: statistics, then sampling
    (72, 8, 64000),    # long rows, 576 positions: the whole call is one launch
])
def test_captured_call_replays_like_eager_and_like_the_oracle(oracle, B, K, V):
    import paper_2512_13194_amd as ears
    from paper_2512_13194_amd import inputs
    ears.lib()
    print("graph capture B=%d K=%d V=%d" % (B, K, V), flush=True)
    T, beta, seed = 0.8, 0.5, 77
    batch = inputs.make_rect(B, K, V, torch.bfloat16, T=T, data_seed=1001, draft_noise=0.5, device="cuda")
    ids = torch.arange(B, dtype=torch.int64, device="cuda")
    ws = torch.empty(ears.ears_workspace_bytes(B * K, B, V), dtype=torch.uint8, device="cuda")
    acc = torch.empty(B, dtype=torch.int32, device="cuda")
    tok = torch.empty(B * (K + 1), dtype=torch.int32, device="cuda")

    def call():
        ears.ears_verify_ex(batch.target, batch.draft, batch.tokens, temperature=T, beta=beta, seed=seed,
                            seq_ids=ids, workspace=ws, out_accept_len=acc, out_tokens=tok)

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        call()                                   # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        call()
    torch.cuda.synchronize()

    tgt, drf = inputs.logits_to_numpy(batch.target), inputs.logits_to_numpy(batch.draft)
    for step in range(4):
        # eager work and synchronisations between replays; new noise through the ids, new tokens
        ids.copy_(torch.arange(B, dtype=torch.int64, device="cuda") + (step << 40))
        if step == 2:
            batch.tokens.copy_(torch.roll(batch.tokens, 1, dims=0))
        torch.cuda.synchronize()
        acc.fill_(-7)
        tok.fill_(-7)
        graph.replay()
        torch.cuda.synchronize()
        g_acc, g_tok = acc.clone(), tok.clone()
        call()                                   # the same call eagerly
        torch.cuda.synchronize()
        assert torch.equal(g_acc, acc) and torch.equal(g_tok, tok), step
        ora = oracle.verify(tgt, drf, batch.tokens.cpu().numpy(), float(np.float32(T)),
                            float(np.float32(beta)), seed, seq_ids=ids.cpu().numpy(), nthreads=NTHREADS)
        assert np.array_equal(g_acc.cpu().numpy(), ora.accept_len), step
        assert np.array_equal(g_tok.view(B, K + 1).cpu().numpy(), ora.tokens), step

    # what the graph buys on a launch-bound shape
    def timed(fn, n=200):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n * 1e6
    print("  eager %.1f us/call, graph replay %.1f us/call" % (timed(call), timed(graph.replay)), flush=True)


def test_producer_side_pipeline_and_greedy_call_in_one_graph(oracle):
    """The projection with its statistics, the draft rows' statistics, their import, DECIDE | SAMPLE
    and a greedy verification, captured together and replayed on new hidden states: every replay
    equals the same calls made eagerly, and the eager result equals the oracle on the emitted logits."""
    import paper_2512_13194_amd as ears
    from paper_2512_13194_amd import inputs
    ears.lib()
    print("graph capture: producer-side pipeline", flush=True)
    B, K, D, V, T, beta, seed = 16, 3, 128, 8192, 0.9, 0.4, 31
    N = B * (K + 1)
    g = torch.Generator(device="cuda").manual_seed(3)
    hidden = torch.randn(N, D, generator=g, device="cuda").to(torch.bfloat16)
    weight = (torch.randn(V, D, generator=g, device="cuda") * (2.5 / D ** 0.5)).to(torch.bfloat16)
    draft = (torch.randn(B, K, V, generator=g, device="cuda") * 2.0).to(torch.bfloat16)
    tokens = torch.randint(0, V, (B, K), generator=g, device="cuda", dtype=torch.int32)
    logits = torch.empty(N, V, dtype=torch.bfloat16, device="cuda")
    tm = torch.empty(N, dtype=torch.float32, device="cuda")
    tz = torch.empty(N, dtype=torch.float64, device="cuda")
    dm = torch.empty(B * K, dtype=torch.float32, device="cuda")
    dz = torch.empty(B * K, dtype=torch.float64, device="cuda")
    lm_ws = torch.empty(ears.ears_lm_head_workspace_bytes(N, V), dtype=torch.uint8, device="cuda")
    ws = torch.empty(ears.ears_workspace_bytes(B * K, B, V), dtype=torch.uint8, device="cuda")
    gws = torch.empty(ears.ears_greedy_workspace_bytes(B * K, B), dtype=torch.uint8, device="cuda")
    acc = torch.empty(B, dtype=torch.int32, device="cuda")
    tok = torch.empty(N, dtype=torch.int32, device="cuda")
    gacc = torch.empty(B, dtype=torch.int32, device="cuda")
    gtok = torch.empty(N, dtype=torch.int32, device="cuda")

    def call():
        ears.ears_lm_head_bf16(hidden, weight, temperature=T, out_logits=logits, out_row_max=tm,
                               out_row_sumexp=tz, workspace=lm_ws)
        ears.ears_row_stats(draft, temperature=T, out_row_max=dm, out_row_sumexp=dz)
        target = logits.view(B, K + 1, V)
        ears.ears_import_stats(target, draft, tokens, tm, tz, dm, dz, ws)
        ears.ears_verify_ex(target, draft, tokens, temperature=T, beta=beta, seed=seed, workspace=ws,
                            stages=ears.EARS_STAGE_DECIDE | ears.EARS_STAGE_SAMPLE,
                            out_accept_len=acc, out_tokens=tok)
        ears.ears_verify_greedy(target, tokens, workspace=gws, out_accept_len=gacc, out_tokens=gtok)

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        call()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        call()
    torch.cuda.synchronize()
    for step in range(3):
        hidden.copy_(torch.randn(N, D, generator=g, device="cuda").to(torch.bfloat16))
        torch.cuda.synchronize()
        for t in (acc, tok, gacc, gtok):
            t.fill_(-7)
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (acc, tok, gacc, gtok, logits)]
        call()
        torch.cuda.synchronize()
        for a, b in zip(got, (acc, tok, gacc, gtok, logits)):
            assert torch.equal(a, b), step
        lb = inputs.logits_to_numpy(logits.view(B, K + 1, V))
        ora = oracle.verify(lb, inputs.logits_to_numpy(draft), tokens.cpu().numpy(), float(np.float32(T)),
                            float(np.float32(beta)), seed, nthreads=NTHREADS)
        assert np.array_equal(got[0].cpu().numpy(), ora.accept_len), step
        assert np.array_equal(got[1].view(B, K + 1).cpu().numpy(), ora.tokens), step
        o_acc, o_out, _ = oracle.verify_greedy(lb, tokens.cpu().numpy())
        assert np.array_equal(got[2].cpu().numpy(), o_acc) and np.array_equal(got[3].view(B, K + 1).cpu().numpy(), o_out)
