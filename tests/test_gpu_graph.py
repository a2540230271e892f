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


def test_captured_call_replays_like_eager_and_like_the_oracle(oracle):
    import paper_2512_13194_amd as ears
    from paper_2512_13194_amd import inputs
    ears.lib()
    print("graph capture", flush=True)
    B, K, V, T, beta, seed = 64, 5, 32000, 0.8, 0.5, 77
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
