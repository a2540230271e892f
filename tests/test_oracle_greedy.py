"""Pins of the oracle's temperature -> 0 corner (no GPU).

What fixes it from outside: numpy's arg-max (first occurrence of the maximum), a hand-worked
batch, and the stochastic oracle itself run at a very small temperature, whose decisions and
tokens must converge to the greedy ones (the limit the corner is defined as).
"""
import numpy as np
import pytest


def _bf16_bits(a):
    return (np.ascontiguousarray(a, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


def test_hand_worked_batch(oracle):
    # V = 4, K = 3.  Target arg-max per row: seq 0 -> 2,0,3,1 ; seq 1 -> 1,1,0,2
    t = np.array([[[0, 1, 5, 2], [9, 1, 5, 2], [0, 1, 5, 7], [0, 8, 5, 2]],
                  [[0, 3, 1, 2], [0, 3, 1, 2], [4, 3, 1, 2], [0, 3, 6, 2]]], dtype=np.float32)
    tok = np.array([[2, 0, 1], [1, 1, 0]], dtype=np.int32)
    acc, out, amax = oracle.verify_greedy(t, tok)
    assert amax.tolist() == [[2, 0, 3, 1], [1, 1, 0, 2]]
    assert acc.tolist() == [2, 3]
    assert out.tolist() == [[2, 0, 3, -1], [1, 1, 0, 2]]
    # first token wrong: nothing accepted, the replacement is the first row's arg-max
    acc, out, _ = oracle.verify_greedy(t, np.array([[3, 0, 3], [0, 1, 0]], dtype=np.int32))
    assert acc.tolist() == [0, 0]
    assert out.tolist() == [[2, -1, -1, -1], [1, -1, -1, -1]]


def test_ties_take_the_lowest_index_and_masked_entries(oracle):
    t = np.full((1, 2, 6), -np.inf, dtype=np.float32)
    t[0, 0, [4, 2, 5]] = 1.5          # three equal maxima
    t[0, 1, 3] = -7.0                 # a single finite entry
    acc, out, amax = oracle.verify_greedy(t, np.array([[2]], dtype=np.int32))
    assert amax.tolist() == [[2, 3]] and acc.tolist() == [1] and out.tolist() == [[2, 3]]
    acc, out, _ = oracle.verify_greedy(t, np.array([[4]], dtype=np.int32))
    assert acc.tolist() == [0] and out.tolist() == [[2, -1]]
    # out-of-range tokens never match
    acc, _, _ = oracle.verify_greedy(t, np.array([[-1]], dtype=np.int32))
    assert acc.tolist() == [0]


@pytest.mark.parametrize("bf16", [False, True])
def test_argmax_against_numpy_and_prefix_rule(oracle, bf16):
    rng = np.random.default_rng(7)
    B, K, V = 9, 5, 777
    t = rng.normal(size=(B, K + 1, V)).astype(np.float32) * 3
    if bf16:
        bits = _bf16_bits(t)                      # many equal values after rounding
        ref = (bits.astype(np.uint32) << 16).view(np.float32)
        arg = bits
    else:
        ref, arg = t, t
    want = ref.argmax(-1).astype(np.int32)        # numpy: first occurrence of the maximum
    tok = want[:, :K].copy()
    wrong = rng.integers(0, K + 1, size=B)        # position of the first planted mismatch (K: none)
    for b in range(B):
        if wrong[b] < K:
            tok[b, wrong[b]] = (tok[b, wrong[b]] + 1) % V
            if wrong[b] + 1 < K:
                tok[b, wrong[b] + 1:] = rng.integers(0, V, size=K - wrong[b] - 1)
    acc, out, amax = oracle.verify_greedy(arg, tok)
    assert np.array_equal(amax, want)
    assert np.array_equal(acc, wrong.astype(np.int32))
    for b in range(B):
        n = acc[b]
        assert np.array_equal(out[b, :n], tok[b, :n]) and out[b, n] == want[b, n]
        assert (out[b, n + 1:] == -1).all()


def test_ragged_equals_rectangular_per_sequence(oracle):
    rng = np.random.default_rng(8)
    V, lens = 300, [1, 4, 2, 8, 3]
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    tgt = rng.normal(size=(off[-1] + len(lens), V)).astype(np.float32)
    tok = rng.integers(0, V, size=off[-1]).astype(np.int32)
    for b in range(len(lens)):                    # make most tokens match so prefixes are long
        rows = tgt[off[b] + b: off[b + 1] + b].argmax(-1)
        keep = rng.random(lens[b]) < 0.7
        tok[off[b]:off[b + 1]][keep] = rows[keep]
    acc, out, amax = oracle.verify_greedy(tgt, tok, off)
    for b, Kb in enumerate(lens):
        a1, o1, m1 = oracle.verify_greedy(tgt[off[b] + b: off[b + 1] + b + 1][None],
                                          tok[off[b]:off[b + 1]][None])
        assert acc[b] == a1[0]
        assert np.array_equal(out[off[b] + b: off[b + 1] + b + 1], o1[0])
        assert np.array_equal(amax[off[b] + b: off[b + 1] + b + 1], m1[0])


def test_stochastic_oracle_converges_to_the_corner(oracle):
    """At T = 0.02 with logit gaps of at least 1 the softmax is one-hot to within e^-50, so the
    stochastic rule (any beta, any seed) must take exactly the greedy decisions and emit the greedy
    tokens, whatever the measure of uncertainty."""
    rng = np.random.default_rng(9)
    B, K, V = 16, 4, 50
    # distinct integers per row: gaps >= 1
    t = np.stack([np.stack([rng.permutation(V) for _ in range(K + 1)]) for _ in range(B)]).astype(np.float32)
    d = np.stack([np.stack([rng.permutation(V) for _ in range(K)]) for _ in range(B)]).astype(np.float32)
    # drafts agree with the target on a random prefix, and propose their own arg-max
    for b in range(B):
        for i in range(rng.integers(0, K + 1)):
            d[b, i] = t[b, i]
    tok = d.argmax(-1).astype(np.int32)
    acc, out, _ = oracle.verify_greedy(t, tok)
    assert 0 < acc.sum() < B * K                    # both outcomes occur
    for seed, beta, unc in ((1, 0.0, oracle.UNC_MAXPROB), (2, 0.5, oracle.UNC_MAXPROB),
                            (3, 1.0, oracle.UNC_ENTROPY)):
        res = oracle.verify(t, d, tok, 0.02, beta, seed, uncertainty=unc)
        assert np.array_equal(res.accept_len, acc)
        assert np.array_equal(res.tokens, out)
