"""Pins of the oracle's vocabulary projection and bf16 rounding (no GPU): numpy's fp64 matrix
product, torch's own float -> bfloat16 conversion, and hand-worked roundings."""
import numpy as np
import torch


def _bits(a):
    return torch.as_tensor(a, dtype=torch.float32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def _val(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def test_round_bf16_hand_worked(oracle):
    r = oracle.round_bf16
    assert r(1.0) == 0x3F80 and r(-2.0) == 0xC000 and r(0.0) == 0 and r(-0.0) == 0x8000
    assert r(1.0 + 2 ** -8) == 0x3F80            # tie between 1 and 1 + 2^-7: even fraction wins
    assert r(1.0 + 3 * 2 ** -8) == 0x3F82        # tie between 1 + 2^-7 and 1 + 2^-6: even wins
    assert r(1.0 + 2 ** -8 + 2 ** -30) == 0x3F81  # just above the tie
    assert r(1.99999) == 0x4000                  # rounds up into the next binade
    assert r(3.3895313892515355e38) == 0x7F7F    # largest finite bf16
    assert r(2.0 ** -133) == 0x0001 and r(2.0 ** -126) == 0x0080


def test_round_bf16_against_torch(oracle):
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.normal(size=4000) * 10.0 ** rng.integers(-6, 6, size=4000),
                        (1.0 + np.arange(-4, 5) * 2.0 ** -9) * 3.0]).astype(np.float32)
    want = _bits(x)
    got = np.array([oracle.round_bf16(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)


def test_projection_against_numpy_matmul(oracle):
    rng = np.random.default_rng(1)
    N, D, V = 7, 96, 53
    h = _bits(rng.normal(size=(N, D)))
    w = _bits(rng.normal(size=(V, D)) * 0.3)
    exact, logits = oracle.lm_head(h, w, nthreads=2)
    ref = _val(h) @ _val(w).T                     # fp64 products of bf16 values are exact; sums differ by order
    assert np.allclose(exact, ref, rtol=0, atol=1e-12)
    assert exact[3, 11] == oracle.lm_head_dot(h, w, 3, 11)
    # transposed operands or a swapped index would fail here
    assert abs(exact[2, 5] - float(_val(h)[2] @ _val(w)[5])) < 1e-12
    assert abs(exact[2, 5] - float(_val(h)[5 % N] @ _val(w)[2])) > 1e-6
    # rounding of the sums: torch's conversion of the fp32-representable cases
    want = _bits(ref.astype(np.float32))
    same = ref.astype(np.float32).astype(np.float64) == ref
    near = np.abs(_val(logits) - ref) <= np.abs(ref) * 2.0 ** -8 + 1e-300
    assert near.all()
    assert np.array_equal(logits[same], want[same])
    assert (logits != want).mean() < 1e-3          # double rounding through fp32 differs almost never
