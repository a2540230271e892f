"""ctypes binding of the plain-C CPU oracle (oracle/ears_oracle.c).  TEST INFRASTRUCTURE ONLY.

Inputs are numpy arrays: fp32 logits as float32, bf16 logits as uint16 (the raw bit pattern).
Nothing here touches the GPU library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ears_oracle.c")
_LIB = os.path.join(_HERE, "libears_oracle.so")
# The mutation tests point this at a deliberately broken build to show that the pins catch it.
_LIB_OVERRIDE = os.environ.get("EARS_ORACLE_LIB")

NDIAG = 10
NSAMP = 5
DIAG_NAMES = ("m_t", "Z_t", "P_t_x", "m_d", "Z_d", "P_d_x", "unc", "R", "U", "thr")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (a second or so).  Returns the path of the shared library."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(
        os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "ears_oracle.h")))
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
             "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if _LIB_OVERRIDE:
        lib = ctypes.CDLL(_LIB_OVERRIDE)
    else:
        build()
        lib = ctypes.CDLL(_LIB)
    c = ctypes
    u32p = c.POINTER(c.c_uint32)
    lib.ears_oracle_philox4x32_10.argtypes = [u32p, u32p, u32p]
    lib.ears_oracle_philox4x32_10.restype = None
    lib.ears_oracle_philox_word.argtypes = [c.c_uint64, c.c_uint64, c.c_uint32, c.c_uint32,
                                            c.c_uint32, c.c_uint32]
    lib.ears_oracle_philox_word.restype = c.c_uint32
    for name in ("ears_oracle_accept_uniform",):
        f = getattr(lib, name)
        f.argtypes = [c.c_uint64, c.c_uint64, c.c_uint32]
        f.restype = c.c_double
    for name in ("ears_oracle_gumbel_uniform", "ears_oracle_gumbel"):
        f = getattr(lib, name)
        f.argtypes = [c.c_uint64, c.c_uint64, c.c_uint32, c.c_uint32]
        f.restype = c.c_double
    lib.ears_oracle_softmax.argtypes = [c.c_void_p, c.c_int, c.c_int, c.c_double, c.c_void_p,
                                        c.POINTER(c.c_double), c.POINTER(c.c_double)]
    lib.ears_oracle_softmax.restype = c.c_double
    lib.ears_oracle_entropy.argtypes = [c.c_void_p, c.c_int]
    lib.ears_oracle_entropy.restype = c.c_double
    lib.ears_oracle_variance.argtypes = [c.c_void_p, c.c_int]
    lib.ears_oracle_variance.restype = c.c_double
    lib.ears_oracle_top2.argtypes = [c.c_void_p, c.c_int, c.c_void_p]
    lib.ears_oracle_top2.restype = c.c_int32
    lib.ears_oracle_verify.argtypes = [
        c.c_void_p, c.c_void_p, c.c_void_p, c.c_int, c.c_int, c.c_int, c.c_int, c.c_double,
        c.c_double, c.c_int, c.c_uint64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_void_p, c.c_int]
    lib.ears_oracle_verify.restype = c.c_int
    lib.ears_oracle_verify_ragged.argtypes = [
        c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int, c.c_int, c.c_int, c.c_void_p,
        c.c_void_p, c.c_int, c.c_uint64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_void_p, c.c_int]
    lib.ears_oracle_verify_ragged.restype = c.c_int
    lib.ears_oracle_verify_greedy.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int, c.c_int,
                                              c.c_int, c.c_int, c.c_void_p, c.c_void_p, c.c_void_p]
    lib.ears_oracle_verify_greedy.restype = None
    lib.ears_oracle_lm_head_dot.argtypes = [c.c_void_p, c.c_void_p, c.c_int, c.c_int64, c.c_int64]
    lib.ears_oracle_lm_head_dot.restype = c.c_double
    lib.ears_oracle_round_bf16.argtypes = [c.c_double]
    lib.ears_oracle_round_bf16.restype = c.c_uint16
    lib.ears_oracle_lm_head.argtypes = [c.c_void_p, c.c_void_p, c.c_int, c.c_int, c.c_int,
                                        c.c_void_p, c.c_void_p, c.c_int]
    lib.ears_oracle_lm_head.restype = None
    _lib = lib
    return lib


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    raise TypeError("logits must be float32 or uint16 (bf16 bit pattern), got %s" % a.dtype)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def philox4x32_10(ctr, key):
    lib = _load()
    c = (ctypes.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (ctypes.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    o = (ctypes.c_uint32 * 4)()
    lib.ears_oracle_philox4x32_10(c, k, o)
    return tuple(int(x) for x in o)


def philox_word(seed, seq, pos, domain, blk, word) -> int:
    return int(_load().ears_oracle_philox_word(seed, seq, pos, domain, blk, word))


def accept_uniform(seed: int, seq: int, pos: int) -> float:
    return float(_load().ears_oracle_accept_uniform(seed, seq, pos))


def gumbel_uniform(seed: int, seq: int, pos: int, v: int) -> float:
    return float(_load().ears_oracle_gumbel_uniform(seed, seq, pos, v))


def gumbel(seed: int, seq: int, pos: int, v: int) -> float:
    return float(_load().ears_oracle_gumbel(seed, seq, pos, v))


def softmax(row: np.ndarray, T: float):
    """Returns (p[V] float64, m, Z, max p) of one logit row."""
    lib = _load()
    row = np.ascontiguousarray(row)
    V = row.shape[0]
    p = np.empty(V, dtype=np.float64)
    m = ctypes.c_double()
    Z = ctypes.c_double()
    pmax = lib.ears_oracle_softmax(_ptr(row), _dtype_code(row), V, float(T), _ptr(p),
                                   ctypes.byref(m), ctypes.byref(Z))
    return p, m.value, Z.value, float(pmax)


def top2(scores: np.ndarray):
    """Arg-max (lowest index on ties) and runner-up of a float64 score vector; -inf entries are not
    candidates.  Returns (winner index, samp[NSAMP]) with samp[3] unused (nan)."""
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    samp = np.full(NSAMP, np.nan)
    arg = _load().ears_oracle_top2(_ptr(scores), scores.shape[0], _ptr(samp))
    return int(arg), samp


@dataclass
class OracleResult:
    accept_len: np.ndarray  # [B] int32
    tokens: np.ndarray      # [B, K+1] int32 (ragged: packed like target rows)
    diag: np.ndarray        # [B, K, NDIAG] float64 (ragged: [rows, NDIAG])
    path: np.ndarray        # [B, K] int32 (ragged: [rows])
    samp: np.ndarray        # [B, NSAMP] float64: best, second, gap, mode, runner-up index
    status: int             # 1 if some draft token was out of range

    def d(self, name: str) -> np.ndarray:
        return self.diag[..., DIAG_NAMES.index(name)]


UNC_MAXPROB, UNC_ENTROPY, UNC_VARIANCE = 0, 1, 2


def entropy(p: np.ndarray) -> float:
    """Shannon entropy (nats) of a float64 probability vector."""
    p = np.ascontiguousarray(p, dtype=np.float64)
    return float(_load().ears_oracle_entropy(_ptr(p), p.shape[0]))


def variance(p: np.ndarray) -> float:
    """Total variance sum_v p_v (1 - p_v) of the one-hot outcome drawn from p (float64 vector)."""
    p = np.ascontiguousarray(p, dtype=np.float64)
    return float(_load().ears_oracle_variance(_ptr(p), p.shape[0]))


def verify(target: np.ndarray, draft: np.ndarray, tokens: np.ndarray, T: float, beta: float,
           seed: int, seq_ids: Optional[np.ndarray] = None, nthreads: int = 1,
           uncertainty: int = UNC_MAXPROB) -> OracleResult:
    """target [B, K+1, V], draft [B, K, V] (float32 or uint16 bf16 bits), tokens [B, K] int32."""
    lib = _load()
    target = np.ascontiguousarray(target)
    draft = np.ascontiguousarray(draft)
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    B, K1, V = target.shape
    K = K1 - 1
    assert draft.shape == (B, K, V) and tokens.shape == (B, K)
    assert _dtype_code(target) == _dtype_code(draft)
    if seq_ids is not None:
        seq_ids = np.ascontiguousarray(seq_ids, dtype=np.int64)
        assert seq_ids.shape == (B,)
    acc = np.empty(B, dtype=np.int32)
    out = np.empty((B, K + 1), dtype=np.int32)
    diag = np.empty((B, K, NDIAG), dtype=np.float64)
    path = np.empty((B, K), dtype=np.int32)
    samp = np.empty((B, NSAMP), dtype=np.float64)
    rc = lib.ears_oracle_verify(_ptr(target), _ptr(draft), _ptr(tokens), _dtype_code(target), B, K,
                                V, float(T), float(beta), int(uncertainty), int(seed), _ptr(seq_ids), _ptr(acc),
                                _ptr(out), _ptr(diag), _ptr(path), _ptr(samp), int(nthreads))
    return OracleResult(acc, out, diag, path, samp, int(rc))


def verify_ragged(target: np.ndarray, draft: np.ndarray, tokens: np.ndarray,
                  row_offsets: np.ndarray, T: np.ndarray, beta: np.ndarray, seed: int,
                  seq_ids: Optional[np.ndarray] = None, nthreads: int = 1,
                  uncertainty: int = UNC_MAXPROB) -> OracleResult:
    """target [R + B, V], draft [R, V], tokens [R]; row_offsets [B+1] int64 over draft rows."""
    lib = _load()
    target = np.ascontiguousarray(target)
    draft = np.ascontiguousarray(draft)
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    row_offsets = np.ascontiguousarray(row_offsets, dtype=np.int64)
    T = np.ascontiguousarray(T, dtype=np.float32)
    beta = np.ascontiguousarray(beta, dtype=np.float32)
    B = row_offsets.shape[0] - 1
    R = int(row_offsets[-1])
    V = target.shape[1]
    assert row_offsets[0] == 0 and np.all(np.diff(row_offsets) >= 0)
    assert target.shape == (R + B, V) and draft.shape == (R, V) and tokens.shape == (R,)
    assert T.shape == (B,) and beta.shape == (B,)
    if seq_ids is not None:
        seq_ids = np.ascontiguousarray(seq_ids, dtype=np.int64)
    acc = np.empty(B, dtype=np.int32)
    out = np.empty(R + B, dtype=np.int32)
    diag = np.empty((R, NDIAG), dtype=np.float64)
    path = np.empty(R, dtype=np.int32)
    samp = np.empty((B, NSAMP), dtype=np.float64)
    rc = lib.ears_oracle_verify_ragged(_ptr(target), _ptr(draft), _ptr(tokens), _ptr(row_offsets),
                                       _dtype_code(target), B, V, _ptr(T), _ptr(beta), int(uncertainty), int(seed),
                                       _ptr(seq_ids), _ptr(acc), _ptr(out), _ptr(diag), _ptr(path),
                                       _ptr(samp), int(nthreads))
    return OracleResult(acc, out, diag, path, samp, int(rc))


def verify_greedy(target: np.ndarray, tokens: np.ndarray, row_offsets: Optional[np.ndarray] = None):
    """Temperature -> 0 corner.  Rectangular: target [B, K+1, V], tokens [B, K].  Ragged: target
    [R + B, V], tokens [R], row_offsets [B+1].  Returns (accept_len, out_tokens, target_argmax)."""
    lib = _load()
    target = np.ascontiguousarray(target)
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    if row_offsets is None:
        B, K1, V = target.shape
        K = K1 - 1
        assert tokens.shape == (B, K)
        nrows = B * K1
        shape = (B, K1)
    else:
        row_offsets = np.ascontiguousarray(row_offsets, dtype=np.int64)
        B = row_offsets.shape[0] - 1
        K = 0
        V = target.shape[1]
        nrows = int(row_offsets[-1]) + B
        assert target.shape == (nrows, V) and tokens.shape == (nrows - B,)
        shape = (nrows,)
    acc = np.empty(B, dtype=np.int32)
    out = np.empty(shape, dtype=np.int32)
    amax = np.empty(shape, dtype=np.int32)
    lib.ears_oracle_verify_greedy(_ptr(target), _ptr(tokens), _ptr(row_offsets), _dtype_code(target),
                                  B, K, V, _ptr(acc), _ptr(out), _ptr(amax))
    return acc, out, amax


def round_bf16(x: float) -> int:
    """Bit pattern of the bfloat16 nearest to x (ties to even)."""
    return int(_load().ears_oracle_round_bf16(float(x)))


def lm_head_dot(hidden: np.ndarray, weight: np.ndarray, n: int, v: int) -> float:
    """One logit, sum_k hidden[n,k] * weight[v,k], in fp64; inputs are uint16 bf16 bit patterns."""
    assert hidden.dtype == np.uint16 and weight.dtype == np.uint16
    assert hidden.flags.c_contiguous and weight.flags.c_contiguous
    assert hidden.shape[1] == weight.shape[1]
    return float(_load().ears_oracle_lm_head_dot(_ptr(hidden), _ptr(weight), hidden.shape[1],
                                                 int(n), int(v)))


def lm_head(hidden: np.ndarray, weight: np.ndarray, nthreads: int = 1):
    """Vocabulary projection: returns (exact [N,V] float64, logits [N,V] uint16 bf16 bits)."""
    hidden = np.ascontiguousarray(hidden)
    weight = np.ascontiguousarray(weight)
    assert hidden.dtype == np.uint16 and weight.dtype == np.uint16
    N, D = hidden.shape
    V = weight.shape[0]
    assert weight.shape[1] == D
    exact = np.empty((N, V), dtype=np.float64)
    logits = np.empty((N, V), dtype=np.uint16)
    _load().ears_oracle_lm_head(_ptr(hidden), _ptr(weight), N, D, V, _ptr(exact), _ptr(logits),
                                int(nthreads))
    return exact, logits
