"""Thin ctypes binding of libears.so (the C ABI of include/ears.h).

Argument marshalling only: torch supplies device memory and the HIP stream; every step of the
verification runs in the library's kernels.  There is no fallback: if the library has not been
built, importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libears.so")

EARS_OK = 0
EARS_ERR_NULL, EARS_ERR_SHAPE, EARS_ERR_PARAM, EARS_ERR_ALIGN = 1, 2, 3, 4
EARS_ERR_DTYPE, EARS_ERR_WORKSPACE, EARS_ERR_HIP = 5, 6, 7
EARS_F32, EARS_BF16 = 0, 1
EARS_STAGE_STATS, EARS_STAGE_DECIDE, EARS_STAGE_SAMPLE, EARS_STAGE_ALL = 1, 2, 4, 7
EARS_UNCERTAINTY_MAXPROB, EARS_UNCERTAINTY_ENTROPY, EARS_UNCERTAINTY_VARIANCE = 0, 1, 2
EARS_NSTATS = 10
STAT_NAMES = ("m_t", "Z_t", "P_t_x", "m_d", "Z_d", "P_d_x", "unc", "R", "U", "thr")

_lib = None


class EarsError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__("ears: %s (status %d)" % (status_string(status), status))


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built (python -m paper_2512_13194_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "libears.so is missing: build it with `python paper_2512_13194_amd/build.py` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        c = ctypes
        vp, i32, i64, f32, u64, sz = c.c_void_p, c.c_int, c.c_int64, c.c_float, c.c_uint64, c.c_size_t
        L.ears_status_string.argtypes = [i32]
        L.ears_status_string.restype = c.c_char_p
        rect = [vp, vp, vp, i32, i32, i32, f32, f32, u64, vp, vp, vp]
        for name in ("ears_verify_f32", "ears_verify_bf16"):
            getattr(L, name).argtypes = rect
            getattr(L, name).restype = i32
        ragged = [vp, vp, vp, vp, i64, i32, i32, vp, vp, u64, vp, vp, vp]
        for name in ("ears_verify_ragged_f32", "ears_verify_ragged_bf16"):
            getattr(L, name).argtypes = ragged
            getattr(L, name).restype = i32
        L.ears_workspace_bytes.argtypes = [i64, i32, i32]
        L.ears_workspace_bytes.restype = sz
        L.ears_verify_ex.argtypes = [i32, vp, vp, vp, vp, i64, i32, i32, i32, f32, f32, vp, vp, i32,
                                     u64, vp, vp, sz, i32, vp, vp, vp, vp, vp, vp]
        L.ears_verify_ex.restype = i32
        L.ears_verify_noalloc.argtypes = [i32, vp, vp, vp, vp, i64, i32, i32, i32, f32, f32, vp, vp,
                                          i32, u64, vp, i32, vp, vp, vp, vp, vp, vp]
        L.ears_verify_noalloc.restype = i32
        L.ears_greedy_workspace_bytes.argtypes = [i64, i32]
        L.ears_greedy_workspace_bytes.restype = sz
        L.ears_verify_greedy.argtypes = [i32, vp, vp, vp, i64, i32, i32, i32, vp, sz, vp, vp, vp]
        L.ears_verify_greedy.restype = i32
        L.ears_lm_head_workspace_bytes.argtypes = [i32, i32]
        L.ears_lm_head_workspace_bytes.restype = sz
        L.ears_lm_head_bf16.argtypes = [vp, vp, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp, sz, vp]
        L.ears_lm_head_bf16.restype = i32
        L.ears_row_stats.argtypes = [i32, vp, i64, i32, f32, vp, vp, vp, vp, vp]
        L.ears_row_stats.restype = i32
        L.ears_import_stats.argtypes = [i32, vp, vp, vp, vp, i64, i32, i32, i32, vp, vp, vp, vp, vp,
                                        vp, sz, vp]
        L.ears_import_stats.restype = i32
        L.ears_release.argtypes = []
        L.ears_release.restype = None
        L.ears_test_single_launch.argtypes = [i32, i32]
        L.ears_test_single_launch.restype = None
        L.ears_bench_read_sink_words.argtypes = []
        L.ears_bench_read_sink_words.restype = i32
        L.ears_bench_read.argtypes = [vp, sz, vp, vp]
        L.ears_bench_read.restype = i32
        L.ears_bench_copy.argtypes = [vp, vp, sz, vp]
        L.ears_bench_copy.restype = i32
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().ears_status_string(int(status)).decode()


def _check(status: int) -> None:
    if status != EARS_OK:
        raise EarsError(status)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream: Optional[torch.cuda.Stream]) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return EARS_F32
    if t.dtype == torch.bfloat16:
        return EARS_BF16
    raise TypeError("logits must be float32 or bfloat16, got %s" % t.dtype)


def _need(t: torch.Tensor, dtype, name: str) -> None:
    if not (t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise TypeError("%s must be a contiguous CUDA tensor of %s" % (name, dtype))


def ears_workspace_bytes(total_draft_rows: int, B: int, V: int) -> int:
    return int(lib().ears_workspace_bytes(int(total_draft_rows), int(B), int(V)))


def _ears_verify_rect(fn, dtype, target, draft, tokens, temperature, beta, seed, out_accept_len,
                      out_tokens, stream):
    B, K1, V = target.shape
    K = K1 - 1
    _need(target, dtype, "target_logits")
    _need(draft, dtype, "draft_logits")
    _need(tokens, torch.int32, "draft_tokens")
    assert tuple(draft.shape) == (B, K, V) and tuple(tokens.shape) == (B, K)
    if out_accept_len is None:
        out_accept_len = torch.empty(B, dtype=torch.int32, device=target.device)
    if out_tokens is None:
        out_tokens = torch.empty(B, K + 1, dtype=torch.int32, device=target.device)
    _need(out_accept_len, torch.int32, "out_accept_len")
    _need(out_tokens, torch.int32, "out_tokens")
    _check(fn(_ptr(target), _ptr(draft), _ptr(tokens), B, K, V, float(temperature), float(beta),
              int(seed), _ptr(out_accept_len), _ptr(out_tokens), _stream(stream)))
    return out_accept_len, out_tokens


def ears_verify_f32(target_logits, draft_logits, draft_tokens, temperature, beta, seed,
                    out_accept_len=None, out_tokens=None, stream=None):
    """target [B,K+1,V] f32, draft [B,K,V] f32, tokens [B,K] i32 -> (accept_len [B], tokens [B,K+1])."""
    return _ears_verify_rect(lib().ears_verify_f32, torch.float32, target_logits, draft_logits,
                             draft_tokens, temperature, beta, seed, out_accept_len, out_tokens, stream)


def ears_verify_bf16(target_logits, draft_logits, draft_tokens, temperature, beta, seed,
                     out_accept_len=None, out_tokens=None, stream=None):
    return _ears_verify_rect(lib().ears_verify_bf16, torch.bfloat16, target_logits, draft_logits,
                             draft_tokens, temperature, beta, seed, out_accept_len, out_tokens, stream)


def _ears_verify_ragged(fn, dtype, target, draft, tokens, row_offsets, temperature, beta, seed,
                        out_accept_len, out_tokens, stream):
    R, V = draft.shape
    B = row_offsets.shape[0] - 1
    _need(target, dtype, "target_logits")
    _need(draft, dtype, "draft_logits")
    _need(tokens, torch.int32, "draft_tokens")
    _need(row_offsets, torch.int64, "row_offsets")
    _need(temperature, torch.float32, "temperature")
    _need(beta, torch.float32, "beta")
    assert tuple(target.shape) == (R + B, V) and tuple(tokens.shape) == (R,)
    assert tuple(temperature.shape) == (B,) and tuple(beta.shape) == (B,)
    if out_accept_len is None:
        out_accept_len = torch.empty(B, dtype=torch.int32, device=target.device)
    if out_tokens is None:
        out_tokens = torch.empty(R + B, dtype=torch.int32, device=target.device)
    _check(fn(_ptr(target), _ptr(draft), _ptr(tokens), _ptr(row_offsets), R, B, V,
              _ptr(temperature), _ptr(beta), int(seed), _ptr(out_accept_len), _ptr(out_tokens),
              _stream(stream)))
    return out_accept_len, out_tokens


def ears_verify_ragged_f32(target_logits, draft_logits, draft_tokens, row_offsets, temperature,
                           beta, seed, out_accept_len=None, out_tokens=None, stream=None):
    """Packed target [R+B,V], draft [R,V], tokens [R], row_offsets [B+1] i64, T/beta [B] f32."""
    return _ears_verify_ragged(lib().ears_verify_ragged_f32, torch.float32, target_logits,
                               draft_logits, draft_tokens, row_offsets, temperature, beta, seed,
                               out_accept_len, out_tokens, stream)


def ears_verify_ragged_bf16(target_logits, draft_logits, draft_tokens, row_offsets, temperature,
                            beta, seed, out_accept_len=None, out_tokens=None, stream=None):
    return _ears_verify_ragged(lib().ears_verify_ragged_bf16, torch.bfloat16, target_logits,
                               draft_logits, draft_tokens, row_offsets, temperature, beta, seed,
                               out_accept_len, out_tokens, stream)


def ears_verify_ex(target_logits, draft_logits, draft_tokens, *, row_offsets=None, K=None,
                   temperature=1.0, beta=0.0, temperature_per_seq=None, beta_per_seq=None,
                   uncertainty=EARS_UNCERTAINTY_MAXPROB, seed=0,
                   seq_ids=None, workspace=None, stages=EARS_STAGE_ALL, out_accept_len=None,
                   out_tokens=None, want_stats=False, want_path=False, status_word=None,
                   stream=None):
    """Full-control call.  Logits may be [B,K+1,V]/[B,K,V] (rectangular, row_offsets None) or packed
    2-D with row_offsets.  Returns a dict with accept_len, tokens, and optionally stats [R,10]
    float64, path [R] int32; `workspace` (uint8 CUDA tensor) is allocated when not given and
    returned so that later stages can reuse the cached statistics."""
    dev = target_logits.device
    V = target_logits.shape[-1]
    if row_offsets is None:
        B, K1, _ = target_logits.shape
        K = K1 - 1
        R = B * K
    else:
        B = row_offsets.shape[0] - 1
        R = draft_logits.shape[0]
        K = 0
    need = ears_workspace_bytes(R, B, V)
    if workspace is None:
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=dev)
    if out_accept_len is None:
        out_accept_len = torch.empty(B, dtype=torch.int32, device=dev)
    if out_tokens is None:
        out_tokens = torch.empty(R + B, dtype=torch.int32, device=dev)
    stats = torch.empty(R, EARS_NSTATS, dtype=torch.float64, device=dev) if want_stats is True else (
        want_stats if isinstance(want_stats, torch.Tensor) else None)
    path = torch.empty(R, dtype=torch.int32, device=dev) if want_path is True else (
        want_path if isinstance(want_path, torch.Tensor) else None)
    _check(lib().ears_verify_ex(
        _dtype_code(target_logits), _ptr(target_logits), _ptr(draft_logits), _ptr(draft_tokens),
        _ptr(row_offsets), R, B, K, V, float(temperature), float(beta), _ptr(temperature_per_seq),
        _ptr(beta_per_seq), int(uncertainty), int(seed), _ptr(seq_ids), _ptr(workspace),
        workspace.numel(),
        int(stages), _ptr(out_accept_len), _ptr(out_tokens), _ptr(stats), _ptr(path),
        _ptr(status_word), _stream(stream)))
    return dict(accept_len=out_accept_len, tokens=out_tokens, stats=stats, path=path,
                workspace=workspace)


EARS_NOALLOC_SCRATCH_BYTES = 4 << 20


def ears_verify_noalloc(target_logits, draft_logits, draft_tokens, out_accept_len, out_tokens, *,
                        row_offsets=None, temperature=1.0, beta=0.0, temperature_per_seq=None,
                        beta_per_seq=None, uncertainty=EARS_UNCERTAINTY_MAXPROB, seed=0, seq_ids=None,
                        stages=EARS_STAGE_ALL, out_stats=None, out_path=None, status_word=None,
                        stream=None):
    """ears_verify_ex on the library's fixed device scratch: allocates nothing, here or in the
    library, so every output tensor is the caller's (accept_len [B], tokens [R + B] int32)."""
    V = target_logits.shape[-1]
    if row_offsets is None:
        B, K1, _ = target_logits.shape
        K = K1 - 1
        R = B * K
    else:
        B = row_offsets.shape[0] - 1
        R = draft_logits.shape[0]
        K = 0
    _check(lib().ears_verify_noalloc(
        _dtype_code(target_logits), _ptr(target_logits), _ptr(draft_logits), _ptr(draft_tokens),
        _ptr(row_offsets), R, B, K, V, float(temperature), float(beta), _ptr(temperature_per_seq),
        _ptr(beta_per_seq), int(uncertainty), int(seed), _ptr(seq_ids), int(stages),
        _ptr(out_accept_len), _ptr(out_tokens), _ptr(out_stats), _ptr(out_path), _ptr(status_word),
        _stream(stream)))
    return out_accept_len, out_tokens


def ears_greedy_workspace_bytes(total_draft_rows: int, B: int) -> int:
    return int(lib().ears_greedy_workspace_bytes(int(total_draft_rows), int(B)))


def ears_verify_greedy(target_logits, draft_tokens, *, row_offsets=None, workspace=None,
                       out_accept_len=None, out_tokens=None, stream=None):
    """Temperature -> 0 corner.  target [B,K+1,V] + tokens [B,K], or packed target [R+B,V] +
    tokens [R] + row_offsets [B+1].  Returns (accept_len [B], tokens [B,K+1] or packed [R+B])."""
    dev = target_logits.device
    V = target_logits.shape[-1]
    _need(target_logits, target_logits.dtype, "target_logits")
    _need(draft_tokens, torch.int32, "draft_tokens")
    if row_offsets is None:
        B, K1, _ = target_logits.shape
        K = K1 - 1
        R = B * K
        assert tuple(draft_tokens.shape) == (B, K)
        shape = (B, K1)
    else:
        _need(row_offsets, torch.int64, "row_offsets")
        B = row_offsets.shape[0] - 1
        R = draft_tokens.shape[0]
        K = 0
        assert tuple(target_logits.shape) == (R + B, V)
        shape = (R + B,)
    if out_accept_len is None:
        out_accept_len = torch.empty(B, dtype=torch.int32, device=dev)
    if out_tokens is None:
        out_tokens = torch.empty(shape, dtype=torch.int32, device=dev)
    _need(out_accept_len, torch.int32, "out_accept_len")
    _need(out_tokens, torch.int32, "out_tokens")
    assert out_accept_len.numel() == B and out_tokens.numel() == R + B
    _check(lib().ears_verify_greedy(
        _dtype_code(target_logits), _ptr(target_logits), _ptr(draft_tokens), _ptr(row_offsets), R, B,
        K, V, _ptr(workspace), 0 if workspace is None else workspace.numel(),
        _ptr(out_accept_len), _ptr(out_tokens), _stream(stream)))
    return out_accept_len, out_tokens


def ears_lm_head_workspace_bytes(N: int, V: int) -> int:
    return int(lib().ears_lm_head_workspace_bytes(int(N), int(V)))


def ears_lm_head_bf16(hidden, weight, *, temperature=1.0, row_temperature=None, out_logits=None,
                      out_row_max=None, out_row_sumexp=None, out_row_entropy=None, workspace=None,
                      stream=None):
    """hidden [N,D] bf16, weight [V,D] bf16 -> (logits [N,V] bf16, row_max [N] f32, row_sumexp [N] f64);
    out_row_entropy (f64 [N]) is filled when given."""
    _need(hidden, torch.bfloat16, "hidden")
    _need(weight, torch.bfloat16, "weight")
    N, D = hidden.shape
    V = weight.shape[0]
    assert weight.shape[1] == D
    dev = hidden.device
    if out_logits is None:
        out_logits = torch.empty(N, V, dtype=torch.bfloat16, device=dev)
    if out_row_max is None:
        out_row_max = torch.empty(N, dtype=torch.float32, device=dev)
    if out_row_sumexp is None:
        out_row_sumexp = torch.empty(N, dtype=torch.float64, device=dev)
    if workspace is None:
        workspace = torch.empty(max(ears_lm_head_workspace_bytes(N, V), 1), dtype=torch.uint8, device=dev)
    _need(out_logits, torch.bfloat16, "out_logits")
    _need(out_row_max, torch.float32, "out_row_max")
    _need(out_row_sumexp, torch.float64, "out_row_sumexp")
    assert tuple(out_logits.shape) == (N, V) and out_row_max.numel() == N and out_row_sumexp.numel() == N
    if row_temperature is not None:
        _need(row_temperature, torch.float32, "row_temperature")
        assert row_temperature.numel() == N
    if out_row_entropy is not None:
        _need(out_row_entropy, torch.float64, "out_row_entropy")
        assert out_row_entropy.numel() == N
    _check(lib().ears_lm_head_bf16(_ptr(hidden), _ptr(weight), N, D, V, float(temperature),
                                   _ptr(row_temperature), _ptr(out_logits), _ptr(out_row_max),
                                   _ptr(out_row_sumexp), _ptr(out_row_entropy), _ptr(workspace),
                                   workspace.numel(), _stream(stream)))
    return out_logits, out_row_max, out_row_sumexp


def ears_row_stats(logits, *, temperature=1.0, row_temperature=None, out_row_max=None,
                   out_row_sumexp=None, out_row_entropy=None, stream=None):
    """Per-row (max, sum-exp) of logits [..., V] (f32 or bf16): returns (row_max f32, row_sumexp f64)
    shaped like the leading dimensions."""
    _need(logits, logits.dtype, "logits")
    V = logits.shape[-1]
    rows = logits.numel() // V
    lead = tuple(logits.shape[:-1])
    if out_row_max is None:
        out_row_max = torch.empty(lead, dtype=torch.float32, device=logits.device)
    if out_row_sumexp is None:
        out_row_sumexp = torch.empty(lead, dtype=torch.float64, device=logits.device)
    _need(out_row_max, torch.float32, "out_row_max")
    _need(out_row_sumexp, torch.float64, "out_row_sumexp")
    assert out_row_max.numel() == rows == out_row_sumexp.numel()
    if row_temperature is not None:
        _need(row_temperature, torch.float32, "row_temperature")
        assert row_temperature.numel() == rows
    if out_row_entropy is not None:
        _need(out_row_entropy, torch.float64, "out_row_entropy")
        assert out_row_entropy.numel() == rows
    _check(lib().ears_row_stats(_dtype_code(logits), _ptr(logits), rows, V, float(temperature),
                                _ptr(row_temperature), _ptr(out_row_max), _ptr(out_row_sumexp),
                                _ptr(out_row_entropy), _stream(stream)))
    return out_row_max, out_row_sumexp


def ears_import_stats(target_logits, draft_logits, draft_tokens, target_row_max, target_row_sumexp,
                      draft_row_max, draft_row_sumexp, workspace, *, target_row_entropy=None,
                      row_offsets=None, stream=None):
    """Fills `workspace` (uint8 CUDA tensor of ears_workspace_bytes) with producer-side statistics."""
    V = target_logits.shape[-1]
    if row_offsets is None:
        B, K1, _ = target_logits.shape
        K = K1 - 1
        R = B * K
    else:
        B = row_offsets.shape[0] - 1
        R = draft_logits.shape[0]
        K = 0
    _need(target_row_max, torch.float32, "target_row_max")
    _need(draft_row_max, torch.float32, "draft_row_max")
    _need(target_row_sumexp, torch.float64, "target_row_sumexp")
    _need(draft_row_sumexp, torch.float64, "draft_row_sumexp")
    assert target_row_max.numel() == R + B == target_row_sumexp.numel()
    assert draft_row_max.numel() == R == draft_row_sumexp.numel()
    if target_row_entropy is not None:
        _need(target_row_entropy, torch.float64, "target_row_entropy")
        assert target_row_entropy.numel() == R + B
    _check(lib().ears_import_stats(
        _dtype_code(target_logits), _ptr(target_logits), _ptr(draft_logits), _ptr(draft_tokens),
        _ptr(row_offsets), R, B, K, V, _ptr(target_row_max), _ptr(target_row_sumexp),
        _ptr(target_row_entropy), _ptr(draft_row_max), _ptr(draft_row_sumexp), _ptr(workspace),
        workspace.numel(), _stream(stream)))
    return workspace


def ears_release() -> None:
    lib().ears_release()


def ears_test_single_launch(force: bool, wait_polls: int = -1) -> None:
    lib().ears_test_single_launch(1 if force else 0, int(wait_polls))


def ears_bench_read(src: torch.Tensor, sink: Optional[torch.Tensor] = None, stream=None):
    if sink is None:
        sink = torch.empty(lib().ears_bench_read_sink_words(), dtype=torch.int32, device=src.device)
    _check(lib().ears_bench_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink),
                                 _stream(stream)))
    return sink


def ears_bench_copy(dst: torch.Tensor, src: torch.Tensor, stream=None):
    _check(lib().ears_bench_copy(_ptr(dst), _ptr(src), src.numel() * src.element_size(),
                                 _stream(stream)))
    return dst
