"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares, and
rejects bad arguments on the host before any GPU work (so these run without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ears.h")


@pytest.fixture(scope="module")
def L():
    from paper_2512_13194_amd import binding, build
    if build.is_stale():
        build.build()
    return binding.lib()


def _declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(ears_[a-z0-9_]+)\s*\(", src)))


def test_header_symbols_are_exported(L):
    names = _declared_functions()
    assert "ears_verify_bf16" in names and "ears_verify_ex" in names and len(names) >= 11
    for n in names:
        assert hasattr(L, n), n


def test_status_strings(L):
    from paper_2512_13194_amd import binding
    seen = {binding.status_string(i) for i in range(8)}
    assert len(seen) == 8 and binding.status_string(0) == "ok"
    assert binding.status_string(99) == "unknown status"


def test_workspace_bytes(L):
    from paper_2512_13194_amd import binding
    w = binding.ears_workspace_bytes(2048, 256, 128256)
    assert w >= 2048 * 2 * 16 and w % 256 == 0
    assert binding.ears_workspace_bytes(4096, 256, 128256) > w
    assert binding.ears_workspace_bytes(0, 1, 8) == 0
    assert binding.ears_workspace_bytes(8, 0, 8) == 0
    assert binding.ears_workspace_bytes(8, 1, 0) == 0
    assert binding.ears_workspace_bytes(3, 4, 8) > 0       # fewer rows than sequences: some have no draft token


P = 0x10000   # a 256-byte aligned stand-in address; never dereferenced on these paths


def _rect(L, fn="ears_verify_bf16", target=P, draft=P, tokens=P, B=2, K=3, V=64, T=1.0, beta=0.1,
          seed=0, acc=P, out=P):
    return getattr(L, fn)(target, draft, tokens, B, K, V, T, beta, seed, acc, out, None)


def test_rect_argument_errors(L):
    from paper_2512_13194_amd import binding as b
    assert _rect(L, target=None) == b.EARS_ERR_NULL
    assert _rect(L, draft=None) == b.EARS_ERR_NULL
    assert _rect(L, tokens=None) == b.EARS_ERR_NULL
    assert _rect(L, acc=None) == b.EARS_ERR_NULL
    assert _rect(L, out=None) == b.EARS_ERR_NULL
    for kw in (dict(B=0), dict(K=0), dict(V=0), dict(B=-1), dict(K=-5)):
        assert _rect(L, **kw) == b.EARS_ERR_SHAPE, kw
    for T in (0.0, -1.0, float("inf"), float("nan")):
        assert _rect(L, T=T) == b.EARS_ERR_PARAM
    for beta in (-0.1, float("inf"), float("nan")):
        assert _rect(L, beta=beta) == b.EARS_ERR_PARAM
    assert _rect(L, target=P + 8) == b.EARS_ERR_ALIGN
    assert _rect(L, draft=P + 2) == b.EARS_ERR_ALIGN
    assert _rect(L, tokens=P + 2) == b.EARS_ERR_ALIGN
    assert _rect(L, fn="ears_verify_f32", out=P + 1) == b.EARS_ERR_ALIGN


def _ex(L, dtype=1, target=P, draft=P, tokens=P, off=None, R=6, B=2, K=3, V=64, T=1.0, beta=0.1,
        Ts=None, betas=None, unc=0, seed=0, ids=None, ws=P, wsb=1 << 20, stages=7, acc=P, out=P,
        stats=None, path=None, status=None):
    return L.ears_verify_ex(dtype, target, draft, tokens, off, R, B, K, V, T, beta, Ts, betas, unc,
                            seed, ids, ws, wsb, stages, acc, out, stats, path, status, None)


def test_ex_argument_errors(L):
    from paper_2512_13194_amd import binding as b
    assert _ex(L, dtype=2) == b.EARS_ERR_DTYPE
    assert _ex(L, dtype=-1) == b.EARS_ERR_DTYPE
    assert _ex(L, R=7) == b.EARS_ERR_SHAPE                 # rectangular: R must be B*K
    assert _ex(L, off=P, R=0, B=2) == b.EARS_ERR_SHAPE     # ragged: at least one draft row in all
    assert _ex(L, stages=0) == b.EARS_ERR_PARAM
    assert _ex(L, stages=8) == b.EARS_ERR_PARAM
    assert _ex(L, unc=3) == b.EARS_ERR_PARAM
    assert _ex(L, unc=-1) == b.EARS_ERR_PARAM
    assert _ex(L, T=0.0) == b.EARS_ERR_PARAM
    assert _ex(L, T=0.0, Ts=P, ws=None) == b.EARS_ERR_WORKSPACE   # per-sequence T: scalar ignored
    assert _ex(L, ws=None) == b.EARS_ERR_WORKSPACE
    assert _ex(L, wsb=16) == b.EARS_ERR_WORKSPACE
    assert _ex(L, ws=P + 64) == b.EARS_ERR_ALIGN
    assert _ex(L, off=P + 4, R=6) == b.EARS_ERR_ALIGN
    assert _ex(L, ids=P + 4) == b.EARS_ERR_ALIGN
    assert _ex(L, stats=P + 4) == b.EARS_ERR_ALIGN
    need = b.ears_workspace_bytes(6, 2, 64)
    assert _ex(L, wsb=need - 1) == b.EARS_ERR_WORKSPACE


def test_noalloc_argument_errors(L):
    """Every check of the entry point without a workspace, its size limit included, happens on the
    host before the first HIP call."""
    from paper_2512_13194_amd import binding as b

    def call(dtype=1, target=P, draft=P, tokens=P, off=None, R=6, B=2, K=3, V=64, T=1.0, beta=0.1,
             unc=0, stages=7, acc=P, out=P):
        return L.ears_verify_noalloc(dtype, target, draft, tokens, off, R, B, K, V, T, beta, None, None,
                                     unc, 0, None, stages, acc, out, None, None, None, None)
    assert call(dtype=5) == b.EARS_ERR_DTYPE
    assert call(target=None) == b.EARS_ERR_NULL
    assert call(acc=None) == b.EARS_ERR_NULL
    assert call(R=7) == b.EARS_ERR_SHAPE
    assert call(T=-1.0) == b.EARS_ERR_PARAM
    assert call(unc=9) == b.EARS_ERR_PARAM
    assert call(stages=0) == b.EARS_ERR_PARAM
    assert call(draft=P + 8) == b.EARS_ERR_ALIGN
    # statistics of 4096 * 64 positions do not fit the fixed scratch
    assert b.ears_workspace_bytes(4096 * 64, 4096, 8) > b.EARS_NOALLOC_SCRATCH_BYTES
    assert call(R=4096 * 64, B=4096, K=64, V=8) == b.EARS_ERR_WORKSPACE


def test_ragged_argument_errors(L):
    from paper_2512_13194_amd import binding as b
    f = L.ears_verify_ragged_bf16
    assert f(P, P, P, None, 6, 2, 64, P, P, 0, P, P, None) == b.EARS_ERR_NULL
    assert f(P, P, P, P, 6, 2, 64, None, P, 0, P, P, None) == b.EARS_ERR_NULL
    assert f(P, P, P, P, 6, 2, 64, P, None, 0, P, P, None) == b.EARS_ERR_NULL
    assert f(P, P, P, P, 0, 2, 64, P, P, 0, P, P, None) == b.EARS_ERR_SHAPE
    assert f(P, P, P, P, 6, 0, 64, P, P, 0, P, P, None) == b.EARS_ERR_SHAPE
    assert f(P + 4, P, P, P, 6, 2, 64, P, P, 0, P, P, None) == b.EARS_ERR_ALIGN


def test_bench_aid_argument_errors(L):
    from paper_2512_13194_amd import binding as b
    assert L.ears_bench_read(None, 1024, P, None) == b.EARS_ERR_NULL
    assert L.ears_bench_read(P, 1000, P, None) == b.EARS_ERR_SHAPE
    assert L.ears_bench_read(P + 8, 1024, P, None) == b.EARS_ERR_ALIGN
    assert L.ears_bench_copy(P, None, 1024, None) == b.EARS_ERR_NULL
    assert L.ears_bench_copy(P, P, 0, None) == b.EARS_ERR_SHAPE
    assert L.ears_bench_read_sink_words() >= 256


def test_binding_and_oracle_do_not_import_each_other():
    pkg = os.path.join(ROOT, "paper_2512_13194_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                assert "oracle" not in open(os.path.join(dirpath, f)).read().replace(
                    "the CPU oracle", "").replace("CPU oracle", ""), f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            src = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2512_13194_amd" not in src and "hip" not in src.lower().replace("relationship", ""), f


def _greedy(L, dtype=1, target=P, tokens=P, off=None, R=6, B=2, K=3, V=64, ws=P, wsb=1 << 20,
            acc=P, out=P):
    return L.ears_verify_greedy(dtype, target, tokens, off, R, B, K, V, ws, wsb, acc, out, None)


def test_greedy_argument_errors(L):
    from paper_2512_13194_amd import binding as b
    assert b.ears_greedy_workspace_bytes(2048, 256) == (2048 + 256) * 4
    assert b.ears_greedy_workspace_bytes(7, 3) % 256 == 0
    assert b.ears_greedy_workspace_bytes(0, 1) == 0 and b.ears_greedy_workspace_bytes(2, 3) == 256
    assert _greedy(L, dtype=2) == b.EARS_ERR_DTYPE
    assert _greedy(L, target=None) == b.EARS_ERR_NULL
    assert _greedy(L, tokens=None) == b.EARS_ERR_NULL
    assert _greedy(L, acc=None) == b.EARS_ERR_NULL
    assert _greedy(L, out=None) == b.EARS_ERR_NULL
    assert _greedy(L, B=0) == b.EARS_ERR_SHAPE
    assert _greedy(L, V=0) == b.EARS_ERR_SHAPE
    assert _greedy(L, K=0) == b.EARS_ERR_SHAPE
    assert _greedy(L, R=7) == b.EARS_ERR_SHAPE              # rectangular: R must be B*K
    assert _greedy(L, off=P, R=0, B=2) == b.EARS_ERR_SHAPE  # no draft row at all
    assert _greedy(L, target=P + 8) == b.EARS_ERR_ALIGN
    assert _greedy(L, tokens=P + 2) == b.EARS_ERR_ALIGN
    assert _greedy(L, off=P + 4) == b.EARS_ERR_ALIGN
    assert _greedy(L, ws=P + 16) == b.EARS_ERR_ALIGN
    assert _greedy(L, wsb=16) == b.EARS_ERR_WORKSPACE


def _lm(L, hidden=P, weight=P, N=8, D=128, V=100, T=1.0, rowT=None, logits=P, rmax=P, rsum=P,
        ws=P, wsb=1 << 20):
    return L.ears_lm_head_bf16(hidden, weight, N, D, V, T, rowT, logits, rmax, rsum, None, ws, wsb, None)


def test_lm_head_argument_errors(L):
    from paper_2512_13194_amd import binding as b
    w = b.ears_lm_head_workspace_bytes(2304, 128256)
    assert w >= 3 * 2304 * 2 * 501 * 4 and w % 256 == 0
    assert b.ears_lm_head_workspace_bytes(0, 5) == 0 and b.ears_lm_head_workspace_bytes(5, 0) == 0
    for name in ("hidden", "weight", "logits", "rmax", "rsum"):
        assert _lm(L, **{name: None}) == b.EARS_ERR_NULL
    assert _lm(L, N=0) == b.EARS_ERR_SHAPE
    assert _lm(L, V=0) == b.EARS_ERR_SHAPE
    assert _lm(L, D=96) == b.EARS_ERR_SHAPE               # D must be a multiple of 64
    assert _lm(L, D=0) == b.EARS_ERR_SHAPE
    assert _lm(L, D=(1 << 20) + 64) == b.EARS_ERR_SHAPE    # a tile's rows beyond 32-bit byte offsets
    assert _lm(L, T=0.0) == b.EARS_ERR_PARAM
    assert _lm(L, T=float("nan")) == b.EARS_ERR_PARAM
    assert _lm(L, hidden=P + 8) == b.EARS_ERR_ALIGN
    assert _lm(L, rsum=P + 4) == b.EARS_ERR_ALIGN
    assert _lm(L, ws=None) == b.EARS_ERR_WORKSPACE
    assert _lm(L, wsb=64) == b.EARS_ERR_WORKSPACE
    assert _lm(L, ws=P + 64) == b.EARS_ERR_ALIGN


def test_import_stats_argument_errors(L):
    from paper_2512_13194_amd import binding as b

    def imp(dtype=1, target=P, draft=P, tokens=P, off=None, R=6, B=2, K=3, V=64, tm=P, ts=P, dm=P,
            ds=P, ws=P, wsb=1 << 20):
        return L.ears_import_stats(dtype, target, draft, tokens, off, R, B, K, V, tm, ts, None, dm, ds,
                                   ws, wsb, None)
    for name in ("tm", "ts", "dm", "ds", "target", "draft", "tokens"):
        assert imp(**{name: None}) == b.EARS_ERR_NULL
    assert imp(dtype=3) == b.EARS_ERR_DTYPE
    assert imp(R=7) == b.EARS_ERR_SHAPE
    assert imp(ts=P + 4) == b.EARS_ERR_ALIGN
    assert imp(wsb=8) == b.EARS_ERR_WORKSPACE


def test_row_stats_argument_errors(L):
    from paper_2512_13194_amd import binding as b

    def rs(dtype=1, logits=P, rows=4, V=64, T=1.0, rowT=None, rmax=P, rsum=P):
        return L.ears_row_stats(dtype, logits, rows, V, T, rowT, rmax, rsum, None, None)
    assert rs(dtype=7) == b.EARS_ERR_DTYPE
    assert rs(logits=None) == b.EARS_ERR_NULL and rs(rmax=None) == b.EARS_ERR_NULL
    assert rs(rows=0) == b.EARS_ERR_SHAPE and rs(V=0) == b.EARS_ERR_SHAPE
    assert rs(T=-1.0) == b.EARS_ERR_PARAM
    assert rs(logits=P + 4) == b.EARS_ERR_ALIGN and rs(rsum=P + 4) == b.EARS_ERR_ALIGN


def test_committed_counter_summaries_belong_to_the_current_kernels():
    """bench.py reports the HBM traffic of the statistics kernel and the instruction count of the
    sampling kernel from counter runs committed under profiles/, and only while the hash of the
    kernel sources, the launch code and the build script matches: a change to any of them without
    new counter runs would silently turn the figures into null."""
    import bench
    assert bench.committed_counters(bench.TRAFFIC_FILE) is not None, "regenerate profiles/traffic_verify_c2.json"
    assert bench.committed_counters(bench.FILTER_FILE) is not None, "regenerate profiles/filter_counters_c2.json"
