"""Host-only checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_2601_07891_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _ensure_built():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2601_07891_amd import build
        build.build(verbose=False)


@pytest.fixture(scope="module")
def lib():
    _ensure_built()
    return binding.lib()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "kvzap.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvzap_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert set(names) == set(binding.SIGNATURES)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(lib):
    seen = set()
    for code in range(0, -9, -1):
        s = lib.kvzap_status_string(code).decode()
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 9
    assert lib.kvzap_status_string(-99).decode() == "unknown status"
    assert re.fullmatch(r"\d+\.\d+\.\d+", lib.kvzap_version().decode())


def test_workspace_queries(lib):
    q = lib.kvzap_workspace_bytes
    assert q(binding.CALL_SCORE, 1, 131072, 4096, 512, 8) == 512 * 4096 * 2   # re-ordered copy of W1
    # a short prompt takes the split first projection: fp32 partial sums of up to 16 K-slices
    n = q(binding.CALL_SCORE, 1, 1024, 4096, 512, 8)
    assert 1024 * 512 * 4 <= n <= 16 * 1024 * 512 * 4 and n % 256 == 0
    assert q(binding.CALL_SCORE, 1, 1024, 4096, 0, 8) == 0
    assert q(binding.CALL_COMPACT, 1, 1024, 0, 0, 8) == 0
    n = q(binding.CALL_MASK, 1, 131072, 0, 0, 8)
    chunks = 8 * 128
    assert n >= chunks * 12 and n % 256 == 0
    assert q(binding.CALL_MASK, 0, 1024, 0, 0, 8) == 0
    assert q(binding.CALL_DECODE_EVICT, 64, 1, 4096, 512, 8) >= 64 * 512 * 4
    assert q(binding.CALL_DECODE_EVICT, 64, 1, 4096, 0, 8) == 0
    assert q(binding.CALL_DECODE_EVICT, 64, 1, 4096, 100, 8) == 0     # unsupported width


P = 0x10000      # fake, aligned, never dereferenced: all calls below fail validation first
ERR = dict(null=-1, shape=-2, align=-3, unsupported=-4, capacity=-5, workspace=-6)


def test_mask_static_rejects_before_any_gpu_call(lib):
    # the allocation-free mask: kvzap_mask's checks, then its own size limit -- all on the host
    f = lib.kvzap_mask_static
    assert f(None, 0.0, 128, None, 1, 8, 1024, P, P, P, None) == ERR["null"]
    assert f(P, 0.0, 128, None, 1, 8, 1024, None, P, P, None) == ERR["null"]
    assert f(P, 0.0, -1, None, 1, 8, 1024, P, P, P, None) == ERR["shape"]
    assert f(P, float("nan"), 128, None, 1, 8, 1024, P, P, P, None) == ERR["shape"]
    assert f(P + 4, 0.0, 128, None, 1, 8, 1024, P, P, P, None) == ERR["align"]
    assert f(P, 0.0, 128, None, 8192, 8, 1024, P, P, P, None) == ERR["unsupported"]   # B*H > 65535
    limit = 65536                                   # KVZAP_MASK_STATIC_MAX_CHUNKS
    text = open(os.path.join(ROOT, "include", "kvzap.h")).read()
    assert int(re.search(r"#define KVZAP_MASK_STATIC_MAX_CHUNKS (\d+)", text).group(1)) == limit
    # one chunk too many: 8 heads x (limit/8 + 1) chunks of 1024 positions
    assert f(P, 0.0, 128, None, 1, 8, (limit // 8) * 1024 + 1, P, P, P, None) == -8
    assert f(P, 0.0, 128, None, 8, 16, 513 * 1024, P, P, P, None) == -8
    assert "built-in scratch" in lib.kvzap_status_string(-8).decode()


def test_score_argument_errors(lib):
    f = lib.kvzap_score
    assert f(None, P, None, None, None, P, 1, 16, 4096, 0, 8, None, 0, None) == ERR["null"]
    assert f(P, P, None, None, None, None, 1, 16, 4096, 0, 8, None, 0, None) == ERR["null"]
    assert f(P, P, None, None, None, P, 1, 16, 4096, 512, 8, None, 0, None) == ERR["null"]   # MLP without W2
    assert f(P, P, None, P, None, P, 1, 16, 4096, 0, 8, None, 0, None) == ERR["shape"]      # linear with W2
    assert f(P, P, None, None, None, P, -1, 16, 4096, 0, 8, None, 0, None) == ERR["shape"]
    assert f(P, P, None, None, None, P, 1, 16, 0, 0, 8, None, 0, None) == ERR["shape"]
    assert f(P, P, None, None, None, P, 1, 16, 4100, 0, 8, None, 0, None) == ERR["unsupported"]
    assert f(P, P, None, P, None, P, 1, 16, 4096, 500, 8, None, 0, None) == ERR["unsupported"]
    assert f(P, P, None, P, None, P, 1, 16, 4096, 768, 8, None, 0, None) == ERR["unsupported"]
    assert f(P, P, None, None, None, P, 1, 16, 4096, 0, 17, None, 0, None) == ERR["unsupported"]
    assert f(P + 2, P, None, None, None, P, 1, 16, 4096, 0, 8, None, 0, None) == ERR["align"]
    assert f(P, P, P + 4, None, None, P, 1, 16, 4096, 0, 8, None, 0, None) == ERR["align"]
    assert f(P, P, None, P, None, P, 1, 16, 4096, 512, 8, None, 0, None) == ERR["workspace"]
    assert f(P, P, None, P, None, P, 1, 16, 4096, 512, 8, 0x20000, 100, None) == ERR["workspace"]
    # empty input is a no-op that needs no pointers
    assert f(None, None, None, None, None, None, 1, 0, 4096, 0, 8, None, 0, None) == 0


def test_prepared_scorer_argument_errors(lib):
    f = lib.kvzap_prepare_scorer
    need = lib.kvzap_workspace_bytes(binding.CALL_SCORE, 1, 131072, 4096, 512, 8)
    Q = 0x4000000
    assert f(None, 4096, 512, Q, need, None) == ERR["null"]
    assert f(P, 4096, 512, None, need, None) == ERR["null"]
    assert f(P, 4096, 0, Q, need, None) == ERR["shape"]          # nothing to prepare
    assert f(P, 4096, 500, Q, need, None) == ERR["unsupported"]
    assert f(P, 4096, 512, Q + 16, need, None) == ERR["align"]
    assert f(P, 4096, 512, Q, need - 1, None) == ERR["workspace"]
    assert f(P, 4096, 512, P + 4096, need, None) == ERR["shape"]  # overlaps W1
    g = lib.kvzap_score_prepared
    assert g(P, Q, None, P, None, P, 1, 16, 4096, 0, 8, None) == ERR["shape"]
    assert g(P, None, None, P, None, P, 1, 16, 4096, 512, 8, None) == ERR["null"]
    assert g(P, Q, None, None, None, P, 1, 16, 4096, 512, 8, None) == ERR["null"]
    assert g(P, Q + 16, None, P, None, P, 1, 16, 4096, 512, 8, None) == ERR["align"]
    assert g(P, Q, None, P, None, P, 1, 16, 4096, 768, 8, None) == ERR["unsupported"]
    assert g(None, None, None, None, None, None, 1, 0, 4096, 512, 8, None) == 0   # empty input


def test_mask_argument_errors(lib):
    f = lib.kvzap_mask
    ws = lib.kvzap_workspace_bytes(binding.CALL_MASK, 1, 1024, 0, 0, 8)
    ok = dict(scores=P, tau=0.0, window=128, seq=None, B=1, H=8, T=1024, idx=P, lens=P, offs=P,
              ws=0x20000, wsb=ws, stream=None)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["scores"], a["tau"], a["window"], a["seq"], a["B"], a["H"], a["T"], a["idx"],
                 a["lens"], a["offs"], a["ws"], a["wsb"], a["stream"])

    assert call(scores=None) == ERR["null"]
    assert call(idx=None) == ERR["null"]
    assert call(window=-1) == ERR["shape"]
    assert call(T=0) == ERR["shape"]
    assert call(tau=float("nan")) == ERR["shape"]
    assert call(B=10000, H=8) == ERR["unsupported"]
    assert call(T=2 ** 31 - 1) == ERR["unsupported"]          # positions are 32-bit with headroom
    assert call(scores=P + 4) == ERR["align"]
    assert call(ws=None) == ERR["workspace"]
    assert call(wsb=ws - 1) == ERR["workspace"]
    assert call(ws=0x20010) == ERR["workspace"]


def test_compact_argument_errors(lib):
    f = lib.kvzap_compact
    big = 1 << 40
    ok = [P, P + (1 << 30), P, P, P, big, big + (1 << 30), 8192, 1, 8, 1024, 128, None]

    def call(i=None, v=None):
        a = list(ok)
        if i is not None:
            a[i] = v
        return f(*a)

    assert call(0, None) == ERR["null"]
    assert call(5, None) == ERR["null"]
    assert call(11, 100) == ERR["unsupported"]
    assert call(11, 1024) == ERR["unsupported"]
    assert call(11, 0) == ERR["shape"]
    assert call(7, -1) == ERR["shape"]
    assert call(1, P + 6) == ERR["align"]
    assert call(5, P) == ERR["shape"]                 # K_out aliases K
    assert call(6, big) == ERR["shape"]               # V_out aliases K_out


def test_compress_argument_errors(lib):
    # the one-call form refuses whatever any of its three stages refuses, before launching
    f = lib.kvzap_compress
    q = lib.kvzap_workspace_bytes
    ws = q(binding.CALL_COMPRESS, 1, 1024, 4096, 512, 8)
    mc = q(binding.CALL_MASK_COMPACT, 1, 1024, 0, 0, 8)
    assert mc == q(binding.CALL_MASK, 1, 1024, 0, 0, 8) and mc % 256 == 0
    assert ws == max(q(binding.CALL_SCORE, 1, 1024, 4096, 512, 8), mc)
    assert q(binding.CALL_COMPRESS, 1, 1024, 4096, 0, 8) == mc
    big = 1 << 40
    ok = dict(hidden=P, W1=P, b1=None, W2=P, b2=None, K=P + (1 << 30), V=P + (2 << 30), tau=0.0,
              window=128, seq=None, scores=P, idx=P, lens=P, offs=P, Ko=big, Vo=big + (1 << 30),
              cap=8192, B=1, T=1024, Dh=4096, M=512, H=8, D=128, ws=0x20000, wsb=ws, stream=None)
    order = list(ok)

    def call(**kw):
        a = dict(ok, **kw)
        return f(*[a[k] for k in order])

    assert call(hidden=None) == ERR["null"]
    assert call(K=None) == ERR["null"]
    assert call(idx=None) == ERR["null"]
    assert call(W2=None) == ERR["null"]
    assert call(T=0) == ERR["shape"]
    assert call(tau=float("nan")) == ERR["shape"]
    assert call(M=500) == ERR["unsupported"]
    assert call(D=100) == ERR["unsupported"]
    assert call(V=P + 6) == ERR["align"]
    assert call(Ko=P + (1 << 30)) == ERR["shape"]      # K_out aliases K
    assert call(wsb=ws - 1) == ERR["workspace"]
    assert call(ws=None) == ERR["workspace"]


def test_mask_compact_argument_errors(lib):
    # the fused threshold + gather refuses whatever kvzap_mask or kvzap_compact refuses
    f = lib.kvzap_mask_compact
    ws = lib.kvzap_workspace_bytes(binding.CALL_MASK_COMPACT, 1, 2048, 0, 0, 8)
    big = 1 << 40
    ok = dict(scores=P, tau=0.0, window=128, seq=None, K=P + (1 << 30), V=P + (2 << 30), idx=P,
              lens=P, offs=P, Ko=big, Vo=big + (1 << 30), cap=16384, B=1, H=8, T=2048, D=128,
              ws=0x20000, wsb=ws, stream=None)
    order = list(ok)

    def call(**kw):
        a = dict(ok, **kw)
        return f(*[a[k] for k in order])

    assert call(scores=None) == ERR["null"]
    assert call(V=None) == ERR["null"]
    assert call(Ko=None) == ERR["null"]
    assert call(window=-1) == ERR["shape"]
    assert call(tau=float("nan")) == ERR["shape"]
    assert call(D=4) == ERR["unsupported"]
    assert call(B=8192) == ERR["unsupported"]
    assert call(K=P + (1 << 30) + 2) == ERR["align"]
    assert call(Vo=big) == ERR["shape"]                # V_out aliases K_out
    assert call(wsb=ws - 1) == ERR["workspace"]
    assert call(ws=None) == ERR["workspace"]
    assert call(ws=0x20010) == ERR["workspace"]


def test_decode_argument_errors(lib):
    f = lib.kvzap_decode_evict
    ws = lib.kvzap_workspace_bytes(binding.CALL_DECODE_EVICT, 4, 1, 4096, 512, 8)
    ok = [P, P, None, P, None, 4096, 512, P, P, P, P, P, P, P, P, P, P, P, P,
          0.0, 128, 4, 8, 128, None, 0x20000, ws, None]

    def call(i=None, v=None):
        a = list(ok)
        if i is not None:
            a[i] = v
        return f(*a)

    assert call(0, None) == ERR["null"]
    assert call(14, None) == ERR["null"]              # ring required when window > 0
    assert call(3, None) == ERR["null"]               # MLP needs W2
    assert call(20, -1) == ERR["shape"]
    assert call(6, 100) == ERR["unsupported"]
    assert call(23, 12) == ERR["unsupported"]
    assert call(9, P + 8) == ERR["align"]
    assert call(25, None) == ERR["workspace"]
    assert call(26, ws - 1) == ERR["workspace"]


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        binding.lib()
