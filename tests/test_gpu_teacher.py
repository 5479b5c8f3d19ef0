"""GPU parity of kvzap_teacher_scores (KVzip Eq. 1 / KVzip+ Eq. 3, log space) against the
float64 oracle.

Tolerance: the logits are bf16 x bf16 products (exact in fp32) accumulated over D = 128 in
fp32 (relative 1e-5 of sum |terms|, i.e. a few 1e-4 absolute on logits of size ~10), the
row statistics sum up to ~1e4 exponentials in fp32 (1e-4 relative -> 1e-4 in the log).  The
test bound on the log score is 2e-3 + 1e-4 * |ref|."""
import numpy as np
import pytest
import torch

from oracle import kvzap_oracle as O
from paper_2601_07891_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
D = 128


def _inputs(H, G, T, instr, Tq, seed, gain=1.0):
    g = torch.Generator().manual_seed(seed)
    Tk = T + instr + Tq
    q = (torch.randn((H * G, Tq, D), generator=g) * gain).bfloat16()
    k = torch.randn((H, Tk, D), generator=g).bfloat16()
    vn = torch.rand((H, T), generator=g) * 3.0 + 0.1
    hn = torch.rand((Tq,), generator=g) * 5.0 + 0.5
    return q, k, vn, hn


def _check(H, G, T, instr, Tq, seed, gain=1.0, norms=True, scale=None):
    q, k, vn, hn = _inputs(H, G, T, instr, Tq, seed, gain)
    scale = D ** -0.5 if scale is None else scale
    got = binding.kvzap_teacher_scores(q.to(DEV), k.to(DEV), T, scale,
                                       vn.to(DEV) if norms else None, hn.to(DEV) if norms else None)
    torch.cuda.synchronize()
    ref = O.teacher_log_scores(synth.f64(q), synth.f64(k), scale, T,
                               vn.double().numpy() if norms else None,
                               hn.double().numpy() if norms else None)
    err = np.abs(got.double().cpu().numpy() - ref)
    bound = 2e-3 + 1e-4 * np.abs(ref)
    assert (err <= bound).all(), f"max err {err.max():.3e} (ref range {ref.min():.2f}..{ref.max():.2f})"
    return ref


def test_small_ragged_shapes():
    for (T, instr, Tq) in [(1, 0, 1), (5, 3, 5), (31, 1, 33), (32, 0, 32), (33, 7, 31), (130, 9, 127)]:
        _check(H=2, G=2, T=T, instr=instr, Tq=Tq, seed=T + Tq)


def test_several_tiles_splits_and_groups():
    _check(H=2, G=4, T=700, instr=25, Tq=700, seed=1)
    _check(H=3, G=1, T=520, instr=11, Tq=300, seed=2)          # fewer repeated tokens than prompt
    _check(H=1, G=8, T=260, instr=40, Tq=513, seed=3)


def test_the_benchmark_shape():
    # bench.py's --stage teacher shape: an 8192-token prompt, 32 instruction tokens, the prompt
    # repeated, 8 KV heads x 4 query heads -- query splits and the longest-block-first order in
    # play.  The oracle recomputes the first and the last KV head (a few seconds each).
    H, G, T, instr = 8, 4, 8192, 32
    q, k, vn, hn = _inputs(H, G, T, instr, T, seed=11)
    scale = D ** -0.5
    got = binding.kvzap_teacher_scores(q.to(DEV), k.to(DEV), T, scale, vn.to(DEV), hn.to(DEV))
    torch.cuda.synchronize()
    got = got.double().cpu().numpy()
    assert np.isfinite(got).all()
    for h in (0, H - 1):
        ref = O.teacher_log_scores(synth.f64(q[h * G:(h + 1) * G]), synth.f64(k[h:h + 1]), scale, T,
                                   vn[h:h + 1].double().numpy(), hn.double().numpy())
        err = np.abs(got[h:h + 1] - ref)
        assert (err <= 2e-3 + 1e-4 * np.abs(ref)).all(), (h, err.max())


def test_kvzip_without_norms_is_the_unit_norm_case():
    ref = _check(H=2, G=2, T=300, instr=10, Tq=300, seed=4, norms=False)
    assert (ref <= 1e-9).all()                                   # attention weights are <= 1


def test_peaked_attention_and_the_copy_pattern():
    _check(H=2, G=2, T=400, instr=16, Tq=400, seed=5, gain=6.0)   # logits ~ N(0, 36)
    # copy pattern: the repeated token's query is a multiple of its original key
    g = torch.Generator().manual_seed(6)
    T, instr = 300, 12
    k = torch.randn((1, T + instr + T, D), generator=g).bfloat16()
    q = (k[:, :T].float() * 3.0).bfloat16().repeat(2, 1, 1)       # two query heads, same pattern
    got = binding.kvzap_teacher_scores(q.to(DEV), k.to(DEV), T, 1.0)
    ref = O.teacher_log_scores(synth.f64(q), synth.f64(k), 1.0, T)
    assert (np.exp(ref) > 0.99).all()
    assert np.abs(got.double().cpu().numpy() - ref).max() <= 2e-3


def test_prompt_shorter_than_the_scored_prefix_and_empty():
    # only the first T positions are scored; T may be smaller than P0
    q, k, vn, hn = _inputs(2, 2, 200, 10, 200, 7)
    got = binding.kvzap_teacher_scores(q.to(DEV), k.to(DEV), 77, D ** -0.5, vn[:, :77].contiguous().to(DEV), hn.to(DEV))
    ref = O.teacher_log_scores(synth.f64(q), synth.f64(k), D ** -0.5, 77, vn[:, :77].double().numpy(),
                               hn.double().numpy())
    assert np.abs(got.double().cpu().numpy() - ref).max() <= 3e-3
    empty = binding.kvzap_teacher_scores(q.to(DEV), k.to(DEV), 0, D ** -0.5)
    assert tuple(empty.shape) == (2, 0)


def test_rejects_bad_arguments():
    L = binding.lib()
    q = torch.zeros((4, 8, D), dtype=torch.bfloat16, device=DEV)
    k = torch.zeros((2, 20, D), dtype=torch.bfloat16, device=DEV)
    out = torch.zeros((2, 8), dtype=torch.float32, device=DEV)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)
    call = lambda **kw: L.kvzap_teacher_scores(
        q.data_ptr(), k.data_ptr(), None, None, 0.1, out.data_ptr(), kw.get("H", 2), kw.get("HQ", 4),
        8, kw.get("Tk", 20), kw.get("T", 8), kw.get("D", D), ws.data_ptr(), kw.get("ws", ws.numel()), None)
    assert call() == 0
    assert call(T=13) == -2          # scored prefix longer than what precedes the repeated prompt
    assert call(HQ=3) == -2
    assert call(Tk=7) == -2          # fewer keys than queries
    assert call(D=64) == -4
    assert call(ws=8) == -6
    torch.cuda.synchronize()
