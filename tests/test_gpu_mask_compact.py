"""GPU parity of kvzap_mask + kvzap_compact against the oracle with INJECTED
scores: indices, lengths, offsets and every gathered byte must be identical, no
exclusion band."""
import math

import numpy as np
import pytest
import torch

from oracle import kvzap_oracle as O
from paper_2601_07891_amd import binding, synth
from tests import parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _kv(B, H, T, D, seed):
    g = torch.Generator().manual_seed(seed)
    # arbitrary bit patterns (NaN payloads, -0, subnormals): the gather is a byte copy
    K = torch.randint(-32768, 32768, (B, H, T, D), generator=g, dtype=torch.int16).view(torch.bfloat16)
    V = torch.randint(-32768, 32768, (B, H, T, D), generator=g, dtype=torch.int16).view(torch.bfloat16)
    return K, V


def _run(scores, tau, window, K, V, seq_lens=None, cap_rows=None):
    s = scores.to(DEV)
    sl = None if seq_lens is None else torch.tensor(seq_lens, dtype=torch.int32, device=DEV)
    idx, n, off = binding.kvzap_mask(s, tau, window, sl)
    Kd, Vd = K.to(DEV), V.to(DEV)
    Ko, Vo = binding.kvzap_compact(Kd, Vd, idx, n, off, cap_rows=cap_rows)
    torch.cuda.synchronize()
    return idx, n, off, Ko, Vo


CASES = [
    # B, H, T, D, window, tau
    (1, 8, 1024, 128, 128, 0.0),
    (1, 8, 1, 128, 128, 0.0),
    (1, 1, 7, 128, 0, 0.3),
    (2, 3, 1000, 128, 17, -0.5),          # T % 4 == 0, ragged chunk tail
    (2, 8, 1027, 128, 128, 0.2),          # T % 4 != 0 -> scalar loads, several chunks
    (3, 8, 5000, 64, 128, 1.0),
    (1, 2, 3333, 256, 4000, 0.0),         # window >= T
    (1, 16, 2049, 8, 1, 0.0),             # smallest row, H = 16
    (1, 8, 4100, 48, 128, 0.0),           # D not a power of two -> generic path
    (4, 8, 16384, 128, 128, 0.67),
    (64, 16, 9000, 8, 128, 0.3),          # > 8192 chunks: the path with the separate scan kernel
    (8, 8, 131072, 8, 128, 1.0),          # exactly 8192 chunks: the largest fused case
]


@pytest.mark.parametrize("B,H,T,D,w,tau", CASES)
def test_injected_scores_exact(B, H, T, D, w, tau):
    scores = synth.make_scores(B, H, T, seed=B * 1000 + T)
    K, V = _kv(B, H, T, D, T)
    idx, n, off, Ko, Vo = _run(scores, tau, w, K, V)
    parity.assert_prune_matches(idx, n, off, Ko, Vo, K, V, scores.double().numpy(), tau, w)


@pytest.mark.parametrize("B,H,T,D,w,tau", CASES)
def test_mask_compact_in_one_call(B, H, T, D, w, tau):
    # threshold + gather in one library call against the oracle, no band, and against the
    # separate calls
    scores = synth.make_scores(B, H, T, seed=B * 1000 + T + 1, ties=True)
    K, V = _kv(B, H, T, D, T + 1)
    s, Kd, Vd = scores.to(DEV), K.to(DEV), V.to(DEV)
    idx, n, off, Ko, Vo = binding.kvzap_mask_compact(s, tau, w, Kd, Vd)
    torch.cuda.synchronize()
    parity.assert_prune_matches(idx, n, off, Ko, Vo, K, V, scores.double().numpy(), tau, w)
    i2, n2, o2 = binding.kvzap_mask(s, tau, w)
    assert torch.equal(n, n2) and torch.equal(off, o2)
    tot = int(off[-1])
    assert torch.equal(idx[:tot], i2[:tot])


def test_mask_compact_in_one_call_padded_and_capped():
    B, H, T, D, w, tau = 4, 8, 5000, 128, 128, 0.1
    scores = synth.make_scores(B, H, T, seed=77)
    K, V = _kv(B, H, T, D, 78)
    lens = [5000, 1025, 100, 0]
    sl = torch.tensor(lens, dtype=torch.int32, device=DEV)
    idx, n, off, Ko, Vo = binding.kvzap_mask_compact(scores.to(DEV), tau, w, K.to(DEV), V.to(DEV), sl)
    torch.cuda.synchronize()
    ref, _ = parity.assert_prune_matches(idx, n, off, Ko, Vo, K, V, scores.double().numpy(), tau, w,
                                         seq_lens=lens)
    # a capacity in the middle of a chunk: rows before it are written, nothing behind it
    total = int(off[-1]); cap = total // 2 + 3
    Kc = torch.full((total, D), 7.0, dtype=torch.bfloat16, device=DEV)
    Vc = torch.full((total, D), 7.0, dtype=torch.bfloat16, device=DEV)
    binding.kvzap_mask_compact(scores.to(DEV), tau, w, K.to(DEV), V.to(DEV), sl, None, None, None,
                               Kc, Vc, cap_rows=cap)
    torch.cuda.synchronize()
    assert torch.equal(Kc[:cap].view(torch.int16), Ko[:cap].view(torch.int16))
    assert torch.equal(Vc[:cap].view(torch.int16), Vo[:cap].view(torch.int16))
    assert (Kc[cap:] == 7.0).all() and (Vc[cap:] == 7.0).all()


@pytest.mark.parametrize("tau", [-math.inf, math.inf])
def test_tau_limits(tau):
    B, H, T, D, w = 2, 8, 3000, 128, 128
    scores = synth.make_scores(B, H, T, seed=5)
    K, V = _kv(B, H, T, D, 6)
    idx, n, off, Ko, Vo = _run(scores, tau, w, K, V)
    parity.assert_prune_matches(idx, n, off, Ko, Vo, K, V, scores.double().numpy(), tau, w)
    if tau < 0:
        assert (parity.to_np(n) == T).all()
        np.testing.assert_array_equal(parity.to_np(Ko)[:B * H * T], parity.to_np(K).reshape(-1, D))
    else:
        assert (parity.to_np(n) == w).all()


def test_ties_nan_inf_scores():
    B, H, T, D, w = 2, 4, 2500, 128, 16
    scores = synth.make_scores(B, H, T, seed=9, ties=True)
    scores[0, 0, ::7] = float("nan")
    scores[1, 2, ::11] = float("inf")
    scores[1, 3, ::13] = float("-inf")
    K, V = _kv(B, H, T, D, 1)
    for tau in (0.25, -2.0, math.inf, -math.inf):
        idx, n, off, Ko, Vo = _run(scores, tau, w, K, V)
        parity.assert_prune_matches(idx, n, off, Ko, Vo, K, V, scores.double().numpy(), tau, w)


def test_seq_lens_right_padded():
    B, H, T, D, w = 4, 8, 2100, 128, 128
    scores = synth.make_scores(B, H, T, seed=3)
    K, V = _kv(B, H, T, D, 2)
    lens = [2100, 1025, 100, 0]
    idx, n, off, Ko, Vo = _run(scores, 0.1, w, K, V, seq_lens=lens)
    parity.assert_prune_matches(idx, n, off, Ko, Vo, K, V, scores.double().numpy(), 0.1, w,
                                seq_lens=lens)
    assert (parity.to_np(n)[3] == 0).all()


@pytest.mark.parametrize("window,tau", [(128, 0.1), (0, -1.0), (5000, 0.0)])
def test_seq_lens_beyond_T_mean_T(window, tau):
    # a length above T (or below 0) names positions that do not exist: the result is the one for
    # a length of T (resp. 0), and nothing is written behind the B*H*T capacity of keep_idx
    B, H, T, D = 3, 8, 2100, 128            # T is not a multiple of the 1024-token chunk
    scores = synth.make_scores(B, H, T, seed=31)
    K, V = _kv(B, H, T, D, 32)
    given = [T + 1000, 2 ** 31 - 1, -5]
    meant = [T, T, 0]
    s = scores.to(DEV)
    sl = torch.tensor(given, dtype=torch.int32, device=DEV)
    guard = 4096
    idx_buf = torch.full((B * H * T + guard,), -7, dtype=torch.int32, device=DEV)
    idx, n, off = binding.kvzap_mask(s, tau, window, sl, idx_buf[:B * H * T])
    Ko, Vo = binding.kvzap_compact(K.to(DEV), V.to(DEV), idx, n, off)
    torch.cuda.synchronize()
    assert (idx_buf[B * H * T:] == -7).all()
    parity.assert_prune_matches(idx, n, off, Ko, Vo, K, V, scores.double().numpy(), tau, window,
                                seq_lens=meant)


def test_cap_rows_is_respected():
    B, H, T, D, w = 1, 8, 2048, 128, 128
    scores = synth.make_scores(B, H, T, seed=4)
    K, V = _kv(B, H, T, D, 3)
    s = scores.to(DEV)
    idx, n, off = binding.kvzap_mask(s, 0.0, w)
    total = int(off[-1].item())
    cap = total // 2
    Ko = torch.full((total, D), 7.0, dtype=torch.bfloat16, device=DEV)
    Vo = torch.full((total, D), 7.0, dtype=torch.bfloat16, device=DEV)
    binding.kvzap_compact(K.to(DEV), V.to(DEV), idx, n, off, Ko, Vo, cap_rows=cap)
    torch.cuda.synchronize()
    ref = O.prune(scores.double().numpy(), 0.0, w, parity.to_np(K), parity.to_np(V))
    np.testing.assert_array_equal(parity.to_np(Ko)[:cap], ref.K_out[:cap])
    assert (Ko[cap:] == 7.0).all() and (Vo[cap:] == 7.0).all()     # nothing written past cap


def test_repeatable_and_buffers_reused():
    # same call twice into poisoned buffers gives identical bytes (no stale reads, no races)
    B, H, T, D, w = 2, 8, 9000, 128, 128
    scores = synth.make_scores(B, H, T, seed=8).to(DEV)
    K, V = _kv(B, H, T, D, 8)
    Kd, Vd = K.to(DEV), V.to(DEV)
    outs = []
    for fill in (0, -1):
        idx = torch.full((B * H * T,), fill, dtype=torch.int32, device=DEV)
        n = torch.full((B, H), fill, dtype=torch.int32, device=DEV)
        off = torch.full((B * H + 1,), fill, dtype=torch.int64, device=DEV)
        binding.kvzap_mask(scores, 0.3, w, None, idx, n, off)
        Ko, Vo = binding.kvzap_compact(Kd, Vd, idx, n, off)
        torch.cuda.synchronize()
        tot = int(off[-1])
        outs.append((idx[:tot].clone(), n.clone(), off.clone(), Ko[:tot].clone(), Vo[:tot].clone()))
    for a, b in zip(*outs):
        assert torch.equal(a.view(torch.uint8) if a.dtype == torch.bfloat16 else a,
                           b.view(torch.uint8) if b.dtype == torch.bfloat16 else b)
