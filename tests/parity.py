"""Comparison protocol between the HIP path and the CPU oracle.

Scores: |gpu - oracle| <= 1e-2 * max(|oracle|, 1) elementwise (bf16 inputs,
fp32 accumulation against float64).
Kept sets: bit-exact, except that non-window tokens whose ORACLE score lies
within 1e-2 of tau may fall on either side; lengths and offsets must be exactly
consistent with the GPU's own index lists; gathered bytes must be exact copies
of the rows the GPU's indices name, and identical to the oracle's wherever no
ambiguous token exists (score injection: always).
"""
import numpy as np
import torch

from oracle import kvzap_oracle as O

SCORE_RTOL = 1e-2
BAND = 1e-2


def to_np(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def assert_scores_close(gpu_scores: torch.Tensor, oracle_scores: np.ndarray):
    g = to_np(gpu_scores).astype(np.float64)
    assert g.shape == oracle_scores.shape
    err = np.abs(g - oracle_scores)
    bound = SCORE_RTOL * np.maximum(np.abs(oracle_scores), 1.0)
    worst = float((err / bound).max()) if err.size else 0.0
    assert worst <= 1.0, f"score error {worst:.3f}x the tolerance (max abs {err.max():.3e})"
    return float(err.max()) if err.size else 0.0


def assert_prune_matches(keep_idx, lengths, offsets, K_out, V_out, K, V,
                         oracle_scores: np.ndarray, tau: float, window: int,
                         seq_lens=None, band: float = 0.0):
    """oracle_scores [B,H,T] float64; band = 0 demands exact equality."""
    B, H, T = oracle_scores.shape
    idx = to_np(keep_idx); n = to_np(lengths).reshape(-1); off = to_np(offsets)
    ref = O.prune(oracle_scores, tau, window, None, None, seq_lens)
    # self-consistency of the bookkeeping, exact
    assert off[0] == 0
    np.testing.assert_array_equal(np.diff(off), n.astype(np.int64))
    Kb = to_np(K) if K is not None else None
    Vb = to_np(V) if V is not None else None
    Ko = to_np(K_out) if K_out is not None else None
    Vo = to_np(V_out) if V_out is not None else None
    n_ambiguous = 0
    for b in range(B):
        Tb = T if seq_lens is None else int(seq_lens[b])
        for h in range(H):
            bh = b * H + h
            got = idx[off[bh]:off[bh] + n[bh]]
            want = ref.idx[b][h]
            if band == 0.0:
                np.testing.assert_array_equal(got, want)
            else:
                assert (np.diff(got) > 0).all() and (got.size == 0 or (got[0] >= 0 and got[-1] < Tb))
                s = oracle_scores[b, h]
                amb = np.zeros(T, dtype=bool)
                amb[:max(Tb - window, 0)] = np.abs(s[:max(Tb - window, 0)] - tau) < band
                n_ambiguous += int(amb.sum())
                np.testing.assert_array_equal(got[~amb[got]], want[~amb[want]])
            if Ko is not None:
                np.testing.assert_array_equal(Ko[off[bh]:off[bh] + n[bh]], Kb[b, h][got])
                np.testing.assert_array_equal(Vo[off[bh]:off[bh] + n[bh]], Vb[b, h][got])
    if band == 0.0:
        np.testing.assert_array_equal(n, ref.lengths.reshape(-1))
        np.testing.assert_array_equal(off, ref.offsets)
    return ref, n_ambiguous
