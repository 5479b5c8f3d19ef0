"""GPU parity at the limits of the launch geometry: the largest number of (sequence, head)
rows a call accepts (65535, the grid's second dimension), rows of millions of tokens
(64-bit offsets, blocks that walk several tiles), and the first shape past each limit is
refused on the host."""
import numpy as np
import pytest
import torch

from oracle import kvzap_oracle as O
from paper_2601_07891_amd import binding, synth
from tests import parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
MAX_BH = 65535


def _flat_idx(ref, B, H):
    return np.concatenate([ref.idx[b][h] for b in range(B) for h in range(H)]) if B else np.zeros(0, np.int64)


def test_mask_and_compact_with_65535_heads():
    B, H, T, D, w = 4369, 15, 40, 8, 3                       # B * H = 65535
    rng = np.random.default_rng(0)
    S = rng.standard_normal((B, H, T)).astype(np.float32)
    seq_lens = rng.integers(0, T + 1, B).astype(np.int32)
    K = torch.from_numpy(rng.integers(0, 1 << 16, (B, H, T, D), dtype=np.uint16).view(np.int16)).view(torch.bfloat16)
    V = torch.from_numpy(rng.integers(0, 1 << 16, (B, H, T, D), dtype=np.uint16).view(np.int16)).view(torch.bfloat16)
    Sd = torch.from_numpy(S).to(DEV)
    idx, n, off = binding.kvzap_mask(Sd, 0.25, w, torch.from_numpy(seq_lens).to(DEV))
    Ko, Vo = binding.kvzap_compact(K.to(DEV), V.to(DEV), idx, n, off)
    torch.cuda.synchronize()
    ref = O.prune(S.astype(np.float64), 0.25, w, synth.bits(K), synth.bits(V), seq_lens)
    total = int(ref.offsets[-1])
    np.testing.assert_array_equal(parity.to_np(n), ref.lengths)
    np.testing.assert_array_equal(parity.to_np(off), ref.offsets)
    np.testing.assert_array_equal(parity.to_np(idx)[:total], _flat_idx(ref, B, H))
    np.testing.assert_array_equal(parity.to_np(Ko)[:total], ref.K_out)
    np.testing.assert_array_equal(parity.to_np(Vo)[:total], ref.V_out)
    # one head more is refused before anything is launched
    S2 = torch.zeros((4096, 16, 4), dtype=torch.float32, device=DEV)
    with pytest.raises(binding.KvzapError) as e:
        binding.kvzap_mask(S2, 0.0, 1)
    assert e.value.status == -4


def test_rows_of_two_million_tokens():
    # one row of 2^21 + 3 scores: thousands of mask chunks, top-k blocks that walk several
    # tiles, offsets beyond what 16 heads of 131072 would reach
    B, H, T, D, w = 1, 2, (1 << 21) + 3, 8, 128
    rng = np.random.default_rng(1)
    S = (rng.standard_normal((B, H, T)) * np.array([1.0, 3.0])[None, :, None]).astype(np.float32)
    Sd = torch.from_numpy(S).to(DEV)
    K = torch.from_numpy(rng.integers(0, 1 << 16, (B, H, T, D), dtype=np.uint16).view(np.int16)).view(torch.bfloat16)
    V = torch.from_numpy(rng.integers(0, 1 << 16, (B, H, T, D), dtype=np.uint16).view(np.int16)).view(torch.bfloat16)
    S64 = S.astype(np.float64)
    for per_layer, k in ((False, 700001), (True, 1234567)):
        tau = binding.kvzap_topk_threshold(Sd, w, k, per_layer)
        ref_tau = O.topk_threshold(S64, w, k, per_layer)
        assert np.array_equal(tau.double().cpu().numpy(), ref_tau)
    idx, n, off = binding.kvzap_mask_per_head(Sd, tau, w)
    Ko, Vo = binding.kvzap_compact(K.to(DEV), V.to(DEV), idx, n, off)
    torch.cuda.synchronize()
    ref = O.prune(S64, ref_tau, w, synth.bits(K), synth.bits(V))
    total = int(ref.offsets[-1])
    assert 1234567 + 2 * w <= total <= 1234567 + 2 * w + 4        # ties with the k-th largest are all kept
    np.testing.assert_array_equal(parity.to_np(off), ref.offsets)
    np.testing.assert_array_equal(parity.to_np(idx)[:total], _flat_idx(ref, B, H))
    np.testing.assert_array_equal(parity.to_np(Ko)[:total], ref.K_out)
    np.testing.assert_array_equal(parity.to_np(Vo)[:total], ref.V_out)


def test_decode_attention_and_pages_with_65535_heads():
    B, H, D, P = 4369, 15, 128, 16
    rng = np.random.default_rng(2)
    lengths = rng.integers(1, 6, (B, H)).astype(np.int32)
    # page assignment: exact against the oracle
    need = int(sum(O.pages_needed(int(x), P) for x in lengths.reshape(-1)))
    free = rng.permutation(need + 7).astype(np.int32)
    table, res = binding.kvzap_assign_pages(torch.from_numpy(lengths).to(DEV), P,
                                            torch.from_numpy(free).to(DEV), 2)
    torch.cuda.synchronize()
    ref_table, used, ok = O.assign_pages(lengths, P, free, 2)
    assert ok and res[:2].tolist() == [used, 0]
    np.testing.assert_array_equal(parity.to_np(table), ref_table)
    # attention over 65535 tiny heads (one query head each), no window
    off = np.zeros(B * H, np.int64); off[1:] = np.cumsum(lengths.reshape(-1).astype(np.int64))[:-1]
    total = int(lengths.sum())
    q, Kg, Vg, _, _ = synth.make_attend_inputs(B, H, H, D, total, 0, 3, DEV)
    out = binding.kvzap_attend_decode(q, Kg, Vg, torch.from_numpy(off).to(DEV),
                                      torch.from_numpy(lengths).to(DEV), None, None, None, 0, 8, D ** -0.5)
    torch.cuda.synchronize()
    Kh, Vh = synth.f64(Kg), synth.f64(Vg)
    # sampled sequences (the oracle loops in Python), first, last and random ones
    for b in [0, B - 1] + rng.integers(0, B, 40).tolist():
        caches = [[(Kh[off[b * H + h]:off[b * H + h] + lengths[b, h]],
                    Vh[off[b * H + h]:off[b * H + h] + lengths[b, h]]) for h in range(H)]]
        want = O.attend_decode(synth.f64(q[b:b + 1]), caches, D ** -0.5)
        assert np.abs(out[b:b + 1].double().cpu().numpy() - want).max() <= 2.0 ** -7 * 6.0
