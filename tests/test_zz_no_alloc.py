"""The allocation-free entry point kvzap_mask_static against kvzap_mask, through the C ABI:
two calls in a row on the library's built-in scratch, the second on a smaller input, every
output equal bit for bit (and therefore equal to the oracle's, which kvzap_mask is checked
against in test_gpu_mask_compact.py); plus the oracle directly on the second call."""
import numpy as np
import pytest
import torch

from oracle import kvzap_oracle as O
from paper_2601_07891_amd import binding, synth
from tests import parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(B, H, T, window, tau, seed, seq_lens=None):
    scores = synth.make_scores(B, H, T, seed=seed, ties=True)
    s = scores.to(DEV)
    sl = None if seq_lens is None else torch.tensor(seq_lens, dtype=torch.int32, device=DEV)
    want = binding.kvzap_mask(s, tau, window, sl)
    torch.cuda.synchronize()
    # poisoned outputs, so that an entry the call leaves unwritten shows
    idx = torch.full((B * H * T,), -3, dtype=torch.int32, device=DEV)
    n = torch.full((B, H), -3, dtype=torch.int32, device=DEV)
    off = torch.full((B * H + 1,), -3, dtype=torch.int64, device=DEV)
    lib = binding.lib()
    rc = lib.kvzap_mask_static(s.data_ptr(), float(tau), int(window),
                               None if sl is None else sl.data_ptr(), B, H, T, idx.data_ptr(),
                               n.data_ptr(), off.data_ptr(),
                               torch.cuda.current_stream().cuda_stream or None)
    assert rc == 0, lib.kvzap_status_string(rc).decode()
    torch.cuda.synchronize()
    tot = int(want[2][-1])
    assert torch.equal(n, want[1]) and torch.equal(off, want[2])
    assert torch.equal(idx[:tot], want[0][:tot])
    assert (idx[tot:] == -3).all()
    return scores, (idx, n, off)


def test_two_calls_second_smaller():
    # first call: several chunks per head, ragged tail, padded batch; the scratch then holds
    # its counts and prefixes when the second, smaller call (fewer heads, fewer chunks) runs
    _both(3, 8, 40000 + 77, 128, 0.2, seed=41, seq_lens=[40077, 1025, 0])
    scores, (idx, n, off) = _both(1, 5, 2500, 16, -0.3, seed=42)
    parity.assert_prune_matches(idx, n, off, None, None, None, None, scores.double().numpy(),
                                -0.3, 16)
    # and a larger one again, through the path with the separate scan kernel (> 8192 chunks)
    _both(64, 16, 9000, 128, 0.3, seed=43)
    _both(1, 1, 1, 0, 0.0, seed=44)


def test_size_limit_is_an_error_and_writes_nothing():
    B, H, T = 1, 8, 1024
    s = synth.make_scores(B, H, T, seed=45).to(DEV)
    idx = torch.full((B * H * T,), -3, dtype=torch.int32, device=DEV)
    n = torch.full((B, H), -3, dtype=torch.int32, device=DEV)
    off = torch.full((B * H + 1,), -3, dtype=torch.int64, device=DEV)
    lib = binding.lib()
    # the same pointers with a T beyond the limit: rejected on the host, nothing launched
    rc = lib.kvzap_mask_static(s.data_ptr(), 0.0, 128, None, B, H, 8193 * 1024, idx.data_ptr(),
                               n.data_ptr(), off.data_ptr(), None)
    assert rc == -8
    torch.cuda.synchronize()
    assert (idx == -3).all() and (n == -3).all() and (off == -3).all()
    # the Python wrapper allocates nothing either and raises on a status
    binding.kvzap_mask_static(s, 0.0, 128, None, idx, n, off)
    want = binding.kvzap_mask(s, 0.0, 128)
    torch.cuda.synchronize()
    assert torch.equal(n, want[1]) and torch.equal(off, want[2])
    with pytest.raises(binding.KvzapError):
        binding.kvzap_mask_static(s, float("nan"), 128, None, idx, n, off)
