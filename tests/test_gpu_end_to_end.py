"""End-to-end parity of score -> mask -> compact on the benchmark configurations
the oracle finishes in seconds, with the exclusion band around tau."""
import numpy as np
import pytest
import torch

from oracle import kvzap_oracle as O
from paper_2601_07891_amd import binding, synth
from tests import parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _pipeline(wl, hid, K, V, w, tau, seq_lens=None):
    d = {k: (None if v is None else v.to(DEV)) for k, v in w.items()}
    scores = binding.kvzap_score(hid.to(DEV), d["W1"], d["b1"], d["W2"], d["b2"])
    sl = None if seq_lens is None else torch.tensor(seq_lens, dtype=torch.int32, device=DEV)
    idx, n, off = binding.kvzap_mask(scores, tau, wl.window, sl)
    Ko, Vo = binding.kvzap_compact(K.to(DEV), V.to(DEV), idx, n, off)
    torch.cuda.synchronize()
    return scores, idx, n, off, Ko, Vo


def _check(wl, seq_lens=None):
    w = synth.make_weights(wl); hid = synth.make_hidden(wl); K, V = synth.make_kv(wl)
    S, _ = O.compress(synth.bits(hid), synth.bits(K), synth.bits(V), synth.oracle_weights(w),
                      0.0, wl.window, seq_lens)
    tau = O.tau_at_keep_fraction(S, wl.window, wl.keep_fraction, seq_lens)
    scores, idx, n, off, Ko, Vo = _pipeline(wl, hid, K, V, w, tau, seq_lens)
    parity.assert_scores_close(scores, S)
    ref, namb = parity.assert_prune_matches(idx, n, off, Ko, Vo, K, V, S, tau, wl.window,
                                            seq_lens, band=parity.BAND)
    total = wl.B * wl.H * wl.T
    assert namb < 0.03 * total                      # the band excludes a few per cent at most
    kept = int(parity.to_np(off)[-1])
    assert abs(kept - int(ref.offsets[-1])) <= namb
    # with the oracle's fp32-rounded scores injected instead, everything is exact
    inj = torch.from_numpy(S.astype(np.float32))
    idx2, n2, off2 = binding.kvzap_mask(inj.to(DEV), tau, wl.window,
                                        None if seq_lens is None else
                                        torch.tensor(seq_lens, dtype=torch.int32, device=DEV))
    Ko2, Vo2 = binding.kvzap_compact(K.to(DEV), V.to(DEV), idx2, n2, off2)
    torch.cuda.synchronize()
    parity.assert_prune_matches(idx2, n2, off2, Ko2, Vo2, K, V, inj.double().numpy(), tau, wl.window,
                                seq_lens)
    return tau


def test_config1_linear_t1k():
    _check(synth.CONFIGS["c1_t1k_linear"])


def test_config2_mlp_t32k():
    _check(synth.CONFIGS["c2_llama8b_32k_mlp"])


def test_config3_shape_reduced_skewed():
    # config 3's recipe (log-normal token scale, 25 % keep) at a length the oracle does quickly
    _check(synth.with_size(synth.CONFIGS["c3_qwen8b_128k_mlp"], L=1, T=6000 + 37))


def test_config4_shape_reduced_batched():
    for name in ("c4_qwen32b_4x64k_mlp", "c4_qwen32b_4x64k_linear"):
        _check(synth.with_size(synth.CONFIGS[name], L=1, T=1500))


def test_batched_right_padded():
    wl = synth.with_size(synth.CONFIGS["c2_llama8b_32k_mlp"], B=3, T=700)
    _check(wl, seq_lens=[700, 401, 128])


@pytest.mark.parametrize("name,T,padded", [("c1_t1k_linear", 1024, False),
                                           ("c2_llama8b_32k_mlp", 5000 + 19, False),
                                           ("c4_qwen32b_4x64k_linear", 700, True)])
def test_compress_is_the_three_calls(name, T, padded):
    # Algorithm 1 through the one-call entry point: bit-identical to score, mask, compact
    wl = synth.with_size(synth.CONFIGS[name], L=1, T=T)
    if padded:
        wl = synth.with_size(wl, B=3)
    w = synth.make_weights(wl); hid = synth.make_hidden(wl); K, V = synth.make_kv(wl)
    seq_lens = [T, T // 2 + 1, 1][:wl.B] if padded else None
    sl = None if seq_lens is None else torch.tensor(seq_lens, dtype=torch.int32, device=DEV)
    d = {k: (None if v is None else v.to(DEV)) for k, v in w.items()}
    tau = float(binding.kvzap_score(hid.to(DEV), d["W1"], d["b1"], d["W2"], d["b2"]).median())
    want = _pipeline(wl, hid, K, V, w, tau, seq_lens)
    got = binding.kvzap_compress(hid.to(DEV), d["W1"], d["b1"], d["W2"], d["b2"], K.to(DEV),
                                 V.to(DEV), tau, wl.window, sl)
    torch.cuda.synchronize()
    kept = int(parity.to_np(want[3])[-1])
    assert 0 < kept < wl.B * wl.H * wl.T
    assert torch.equal(got[0], want[0])
    assert torch.equal(got[2], want[2]) and torch.equal(got[3], want[3])
    assert torch.equal(got[1][:kept], want[1][:kept])
    assert torch.equal(got[4][:kept].view(torch.int16), want[4][:kept].view(torch.int16))
    assert torch.equal(got[5][:kept].view(torch.int16), want[5][:kept].view(torch.int16))
