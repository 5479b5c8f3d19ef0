"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle cannot score 131k x 4096 x 512 in float64 inside a test budget for every
layer, so scores are checked on a sample of tokens it computes one by one (tile
boundaries, the ragged tail, the window edge and random positions); mask and compact
are checked in full: the oracle prunes with the GPU's own fp32 scores injected, so
indices, lengths, offsets and all gathered bytes must match exactly.  On the sampled
tokens the keep decision must also agree with the float64 oracle outside the band."""
import numpy as np
import pytest
import torch

from oracle import kvzap_oracle as O
from paper_2601_07891_amd import binding, synth
from tests import parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _sample_positions(T, window, n_random, seed):
    rng = np.random.default_rng(seed)
    fixed = [0, 1, 127, 128, 129, 255, 256, 1023, 1024, 1025, T // 2 - 1, T // 2,
             T - window - 2, T - window - 1, T - window, T - window + 1, T - 2, T - 1]
    pos = set(p for p in fixed if 0 <= p < T)
    pos.update(int(p) for p in rng.integers(0, T, n_random))
    return np.array(sorted(pos))


def _full_size_case(name, n_random=1500):
    wl = synth.CONFIGS[name]
    w = synth.make_weights(wl, 0, DEV)
    hid = synth.make_hidden(wl, 0, DEV)
    K, V = synth.make_kv(wl, 0, DEV)
    B, T, H = wl.B, wl.T, wl.H
    scores = binding.kvzap_score(hid, w["W1"], w["b1"], w["W2"], w["b2"])
    torch.cuda.synchronize()

    # ---- scores on sampled tokens against the float64 oracle ----
    ow = synth.oracle_weights(w)
    pos = _sample_positions(T, wl.window, n_random, seed=1)
    S_gpu = scores.cpu().numpy()
    S_ref = np.empty((B, H, len(pos)))
    for b in range(B):
        h64 = O.bf16_bits_to_f64(synth.bits(hid[b, torch.from_numpy(pos).to(DEV)]))
        S_ref[b] = (O.score_mlp(h64, ow["W1"], ow["b1"], ow["W2"], ow["b2"]) if "W1" in ow
                    else O.score_linear(h64, ow["W"], ow["b"]))
    err = np.abs(S_gpu[:, :, pos] - S_ref)
    assert (err <= parity.SCORE_RTOL * np.maximum(np.abs(S_ref), 1.0)).all(), err.max()

    # tau from the sample's quantile (the recipe's quantile needs every score; the sample
    # estimates it, and the test only needs a tau that splits the scores realistically)
    non_window = pos < T - wl.window
    tau = O.tau_at_keep_fraction(S_ref[:, :, non_window], 0, wl.keep_fraction)

    # ---- mask + compact in full, oracle run on the GPU's own scores ----
    idx, n, off = binding.kvzap_mask(scores, tau, wl.window)
    Ko, Vo = binding.kvzap_compact(K, V, idx, n, off)
    torch.cuda.synchronize()
    ref = O.prune(S_gpu.astype(np.float64), tau, wl.window)
    idx_h, n_h, off_h = idx.cpu().numpy(), n.cpu().numpy(), off.cpu().numpy()
    np.testing.assert_array_equal(n_h, ref.lengths)
    np.testing.assert_array_equal(off_h, ref.offsets)
    np.testing.assert_array_equal(idx_h[:off_h[-1]], ref.flat_idx())
    total = int(off_h[-1])
    kept_frac = total / (B * H * T)
    assert abs(kept_frac - wl.keep_fraction) < 0.05
    # gathered bytes: compare against a gather done with the oracle's index lists, head by head
    Kb = K.view(torch.int16); Vb = V.view(torch.int16)
    Kob = Ko.view(torch.int16); Vob = Vo.view(torch.int16)
    for b in range(B):
        for h in range(H):
            bh = b * H + h
            want = torch.from_numpy(ref.idx[b][h].astype(np.int64)).to(DEV)
            sl = slice(int(off_h[bh]), int(off_h[bh]) + int(n_h[b, h]))
            assert torch.equal(Kob[sl], Kb[b, h].index_select(0, want))
            assert torch.equal(Vob[sl], Vb[b, h].index_select(0, want))

    # ---- keep decisions on the sampled tokens agree with float64 outside the band ----
    keep_gpu = np.zeros((B, H, T), dtype=bool)
    for b in range(B):
        for h in range(H):
            bh = b * H + h
            keep_gpu[b, h, idx_h[off_h[bh]:off_h[bh] + n_h[b, h]]] = True
    want_keep = (S_ref >= tau) | (pos >= T - wl.window)[None, None, :]
    clear = (np.abs(S_ref - tau) >= parity.BAND) | (pos >= T - wl.window)[None, None, :]
    assert (keep_gpu[:, :, pos][clear] == want_keep[clear]).all()
    assert clear.mean() > 0.9


def test_config3_full_layer():
    _full_size_case("c3_qwen8b_128k_mlp")


def test_config4_full_layer_mlp():
    _full_size_case("c4_qwen32b_4x64k_mlp", n_random=600)


def test_config4_full_layer_linear():
    _full_size_case("c4_qwen32b_4x64k_linear", n_random=600)


def test_decode_attention_at_the_benchmark_shape():
    """kvzap_attend_decode at the decode workload's cache shape (64 sequences x 8 KV heads of
    4096..32768 rows + a full 128-row ring, 32 query heads), as bench.py launches it; the
    oracle recomputes a sample of heads one by one: the shortest, the longest, the first, the
    last and a few random ones."""
    wl = synth.CONFIGS["c5_qwen8b_decode"]
    B, H, D, w, HQ = wl.B, wl.H, wl.D, wl.window, 32
    G = HQ // H
    g = torch.Generator().manual_seed(wl.seed)
    lens = torch.randint(4096, 32768 + 1, (B, H), generator=g).to(torch.int32)
    off = torch.zeros(B * H, dtype=torch.int64)
    off[1:] = torch.cumsum(lens.reshape(-1).to(torch.int64), 0)[:-1]
    total = int(lens.sum())
    q, Kr, Vr, Kg, Vg = synth.make_attend_inputs(B, H, HQ, D, total, w, wl.seed, DEV)
    sp = torch.full((B,), 40000, dtype=torch.int32, device=DEV)
    scale = D ** -0.5
    out = binding.kvzap_attend_decode(q, Kr, Vr, off.to(DEV), lens.to(DEV), Kg, Vg, sp, w, 32768,
                                      scale)
    torch.cuda.synchronize()
    flat = lens.reshape(-1)
    rng = np.random.default_rng(3)
    heads = {0, B * H - 1, int(flat.argmin()), int(flat.argmax())}
    heads.update(int(x) for x in rng.integers(0, B * H, 6))
    for bh in sorted(heads):
        b, h = divmod(bh, H)
        o, n = int(off[bh]), int(flat[bh])
        K = synth.f64(torch.cat([Kr[o:o + n], Kg[b, h]]))
        V = synth.f64(torch.cat([Vr[o:o + n], Vg[b, h]]))
        ref = O.attend_decode(synth.f64(q[b:b + 1, h * G:(h + 1) * G]), [[(K, V)]], scale)[0]
        got = out[b, h * G:(h + 1) * G].to(torch.float64).cpu().numpy()
        err = np.abs(got - ref)
        assert err.max() <= 2.0 ** -7 * max(1.0, float(np.abs(V).max())), (bh, err.max())
        assert np.sqrt((err ** 2).mean()) <= 2e-3 * np.sqrt((ref ** 2).mean()) + 1e-3, bh
