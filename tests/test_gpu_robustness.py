"""Robustness of the HIP path: stream ordering, run-to-run determinism, randomised
shapes, reuse of poisoned workspaces.  All comparisons are against the CPU oracle
or bit-for-bit between runs."""
import numpy as np
import pytest
import torch

from oracle import kvzap_oracle as O
from paper_2601_07891_amd import binding, synth
from tests import parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _bits_kv(B, H, T, D, seed):
    g = torch.Generator().manual_seed(seed)
    K = torch.randint(-32768, 32768, (B, H, T, D), generator=g, dtype=torch.int16).view(torch.bfloat16)
    V = torch.randint(-32768, 32768, (B, H, T, D), generator=g, dtype=torch.int16).view(torch.bfloat16)
    return K, V


def test_randomised_shapes_mask_compact():
    rng = np.random.default_rng(2024)
    for case in range(40):
        B = int(rng.integers(1, 4)); H = int(rng.integers(1, 17))
        T = int(rng.choice([1, 2, 3, 5, 63, 64, 65, 255, 1023, 1024, 1025, 2047, 3001, 4096]))
        D = int(rng.choice([8, 16, 64, 128, 136, 256]))
        w = int(rng.choice([0, 1, 7, 128, T, T + 5]))
        tau = float(rng.choice([-np.inf, -1.0, 0.0, 0.25, 2.0, np.inf]))
        ties = bool(rng.integers(0, 2))
        scores = synth.make_scores(B, H, T, seed=case, ties=ties)
        lens = None
        if B > 1 and rng.integers(0, 2):
            lens = [int(x) for x in rng.integers(0, T + 1, B)]
        K, V = _bits_kv(B, H, T, D, case)
        sl = None if lens is None else torch.tensor(lens, dtype=torch.int32, device=DEV)
        idx, n, off = binding.kvzap_mask(scores.to(DEV), tau, w, sl)
        Ko, Vo = binding.kvzap_compact(K.to(DEV), V.to(DEV), idx, n, off)
        torch.cuda.synchronize()
        parity.assert_prune_matches(idx, n, off, Ko, Vo, K, V, scores.double().numpy(), tau, w, lens)


def test_non_default_stream_and_back_to_back_calls():
    wl = synth.with_size(synth.CONFIGS["c2_llama8b_32k_mlp"], T=5000)
    w = synth.make_weights(wl, 0, DEV); hid = synth.make_hidden(wl, 0, DEV)
    K, V = synth.make_kv(wl, 0, DEV)
    # reference on the default stream
    s0 = binding.kvzap_score(hid, w["W1"], w["b1"], w["W2"], w["b2"])
    i0, n0, o0 = binding.kvzap_mask(s0, 0.1, wl.window)
    K0, V0 = binding.kvzap_compact(K, V, i0, n0, o0)
    torch.cuda.synchronize()
    tot = int(o0[-1])
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        big = torch.empty(1 << 28, dtype=torch.uint8, device=DEV)
        for _ in range(4):
            big.fill_(3)                         # keeps the side stream busy before our kernels
        s1 = binding.kvzap_score(hid, w["W1"], w["b1"], w["W2"], w["b2"])
        i1, n1, o1 = binding.kvzap_mask(s1, 0.1, wl.window)
        K1, V1 = binding.kvzap_compact(K, V, i1, n1, o1)
        # immediately again into the same outputs, no synchronisation in between
        binding.kvzap_score(hid, w["W1"], w["b1"], w["W2"], w["b2"], s1)
        binding.kvzap_mask(s1, 0.1, wl.window, None, i1, n1, o1)
        binding.kvzap_compact(K, V, i1, n1, o1, K1, V1)
    side.synchronize()
    assert torch.equal(s0, s1) and torch.equal(n0, n1) and torch.equal(o0, o1)
    assert torch.equal(i0[:tot], i1[:tot])
    assert torch.equal(K0[:tot].view(torch.int16), K1[:tot].view(torch.int16))
    assert torch.equal(V0[:tot].view(torch.int16), V1[:tot].view(torch.int16))


def test_explicit_stream_that_is_not_current():
    # stream= names a side stream while torch's current stream stays the default one: the
    # wrappers' temporary workspaces are allocated on the current stream and must not be
    # recycled (and overwritten by the allocations below) before the side stream has run
    wl = synth.with_size(synth.CONFIGS["c2_llama8b_32k_mlp"], T=6000)
    w = synth.make_weights(wl, 0, DEV); hid = synth.make_hidden(wl, 0, DEV)
    K, V = synth.make_kv(wl, 0, DEV)
    s0 = binding.kvzap_score(hid, w["W1"], w["b1"], w["W2"], w["b2"])
    i0, n0, o0 = binding.kvzap_mask(s0, 0.1, wl.window)
    K0, V0 = binding.kvzap_compact(K, V, i0, n0, o0)
    torch.cuda.synchronize()
    tot = int(o0[-1])
    side = torch.cuda.Stream()
    big = torch.empty(1 << 28, dtype=torch.uint8, device=DEV)
    for rep in range(3):
        with torch.cuda.stream(side):
            for _ in range(4):
                big.fill_(rep)                   # the side stream is busy when our kernels arrive
        s1 = binding.kvzap_score(hid, w["W1"], w["b1"], w["W2"], w["b2"], stream=side)
        # what a recycled workspace block would be overwritten by, on the current stream
        junk = [torch.full((n,), 255, dtype=torch.uint8, device=DEV) for n in (1 << 22, 1 << 23, 1 << 16)]
        i1, n1, o1 = binding.kvzap_mask(s1, 0.1, wl.window, stream=side)
        junk += [torch.full((n,), 255, dtype=torch.uint8, device=DEV) for n in (1 << 12, 1 << 16, 1 << 20)]
        K1, V1 = binding.kvzap_compact(K, V, i1, n1, o1, stream=side)
        side.synchronize()
        torch.cuda.synchronize()
        del junk
        assert torch.equal(s0, s1) and torch.equal(n0, n1) and torch.equal(o0, o1)
        assert torch.equal(i0[:tot], i1[:tot])
        assert torch.equal(K0[:tot].view(torch.int16), K1[:tot].view(torch.int16))
        assert torch.equal(V0[:tot].view(torch.int16), V1[:tot].view(torch.int16))


def test_bitwise_repeatability_and_poisoned_workspaces():
    wl = synth.with_size(synth.CONFIGS["c3_qwen8b_128k_mlp"], L=1, T=9000)
    w = synth.make_weights(wl, 0, DEV); hid = synth.make_hidden(wl, 0, DEV)
    K, V = synth.make_kv(wl, 0, DEV)
    B, T, H = wl.B, wl.T, wl.H
    ws_s = torch.empty(binding.kvzap_workspace_bytes(binding.CALL_SCORE, B, T, wl.Dh, wl.M, H),
                       dtype=torch.uint8, device=DEV)
    ws_m = torch.empty(binding.kvzap_workspace_bytes(binding.CALL_MASK, B, T, 0, 0, H),
                       dtype=torch.uint8, device=DEV)
    outs = []
    for poison in (0, 255, 170, 85, 1):
        ws_s.fill_(poison); ws_m.fill_(poison)
        s = binding.kvzap_score(hid, w["W1"], w["b1"], w["W2"], w["b2"], None, ws_s)
        i, n, o = binding.kvzap_mask(s, 0.3, wl.window, None, None, None, None, ws_m)
        Ko, Vo = binding.kvzap_compact(K, V, i, n, o)
        torch.cuda.synchronize()
        tot = int(o[-1])
        outs.append((s.clone(), i[:tot].clone(), n.clone(), o.clone(),
                     Ko[:tot].view(torch.int16).clone(), Vo[:tot].view(torch.int16).clone()))
    for other in outs[1:]:
        for a, b in zip(outs[0], other):
            assert torch.equal(a, b)


def test_decode_repeatable():
    B, H, D, Dh, M, w = 6, 8, 128, 1024, 256, 8
    g = torch.Generator().manual_seed(5)
    wts = {"W1": (torch.randn((M, Dh), generator=g) * Dh ** -0.5).bfloat16().to(DEV),
           "b1": (torch.randn((M,), generator=g) * 0.1).bfloat16().to(DEV),
           "W2": (torch.randn((H, M), generator=g) * M ** -0.5).bfloat16().to(DEV),
           "b2": (torch.randn((H,), generator=g) * 0.1).bfloat16().to(DEV)}
    hid = torch.randn((40, B, Dh), generator=g).bfloat16().to(DEV)
    kv = torch.randn((40, 2, B, H, D), generator=g).bfloat16().to(DEV)
    finals = []
    for rep in range(3):
        st = binding.DecodeState(B, H, D, w, np.full((B, H), 64), DEV)
        for t in range(40):
            binding.kvzap_decode_evict(hid[t], wts["W1"], wts["b1"], wts["W2"], wts["b2"],
                                       kv[t, 0], kv[t, 1], st, 0.0)
        torch.cuda.synchronize()
        finals.append((st.lengths.clone(), st.prefix_pos.clone(), st.K_prefix.view(torch.int16).clone(),
                       st.V_ring.view(torch.int16).clone(), st.score_ring.clone(), st.seq_pos.clone()))
    for other in finals[1:]:
        for a, b in zip(finals[0], other):
            assert torch.equal(a, b)
    assert int(finals[0][5][0]) == 40
