"""GPU parity of kvzap_score (linear and MLP surrogates) against the float64 oracle."""
import numpy as np
import pytest
import torch

from oracle import kvzap_oracle as O
from paper_2601_07891_amd import binding, synth
from tests import parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(w):
    return {k: (None if v is None else v.to(DEV)) for k, v in w.items()}


def _oracle_scores(hid, w):
    ow = synth.oracle_weights(w)
    out = []
    for b in range(hid.shape[0]):
        h64 = O.bf16_bits_to_f64(synth.bits(hid[b]))
        if "W1" in ow:
            out.append(O.score_mlp(h64, ow["W1"], ow["b1"], ow["W2"], ow["b2"]))
        else:
            out.append(O.score_linear(h64, ow["W"], ow["b"]))
    return np.stack(out)


def _gpu_scores(hid, w):
    d = _dev(w)
    s = binding.kvzap_score(hid.to(DEV), d["W1"], d["b1"], d["W2"], d["b2"])
    torch.cuda.synchronize()
    return s


# up to 8192 tokens (and D_h a multiple of 128) the short-input kernel runs, above it or with
# other widths the one that stages W in LDS
LINEAR_SHAPES = [(1, 1024, 4096, 8), (2, 333, 5120, 8), (1, 1, 64, 1), (3, 17, 192, 5),
                 (1, 4099, 4096, 8), (1, 50, 1024, 16), (1, 8192, 4096, 8), (1, 9001, 4096, 8),
                 (2, 5003, 5120, 8), (1, 8200, 1024, 16)]


@pytest.mark.parametrize("B,T,Dh,H", LINEAR_SHAPES)
def test_linear_random(B, T, Dh, H):
    wl = synth.Workload("t", L=1, B=B, T=T, Dh=Dh, H=H, scorer="linear", seed=T, bias_std=0.1)
    w = synth.make_weights(wl); hid = synth.make_hidden(wl)
    parity.assert_scores_close(_gpu_scores(hid, w), _oracle_scores(hid, w))


@pytest.mark.parametrize("T,Dh,H", [(1000, 4096, 8), (77, 320, 3)])
def test_linear_exact_integers(T, Dh, H):
    # every partial sum is a small integer: fp32 accumulation in any order is exact
    hid, w = synth.make_exact_case(T, Dh, H, 0, seed=T)
    got = parity.to_np(_gpu_scores(hid, w)).astype(np.float64)
    np.testing.assert_array_equal(got, _oracle_scores(hid, w))


def test_linear_one_hot_weights_pick_columns():
    T, Dh, H = 130, 4096, 8
    wl = synth.Workload("t", L=1, B=1, T=T, Dh=Dh, H=H, scorer="linear", seed=1)
    hid = synth.make_hidden(wl)
    W = torch.zeros((H, Dh), dtype=torch.bfloat16)
    cols = [0, 7, 8, 31, 32, 2047, 4000, 4095]
    for h, c in enumerate(cols):
        W[h, c] = 1.0
    got = parity.to_np(_gpu_scores(hid, {"W1": W, "b1": None, "W2": None, "b2": None}))
    want = hid[0].float().numpy()[:, cols].T
    np.testing.assert_array_equal(got[0], want)


MLP_SHAPES = [(1, 300, 256, 128, 8), (2, 129, 1024, 128, 8), (1, 1000, 4096, 512, 8),
              (1, 257, 5120, 640, 8), (1, 64, 2048, 256, 3), (1, 1, 3072, 384, 16),
              (3, 50, 4096, 512, 8), (1, 200, 448, 128, 8), (2, 70, 320, 256, 4),   # odd K-tile counts
              (1, 97, 256, 640, 8), (1, 500, 192, 512, 8),                          # 4 tiles; D_h < 256
              # the single kernel keeps two K tiles of W1 fragments in flight in alternating
              # register sets: odd and even tile counts at every unit-block count, 5 to 65 tiles
              (1, 300, 4160, 512, 8), (1, 260, 384, 512, 8), (1, 150, 576, 384, 8),
              (1, 140, 320, 128, 8), (1, 131, 5184, 640, 8),
              # more than one block per CU and a ragged last block: blocks touch the first hidden
              # tiles of the block 256 further on, up to the end of the input and not beyond
              (1, 40077, 1024, 128, 8), (2, 16500, 512, 256, 8)]


# kvzap_score splits the first projection of short and mid-length prompts (a skinny GEMM up
# to 384 tokens, the main kernel cut over K while its token blocks do not fill the chip);
# kvzap_score_prepared always takes the one-kernel path, so both see every shape
@pytest.mark.parametrize("entry", ["score", "prepared"])
@pytest.mark.parametrize("B,T,Dh,M,H", MLP_SHAPES)
def test_mlp_random(B, T, Dh, M, H, entry):
    wl = synth.Workload("t", L=1, B=B, T=T, Dh=Dh, H=H, scorer="mlp", seed=T + M, bias_std=0.1)
    g = torch.Generator().manual_seed(T)
    w = {"W1": (torch.randn((M, Dh), generator=g) * Dh ** -0.5).bfloat16(),
         "b1": (torch.randn((M,), generator=g) * 0.1).bfloat16(),
         "W2": (torch.randn((H, M), generator=g) * M ** -0.5).bfloat16(),
         "b2": (torch.randn((H,), generator=g) * 0.1).bfloat16()}
    hid = synth.make_hidden(wl)
    if entry == "score":
        got = _gpu_scores(hid, w)
    else:
        d = _dev(w)
        got = binding.kvzap_score_prepared(hid.to(DEV), binding.kvzap_prepare_scorer(d["W1"]), d["b1"],
                                           d["W2"], d["b2"])
        torch.cuda.synchronize()
    err = parity.assert_scores_close(got, _oracle_scores(hid, w))
    assert err < 5e-3


def test_mlp_randomised_shapes():
    # 30 seeded shapes through the one-kernel path (kvzap_score_prepared) and through
    # kvzap_score: every unit-block count, 4 to 40 K tiles (odd and even), 1 to 16 heads,
    # ragged token counts, with and without the biases
    rng = np.random.default_rng(7)
    for case in range(30):
        M = int(rng.choice([128, 256, 384, 512, 640]))
        Dh = 64 * int(rng.integers(4, 41))
        H = int(rng.integers(1, 17))
        B = int(rng.integers(1, 4))
        T = int(rng.choice([1, 31, 96, 127, 128, 129, 300, 517, 1000]))
        g = torch.Generator().manual_seed(1000 + case)
        bias = bool(rng.integers(0, 2))
        w = {"W1": (torch.randn((M, Dh), generator=g) * Dh ** -0.5).bfloat16(),
             "b1": (torch.randn((M,), generator=g) * 0.3).bfloat16() if bias else None,
             "W2": (torch.randn((H, M), generator=g) * M ** -0.5).bfloat16(),
             "b2": (torch.randn((H,), generator=g) * 0.3).bfloat16() if bias else None}
        wl = synth.Workload("t", L=1, B=B, T=T, Dh=Dh, H=H, scorer="mlp", seed=case)
        hid = synth.make_hidden(wl)
        d = _dev(w)
        want = _oracle_scores(hid, w)
        got = binding.kvzap_score_prepared(hid.to(DEV), binding.kvzap_prepare_scorer(d["W1"]), d["b1"],
                                           d["W2"], d["b2"])
        torch.cuda.synchronize()
        parity.assert_scores_close(got, want)
        parity.assert_scores_close(_gpu_scores(hid, w), want)


@pytest.mark.parametrize("B,T,Dh,M,H", [(1, 1024 + 77, 4096, 512, 8), (3, 731, 1024, 128, 8),
                                        (1, 1025, 5120, 640, 8), (1, 900, 2048, 256, 3),
                                        (1, 700, 3072, 384, 16), (1, 20000, 4096, 512, 8)])
def test_mlp_split_k_path_through_kvzap_score(B, T, Dh, M, H):
    # just past the short-prompt limit: the main kernel cut over K, ragged last block,
    # several sequences
    wl = synth.Workload("t", L=1, B=B, T=T, Dh=Dh, H=H, scorer="mlp", seed=T, bias_std=0.1)
    w = synth.make_weights(wl); hid = synth.make_hidden(wl)
    assert B * T > 384
    err = parity.assert_scores_close(_gpu_scores(hid, w), _oracle_scores(hid, w))
    assert err < 5e-3


def test_mlp_no_bias_and_unit_selectivity():
    # W2 one-hot: score[h] = GELU(z[unit_h]); checks the unit <-> lane/register mapping
    # of the fused second projection for every unit position in a 32-block
    T, Dh, M, H = 70, 512, 512, 8
    wl = synth.Workload("t", L=1, B=1, T=T, Dh=Dh, H=H, scorer="mlp", seed=2)
    hid = synth.make_hidden(wl)
    g = torch.Generator().manual_seed(0)
    W1 = (torch.randn((M, Dh), generator=g) * Dh ** -0.5).bfloat16()
    for base in range(0, 64, 8):
        W2 = torch.zeros((H, M), dtype=torch.bfloat16)
        units = [(base + 37 * h + 64 * h) % M for h in range(H)]
        for h, u in enumerate(units):
            W2[h, u] = 1.0
        w = {"W1": W1, "b1": None, "W2": W2, "b2": None}
        parity.assert_scores_close(_gpu_scores(hid, w), _oracle_scores(hid, w))
        z = hid[0].double().numpy() @ W1.double().numpy().T
        want = O.gelu(z)[:, units].T
        got = parity.to_np(_gpu_scores(hid, w))[0].astype(np.float64)
        assert np.abs(got - want).max() < 2e-4


@pytest.mark.parametrize("Dh,M", [(512, 512), (1024, 640), (256, 128)])
def test_fused_epilogue_unit_selectivity(Dh, M):
    # The same one-hot W2 through kvzap_score_prepared, which always runs the single kernel with
    # the fused epilogue (GELU fitted to 2.6e-5, result rounded to fp16 for the second matrix
    # product): every unit position of a wavefront's accumulator blocks must reach the head
    # that W2 names, and b1 must reach its unit through the accumulators' initial value.
    T, H = 300, 8
    wl = synth.Workload("t", L=1, B=1, T=T, Dh=Dh, H=H, scorer="mlp", seed=4)
    hid = synth.make_hidden(wl)
    g = torch.Generator().manual_seed(1)
    W1 = (torch.randn((M, Dh), generator=g) * Dh ** -0.5).bfloat16()
    b1 = (torch.randn((M,), generator=g)).bfloat16()
    z = hid[0].double().numpy() @ W1.double().numpy().T + b1.double().numpy()
    G = O.gelu(z)
    prep = binding.kvzap_prepare_scorer(W1.to(DEV))
    for base in range(0, 128, 8):
        W2 = torch.zeros((H, M), dtype=torch.bfloat16)
        units = [(base + h + 133 * h) % M for h in range(H)]
        for h, u in enumerate(units):
            W2[h, u] = 1.0
        got = binding.kvzap_score_prepared(hid.to(DEV), prep, b1.to(DEV), W2.to(DEV), None)
        torch.cuda.synchronize()
        got = parity.to_np(got)[0].astype(np.float64)
        want = G[:, units].T
        assert (np.abs(got - want) <= 6e-4 * np.abs(want) + 6e-5).all(), np.abs(got - want).max()


def test_fused_gelu_over_its_whole_range():
    # z swept over [-12, 12] (and far beyond) through the fused kernel: identity weights pick
    # hidden columns, so z is exact and the score is GELU(z) as the kernel evaluates it
    T, Dh, M, H = 4096, 256, 128, 8
    hid = torch.zeros((1, T, Dh), dtype=torch.bfloat16)
    zs = torch.linspace(-12.0, 12.0, T).bfloat16()
    zs[:8] = torch.tensor([-200.0, -50.0, -14.0, 14.0, 50.0, 200.0, 0.0, -0.0]).bfloat16()
    for h in range(H):
        hid[0, :, h] = zs * (1.0 if h % 2 == 0 else -1.0)
    W1 = torch.zeros((M, Dh), dtype=torch.bfloat16)
    W2 = torch.zeros((H, M), dtype=torch.bfloat16)
    for h in range(H):
        W1[17 * h + 3, h] = 1.0
        W2[h, 17 * h + 3] = 1.0
    prep = binding.kvzap_prepare_scorer(W1.to(DEV))
    got = binding.kvzap_score_prepared(hid.to(DEV), prep, None, W2.to(DEV), None)
    torch.cuda.synchronize()
    got = parity.to_np(got)[0].astype(np.float64)
    z = hid[0].double().numpy()[:, :H].T
    want = O.gelu(z)
    assert np.isfinite(got).all()
    assert (np.abs(got - want) <= 6e-4 * np.abs(want) + 6e-5).all(), np.abs(got - want).max()


def test_mlp_exact_first_projection():
    # integer inputs: z is exact, so the only error left is GELU + second projection
    T, Dh, M, H = 200, 256, 128, 8
    hid, w = synth.make_exact_case(T, Dh, H, M, seed=3)
    got = parity.to_np(_gpu_scores(hid, w)).astype(np.float64)
    want = _oracle_scores(hid, w)
    assert np.abs(got - want).max() <= 1e-4 * np.maximum(np.abs(want), 1).max()


def test_scores_deterministic():
    wl = synth.with_size(synth.CONFIGS["c2_llama8b_32k_mlp"], T=2000)
    w = synth.make_weights(wl); hid = synth.make_hidden(wl)
    a = _gpu_scores(hid, w).clone()
    b = _gpu_scores(hid, w)
    assert torch.equal(a, b)


# exact: kvzap_score runs the same single kernel as kvzap_score_prepared (enough token blocks
# to fill the chip, or too few K tiles to split); otherwise it splits K and finishes in fp32
@pytest.mark.parametrize("B,T,Dh,M,H,exact", [(1, 17000, 4096, 512, 8, True), (1, 3000, 4096, 512, 8, False),
                                              (1, 1024 + 257, 5120, 640, 8, False),
                                              (2, 700, 320, 256, 4, True), (1, 1500, 192, 512, 8, True),
                                              (1, 1000, 4096, 512, 8, False)])
def test_prepared_weights_give_the_same_scores(B, T, Dh, M, H, exact):
    # W1 re-ordered once and reused, also after the original W1 is gone and on repeated calls:
    # the scores of kvzap_score, bit for bit where both run the same kernel, within rounding
    # where kvzap_score uses its workspace to split the first projection
    wl = synth.Workload("t", L=1, B=B, T=T, Dh=Dh, H=H, scorer="mlp", seed=T + M, bias_std=0.1)
    g = torch.Generator().manual_seed(T)
    w = _dev({"W1": (torch.randn((M, Dh), generator=g) * Dh ** -0.5).bfloat16(),
              "b1": (torch.randn((M,), generator=g) * 0.1).bfloat16(),
              "W2": (torch.randn((H, M), generator=g) * M ** -0.5).bfloat16(),
              "b2": (torch.randn((H,), generator=g) * 0.1).bfloat16()})
    hid = synth.make_hidden(wl).to(DEV)
    want = binding.kvzap_score(hid, w["W1"], w["b1"], w["W2"], w["b2"]).clone()
    prep = binding.kvzap_prepare_scorer(w["W1"])
    w["W1"].zero_()
    first = None
    for _ in range(2):
        got = binding.kvzap_score_prepared(hid, prep, w["b1"], w["W2"], w["b2"])
        torch.cuda.synchronize()
        if exact:
            assert torch.equal(got, want)
        else:
            assert (got - want).abs().max().item() < 1e-3
        first = got.clone() if first is None else first
        assert torch.equal(got, first)
