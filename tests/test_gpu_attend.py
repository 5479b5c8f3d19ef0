"""GPU parity of kvzap_attend_decode against the float64 attention oracle.

Tolerance (derived from the arithmetic the header states): the softmax weights enter the
second product rounded to bf16 (relative 2^-9 each) and the denominator sums the same
rounded weights, so |out - ref| <= 2^-8 * max_i |V_i| per head before the final bf16
rounding of the output (another 2^-9 * |out|); fp32 accumulation errors are orders of
magnitude below that.  The test bound is 2^-7 * max(1, max|V|) elementwise and, sharper
because rounding errors average out, an RMS error below 2e-3 * rms(ref) + 1e-3.
"""
import numpy as np
import pytest
import torch

from oracle import kvzap_oracle as O
from paper_2601_07891_amd import binding, synth
from tests import parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
D = 128


def _layout(lengths, gap, rng):
    """Row offsets with random gaps between the heads' slabs (the layout of the decode
    state; gap = 0 gives the packed prefill layout)."""
    n = np.asarray(lengths, np.int64).reshape(-1)
    gaps = rng.integers(0, gap + 1, size=n.size) if gap > 0 else np.zeros(n.size, np.int64)
    off = np.zeros(n.size, np.int64)
    pos = 0
    for i in range(n.size):
        pos += int(gaps[i])
        off[i] = pos
        pos += int(n[i])
    return off, pos + (int(gap) if gap > 0 else 0)


def _run_case(lengths, window, seq_pos, HQ, seed, gap=5, q_gain=1.0, max_rows=None,
              scale=None):
    lengths = np.asarray(lengths, np.int32)
    B, H = lengths.shape
    rng = np.random.default_rng(seed)
    off, total = _layout(lengths, gap, rng)
    q, Kr, Vr, Kg, Vg = synth.make_attend_inputs(B, H, HQ, D, total, window, seed, DEV, q_gain)
    scale = D ** -0.5 if scale is None else scale
    mr = int(lengths.max()) if max_rows is None else max_rows
    sp = None if window == 0 else torch.tensor(seq_pos, dtype=torch.int32, device=DEV)
    out = binding.kvzap_attend_decode(
        q, Kr, Vr, torch.from_numpy(off).to(DEV), torch.from_numpy(lengths).to(DEV),
        Kg if window else None, Vg if window else None, sp, window, mr, scale)
    torch.cuda.synchronize()
    got = out.to(torch.float64).cpu().numpy()

    Kf, Vf, Kgf, Vgf = synth.f64(Kr), synth.f64(Vr), synth.f64(Kg), synth.f64(Vg)
    G = HQ // H
    worst = 0.0
    for b in range(B):
        for h in range(H):
            o, n = int(off[b * H + h]), int(lengths[b, h])
            nr = min(int(seq_pos[b]), window) if window else 0
            K = np.concatenate([Kf[o:o + n], Kgf[b, h, :nr]])
            V = np.concatenate([Vf[o:o + n], Vgf[b, h, :nr]])
            g0 = h * G
            mine = got[b, g0:g0 + G]
            if n + nr == 0:
                assert np.all(mine == 0.0), f"empty head ({b},{h}) must give zeros"
                continue
            ref = O.attend_decode(synth.f64(q)[b:b + 1, g0:g0 + G], [[(K, V)]], scale)[0]
            err = np.abs(mine - ref)
            bound = 2.0 ** -7 * max(1.0, float(np.abs(V).max()))
            assert err.max() <= bound, \
                f"head ({b},{h}) n={n}+{nr}: max err {err.max():.3e} > {bound:.3e}"
            rms = float(np.sqrt((err ** 2).mean()))
            lim = 2e-3 * float(np.sqrt((ref ** 2).mean())) + 1e-3
            assert rms <= lim, f"head ({b},{h}) n={n}+{nr}: rms err {rms:.3e} > {lim:.3e}"
            worst = max(worst, float(err.max()))
    return worst


def test_ragged_lengths_no_ring():
    # tails around the 16- and 32-row tiles, a head of one row, an empty head, several splits
    lengths = [[1, 0, 15, 16], [17, 31, 32, 33], [63, 64, 65, 511], [512, 513, 1100, 2049]]
    _run_case(lengths, 0, None, HQ=16, seed=1)


def test_ring_partially_filled_and_full():
    lengths = [[0, 5, 300], [40, 0, 1000], [7, 700, 33], [0, 0, 0]]
    _run_case(lengths, 128, [0, 5, 128, 100000], HQ=12, seed=2)     # G = 4


def test_ring_only_heads():
    # no packed row at all: only the window (a short prompt); a sequence with seq_pos = 0 is empty
    _run_case([[0, 0], [0, 0], [0, 0]], 128, [1, 77, 0], HQ=8, seed=3)


def test_window_not_multiple_of_chunk():
    _run_case([[10, 200], [45, 3]], 50, [50, 13], HQ=8, seed=4)


@pytest.mark.parametrize("G", [1, 2, 4, 8, 16])
def test_group_sizes(G):
    H = 2
    _run_case([[100, 777], [1300, 64]], 128, [500, 64], HQ=H * G, seed=10 + G)


def test_packed_prefill_layout():
    # the output layout of the compaction step: no gaps, offsets = exclusive prefix sum
    _run_case([[900, 1, 0, 257], [128, 129, 640, 31]], 0, None, HQ=32, seed=5, gap=0)


def test_peaked_softmax():
    # logits ~ N(0, 8^2): a few rows carry almost all the weight, the running reference
    # has to move by far more than the lazy margin
    _run_case([[2000, 600], [1500, 40]], 128, [128, 9], HQ=8, seed=6, q_gain=8.0)


def test_huge_logits_do_not_overflow():
    # |logit| up to ~1e3: exp() of the raw values would overflow fp32
    _run_case([[700, 90]], 0, None, HQ=8, seed=7, q_gain=8.0, scale=10.0 * D ** -0.5)


def test_bound_smaller_than_lengths_still_exact():
    # max_rows is only a launch-size hint: heads longer than it are still covered in full
    _run_case([[3000, 40], [1200, 5000]], 128, [128, 128], HQ=8, seed=8, max_rows=100)


def test_bound_larger_than_lengths():
    _run_case([[30, 40], [12, 50]], 128, [3, 128], HQ=8, seed=9, max_rows=40000)


def test_ascending_logits_trigger_rescale_late():
    # rows sorted so the logits of query head 0 rise steadily over 3000 rows: the reference
    # has to be raised many times, each time well after the first chunk
    B, H, HQ, n = 1, 1, 4, 3000
    q, Kr, Vr, _, _ = synth.make_attend_inputs(B, H, HQ, D, n, 0, 21, DEV, q_gain=6.0)
    s = (Kr.float() @ q[0, 0].float())
    order = torch.argsort(s)
    Kr, Vr = Kr[order].contiguous(), Vr[order].contiguous()
    off = torch.zeros(1, dtype=torch.int64, device=DEV)
    ln = torch.tensor([[n]], dtype=torch.int32, device=DEV)
    out = binding.kvzap_attend_decode(q, Kr, Vr, off, ln, None, None, None, 0, n, D ** -0.5)
    ref = O.attend_decode(synth.f64(q), [[(synth.f64(Kr), synth.f64(Vr))]], D ** -0.5)
    err = np.abs(out.to(torch.float64).cpu().numpy() - ref)
    assert err.max() <= 2.0 ** -7 * max(1.0, float(Vr.abs().max()))


def test_uniform_values_are_reproduced_exactly():
    # all V rows equal: a convex combination must return that row bit for bit
    B, H, HQ, n = 2, 2, 8, 1500
    q, Kr, Vr, Kg, Vg = synth.make_attend_inputs(B, H, HQ, D, B * H * n, 64, 22, DEV)
    Vr[:] = Vr[0]
    Vg[:] = Vr[0]
    off = (torch.arange(B * H, dtype=torch.int64) * n).to(DEV)
    ln = torch.full((B, H), n, dtype=torch.int32, device=DEV)
    sp = torch.tensor([64, 20], dtype=torch.int32, device=DEV)
    out = binding.kvzap_attend_decode(q, Kr, Vr, off, ln, Kg, Vg, sp, 64, n, D ** -0.5)
    want = parity.to_np(Vr[0])
    got = parity.to_np(out).reshape(-1, D)
    assert np.array_equal(got, np.broadcast_to(want, got.shape))


def test_order_of_rows_does_not_matter_beyond_rounding():
    B, H, HQ, n = 1, 2, 8, 900
    q, Kr, Vr, _, _ = synth.make_attend_inputs(B, H, HQ, D, H * n, 0, 23, DEV)
    off = (torch.arange(H, dtype=torch.int64) * n).to(DEV)
    ln = torch.full((B, H), n, dtype=torch.int32, device=DEV)
    a = binding.kvzap_attend_decode(q, Kr, Vr, off, ln, None, None, None, 0, n, D ** -0.5)
    perm = torch.cat([torch.randperm(n, device=DEV) + h * n for h in range(H)])
    b = binding.kvzap_attend_decode(q, Kr[perm].contiguous(), Vr[perm].contiguous(), off, ln,
                                    None, None, None, 0, n, D ** -0.5)
    assert (a.float() - b.float()).abs().max().item() <= 2.0 ** -7


def test_attends_to_the_state_decode_evict_maintains():
    """Decode steps on the device (their parity with the decode oracle is tested on its own),
    then attention over prefix + ring of every head, against the oracle applied to the rows
    the state holds."""
    from tests.test_gpu_decode import _canonical_gpu
    wl = synth.with_size(synth.CONFIGS["c5_qwen8b_decode"], B=2, Dh=1024)
    B, H, w, steps, tau = 2, wl.H, 16, 45, 0.0
    st = binding.DecodeState(B, H, D, w, np.full((B, H), steps + 2), DEV)
    wt = synth.make_weights(wl, 0, DEV)
    for i in range(steps):
        hid = synth.make_hidden(wl, 100 + i, DEV, B=1, T=B)[0].contiguous()
        k, v = synth.make_kv(wl, 200 + i, DEV, B=B, T=1)
        binding.kvzap_decode_evict(hid, wt["W1"], wt["b1"], wt["W2"], wt["b2"],
                                   k[:, :, 0].contiguous(), v[:, :, 0].contiguous(), st, tau)
    torch.cuda.synchronize()
    assert int(st.error_flag[0]) == 0
    HQ = 4 * H
    q = synth.make_attend_inputs(B, H, HQ, D, 1, 0, 33, DEV)[0]
    out = binding.kvzap_attend_decode(q, st.K_prefix, st.V_prefix, st.slab_offsets, st.lengths,
                                      st.K_ring, st.V_ring, st.seq_pos, w, steps + 2, D ** -0.5)
    caches = []
    kept = 0
    for b in range(B):
        row = []
        for h in range(H):
            _, Kc, Vc = _canonical_gpu(st, b, h)
            kept += Kc.shape[0]
            row.append((O.bf16_bits_to_f64(Kc), O.bf16_bits_to_f64(Vc)))
        caches.append(row)
    assert B * H * w < kept < B * H * steps        # some tokens evicted, some kept
    ref = O.attend_decode(synth.f64(q), caches, D ** -0.5)
    err = np.abs(out.to(torch.float64).cpu().numpy() - ref)
    assert err.max() <= 2.0 ** -7 * 6.0, f"max err {err.max():.3e}"


def test_rejects_bad_arguments():
    q, Kr, Vr, Kg, Vg = synth.make_attend_inputs(1, 2, 8, D, 10, 4, 40, DEV)
    off = torch.zeros(2, dtype=torch.int64, device=DEV)
    ln = torch.zeros((1, 2), dtype=torch.int32, device=DEV)
    L = binding.lib()
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)
    out = torch.empty_like(q)

    def call(D_=D, HQ=8, H=2, ws_bytes=ws.numel(), ring=True, window=4):
        return L.kvzap_attend_decode(
            q.data_ptr(), Kr.data_ptr(), Vr.data_ptr(), 10, off.data_ptr(), ln.data_ptr(),
            Kg.data_ptr() if ring else None, Vg.data_ptr() if ring else None,
            torch.zeros(1, dtype=torch.int32, device=DEV).data_ptr() if ring else None,
            window, 10, 0.1, out.data_ptr(), 1, H, HQ, D_, ws.data_ptr(), ws_bytes, None)

    assert call() == 0
    assert call(D_=64) == -4          # unsupported head dimension
    assert call(HQ=7) == -2           # HQ not a multiple of H
    assert call(ws_bytes=16) == -6    # workspace too small
    assert call(ring=False) == -1     # window > 0 without ring pointers
    torch.cuda.synchronize()
