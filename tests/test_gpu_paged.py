"""GPU parity of the paged layout: kvzap_assign_pages, kvzap_compact_paged and
kvzap_attend_decode_paged against the oracle (page assignment and scatter: bit-exact;
attention: the bound derived in test_gpu_attend.py)."""
import numpy as np
import pytest
import torch

from oracle import kvzap_oracle as O
from paper_2601_07891_amd import binding, synth
from tests import parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _i32(a):
    return torch.as_tensor(np.asarray(a), dtype=torch.int32).to(DEV)


@pytest.mark.parametrize("P,reserve", [(16, 0), (16, 5), (64, 0), (128, 128), (1024, 0)])
def test_assign_pages_matches_oracle(P, reserve):
    rng = np.random.default_rng(P + reserve)
    B, H = 5, 8
    lengths = rng.integers(0, 700, (B, H)).astype(np.int32)
    lengths[0, 0] = 0
    lengths[1, 3] = P
    lengths[2, 2] = P + 1
    max_pages = 700 // P + 3 + reserve // P
    need = sum(O.pages_needed(int(n), P, reserve) for n in lengths.reshape(-1))
    free = rng.permutation(need + 20).astype(np.int32)
    table, res = binding.kvzap_assign_pages(_i32(lengths), P, _i32(free), max_pages, reserve)
    torch.cuda.synchronize()
    ref_table, used, ok = O.assign_pages(lengths, P, free, max_pages, reserve)
    assert ok
    assert res[:2].tolist() == [used, 0]
    np.testing.assert_array_equal(parity.to_np(table), ref_table)


def test_assign_pages_many_heads():
    # more heads than scan threads: every thread handles several
    rng = np.random.default_rng(0)
    B, H = 300, 16
    lengths = rng.integers(0, 100, (B, H)).astype(np.int32)
    free = np.arange(10 ** 5, dtype=np.int32)[::-1].copy()
    table, res = binding.kvzap_assign_pages(_i32(lengths), 16, _i32(free), 8)
    ref_table, used, ok = O.assign_pages(lengths, 16, free, 8)
    assert ok and res[:2].tolist() == [used, 0]
    np.testing.assert_array_equal(parity.to_np(table), ref_table)


def test_assign_pages_failures_assign_nothing():
    lengths = np.array([[20, 20], [3, 0]], np.int32)
    t, res = binding.kvzap_assign_pages(_i32(lengths), 16, _i32([1, 2, 3, 4]), 4)   # needs 5
    assert res[:2].tolist() == [0, 1] and (parity.to_np(t) == -1).all()
    t, res = binding.kvzap_assign_pages(_i32(lengths), 16, _i32(range(10)), 1)      # 2 per head
    assert res[:2].tolist() == [0, 2] and (parity.to_np(t) == -1).all()
    t, res = binding.kvzap_assign_pages(_i32(np.zeros((2, 2))), 16, _i32([]), 1)    # nothing needed
    assert res[:2].tolist() == [0, 0] and (parity.to_np(t) == -1).all()


def _pruned_case(B, H, T, D, w, seed, keep=0.4):
    S = synth.make_scores(B, H, T, seed=seed, device=DEV)
    wl = synth.Workload("p", L=1, B=B, T=T, Dh=256, H=H, D=D, seed=seed)
    K, V = synth.make_kv(wl, 0, DEV)
    S64 = S.double().cpu().numpy()
    tau = O.tau_at_keep_fraction(S64, w, keep)
    idx, n, off = binding.kvzap_mask(S, tau, w)
    ref = O.prune(S64, tau, w, synth.bits(K), synth.bits(V))
    return K, V, idx, n, off, ref


@pytest.mark.parametrize("P,D", [(16, 128), (32, 128), (128, 128), (64, 64), (16, 256)])
def test_compact_paged_matches_oracle_scatter(P, D):
    B, H, T, w = 2, 4, 1500, 100
    K, V, idx, n, off, ref = _pruned_case(B, H, T, D, w, seed=P + D)
    lengths = ref.lengths
    max_pages = T // P + 1
    need = sum(O.pages_needed(int(x), P) for x in lengths.reshape(-1))
    rng = np.random.default_rng(1)
    num_pages = need + 7
    free = rng.permutation(num_pages).astype(np.int32)
    table, res = binding.kvzap_assign_pages(n, P, _i32(free), max_pages)
    assert res[:2].tolist() == [need, 0]
    # pools start with a recognisable pattern: nothing but the kept rows may change
    Kp = torch.full((num_pages, P, D), -7.0, dtype=torch.bfloat16, device=DEV)
    Vp = torch.full((num_pages, P, D), -9.0, dtype=torch.bfloat16, device=DEV)
    binding.kvzap_compact_paged(K, V, idx, n, off, table, P, Kp, Vp)
    torch.cuda.synchronize()
    ref_table, _, _ = O.assign_pages(lengths, P, free, max_pages)
    rows_k = [ref.K_out[ref.offsets[i]:ref.offsets[i + 1]] for i in range(B * H)]
    rows_v = [ref.V_out[ref.offsets[i]:ref.offsets[i + 1]] for i in range(B * H)]
    want_k = O.scatter_to_pages(rows_k, ref_table, P, num_pages, D)
    want_v = O.scatter_to_pages(rows_v, ref_table, P, num_pages, D)
    written = np.zeros((num_pages, P), bool)
    for i, r in enumerate(rows_k):
        for j in range(r.shape[0]):
            written[ref_table[i, j // P], j % P] = True
    got_k, got_v = parity.to_np(Kp), parity.to_np(Vp)
    np.testing.assert_array_equal(got_k[written], want_k[written])
    np.testing.assert_array_equal(got_v[written], want_v[written])
    fill_k = parity.to_np(torch.tensor([-7.0], dtype=torch.bfloat16))[0]
    fill_v = parity.to_np(torch.tensor([-9.0], dtype=torch.bfloat16))[0]
    assert (got_k[~written] == fill_k).all() and (got_v[~written] == fill_v).all()
    # reading back through the table gives the contiguous result of kvzap_compact
    Ko, Vo = binding.kvzap_compact(K, V, idx, n, off)
    for i in range(B * H):
        nn = int(lengths.reshape(-1)[i])
        back = O.gather_from_pages(got_k, parity.to_np(table)[i], nn, P)
        np.testing.assert_array_equal(back, parity.to_np(Ko)[int(ref.offsets[i]):int(ref.offsets[i]) + nn])


def test_compact_paged_skips_rows_without_a_valid_page():
    B, H, T, D, P, w = 1, 2, 300, 128, 16, 10
    K, V, idx, n, off, ref = _pruned_case(B, H, T, D, w, seed=3)
    max_pages = 4                                   # far too few slots: rows beyond 64 are skipped
    table = torch.tensor([[0, 1, 99, -1], [2, 3, 4, 5]], dtype=torch.int32, device=DEV)
    num_pages = 6
    Kp = torch.zeros((num_pages, P, D), dtype=torch.bfloat16, device=DEV)
    Vp = torch.zeros_like(Kp)
    binding.kvzap_compact_paged(K, V, idx, n, off, table, P, Kp, Vp)
    torch.cuda.synchronize()
    got = parity.to_np(Kp)
    r0 = ref.K_out[ref.offsets[0]:ref.offsets[1]]
    r1 = ref.K_out[ref.offsets[1]:ref.offsets[2]]
    np.testing.assert_array_equal(got[0], r0[:16]); np.testing.assert_array_equal(got[1], r0[16:32])
    for pg in range(4):
        np.testing.assert_array_equal(got[2 + pg], r1[16 * pg:16 * pg + 16])


def _attend_case(lengths, P, window, seq_pos, HQ, seed, q_gain=1.0, max_rows=None):
    lengths = np.asarray(lengths, np.int32)
    B, H = lengths.shape
    D = 128
    rng = np.random.default_rng(seed)
    max_pages = int(lengths.max()) // P + 2
    need = sum(O.pages_needed(int(x), P) for x in lengths.reshape(-1))
    num_pages = need + 9
    free = rng.permutation(num_pages).astype(np.int32)
    ref_table, used, ok = O.assign_pages(lengths, P, free, max_pages)
    assert ok
    q, Kflat, Vflat, Kg, Vg = synth.make_attend_inputs(B, H, HQ, D, num_pages * P, window, seed, DEV,
                                                       q_gain)
    Kp, Vp = Kflat.view(num_pages, P, D), Vflat.view(num_pages, P, D)
    sp = None if window == 0 else _i32(seq_pos)
    mr = int(lengths.max()) if max_rows is None else max_rows
    out = binding.kvzap_attend_decode_paged(q, Kp, Vp, _i32(ref_table), P, _i32(lengths),
                                            Kg if window else None, Vg if window else None, sp,
                                            window, mr, D ** -0.5)
    torch.cuda.synchronize()
    got = out.to(torch.float64).cpu().numpy()
    Kb, Vb = synth.bits(Kp), synth.bits(Vp)
    G = HQ // H
    for b in range(B):
        for h in range(H):
            bh = b * H + h
            n = int(lengths[b, h])
            nr = min(int(seq_pos[b]), window) if window else 0
            K = np.concatenate([O.bf16_bits_to_f64(O.gather_from_pages(Kb, ref_table[bh], n, P)),
                                synth.f64(Kg[b, h, :nr])])
            V = np.concatenate([O.bf16_bits_to_f64(O.gather_from_pages(Vb, ref_table[bh], n, P)),
                                synth.f64(Vg[b, h, :nr])])
            mine = got[b, h * G:(h + 1) * G]
            if n + nr == 0:
                assert np.all(mine == 0.0)
                continue
            ref = O.attend_decode(synth.f64(q)[b:b + 1, h * G:(h + 1) * G], [[(K, V)]], D ** -0.5)[0]
            err = np.abs(mine - ref)
            assert err.max() <= 2.0 ** -7 * max(1.0, float(np.abs(V).max())), (b, h, n, nr, err.max())
            assert np.sqrt((err ** 2).mean()) <= 2e-3 * np.sqrt((ref ** 2).mean()) + 1e-3


@pytest.mark.parametrize("P", [16, 32, 64, 256])
def test_attend_paged_ragged(P):
    lengths = [[1, 0, 15, 16], [17, 31, 32, 33], [63, 64, 65, 511], [512, 513, 1100, 2049]]
    _attend_case(lengths, P, 0, None, HQ=16, seed=P)


@pytest.mark.parametrize("P", [16, 128])
def test_attend_paged_with_ring(P):
    lengths = [[0, 5, 300], [40, 0, 1000], [7, 700, 33], [0, 0, 0]]
    _attend_case(lengths, P, 128, [0, 5, 128, 100000], HQ=12, seed=100 + P)


def test_attend_paged_peaked_and_small_bound():
    _attend_case([[2000, 600], [1500, 40]], 16, 128, [128, 9], HQ=16, seed=7, q_gain=8.0, max_rows=100)


def test_paged_pipeline_end_to_end():
    """mask -> assign_pages -> compact_paged -> attend_decode_paged equals attention over the
    oracle's pruned cache."""
    B, H, T, D, w, P, HQ = 2, 4, 3000, 128, 128, 32, 16
    K, V, idx, n, off, ref = _pruned_case(B, H, T, D, w, seed=11, keep=0.3)
    max_pages = T // P + 1
    num_pages = int(ref.lengths.sum()) // P + B * H + 3
    free = torch.randperm(num_pages, dtype=torch.int32).to(DEV)
    table, res = binding.kvzap_assign_pages(n, P, free, max_pages)
    assert int(res[1]) == 0
    Kp = torch.zeros((num_pages, P, D), dtype=torch.bfloat16, device=DEV)
    Vp = torch.zeros_like(Kp)
    binding.kvzap_compact_paged(K, V, idx, n, off, table, P, Kp, Vp)
    q = synth.make_attend_inputs(B, H, HQ, D, 1, 0, 12, DEV)[0]
    out = binding.kvzap_attend_decode_paged(q, Kp, Vp, table, P, n, None, None, None, 0, T, D ** -0.5)
    caches = []
    for b in range(B):
        row = []
        for h in range(H):
            i = b * H + h
            row.append((O.bf16_bits_to_f64(ref.K_out[ref.offsets[i]:ref.offsets[i + 1]]),
                        O.bf16_bits_to_f64(ref.V_out[ref.offsets[i]:ref.offsets[i + 1]])))
        caches.append(row)
    want = O.attend_decode(synth.f64(q), caches, D ** -0.5)
    err = np.abs(out.to(torch.float64).cpu().numpy() - want)
    assert err.max() <= 2.0 ** -7 * 6.0, err.max()


def test_paged_calls_reject_bad_arguments():
    L = binding.lib()
    z = torch.zeros(64, dtype=torch.int32, device=DEV)
    ws = torch.empty(4096, dtype=torch.uint8, device=DEV)
    args = lambda page_rows, max_pages: (z.data_ptr(), 1, 2, page_rows, 0, z.data_ptr(), 4, z.data_ptr(),
                                         max_pages, z.data_ptr(), ws.data_ptr(), ws.numel(), None)
    assert L.kvzap_assign_pages(*args(16, 4)) == 0
    assert L.kvzap_assign_pages(*args(24, 4)) == -2       # not a power of two
    assert L.kvzap_assign_pages(*args(8, 4)) == -2        # below 16
    assert L.kvzap_assign_pages(*args(16, 0)) == -2
    torch.cuda.synchronize()


def test_extend_pages_matches_oracle_over_many_rounds():
    rng = np.random.default_rng(21)
    B, H, P, max_pages = 3, 5, 16, 40
    lengths = np.zeros((B, H), np.int64)
    counts = np.zeros(B * H, np.int32)
    table = np.full((B * H, max_pages), -1, np.int32)
    free = rng.permutation(2000).astype(np.int32)
    d_counts = _i32(counts).reshape(B, H).contiguous()
    d_table = _i32(table)
    used_total = 0
    for rnd in range(12):
        lengths += rng.integers(0, 40, (B, H))
        res = binding.kvzap_extend_pages(_i32(lengths), d_counts, P, _i32(free[used_total:]), d_table,
                                         reserve_rows=8)
        table, counts, used, ok = O.extend_pages(lengths, counts, table, P, free[used_total:], 8)
        assert ok and res[:2].tolist() == [used, 0], rnd
        used_total += used
        np.testing.assert_array_equal(parity.to_np(d_table), table)
        np.testing.assert_array_equal(parity.to_np(d_counts).reshape(-1), counts)
    # failure leaves table and counts as they were
    before_t, before_c = parity.to_np(d_table).copy(), parity.to_np(d_counts).copy()
    res = binding.kvzap_extend_pages(_i32(lengths + 400), d_counts, P, _i32(free[used_total:]), d_table)
    assert res[:2].tolist() == [0, 2]                  # a head would exceed the table width
    res = binding.kvzap_extend_pages(_i32(lengths + 64), d_counts, P, _i32(free[:3]), d_table)
    assert res[:2].tolist() == [0, 1]                  # free list too short
    np.testing.assert_array_equal(parity.to_np(d_table), before_t)
    np.testing.assert_array_equal(parity.to_np(d_counts), before_c)


def _paged_canonical(st, b, h):
    bh = b * st.H + h
    n = int(st.lengths.reshape(-1)[bh]); p = int(st.seq_pos[b]); P = st.page_rows
    row = parity.to_np(st.block_table)[bh]
    Kc = O.gather_from_pages(parity.to_np(st.K_pool), row, n, P)
    Vc = O.gather_from_pages(parity.to_np(st.V_pool), row, n, P)
    pos = O.gather_from_pages(parity.to_np(st.pos_pool)[:, :, None], row, n, P)[:, 0].astype(np.int64)
    w = st.window
    win = list(range(max(p - w, 0), p)) if w > 0 else []
    slots = [t % w for t in win]
    Kw = parity.to_np(st.K_ring[b, h])[slots] if win else np.zeros((0, st.D), np.uint16)
    Vw = parity.to_np(st.V_ring[b, h])[slots] if win else np.zeros((0, st.D), np.uint16)
    return (np.concatenate([pos, np.array(win, np.int64)]),
            np.concatenate([Kc, Kw]), np.concatenate([Vc, Vw]))


@pytest.mark.parametrize("w,P,steps", [(0, 16, 70), (4, 16, 90), (128, 32, 300)])
def test_decode_evict_paged_equals_the_slab_form_and_the_oracle(w, P, steps):
    """The same token stream through kvzap_decode_evict (slabs) and kvzap_decode_evict_paged
    (pages topped up every few steps by kvzap_extend_pages): identical canonical caches, and
    equal to the decode oracle's with exact-integer linear scores."""
    from tests.test_gpu_decode import _canonical_gpu
    B, H, D, Dh, tau = 3, 4, 128, 256, 1.0
    T = steps
    hid, wts = synth.make_exact_case(T, Dh, H, 0, seed=w + P)
    hid = hid.expand(B, T, Dh).contiguous()
    hid = hid + torch.arange(B).view(B, 1, 1).to(torch.bfloat16)          # sequences differ
    K = synth.make_scores(B, H, T * D, seed=1).view(B, H, T, D).bfloat16()
    V = synth.make_scores(B, H, T * D, seed=2).view(B, H, T, D).bfloat16()
    ow = synth.oracle_weights(wts)
    S = np.stack([O.score_linear(O.bf16_bits_to_f64(synth.bits(hid[b])), ow["W"], ow["b"])
                  for b in range(B)])
    dec = O.DecodeOracle(B, H, w, tau)
    slab = binding.DecodeState(B, H, D, w, np.full((B, H), T + 1), DEV)
    max_pages = T // P + 2
    paged = binding.PagedDecodeState(B, H, D, w, P, B * H * max_pages, max_pages, DEV)
    free = torch.randperm(paged.num_pages, dtype=torch.int32).to(DEV)
    used = 0
    d = {k: (None if v is None else v.to(DEV)) for k, v in wts.items()}
    hid_d, K_d, V_d = hid.to(DEV), K.to(DEV), V.to(DEV)
    every = 5                                           # pages topped up every 5 steps, room for 5 rows
    for t in range(T):
        if t % every == 0:
            res = binding.kvzap_extend_pages(paged.lengths, paged.page_counts, P, free[used:],
                                             paged.block_table, reserve_rows=every)
            assert int(res[1]) == 0
            used += int(res[0])
        args = (hid_d[:, t].contiguous(), d["W1"], d["b1"], None, None,
                K_d[:, :, t].contiguous(), V_d[:, :, t].contiguous())
        binding.kvzap_decode_evict(*args, slab, tau)
        binding.kvzap_decode_evict_paged(*args, paged, tau)
        dec.step(S[:, :, t], synth.bits(K[:, :, t]), synth.bits(V[:, :, t]))
    torch.cuda.synchronize()
    assert int(paged.error_flag[0]) == 0 and int(slab.error_flag[0]) == 0
    np.testing.assert_array_equal(parity.to_np(paged.lengths), parity.to_np(slab.lengths))
    kept = 0
    for b in range(B):
        for h in range(H):
            pp, Kp_, Vp_ = _paged_canonical(paged, b, h)
            ps, Ks_, Vs_ = _canonical_gpu(slab, b, h)
            rpos, rK, rV = dec.canonical(b, h)
            np.testing.assert_array_equal(pp, ps)
            np.testing.assert_array_equal(Kp_, Ks_); np.testing.assert_array_equal(Vp_, Vs_)
            np.testing.assert_array_equal(pp, rpos)
            np.testing.assert_array_equal(Kp_, rK.reshape(-1, D))
            kept += len(pp)
    assert kept < B * H * T                             # something was evicted


def test_decode_evict_paged_without_a_page_sets_the_error_flag():
    B, H, D, Dh, w, P = 1, 2, 128, 256, 2, 16
    hid, wts = synth.make_exact_case(40, Dh, H, 0, seed=1)
    st = binding.PagedDecodeState(B, H, D, w, P, 4, 2, DEV)
    st.block_table.copy_(torch.tensor([[0, -1], [1, 77]], dtype=torch.int32))     # one page each
    d = {k: (None if v is None else v.to(DEV)) for k, v in wts.items()}
    kv = torch.ones((B, H, D), dtype=torch.bfloat16, device=DEV)
    for t in range(40):
        binding.kvzap_decode_evict_paged(hid[:, t].to(DEV).contiguous(), d["W1"], d["b1"], None, None,
                                         kv, kv, st, float("-inf"))
    torch.cuda.synchronize()
    assert int(st.error_flag[0]) == 1
    assert (parity.to_np(st.lengths) == P).all()        # never beyond the pages a head owns
    assert (parity.to_np(st.pos_pool)[2:] == -1).all()  # pages 2, 3 untouched
