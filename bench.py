#!/usr/bin/env python3
"""Benchmark of the KVzap prune step (score -> mask -> compact) on one MI355X.

One "step" is one pass of the whole prune path over every layer of the workload
(default: the Qwen3-8B-shaped 128k-token prefill, 36 layers resident in HBM).
Prints ONE JSON line; `value` is prune-step tokens/sec per layer, i.e. layer-tokens
pruned per second with all inputs already in HBM.  The CPU oracle is timed next
to it on a bounded sample (a baseline, not the target) and also supplies tau.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2601_07891_amd import binding, synth  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by a plain
# streaming kernel of known size): (workload, kernel) -> bytes.  These are CONSTANTS copied from
# the named profile summaries, not re-measured by this program; the bench line says so
# (`traffic_source`), and they are refreshed whenever a kernel changes.
TRAFFIC_SOURCE = {"c3_qwen8b_128k_mlp": "constant from profiles/c3_hbm_traffic.txt",
                  "c5_qwen8b_decode+attend": "constant from profiles/c5_attend_hbm_traffic.txt"}
MEASURED_HBM_TRAFFIC = {
    ("c3_qwen8b_128k_mlp", "score_mlp_frag_kernel"): 1213.9e6 + 4.2e6,
    ("c3_qwen8b_128k_mlp", "compact_kernel"): 146.5e6 + 143.3e6,
    # profiles/c5_attend_hbm_traffic.txt (default rows-per-head range, 32 query heads)
    ("c5_qwen8b_decode+attend", "attend_partial_kernel"): 4926.1e6 + 10.4e6,
}


def _host_numerics() -> dict:
    """What the oracle's timing depends on: the cores this process may use and the BLAS behind
    numpy's float64 GEMM (the mask and the gather are single-threaded numpy)."""
    info = {"affinity_cores": len(os.sched_getaffinity(0)), "numpy": np.__version__}
    try:
        blas = np.__config__.show(mode="dicts").get("Build Dependencies", {}).get("blas", {})
        info["blas"] = f"{blas.get('name')} {blas.get('version')}"
    except Exception:
        info["blas"] = "unknown"
    return info


def _oracle_sample(wl, layer0, sample_tokens):
    """Run the float64 oracle on the first `sample_tokens` tokens of every sequence
    of layer 0 (all of them, window included, when sample_tokens == T).
    Returns (tau, cpu_baseline dict, oracle scores [B,H,sample_tokens])."""
    from oracle import kvzap_oracle as O       # cpu_baseline leg only
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    full = sample_tokens == wl.T
    window = wl.window if full else 0          # a proper prefix holds no window token
    hb = synth.bits(layer0["hidden"][:, :sample_tokens])
    Kb = synth.bits(layer0["K"][:, :, :sample_tokens])
    Vb = synth.bits(layer0["V"][:, :, :sample_tokens])
    ow = synth.oracle_weights(layer0["w"])
    B = hb.shape[0]
    t0 = time.perf_counter()
    S = []
    for b in range(B):
        h64 = O.bf16_bits_to_f64(hb[b])
        S.append(O.score_mlp(h64, ow["W1"], ow["b1"], ow["W2"], ow["b2"]) if "W1" in ow
                 else O.score_linear(h64, ow["W"], ow["b"]))
        del h64
    S = np.stack(S)
    t1 = time.perf_counter()
    tau = O.tau_at_keep_fraction(S, window, wl.keep_fraction)     # workload recipe, untimed
    t2 = time.perf_counter()
    res = O.prune(S, tau, window, Kb, Vb)
    t3 = time.perf_counter()
    total = (t1 - t0) + (t3 - t2)
    what = "all" if full else "first"
    info = {"value": B * sample_tokens / total, "unit": "tokens/s",
            "cores": int(threads), "kind": "oracle",
            "sample": f"layer 0 of {wl.name}: {what} {sample_tokens} tokens of each of {B} "
                      f"sequence(s); float64 numpy score + mask + compact, one pass",
            "score_s": t1 - t0, "mask_compact_s": t3 - t2,
            "kept_fraction": float(res.lengths.sum()) / (B * wl.H * sample_tokens),
            "host": _host_numerics()}
    return tau, info, S


def bench_decode(wl, args) -> dict:
    """Decode-phase eviction (non-default workload): every step appends one token to each of
    B sequences in each of L layers: L calls of kvzap_decode_evict per step."""
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    B, H, D, Dh, M, w = wl.B, wl.H, wl.D, wl.Dh, wl.M, wl.window
    L = args.layers or wl.L
    steps, warm = args.steps, args.warmup
    tau = 0.0
    g = torch.Generator().manual_seed(wl.seed)
    len0 = torch.randint(args.decode_cache_rows[0], args.decode_cache_rows[1] + 1, (B, H), generator=g)          # rows already kept per head
    caps = len0 + steps + warm + 8
    layers = []
    for l in range(L):
        st = binding.DecodeState(B, H, D, w, caps, dev)               # prefix content is never read
        st.lengths.copy_(len0.to(torch.int32))
        st.seq_pos.fill_(40000)
        st.score_ring.copy_(synth.make_scores(B, H, w, seed=wl.seed + l, device=dev))
        layers.append((st, synth.make_weights(wl, l, dev)))
    n_in = 8                                                           # rotating per-step inputs
    hid = [synth.make_hidden(wl, i, dev, B=1, T=B)[0].contiguous() for i in range(n_in)]
    kv = [synth.make_kv(wl, i, dev, B=B, T=1) for i in range(n_in)]
    kv = [(k[:, :, 0].contiguous(), v[:, :, 0].contiguous()) for k, v in kv]
    ws = torch.empty(max(binding.kvzap_workspace_bytes(binding.CALL_DECODE_EVICT, B, 1, Dh, M, H), 256),
                     dtype=torch.uint8, device=dev)

    def step(i):
        h, (k, v) = hid[i % n_in], kv[i % n_in]
        for st, wt in layers:
            binding.kvzap_decode_evict(h, wt["W1"], wt["b1"], wt["W2"], wt["b2"], k, v, st, tau, ws)

    for i in range(warm):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(warm + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    grown = float(torch.stack([st.lengths.float().mean() for st, _ in layers]).mean()
                  - len0.float().mean())

    # second figure: the same L calls captured once in a HIP graph and replayed (inputs are
    # copied into fixed buffers before every replay, as a model's previous layer would write
    # them); the slabs have room for exactly `steps` more tokens
    graph_ms = None
    if args.graph:
        h_in, k_in, v_in = (torch.empty_like(hid[0]), torch.empty_like(kv[0][0]),
                            torch.empty_like(kv[0][1]))

        def gstep():
            for st, wt in layers:
                binding.kvzap_decode_evict(h_in, wt["W1"], wt["b1"], wt["W2"], wt["b2"], k_in, v_in,
                                           st, tau, ws)

        for st, _ in layers:                     # back to the initial lengths: capacity for the replays
            st.lengths.copy_(len0.to(torch.int32))
        torch.cuda.synchronize()
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            gstep()
        torch.cuda.synchronize()
        reps = max(1, min(steps, warm + steps - 1))
        g0 = time.perf_counter()
        for i in range(reps):
            h, (k, v) = hid[i % n_in], kv[i % n_in]
            h_in.copy_(h); k_in.copy_(k); v_in.copy_(v)
            gr.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - g0) * 1e3 / reps
    out = {"metric": "decode-evict tokens/sec (all layers per token)", "value": B / (ms_per_step * 1e-3),
           "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warm,
           "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": wl.name, "layers": L, "batch": B, "d_model": Dh, "mlp_width": M,
                      "kv_heads": H, "head_dim": D, "window": w, "tau": tau,
                      "kept_per_step_fraction": grown / (steps + warm)},
           "us_per_layer_step": ms_per_step * 1e3 / L,
           "hip_graph": (None if graph_ms is None else
                         {"ms_per_step": graph_ms, "us_per_layer_step": graph_ms * 1e3 / L,
                          "tokens_per_s": B / (graph_ms * 1e-3)}),
           "roofline": None, "cpu_baseline": None,
           "note": "latency-bound: ~5.5 MB per layer-step; one library call per layer per step, eager"}
    return out


def bench_attend(wl, args) -> dict:
    """Decode-step attention over the ragged per-head cache (non-default stage of the decode
    workload): one step = one kvzap_attend_decode call per layer for B sequences, every
    (sequence, head) holding its own number of kept rows plus a full window ring."""
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    B, H, D, w = wl.B, wl.H, wl.D, wl.window
    HQ = args.query_heads
    L = args.layers or 4                       # 4 distinct caches (~19 GB) rotate: no reuse
    steps, warm = args.steps, args.warmup
    lo, hi = args.decode_cache_rows
    g = torch.Generator().manual_seed(wl.seed)
    lens = torch.randint(lo, hi + 1, (B, H), generator=g).to(torch.int32)
    off = torch.zeros(B * H, dtype=torch.int64)
    off[1:] = torch.cumsum(lens.reshape(-1).to(torch.int64), 0)[:-1]
    total = int(lens.sum())
    P = args.page_rows
    layers = []
    table = None
    if P:       # every head's pages scattered over the pool by a random permutation
        pages_per_head = (lens.reshape(-1).to(torch.int64) + P - 1) // P
        num_pages = int(pages_per_head.sum())
        perm = torch.randperm(num_pages, generator=g).to(torch.int32)
        table = torch.full((B * H, int(pages_per_head.max())), -1, dtype=torch.int32)
        pos = 0
        for i, c in enumerate(pages_per_head.tolist()):
            table[i, :c] = perm[pos:pos + c]
            pos += c
        table = table.to(dev)
        total = num_pages * P
    for l in range(L):
        q, Kr, Vr, Kg, Vg = synth.make_attend_inputs(B, H, HQ, D, total, w, wl.seed + l, dev)
        if P:
            Kr, Vr = Kr.view(-1, P, D), Vr.view(-1, P, D)
        layers.append((q, Kr, Vr, Kg, Vg))
    lens_d, off_d = lens.to(dev), off.to(dev)
    sp = torch.full((B,), 40000, dtype=torch.int32, device=dev)
    out = torch.empty((B, HQ, D), dtype=torch.bfloat16, device=dev)
    ws = torch.empty(binding.kvzap_workspace_bytes(binding.CALL_ATTEND_DECODE, B, hi, HQ, w, H),
                     dtype=torch.uint8, device=dev)
    scale = D ** -0.5

    def attend(q, Kr, Vr, Kg, Vg, out_):
        if P:
            return binding.kvzap_attend_decode_paged(q, Kr, Vr, table, P, lens_d, Kg, Vg, sp, w, hi,
                                                     scale, out=out_, workspace=ws)
        return binding.kvzap_attend_decode(q, Kr, Vr, off_d, lens_d, Kg, Vg, sp, w, hi, scale,
                                           out=out_, workspace=ws)

    def step():
        for q, Kr, Vr, Kg, Vg in layers:
            attend(q, Kr, Vr, Kg, Vg, out)

    for _ in range(warm):
        step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    ms_call = ev0.elapsed_time(ev1) / (steps * L)          # both kernels of one call
    rows = int(lens.sum()) + B * H * w
    bytes_call = rows * 2 * D * 2                          # K and V rows, read once
    achieved = bytes_call / (ms_call * 1e-3) / 1e9

    # CPU oracle on a bounded sample: the heads of sequence 0 of layer 0
    from oracle import kvzap_oracle as O       # cpu_baseline leg only
    q, Kr, Vr, Kg, Vg = layers[0]
    G = HQ // H
    caches = []
    for h in range(H):
        o, n = int(off[h]), int(lens[0, h])
        if P:       # rows of head (0,h) in block-table order
            pg = table[h, :(n + P - 1) // P].long()
            kh, vh = Kr[pg].reshape(-1, D)[:n], Vr[pg].reshape(-1, D)[:n]
        else:
            kh, vh = Kr[o:o + n], Vr[o:o + n]
        caches.append((synth.f64(torch.cat([kh, Kg[0, h]])), synth.f64(torch.cat([vh, Vg[0, h]]))))
    q0 = synth.f64(q[:1])
    c0 = time.perf_counter()
    ref = O.attend_decode(q0, [caches], scale)
    c1 = time.perf_counter()
    got = out  # last layer's output; recompute layer 0 for the check
    got = attend(q, Kr, Vr, Kg, Vg, None)
    err = float(np.abs(got[:1].to(torch.float64).cpu().numpy() - ref).max())
    sample_rows = sum(c[0].shape[0] for c in caches)
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    return ({
        "metric": "decode-attention tokens/sec (all layers per token)",
        "value": B / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": steps,
        "warmup": warm, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name + "+attend", "layers": L, "batch": B, "kv_heads": H,
                   "query_heads": HQ, "head_dim": D, "window": w,
                   "rows_per_head": [lo, hi], "cache_rows_per_layer": rows,
                   "layout": f"paged, {P} rows per page, pages shuffled" if P else "contiguous slabs"},
        "ms_per_call": ms_call,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": achieved / PEAK_HBM_GBS,
                     "traffic": (MEASURED_HBM_TRAFFIC.get((wl.name + "+attend", "attend_partial_kernel"))
                                 if (lo, hi, HQ, B, P) == (4096, 32768, 32, 64, 0) else None),
                     "kernel": "attend_partial_kernel (+ attend_combine_kernel in the same interval)",
                     "bytes_per_launch": bytes_call},
        "cpu_baseline": {"value": sample_rows / (c1 - c0), "unit": "cache rows/s",
                         "gpu_value_same_unit": rows / (ms_call * 1e-3),
                         "cores": int(threads), "kind": "oracle",
                         "sample": f"sequence 0 of layer 0: {H} KV heads x {G} query heads over "
                                   f"{sample_rows} cache rows, float64 numpy",
                         "max_abs_diff_vs_gpu": err}})


def bench_teacher(wl, args) -> dict:
    """Teacher scores (KVzip+ of Eq. 3) of one layer of one extended prompt: a prompt of
    --teacher-tokens tokens, a 32-token instruction, the prompt repeated (non-default stage)."""
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    H, D, HQ = wl.H, wl.D, args.query_heads
    T = Tq = args.teacher_tokens
    instr = 32
    Tk = T + instr + Tq
    nbuf = 3
    g = torch.Generator(device=dev).manual_seed(wl.seed)
    bufs = []
    for _ in range(nbuf):
        q = torch.randn((HQ, Tq, D), generator=g, device=dev).bfloat16()
        k = torch.randn((H, Tk, D), generator=g, device=dev).bfloat16()
        vn = torch.rand((H, T), generator=g, device=dev) * 3.0 + 0.1
        hn = torch.rand((Tq,), generator=g, device=dev) * 5.0 + 0.5
        bufs.append((q, k, vn, hn))
    scale = D ** -0.5
    out = torch.empty((H, T), dtype=torch.float32, device=dev)
    ws = torch.empty(binding.kvzap_workspace_bytes(binding.CALL_TEACHER_SCORES, 1, T, HQ, Tq, H),
                     dtype=torch.uint8, device=dev)

    def step(i):
        q, k, vn, hn = bufs[i % nbuf]
        binding.kvzap_teacher_scores(q, k, T, scale, vn, hn, out, ws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for i in range(args.steps):
        step(i)
    ev1.record()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_call = ev0.elapsed_time(ev1) / args.steps
    P0 = Tk - Tq
    # Eq. 1 / Eq. 3 need every a_ji of a visible (query, key) pair once: that is the method's own
    # work.  The kernels compute q.k a second time for the (query, prompt key) pairs of the
    # column pass instead of storing the first result: executed, not algorithmic.
    pairs1 = sum(P0 + j + 1 for j in range(Tq))
    flops = 2 * D * HQ * pairs1
    executed_flops = 2 * D * HQ * (pairs1 + Tq * T)
    achieved = flops / (ms_call * 1e-3) / 1e12

    from oracle import kvzap_oracle as O       # cpu_baseline leg only
    q, k, vn, hn = bufs[0]
    G = HQ // H
    c0 = time.perf_counter()
    ref = O.teacher_log_scores(synth.f64(q[:G]), synth.f64(k[:1]), scale, T, synth.f64(vn[:1]),
                               synth.f64(hn))
    c1 = time.perf_counter()
    got = binding.kvzap_teacher_scores(q, k, T, scale, vn, hn)
    err = float(np.abs(got[:1].double().cpu().numpy() - ref).max())
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    return ({
        "metric": "teacher-score prompt tokens/sec per layer (KVzip+ scores, all KV heads)",
        "value": T / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"teacher scores, prompt {T} + instruction {instr} + repeat {Tq}",
                   "kv_heads": H, "query_heads": HQ, "head_dim": D},
        "ms_per_call": ms_call,
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": None,
                     "kernel": "teacher_rowstat_kernel + teacher_colmax_kernel (one interval)",
                     "algorithmic_flops_per_launch": flops,
                     "executed_flops_per_launch": executed_flops,
                     "executed_TFLOP/s": executed_flops / (ms_call * 1e-3) / 1e12},
        "cpu_baseline": {"value": T / (c1 - c0) / H, "unit": "tokens/s", "cores": int(threads),
                         "kind": "oracle",
                         "sample": f"KV head 0 ({G} query heads) of the same prompt, float64 numpy; "
                                   f"value scaled to all {H} KV heads",
                         "max_abs_diff_vs_gpu": err}})


def bench_fused_norm(wl, args) -> dict:
    """The MLP surrogate fused into the layer's input RMSNorm (--stage fused-norm, a prefill
    workload): kvzap_score_rmsnorm reading the residual stream, with and without the normalised
    states as an output, next to kvzap_score_prepared on states normalised beforehand -- the
    scorer's cost when the norm is a kernel of its own, whose output it has to read again."""
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    B, T, H, Dh, M = wl.B, wl.T, wl.H, wl.Dh, wl.M
    L = args.layers or 6
    eps = 1e-6
    layers = []
    for l in range(L):
        w = synth.make_weights(wl, l, dev)
        x = synth.make_hidden(wl, l, dev)                 # stands for the residual stream
        g = torch.Generator(device=dev).manual_seed(900 + l)
        gain = (1.0 + 0.3 * torch.randn((Dh,), generator=g, device=dev)).bfloat16()
        layers.append(dict(w=w, x=x, gain=gain, normed=torch.empty_like(x),
                           prep=binding.kvzap_prepare_scorer(w["W1"]),
                           prep_n=binding.kvzap_prepare_scorer_rmsnorm(w["W1"], gain),
                           scores=torch.empty((B, H, T), dtype=torch.float32, device=dev),
                           rstd=torch.empty((B, T), dtype=torch.float32, device=dev)))
    torch.cuda.synchronize()

    def plain(ly):      # the norm ran as its own kernel before: its output is read here
        w = ly["w"]
        binding.kvzap_score_prepared(ly["normed"], ly["prep"], w["b1"], w["W2"], w["b2"], ly["scores"])

    def fused(ly):
        w = ly["w"]
        binding.kvzap_score_rmsnorm(ly["x"], ly["prep_n"], ly["gain"], eps, w["b1"], w["W2"], w["b2"],
                                    False, ly["scores"], ly["rstd"])

    def fused_normed(ly):
        w = ly["w"]
        binding.kvzap_score_rmsnorm(ly["x"], ly["prep_n"], ly["gain"], eps, w["b1"], w["W2"], w["b2"],
                                    True, ly["scores"], ly["rstd"], ly["normed"])

    def torch_norm(ly):  # context only: the framework's own RMSNorm kernel, bf16 in and out
        torch.nn.functional.rms_norm(ly["x"], (Dh,), ly["gain"], eps)

    def timed(fn):
        for ly in layers:
            fn(ly)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(args.steps):
            for ly in layers:
                fn(ly)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (args.steps * L), (time.perf_counter() - t0) * 1e3 / args.steps

    for ly in layers:
        fused_normed(ly)                                  # fills `normed` for the plain variant
    ms_plain, _ = timed(plain)
    ms_fused, ms_step = timed(fused)
    ms_fused_normed, _ = timed(fused_normed)
    ms_torch, _ = timed(torch_norm)
    row = B * T * Dh * 2                                  # bytes of one [B,T,Dh] bf16 tensor
    flops = (2 * Dh * M + 2 * M * H) * B * T
    return {
        "metric": "fused-norm scorer tokens/sec per layer (scores + row scales from the residual stream)",
        "value": L * B * T / (ms_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": 1, "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name + "+fused-norm", "layers": L, "batch": B, "seq_len": T,
                   "d_model": Dh, "mlp_width": M, "kv_heads": H, "eps": eps},
        "ms_per_layer": {"kvzap_score_prepared on normalised states": ms_plain,
                         "kvzap_score_rmsnorm (scores + rstd)": ms_fused,
                         "kvzap_score_rmsnorm (scores + rstd + normalised states)": ms_fused_normed,
                         "context: torch rms_norm kernel alone": ms_torch},
        "hbm_bytes_per_layer": {
            "separate norm, then scorer": {"norm": 2 * row, "scorer": row, "total": 3 * row},
            "fused, consumer applies rstd itself": {"scorer": row, "total": row,
                                                    "saved_vs_separate_scorer_read": row},
            "fused, normalised states written": {"scorer": 3 * row, "total": 3 * row}},
        "roofline": {"kernel": "score_mlp_frag_kernel (normalising form)", "bound": "mfma",
                     "achieved": flops / (ms_fused * 1e-3) / 1e12, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": flops / (ms_fused * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                     "traffic": None, "avg_launch_ms": ms_fused,
                     "algorithmic_flops_per_launch": flops},
        "cpu_baseline": None}


def bench_prefill(wl, args, L, oracle: bool, extras: bool) -> dict:
    """Prune step (score, mask, compact) over L resident layers of a prefill workload.
    oracle: tau and the cpu_baseline come from the float64 oracle on layer 0 (the headline
    workload); otherwise tau is the keep-fraction quantile of the GPU's own layer-0 scores (it
    only sets how many rows are kept).  extras: the vendor GEMM for context."""
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    B, T, H, D, Dh, M = wl.B, wl.T, wl.H, wl.D, wl.Dh, wl.M
    P = args.page_rows

    # ---- resident inputs and preallocated outputs for every layer ----
    layers = []
    for l in range(L):
        w = synth.make_weights(wl, l, dev)
        hidden = synth.make_hidden(wl, l, dev)
        K, V = synth.make_kv(wl, l, dev)
        cap = B * H * T
        layers.append(dict(
            w=w, hidden=hidden, K=K, V=V,
            scores=torch.empty((B, H, T), dtype=torch.float32, device=dev),
            idx=torch.empty(cap, dtype=torch.int32, device=dev),
            n=torch.empty((B, H), dtype=torch.int32, device=dev),
            off=torch.empty(B * H + 1, dtype=torch.int64, device=dev),
            K_out=None if P else torch.empty((cap, D), dtype=torch.bfloat16, device=dev),
            V_out=None if P else torch.empty((cap, D), dtype=torch.bfloat16, device=dev)))
        if P:       # paged layout: room for 55 % of the rows (the configs keep 25-50 %)
            num_pages = int(cap * 0.55) // P + B * H
            layers[-1].update(
                K_pool=torch.empty((num_pages, P, D), dtype=torch.bfloat16, device=dev),
                V_pool=torch.empty((num_pages, P, D), dtype=torch.bfloat16, device=dev),
                free=torch.arange(num_pages, dtype=torch.int32, device=dev),
                table=torch.empty((B * H, T // P + 1), dtype=torch.int32, device=dev),
                pages=torch.zeros(4, dtype=torch.int32, device=dev))
    ws = torch.empty(max(binding.kvzap_workspace_bytes(binding.CALL_MASK, B, T, 0, 0, H), 256),
                     dtype=torch.uint8, device=dev)
    ws_score = torch.empty(max(binding.kvzap_workspace_bytes(binding.CALL_SCORE, B, T, Dh, M, H), 256),
                           dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()

    # ---- CPU oracle on a bounded sample: the reported baseline, and tau ----
    sample_tokens = T if args.sample_tokens <= 0 else min(args.sample_tokens, T)
    if sample_tokens < T:
        sample_tokens = min(sample_tokens, max(T - wl.window, 1))
    if oracle:
        tau, cpu_info, S_ref = _oracle_sample(wl, layers[0], sample_tokens)
    else:
        # tau only sets how many rows are kept: the keep-fraction quantile of the GPU's own
        # layer-0 scores over the non-window positions (every 8th position of every head)
        w0 = layers[0]["w"]
        s0 = binding.kvzap_score(layers[0]["hidden"], w0["W1"], w0["b1"], w0["W2"], w0["b2"])
        pool = s0[:, :, :max(T - wl.window, 1)][:, :, ::8].reshape(-1).float()
        tau = float(torch.quantile(pool[:4_000_000], 1.0 - wl.keep_fraction))
        cpu_info, S_ref, sample_tokens = None, None, 0
        del s0, pool
    if args.copy_calibration:                   # 1 GiB read + 1 GiB written by a plain copy
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.prepared_weights and M:
        for ly in layers:                            # at weight-load time, outside every timed region
            ly["w1p"] = binding.kvzap_prepare_scorer(ly["w"]["W1"])
        torch.cuda.synchronize()

    def score(ly):
        w = ly["w"]
        if args.prepared_weights and M:
            binding.kvzap_score_prepared(ly["hidden"], ly["w1p"], w["b1"], w["W2"], w["b2"], ly["scores"])
        else:
            binding.kvzap_score(ly["hidden"], w["W1"], w["b1"], w["W2"], w["b2"], ly["scores"], ws_score)

    ws_topk = torch.empty(max(binding.kvzap_workspace_bytes(binding.CALL_TOPK_THRESHOLD, B, T, 0, 1, H),
                              binding.kvzap_workspace_bytes(binding.CALL_TOPK_THRESHOLD, B, T, 0, 0, H), 256),
                          dtype=torch.uint8, device=dev)
    tau_heads = torch.empty((B, H), dtype=torch.float32, device=dev)
    k_head = int(round(wl.keep_fraction * max(T - wl.window, 0)))

    def mask(ly):
        if args.select == "threshold":
            binding.kvzap_mask(ly["scores"], tau, wl.window, None, ly["idx"], ly["n"], ly["off"], ws)
        else:       # fixed budget: the same kept fraction as a top-k per head / per layer
            per_layer = args.select == "topk-layer"
            binding.kvzap_topk_threshold(ly["scores"], wl.window, k_head * (H if per_layer else 1),
                                         per_layer, None, tau_heads, ws_topk)
            binding.kvzap_mask_per_head(ly["scores"], tau_heads, wl.window, None, ly["idx"],
                                        ly["n"], ly["off"], ws)

    ws_pages = torch.empty(max(binding.kvzap_workspace_bytes(binding.CALL_ASSIGN_PAGES, B, 1, 0, 0, H), 256),
                           dtype=torch.uint8, device=dev)

    def assign(ly):
        binding.kvzap_assign_pages(ly["n"], P, ly["free"], ly["table"].shape[1], 0, ly["table"],
                                   ly["pages"], ws_pages)

    def compact(ly):
        if P:
            assign(ly)
            binding.kvzap_compact_paged(ly["K"], ly["V"], ly["idx"], ly["n"], ly["off"], ly["table"],
                                        P, ly["K_pool"], ly["V_pool"])
        else:
            binding.kvzap_compact(ly["K"], ly["V"], ly["idx"], ly["n"], ly["off"], ly["K_out"],
                                  ly["V_out"], B * H * T)

    # Layers are independent in the prune step, so the scorer of layer l+1 may run while the
    # HBM-bound mask + compact of layer l run on a second stream (--two-streams, default priority).
    main_stream = torch.cuda.current_stream()
    side_stream = torch.cuda.Stream() if args.two_streams else main_stream

    def step(events=None):
        for ly in layers:
            if events is not None:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(main_stream)
                score(ly)
                e1.record(main_stream)
                events.append((e0, e1))
            else:
                score(ly)
            if side_stream is not main_stream:
                scored = torch.cuda.Event()
                scored.record(main_stream)
                side_stream.wait_event(scored)
            with torch.cuda.stream(side_stream):
                mask(ly)
                compact(ly)
        if side_stream is not main_stream:
            main_stream.wait_stream(side_stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # sanity: the GPU scores of the sample agree with the oracle's (not a timed part)
    score_err = None
    if S_ref is not None:
        got = layers[0]["scores"][:, :, :sample_tokens].double().cpu().numpy()
        score_err = float(np.max(np.abs(got - S_ref) / np.maximum(np.abs(S_ref), 1.0)))

    score_events = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(score_events)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_step = L * B * T
    value = tokens_per_step / (ms_per_step * 1e-3)
    score_ms = float(np.mean([a.elapsed_time(b) for a, b in score_events]))

    # ---- per-stage figures (outside the timed region) ----
    def time_stage(fn, reps=3):
        ev = []
        for _ in range(reps):
            for ly in layers:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(); fn(ly); e1.record()
                ev.append((e0, e1))
        torch.cuda.synchronize()
        return float(np.mean([a.elapsed_time(b) for a, b in ev]))

    mask_ms = time_stage(mask)
    compact_ms = time_stage(compact)
    # Algorithm 1's last three lines as ONE stage: both calls between one pair of events
    # (their kernels queue back to back), against the bytes of both
    mask_compact_ms = time_stage(lambda ly: (mask(ly), compact(ly)))
    assign_ms = None
    if P:
        if any(int(ly["pages"][1]) != 0 for ly in layers):
            print("bench.py: the page pool was too small for this workload", file=sys.stderr)
            return 1
        assign_ms = time_stage(assign)
        compact_ms -= assign_ms                   # the gather alone, for the HBM figure
    kept_rows = float(np.mean([int(ly["off"][-1]) for ly in layers]))
    kept_fraction = kept_rows / (B * H * T)

    flops_per_token = 2 * Dh * M + 2 * M * H if M else 2 * Dh * H          # App. B Eq. 5 / Eq. 6
    score_flops = flops_per_token * B * T
    row_bytes = D * 2
    compact_bytes = kept_rows * (2 * 2 * row_bytes + 4)      # read+write K and V rows, read idx
    if M:
        roofline = {"kernel": "score_mlp_frag_kernel", "bound": "mfma",
                    "achieved": score_flops / (score_ms * 1e-3) / 1e12, "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "traffic": None}
    else:
        roofline = {"kernel": "score_linear_kernel", "bound": "hbm",
                    "achieved": (B * T * (2 * Dh + 4 * H)) / (score_ms * 1e-3) / 1e9,
                    "peak": PEAK_HBM_GBS, "unit": "GB/s", "traffic": None}
    roofline["frac"] = roofline["achieved"] / roofline["peak"]
    roofline["avg_launch_ms"] = score_ms
    roofline["algorithmic_flops_per_launch" if M else "algorithmic_bytes_per_launch"] = (
        score_flops if M else B * T * (2 * Dh + 4 * H))
    if L == wl.L:
        roofline["traffic"] = MEASURED_HBM_TRAFFIC.get((wl.name, roofline["kernel"]))
        if roofline["traffic"] is not None:
            roofline["traffic_source"] = TRAFFIC_SOURCE[wl.name]
        compact_traffic = None if P else MEASURED_HBM_TRAFFIC.get((wl.name, "compact_kernel"))
    else:
        compact_traffic = None
    compact_roof = {"kernel": "compact_paged_kernel" if P else "compact_kernel", "bound": "hbm",
                    "achieved": compact_bytes / (compact_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "traffic": compact_traffic, "avg_launch_ms": compact_ms,
                    "algorithmic_bytes_per_launch": compact_bytes}
    compact_roof["frac"] = compact_roof["achieved"] / compact_roof["peak"]
    # mask: every score read once (4 B), every kept position written once (4 B)
    mc_bytes = compact_bytes + B * H * T * 4 + kept_rows * 4
    mc_roof = {"kernel": "mask_count_kernel + mask_emit_kernel + compact_kernel (one interval)",
               "bound": "hbm", "achieved": mc_bytes / (mask_compact_ms * 1e-3) / 1e9,
               "peak": PEAK_HBM_GBS, "unit": "GB/s", "traffic": None,
               "avg_launch_ms": mask_compact_ms, "algorithmic_bytes_per_launch": mc_bytes}
    mc_roof["frac"] = mc_roof["achieved"] / mc_roof["peak"]

    # context, not a target and not on the product path: the vendor library's GEMM (torch.matmul,
    # i.e. hipBLASLt) on the scorer's FIRST projection alone, same operands, bf16 output
    library_gemm = None
    if M and extras:
        hid2d = [ly["hidden"].reshape(B * T, Dh) for ly in layers]
        w1 = [ly["w"]["W1"] for ly in layers]
        z = torch.empty((B * T, M), dtype=torch.bfloat16, device=dev)
        for i in range(2):
            torch.matmul(hid2d[i % L], w1[i % L].t(), out=z)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = max(10, L)
        e0.record()
        for i in range(reps):
            torch.matmul(hid2d[i % L], w1[i % L].t(), out=z)
        e1.record(); torch.cuda.synchronize()
        gemm_ms = e0.elapsed_time(e1) / reps
        library_gemm = {"what": "torch.matmul hidden[B*T,Dh] x W1^T -> bf16 [B*T,M]; no bias, GELU or "
                                "second projection", "avg_ms": gemm_ms,
                        "TFLOP/s": 2.0 * B * T * Dh * M / (gemm_ms * 1e-3) / 1e12}
        del z

    out = {
        "metric": "prune-step tokens/sec per layer (score+mask+compact)",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "layers": L, "batch": B, "seq_len": T, "d_model": Dh,
                   "mlp_width": M, "kv_heads": H, "head_dim": D, "window": wl.window,
                   "keep_fraction_target": wl.keep_fraction, "tau": tau,
                   "kept_fraction_measured": kept_fraction, "scorer": wl.scorer,
                   "output_layout": f"paged, {P} rows per page" if P else "packed contiguous",
                   "selection": args.select,
                   "scorer_entry": "kvzap_score_prepared" if (args.prepared_weights and M) else "kvzap_score",
                   "generator": f"torch {torch.__version__} cuda philox, seeds per layer"},
        "roofline": roofline,
        "roofline_compact": compact_roof,
        "roofline_mask_compact": mc_roof,
        "stages_ms_per_layer": {"score": score_ms, "mask": mask_ms, "compact": compact_ms,
                                "mask_compact": mask_compact_ms,
                                "assign_pages": assign_ms,
                                "sum": score_ms + mask_ms + compact_ms + (assign_ms or 0.0),
                                "wall": ms_per_step / L,
                                "streams": 2 if args.two_streams else 1,
                                "note": "score timed inside the step; mask, compact and the two "
                                        "together (mask_compact, one event pair) timed alone on "
                                        "one stream after it"},
        "score_max_rel_err_vs_oracle_sample": score_err,
        "library_gemm_context": library_gemm,
        "cpu_baseline": cpu_info,
    }
    return out


def other_workloads(args) -> list:
    """The remaining configurations, each timed in this same run after the headline workload has
    released its memory: short figures (tokens/s, per-stage times, the roofline of the dominant
    kernel, kept fraction), no CPU baseline.  Layers resident: enough to exceed the 256 MB
    last-level cache several times over."""
    import copy
    import gc
    res = []

    def brief(d, keys):
        return {k: d[k] for k in keys if k in d}

    keys = ("metric", "value", "unit", "steps", "warmup", "ms_per_step", "config", "roofline",
            "roofline_compact", "roofline_mask_compact", "stages_ms_per_layer")
    for name, layers, steps in (("c1_t1k_linear", 16, 20), ("c2_llama8b_32k_mlp", 12, 10),
                                ("c4_qwen32b_4x64k_linear", 4, 5), ("c4_qwen32b_4x64k_mlp", 4, 5)):
        a = copy.copy(args)
        a.steps, a.warmup, a.sample_tokens, a.page_rows, a.select = steps, 2, 0, 0, "threshold"
        a.two_streams, a.copy_calibration = False, False
        gc.collect(); torch.cuda.empty_cache()
        res.append(brief(bench_prefill(synth.CONFIGS[name], a, layers, oracle=False, extras=False), keys))
    gc.collect(); torch.cuda.empty_cache()
    wl5 = synth.CONFIGS["c5_qwen8b_decode"]
    a = copy.copy(args)
    a.steps, a.warmup, a.layers, a.graph, a.page_rows = 32, 4, 0, True, 0
    res.append(brief(bench_decode(wl5, a), ("metric", "value", "unit", "steps", "warmup", "ms_per_step",
                                            "config", "us_per_layer_step", "hip_graph", "note")))
    gc.collect(); torch.cuda.empty_cache()
    a = copy.copy(args)
    a.steps, a.warmup, a.layers, a.page_rows = 5, 1, 0, 0
    res.append(brief(bench_attend(wl5, a), ("metric", "value", "unit", "steps", "warmup", "ms_per_step",
                                            "config", "ms_per_call", "roofline")))
    gc.collect(); torch.cuda.empty_cache()
    a = copy.copy(args)
    a.steps, a.layers = 5, 6
    res.append(brief(bench_fused_norm(synth.CONFIGS["c3_qwen8b_128k_mlp"], a),
                     ("metric", "value", "unit", "steps", "ms_per_step", "config", "ms_per_layer",
                      "hbm_bytes_per_layer", "roofline")))
    gc.collect(); torch.cuda.empty_cache()
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default=None, choices=sorted(synth.CONFIGS),
                    help="one workload only; default: the 128k-token Qwen3-8B prefill (the headline) "
                         "followed by the other configurations under the key other_workloads")
    ap.add_argument("--no-others", action="store_true",
                    help="default run: skip the other configurations")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (0 = config's)")
    ap.add_argument("--sample-tokens", type=int, default=0,
                    help="tokens per sequence the CPU oracle is timed on (0 = all of layer 0)")
    ap.add_argument("--two-streams", action="store_true",
                    help="run mask+compact of layer l on a second stream while the scorer of layer "
                         "l+1 runs (measured: +1 %% throughput, the scorer slows under contention); "
                         "default is one stream, which keeps per-kernel timings clean")
    ap.add_argument("--per-call-weights", dest="prepared_weights", action="store_false",
                    help="MLP surrogate: score with kvzap_score, which re-orders W1 into the matrix "
                         "cores' operand order on every call (5 us).  Default: the weights are "
                         "re-ordered once with kvzap_prepare_scorer when they are loaded, before the "
                         "timed region, and scored with kvzap_score_prepared, so that the event "
                         "pair around the scorer brackets its one kernel")
    ap.add_argument("--decode-cache-rows", type=int, nargs=2, default=[4096, 32768],
                    help="decode workload: range of rows already kept per (sequence, head)")
    ap.add_argument("--select", default="threshold", choices=["threshold", "topk-head", "topk-layer"],
                    help="eviction rule of the mask stage: the paper's global threshold (default) or "
                         "the fixed-budget variants of its ablation at the same kept fraction")
    ap.add_argument("--page-rows", type=int, default=0,
                    help="0 (default): packed contiguous output; a power of two >= 16: paged output "
                         "(kvzap_assign_pages + kvzap_compact_paged) and, for --stage attend, the "
                         "paged attention over a shuffled page pool")
    ap.add_argument("--graph", action="store_true",
                    help="decode workload: also time the step replayed from a HIP graph")
    ap.add_argument("--stage", default="evict", choices=["evict", "attend", "teacher", "fused-norm"],
                    help="decode workload: time the eviction step (default) or the attention "
                         "over the ragged cache it maintains; 'teacher' (any config): the "
                         "KVzip+ training scores of one extended prompt; 'fused-norm' (a prefill "
                         "config with an MLP surrogate): the surrogate fused into the layer's "
                         "input RMSNorm")
    ap.add_argument("--teacher-tokens", type=int, default=8192,
                    help="--stage teacher: prompt length (the extended prompt is twice that + 32)")
    ap.add_argument("--query-heads", type=int, default=32,
                    help="decode attention: number of query heads (Qwen3-8B: 32 over 8 KV heads)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(the path shards by layer / sequence / KV head with no communication)",
              file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    binding.lib()                                   # fail loudly if the library is not built
    wl = synth.CONFIGS[args.config or "c3_qwen8b_128k_mlp"]
    if args.stage == "teacher":
        print(json.dumps(bench_teacher(wl, args)))
        return 0
    if args.stage == "fused-norm":
        if wl.T == 1 or not wl.M:
            print("bench.py: --stage fused-norm needs a prefill workload with an MLP surrogate",
                  file=sys.stderr)
            return 2
        print(json.dumps(bench_fused_norm(wl, args)))
        return 0
    if wl.T == 1:
        print(json.dumps(bench_attend(wl, args) if args.stage == "attend" else bench_decode(wl, args)))
        return 0
    L = args.layers or wl.L
    if args.config is not None:                      # one named workload, nothing else
        print(json.dumps(bench_prefill(wl, args, L, oracle=True, extras=True)))
        return 0
    out = bench_prefill(wl, args, L, oracle=True, extras=True)
    if not args.no_others:
        out["other_workloads"] = other_workloads(args)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
