#!/usr/bin/env python3
"""Benchmark of the verification step (vote -> verify forward -> accept + commit) on one MI355X.

A step is one pass of the whole path over one batch of synthetic input, everything resident in HBM.
Default workload: the Llama-2-70B-shaped configuration, batch 16, context 1024, k = 8 (M = 144 scored
positions), bf16 weights, 16-bit KV pages (bf16-valued draws held as fp16), random-init weights, synthetic KV pages and drafts.

Prints one JSON line: throughput in verified positions/s, the roofline of the dominant kernel (the
weight-streaming projection GEMM; its device time comes from HIP events the library records around
every launch of that kernel on the launch stream), and the CPU oracle timed on the host cores on a
bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X published HBM3E bandwidth
MFMA_PEAK_TFLOPS = 2500.0    # dense bf16/fp16 MFMA


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", type=int, default=2, help="index into the workload list (default: 70B b16 k8)")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (0 = the real depth); for experiments")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="also replay the step from a captured graph and report its time beside the eager one")
    ap.add_argument("--profile-steps", type=int, default=3, help="extra steps run with the timing taps on")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device copy (a kernel of known traffic, for scaling rocprofv3 byte counters)")
    return ap.parse_args()


def measured_traffic(workload_name, kernel="gemm_w16_kernel"):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary (FETCH_SIZE +
    WRITE_SIZE scaled by a copy kernel of known size), or None when there is no summary for this workload."""
    path = os.path.join(ROOT, "profiles", "%s_%s.hbm_traffic.txt" % (kernel, workload_name))
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split("=")[1])
    except OSError:
        pass
    return None


def calibration_copy(torch, dev):
    """One 1 GiB device-to-device copy: a kernel that reads and writes a known number of bytes."""
    src = torch.empty((1 << 30,), dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


def cpu_baseline(wl, desc, M, ks, ctx, n_drafts):
    """The oracle as it stands, on the host cores: one full-shape layer at the real M and context, the LM
    head, the vote and the acceptance are timed; the layer time is multiplied by the layer count
    (the full depth would need the 137 GB of weights on the host)."""
    import numpy as np
    from oracle import minions_oracle as orc
    from paper_2402_15678_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        cores = os.cpu_count() or 1
    d1 = desc.with_layers(1)
    W = synth.make_weights(d1, wl.seed)
    kvh = synth.make_paged_kv(d1, ctx, ks, wl.seed)
    B = len(ctx)
    kv_rows = [synth.gather_sequence_kv(kvh, 0, b, int(ctx[b])) for b in range(B)]

    def fresh_caches():
        return [orc.SeqCache(1, d1.n_kv_heads, d1.head_dim, [K], [V]) for K, V in kv_rows]
    g = synth.stream(wl.seed, 900)
    k_max = int(max(ks))
    drafts = g.integers(0, desc.vocab, size=(B, n_drafts, max(1, k_max))).astype(np.int32)
    last = g.integers(0, desc.vocab, size=B).astype(np.int32)
    ssm_w = np.ones(n_drafts, np.float32)
    t0 = time.perf_counter()
    voted, _ = orc.vote_batch(drafts, ks, ssm_w)
    t_vote = time.perf_counter() - t0
    toks = [[int(last[b])] + [int(t) for t in voted[b, :ks[b]]] for b in range(B)]
    # one layer + head through the oracle's own step, repeated on fresh caches until about ten seconds of CPU
    # work have been sampled (the mean is taken); the head is timed on its own and subtracted
    reps, t_sum = 0, 0.0
    while reps < 24 and (reps < 2 or t_sum < 10.0):
        cs = fresh_caches()
        t0 = time.perf_counter()
        logits = orc.decoder_step(d1, W, toks, cs)
        t_sum += time.perf_counter() - t0
        reps += 1
    t_layer_head = t_sum / reps
    x = np.zeros((M, desc.d_model))
    t0 = time.perf_counter()
    h = orc._norm(d1, x + 1.0, W["final_norm_g"], W.get("final_norm_b"))
    orc._linear(h, W["lm_head"])
    t_head = time.perf_counter() - t0
    greedy = np.full((B, k_max + 1), -1, np.int32)
    t0 = time.perf_counter()
    for b in range(B):
        greedy[b, :len(toks[b])] = orc.greedy_tokens(logits[b])
    orc.accept_batch(voted, greedy, ks, ctx, wl.block_size)
    t_accept = time.perf_counter() - t0
    t_layer = max(t_layer_head - t_head, 1e-9)
    total = t_vote + desc.n_layers * t_layer + t_head + t_accept
    return {"value": M / total, "unit": "positions/s", "cores": int(cores), "kind": "oracle",
            "sample": "1 of %d layers at the full shape (M=%d rows, real contexts) + LM head + vote + accept, run %d "
                      "times (%.1f s of CPU work, mean taken); layer time x %d (extrapolated): layer %.2fs, head %.2fs"
                      % (desc.n_layers, M, reps, t_sum, desc.n_layers, t_layer, t_head)}


def measure_ceilings(torch, binding, harness):
    """What this machine sustains: a plain streaming read over 1 GiB and a dense fp16 MFMA loop (both in the
    library, timed here with events on the launch stream)."""
    dev = torch.device("cuda:0")
    buf = torch.empty((1 << 30,), dtype=torch.uint8, device=dev).fill_(3)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    st = harness.stream_ptr()
    for _ in range(2):
        binding.mn_probe_stream_read(buf.data_ptr(), buf.numel(), st)
    e0.record()
    for _ in range(10):
        binding.mn_probe_stream_read(buf.data_ptr(), buf.numel(), st)
    e1.record()
    torch.cuda.synchronize()
    hbm = 10.0 * buf.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del buf
    binding.mn_probe_mfma(2000, st)
    e0.record()
    flop = binding.mn_probe_mfma(100000, st)      # about 40 ms: long enough for the clocks to settle
    e1.record()
    torch.cuda.synchronize()
    mfma = flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
    binding.mn_probe_mfma_data(2000, st)
    e0.record()
    flop = binding.mn_probe_mfma_data(100000, st)
    e1.record()
    torch.cuda.synchronize()
    mfma_data = flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
    return {"hbm_stream_read_GBps": hbm, "mfma_f16_dense_TFLOPs": mfma, "mfma_f16_dense_TFLOPs_on_data": mfma_data,
            "note": "measured on this box by mn_probe_stream_read / mn_probe_mfma (constant operands, boost clock) / "
                    "mn_probe_mfma_data (operands of random sign and mantissa: the clock the chip holds on data); "
                    "the roofline peaks above are the published ones"}


def attention_only(args, wl):
    """Workload 4: the paged multi-query attention of one layer at its own shape (no model around it).
    One JSON line: KV bytes streamed per second by attn_mfma_kernel + attn_merge_kernel."""
    import numpy as np
    import torch
    from paper_2402_15678_amd import binding, harness, synth
    dev = torch.device("cuda:0")
    desc = wl.desc
    ctx = synth.draw_ctx_lens(wl)
    ks = synth.draw_spec_lens(wl)
    B = wl.batch
    total = ctx + ks + 1
    M = int((ks + 1).sum())
    tiny = synth.ModelDesc(desc.arch, desc.dtype, 1, 128, desc.n_heads, desc.n_kv_heads, desc.head_dim, 128, 8, desc.max_pos + 64)
    model = harness.DeviceModel.from_host(tiny, synth.make_weights(tiny, wl.seed))
    kvd = harness.DeviceKV.random_on_device(desc, ctx, ks, wl.seed, wl.block_size)
    q = torch.randn((M, desc.n_heads, desc.head_dim), device=dev, dtype=torch.float16)
    out = torch.empty((M, desc.n_heads * desc.head_dim), device=dev, dtype=torch.float16)
    max_ctx = int(total.max())
    wsb = binding.mn_workspace_bytes(model.ctx, B, M, max_ctx)
    ws = torch.empty((wsb,), dtype=torch.uint8, device=dev)
    spec = torch.tensor(ks, dtype=torch.int32, device=dev)
    hs = binding.host_i32(ks.tolist())
    status = torch.zeros(1, dtype=torch.int32, device=dev)

    def step():
        binding.mn_attention(model.ctx, q.data_ptr(), spec.data_ptr(), hs, B, max_ctx, kvd.c, 0, out.data_ptr(),
                             ws.data_ptr(), wsb, status.data_ptr(), harness.stream_ptr())

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    assert status.item() == 0
    if args.calibrate_copy:
        calibration_copy(torch, dev)
    binding.mn_profile_enable(model.ctx, True)
    for _ in range(max(1, args.profile_steps)):
        step()
    torch.cuda.synchronize()
    prof = binding.mn_profile_collect(model.ctx)
    binding.mn_profile_enable(model.ctx, False)
    att_ms = prof["attention"][0] / max(1, prof["attention"][1])      # attention + merge, per call
    kv_bytes = float(total.astype(np.int64).sum()) * 2 * desc.n_kv_heads * desc.head_dim * 2
    achieved = kv_bytes / (att_ms * 1e-3) / 1e9
    flops = 4.0 * desc.n_heads * desc.head_dim * float(((ks + 1).astype(np.int64) * total).sum())
    out_line = {
        "metric": "attention_kv_stream", "value": achieved, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "storage_dtype": "bf16", "accumulate_dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "batch": B, "rows": M, "ctx_min": int(ctx.min()), "ctx_max": int(ctx.max()),
                   "heads": desc.n_heads, "kv_heads": desc.n_kv_heads, "head_dim": desc.head_dim,
                   "block_size": wl.block_size, "seed": wl.seed},
        "note": "ms_per_step is one mn_attention call (row bookkeeping kernel + attention + merge); the roofline "
                "covers the attention and merge kernels, timed by the library's event taps",
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(wl.name, "attn_mfma_kernel"),
                     "algorithmic_bytes_per_launch": kv_bytes,
                     "kernel": "attn_mfma_kernel + attn_merge_kernel", "avg_launch_us": att_ms * 1e3,
                     "mfma_tflops": flops / (att_ms * 1e-3) / 1e12,
                     "mfma_frac": flops / (att_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS},
        "ceilings": measure_ceilings(torch, binding, harness),
        "cpu_baseline": None,
    }
    print(json.dumps(out_line))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); --gpus %d is not supported. "
              "Run with --gpus 1." % args.gpus, file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2402_15678_amd import binding, harness, synth

    wl = synth.WORKLOADS[args.workload]
    if wl.desc is synth.LLAMA2_70B_ATTN:
        attention_only(args, wl)
        return
    desc = wl.desc if args.layers <= 0 else wl.desc.with_layers(args.layers)
    dev = torch.device("cuda:0")
    t_setup = time.perf_counter()
    model = harness.DeviceModel.random_on_device(desc, wl.seed)
    ctx = synth.draw_ctx_lens(wl)
    ks = synth.draw_spec_lens(wl)
    B, k_max, n = wl.batch, int(ks.max()), wl.n_drafts
    M = int((ks + 1).sum())
    kvd = harness.DeviceKV.random_on_device(desc, ctx, ks, wl.seed, wl.block_size)
    max_ctx = int((ctx + ks + 1).max())
    ses = harness.VerifySession(model, kvd, B, k_max, n, max_ctx, max_rows=M)
    ctx0 = kvd.ctx_lens.clone()
    g = synth.stream(wl.seed, 600)
    last = torch.tensor(g.integers(0, desc.vocab, size=B).astype(np.int32), device=dev)

    # greedy continuation by k_max sequential single-token steps of the library itself, then roll back
    one = harness.VerifySession(model, kvd, B, 0, 1, max_ctx, max_rows=B)
    zeros = torch.zeros((B,), dtype=torch.int32, device=dev)
    cur = last.clone()
    cont = []
    dummy_voted = torch.zeros((B, 1), dtype=torch.int32, device=dev)
    for _ in range(k_max):
        one.forward(cur, zeros, [0] * B, voted=dummy_voted)
        one.accept(zeros, voted=dummy_voted)
        cur = one.next_last_tok.clone()
        cont.append(cur.cpu().numpy())
    kvd.ctx_lens.copy_(ctx0)
    cont = np.stack(cont, axis=1) if cont else np.zeros((B, 0), np.int32)   # [B][k_max]
    per = [synth.drafts_corrupted(cont[b, :ks[b]], n, wl.p_corrupt, desc.vocab, g) for b in range(B)]
    drafts = torch.tensor(synth.pack_drafts(per, max(1, k_max)), device=dev)
    spec = torch.tensor(ks, dtype=torch.int32, device=dev)
    ssm_w = torch.ones((n,), dtype=torch.float32, device=dev)
    h_spec = ks.tolist()
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup

    def step():
        kvd.ctx_lens.copy_(ctx0)          # 4*B-byte device copy: the commit of the previous step is undone
        ses.step(last, drafts, spec, h_spec, ssm_w)

    for _ in range(args.warmup):
        step()
    # one event per step boundary on the launch stream: per-step device times for the median and the minimum
    # (the headline stays wall clock over exactly K steps between two synchronisations)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    assert ses.dev_status.item() == 0
    ms_per_step = dt / args.steps * 1e3
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    acc = ses.accepted_len.cpu().numpy()

    # the same step captured once and replayed (the library only launches kernels on the caller's stream, so a
    # serving loop may do this): informational, the headline stays the eager launch sequence
    graph_ms = None
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(gr, stream=side):
                step()
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(2):
            gr.replay()
        torch.cuda.synchronize()
        tg = time.perf_counter()
        for _ in range(args.steps):
            gr.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - tg) / args.steps * 1e3
        assert ses.dev_status.item() == 0 and np.array_equal(ses.accepted_len.cpu().numpy(), acc)
        del gr

    # the two rows that close the loop after the step (not part of the timed step): the SSM weight update
    # on the device and the host-side speculation length selector
    acr_buf = torch.zeros((n,), dtype=torch.float64, device=dev)
    w_scratch = ssm_w.clone()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ses.acr_update(spec, w_scratch, 0.8, 0.4, 1.1, 0.9, acr=acr_buf)
    e0.record()
    for _ in range(50):
        ses.acr_update(spec, w_scratch, 0.8, 0.4, 1.1, 0.9, acr=acr_buf)
    e1.record()
    torch.cuda.synchronize()
    acr_us = e0.elapsed_time(e1) / 50 * 1e3
    # the general (stochastic) verification rule on this step's own scores: q = softmax(scores + N(0,1)) stands
    # in for the SSM's distributions (harness arithmetic); device time of mn_verify_sample per call; informational
    ses.logits = torch.empty((M, desc.vocab), dtype=torch.float32, device=dev)
    kvd.ctx_lens.copy_(ctx0)
    ses.forward(last, spec, h_spec)
    gq = torch.Generator(device=dev).manual_seed(wl.seed)
    q_probs = torch.zeros((B, max(1, k_max), desc.vocab), dtype=torch.float32, device=dev)
    row = 0
    for b in range(B):
        kb = int(ks[b])
        if kb:
            z = ses.logits[row:row + kb] + torch.randn((kb, desc.vocab), generator=gq, device=dev)
            q_probs[b, :kb] = torch.softmax(z, dim=-1)
        row += kb + 1
    ses.sample(spec, M, q_probs, 1.0, wl.seed, 0)
    e0.record()
    for i in range(20):
        ses.sample(spec, M, q_probs, 1.0, wl.seed, i + 1)
    e1.record()
    torch.cuda.synchronize()
    sample_us = e0.elapsed_time(e1) / 20 * 1e3
    sample_survivors = int((ses.sampled[:, :max(1, k_max)] == ses.voted)[torch.arange(max(1, k_max), device=dev)[None, :]
                                                                        < spec[:, None]].sum().item())
    kvd.ctx_lens.copy_(ctx0)
    ses.logits = None
    del q_probs
    # the step before the path: n SSMs of the paper's small-model shape drafting k tokens each through the
    # same library (random weights, synthetic caches of the same contexts); informational
    draft_ms = None
    draft_graph_ms = None
    draft_seq_ms = None
    if desc.arch == synth.ARCH_LLAMA and desc.dtype == synth.DT_BF16 and args.layers <= 0:
        sd = synth.LLAMA_160M
        s_models = [harness.DeviceModel.random_on_device(sd, wl.seed + 100 + j) for j in range(n)]
        s_kvs = [harness.DeviceKV.random_on_device(sd, ctx, ks, wl.seed + 200 + j, wl.block_size) for j in range(n)]
        dsn = harness.DraftSession(s_models, s_kvs, B, k_max, max_ctx)
        s_ctx0 = [kv.ctx_lens.clone() for kv in s_kvs]
        dsn.draft(last, k_max)
        for kv, c0 in zip(s_kvs, s_ctx0):
            kv.ctx_lens.copy_(c0)
        torch.cuda.synchronize()
        t_d = time.perf_counter()
        dsn.draft(last, k_max)
        torch.cuda.synchronize()
        draft_ms = (time.perf_counter() - t_d) * 1e3
        for kv, c0 in zip(s_kvs, s_ctx0):
            kv.ctx_lens.copy_(c0)
        torch.cuda.synchronize()
        t_d = time.perf_counter()
        dsn.draft(last, k_max, concurrent=False)
        torch.cuda.synchronize()
        draft_seq_ms = (time.perf_counter() - t_d) * 1e3
        if args.graph:
            # the drafting of all SSMs (a few thousand small launches, no host decision in between) as one graph
            for kv, c0 in zip(s_kvs, s_ctx0):
                kv.ctx_lens.copy_(c0)
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            gd = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(gd, stream=side):
                    dsn.draft(last, k_max)
            torch.cuda.current_stream().wait_stream(side)
            want_drafts = dsn.drafts.clone()
            times = []
            for _ in range(3):
                for kv, c0 in zip(s_kvs, s_ctx0):
                    kv.ctx_lens.copy_(c0)
                torch.cuda.synchronize()
                t_d = time.perf_counter()
                gd.replay()
                torch.cuda.synchronize()
                times.append((time.perf_counter() - t_d) * 1e3)
                assert torch.equal(dsn.drafts, want_drafts)
            draft_graph_ms = min(times)
            del gd
        del dsn, s_models, s_kvs
    sel = binding.mn_selector_create(max(1, k_max), 1, 64, 8, 1, 1)
    t_sel = time.perf_counter()
    for i in range(10000):
        binding.mn_selector_observe(sel, ms_per_step * (1.0 + 1e-3 * (i % 7)), float((acc + 1).mean()))
    sel_ns = (time.perf_counter() - t_sel) / 10000 * 1e9
    binding.mn_selector_destroy(sel)

    # the same steps again with the timing taps on: per-family device time from HIP events on the launch stream
    prof = None
    if args.profile_steps > 0:
        binding.mn_profile_enable(model.ctx, True)
        t0 = time.perf_counter()
        for _ in range(args.profile_steps):
            step()
        torch.cuda.synchronize()
        dt_prof = time.perf_counter() - t0
        prof = binding.mn_profile_collect(model.ctx)
        binding.mn_profile_enable(model.ctx, False)

    if args.calibrate_copy:
        calibration_copy(torch, dev)

    gemm_bytes_step = 2.0 * desc.gemm_params()          # every matrix parameter (2 bytes) is needed once per step
    roofline = None
    families = None
    if prof:
        ps = args.profile_steps
        gemm_ms, gemm_n = prof["gemm"]
        per_launch_ms = gemm_ms / max(1, gemm_n)
        achieved = gemm_bytes_step * ps / (gemm_ms * 1e-3) / 1e9 if gemm_ms > 0 else 0.0
        flops = 2.0 * M * desc.gemm_params() * ps
        tflops = flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
        roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS,
                    "traffic": measured_traffic(wl.name) if args.layers <= 0 else None,
                    "algorithmic_bytes_per_launch": gemm_bytes_step / max(1, gemm_n // ps), "kernel": "gemm_w16_kernel",
                    "launches_per_step": gemm_n // ps, "avg_launch_us": per_launch_ms * 1e3,
                    "mfma_tflops": tflops, "mfma_frac": tflops / MFMA_PEAK_TFLOPS}
        if M > MFMA_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9):
            # more rows than the machine balance (flop per weight byte = M): the projections are bound by the matrix pipe
            roofline.update({"bound": "mfma", "achieved": tflops, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                             "frac": tflops / MFMA_PEAK_TFLOPS, "traffic": None, "kernel": "gemm_big_kernel",
                             "algorithmic_flop_per_launch": flops / ps / max(1, gemm_n // ps),
                             "hbm_GBps": achieved, "hbm_frac": achieved / HBM_PEAK_GBS})
        families = {k: {"ms_per_step": v[0] / ps, "launches_per_step": v[1] // ps} for k, v in prof.items()}
        families["_instrumented_ms_per_step"] = dt_prof / ps * 1e3
        # attention: KV bytes streamed per step
        kv_bytes = float(((ctx + ks + 1).astype(np.int64)).sum()) * 2 * desc.n_kv_heads * desc.head_dim * 2 * desc.n_layers
        att_ms = prof["attention"][0] / ps
        families["attention"]["kv_GBps"] = kv_bytes / (att_ms * 1e-3) / 1e9 if att_ms > 0 else 0.0

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(wl, desc, M, ks, ctx, n)

    out = {
        "metric": "verified_positions_per_sec", "value": M / (ms_per_step * 1e-3), "unit": "positions/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "storage_dtype": "bf16 (16 bits per parameter; weights re-encoded as fp16 when packed, KV pages fp16)",
        "accumulate_dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "arch": "llama" if desc.arch == synth.ARCH_LLAMA else "opt",
                   "n_layers": desc.n_layers, "d_model": desc.d_model, "batch": B, "k_max": k_max, "rows": M,
                   "ctx_min": int(ctx.min()), "ctx_max": int(ctx.max()), "n_drafts": n, "block_size": wl.block_size,
                   "seed": wl.seed},
        "accepted_tokens_per_sec": float((acc + 1).sum()) / (ms_per_step * 1e-3),
        "acceptance_rate": float(acc.sum()) / max(1, int(ks.sum())),
        "ms_per_step_median": per_step[len(per_step) // 2], "ms_per_step_min": per_step[0],
        "setup_s": t_setup, "ms_per_step_graph_replay": graph_ms,
        "stochastic_rule": {"verify_sample_us": sample_us, "temperature": 1.0, "positions": M,
                            "speculated_tokens_surviving": sample_survivors, "speculated_tokens": int(ks.sum()),
                            "note": "mn_verify_sample on this step's scores; q = softmax(scores + N(0,1))"},
        "after_step": {"acr_update_us": acr_us, "acr": [None if x != x else x for x in acr_buf.cpu().tolist()],
                       "selector_observe_ns_incl_binding": sel_ns,
                       "ssm_drafting_ms": draft_ms, "ssm_drafting_ms_one_after_the_other": draft_seq_ms,
                       "ssm_drafting_ms_graph_replay": draft_graph_ms,
                       "ssm_drafting_note": "n SSMs of Llama-160M shape, k_max tokens each, on this GPU, one stream per SSM"},
        "roofline": roofline, "kernel_families": families,
        "ceilings": measure_ceilings(torch, binding, harness), "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
