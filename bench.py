#!/usr/bin/env python3
"""Benchmark of the WindowQuant hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch:
    wq_window_scores -> wq_assign_bits -> wq_reorder_quantize -> wq_decode_attention
on the long-video 7B-shaped configuration (4 sequences x (256 frames x 196 visual + 512 text tokens),
28 query / 4 KV heads, head_dim 128, bf16, bit mix 10/40/50 % at 8/4/2 bits, group 64).

The packed cache of one layer (about 105 MB) fits the GPU's last-level cache, which a real decoder never
enjoys (27 other layers stream through between two visits).  So the step quantizes into one of N_COPIES packed
caches and decodes from the one written longest ago; with 8 copies about 3 GB of other traffic separate the
write of a cache from its read.

Prints ONE JSON line.  `value` is the decode-attention rate: algorithmic bytes of the packed cache divided
by the duration of a decode call: 10 warm-up calls, then 512 calls on rotated caches timed as 16 batches of 32
back-to-back calls (HIP events on the launch stream around each batch); the median of the batch means, with
p10/p90 next to it.  The call is one kernel (it streams the cache and its last workgroups merge the splits).  The
roofline entry takes that kernel's own duration: the same calls captured in a HIP graph (64 per replay, 20 replays, one
event pair per replay), which leaves 0.15 us between two kernels where eager launches leave about 0.8 us and agrees with
rocprofv3's per-dispatch durations; the eager figure stands next to it (`call_us_eager`).  `streaming_only_us` is the
kernel without the merge.
The line also carries the 7B-shaped 28-layer decode loop (`decode_loop_cfg2`, one HIP graph replay per step).

`--decode-only [--mix P8,P4]` times only the decode call (optionally with every sequence at the given bit mix): the
command that the rocprofv3 counter summaries under profiles/ are made with.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
N_COPIES = 8
DECODE_BATCHES, DECODE_PER_BATCH = 16, 32     # 512 timed decode calls (8 calls per event pair read 1-2 us more per call: the markers)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measured_traffic():
    """HBM bytes per launch of the decode kernel from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE, each scaled by what the same counter reads for the plain copy probe), or None."""
    path = os.path.join(ROOT, "profiles", "decode_attention_cfg3_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(line.split(":")[1])
    except (OSError, ValueError):
        pass
    return None


def decode_loop(args):
    """The 7B-shaped decoder loop (28 layers, 8 sequences of 64 frames x 196 + 256 text tokens, bit mix 20/50/30 %):
    every decode step appends one generated token per sequence to every layer's 16-bit segment and attends over that
    layer's packed cache.  One step (28 wq_decode_append_attention calls, one kernel launch each) is captured in a HIP
    graph and replayed.
    K, V, queries and scores are drawn on the device (torch generator, same distributions as the host generator)."""
    import torch
    from paper_2605_02262_amd import binding as W
    from paper_2605_02262_amd import synth

    torch.cuda.set_device(0)
    w = synth.workload(2)
    t = synth.tables(w)
    B, L = w.B, w.layers
    steps, warm = args.steps, args.warmup
    gen = torch.Generator(device="cuda").manual_seed(w.seed)
    i32 = lambda x: torch.as_tensor(np.ascontiguousarray(x, dtype=np.int32)).cuda()
    kv_off, win_size, win_off, quota = i32(t.kv_off), i32(t.win_size), i32(t.win_off), i32(t.quota)
    total_rows, total_win = int(t.kv_off[-1]), int(t.win_off[-1])
    max_tok = int(np.diff(t.kv_off).max()) + steps + warm
    max_win = int(np.diff(t.win_off).max())
    nsplit = args.splits or W.auto_splits(B, w.Hkv, max_tok)
    ctx = W.Context(W.workspace_bytes(B, w.Hq, w.hd, nsplit))
    cap = [0, 0, 0]
    n16 = []
    for sq in w.seqs:
        n_top, n4, n2 = sq.quota
        for c, n in enumerate((n2, n4, n_top)):
            cap[c] += (n * sq.win_size + 31) // 32 * 32
        n16.append(sq.n_text + steps + warm + 8)
    off16 = np.concatenate([[0], np.cumsum(n16)]).astype(np.int32)
    sm_scale = 1.0 / float(np.sqrt(w.hd))
    caches, qs, kn, vn = [], [], [], []
    randn = lambda *s: torch.randn(*s, generator=gen, device="cuda", dtype=torch.float32)
    for layer in range(L):
        csc = torch.exp(w.sigma_k * randn(w.Hkv, w.hd))                      # key channel outliers, lognormal
        K = (randn(total_rows, w.Hkv, w.hd) * csc).to(torch.bfloat16)
        V = randn(total_rows, w.Hkv, w.hd).to(torch.bfloat16)
        scores = torch.rand(total_win, generator=gen, device="cuda")
        bits, perm, seg = W.wq_assign_bits(ctx, scores, win_off, max_win, W.MODE_QUOTA, quota, None, w.top_bits, w.pin_first)
        pk = W.PackedKV(B, w.Hkv, w.hd, w.group, torch.bfloat16, cap, off16)
        W.wq_reorder_quantize(ctx, K, V, kv_off, win_size, win_off, perm, seg, total_rows, pk)
        caches.append(pk)
        q = randn(B, w.Hq, w.hd)
        rep = w.Hq // w.Hkv                                                  # logits over the sequence: std 2
        sd = sm_scale * torch.sqrt(((q.view(B, w.Hkv, rep, w.hd) * csc[None, :, None, :]) ** 2).sum(-1)).view(B, w.Hq, 1)
        qs.append((q * (w.logit_std / sd)).to(torch.bfloat16))
        kn.append((randn(B, w.Hkv, w.hd) * csc).to(torch.bfloat16))
        vn.append(randn(B, w.Hkv, w.hd).to(torch.bfloat16))
        del K, V
    torch.cuda.synchronize()
    assert ctx.device_status() == 0
    outs = [torch.empty(B, w.Hq, w.hd, dtype=torch.float32, device="cuda") for _ in range(L)]

    def one_step():
        for layer in range(L):
            if args.separate_append:
                W.wq_append_kv(ctx, kn[layer], vn[layer], caches[layer])
                W.wq_decode_attention(ctx, qs[layer], caches[layer], sm_scale, nsplit, max_tok, W.DECODE_AUTO, out=outs[layer])
            else:
                W.wq_decode_append_attention(ctx, qs[layer], caches[layer], kn[layer], vn[layer], sm_scale, nsplit, max_tok,
                                             W.DECODE_AUTO, out=outs[layer])

    bytes0 = sum(pk.bytes_algorithmic() for pk in caches)
    row_bytes = L * B * w.Hkv * w.hd * 2 * 2                                 # 16-bit rows added per step, all layers
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    # eager reference of the first step's outputs (the graph must reproduce them: same cache state, fixed order)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        ctx.set_stream(side)
        one_step()                                                           # step 1, eager, also warms the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            one_step()
    ctx.set_stream(side)
    with torch.cuda.stream(side):
        for _ in range(max(warm - 2, 0)):
            graph.replay()
        side.synchronize()
        e0.record(side)
        for _ in range(steps):
            graph.replay()
        e1.record(side)
        side.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / steps
    status = ctx.device_status()
    len16 = caches[0].len16.cpu().numpy()
    mean_rows = max(warm, 2) + (steps + 1) / 2.0                             # rows appended before + during the timed steps
    bytes_step = bytes0 + mean_rows * row_bytes
    # eager loop for comparison (launch-bound without the graph)
    with torch.cuda.stream(side):
        e0.record(side)
        n_eager = 8
        for _ in range(n_eager):
            one_step()
        e1.record(side)
        side.synchronize()
    us_eager = e0.elapsed_time(e1) * 1e3 / n_eager
    finite = all(bool(torch.isfinite(o).all().item()) for o in outs)
    res = {"metric": "mixed-precision KV decode loop us/step (28 layers, HIP graph) and GB/s", "value": round(bytes_step / (us * 1e-6) / 1e9, 1),
           "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warm, "ms_per_step": round(us * 1e-3, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16 cache in, 2/4/8-bit codes, f16 MFMA, fp32 accumulate",
           "data": "synthetic (device generator, LLaVA-OneVision-shaped)",
           "config": {"workload": w.name + "-decode-loop", "layers": L, "B": B, "Hq": w.Hq, "Hkv": w.Hkv, "head_dim": w.hd,
                      "group": w.group, "visual_tokens_per_seq": w.seqs[0].n_vis, "text_tokens_per_seq": w.seqs[0].n_text,
                      "bit_mix_windows_8_4_2": list(map(int, w.seqs[0].quota)), "splits": nsplit},
           "us_per_step_graph": round(us, 1), "us_per_layer": round(us / L, 2), "us_per_step_eager": round(us_eager, 1),
           "bytes_per_step": int(bytes_step), "pct_hbm_peak": round(100 * bytes_step / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 1),
           "launches_per_layer": 2 if args.separate_append else 1,
           "rows_appended_per_sequence": int(len16[0] - w.seqs[0].n_text), "device_status": status, "outputs_finite": finite}
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--config", type=int, default=3, help="workload id (3 = long-video 7B-shaped layer)")
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--separate-append", action="store_true",
                    help="with --decode-loop: wq_append_kv + wq_decode_attention per layer instead of the one-call step")
    ap.add_argument("--decode-loop", action="store_true",
                    help="only time the 28-layer decode loop of the 7B-shaped batch-8 workload (one step = one HIP graph replay)")
    ap.add_argument("--no-decode-loop", action="store_true", help="leave the 28-layer decode loop out of the default run")
    ap.add_argument("--decode-only", action="store_true",
                    help="only the decode call on rotated caches (prints its timing line); with --mix P8,P4 all sequences get that bit mix")
    ap.add_argument("--mix", type=str, default="", help="with --decode-only: percentages of 8- and 4-bit windows, e.g. 0,0 = all 2-bit")
    ap.add_argument("--frames", type=int, default=0,
                    help="with --decode-only: every sequence gets this many video frames (the bit mix keeps its percentages): decode time against cache size")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_02262_amd import binding as W
    from paper_2605_02262_amd import synth

    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.decode_loop:
        if args.steps == 40:
            args.steps = 128
        print(json.dumps(decode_loop(args)), flush=True)
        return
    torch.cuda.set_device(0)
    TD = {synth.F32: torch.float32, synth.BF16: torch.bfloat16, synth.F16: torch.float16}

    w = synth.workload(args.config)
    if args.frames and not args.decode_only:
        raise SystemExit("bench.py: --frames goes with --decode-only")
    if args.mix or args.frames:
        for sq in w.seqs:
            if args.mix:
                p8, p4 = [int(x) for x in args.mix.split(",")]
            else:
                p8, p4 = round(100 * sq.quota[0] / sq.n_win), round(100 * sq.quota[1] / sq.n_win)
            if args.frames:
                sq.frames = args.frames
            sq.quota = synth.mix_to_quota(sq.n_win, p8, p4)
        w.pin_first = 0                     # (a pinned first window would not fit a mix without 8-bit windows)
    t = synth.tables(w)
    B = w.B
    t0 = time.time()
    # ---- seeded synthetic inputs, resident in HBM before anything is timed ----------------------------------
    ev_parts, et_parts, k_parts, v_parts, q_parts = [], [], [], [], []
    for b in range(B):
        if not args.decode_only:
            et, ev = synth.embeddings(w, b)
            ev_parts.append(torch.from_numpy(ev).to(TD[w.dtype]).cuda())
            et_parts.append(torch.from_numpy(et).to(TD[w.dtype]).cuda())
            del ev, et
        k, v = synth.keys_values(w, b)
        q_parts.append(synth.query(w, b, k))
        k_parts.append(torch.from_numpy(k).to(TD[w.dtype]).cuda())
        v_parts.append(torch.from_numpy(v).to(TD[w.dtype]).cuda())
        if b == 0:
            k0_host, v0_host = k, v
        del k, v
    if not args.decode_only:
        E_v, E_t = torch.cat(ev_parts), torch.cat(et_parts)
    K, V = torch.cat(k_parts), torch.cat(v_parts)
    q_host = np.stack(q_parts)
    q = torch.from_numpy(q_host).to(TD[w.dtype]).cuda()
    del ev_parts, et_parts, k_parts, v_parts
    log(f"[bench] inputs ready in {time.time() - t0:.1f}s: K {tuple(K.shape)}")

    i32 = lambda x: torch.as_tensor(np.ascontiguousarray(x, dtype=np.int32)).cuda()
    vis_off, txt_off, kv_off = i32(t.vis_off), i32(t.txt_off), i32(t.kv_off)
    win_size, win_off, quota = i32(t.win_size), i32(t.win_off), i32(t.quota)
    total_vis, total_txt, total_win = int(t.vis_off[-1]), int(t.txt_off[-1]), int(t.win_off[-1])
    total_rows = int(t.kv_off[-1])
    max_tok = int(np.diff(t.kv_off).max())
    max_win = int(np.diff(t.win_off).max())
    cap = [0, 0, 0]
    n16 = []
    for s in w.seqs:
        n_top, n4, n2 = s.quota
        for c, n in enumerate((n2, n4, n_top if w.top_bits == 8 else 0)):
            cap[c] += (n * s.win_size + 31) // 32 * 32
        n16.append((n_top if w.top_bits == 16 else 0) * s.win_size + (s.n_vis - s.n_win * s.win_size) + s.n_text + 64)
    off16 = np.concatenate([[0], np.cumsum(n16)]).astype(np.int32)
    # sequences of very different lengths (workload 4): splits by length, the library's count for them; nsplit is the count
    # the decode calls end up with, for the workspace and the report
    plain = W.auto_splits(B, w.Hkv, max_tok)
    ragged = W.auto_splits_ragged(B, w.Hkv, max_tok, sum(cap) + int(off16[-1]))
    by_length = W.DECODE_BY_LENGTH if (ragged > plain and not args.splits) else 0
    nsplit = args.splits or (ragged if by_length else plain)
    ctx = W.Context(W.workspace_bytes(B, w.Hq, w.hd, nsplit, total_vis, total_txt, w.D))
    copies = [W.PackedKV(B, w.Hkv, w.hd, w.group, TD[w.dtype16], cap, off16) for _ in range(N_COPIES)]
    sm_scale = 1.0 / float(np.sqrt(w.hd))
    out = torch.empty(B, w.Hq, w.hd, dtype=torch.float32, device="cuda")
    lse = torch.empty(B, w.Hq, dtype=torch.float32, device="cuda")
    scores = torch.empty(total_win, dtype=torch.float32, device="cuda")

    def prefill(pk):
        if args.decode_only:
            scores.copy_(torch.rand(total_win, generator=torch.Generator(device="cuda").manual_seed(w.seed), device="cuda"))
        else:
            W.wq_window_scores(ctx, E_v, E_t, vis_off, txt_off, win_size, win_off, total_vis, total_txt, total_win, scores=scores)
        bits, perm, seg = W.wq_assign_bits(ctx, scores, win_off, max_win, W.MODE_QUOTA, quota, None, w.top_bits, w.pin_first)
        W.wq_reorder_quantize(ctx, K, V, kv_off, win_size, win_off, perm, seg, total_rows, pk)
        return bits, perm, seg

    for pk in copies:                       # every copy holds a valid cache before the first decode
        bits, perm, seg = prefill(pk)
    torch.cuda.synchronize()
    assert ctx.device_status() == 0
    alg_bytes = copies[0].bytes_algorithmic()

    def step(i):
        pk_w, pk_r = copies[i % N_COPIES], copies[(i + 1) % N_COPIES]
        W.wq_window_scores(ctx, E_v, E_t, vis_off, txt_off, win_size, win_off, total_vis, total_txt, total_win, scores=scores)
        bits_, perm_, seg_ = W.wq_assign_bits(ctx, scores, win_off, max_win, W.MODE_QUOTA, quota, None, w.top_bits, w.pin_first)
        W.wq_reorder_quantize(ctx, K, V, kv_off, win_size, win_off, perm_, seg_, total_rows, pk_w)
        W.wq_decode_attention(ctx, q, pk_r, sm_scale, args.splits, max_tok, W.DECODE_AUTO | by_length, out=out, lse=lse)

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn, n):
        """mean microseconds of fn(i) over n back-to-back calls: one HIP event before the first, one after the last"""
        torch.cuda.synchronize()
        e0.record()
        for i in range(n):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / n

    # ---- the decode call on rotated caches: 10 warm-up calls, then DECODE_BATCHES batches of DECODE_PER_BATCH back-to-back
    #      calls, one pair of HIP events around each batch (a pair around every call puts 1-3 us of marker overhead into a
    #      kernel of under 30 us, a pair around 8 calls still 1-2 us per call); median and spread over the batch means ------
    dec = lambda algo: (lambda i: W.wq_decode_attention(ctx, q, copies[i % N_COPIES], sm_scale, args.splits, max_tok, algo | by_length, out=out, lse=lse))

    def decode_stats(algo):
        for i in range(10):
            dec(algo)(i)
        means = np.array([timed(dec(algo), DECODE_PER_BATCH) for _ in range(DECODE_BATCHES)])
        return {"median": float(np.median(means)), "p10": float(np.percentile(means, 10)), "p90": float(np.percentile(means, 90)),
                "mean": float(means.mean()), "calls": DECODE_BATCHES * DECODE_PER_BATCH, "calls_per_event_pair": DECODE_PER_BATCH}

    def decode_graph_stats(algo, calls=64, replays=20):
        """the decode call as a serving loop would launch it: `calls` calls (over the rotated caches) captured once in a HIP
        graph, one event pair on the replay's stream around every replay.  A replay leaves 0.15 us between two kernels
        (eager launches: about 0.8 us) and repeats to 0.2 %."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        means = []
        with torch.cuda.stream(side):
            ctx.set_stream(side)
            for i in range(N_COPIES):
                dec(algo)(i)
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                for i in range(calls):
                    dec(algo)(i)
            for _ in range(3):
                graph.replay()
            side.synchronize()
            for _ in range(replays):
                g0.record(side)
                graph.replay()
                g1.record(side)
                side.synchronize()
                means.append(g0.elapsed_time(g1) * 1e3 / calls)
        ctx.set_stream(torch.cuda.current_stream())
        means = np.array(means)
        return {"median": float(np.median(means)), "p10": float(np.percentile(means, 10)), "p90": float(np.percentile(means, 90)),
                "mean": float(means.mean()), "calls": calls * replays, "calls_per_replay": calls}

    dstat = decode_stats(W.DECODE_AUTO)                                       # the whole call: one kernel
    gstat = decode_graph_stats(W.DECODE_AUTO)                                 # ... launched from a captured graph
    kstat = decode_stats(W.DECODE_AUTO | W.DECODE_PARTIALS_ONLY)             # ... without the merge of the splits
    # the library's own ring of event pairs around the kernel of every call (includes the markers' overhead)
    ctx.decode_timing(True)
    for i in range(64):
        dec(W.DECODE_AUTO)(i)
    ring = np.array(ctx.decode_times_us(64))
    ctx.decode_timing(False)
    dec_us, kern_mean_us = dstat["median"], kstat["median"]
    if args.decode_only:
        alg_bytes = copies[0].bytes_algorithmic()
        print(json.dumps({"workload": w.name, "mix_8_4": args.mix or "config", "frames_per_sequence": w.seqs[0].frames,
                          "tokens_per_sequence": max_tok, "splits": nsplit, "bytes": alg_bytes,
                          "decode_us": {k: round(v, 2) for k, v in dstat.items()},
                          "decode_us_graph_replay": {k: round(v, 2) for k, v in gstat.items()}, "kernel_without_merge_us": {k: round(v, 2) for k, v in kstat.items()},
                          "GBs": round(alg_bytes / dec_us / 1e3, 1), "pct_hbm_peak": round(100 * alg_bytes / dec_us / 1e3 / HBM_PEAK_GBS, 1),
                          "per_call_event_pairs_us": {"median": round(float(np.median(ring)), 2), "p10": round(float(np.percentile(ring, 10)), 2),
                                                      "p90": round(float(np.percentile(ring, 90)), 2)}}), flush=True)
        return

    # ---- the timed region: K passes of the whole hot path --------------------------------------------------
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    step_us = timed(lambda i: step(args.warmup + i), args.steps)
    wall = time.perf_counter() - t_start

    # ---- the other stages, each over back-to-back calls -----------------------------------------------------
    n = max(args.steps, 2 * N_COPIES)
    sc_us = timed(lambda i: W.wq_window_scores(ctx, E_v, E_t, vis_off, txt_off, win_size, win_off, total_vis, total_txt,
                                               total_win, scores=scores), n)
    pairwise = lambda i: W.wq_window_scores(ctx, E_v, E_t, vis_off, txt_off, win_size, win_off, total_vis, total_txt,
                                            total_win, algo=W.SCORE_PAIRWISE_MFMA, scores=scores)
    pairwise(0)                                            # (its first call loads the kernel)
    scm_us = timed(pairwise, 8)
    pair_flops = sum(2.0 * sq.n_win * sq.win_size * sq.n_text * w.D for sq in w.seqs)
    as_us = timed(lambda i: W.wq_assign_bits(ctx, scores, win_off, max_win, W.MODE_QUOTA, quota, None, w.top_bits, w.pin_first), n)
    rq_us = timed(lambda i: W.wq_reorder_quantize(ctx, K, V, kv_off, win_size, win_off, perm, seg, total_rows, copies[i % N_COPIES]), n)
    st_mean = [sc_us, as_us, rq_us, dec_us]

    # ---- operator-fusion ablation: dequantize the packed cache to 16-bit rows in memory, then plain 16-bit attention
    #      over them (what runs at every decode step without the fused kernel); two dense copies, rotated ------------
    tot = [int(sum(copies[0].cls_len[c][b].item() for c in range(3)) + copies[0].len16[b].item()) for b in range(B)]
    dense_off = np.concatenate([[0], np.cumsum(tot)]).astype(np.int32)
    dense = [W.PackedKV(B, w.Hkv, w.hd, w.group, TD[w.dtype16], [0, 0, 0], dense_off) for _ in range(2)]
    for i in range(2):
        W.wq_dequantize(ctx, copies[i], dense[i])
        W.wq_decode_attention(ctx, q, dense[i], sm_scale, args.splits, max_tok, W.DECODE_AUTO | by_length, out=out, lse=lse)
    nd = max(8, n // 4)
    deq_us = timed(lambda i: W.wq_dequantize(ctx, copies[i % N_COPIES], dense[i % 2]), nd)
    att16_us = timed(lambda i: W.wq_decode_attention(ctx, q, dense[i % 2], sm_scale, args.splits, max_tok, W.DECODE_AUTO | by_length, out=out, lse=lse), nd)
    unf_us = timed(lambda i: (W.wq_dequantize(ctx, copies[i % N_COPIES], dense[i % 2]),
                              W.wq_decode_attention(ctx, q, dense[i % 2], sm_scale, args.splits, max_tok, W.DECODE_AUTO | by_length, out=out, lse=lse)), nd)
    dense_bytes = sum(tot) * w.Hkv * w.hd * 2 * 2
    del dense
    gbs = alg_bytes / (dec_us * 1e-6) / 1e9
    # the kernel's own duration: a graph replay leaves 0.15 us between two kernels and agrees with rocprofv3's per-dispatch
    # durations (profiles/decode_attention_cfg3_kernel_trace.txt); back-to-back eager calls add the launch gap (about 0.8 us)
    kern_us = gstat["median"]
    kern_gbs = alg_bytes / (kern_us * 1e-6) / 1e9

    # ---- achievable stream-read rate of this GPU (plain 16-byte loads over 2 GiB) ------------------------------
    big = torch.empty(2 << 30, dtype=torch.uint8, device="cuda")
    big.zero_()
    W.wq_probe_stream(ctx, big)
    read_gbs = big.numel() / (timed(lambda i: W.wq_probe_stream(ctx, big), 5) * 1e-6) / 1e9
    # ... and how long a plain read of just this job's bytes takes (slices of the big buffer in turn, so each one is cold):
    # launch, first round trips and the last blocks weigh more at 100 MB than at 2 GiB
    job = (alg_bytes + 4095) // 4096 * 4096
    nslice = big.numel() // job
    same_us = timed(lambda i: W.wq_probe_stream(ctx, big[(i % nslice) * job:(i % nslice + 1) * job]), 40)
    half = big.numel() // 2
    W.wq_probe_stream(ctx, big[:half], big[half:])      # plain copy of 1 GiB: the reference for byte counters
    torch.cuda.synchronize()
    del big
    # ---- matrix-core rate this GPU sustains on register operands that change from product to product ---------
    W.wq_probe_mfma(ctx, True, 2048, 100)
    probe_flops = W.wq_probe_mfma(ctx, True, 2048, 1000)
    mfma_tflops = probe_flops / (timed(lambda i: W.wq_probe_mfma(ctx, True, 2048, 1000), 3) * 1e-6) / 1e12

    res = {
        "metric": "mixed-precision KV decode-attention GB/s (% HBM peak) + us/step at 50K ctx",
        "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(step_us * 1e-3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16 cache in, 2/4/8-bit codes, f16 MFMA, fp32 accumulate",
        "data": "synthetic (seeded, LLaVA-OneVision-shaped; stands in for the paper's video workloads)",
        "config": {"workload": w.name, "B": B, "Hq": w.Hq, "Hkv": w.Hkv, "head_dim": w.hd, "group": w.group,
                   "visual_tokens_per_seq": w.seqs[0].n_vis, "text_tokens_per_seq": w.seqs[0].n_text,
                   "window": w.seqs[0].win_size, "bit_mix_windows_8_4_2": list(map(int, w.seqs[0].quota)),
                   "splits": nsplit, "splits_by_length": bool(by_length), "kv_copies_rotated": N_COPIES, "calls_per_stage_timing": n},
        "decode_us_per_step": round(dec_us, 2),
        "decode_us": {k: (round(v, 2) if isinstance(v, float) else v) for k, v in dstat.items()},
        "decode_us_graph_replay": {k: (round(v, 2) if isinstance(v, float) else v) for k, v in gstat.items()},
        "decode_us_per_call_event_pairs": {"median": round(float(np.median(ring)), 2), "p10": round(float(np.percentile(ring, 10)), 2),
                                           "p90": round(float(np.percentile(ring, 90)), 2), "calls": int(ring.size),
                                           "note": "one HIP event pair per call around the kernel (wq_decode_times_us): includes the markers' overhead"},
        "pct_hbm_peak": round(100 * gbs / HBM_PEAK_GBS, 1),
        "stage_us": {"window_scores": round(float(st_mean[0]), 1), "assign_bits": round(float(st_mean[1]), 1),
                     "reorder_quantize": round(float(st_mean[2]), 1), "decode_attention": round(dec_us, 2)},
        "stream_read_GBs": round(read_gbs, 0), "plain_read_of_the_same_bytes_us": round(same_us, 2),
        "ablation_operator_fusion": {"fused_decode_us": round(dec_us, 2), "unfused_decode_us": round(unf_us, 2),
                                     "dequantize_to_memory_us": round(deq_us, 2), "attention_16bit_us": round(att16_us, 2),
                                     "bytes_16bit_cache": dense_bytes, "speedup_of_fusion": round(unf_us / dec_us, 2),
                                     "note": "unfused = wq_dequantize (packed -> 16-bit rows in HBM) + wq_decode_attention over those rows, per step"},
        "roofline": {"kernel": "k_decode_mfma<128>", "bound": "hbm", "achieved": round(kern_gbs, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(kern_gbs / HBM_PEAK_GBS, 4),
                     "traffic": measured_traffic() if args.config == 3 else None,
                     "traffic_source": "profiles/decode_attention_cfg3_hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command, committed; not re-measured in this run)",
                     "algorithmic_bytes_per_launch": alg_bytes,
                     "kernel_us": round(kern_us, 2), "kernel_us_p10_p90": [round(gstat["p10"], 2), round(gstat["p90"], 2)],
                     "kernel_us_source": "graph replay of 64 calls over the rotated caches, 20 replays, one HIP event pair per replay on the replay's stream",
                     "call_us_eager": round(dec_us, 2), "call_us_eager_p10_p90": [round(dstat["p10"], 2), round(dstat["p90"], 2)],
                     "frac_eager_calls": round(gbs / HBM_PEAK_GBS, 4),
                     "streaming_only_us": round(kern_mean_us, 2),
                     "frac_of_stream_ceiling": round(kern_gbs / read_gbs, 4), "frac_of_plain_read": round(same_us / kern_us, 4)},
        "roofline_other": {
            "reorder_quantize": {"bound": "hbm", "unit": "GB/s",
                                 "achieved": round((total_rows * w.Hkv * w.hd * 2 * 2 + alg_bytes) / (st_mean[2] * 1e-6) / 1e9, 1)
                                 if st_mean[2] > 0 else None},
            "window_scores_pairwise_mfma": {"bound": "mfma", "unit": "TFLOP/s", "peak": 2500.0, "us": round(scm_us, 1),
                                            "achieved": round(pair_flops / (scm_us * 1e-6) / 1e12, 1),
                                            "frac": round(pair_flops / (scm_us * 1e-6) / 1e12 / 2500.0, 4),
                                            "probe_random_operands_TFLOPs": round(mfma_tflops, 1),
                                            "note": "literal pairwise form on the matrix cores; the default is the pooled form; "
                                                    "the probe is the rate of the same instruction on register operands"},
            "window_scores": {"bound": "hbm", "unit": "GB/s",
                              "achieved": round((total_vis + total_txt) * w.D * 2 / (st_mean[0] * 1e-6) / 1e9, 1)
                              if st_mean[0] > 0 else None}},
    }

    if not args.no_cpu_baseline:
        from oracle import wq_oracle as O
        # bounded sample: sequence 0 only (1 of B), decode attention over its packed cache, all Hq heads
        s0 = w.seqs[0]
        nw = s0.n_win
        bits_h, perm_h, seg_h = bits.cpu().numpy()[:nw], perm.cpu().numpy()[:nw], seg.cpu().numpy()[:1]
        rows0 = int(t.kv_off[1])
        pk0 = O.reorder_quantize(k0_host, v0_host, [0, rows0], [s0.win_size], [0, nw], perm_h, seg_h, w.group)
        tc = time.perf_counter()
        reps = 0
        while True:                         # about 10 s of CPU work on the sample
            ref = O.decode_attention(q_host[:1], pk0, sm_scale)
            reps += 1
            if time.perf_counter() - tc >= 10.0:
                break
        dt = (time.perf_counter() - tc) / reps
        bytes0 = alg_bytes / B
        # the same on one thread (the OpenMP runtime the oracle already runs on, told to use one thread; about 3 s)
        import ctypes
        gomp = ctypes.CDLL("libgomp.so.1")
        nthreads = O.num_threads()
        gomp.omp_set_num_threads(1)
        t1 = time.perf_counter()
        reps1 = 0
        while True:
            O.decode_attention(q_host[:1], pk0, sm_scale)
            reps1 += 1
            if time.perf_counter() - t1 >= 3.0:
                break
        dt1 = (time.perf_counter() - t1) / reps1
        gomp.omp_set_num_threads(nthreads)
        W.wq_decode_attention(ctx, q, copies[0], sm_scale, args.splits, max_tok, W.DECODE_AUTO | by_length, out=out)
        torch.cuda.synchronize()
        got = out[0].cpu().numpy().astype(np.float64)
        err = float((np.abs(got - ref[0]).max(axis=-1) / np.abs(ref[0]).max(axis=-1)).max())
        res["cpu_baseline"] = {"value": round(bytes0 / dt / 1e9, 4), "unit": "GB/s", "cores": nthreads,
                               "kind": "oracle", "seconds_per_pass": round(dt, 3), "passes": reps,
                               "one_thread": {"value": round(bytes0 / dt1 / 1e9, 4), "seconds_per_pass": round(dt1, 3)},
                               "sample": f"decode attention of sequence 0 of {B} (all {w.Hq} heads, {rows0} tokens), fp64"}
        res["parity_max_rel_err_seq0"] = err
    if not args.no_decode_loop:
        # the 7B-shaped decoder loop (28 layers, batch 8, 128 steps in a HIP graph) as one more key of the line
        del E_v, E_t, K, V, copies, out
        torch.cuda.empty_cache()
        la = argparse.Namespace(**vars(args))
        la.steps, la.warmup, la.splits, la.separate_append = 128, 8, 0, False
        lp = decode_loop(la)
        res["decode_loop_cfg2"] = {k: lp[k] for k in ("us_per_step_graph", "us_per_layer", "us_per_step_eager", "bytes_per_step", "pct_hbm_peak",
                                                      "launches_per_layer", "rows_appended_per_sequence", "device_status", "outputs_finite")}
        res["decode_loop_cfg2"].update({"GBs": lp["value"], "workload": lp["config"]["workload"], "steps": lp["steps"], "splits": lp["config"]["splits"]})

    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
