#!/usr/bin/env python3
"""Benchmark of the ragged-cache attention path on one MI355X.

Workload (default): the full 30-layer denoising step at Wan-1.3B shape -- 30 layers x 12 heads, head_dim 128,
1560 tokens/frame, a 3-frame query chunk (4680 tokens) and 57 history frames; head types drawn 40/30/30 from the
seed (Anchor = 18 best-scored frames, Wave period 2-4, Veil = first + last 3 frames).  Every layer's pool is filled
through pf_cache_append (19 appends of 3 frames).  One timed "step" = for each of the 30 layers: pf_build_index +
pf_ragged_attn_fwd; the attention launches run back to back on one stream (layer l+1 depends on layer l in a real
model), the index builds, which depend on the pools only, on a second stream ahead of them.

The value is effective TFLOP/s over retained keys: sum over (layer, head) of 4*Lq*Lkv*D / step time.
Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np
import torch

PEAK_BF16_TFLOPS = 2516.6      # MI355X dense bf16 MFMA: 256 CU x 4096 flop/clk x 2.4 GHz
PEAK_HBM_GBS = 8000.0
APPEND_STREAMS = 4                    # side streams that take the layers' write-backs (appends, index builds) in a rollout


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c3_step", choices=["c2_layer", "c3_step", "c4_skew", "c5_stream", "c6_paper", "c7_headwin"],
                    help="c5_stream / c6_paper / c7_headwin: streaming rollouts, a step = one chunk (4 attention passes over all layers, "
                         "then append + index build per layer); --steps = chunks from an empty cache (default there: "
                         "the whole rollout)")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (0 = the workload's)")
    ap.add_argument("--layout", default="packed", choices=["packed", "model"],
                    help="chunk tensors per head [heads][tokens][D] (default) or as the model holds them, "
                         "[tokens][heads][D], through the strided entry point")
    ap.add_argument("--cpu-rows", type=int, default=3072, help="query rows per head of layer 0 timed on the CPU oracle")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--block-trace", action="store_true",
                    help="after the timed steps, run one more attention launch per layer with the library's per-workgroup "
                         "diagnostics on and report how busy each compute unit's resident workgroup was (cu_busy)")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MiB",
                    help="also run one plain device-to-device copy of this many MiB (a dispatch of known size "
                         "against which hardware traffic counters are scaled)")
    ap.add_argument("--append-probe", action="store_true",
                    help="instead of the benchmark: a few pool appends of known size (12 heads that keep every frame, then "
                         "12 top-6 heads whose survivors move) and a 64 MiB device copy, each announced with its "
                         "algorithmic bytes; for reading hardware traffic counters of the append kernel")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)
    from paper_2605_13111_amd import binding as B
    from paper_2605_13111_amd import synth
    B.lib()                                           # fail loudly if libpf.so is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.append_probe:
        return append_probe(B, synth, dev)
    if args.workload in ("c5_stream", "c6_paper", "c7_headwin"):
        return stream_bench(args, B, synth, dev)
    w = synth.WORKLOADS[args.workload]
    n_layers = args.layers or w.n_layers
    H, D, tpf = w.n_heads, w.head_dim, w.tokens_per_frame
    Lq = w.chunk_frames * tpf
    T = w.history_frames
    frame_bytes = tpf * D * 2

    # ---------------------------------------------------------------- setup: pools filled through the library
    layers = []
    hist0 = None
    append_ms, append_bytes, last_appends = [], [], []
    ev = lambda: torch.cuda.Event(enable_timing=True)
    for layer in range(n_layers):
        pols = synth.policies(w.name, layer=layer)
        pool = B.Pool(pols, tpf, D, device=dev)
        B.pf_pool_reset(pool)
        keep_k, keep_v, keep_s = [], [], []
        for ci, t0 in enumerate(range(0, T, w.chunk_frames)):
            n_new = min(w.chunk_frames, T - t0)
            seed = 100000 * (layer + 1) + 10 * ci
            k_new = synth.randn_bf16((H, n_new, tpf, D), seed, device=dev)
            v_new = synth.randn_bf16((H, n_new, tpf, D), seed + 1, device=dev)
            sc = synth.frame_scores(H, n_new, seed + 2, device=dev)
            last = t0 + n_new >= T
            if last:                                   # the append that brings the pool to T frames is timed below
                last_appends.append((pool, k_new, v_new, sc, t0, n_new))
            else:
                B.pf_cache_append(pool, k_new, v_new, sc)
            if layer == 0 and not args.no_cpu:
                keep_k.append(k_new.cpu())
                keep_v.append(v_new.cpu())
                keep_s.append(sc.cpu())
        if layer == 0 and not args.no_cpu:
            hist0 = (pols, keep_k, keep_v, keep_s)
        index = B.Index(pool, Lq)
        q = synth.randn_bf16((H, Lq, D), 900000 + layer, device=dev)
        k_cur = synth.randn_bf16((H, Lq, D), 910000 + layer, device=dev)
        v_cur = synth.randn_bf16((H, Lq, D), 920000 + layer, device=dev)
        if args.layout == "model":                 # same values, held as [tokens][heads][D]; the views are heads-first
            q, k_cur, v_cur = [t.permute(1, 0, 2).contiguous().permute(1, 0, 2) for t in (q, k_cur, v_cur)]
        out = torch.empty_like(q)                  # preserves the strides
        layers.append((pool, index, q, k_cur, v_cur, out))
    # The last append of every layer (the one that brings its pool to T frames), enqueued as in a rollout, where the
    # layers' write-backs are independent of each other and go round-robin onto four side streams (default priority),
    # and timed as one region on the main stream; bytes = new frames + survivors that changed slot, K and V, read + write.
    torch.cuda.synchronize()
    ids_before = [a[0].frame_ids.cpu().numpy().copy() for a in last_appends]
    wb_streams = [torch.cuda.Stream() for _ in range(APPEND_STREAMS)]
    for s_ in wb_streams:                            # first use of a stream costs the host a few hundred microseconds
        with torch.cuda.stream(s_):
            torch.zeros(1024, device=dev).add_(1)
    torch.cuda.synchronize()
    main0 = torch.cuda.current_stream()
    e0, e1 = ev(), ev()
    e0.record()
    for s_ in wb_streams:
        s_.wait_stream(main0)
    for li, (pool, k_new, v_new, sc, t0, n_new) in enumerate(last_appends):
        B.pf_cache_append(pool, k_new, v_new, sc, stream=wb_streams[li % APPEND_STREAMS].cuda_stream)
    for s_ in wb_streams:
        main0.wait_stream(s_)
    e1.record()
    torch.cuda.synchronize()
    append_ms.append(e0.elapsed_time(e1) / len(last_appends))
    for (pool, k_new, v_new, sc, t0, n_new), before in zip(last_appends, ids_before):
        after = pool.frame_ids.cpu().numpy()
        moved = int(((after != before) & (after >= 0) & (after < t0)).sum())
        append_bytes.append(2 * 2 * frame_bytes * (H * n_new + moved) / len(last_appends))
    del last_appends
    ws_bytes = max(B.pf_attn_workspace_bytes(L[0], Lq) for L in layers)
    workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)     # layers run one after another: shared
    torch.cuda.synchronize()

    # The frame indices depend on the pools only, not on the previous layer's output: they are built on a side
    # stream (default priority) and each attention launch waits for its own layer's index.  A step still
    # contains all 30 builds and all 30 attention launches.
    main = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    built = [torch.cuda.Event() for _ in layers]

    attn_fwd = B.pf_ragged_attn_fwd_strided if args.layout == "model" else B.pf_ragged_attn_fwd

    def step(events=None):
        side.wait_stream(main)                     # the previous step's launches have read their plans
        with torch.cuda.stream(side):
            for li, (pool, index, *_r) in enumerate(layers):
                B.pf_build_index(pool, index, Lq)
                built[li].record(side)
        for li, (pool, index, q, k_cur, v_cur, out) in enumerate(layers):
            main.wait_event(built[li])
            if events is not None:
                e0, e1 = ev(), ev()
                e0.record()
            attn_fwd(pool, index, q, k_cur, v_cur, out, workspace)
            if events is not None:
                e1.record()
                events.append((e0, e1))

    if args.copy_probe > 0:
        src = torch.empty(args.copy_probe << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # effective work from the index the library built (history frames selected per head)
    flops = 0.0
    kv_bytes = 0.0
    for (pool, index, *_rest) in layers:
        for n in index.sel_count.cpu().tolist():
            lkv = n * tpf + Lq
            flops += 4.0 * Lq * lkv * D
            kv_bytes += 2.0 * lkv * D * 2

    events = []
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(args.steps):
        step(events)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    ms_per_step = wall * 1e3 / args.steps
    attn_ms = [a.elapsed_time(b) for a, b in events]
    attn_ms_avg = float(np.mean(attn_ms))
    flops_per_launch = flops / n_layers
    achieved = flops_per_launch / (attn_ms_avg * 1e-3) / 1e12
    value = flops / (ms_per_step * 1e-3) / 1e12

    traffic, traffic_source = profiled_traffic(w.name, int(layers[0][1].c.variant), args.layout)
    result = {
        "metric": "ragged-attn effective TFLOP/s (retained keys)",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: %d layers x %d heads, head_dim %d, %d tokens/frame, %d-token query chunk, "
                               "%d history frames" % (w.name, n_layers, H, D, tpf, Lq, T),
                   "step": "per layer pf_build_index (side stream) + pf_ragged_attn_fwd, %d layers back to back" % n_layers,
                   "effective_tflop_per_step": round(flops / 1e12, 3),
                   "attn_variant": int(layers[0][1].c.variant), "chunk_layout": args.layout,
                   "seg_tiles": int(os.environ.get("PF_SEG_TILES", "0")) or "default"},
        "frac_of_bf16_peak": round(value / PEAK_BF16_TFLOPS, 4),
        "roofline": {"kernel": "pf_attn_pp_kernel" if int(layers[0][1].c.variant) >= 1 else "pf_attn_kernel", "bound": "mfma", "achieved": round(achieved, 2),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                     "traffic": traffic, "traffic_source": traffic_source,
                     "avg_launch_ms": round(attn_ms_avg, 4),
                     "flop_per_launch": flops_per_launch, "launches_timed": len(attn_ms)},
        "pool_append": {"kernel": "pf_pool_append_kernel", "bound": "hbm",
                        "what": "the append of %d frames that brings each layer's pool to %d frames "
                                "(new frames + left-packed survivors, K and V, read + write), the layers' appends enqueued "
                                "round-robin on %d streams as in a rollout, timed as one region" % (w.chunk_frames, T, APPEND_STREAMS),
                        "avg_launch_ms": round(float(np.mean(append_ms)), 4),
                        "achieved": round(float(np.sum(append_bytes)) / (float(np.sum(append_ms)) * 1e-3) / 1e9, 1),
                        "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": round(float(np.sum(append_bytes)) / (float(np.sum(append_ms)) * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
    }

    if args.block_trace:
        # one resident workgroup per compute unit: ticks (10 ns) inside work items over the launch's span
        trace = torch.zeros(8 * 1024, dtype=torch.int64, device=dev)
        B.pf_set_block_trace(trace)
        fracs, spans, mhz = [], [], []
        for (pool, index, q, k_cur, v_cur, out) in layers:
            trace.zero_()
            attn_fwd(pool, index, q, k_cur, v_cur, out, workspace)
            torch.cuda.synchronize()
            t = trace.cpu().numpy().reshape(-1, 8)
            t = t[t[:, 3] > 0]
            mhz.append(100.0 * t[:, 4] / np.maximum(t[:, 0], 1))
            span = float(t[:, 2].max() - t[:, 1].min())
            fracs.append(t[:, 0] / span)
            spans.append(span * 1e-2)
        B.pf_set_block_trace(None)
        allf = np.concatenate(fracs)
        result["cu_busy"] = {"what": "fraction of the launch's span (first item start to last item end over all workgroups) that each "
                                     "resident workgroup (one per compute unit) spent inside work items, over %d launch(es)" % len(layers),
                             "workgroups_per_launch": int(len(fracs[0])), "mean": round(float(allf.mean()), 4),
                             "min": round(float(allf.min()), 4), "p05": round(float(np.percentile(allf, 5)), 4),
                             "max": round(float(allf.max()), 4), "mean_span_us": round(float(np.mean(spans)), 1),
                             "shader_clock_mhz": {"what": "shader-clock cycles per 100 MHz tick inside work items, per workgroup",
                                                  "mean": round(float(np.concatenate(mhz).mean()), 0),
                                                  "min": round(float(np.concatenate(mhz).min()), 0),
                                                  "max": round(float(np.concatenate(mhz).max()), 0)}}

    # ---------------------------------------------------------------- cpu_baseline: the oracle on a bounded sample
    if not args.no_cpu:
        from oracle import attention as OA
        from oracle import check as G
        from oracle.pool import PoolOracle
        pols, keep_k, keep_v, keep_s = hist0
        pool_o = PoolOracle(pols, tpf, D)
        for k_new, v_new, sc in zip(keep_k, keep_v, keep_s):
            pool_o.append(synth.bits(k_new), synth.bits(v_new), sc.numpy())
        sel_count, sel_frames, _, _ = pool_o.build_index(layers[0][1].max_sel)
        rows = G.sample_rows(Lq, args.cpu_rows, 12345)
        pool, index, q, k_cur, v_cur, out = layers[0]
        qc, kc, vc = q.cpu(), k_cur.cpu(), v_cur.cpu()
        OA.num_threads()
        t0 = time.perf_counter()
        want = G.oracle_attention(pool_o, sel_count, sel_frames, qc, kc, vc, rows=rows)
        cpu_s = time.perf_counter() - t0
        cpu_flops = sum(4.0 * len(rows) * (int(n) * tpf + Lq) * D for n in sel_count)
        worst_abs, worst_rel = G.compare_attention(out.float().cpu().numpy(), want, rows=rows, label="bench layer 0")
        result["cpu_baseline"] = {"value": round(cpu_flops / cpu_s / 1e12, 6), "unit": "TFLOP/s",
                                  "cores": OA.num_threads(), "kind": "oracle",
                                  "sample": "layer 0, all %d heads, %d seeded query rows per head (%.1f GFLOP effective, "
                                            "%.1f s incl. assembling each head's keys)" % (H, len(rows), cpu_flops / 1e9, cpu_s),
                                  "parity_max_abs": float(worst_abs), "parity_rel_l2": float(worst_rel)}
    print(json.dumps(result))


def profiled_traffic(workload, variant, layout):
    """(HBM bytes per attention launch, where the figure comes from): counters cannot be read inside a timed run, so
    the bytes are those of the committed rocprofv3 counter summary of this command (FETCH_SIZE and WRITE_SIZE passes,
    scaled by the copy probe).  The summary names the commit it was made from and the SHA-256 of the attention
    kernel's source at that time; when the source here differs, or the summary does not cover this workload /
    kernel, the bytes are None and the second value says why."""
    rel = "profiles/pf_attn_pp_kernel_c3_step.md"
    if workload != "c3_step" or variant != 1 or layout != "packed":
        return None, "no stored counter summary for this workload / kernel / layout"
    import hashlib
    fields = {}
    try:
        for line in open(os.path.join(ROOT, rel)):
            for key in ("traffic_bytes_per_launch", "commit", "kernel_source_sha256"):
                if line.startswith(key + ":"):
                    fields[key] = line.split(":", 1)[1].strip()
        with open(os.path.join(ROOT, "paper_2605_13111_amd", "csrc", "pf_attn.hip"), "rb") as f:
            sha = hashlib.sha256(f.read()).hexdigest()
    except OSError:
        return None, "no stored counter summary"
    if "traffic_bytes_per_launch" not in fields:
        return None, "no stored counter summary"
    where = "%s @ %s" % (rel, fields.get("commit", "unknown commit"))
    if fields.get("kernel_source_sha256") != sha:
        return None, "stale: %s was measured on another version of the attention kernel" % where
    return int(fields["traffic_bytes_per_launch"]), "stored rocprofv3 counters, " + where


def append_probe(B, synth, dev):
    """Pool appends whose algorithmic bytes are known exactly, beside a plain copy (see --append-probe)."""
    H, D, tpf = 12, 128, 1560
    frame = tpf * D * 2

    def run(pols, n_app, label):
        pool = B.Pool(pols, tpf, D, device=dev)
        B.pf_pool_reset(pool)
        k = synth.randn_bf16((H, 3, tpf, D), 1, device=dev)
        v = synth.randn_bf16((H, 3, tpf, D), 2, device=dev)
        sc = synth.frame_scores(H, 3, 3, device=dev)
        torch.cuda.synchronize()
        for i in range(n_app):
            before = pool.frame_ids.cpu().numpy().copy()
            B.pf_cache_append(pool, k, v, sc)
            torch.cuda.synchronize()
            after = pool.frame_ids.cpu().numpy()
            moved = int(((after != before) & (after >= 0) & (after < 3 * i)).sum())
            print("%s append %d: %d new frames, %d survivors moved -> algorithmic read = write = %.2f MB (K and V)"
                  % (label, i, H * 3, moved, 2 * frame * (H * 3 + moved) / 1e6), flush=True)

    run([synth.anchor_all(30)] * H, 4, "keep-all")
    run([synth.anchor_topk(6, 6)] * H, 6, "top-6")
    src = torch.empty(64 << 20, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    print("copy probe: 64 MiB read, 64 MiB written", flush=True)


def stream_bench(args, B, synth, dev):
    """Streaming rollout: per chunk, 4 denoising passes of 30 attention launches, then the chunk's
    K/V are appended to every layer's pool and the indices rebuilt.  Everything is enqueued without a host sync."""
    w = synth.WORKLOADS[args.workload]
    n_layers = args.layers or w.n_layers
    H, D, tpf = w.n_heads, w.head_dim, w.tokens_per_frame
    Lq = w.chunk_frames * tpf
    n_chunks = args.steps if args.steps != 10 else w.history_frames // w.chunk_frames
    passes = 4
    layers = []
    for layer in range(n_layers):
        pols = synth.policies(w.name, layer=layer, slots_of=lambda p: B.slots_needed(p, w.history_frames))
        pool = B.Pool(pols, tpf, D, device=dev)
        index = B.Index(pool, Lq)
        q = synth.randn_bf16((H, Lq, D), 900000 + layer, device=dev)
        k_cur = synth.randn_bf16((H, w.chunk_frames, tpf, D), 910000 + layer, device=dev)
        v_cur = synth.randn_bf16((H, w.chunk_frames, tpf, D), 920000 + layer, device=dev)
        sc = synth.frame_scores(H, w.chunk_frames, 930000 + layer, device=dev)
        layers.append((pols, pool, index, q, k_cur, v_cur, sc, torch.empty_like(q)))
    ws_bytes = max(B.pf_attn_workspace_bytes(L[1], Lq) for L in layers)
    workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)

    # The write-back of a layer (append + index build) depends on that layer's last attention pass only, and the next
    # chunk's first pass of the layer depends on it: it is enqueued on a side stream (default priority, four of them
    # round-robin) right behind the layer's last pass and runs next to the attention launches of the following layers.
    main = torch.cuda.current_stream()
    sides = [torch.cuda.Stream() for _ in range(4)]
    attn_done = [torch.cuda.Event() for _ in layers]
    index_ready = [torch.cuda.Event() for _ in layers]

    def rollout(chunks):
        flops = 0.0
        for li, (pols, pool, index, *_r) in enumerate(layers):
            B.pf_pool_reset(pool)
            B.pf_build_index(pool, index, Lq)
            index_ready[li].record(main)
        for c in range(chunks):
            for ps in range(passes):
                for li, (pols, pool, index, q, k_cur, v_cur, sc, out) in enumerate(layers):
                    if ps == 0:
                        main.wait_event(index_ready[li])
                    B.pf_ragged_attn_fwd(pool, index, q, k_cur.view(H, Lq, D), v_cur.view(H, Lq, D), out, workspace)
                    if ps == passes - 1:
                        attn_done[li].record(main)
                        st = sides[li % len(sides)]
                        st.wait_event(attn_done[li])
                        with torch.cuda.stream(st):
                            B.pf_cache_append(pool, k_cur, v_cur, sc)
                            B.pf_build_index(pool, index, Lq)
                            index_ready[li].record(st)
            for li, (pols, *_r) in enumerate(layers):
                flops += passes * sum(4.0 * Lq * (B.pf_selected_count(p, c * w.chunk_frames) * tpf + Lq) * D for p in pols)
        for st in sides:
            main.wait_stream(st)
        return flops

    # warm-up: one whole rollout when any is asked for -- the library remembers the launch plan of every (layer,
    # history length) it has seen, as a serving process that generates one video after another would have them
    warm = n_chunks if args.warmup > 0 else 0
    rollout(warm)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    flops = rollout(n_chunks)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_chunk = wall * 1e3 / n_chunks
    value = flops / wall / 1e12
    print(json.dumps({
        "metric": "ragged-attn effective TFLOP/s (retained keys)", "value": round(value, 2), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": n_chunks, "warmup": warm, "ms_per_step": round(ms_per_chunk, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: %d layers x %d heads, head_dim %d, %d-token chunks, history 0..%d frames, "
                               "%d attention passes per chunk" % (w.name, n_layers, H, D, Lq, (n_chunks - 1) * w.chunk_frames,
                                                                  passes),
                   "step": "one chunk = %d x %d pf_ragged_attn_fwd; each layer's pf_cache_append + pf_build_index follows its last "
                           "pass on a side stream; no host sync inside the rollout; warm-up = one whole rollout (launch plans "
                           "remembered)" % (passes, n_layers),
                   "effective_tflop_total": round(flops / 1e12, 2), "ms_per_chunk": round(ms_per_chunk, 4)},
        "frac_of_bf16_peak": round(value / PEAK_BF16_TFLOPS, 4),
        "roofline": {"kernel": "pf_attn_pp_kernel", "bound": "mfma", "achieved": round(value, 2), "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(value / PEAK_BF16_TFLOPS, 4), "traffic": None,
                     "traffic_source": "no stored counter summary for this workload",
                     "note": "whole-rollout rate (appends and index builds included in the time)"}}))


if __name__ == "__main__":
    main()
