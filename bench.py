#!/usr/bin/env python3
"""Benchmark of the per-chunk streaming sparse-attention step on one MI355X.

One "step" streams a whole synthetic context through one attention layer: for every chunk,
append (segment + index) -> retrieve (score + select) -> attend.  Inputs are resident in HBM
before the timed region starts.  Prints one JSON line:
  metric  = prefill tokens/s per layer (the context length is in config.workload),
  roofline = the attend kernel's achieved bf16 matrix-core rate against the published peak,
  cpu_baseline = the CPU oracle timed on a bounded sample of the same workload.
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

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 matrix rate
PEAK_HBM_GBPS = 8000.0
PROFILES = os.path.join(ROOT, "profiles")


def profile_traffic_bytes(filename, kernels):
    """HBM bytes per launch of the named kernels, summed, from a committed rocprofv3 counter summary under
    profiles/: table rows `kernel  launches  FETCH_SIZE  read-KiB  WRITE_SIZE` (KiB per dispatch, the read
    column already scaled by the calibration factor stated in the file). None if the file or a row is missing."""
    try:
        lines = open(os.path.join(PROFILES, filename)).read().splitlines()
    except OSError:
        return None
    total = 0.0
    for k in kernels:
        row = [l.split() for l in lines if l.startswith(k) and len(l.split()) >= 5]
        if not row:
            return None
        r = row[0]
        try:
            nums = [float(x) for x in r[1:] if x.replace(".", "", 1).isdigit()]
        except ValueError:
            return None
        if len(nums) < 4:
            return None
        total += (nums[2] + nums[3]) * 1024.0      # read KiB (scaled) + written KiB
    return int(total)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def attend_flops(w, n_q, list_lens):
    """Algorithmic work of one attend launch: 4 * d * (group size) * n_q * (N_att + (n_q + 1) / 2)
    per KV head, N_att = that head's context-list length; causal part counted at half."""
    g = w.n_q_heads // w.n_kv_heads
    return sum(4.0 * w.head_dim * g * n_q * (n + (n_q + 1) / 2.0) for n in list_lens)


def cpu_baseline(w, K, V, Q, bounds, theta, rows_sampled=256):
    """The oracle, as it stands, on the last (full-context) chunk of the workload: once with the numeric library's
    thread pool as it comes up on this host, once limited to one thread."""
    import numpy as np
    import torch
    from oracle import ltri_oracle as O
    T, L = w.context, w.chunk
    t_setup = time.time()
    Kn = K.double().cpu().numpy()
    Vn = V.double().cpu().numpy()
    cfg = O.OracleConfig(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, w.n_sink, w.window,
                         k_max=w.k_max, budget_tokens=w.budget_tokens, seg_map=O.MAP_LOGIT,
                         theta=float(np.float32(theta)), phi=0.0)
    qn = Q[T - L:].double().cpu().numpy()
    rows = list(range(0, L, L // rows_sampled))[:rows_sampled]

    def history():
        # the planted boundaries (cut at chunk edges) stand in for the earlier chunks' spans; building them is
        # not part of the timed chunk
        st = O.OracleStream(cfg, Kn, Vn)
        for c0 in range(0, T - L, L):
            b = [np.asarray(sorted({0, L} | {int(x - c0) for x in bounds[h][(bounds[h] > c0) & (bounds[h] < c0 + L)]}),
                            np.int64) for h in range(w.n_kv_heads)]
            st.append_chunk(L, bounds=b)
        return st

    def timed_chunk(st):
        c0, t0 = time.process_time(), time.time()
        st.append_chunk(L)
        t1 = time.time()
        st.retrieve(qn)
        t2 = time.time()
        st.attend(qn, rows=rows)
        t3, c1 = time.time(), time.process_time()
        seg, ret, att = t1 - t0, t2 - t1, (t3 - t2) * (L / len(rows))
        return seg, ret, att, (c1 - c0) / max(t3 - t0, 1e-9)

    st = history()
    log(f"[cpu_baseline] setup {time.time() - t_setup:.1f}s; timing the last chunk")
    seg, ret, att, busy = timed_chunk(st)
    total = seg + ret + att
    try:
        import threadpoolctl
        pool = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] or [1])
    except Exception:
        threadpoolctl, pool = None, (os.cpu_count() or 1)
    one = None
    if threadpoolctl is not None:
        with threadpoolctl.threadpool_limits(limits=1):
            s1, r1, a1, _ = timed_chunk(history())
        one = s1 + r1 + a1
        log(f"[cpu_baseline] one thread: segment {s1:.2f}s retrieve {r1:.2f}s attend (scaled) {a1:.2f}s")
    log(f"[cpu_baseline] {pool} threads: segment {seg:.2f}s retrieve {ret:.2f}s attend (scaled) {att:.2f}s "
        f"-> {total:.1f}s per chunk; {busy:.1f} cores busy on average over the sample")
    return {"value": L / total, "unit": "tokens/s", "cores": int(pool), "kind": "oracle",
            "cores_busy_on_average": round(busy, 1),
            "value_one_thread": (L / one) if one else None,
            "seconds_per_chunk": {"segment": round(seg, 2), "retrieve": round(ret, 2), "attend_scaled": round(att, 2)},
            "sample": f"last chunk of {w.name} (tokens {T - L}..{T}, full context): segmentation and retrieval of all "
                      f"{w.n_kv_heads} KV heads timed whole, attention timed on {len(rows)} of {L} query rows x "
                      f"{w.n_q_heads} heads and scaled by {L // len(rows)}; earlier chunks' spans taken from the planted "
                      f"boundaries (setup, untimed); fp64 numpy. `cores` is the size of the numeric library's thread pool "
                      f"(its matrix products use it; the cumulative sums and the loop over anti-diagonals of the "
                      f"segmentation run on one thread), `cores_busy_on_average` is process CPU time over wall time "
                      f"of the sample, `value_one_thread` the same sample with the pool limited to one thread"}


def run_decode(args, torch, dev):
    """Batched decode at the cfg5 shape (not the headline line): 16 sequences with `context` tokens
    each, one new token per step; every step appends, re-scores all stored spans, selects under the
    budget and attends. The index is built from the planted boundaries (the prefill path measures
    the segmentation). Prints one JSON line of its own."""
    import numpy as np
    from paper_2412_04757_amd import LtriContext, config_from_workload
    from workloads import CONFIGS, planted_stream, theta_default
    w = CONFIGS["cfg5"]
    T0 = args.context or w.context
    n_seqs, L, steps, warm = 16, 2048, max(8, args.steps * 8), 4
    T = T0 + 3 * steps + warm                   # a third of the steps keeps the selection (persistent mechanism), a third goes through ltri_step
    cfg = config_from_workload(w, max_tokens=T, theta=theta_default(w.head_dim), n_layers=1, n_seqs=n_seqs)
    ctx = LtriContext(cfg, dev)
    ka, va = ctx.arena_views()
    Qs = []
    for s in range(n_seqs):
        K, V, Q, bounds = planted_stream(w, args.seed, device="cuda:0", context=T, seq=s)
        ka[0, s, :, :T].copy_(K)
        va[0, s, :, :T].copy_(V)
        Qs.append(Q[T0:T].clone())
        for c0 in range(0, T0, L):
            n = min(L, T0 - c0)
            b = [np.asarray(sorted({0, n} | {int(x - c0) for x in bounds[h][(bounds[h] > c0) & (bounds[h] < c0 + n)]}), np.int32)
                 for h in range(w.n_kv_heads)]
            ctx.append_chunk_with_spans(0, s, n, b)
        del K, V, Q
    out = torch.empty((n_seqs, 1, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
    qsteps = [torch.stack([Qs[s][k:k + 1] for s in range(n_seqs)]).contiguous() for k in range(3 * steps + warm)]
    for k in range(warm):
        ctx.append_chunk(0, 0, n_seqs, 1)
        ctx.retrieve(0, 0, n_seqs, qsteps[k])
        ctx.attend(0, 0, n_seqs, qsteps[k], out=out)
    torch.cuda.synchronize()
    n_att = sum(len(ctx.get_token_list(0, s, h)) for s in range(n_seqs) for h in range(w.n_kv_heads))
    evs = []
    for k in range(warm, warm + steps):
        e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        e[0].record(); ctx.append_chunk(0, 0, n_seqs, 1)
        e[1].record(); ctx.retrieve(0, 0, n_seqs, qsteps[k])
        e[2].record(); ctx.attend(0, 0, n_seqs, qsteps[k], out=out)
        e[3].record(); evs.append(e)
    pevs = []
    for k in range(warm + steps, warm + 2 * steps):
        e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        e[0].record(); ctx.append_chunk(0, 0, n_seqs, 1)
        e[1].record(); ctx.retrieve_persistent(0, 0, n_seqs)
        e[2].record(); ctx.attend(0, 0, n_seqs, qsteps[k], out=out)
        e[3].record(); pevs.append(e)
    sevs = []                                   # ltri_step: steps 1 and 2 in one launch, then step 3
    for k in range(warm + 2 * steps, warm + 3 * steps):
        e = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        e[0].record(); ctx.step(0, 0, n_seqs, None, None, qsteps[k], out=out)
        e[1].record(); sevs.append(e)
    torch.cuda.synchronize()
    if ctx.sync_status() != 0:
        print("bench.py: device status", ctx.sync_status(), file=sys.stderr)
        sys.exit(1)
    med = lambda i, ev=None: float(np.median([e[i].elapsed_time(e[i + 1]) for e in (ev or evs)]) * 1e3)
    ap_us, rt_us, at_us = med(0), med(1), med(2)
    pers = [med(i, pevs) for i in range(3)]
    kv_bytes = n_att * w.head_dim * 2 * 2
    calls_us = ap_us + rt_us + at_us
    step_us = med(0, sevs) if args.schedule == "step" else calls_us
    print(json.dumps({
        "metric": "decode step time per layer", "value": round(step_us, 1), "unit": "us", "n_gpus": 1, "steps": steps,
        "warmup": warm, "higher_is_better": False, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"cfg5: 16 sequences x {T0} tokens, 32 query / 8 KV heads, head_dim 128, bf16, 4 sink tokens, "
                               f"window {w.window}, retrieval budget {w.budget_tokens} tokens, one token per step"},
        "schedule": "ltri_step (append and retrieve in one launch, then attend)" if args.schedule == "step" else "three calls",
        "three_calls_us": round(calls_us, 1),
        "breakdown_us": {"append": round(ap_us, 1), "retrieve": round(rt_us, 1), "attend": round(at_us, 1)},
        "persistent_selection": {"step_us": round(sum(pers), 1), "append": round(pers[0], 1),
                                 "rebuild_list": round(pers[1], 1), "attend": round(pers[2], 1)},
        "roofline": {"bound": "hbm", "kernel": "attend_decode_kernel + attend_merge_kernel",
                     "achieved": round(kv_bytes / at_us / 1e3, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                     "frac": round(kv_bytes / at_us / 1e3 / PEAK_HBM_GBPS, 4), "kv_bytes_per_step": kv_bytes,
                     "traffic": (profile_traffic_bytes("attend_decode_cfg5_hbm_traffic.txt",
                                                       ["attend_decode_kernel", "attend_merge_kernel"])
                                 if not args.context else None),
                     "whole_step_GBps": round(kv_bytes / step_us / 1e3, 1)}}))


def run_layers(args, torch, dev):
    """All layers resident at the cfg4 shape (not the headline line): 32 layers x 256K tokens of K/V
    (34 GB) plus every layer's span index stay in HBM; the last chunk of the stream is run through
    every layer in turn (real segmentation, retrieval, attention). Prints one JSON line of its own:
    per-chunk time per layer, its spread over the layers, and the resident bytes."""
    import numpy as np
    from paper_2412_04757_amd import LtriContext, config_from_workload
    from workloads import CONFIGS, planted_stream, theta_default
    w = CONFIGS["cfg4"]
    T = args.context or w.context
    L, n_layers = w.chunk, w.n_layers
    cfg = config_from_workload(w, max_tokens=T, theta=theta_default(w.head_dim), n_layers=n_layers, n_seqs=1)
    ctx = LtriContext(cfg, dev)
    ka, va = ctx.arena_views()
    T0 = T - L                                  # history through the planted boundaries, last chunk for real
    qs = []
    for layer in range(n_layers):
        K, V, Q, bounds = planted_stream(w, args.seed, device="cuda:0", context=T, layer=layer)
        ka[layer, 0].copy_(K)
        va[layer, 0].copy_(V)
        qs.append(Q[T0:T].clone())
        for c0 in range(0, T0, L):
            b = [np.asarray(sorted({0, L} | {int(x - c0) for x in bounds[h][(bounds[h] > c0) & (bounds[h] < c0 + L)]}), np.int32)
                 for h in range(w.n_kv_heads)]
            ctx.append_chunk_with_spans(layer, 0, L, b)
        del K, V, Q
        log(f"[bench] layer {layer} resident")
    out = torch.empty((1, L, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
    torch.cuda.synchronize()
    times = []
    for layer in range(n_layers):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        if args.schedule == "step":
            ctx.step(layer, 0, 1, None, None, qs[layer], out=out)
        else:
            ctx.append_chunk(layer, 0, 1, L)
            ctx.retrieve(layer, 0, 1, qs[layer])
            ctx.attend(layer, 0, 1, qs[layer], out=out)
        e1.record()
        times.append((e0, e1))
    torch.cuda.synchronize()
    if ctx.sync_status() != 0:
        print("bench.py: device status", ctx.sync_status(), file=sys.stderr)
        sys.exit(1)
    us = np.asarray([a.elapsed_time(b) * 1e3 for a, b in times])
    spans = [ctx.span_count(layer, 0, 0) for layer in (0, n_layers - 1)]
    print(json.dumps({
        "metric": "last-chunk time per layer with all layers resident", "value": round(float(np.median(us[1:])), 1), "unit": "us",
        "n_gpus": 1, "higher_is_better": False, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"cfg4: {n_layers} layers x {T} tokens resident, 32 query / 8 KV heads, head_dim 128, bf16, "
                               f"chunk {L}, window {w.window}, budget {w.budget_tokens}",
                   "schedule": "ltri_step" if args.schedule == "step" else "three calls"},
        "per_layer_us": {"first_layer_incl_warmup": round(float(us[0]), 1), "min": round(float(us[1:].min()), 1),
                         "median": round(float(np.median(us[1:])), 1), "max": round(float(us[1:].max()), 1)},
        "resident_bytes": {"kv_arenas": int(ka.numel() * ka.element_size() * 2), "index_state": int(ctx.state.numel()),
                           "scratch": int(ctx.scratch.numel())},
        "spans_kv_head0": {"layer0": spans[0], f"layer{n_layers - 1}": spans[1]}}))


def run_attend_occupancy(args, torch, dev):
    """The attend kernel of the default workload with fewer and fewer compute units busy (not the
    headline line): the last chunk of the cfg3 stream is cut to 2048, 1024, 512 and 256 queries, which
    gives 256, 128, 64 and 32 workgroups (one per compute unit) over the same ~12K-key context. If the
    rate per busy compute unit rises as the chip empties, the full launch is held back by a chip-wide
    limit (power, clocks) and not by the kernel's instruction schedule. Prints one JSON line of its own."""
    import numpy as np
    from paper_2412_04757_amd import LtriContext, config_from_workload
    from workloads import CONFIGS, planted_stream, theta_default
    w = CONFIGS["cfg3"]
    T, L = w.context, w.chunk
    K, V, Q, bounds = planted_stream(w, args.seed, device="cuda:0")
    rows = []
    for n_q in (2048, 1024, 512, 256):
        cfg = config_from_workload(w, theta=theta_default(w.head_dim), n_layers=1, n_seqs=1)
        ctx = LtriContext(cfg, dev)
        ka, va = ctx.arena_views()
        ka[0, 0].copy_(K)
        va[0, 0].copy_(V)
        T0 = T - L
        for c0 in list(range(0, T0, L)) + [T0]:
            n = L if c0 < T0 else n_q
            b = [np.asarray(sorted({0, n} | {int(x - c0) for x in bounds[h][(bounds[h] > c0) & (bounds[h] < c0 + n)]}), np.int32)
                 for h in range(w.n_kv_heads)]
            ctx.append_chunk_with_spans(0, 0, n, b)
        q = Q[T0:T0 + n_q].contiguous()
        ctx.retrieve(0, 0, 1, q)
        out = torch.empty((1, n_q, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
        lens = [len(ctx.get_token_list(0, 0, h)) for h in range(w.n_kv_heads)]
        flops = attend_flops(w, n_q, lens)
        reps = 10 * max(1, args.steps)
        for _ in range(3):
            ctx.attend(0, 0, 1, q, out=out)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            ctx.attend(0, 0, 1, q, out=out)
        e1.record()
        torch.cuda.synchronize()
        if ctx.sync_status() != 0:
            print("bench.py: device status", ctx.sync_status(), file=sys.stderr)
            sys.exit(1)
        us = e0.elapsed_time(e1) / reps * 1e3
        groups = w.n_kv_heads * (n_q // 64)
        rows.append({"queries": n_q, "workgroups": groups, "us": round(us, 1), "tflops": round(flops / us / 1e6, 1),
                     "tflops_per_workgroup": round(flops / us / 1e6 / groups, 3)})
        log(f"[bench] attend, {n_q} queries on {groups} workgroups: {us:.1f} us, {flops / us / 1e6:.1f} TFLOP/s")
        del ctx
    full, least = rows[0], rows[-1]
    print(json.dumps({
        "metric": "attend rate per busy compute unit, 32 workgroups over 256", "unit": "ratio",
        "value": round(least["tflops_per_workgroup"] / full["tflops_per_workgroup"], 3),
        "n_gpus": 1, "higher_is_better": False, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "cfg3, last chunk cut to 2048 / 1024 / 512 / 256 queries over the full 128K stream's index"},
        "launches": rows}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--context", type=int, default=0, help="override the context length (debugging)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-single-launch", action="store_true",
                    help="skip the comparison pass with the three plain calls")
    ap.add_argument("--overlap", action="store_true",
                    help="segment chunk c+1 on a second stream next to attend(c) (measured: no gain, the kernels\n"
                         "compete for the same compute units)")
    ap.add_argument("--schedule", choices=["calls", "step"], default="step",
                    help="calls: append, retrieve, attend one after the other; step: ltri_step per chunk (one stream "
                         "and fused step-2 kernels; with --kv-offload the attention over initial | window | chunk "
                         "runs beside steps 1 and 2 on a second stream)")
    ap.add_argument("--attend-stages", type=int, default=0, choices=[0, 3, 4],
                    help="LDS ring depth of the attention kernel (default: the library's)")
    ap.add_argument("--index-vectors", choices=["mean", "dynamic"], default="mean",
                    help="what a span stores: the mean key (headline) or the sum of its index tokens' keys\n"
                         "(dynamic span index vectors, row ratio, lambda 3); not the headline configuration")
    ap.add_argument("--theta-quantile", type=float, default=0.0,
                    help="take theta as this percentile of every chunk's map (e.g. 0.9) instead of the absolute\n"
                         "value; not the headline configuration")
    ap.add_argument("--unit-tokens", type=int, default=0,
                    help="retrieve whole memory units of this many tokens (Eq. 9 as written) instead of spans;\n"
                         "not the headline configuration")
    ap.add_argument("--index-block-max", type=int, default=0,
                    help="with --index-vectors dynamic and --unit-tokens U: at most this many index vectors per block of\n"
                         "U tokens (the paper's M, 12 or 24), shared over the block's spans")
    ap.add_argument("--kv-offload", action="store_true",
                    help="host-offloaded KV (Sec. 3.4 first step): the arenas are pinned host memory, the device keeps\n"
                         "initial tokens, a ring of the latest tokens and the rows fetched for each selection; not the\n"
                         "headline configuration")
    ap.add_argument("--seed", type=int, default=1)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path has no collective: KV heads, sequences and "
              "layers would shard without any exchange); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2412_04757_amd import LtriContext, config_from_workload
    from workloads import CONFIGS, planted_stream, theta_default

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    if args.workload == "cfg5":
        run_decode(args, torch, dev)
        return
    if args.workload == "cfg4":
        run_layers(args, torch, dev)
        return
    if args.workload == "attend-occupancy":
        run_attend_occupancy(args, torch, dev)
        return
    w = CONFIGS[args.workload]
    if args.context:
        from dataclasses import replace
        w = replace(w, context=args.context)
    T, L = w.context, w.chunk
    n_chunks = T // L
    theta = theta_default(w.head_dim)
    log(f"[bench] workload {w.name}: T={T} L={L} Hq={w.n_q_heads} Hkv={w.n_kv_heads} d={w.head_dim} {w.dtype}")
    t0 = time.time()
    K, V, Q, bounds = planted_stream(w, args.seed, device="cuda:0")
    torch.cuda.synchronize()
    log(f"[bench] inputs generated in {time.time() - t0:.1f}s")
    cfg = config_from_workload(w, theta=theta, n_layers=1, n_seqs=1,
                               rep_mode=1 if args.index_vectors == "dynamic" else 0, lam=3.0,
                               theta_quantile=args.theta_quantile, unit_tokens=args.unit_tokens,
                               kv_offload=int(args.kv_offload), index_block_max=args.index_block_max)
    ctx = LtriContext(cfg, dev)
    ka, va = ctx.arena_views()
    if not args.kv_offload:
        ka[0, 0].copy_(K)
        va[0, 0].copy_(V)
    # host-offloaded KV: the rows come with every call
    kcs = [K[:, c * L:(c + 1) * L].unsqueeze(0).contiguous() if args.kv_offload else None for c in range(n_chunks)]
    vcs = [V[:, c * L:(c + 1) * L].unsqueeze(0).contiguous() if args.kv_offload else None for c in range(n_chunks)]
    out = torch.empty((1, L, w.n_q_heads, w.head_dim), dtype=w.torch_dtype, device=dev)
    qs = [Q[c * L:(c + 1) * L] for c in range(n_chunks)]          # contiguous views

    list_lens = []          # per chunk: context-list length of every KV head
    n_index_tokens = [0]    # dynamic index vectors: index tokens of all chunks and KV heads (first pass)
    SEPARATE = []           # events of the pass that times the attention kernel alone (--schedule step)

    # The segmentation of chunk c + 1 does not depend on the attention of chunk c; with --overlap it is
    # enqueued on a second stream between retrieve(c) and retrieve(c + 1) and runs next to attend(c).
    overlap = args.overlap
    main = torch.cuda.current_stream(dev)
    side = torch.cuda.Stream(dev) if overlap else None
    ev_r = [torch.cuda.Event() for _ in range(n_chunks)]
    ev_a = [torch.cuda.Event() for _ in range(n_chunks)]
    if overlap:
        ctx.set_attend_stages(3)          # leaves LDS for the segmentation kernels on every compute unit

    step_schedule = args.schedule == "step" and not overlap
    if args.attend_stages:
        ctx.set_attend_stages(args.attend_stages)

    def one_stream_steps():
        ctx.reset(0)
        for c in range(n_chunks):
            ctx.step(0, 0, 1, kcs[c], vcs[c], qs[c], out=out)

    def one_stream(record_lens=False, events=None):
        if step_schedule and events is not None and events is not SEPARATE:
            one_stream_steps()
            return
        ctx.reset(0)
        ctx.append_chunk(0, 0, 1, L, k_chunk=kcs[0], v_chunk=vcs[0])
        for c in range(n_chunks):
            ctx.retrieve(0, 0, 1, qs[c])
            nxt = c + 1 < n_chunks
            if nxt and overlap:
                ev_r[c].record(main)
            if events is not None:
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record(main)
            ctx.attend(0, 0, 1, qs[c], out=out)
            if events is not None:
                e1.record(main)
                events.append((e0, e1))
            if record_lens:
                list_lens.append([len(ctx.get_token_list(0, 0, h)) for h in range(w.n_kv_heads)])
                if args.index_vectors == "dynamic":
                    n_index_tokens[0] += sum(len(ctx.get_index_tokens(0, 0, h, L)) for h in range(w.n_kv_heads))
            if nxt:
                if overlap:
                    side.wait_event(ev_r[c])
                    ctx.set_stream(side)
                    ctx.append_chunk(0, 0, 1, L, k_chunk=kcs[c + 1], v_chunk=vcs[c + 1])
                    ev_a[c].record(side)
                    ctx.set_stream(main)
                    main.wait_event(ev_a[c])
                else:
                    ctx.append_chunk(0, 0, 1, L, k_chunk=kcs[c + 1], v_chunk=vcs[c + 1])

    # warmup (the first pass also records the list lengths, which need a synchronising read-back)
    one_stream(record_lens=True)
    for _ in range(max(0, args.warmup - 1)):
        one_stream()
    if step_schedule:
        one_stream_steps()
    status = ctx.sync_status()
    if status != 0:
        print(f"bench.py: device status {status}", file=sys.stderr)
        sys.exit(1)
    n_spans = [ctx.span_count(0, 0, h) for h in range(w.n_kv_heads)]
    log(f"[bench] spans per KV head: {n_spans}; last chunk list lengths {list_lens[-1]}")

    events = []
    if step_schedule:
        ctx.set_step_timing(True)     # events around the attention launches of every step, on their own streams
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_stream(events=events)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    value = T * args.steps / elapsed

    traffic = None
    if step_schedule:
        # The library brackets the attention launches of every step with events on the context's stream, inside the
        # timed region above. Resident keys and values: one launch of attend_bf16_kernel per chunk (the events ride in
        # its dispatch). Host-offloaded: two (initial | window | chunk beside the fetch of the retrieved rows, which a
        # second stream carries and which slows it, then the retrieved tokens); achieved = the chunk's algorithmic
        # flops over the sum of the two durations.
        t_loc, t_ret = ctx.read_step_timing(cap=args.steps * n_chunks + 8)
        ctx.set_step_timing(False)
        assert len(t_loc) == args.steps * n_chunks, (len(t_loc), args.steps * n_chunks)
        if args.kv_offload:
            att_ms = [float(a + b) for a, b in zip(t_loc, t_ret)]
            part_ms = {"initial_window_chunk": float(sum(t_loc)) / len(t_loc), "retrieved": float(sum(t_ret)) / len(t_ret)}
        else:
            att_ms = [float(a) for a in t_loc]
            part_ms = None
            if args.workload == "cfg3" and not args.context:
                traffic = profile_traffic_bytes("attend_gather_hbm_traffic_cfg3.txt", ["attend_bf16_kernel"])
    else:
        att_ms = [e0.elapsed_time(e1) for e0, e1 in events]
        part_ms = None
        if args.workload == "cfg3" and not args.context:
            traffic = profile_traffic_bytes("attend_gather_hbm_traffic_cfg3.txt", ["attend_bf16_kernel"])
    flops = [attend_flops(w, L, list_lens[i % n_chunks]) for i in range(len(att_ms))]
    tot_flops, tot_ms = sum(flops), sum(att_ms)
    achieved = tot_flops / (tot_ms * 1e-3) / 1e12
    last = [i for i in range(len(att_ms)) if i % n_chunks == n_chunks - 1]
    last_tflops = sum(flops[i] for i in last) / (sum(att_ms[i] for i in last) * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": "attend_bf16_kernel", "achieved": round(achieved, 2),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                "traffic": traffic,
                "avg_launch_us": round(tot_ms / len(att_ms) * 1e3, 1),
                "launches_timed": (("the two attention launches of every ltri_step of the timed streams (events recorded by "
                                    "the library on the context's stream); durations summed per chunk"
                                    if args.kv_offload else
                                    "the attention launch of every ltri_step of the timed streams (events recorded by the "
                                    "library around the launch)")
                                   if step_schedule else "every launch of the timed streams"),
                "avg_part_us": {k: round(v * 1e3, 1) for k, v in part_ms.items()} if part_ms else None,
                "full_context_launch_us": round(sum(att_ms[i] for i in last) / len(last) * 1e3, 1),
                "full_context_achieved": round(last_tflops, 2)}

    # what the timing events of the timed region cost: the same streams once more without them (not the headline)
    untimed_ms_per_step = None
    if step_schedule and not args.no_single_launch:
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            one_stream_steps()
        torch.cuda.synchronize()
        untimed_ms_per_step = (time.perf_counter() - t1) / args.steps * 1e3

    calls_ms_per_step = None
    single = None
    if step_schedule and not args.no_single_launch:
        # for comparison: the three plain calls, the attention as one launch per chunk
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            one_stream(events=SEPARATE)
        torch.cuda.synchronize()
        calls_ms_per_step = (time.perf_counter() - t1) / args.steps * 1e3
        s_ms = [e0.elapsed_time(e1) for e0, e1 in SEPARATE]
        s_fl = [attend_flops(w, L, list_lens[i % n_chunks]) for i in range(len(s_ms))]
        single = {"schedule": "three plain calls, one attention launch per chunk", "ms_per_step": round(calls_ms_per_step, 3),
                  "avg_launch_us": round(sum(s_ms) / len(s_ms) * 1e3, 1),
                  "achieved": round(sum(s_fl) / (sum(s_ms) * 1e-3) / 1e12, 2),
                  "frac": round(sum(s_fl) / (sum(s_ms) * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
    roofline["single_launch"] = single

    # the gather on its own (HBM-bound): context set of the last chunk into packed buffers. Warm = launches back to
    # back (the 99 MB working set then sits in the 256 MB last-level cache); cold = every launch after a pass over
    # 1 GiB of other memory, timed alone.
    kp = torch.empty((w.n_kv_heads, ctx.list_cap, w.head_dim), dtype=w.torch_dtype, device=dev)
    vp = torch.empty_like(kp)
    for _ in range(3):
        ctx.gather_pack(0, 0, kp, vp)
    g0 = torch.cuda.Event(enable_timing=True)
    g1 = torch.cuda.Event(enable_timing=True)
    reps = 20
    g0.record()
    for _ in range(reps):
        ctx.gather_pack(0, 0, kp, vp)
    g1.record()
    torch.cuda.synchronize()
    g_us = g0.elapsed_time(g1) / reps * 1e3
    flush = torch.empty(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB
    flush.zero_()
    cold = []
    for _ in range(10):
        flush.add_(1.0)
        c0e, c1e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        c0e.record()
        ctx.gather_pack(0, 0, kp, vp)
        c1e.record()
        cold.append((c0e, c1e))
    torch.cuda.synchronize()
    import statistics
    g_cold_us = statistics.median(a.elapsed_time(b) for a, b in cold) * 1e3
    elt = 2 if w.dtype == "bf16" else 4
    g_bytes = sum(list_lens[-1]) * w.head_dim * elt * 2 * 2            # K and V, read + write
    # what a plain contiguous device copy of the same size reaches in the same cold state (torch's copy kernel):
    # a launch this short spends a good part of its time ramping up and draining
    ref_src = torch.empty(g_bytes // 2, dtype=torch.uint8, device=dev)
    ref_dst = torch.empty_like(ref_src)
    ref_src.zero_()
    ref_dst.copy_(ref_src)
    cold_ref = []
    for _ in range(10):
        flush.add_(1.0)
        c0e, c1e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        c0e.record()
        ref_dst.copy_(ref_src)
        c1e.record()
        cold_ref.append((c0e, c1e))
    torch.cuda.synchronize()
    ref_cold_us = statistics.median(a.elapsed_time(b) for a, b in cold_ref) * 1e3
    del flush, ref_src, ref_dst
    gather = {"bound": "hbm", "kernel": "gather_pack_kernel", "achieved": round(g_bytes / g_cold_us / 1e3, 1),
              "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": round(g_bytes / g_cold_us / 1e3 / PEAK_HBM_GBPS, 4),
              "launch_us": round(g_cold_us, 2), "bytes": g_bytes,
              "state": "cold: timed alone after a pass over 1 GiB of other memory (median of 10)",
              "plain_copy_same_size_cold": {"achieved": round(g_bytes / ref_cold_us / 1e3, 1), "launch_us": round(ref_cold_us, 2),
                                            "note": "contiguous device-to-device copy of the same bytes in the same cold state"},
              "warm": {"achieved": round(g_bytes / g_us / 1e3, 1), "frac": round(g_bytes / g_us / 1e3 / PEAK_HBM_GBPS, 4),
                       "launch_us": round(g_us, 2),
                       "state": "back-to-back launches: the working set stays in the last-level cache"}}

    # measured ceilings of this GPU next to the published ones: back-to-back bf16 matrix-core
    # products, and a streaming copy / read of 1 GiB
    from paper_2412_04757_amd import measure_mfma_peak, measure_copy_peak, measure_read_peak
    mfma_meas = measure_mfma_peak(dev)
    mfma_meas_rnd = measure_mfma_peak(dev, random_operands=True)
    copy_meas = measure_copy_peak(dev)
    read_meas = measure_read_peak(dev)
    roofline["measured_peak"] = round(mfma_meas, 1)
    roofline["frac_of_measured"] = round(achieved / mfma_meas, 4)
    roofline["measured_peak_random_operands"] = round(mfma_meas_rnd, 1)
    roofline["frac_of_measured_random_operands"] = round(achieved / mfma_meas_rnd, 4)
    gather["measured_peak"] = round(copy_meas, 1)
    gather["measured_read_peak"] = round(read_meas, 1)
    gather["frac_of_measured"] = round(g_bytes / g_cold_us / 1e3 / copy_meas, 4)
    log(f"[bench] measured ceilings: {mfma_meas:.0f} TFLOP/s bf16 matrix products ({mfma_meas_rnd:.0f} with random operands), "
        f"{copy_meas:.0f} GB/s streaming copy (read + write), {read_meas:.0f} GB/s streaming read")

    # share of the step spent outside attend (append + retrieve + launch gaps)
    other_ms = ms_per_step - tot_ms / args.steps
    log(f"[bench] {ms_per_step:.2f} ms per stream" +
        (f" (with the three plain calls {calls_ms_per_step:.2f} ms" +
         (f", without the timing events {untimed_ms_per_step:.2f} ms" if untimed_ms_per_step else "") + ")"
         if calls_ms_per_step else "") +
        f": attend {tot_ms / args.steps:.2f} ms, rest {other_ms:.2f} ms; roofline frac {achieved / PEAK_BF16_TFLOPS:.4f}")

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(w, K, V, Q, bounds, theta)

    index_footprint = None
    if args.index_vectors == "dynamic":
        # What the index of the evicted tokens takes (Sec. 4, "Compression Ratio" and the table of occupied GPU
        # memory): the paper keeps every index vector (up to M per block of 128 tokens); this build keeps their sum,
        # one vector per span (Eq. 8 is bilinear). Bytes per token and KV head, next to the paper's figure.
        blk = args.unit_tokens or 128
        elt = 2 if w.dtype == "bf16" else 4
        per_block = n_index_tokens[0] / (w.n_kv_heads * T / blk)
        spans_per_block = sum(n_spans) / (w.n_kv_heads * T / blk)
        index_footprint = {
            "block_tokens": blk, "index_block_max": args.index_block_max or None,
            "index_vectors_per_block": round(per_block, 2), "spans_per_block": round(spans_per_block, 2),
            "bytes_per_token_and_head_if_every_index_vector_were_stored": round(per_block * w.head_dim * elt / blk, 2),
            "bytes_per_token_and_head_stored_here": round(spans_per_block * w.head_dim * elt / blk, 2),
            "paper": "0.027 GiB for the index of 100K tokens (M = 12, lambda = 3, 16-bit, 32 layers with one retrieval "
                     "head each; window 4096 and 128 initial tokens stay out): 9.5 bytes per evicted token and head, "
                     "i.e. 4.7 index vectors per block of 128 tokens on the real model's maps"}
    host_link = None
    if args.kv_offload:
        elt = 2 if w.dtype == "bf16" else 4
        row = w.head_dim * elt * 2                                            # K and V
        n_init_win = [min(w.n_sink, c * L) + (c * L - max(min(w.n_sink, c * L), c * L - w.window)) for c in range(n_chunks)]
        h2d = sum(sum(n - n_init_win[c] for n in list_lens[c]) for c in range(n_chunks)) * row
        d2h = T * w.n_kv_heads * row
        host_link = {"fetched_bytes_per_stream": int(h2d), "written_back_bytes_per_stream": int(d2h),
                     "sustained_GBps": round((h2d + d2h) / (ms_per_step * 1e-3) / 1e9, 2),
                     "note": "bytes crossing the host link per stream over the stream's wall time (reads and writes share "
                             "the time, the link is full duplex)"}
    result = {
        "metric": "prefill tokens/s per layer", "value": round(value, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": f"{w.name}: Llama-3-8B layer shape, {w.n_q_heads} query / {w.n_kv_heads} KV heads, "
                               f"head_dim {w.head_dim}, {w.dtype}, context {T} streamed in chunks of {L}, "
                               f"{w.n_sink} sink tokens, window {w.window}, retrieval budget {w.budget_tokens} tokens, "
                               f"planted-span keys ({w.len_dist} lengths in [{w.len_lo},{w.len_hi}]), seed {args.seed}",
                   "step": "one full stream through one layer (append + retrieve + attend per chunk)",
                   "seg_map": "logit", "theta": theta if not args.theta_quantile else f"percentile {args.theta_quantile}",
                   "phi": 0.0,
                   "retrieval_unit": "span" if not args.unit_tokens else f"memory units of {args.unit_tokens} tokens",
                   "kv": ("host-offloaded: pinned host arenas, device ring + fetched rows" if args.kv_offload
                          else "resident in HBM"),
                   "index_vectors": "mean key per span" if args.index_vectors == "mean"
                   else "dynamic (row ratio, lambda 3): sum of the keys of each span's index tokens",
                   "schedule": "append(c+1) on a second stream next to attend(c)" if overlap else
                   (("ltri_step per chunk: steps 1 and 2, then the fetch of the retrieved rows on a second stream beside "
                     "the attention over initial | window | chunk, retrieved tokens after, merged" if args.kv_offload else
                     "ltri_step per chunk: the kernels of the three steps on one stream, one attention launch")
                    if step_schedule else "three calls per chunk, serial")},
        "roofline": roofline, "gather": gather, "cpu_baseline": cpu, "host_link": host_link, "index_footprint": index_footprint,
        "breakdown_ms": {"attend": round(tot_ms / args.steps, 3), "rest_of_step": round(other_ms, 3),
                         "note": (("attend = sum of the two attention launches of every step; the first one shares the "
                                   "chip with the fetch over the host link and lasts about as long" if args.kv_offload else
                                   "attend = the attention launch of every step") if step_schedule else "serial calls"),
                         "ms_per_step_three_calls": round(calls_ms_per_step, 3) if calls_ms_per_step else None,
                         "ms_per_step_without_timing_events": round(untimed_ms_per_step, 3) if untimed_ms_per_step else None},
    }
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
