#!/usr/bin/env python3
"""Benchmark of the Kitty decode hot path on one MI355X.

A step is one pass of the whole hot path over one batch: kitty_append_token (window insert, and the
page quantizer whenever a window is full) followed by kitty_decode_attention — one decode step of one
attention layer, issued as the single call kitty_decode_step (or as the two calls with --two-calls).  Inputs are resident in HBM before the timed
region.  Steps rotate over several copies of the cache so that every step streams its records
from HBM rather than from the 256 MB last-level cache.

Prints one JSON line: effective HBM GB/s of the step (algorithmic bytes / time), the roofline
record of the dominant kernel (decode split-K, timed on its own with HIP events) and the CPU
oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps (default 200; 256 for c5)")
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c3", choices=["c2", "c3", "c4", "c5"],
                    help="c5 = the 36-layer variable-length decode loop (a step = one token for every sequence through all layers)")
    ap.add_argument("--layers", type=int, default=0, help="c5 only: number of layers (default 36)")
    ap.add_argument("--copies", type=int, default=0, help="cache copies to rotate over (0 = enough for >= 1.2 GB)")
    ap.add_argument("--n-splits", type=int, default=0)
    ap.add_argument("--src-seqs", type=int, default=2, help="distinct synthetic sequences tiled over the batch")
    ap.add_argument("--launch", default="eager", choices=["graph", "eager"],
                    help="graph: each step (4 kernel launches) is replayed from a captured HIP graph")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (scale reference for FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--prewarm-ms", type=float, default=300.0,
                    help="untimed launches of the streaming kernel before the warm-up steps (clocks and TLBs settle)")
    ap.add_argument("--two-calls", action="store_true",
                    help="step = kitty_append_token + kitty_decode_attention instead of the single kitty_decode_step call")
    ap.add_argument("--n-boost", type=int, default=-1,
                    help="override the workload's boosted-channel count (a multiple of 16 up to 128): the variant sweep")
    ap.add_argument("--batch", type=int, default=0, help="c2-c4: override the workload's batch size (1 = one sequence: latency)")
    ap.add_argument("--v-bits", type=int, default=2, choices=[2, 4],
                    help="4: Values quantized to 4 bits (the K2V4- and K4V4-like variants)")
    ap.add_argument("--sink-tokens", type=int, default=0,
                    help="keep this many initial tokens in full precision (the paper's Sink; parity covered by the tests, "
                         "the CPU baseline leg is skipped)")
    ap.add_argument("--v-local", type=int, default=0, choices=[0, 128],
                    help="128: Values of the newest page are read from the bf16 Local window")
    ap.add_argument("--no-seq-order", action="store_true", help="c5 only: dispatch sequences in batch order instead of longest first")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true",
                    help="default run only: leave out the summary of the other workloads (c2, c4, c5)")
    ap.add_argument("--cpu-pairs", type=int, default=0, help="(sequence, kv-head) pairs in the oracle sample (0 = auto)")
    return ap.parse_args()


def step_bytes(payload, n_pages, n_resid, w, sink=0, v_local=0):
    """Algorithmic bytes of one decode_attention call: records + full-precision rows + q + out.  With the Value
    Local window the newest page's Values are 128 bf16 rows instead of its 2-bit plane and per-token metadata."""
    per_pair = n_pages * payload + (n_resid + sink) * 128 * 2 * 2
    if v_local and n_pages:
        per_pair += 128 * 128 * 2 - (4096 + 512)
    return w.batch * w.n_kv_heads * per_pair + 2 * w.batch * w.n_q_heads * 128 * 2


def recorded_traffic(workload):
    """HBM bytes per decode_split launch as the committed rocprofv3 counter summary of this workload holds them
    (two --pmc runs of this command, FETCH_SIZE then WRITE_SIZE, scaled by a plain copy of known size).  It is a
    recorded figure, not one measured in the present run (counters need the profiler), so it comes with its
    source and with the algorithmic bytes of the run it was taken in."""
    rel = f"profiles/decode_split_{workload}_traffic.txt"
    got = {}
    try:
        for line in open(os.path.join(ROOT, rel)):
            for key in ("traffic_bytes_per_launch", "algorithmic_bytes_per_launch"):
                if line.startswith(key):
                    got[key] = int(float(line.split("=")[1].split()[0]))
    except OSError:
        pass
    if "traffic_bytes_per_launch" not in got:
        return {"traffic": None}
    return {"traffic": got["traffic_bytes_per_launch"],
            "traffic_source": f"recorded in {rel} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command), not measured in this run",
            "traffic_run_algorithmic_bytes": got.get("algorithmic_bytes_per_launch")}


def gpu_clocks(busy):
    """Clock speeds rocm-smi reports while `busy()` keeps the GPU loaded (a child process; None if unusable)."""
    import subprocess
    # under a profiler every child inherits its preloaded library (which touches the GPU before the child's own
    # exec of the script interpreter): no child processes then
    if "rocprof" in os.environ.get("LD_PRELOAD", "") or any(k.startswith("ROCPROF") for k in os.environ):
        return None
    try:
        pr = subprocess.Popen(["rocm-smi", "-d", "0", "--showclocks", "--json"], stdout=subprocess.PIPE,
                              stderr=subprocess.DEVNULL, text=True)
        t0 = time.perf_counter()
        while pr.poll() is None and time.perf_counter() - t0 < 20.0:
            busy()
        txt = pr.communicate(timeout=5)[0]
        card = next(iter(json.loads(txt).values()))
        return {k.split()[0]: v.strip("()") for k, v in card.items() if "clock speed" in k}
    except Exception:
        return None


def run_c5(args):
    """Config 5: `layers` attention layers of a Qwen3-8B-shaped model, batch 128 with seeded lengths uniform in
    [1024, 32768]; prefill through kitty_quantize_pages, then `steps` decode steps, each appending one token per
    sequence and attending in every layer (kitty_decode_step: one launch per layer).  Every layer has its own
    cache (pool, page table, windows); the caches are filled from two synthetic source sequences, shifted by one
    page per layer.  Page ids are handed out per sequence from a contiguous run, as a serving engine's allocator
    would: fresh id = run base + pages so far, computed on the device once per step."""
    import torch
    from paper_2511_18643_amd import kitty, synth
    from paper_2511_18643_amd import devcache as H
    dev = "cuda"
    w = synth.WORKLOADS["c5"]
    layers = args.layers or synth.C5_LAYERS
    steps = args.steps or synth.C5_STEPS
    B, hkv, hq = w.batch, w.n_kv_heads, w.n_q_heads
    S, VL = args.sink_tokens, args.v_local        # the paper's full cache organisation (Fig. 1) if given
    if S or VL or args.v_bits != 2:
        args.no_cpu_baseline = True               # the live oracle replay below is written for the default layout
    layout = kitty.make_layout(hq, hkv, w.n_boost, w.residual_window, w.rank_metric, sink_tokens=S, v_local=VL,
                               v_bits=args.v_bits)
    payload, rec_bytes = kitty.kitty_page_payload_bytes(layout), kitty.kitty_page_bytes(layout)
    lengths = synth.sequence_lengths(w)
    total = args.warmup + steps
    plan = H.VarLenPlan(lengths, total, S)
    np0, r0, max_pages, base, n_pool = plan.np0, plan.r0, plan.max_pages, plan.base, plan.n_pool

    t0 = time.time()
    nsrc = 2
    Ls = max(lengths) + 128 * layers
    ksrc, vsrc = H.varlen_sources(w, nsrc, Ls)
    kt, vt = H.bf16_tensor(ksrc, dev), H.bf16_tensor(vsrc, dev)
    gen_s = time.time() - t0

    tq0 = time.time()
    caches = [H.varlen_layer_cache(layout, w, plan, kt, vt, layer, S, VL, dev) for layer in range(layers)]
    # dispatch order: longest sequences first (every sequence grows by one token per step, so the order holds)
    if not args.no_seq_order:
        order = torch.argsort(caches[0].n_pages * 128 + caches[0].n_resid, descending=True).to(torch.int32)
        for c in caches:
            c.seq_order = order
    torch.cuda.synchronize()
    prefill_s = time.time() - tq0

    ns, pps = kitty.kitty_decode_plan(layout, B, max_pages, args.n_splits)
    ws = kitty.new_workspace(layout, B, max_pages, args.n_splits, device=dev)
    n_rot = 4
    qs = [H.bf16_tensor(synth.query(w, s), dev) for s in range(n_rot)]
    new_np = [synth.new_token(w, s) for s in range(n_rot)]
    newt = [tuple(H.bf16_tensor(x, dev) for x in kv) for kv in new_np]
    out = torch.empty((B, hq, 128), dtype=torch.bfloat16, device=dev)
    base_t = torch.tensor(base[:-1], dtype=torch.int32, device=dev)
    fresh = torch.empty((B,), dtype=torch.int32, device=dev)

    def launch_step(j):
        torch.add(base_t, caches[0].n_pages, out=fresh)      # next free page of every sequence's run
        kn, vn = newt[j]
        for c in caches:
            if args.two_calls:
                kitty.kitty_append_token(layout, c, kn, vn, fresh)
                kitty.kitty_decode_attention(layout, c, qs[j], out, w.sm_scale, ws, args.n_splits)
            else:
                kitty.kitty_decode_step(layout, c, kn, vn, fresh, qs[j], out, w.sm_scale, ws, args.n_splits)

    graphs = None
    if args.launch == "graph":      # one graph per input variant: 1 + layers kernel nodes each
        snap = [(c.n_pages.clone(), c.n_resid.clone(), c.resid_k.clone(), c.resid_v.clone(), c.page_table.clone()) for c in caches]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            launch_step(0)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graphs = []
        for j in range(n_rot):
            gph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gph):
                launch_step(j)
            graphs.append(gph)
        torch.cuda.synchronize()
        for c, (a, b_, k_, v_, p_) in zip(caches, snap):
            c.n_pages.copy_(a); c.n_resid.copy_(b_); c.resid_k.copy_(k_); c.resid_v.copy_(v_); c.page_table.copy_(p_)
        torch.cuda.synchronize()

    st_np, st_r = list(np0), list(r0)

    def do_step(i):
        nbytes = 0
        for b in range(B):
            if st_r[b] == 128:
                st_np[b] += 1
                st_r[b] = 0
            st_r[b] += 1
            nbytes += st_np[b] * payload + (st_r[b] + S) * 512 + (128 * 128 * 2 - (4096 + 512) if VL else 0)
        if graphs is not None:
            graphs[i % n_rot].replay()
        else:
            launch_step(i % n_rot)
        return layers * (hkv * nbytes + 2 * B * hq * 256)

    t_pre = time.perf_counter()
    while (time.perf_counter() - t_pre) * 1e3 < args.prewarm_ms:
        for c in caches[:4]:
            kitty.kitty_decode_split(layout, c, qs[0], w.sm_scale, ws, args.n_splits)
        torch.cuda.synchronize()
    for i in range(args.warmup):
        do_step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    total_bytes = 0
    for i in range(args.warmup, total):
        total_bytes += do_step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    # ---- the streaming kernel alone on the final state, HIP events on the launch stream ------------
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    kbytes = hkv * sum(p * payload + (r + S) * 512 + (128 * 128 * 2 - (4096 + 512) if VL else 0) for p, r in zip(st_np, st_r)) \
        + 2 * B * hq * 256
    for c in caches[:2]:
        kitty.kitty_decode_split(layout, c, qs[0], w.sm_scale, ws, args.n_splits)
    torch.cuda.synchronize()
    reps = 3
    ev0.record()
    for _ in range(reps):
        for c in caches:
            kitty.kitty_decode_split(layout, c, qs[0], w.sm_scale, ws, args.n_splits)
    ev1.record()
    torch.cuda.synchronize()
    kern_ms = ev0.elapsed_time(ev1) / (reps * layers)
    kern_gbps = kbytes / (kern_ms * 1e-3) / 1e9

    if args.calib_copy_mib:      # scale reference for the FETCH_SIZE / WRITE_SIZE counters
        src_c = torch.ones(args.calib_copy_mib << 20, dtype=torch.uint8, device=dev)
        dst_c = torch.empty_like(src_c)
        dst_c.copy_(src_c)
        torch.cuda.synchronize()
        del src_c, dst_c

    # ---- CPU oracle on a sample of layer 0: rebuilt from the inputs, appended tokens replayed ----------
    cpu, max_err = None, None
    if not args.no_cpu_baseline:
        from oracle import kitty_oracle as ko
        order = np.argsort(lengths)
        n_seq = args.cpu_pairs or 32
        sample_b = [int(x) for x in order[::max(len(order) // n_seq, 1)]] + [int(order[-1])]   # evenly over the lengths + the longest
        sample = [(b, h) for b in sample_b for h in (0, hkv - 1)]
        g = w.gqa
        out32 = torch.empty((B, hq, 128), dtype=torch.float32, device=dev)
        kitty.kitty_decode_attention(layout, caches[0], qs[0], out32, w.sm_scale, ws, args.n_splits)
        torch.cuda.synchronize()
        got = out32.cpu().numpy()
        qbits = synth.query(w, 0)
        wall, cpu_used, sample_bytes, worst = 0.0, 0.0, 0, 0.0
        for b, h in sample:
            sb = b % nsrc
            oc = ko.KittyCacheOracle(1, 1, g, w.n_boost, 128, max_pages, max_pages, w.rank_metric)
            n_p = np0[b]
            oc.quantize_pages(ksrc[sb, h, 0:n_p * 128].reshape(n_p, 1, 128, 128),
                              vsrc[sb, h, 0:n_p * 128].reshape(n_p, 1, 128, 128), list(range(n_p)))
            oc.page_table[0] = np.arange(max_pages); oc.n_pages[0] = n_p; oc.n_resid[0] = r0[b]
            oc.resid_k[0, 0, :r0[b]] = ksrc[sb, h, n_p * 128:n_p * 128 + r0[b]]
            oc.resid_v[0, 0, :r0[b]] = vsrc[sb, h, n_p * 128:n_p * 128 + r0[b]]
            for i in range(total):
                kn, vn = new_np[i % n_rot]
                oc.append_token(kn[b:b + 1, h:h + 1], vn[b:b + 1, h:h + 1], np.array([oc.n_pages[0]]))
            c0, w0 = time.process_time(), time.perf_counter()
            want = oc.decode_attention(qbits[b:b + 1, h * g:(h + 1) * g], w.sm_scale)[0]
            wall += time.perf_counter() - w0
            cpu_used += time.process_time() - c0
            worst = max(worst, float(np.abs(got[b, h * g:(h + 1) * g] - want).max()))
            sample_bytes += int(oc.n_pages[0]) * payload + int(oc.n_resid[0]) * 512 + 2 * g * 256
        max_err = worst
        cpu = {"value": round(sample_bytes / wall / 1e9, 4), "unit": "GB/s",
               "cores": max(1, int(round(cpu_used / max(wall, 1e-9)))), "kind": "oracle",
               "sample": f"layer 0, {len(sample)} (sequence, kv-head) pairs ({len(sample_b)} sequences spread evenly over the lengths, the longest among them; "
                         f"first and last kv-head) after the decode loop, all {g} query heads each, {wall:.1f} s wall "
                         f"(decode attention only)"}

    res = {
        "metric": "decode_attn_effective_hbm_gbps", "value": round(total_bytes / dt / 1e9, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup, "ms_per_step": round(dt / steps * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {
            "workload": f"c5: {layers} layers, batch {B}, {hq}q/{hkv}kv heads, head_dim 128, lengths uniform in [1024, 32768] "
                        f"(seeded; mean {np.mean(lengths):.0f}), n_boost {w.n_boost}, {args.v_bits}-bit Values"
                        f"{f', {S}-token Sink' if S else ''}{', Value Local window' if VL else ''}, step = one token per sequence through "
                        f"all layers ({'append_token + decode_attention' if args.two_calls else 'kitty_decode_step'} per layer, "
                        f"{args.launch} launch)",
            "n_splits": ns, "min_pages_per_split": pps, "record_bytes": rec_bytes, "payload_bytes_per_page": payload,
            "cache_bytes_resident": int(layers * n_pool * hkv * rec_bytes), "distinct_source_sequences": nsrc,
            "dispatch_order": "batch order" if args.no_seq_order else "longest sequence first (seq_order)",
        },
        "pct_of_hbm_peak": round(100.0 * total_bytes / dt / 1e9 / HBM_PEAK_GBPS, 2),
        "decode_tokens_per_s": round(B * steps / dt, 1),
        "roofline": {"bound": "hbm", "kernel": "decode_split_kernel", "achieved": round(kern_gbps, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(kern_gbps / HBM_PEAK_GBPS, 4), "traffic": None,
                     "avg_launch_ms": round(kern_ms, 5), "algorithmic_bytes_per_launch": int(kbytes)},
        "cpu_baseline": cpu,
        "max_abs_err_vs_oracle_sample": max_err,
        "setup_s": {"generate": round(gen_s, 1), "prefill_quantize_all_layers": round(prefill_s, 2)},
    }
    del caches, kt, vt
    torch.cuda.empty_cache()
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2511_18643_amd import kitty

    kitty.lib()      # fails loudly if libkitty.so is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.workload == "c5":
        print(json.dumps(run_c5(args)))
        return
    default_run = args.workload == "c3" and args.n_boost < 0 and args.v_bits == 2 and not (args.sink_tokens or args.v_local) \
        and not args.no_others
    res = run_layer(args, args.workload, headline=True)
    if default_run:
        res["other_workloads"] = other_workloads(args)
    print(json.dumps(res))


def compact(res):
    """The figures of a full result line that the summary of the other workloads keeps."""
    rf = res["roofline"]
    return {"workload": res["config"]["workload"], "n_splits": res["config"]["n_splits"], "steps": res["steps"],
            "algorithmic_bytes_per_launch": rf["algorithmic_bytes_per_launch"], "kernel_ms": rf["avg_launch_ms"],
            "kernel_gbps": rf["achieved"], "frac": rf["frac"], "ms_per_step": res["ms_per_step"],
            "step_gbps": res["value"], "decode_tokens_per_s": res["decode_tokens_per_s"],
            "max_abs_err_vs_oracle_sample": res["max_abs_err_vs_oracle_sample"],
            "oracle_sample": (res.get("cpu_baseline") or {}).get("sample")}


def other_workloads(args):
    """The configurations that are not the headline, each at its full size with fewer steps: the 8k and the 128k
    layer (same step, same timing as the headline, live oracle check on a few pairs) and the 36-layer
    variable-length loop; the page quantizer's figures come from the headline run's own prefill shape."""
    import copy
    import torch
    out = {}
    for key, name, pairs, batch in (("c2", "c2", 16, 0), ("c4", "c4", 2, 0), ("c4_one_sequence", "c4", 1, 1)):
        a = copy.copy(args)
        a.steps, a.warmup, a.cpu_pairs, a.prewarm_ms = min(args.steps or 200, 100), min(args.warmup, 10), pairs, 150.0
        a.batch = batch      # (c4_one_sequence: one 128k-token sequence, the latency case; 32 ranges and a merge)
        out[key] = compact(run_layer(a, name, headline=False))
        torch.cuda.empty_cache()
    a = copy.copy(args)
    a.steps, a.warmup, a.layers, a.prewarm_ms, a.cpu_pairs = min(args.steps or 16, 16), 2, 0, 150.0, 6
    out["c5"] = compact(run_c5(a))
    return out


def run_layer(args, wname, headline):
    """One attention layer's decode step on workload `wname` (c2, c3 or c4); see the module docstring."""
    import torch
    from paper_2511_18643_amd import kitty, synth
    from paper_2511_18643_amd import devcache as H
    dev = "cuda"
    args.steps = args.steps or 200
    w = synth.WORKLOADS[wname]
    if args.n_boost >= 0:
        w = synth.scaled(w, n_boost=args.n_boost)
    if getattr(args, "batch", 0):
        w = synth.scaled(w, batch=args.batch)
    S, VL = args.sink_tokens, args.v_local
    full_scheme = bool(S or VL)
    if full_scheme:
        args.no_cpu_baseline = True
    layout = kitty.make_layout(w.n_q_heads, w.n_kv_heads, w.n_boost, w.residual_window, w.rank_metric,
                               sink_tokens=S, v_local=VL, v_bits=args.v_bits)
    if args.v_bits != 2:
        args.no_cpu_baseline = True      # the live oracle replay below is written for the default record
    payload = kitty.kitty_page_payload_bytes(layout)
    rec_bytes = kitty.kitty_page_bytes(layout)
    n_pages0, r0 = w.pages_and_resid()                      # c3: 255 pages + 128 window rows
    hkv, B = w.n_kv_heads, w.batch
    copy_bytes = B * hkv * (n_pages0 * rec_bytes + 128 * 128 * 4)
    n_copies = args.copies or max(2, int(np.ceil(1.2e9 / copy_bytes)))
    total_steps = args.warmup + args.steps
    steps_per_copy = (total_steps + n_copies - 1) // n_copies
    extra_pages = (r0 + steps_per_copy) // 128 + 1
    max_pages = n_pages0 + extra_pages

    # ---- synthetic K/V: `src_seqs` distinct sequences (all kv-heads), tiled over the batch ----------
    t0 = time.time()
    nsrc = min(args.src_seqs, B)
    L = n_pages0 * 128 + 128
    ksrc = np.zeros((nsrc, hkv, L, 128), np.uint16)
    vsrc = np.zeros_like(ksrc)
    for sb in range(nsrc):
        for h in range(hkv):
            ksrc[sb, h], vsrc[sb, h] = synth.kv_block(w, sb, h, L)
    kt, vt = H.bf16_tensor(ksrc, dev), H.bf16_tensor(vsrc, dev)
    gen_s = time.time() - t0

    # ---- caches: prefill pages through kitty_quantize_pages, window = the tail tokens ---------------
    # the window starts `warm_per_copy + 1` rows short of full, so that the first timed step of each copy
    # runs at exactly the workload's shape (n_pages0 pages + 128 window rows)
    warm_per_copy = (args.warmup + n_copies - 1) // n_copies
    r_init = max(128 - 1 - warm_per_copy, 0)
    caches, states = [], []
    offs = torch.tensor([(b % nsrc) * hkv * L * 128 + i * 128 * 128 for b in range(B) for i in range(n_pages0)],
                        dtype=torch.int64, device=dev)
    ids = torch.tensor([b * max_pages + i for b in range(B) for i in range(n_pages0)], dtype=torch.int32, device=dev)
    tq0 = time.time()
    for c in range(n_copies):
        cache = kitty.Cache(layout, B, max_pages, B * max_pages, device=dev)
        kitty.kitty_quantize_pages(layout, kt, vt, 128 * 128, L * 128, 128, ids, B * n_pages0, cache.pool,
                                   cache.n_pool_pages, src_page_offsets=offs)
        pt = torch.arange(max_pages, dtype=torch.int32, device=dev)[None, :] + \
            (torch.arange(B, dtype=torch.int32, device=dev) * max_pages)[:, None]
        cache.page_table.copy_(pt)
        cache.n_pages.fill_(n_pages0)
        for b in range(B):
            cache.resid_k[b] = kt[b % nsrc, :, n_pages0 * 128:]
            if VL:      # the window's half, and the bf16 Value rows of the newest page in the other half
                cache.resid_v[b, :, n_pages0 & 1] = vt[b % nsrc, :, n_pages0 * 128:]
                cache.resid_v[b, :, (n_pages0 - 1) & 1] = vt[b % nsrc, :, (n_pages0 - 1) * 128:n_pages0 * 128]
            else:
                cache.resid_v[b] = vt[b % nsrc, :, n_pages0 * 128:]
            if S:       # Sink rows: any tokens of the right distribution (the timed path only reads them)
                cache.sink_k[b] = kt[b % nsrc, :, :S]
                cache.sink_v[b] = vt[b % nsrc, :, :S]
        if S:
            cache.n_sink.fill_(S)
        cache.n_resid.fill_(r_init)
        caches.append(cache)
        states.append([n_pages0, r_init])
    torch.cuda.synchronize()
    quant_s = time.time() - tq0

    ws = kitty.new_workspace(layout, B, max_pages, args.n_splits, device=dev)
    ns, pps = kitty.kitty_decode_plan(layout, B, max_pages, args.n_splits)
    n_rot = 4
    qs = [H.bf16_tensor(synth.query(w, s), dev) for s in range(n_rot)]
    newt = [tuple(H.bf16_tensor(x, dev) for x in synth.new_token(w, s)) for s in range(n_rot)]
    out = torch.empty((B, w.n_q_heads, 128), dtype=torch.bfloat16, device=dev)
    fresh = [torch.tensor([b * max_pages + n_pages0 for b in range(B)], dtype=torch.int32, device=dev) for _ in range(n_copies)]

    def launch_step(c, j):
        kn, vn = newt[j]
        if args.two_calls:
            kitty.kitty_append_token(layout, caches[c], kn, vn, fresh[c])
            kitty.kitty_decode_attention(layout, caches[c], qs[j], out, w.sm_scale, ws, args.n_splits)
        else:
            kitty.kitty_decode_step(layout, caches[c], kn, vn, fresh[c], qs[j], out, w.sm_scale, ws, args.n_splits)

    # one captured graph per cache copy (fixed q / new-token buffers per copy); the kernels read the
    # sequence state from device memory, so the same graph serves every step, flushes included
    graphs = None
    if args.launch == "graph":
        snap = [(c.n_pages.clone(), c.n_resid.clone(), c.resid_k.clone(), c.resid_v.clone()) for c in caches]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for c in range(n_copies):
                launch_step(c, c % n_rot)          # warm the launch path outside capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graphs = []
        for c in range(n_copies):
            gph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gph):
                launch_step(c, c % n_rot)
            graphs.append(gph)
        torch.cuda.synchronize()
        for c, (a, b_, k_, v_) in zip(caches, snap):     # undo the warm-up appends (capture itself runs nothing)
            c.n_pages.copy_(a); c.n_resid.copy_(b_); c.resid_k.copy_(k_); c.resid_v.copy_(v_)
        torch.cuda.synchronize()

    def do_step(i):
        c = i % n_copies
        st = states[c]
        flushed = st[1] == 128
        if flushed:
            st[0] += 1
            st[1] = 0
        st[1] += 1
        if graphs is not None:
            graphs[c].replay()
        else:
            launch_step(c, i % n_rot)
        if flushed:      # the id was consumed: point at the next free slot for the flush 128 steps from now
            fresh[c].copy_(torch.arange(B, dtype=torch.int32, device=dev) * max_pages + st[0])
        return step_bytes(payload, st[0], st[1], w, S, VL)

    # bring the GPU to its steady state first (the first ~100 ms after set-up run ~8 % slower); these launches
    # do not touch the sequence state
    t_pre = time.perf_counter()
    while (time.perf_counter() - t_pre) * 1e3 < args.prewarm_ms:
        for c in range(n_copies):
            kitty.kitty_decode_split(layout, caches[c], qs[0], w.sm_scale, ws, args.n_splits)
        torch.cuda.synchronize()
    for i in range(args.warmup):
        do_step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    total_bytes = 0
    for i in range(args.warmup, total_steps):
        total_bytes += do_step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    gbps = total_bytes / dt / 1e9
    tokens_per_s = B * args.steps / dt

    # ---- dominant kernel on its own: decode split-K, HIP events on the launch stream ----------------
    n_kern = max(args.steps, 50)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    kbytes = 0
    for i in range(4):
        kitty.kitty_decode_split(layout, caches[i % n_copies], qs[0], w.sm_scale, ws, args.n_splits)
    torch.cuda.synchronize()
    ev0.record()
    for i in range(n_kern):
        c = i % n_copies
        kitty.kitty_decode_split(layout, caches[c], qs[i % n_rot], w.sm_scale, ws, args.n_splits)
        kbytes += step_bytes(payload, states[c][0], states[c][1], w, S, VL)
    ev1.record()
    torch.cuda.synchronize()
    kern_ms = ev0.elapsed_time(ev1) / n_kern
    kern_gbps = kbytes / n_kern / (kern_ms * 1e-3) / 1e9
    spread, clocks, quant = None, None, None
    if headline:
        # spread of single launches (each bracketed by its own event pair; includes ~2 us of event overhead)
        pairs_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(100)]
        for i, (a, b_) in enumerate(pairs_ev):
            a.record()
            kitty.kitty_decode_split(layout, caches[i % n_copies], qs[i % n_rot], w.sm_scale, ws, args.n_splits)
            b_.record()
        torch.cuda.synchronize()
        single = np.sort(np.array([a.elapsed_time(b_) for a, b_ in pairs_ev]))
        spread = {"p10_ms": round(float(single[10]), 5), "median_ms": round(float(single[50]), 5),
                  "p90_ms": round(float(single[90]), 5)}

        def busy():
            for i in range(16):
                kitty.kitty_decode_split(layout, caches[i % n_copies], qs[0], w.sm_scale, ws, args.n_splits)
            torch.cuda.synchronize()
        clocks = gpu_clocks(busy)

        # ---- page quantizer on its own (the prefill of this workload: every page of every sequence and kv-head).
        # Every sequence reads its own copy of the source tokens, so that the input comes from HBM and not from
        # the last-level cache.  Bound: HBM; algorithmic bytes per (page, kv-head) = 2 x 32 KiB of bf16 in + the
        # record's payload out. -------------------------------------------------------------------------------
        reps_src = (B + nsrc - 1) // nsrc
        kt_all, vt_all = kt.repeat(reps_src, 1, 1, 1)[:B].contiguous(), vt.repeat(reps_src, 1, 1, 1)[:B].contiguous()
        offs_all = torch.tensor([b * hkv * L * 128 + i * 128 * 128 for b in range(B) for i in range(n_pages0)],
                                dtype=torch.int64, device=dev)
        quant_ms = []
        for _ in range(5):
            ev0.record()
            kitty.kitty_quantize_pages(layout, kt_all, vt_all, 128 * 128, L * 128, 128, ids, B * n_pages0, caches[0].pool,
                                       caches[0].n_pool_pages, src_page_offsets=offs_all)
            ev1.record()
            torch.cuda.synchronize()
            quant_ms.append(ev0.elapsed_time(ev1))
        quant_ms = float(np.median(quant_ms))
        quant_pages = B * n_pages0 * hkv
        del kt_all, vt_all
        # (the records just rewritten are identical: same inputs)
        qbytes = quant_pages * (65536 + payload)
        quant = {"kernel": "quantize_pages_kernel", "bound": "hbm", "page_heads": quant_pages, "ms": round(quant_ms, 4),
                 "algorithmic_bytes_per_launch": int(qbytes), "achieved": round(qbytes / (quant_ms * 1e-3) / 1e9, 1),
                 "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(qbytes / (quant_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                 "input_gbps": round(quant_pages * 65536 / (quant_ms * 1e-3) / 1e9, 1)}

    if args.calib_copy_mib:
        src_c = torch.ones(args.calib_copy_mib << 20, dtype=torch.uint8, device=dev)
        dst_c = torch.empty_like(src_c)
        dst_c.copy_(src_c)
        torch.cuda.synchronize()
        del src_c, dst_c

    # ---- CPU oracle on a bounded sample of the same workload + live parity on that sample -------
    cpu = None
    max_err = None
    if not args.no_cpu_baseline:
        from oracle import kitty_oracle as ko
        c0 = caches[0]
        n_pairs = min(args.cpu_pairs or 160, B * hkv)       # ~70 ms of oracle attention per pair at 32k context
        pairs_kv = [(b, h) for b in range(B) for h in range(hkv)][:n_pairs]
        # rebuild the sampled sequences on the CPU from the inputs (never from GPU results); sequences
        # tiled from the same source sequence share their prefill records
        oc = ko.KittyCacheOracle(B, hkv, w.n_q_heads, w.n_boost, w.residual_window, max_pages, B * max_pages,
                                 w.rank_metric)
        tq = time.time()
        src_recs = {}
        for (b, h) in pairs_kv:
            key = (b % nsrc, h)
            if key not in src_recs:
                recs = []
                for i in range(n_pages0):
                    kp = ko.quantize_k_page(ko.bf16_bits_to_f32(ksrc[key[0], h, 128 * i:128 * (i + 1)]), w.n_boost, w.rank_metric)
                    vp = ko.quantize_v_page(ko.bf16_bits_to_f32(vsrc[key[0], h, 128 * i:128 * (i + 1)]))
                    recs.append(ko.pack_record(kp, vp))
                src_recs[key] = np.stack(recs)
            oc.pool[b * max_pages:b * max_pages + n_pages0, h] = src_recs[key]
        oracle_quant_s = time.time() - tq
        # replay copy 0's history on the oracle for the sampled pairs: window tail + appended tokens
        oc.page_table[:] = np.arange(max_pages)[None, :] + (np.arange(B) * max_pages)[:, None]
        oc.n_pages[:] = n_pages0
        oc.n_resid[:] = r_init
        for b in range(B):
            oc.resid_k[b] = ksrc[b % nsrc, :, n_pages0 * 128:]
            oc.resid_v[b] = vsrc[b % nsrc, :, n_pages0 * 128:]
        sample_b = sorted({b for b, _ in pairs_kv})
        steps_c0 = [i for i in range(total_steps) if i % n_copies == 0]
        new_np = [tuple(x for x in synth.new_token(w, s)) for s in range(n_rot)]
        for i in steps_c0:
            kn, vn = new_np[0 if graphs is not None else i % n_rot]
            for b in sample_b:          # the oracle's append, restricted to the sampled sequences
                if oc.n_resid[b] == 128:
                    pid = b * max_pages + int(oc.n_pages[b])
                    for h in range(hkv):
                        if (b, h) in pairs_kv:
                            kp = ko.quantize_k_page(ko.bf16_bits_to_f32(oc.resid_k[b, h]), w.n_boost, w.rank_metric)
                            vp = ko.quantize_v_page(ko.bf16_bits_to_f32(oc.resid_v[b, h]))
                            oc.pool[pid, h] = ko.pack_record(kp, vp)
                    oc.n_pages[b] += 1
                    oc.n_resid[b] = 0
                oc.resid_k[b, :, oc.n_resid[b]] = kn[b]
                oc.resid_v[b, :, oc.n_resid[b]] = vn[b]
                oc.n_resid[b] += 1
        # GPU result for the current state of copy 0 with query 0
        out32 = torch.empty((B, w.n_q_heads, 128), dtype=torch.float32, device=dev)
        kitty.kitty_decode_attention(layout, c0, qs[0], out32, w.sm_scale, ws, args.n_splits)
        torch.cuda.synchronize()
        got = out32.cpu().numpy()
        qbits = synth.query(w, 0)
        g = w.gqa
        hq_pairs = [(b, h * g + e) for (b, h) in pairs_kv for e in range(g)]
        cpu_t0, wall_t0 = time.process_time(), time.perf_counter()
        want = oc.decode_attention(qbits, w.sm_scale, pairs=hq_pairs)
        wall = time.perf_counter() - wall_t0
        cpu_used = time.process_time() - cpu_t0
        max_err = max(float(np.abs(got[b, hq] - want[b, hq]).max()) for b, hq in hq_pairs)
        sample_bytes = len(pairs_kv) * (int(oc.n_pages[sample_b[0]]) * payload + int(oc.n_resid[sample_b[0]]) * 512) \
            + 2 * len(hq_pairs) * 256
        cpu = {
            "value": round(sample_bytes / wall / 1e9, 4), "unit": "GB/s",
            "cores": max(1, int(round(cpu_used / max(wall, 1e-9)))), "kind": "oracle",
            "sample": f"{len(pairs_kv)} of {B * hkv} (sequence, kv-head) pairs at full context, all {g} query heads each, "
                      f"{wall:.1f} s wall (decode attention only; oracle quantization of the sample took {oracle_quant_s:.1f} s)",
        }

    traffic = {"traffic": None}
    if args.n_boost < 0 and not full_scheme and args.v_bits == 2:
        traffic = recorded_traffic(w.name)
    res = {
        "metric": "decode_attn_effective_hbm_gbps", "value": round(gbps, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8",
        "data": "synthetic",
        "config": {
            "workload": f"{w.name}: batch {B}, {w.n_q_heads}q/{hkv}kv heads, head_dim 128, context {w.context} "
                        f"({n_pages0} pages + 128-token bf16 window at the first timed step"
                        f"{f' + {S}-token Sink' if S else ''}{', Values of the newest page in the bf16 Local window' if VL else ''}), n_boost {w.n_boost}, "
                        f"{args.v_bits}-bit Values, "
                        f"step = append_token + decode_attention ({'two calls' if args.two_calls else 'kitty_decode_step'}, {args.launch} launch)",
            "n_splits": ns, "min_pages_per_split": pps, "cache_copies": n_copies, "record_bytes": rec_bytes,
            "payload_bytes_per_page": payload, "distinct_source_sequences": nsrc,
        },
        "pct_of_hbm_peak": round(100.0 * gbps / HBM_PEAK_GBPS, 2),
        "decode_tokens_per_s": round(tokens_per_s, 1),
        "roofline": {
            "bound": "hbm", "kernel": "decode_split_kernel", "achieved": round(kern_gbps, 1), "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": round(kern_gbps / HBM_PEAK_GBPS, 4),
            "avg_launch_ms": round(kern_ms, 5), "algorithmic_bytes_per_launch": int(kbytes / n_kern),
            "single_launch": spread, **traffic,
        },
        "cpu_baseline": cpu,
        "max_abs_err_vs_oracle_sample": max_err,
        "quantize_pages": quant,
        "clocks_under_load": clocks,
        "setup_s": {"generate": round(gen_s, 1), "prefill_quantize_all_copies": round(quant_s, 2)},
    }
    return res


if __name__ == "__main__":
    main()
