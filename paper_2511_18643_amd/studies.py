"""Two measurements around the hot path, each printing one JSON line (run on one MI355X):

  python -m paper_2511_18643_amd.studies prefill [--tokens N] [--hidden H]
      Prefill of one attention layer's cache for a Llama-3-8B-shaped layer (8 kv-heads of 128 channels): the
      Key/Value projection of `tokens` tokens followed by the page quantizer, three ways:
        two_step   one library GEMM for all tokens (torch.matmul), bf16 K/V written to device memory, then
                   kitty_quantize_pages reading them in place (token-major layout, no repacking copy);
        chunked    the same two calls per chunk of tokens small enough that the chunk's bf16 K/V are still in the
                   last-level cache when the quantizer reads them;
        fused      kitty_project_quantize_pages (projection tile and quantizer in one kernel; the bf16 K/V never
                   reach device memory).
      Records written by two_step and chunked are compared byte for byte; fused is compared by the fraction of
      equal bytes (its fp32 sums are taken in another order).

  python -m paper_2511_18643_amd.studies memory [--context L] [--decode-steps K]
      The batch-size-until-out-of-memory experiment of the paper's system evaluation (Sec. 5.5, the memory and
      throughput figure) for a Qwen3-8B-shaped cache (36 layers, 8 kv-heads, head size 128) at `context` tokens per
      sequence: the batch is doubled and the whole cache allocated (and touched) for a bf16 cache and for the packed
      records + bf16 windows, until the allocator refuses; the refusal is an exception caught on the host, nothing
      is launched after it.  For every batch the packed cache fits, `decode-steps` decode steps through all layers
      are timed (kitty_decode_step; the records hold whatever the allocator returned: timing only).

Inputs are synthetic (seeded Gaussians); nothing here touches the CPU oracle.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np


def prefill(args):
    import torch
    from . import kitty
    dev = "cuda"
    hkv, hq, D = 8, 32, 128
    T, Hd = args.tokens, args.hidden
    assert T % 128 == 0
    n_pages = T // 128
    g = torch.Generator(device=dev).manual_seed(1234)
    x = torch.randn((T, Hd), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    wk = (torch.randn((hkv * D, Hd), generator=g, device=dev, dtype=torch.float32) / Hd ** 0.5)
    wk[::21] *= 8.0                                    # a few high-magnitude Key channels per head
    wk = wk.to(torch.bfloat16)
    wv = (torch.randn((hkv * D, Hd), generator=g, device=dev, dtype=torch.float32) / Hd ** 0.5).to(torch.bfloat16)
    layout = kitty.make_layout(hq, hkv, 16)
    rb = kitty.kitty_page_bytes(layout)
    pools = {k: torch.empty((n_pages, hkv, rb), dtype=torch.uint8, device=dev) for k in ("two_step", "chunked", "fused")}
    ids = torch.arange(n_pages, dtype=torch.int32, device=dev)
    tok_off = torch.arange(n_pages, dtype=torch.int64, device=dev) * 128
    kbuf = torch.empty((T, hkv * D), dtype=torch.bfloat16, device=dev)
    vbuf = torch.empty_like(kbuf)

    def two_step(pool, t0=0, t1=T):
        torch.matmul(x[t0:t1], wk.t(), out=kbuf[t0:t1])
        torch.matmul(x[t0:t1], wv.t(), out=vbuf[t0:t1])
        p0, p1 = t0 // 128, t1 // 128
        offs = tok_off[p0:p1] * (hkv * D)
        kitty.kitty_quantize_pages(layout, kbuf, vbuf, 0, D, hkv * D, ids[p0:p1], p1 - p0, pool, n_pages, src_page_offsets=offs)

    chunk = args.chunk_tokens

    def chunked(pool):
        for t0 in range(0, T, chunk):
            two_step(pool, t0, min(t0 + chunk, T))

    def fused(pool):
        kitty.kitty_project_quantize_pages(layout, x, Hd, Hd, wk, wv, tok_off, ids, n_pages, pool, n_pages)

    def timed(fn, pool, reps=3):
        fn(pool)
        torch.cuda.synchronize()
        best = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn(pool)
            e1.record()
            torch.cuda.synchronize()
            best.append(e0.elapsed_time(e1))
        return float(np.median(best))

    ms = {"two_step": timed(two_step, pools["two_step"]), "chunked": timed(chunked, pools["chunked"]),
          "fused": timed(fused, pools["fused"])}
    # the parts of two_step on their own
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    torch.matmul(x, wk.t(), out=kbuf)
    torch.matmul(x, wv.t(), out=vbuf)
    e1.record()
    torch.cuda.synchronize()
    gemm_ms = e0.elapsed_time(e1)
    # the quantizer alone, reading the token-major projection output in place
    def quant_only(pool):
        kitty.kitty_quantize_pages(layout, kbuf, vbuf, 0, D, hkv * D, ids, n_pages, pool, n_pages, src_page_offsets=tok_off * (hkv * D))
    quant_ms = timed(quant_only, pools["two_step"], reps=5)
    flops = 2.0 * T * Hd * (2 * hkv * D)
    same_chunked = bool(torch.equal(pools["two_step"], pools["chunked"]))
    same_fused = float((pools["two_step"] == pools["fused"]).float().mean())
    print(json.dumps({
        "study": "prefill", "tokens": T, "hidden": Hd, "kv_heads": hkv, "pages": n_pages * hkv, "chunk_tokens": chunk,
        "projection_flop": flops, "ms": {k: round(v, 3) for k, v in ms.items()},
        "two_step_parts_ms": {"projection_gemms": round(gemm_ms, 3), "quantize_pages": round(quant_ms, 3)},
        "quantize_pages_traffic_gbps": round(n_pages * hkv * (65536 + rb) / (quant_ms * 1e-3) / 1e9, 1),
        "tflops": {k: round(flops / (v * 1e-3) / 1e12, 1) for k, v in ms.items()},
        "bf16_kv_round_trip_bytes_saved_by_fusion": int(2 * 2 * T * hkv * D * 2),
        "records_equal_two_step_vs_chunked": same_chunked, "fraction_of_equal_record_bytes_fused_vs_two_step": round(same_fused, 5),
    }))


def memory(args):
    import torch
    from . import kitty
    dev = "cuda"
    layers, hkv, hq, D = 36, 8, 32, 128
    L = args.context
    np_seq, r = (L + 127) // 128 - 1, L - 128 * ((L + 127) // 128 - 1)
    layout = kitty.make_layout(hq, hkv, args.n_boost)
    rb = kitty.kitty_page_bytes(layout)
    total_mem = torch.cuda.get_device_properties(0).total_memory
    free0, _ = torch.cuda.mem_get_info()
    rows = []

    def try_alloc(kind, B):
        """Allocates the whole cache of `kind` for batch B, layer by layer, touching every byte.  Returns
        (tensors, bytes) or (None, reason) when the allocator refuses."""
        held = []
        try:
            for _ in range(layers):
                if kind == "bf16":
                    t = torch.empty((2, B, hkv, L, D), dtype=torch.bfloat16, device=dev)       # K and V
                    t.zero_()
                    held.append(t)
                else:
                    c = kitty.Cache(layout, B, np_seq + 1, B * (np_seq + 1), device=dev)       # zero-filled by the binding
                    held.append(c)
            torch.cuda.synchronize()
            return held, torch.cuda.memory_allocated()
        except torch.OutOfMemoryError as e:       # the allocator refused: free what this attempt holds, launch nothing
            held.clear()
            torch.cuda.empty_cache()
            return None, str(e).split("\n")[0][:160]

    for kind in ("bf16", "kitty"):
        B = args.first_batch
        while True:
            torch.cuda.empty_cache()
            need = layers * (2 * B * hkv * L * D * 2 if kind == "bf16"
                             else B * (np_seq + 1) * hkv * rb + 2 * B * hkv * 128 * D * 2)
            t0 = time.time()
            held, info = try_alloc(kind, B)
            row = {"cache": kind, "batch": B, "bytes_by_formula": int(need)}
            if held is None:
                row.update({"fits": False, "allocator_said": info})
                rows.append(row)
                break
            row.update({"fits": True, "bytes_allocated": int(info), "gb_allocated": round(info / 1e9, 2),
                        "alloc_s": round(time.time() - t0, 2)})
            if kind == "kitty" and args.decode_steps:
                # decode throughput at this batch: every sequence at `context` tokens, one token per step through all layers
                ws = kitty.new_workspace(layout, B, np_seq + 1)
                q = torch.randn((B, hq, D), device=dev, dtype=torch.float32).to(torch.bfloat16)
                kn = torch.randn((B, hkv, D), device=dev, dtype=torch.float32).to(torch.bfloat16)
                out = torch.empty((B, hq, D), dtype=torch.bfloat16, device=dev)
                fresh = torch.arange(B, dtype=torch.int32, device=dev) * (np_seq + 1) + np_seq
                for c in held:
                    c.page_table.copy_(torch.arange(B * (np_seq + 1), dtype=torch.int32, device=dev).view(B, np_seq + 1))
                    c.n_pages.fill_(np_seq)
                    c.n_resid.fill_(max(r - args.decode_steps - 2, 1))      # no flush inside the timed steps
                def step():
                    for c in held:
                        kitty.kitty_decode_step(layout, c, kn, kn, fresh, q, out, 0.088, ws)
                step(); step()
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                for _ in range(args.decode_steps):
                    step()
                torch.cuda.synchronize()
                dt = (time.perf_counter() - t1) / args.decode_steps
                row.update({"ms_per_decode_step": round(dt * 1e3, 3), "decode_tokens_per_s": round(B / dt, 1)})
                del ws, q, kn, out, fresh
            rows.append(row)
            del held
            B *= 2
    best = {k: max([r_["batch"] for r_ in rows if r_["cache"] == k and r_["fits"]], default=0) for k in ("bf16", "kitty")}
    print(json.dumps({
        "study": "memory", "model_shape": f"{layers} layers x {hkv} kv-heads x {D}", "context": L, "n_boost": args.n_boost,
        "device_total_bytes": int(total_mem), "device_free_bytes_at_start": int(free0),
        "bytes_per_token_bf16": layers * 2 * hkv * D * 2, "bytes_per_token_kitty_records": round(layers * hkv * rb / 128, 1),
        "largest_batch_that_fits": best, "batch_ratio": (best["kitty"] / best["bf16"]) if best["bf16"] else None,
        "rows": rows,
    }))


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    p = sub.add_parser("prefill")
    p.add_argument("--tokens", type=int, default=131072)
    p.add_argument("--hidden", type=int, default=4096)
    p.add_argument("--chunk-tokens", type=int, default=8192)
    m = sub.add_parser("memory")
    m.add_argument("--context", type=int, default=8192)
    m.add_argument("--n-boost", type=int, default=32)
    m.add_argument("--first-batch", type=int, default=8)
    m.add_argument("--decode-steps", type=int, default=4)
    args = ap.parse_args()
    import torch
    from . import kitty
    kitty.lib()
    assert torch.cuda.is_available(), "needs a GPU"
    {"prefill": prefill, "memory": memory}[args.cmd](args)


if __name__ == "__main__":
    sys.exit(main())
