"""Device-side cache builders for tests, the smoke check and the benchmark: they generate seeded sequences and
fill a `kitty.Cache` through the library's own entry points (kitty_quantize_pages + plain tensor copies for the
full-precision rows).  Argument plumbing only: none of the method's arithmetic lives here, and nothing here
touches the CPU oracle."""
from __future__ import annotations

import numpy as np

from . import synth


def gen_sequences(w, lengths):
    """bf16 bits [B][Hkv][Lmax][D] for K and V (rows beyond a sequence's length are zero)."""
    lmax = max(max(lengths), 1)
    k = np.zeros((w.batch, w.n_kv_heads, lmax, 128), np.uint16)
    v = np.zeros_like(k)
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            if lengths[b]:
                kb, vb = synth.kv_block(w, b, h, lengths[b])
                k[b, h, :lengths[b]] = kb
                v[b, h, :lengths[b]] = vb
    return k, v


def bf16_tensor(bits, device="cuda"):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def gpu_cache(w, lengths, k, v, max_pages, poison=True, v_bits=2):
    """Cache filled by kitty_quantize_pages + window copies.  Returns (layout, Cache)."""
    import torch
    from . import kitty
    layout = kitty.make_layout(w.n_q_heads, w.n_kv_heads, w.n_boost, w.residual_window, w.rank_metric, v_bits=v_bits)
    c = kitty.Cache(layout, w.batch, max_pages, w.batch * max_pages)
    if poison:
        c.pool.fill_(0xA5)      # every byte of a written record must be overwritten
    kt, vt = bf16_tensor(k), bf16_tensor(v)
    lmax = k.shape[2]
    offs, ids, npg, nres = [], [], [], []
    for b in range(w.batch):
        n_pages, r = w.pages_and_resid(lengths[b]) if lengths[b] else (0, 0)
        for i in range(n_pages):
            offs.append(b * w.n_kv_heads * lmax * 128 + i * 128 * 128)
            ids.append(b * max_pages + i)
        npg.append(n_pages)
        nres.append(r)
        c.page_table[b, :n_pages] = torch.arange(n_pages, dtype=torch.int32, device="cuda") + b * max_pages
        if r:
            c.resid_k[b, :, :r] = kt[b, :, n_pages * 128:n_pages * 128 + r]
            c.resid_v[b, :, :r] = vt[b, :, n_pages * 128:n_pages * 128 + r]
    c.n_pages.copy_(torch.tensor(npg, dtype=torch.int32))
    if c.n_resid is not None:
        c.n_resid.copy_(torch.tensor(nres, dtype=torch.int32))
    if ids:
        offs_t = torch.tensor(offs, dtype=torch.int64, device="cuda")
        ids_t = torch.tensor(ids, dtype=torch.int32, device="cuda")
        kitty.kitty_quantize_pages(layout, kt, vt, 128 * 128, lmax * 128, 128, ids_t, len(ids), c.pool,
                                   c.n_pool_pages, src_page_offsets=offs_t)
    torch.cuda.synchronize()
    return layout, c


def gpu_decode(layout, c, q_bits, sm_scale, n_splits=0, fp32=True):
    import torch
    from . import kitty
    q = bf16_tensor(q_bits)
    out = torch.full(q.shape, float("nan"), dtype=torch.float32 if fp32 else torch.bfloat16, device="cuda")
    ws = kitty.new_workspace(layout, c.batch, c.max_pages, n_splits)
    ws.fill_(float("nan"))
    kitty.kitty_decode_attention(layout, c, q, out, sm_scale, ws, n_splits)
    torch.cuda.synchronize()
    return out.float().cpu().numpy()


def gpu_full_cache(w, lengths, k, v, max_pages, sink, v_local, poison=True, v_bits=2):
    """Prefilled cache with a Sink of `sink` tokens and (v_local = 128) the Value Local window: the first tokens
    go to the Sink, whole pages behind it through kitty_quantize_pages, the tail to the window; the bf16 Value
    rows of the newest page are placed in their half of resid_v."""
    import torch
    from . import kitty
    layout = kitty.make_layout(w.n_q_heads, w.n_kv_heads, w.n_boost, w.residual_window, w.rank_metric,
                               sink_tokens=sink, v_local=v_local, v_bits=v_bits)
    c = kitty.Cache(layout, w.batch, max_pages, w.batch * max_pages)
    if poison:
        c.pool.fill_(0xA5)
    kt, vt = bf16_tensor(k), bf16_tensor(v)
    lmax = k.shape[2]
    offs, ids, npg, nres, nsk = [], [], [], [], []
    for b in range(w.batch):
        n = lengths[b]
        s = min(n, sink)
        post = n - s
        if w.residual_window:
            n_pages = max((post + 127) // 128 - 1, 0)
        else:
            assert post % 128 == 0
            n_pages = post // 128
        r = post - n_pages * 128
        if s:
            c.sink_k[b, :, :s] = kt[b, :, :s]
            c.sink_v[b, :, :s] = vt[b, :, :s]
        for i in range(n_pages):
            offs.append(b * w.n_kv_heads * lmax * 128 + (s + i * 128) * 128)
            ids.append(b * max_pages + i)
        c.page_table[b, :n_pages] = torch.arange(n_pages, dtype=torch.int32, device="cuda") + b * max_pages
        t0 = s + n_pages * 128
        if r:
            c.resid_k[b, :, :r] = kt[b, :, t0:t0 + r]
            if v_local:
                c.resid_v[b, :, n_pages & 1, :r] = vt[b, :, t0:t0 + r]
            else:
                c.resid_v[b, :, :r] = vt[b, :, t0:t0 + r]
        if v_local and n_pages:
            c.resid_v[b, :, (n_pages - 1) & 1] = vt[b, :, t0 - 128:t0]
        npg.append(n_pages); nres.append(r); nsk.append(s)
    c.n_pages.copy_(torch.tensor(npg, dtype=torch.int32))
    if c.n_resid is not None:
        c.n_resid.copy_(torch.tensor(nres, dtype=torch.int32))
    if c.n_sink is not None:
        c.n_sink.copy_(torch.tensor(nsk, dtype=torch.int32))
    if ids:
        kitty.kitty_quantize_pages(layout, kt, vt, 128 * 128, lmax * 128, 128,
                                   torch.tensor(ids, dtype=torch.int32, device="cuda"), len(ids), c.pool, c.n_pool_pages,
                                   src_page_offsets=torch.tensor(offs, dtype=torch.int64, device="cuda"))
    torch.cuda.synchronize()
    return layout, c


# ---------------------------------------------------------------------------------------------------
# Variable-length batch of the 36-layer decode loop: one cache per layer, page ids handed out per sequence
# from a contiguous run (as a serving engine's allocator would)
# ---------------------------------------------------------------------------------------------------
class VarLenPlan:
    """Page bookkeeping of a variable-length batch that will run `total_steps` decode steps: pages and window
    rows of every sequence at the start, row length of the page table, the first page id of every sequence's
    run (one spare page per run) and the pool size."""

    def __init__(self, lengths, total_steps, sink=0):
        self.lengths = list(lengths)
        self.np0 = [(n - sink + 127) // 128 - 1 for n in lengths]           # the first `sink` tokens sit in the Sink
        self.r0 = [n - sink - 128 * p for n, p in zip(lengths, self.np0)]
        np_end = [(n - sink + total_steps + 127) // 128 - 1 for n in lengths]
        self.max_pages = max(np_end) + 1
        self.base = np.concatenate([[0], np.cumsum([p + 1 for p in np_end])]).astype(np.int64)
        self.n_pool = int(self.base[-1])


def varlen_sources(w, n_src, n_tokens):
    """bf16 bits [n_src][Hkv][n_tokens][D] of K and V: the distinct synthetic sequences a batch is tiled from."""
    ksrc = np.zeros((n_src, w.n_kv_heads, n_tokens, 128), np.uint16)
    vsrc = np.zeros_like(ksrc)
    for sb in range(n_src):
        for h in range(w.n_kv_heads):
            ksrc[sb, h], vsrc[sb, h] = synth.kv_block(w, sb, h, n_tokens)
    return ksrc, vsrc


def varlen_layer_cache(layout, w, plan, kt, vt, layer, sink=0, v_local=0, device="cuda"):
    """Cache of one layer: sequence b holds tokens [128*layer, 128*layer + length) of source sequence b % n_src
    (kt, vt: bf16 tensors [n_src][Hkv][Ls][D] on the device), prefilled through kitty_quantize_pages."""
    import torch
    from . import kitty
    B, hkv = w.batch, w.n_kv_heads
    nsrc, Ls = kt.shape[0], kt.shape[2]
    S, VL = sink, v_local
    c = kitty.Cache(layout, B, plan.max_pages, plan.n_pool, device=device)
    ids = torch.tensor([plan.base[b] + i for b in range(B) for i in range(plan.np0[b])], dtype=torch.int32, device=device)
    offs = torch.tensor([(b % nsrc) * hkv * Ls * 128 + (S + (layer + i) * 128) * 128 for b in range(B) for i in range(plan.np0[b])],
                        dtype=torch.int64, device=device)
    if ids.numel():
        kitty.kitty_quantize_pages(layout, kt, vt, 128 * 128, Ls * 128, 128, ids, ids.numel(), c.pool, plan.n_pool,
                                   src_page_offsets=offs)
    pt = torch.zeros((B, plan.max_pages), dtype=torch.int32)
    for b in range(B):
        pt[b, :plan.np0[b]] = torch.arange(plan.np0[b], dtype=torch.int32) + int(plan.base[b])
    c.page_table.copy_(pt)
    c.n_pages.copy_(torch.tensor(plan.np0, dtype=torch.int32))
    c.n_resid.copy_(torch.tensor(plan.r0, dtype=torch.int32))
    for b in range(B):
        a = S + (layer + plan.np0[b]) * 128
        r = plan.r0[b]
        c.resid_k[b, :, :r] = kt[b % nsrc, :, a:a + r]
        if VL:      # the window's half, and the bf16 Value rows of the newest page in the other half
            c.resid_v[b, :, plan.np0[b] & 1, :r] = vt[b % nsrc, :, a:a + r]
            c.resid_v[b, :, (plan.np0[b] - 1) & 1] = vt[b % nsrc, :, a - 128:a]
        else:
            c.resid_v[b, :, :r] = vt[b % nsrc, :, a:a + r]
        if S:
            c.sink_k[b] = kt[b % nsrc, :, :S]
            c.sink_v[b] = vt[b % nsrc, :, :S]
    if S:
        c.n_sink.fill_(S)
    return c
