"""Builds the same cache twice from one seeded workload: once through the CPU oracle, once on the
GPU through the C-ABI binding.  The two sides share only the input bits."""
from __future__ import annotations

import numpy as np

from oracle import kitty_oracle as ko
from paper_2511_18643_amd import synth


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


def oracle_cache(w, lengths, k, v, max_pages, v_bits=2):
    c = ko.KittyCacheOracle(w.batch, w.n_kv_heads, w.n_q_heads, w.n_boost, w.residual_window,
                            max_pages, w.batch * max_pages, w.rank_metric, v_bits)
    for b in range(w.batch):
        n_pages, r = w.pages_and_resid(lengths[b]) if lengths[b] else (0, 0)
        ids = np.arange(n_pages) + b * max_pages
        if n_pages:
            kb = k[b, :, :n_pages * 128].reshape(w.n_kv_heads, n_pages, 128, 128).transpose(1, 0, 2, 3)
            vb = v[b, :, :n_pages * 128].reshape(w.n_kv_heads, n_pages, 128, 128).transpose(1, 0, 2, 3)
            c.quantize_pages(kb, vb, ids)
        c.page_table[b, :n_pages] = ids
        c.n_pages[b] = n_pages
        if r:
            c.resid_k[b, :, :r] = k[b, :, n_pages * 128:n_pages * 128 + r]
            c.resid_v[b, :, :r] = v[b, :, n_pages * 128:n_pages * 128 + r]
        c.n_resid[b] = r
    return c


def bf16_tensor(bits, device="cuda"):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def gpu_cache(w, lengths, k, v, max_pages, poison=True, v_bits=2):
    """Cache filled by kitty_quantize_pages + window copies.  Returns (layout, Cache)."""
    import torch
    from paper_2511_18643_amd import kitty
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
    from paper_2511_18643_amd import kitty
    q = bf16_tensor(q_bits)
    out = torch.full(q.shape, float("nan"), dtype=torch.float32 if fp32 else torch.bfloat16, device="cuda")
    ws = kitty.new_workspace(layout, c.batch, c.max_pages, n_splits)
    ws.fill_(float("nan"))
    kitty.kitty_decode_attention(layout, c, q, out, sm_scale, ws, n_splits)
    torch.cuda.synchronize()
    return out.float().cpu().numpy()


# ---------------------------------------------------------------------------------------------------
# Full scheme (Sink + Value Local window): the oracle side is one KittyUnitOracle per (sequence, kv-head)
# ---------------------------------------------------------------------------------------------------
def unit_oracles(w, lengths, k, v, sink, local, v_bits=2):
    """Units fed token by token (steps 1 and 3 of the pipeline) with the first lengths[b] tokens, left in the
    state attention sees right after the last insert (step 3 of that last step still pending).  Without a
    residual window the cache is static and every token behind the Sink has been quantized."""
    units = {}
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            u = ko.KittyUnitOracle(w.n_boost, sink=sink, local=local, rank_metric=w.rank_metric, v_bits=v_bits)
            n = lengths[b]
            if n and w.residual_window == 0:       # static cache: everything behind the Sink is in pages
                u.prefill(k[b, h, :n], v[b, h, :n])
            elif n:
                u.prefill(k[b, h, :n - 1], v[b, h, :n - 1])
                u.insert(k[b, h, n - 1], v[b, h, n - 1])
            units[(b, h)] = u
    return units


def units_attention(w, units, q_bits, sm_scale):
    g = w.gqa
    out = np.zeros((w.batch, w.n_q_heads, 128), np.float64)
    for (b, h), u in units.items():
        out[b, h * g:(h + 1) * g] = u.attention(q_bits[b, h * g:(h + 1) * g], sm_scale)
    return out


def gpu_full_cache(w, lengths, k, v, max_pages, sink, v_local, poison=True, v_bits=2):
    """Prefilled cache with a Sink of `sink` tokens and (v_local = 128) the Value Local window: the first tokens
    go to the Sink, whole pages behind it through kitty_quantize_pages, the tail to the window; the bf16 Value
    rows of the newest page are placed in their half of resid_v."""
    import torch
    from paper_2511_18643_amd import kitty
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
