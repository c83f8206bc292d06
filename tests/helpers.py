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


def oracle_cache(w, lengths, k, v, max_pages):
    c = ko.KittyCacheOracle(w.batch, w.n_kv_heads, w.n_q_heads, w.n_boost, w.residual_window,
                            max_pages, w.batch * max_pages, w.rank_metric)
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


def gpu_cache(w, lengths, k, v, max_pages, poison=True):
    """Cache filled by kitty_quantize_pages + window copies.  Returns (layout, Cache)."""
    import torch
    from paper_2511_18643_amd import kitty
    layout = kitty.make_layout(w.n_q_heads, w.n_kv_heads, w.n_boost, w.residual_window, w.rank_metric)
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
