"""Builds the same cache twice from one seeded workload: once through the CPU oracle (here), once on the
GPU through the C-ABI binding (paper_2511_18643_amd.devcache).  The two sides share only the input bits."""
from __future__ import annotations

import numpy as np

from oracle import kitty_oracle as ko
from paper_2511_18643_amd.devcache import (VarLenPlan, bf16_tensor, gen_sequences, gpu_cache,  # noqa: F401
                                           gpu_decode, gpu_full_cache, varlen_layer_cache, varlen_sources)


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


