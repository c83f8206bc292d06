"""GPU parity of the paper's full cache organisation (Fig. 1, Sec. 4.3): Sink tokens in full precision, and the
Value Local window that keeps the Values of the newest page in full precision one page longer than its Keys.
The oracle side is the buffer-by-buffer state machine (KittyUnitOracle); the GPU side goes through the C ABI."""
import os

import numpy as np
import pytest

from oracle import kitty_oracle as ko
from paper_2511_18643_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu

TOL_FP32 = 3e-4


def small(batch=3, hq=8, hkv=2, nb=16, **kw):
    return synth.scaled(synth.WORKLOADS["c2"], batch=batch, n_q_heads=hq, n_kv_heads=hkv, n_boost=nb, context=0, **kw)


@pytest.mark.parametrize("sink,v_local,hq,nb,n_splits", [
    (32, 128, 8, 16, 0), (32, 0, 8, 16, 0), (0, 128, 8, 16, 0), (32, 128, 16, 32, 0), (32, 128, 2, 0, 0),
    (32, 128, 8, 16, 3), (128, 128, 8, 16, 2), (5, 128, 4, 16, 1)])
def test_prefilled_cache_matches_unit_oracle(sink, v_local, hq, nb, n_splits):
    """Lengths cover: empty, inside the Sink, Sink exactly full, first window token, window full, one page + 1
    (the first step with a page whose Values are still in the Local window), several pages."""
    lengths = [0, 3, sink, sink + 1, sink + 128, sink + 129, sink + 2 * 128 + 77, sink + 9 * 128, sink + 40 * 128 + 1]
    w = small(batch=len(lengths), hq=hq, nb=nb)
    k, v = H.gen_sequences(w, lengths)
    max_pages = 48
    units = H.unit_oracles(w, lengths, k, v, sink, v_local)
    layout, gc = H.gpu_full_cache(w, lengths, k, v, max_pages, sink, v_local)
    q = synth.query(w)
    want = H.units_attention(w, units, q, w.sm_scale)
    got = H.gpu_decode(layout, gc, q, w.sm_scale, n_splits, fp32=True)
    assert np.isfinite(got).all()
    err = np.abs(got - want).max(axis=(1, 2))
    assert err.max() <= (TOL_FP32 if w.gqa <= 4 else 1e-3), err
    got16 = H.gpu_decode(layout, gc, q, w.sm_scale, n_splits, fp32=False)
    assert np.array_equal(got16, ko.bf16_bits_to_f32(ko.f32_to_bf16_bits(got)))


def test_sink_without_window():
    """Static cache (R = 0) with a Sink: Sink rows + whole pages."""
    w = small(batch=3, residual_window=0)
    lengths = [32, 32 + 128, 32 + 6 * 128]
    k, v = H.gen_sequences(w, lengths)
    units = H.unit_oracles(w, lengths, k, v, 32, 0)
    layout, gc = H.gpu_full_cache(w, lengths, k, v, 8, 32, 0)
    q = synth.query(w)
    got = H.gpu_decode(layout, gc, q, w.sm_scale, 0, fp32=True)
    err = float(np.abs(got - H.units_attention(w, units, q, w.sm_scale)).max())
    assert err <= TOL_FP32


@pytest.mark.parametrize("fused,max_pages,n_splits,VL", [(False, 4, 0, 128), (True, 4, 0, 128), (True, 40, 1, 128), (True, 4, 2, 128),
                                                         (True, 40, 1, 0), (False, 40, 1, 0)])
def test_decode_loop_from_empty_matches_unit_oracle(fused, max_pages, n_splits, VL):
    """Token-by-token decode from an empty cache through the Sink, the first pages and the Local window,
    either as kitty_append_token + kitty_decode_attention or as the single kitty_decode_step call.  Sequences
    start at different lengths so that Sink fill, flushes and the first Value-lagging page fall on different
    steps.  State, flushed records (bit-exact) and outputs are checked against the unit oracles.  VL = 0: Sink and
    the single window only (with 40 pages per sequence: the 8-wavefront blocks with a row wavefront)."""
    import torch
    from paper_2511_18643_amd import kitty
    S = 32
    w = small(batch=4)
    start = [0, 31, 32 + 127, 32 + 128 + 120]
    k0, v0 = H.gen_sequences(w, start)
    units = H.unit_oracles(w, start, k0, v0, S, VL)
    layout, gc = H.gpu_full_cache(w, start, k0, v0, max_pages, S, VL)
    ws = kitty.new_workspace(layout, 4, max_pages, n_splits)
    out = torch.empty((4, 8, 128), dtype=torch.float32, device="cuda")
    n_steps = 150
    for step in range(1, n_steps + 1):
        kn, vn = synth.new_token(w, step)
        q = synth.query(w, step)
        # the oracle's pipeline: insert, attention, then quantize-if-full
        # (the library flushes a full window at the next append; the oracle's step (3) is therefore run at the
        # top of the next iteration, so both sides name the same next page)
        fresh = np.array([b * max_pages + len(units[(b, 0)].k_pages) for b in range(4)], np.int32)
        for (b, h), u in units.items():
            u.quantize_if_full()           # step (3) of the previous step
            u.insert(kn[b, h], vn[b, h])
        args = (H.bf16_tensor(kn), H.bf16_tensor(vn), torch.from_numpy(fresh).cuda())
        if fused:
            kitty.kitty_decode_step(layout, gc, *args, H.bf16_tensor(q), out, w.sm_scale, ws, n_splits)
        else:
            kitty.kitty_append_token(layout, gc, *args)
            kitty.kitty_decode_attention(layout, gc, H.bf16_tensor(q), out, w.sm_scale, ws, n_splits)
        if step in (1, 2, 32, 33, 34) or step % 16 == 0 or step >= n_steps - 2:
            torch.cuda.synchronize()
            want = H.units_attention(w, units, q, w.sm_scale)
            got = out.cpu().numpy()
            err = float(np.abs(got - want).max())
            assert err <= TOL_FP32, step
            # state: Sink rows, pages formed so far (the GPU flushes at the next append: one behind after a
            # step that filled the window), window rows
            ns_g, np_g, nr_g = (x.cpu().numpy() for x in (gc.n_sink, gc.n_pages, gc.n_resid))
            for b in range(4):
                u = units[(b, 0)]
                assert ns_g[b] == len(u.sink_k), (step, b)
                assert (np_g[b], nr_g[b]) == (len(u.k_pages), len(u.k_qbuf)), (step, b)
    torch.cuda.synchronize()
    # every page the GPU has formed is bit-identical to the oracle's quantizer on the same tokens, Keys and Values
    pool = gc.pool.cpu().numpy()
    pt = gc.page_table.cpu().numpy()
    checked = 0
    for b in range(4):
        total = start[b] + n_steps
        kall = np.concatenate([k0[b, :, :start[b]], np.stack([synth.new_token(w, s)[0][b] for s in range(1, n_steps + 1)], axis=1)], axis=1)
        vall = np.concatenate([v0[b, :, :start[b]], np.stack([synth.new_token(w, s)[1][b] for s in range(1, n_steps + 1)], axis=1)], axis=1)
        for i in range(int(gc.n_pages[b])):
            for h in range(2):
                kp = ko.quantize_k_page(ko.bf16_bits_to_f32(kall[h, S + 128 * i:S + 128 * (i + 1)]), w.n_boost, w.rank_metric)
                vp = ko.quantize_v_page(ko.bf16_bits_to_f32(vall[h, S + 128 * i:S + 128 * (i + 1)]))
                assert np.array_equal(pool[pt[b, i], h], ko.pack_record(kp, vp)), (b, i, h)
                checked += 1
        assert int(gc.n_pages[b]) == max((total - S + 127) // 128 - 1, 0)
    assert checked >= 8


def test_c3_shape_full_scheme_sampled():
    """The 32k-context workload at full size with the Sink and the Value Local window switched on, in the
    launch configuration the benchmark uses (cache tiled from two source sequences); sampled (sequence,
    kv-head) pairs are rebuilt by the unit oracle from the inputs."""
    import torch
    from paper_2511_18643_amd import kitty
    S, VL, n_src = 32, 128, 2
    w = synth.WORKLOADS["c3"]
    B, hkv, g = w.batch, w.n_kv_heads, w.gqa
    L = w.context
    post = L - S
    n_pages = (post + 127) // 128 - 1
    r = post - n_pages * 128
    sample = [(0, 0), (1, 7), (18, 2), (31, 4)]
    ksrc = np.zeros((n_src, hkv, L, 128), np.uint16)
    vsrc = np.zeros_like(ksrc)
    for sb, h in sorted({(b % n_src, h) for b, h in sample}):
        ksrc[sb, h], vsrc[sb, h] = synth.kv_block(w, sb, h, L)
    kt, vt = H.bf16_tensor(ksrc), H.bf16_tensor(vsrc)
    layout = kitty.make_layout(w.n_q_heads, hkv, w.n_boost, w.residual_window, w.rank_metric, sink_tokens=S, v_local=VL)
    cache = kitty.Cache(layout, B, n_pages, B * n_pages)
    offs = torch.tensor([(b % n_src) * hkv * L * 128 + (S + i * 128) * 128 for b in range(B) for i in range(n_pages)],
                        dtype=torch.int64, device="cuda")
    ids = torch.arange(B * n_pages, dtype=torch.int32, device="cuda")
    kitty.kitty_quantize_pages(layout, kt, vt, 128 * 128, L * 128, 128, ids, B * n_pages, cache.pool,
                               cache.n_pool_pages, src_page_offsets=offs)
    cache.page_table.copy_(ids.view(B, n_pages))
    cache.n_pages.fill_(n_pages)
    t0 = S + n_pages * 128
    for b in range(B):
        sb = b % n_src
        cache.sink_k[b] = kt[sb, :, :S]
        cache.sink_v[b] = vt[sb, :, :S]
        cache.resid_k[b, :, :r] = kt[sb, :, t0:]
        cache.resid_v[b, :, n_pages & 1, :r] = vt[sb, :, t0:]
        cache.resid_v[b, :, (n_pages - 1) & 1] = vt[sb, :, t0 - 128:t0]
    cache.n_sink.fill_(S)
    cache.n_resid.fill_(r)
    q = synth.query(w)
    ws = kitty.new_workspace(layout, B, n_pages)
    out = torch.empty((B, w.n_q_heads, 128), dtype=torch.float32, device="cuda")
    kitty.kitty_decode_attention(layout, cache, H.bf16_tensor(q), out, w.sm_scale, ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.isfinite(got).all()
    worst = 0.0
    for b, h in sample:
        sb = b % n_src
        u = ko.KittyUnitOracle(w.n_boost, sink=S, local=VL, rank_metric=w.rank_metric)
        u.prefill(ksrc[sb, h, :L - 1], vsrc[sb, h, :L - 1])
        u.insert(ksrc[sb, h, L - 1], vsrc[sb, h, L - 1])
        assert (len(u.k_pages), len(u.k_qbuf), len(u.v_pages)) == (n_pages, r, n_pages - 1)
        want = u.attention(q[b, h * g:(h + 1) * g], w.sm_scale)
        worst = max(worst, float(np.abs(got[b, h * g:(h + 1) * g] - want).max()))
    assert worst <= TOL_FP32, worst


def test_randomized_configurations():
    """Seeded random draws over the layout knobs (heads, GQA group, boost count, Value bits, Sink size, Local
    window, ranking metric), batch shapes (ragged lengths incl. empty), split plans and dispatch orders; each
    cache is prefilled, then advanced by three decode steps (alternating the one-call and two-call paths), and
    every output is compared with the unit oracles."""
    import torch
    from paper_2511_18643_amd import kitty
    # KITTY_RANDOM_SEED / KITTY_RANDOM_DRAWS widen the search by hand; the defaults are what the suite runs
    rng = np.random.default_rng(int(os.environ.get("KITTY_RANDOM_SEED", "20251127")))
    for trial in range(int(os.environ.get("KITTY_RANDOM_DRAWS", "14"))):
        hkv = int(rng.choice([1, 2, 4]))
        g = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8]))
        v_bits = int(rng.choice([2, 2, 4]))
        nb = int(rng.choice([0, 16, 32, 48, 64, 80, 96, 112, 128]))
        sink = int(rng.choice([0, 0, 7, 32, 128]))
        v_local = int(rng.choice([0, 128]))
        metric = int(rng.choice([0, 1]))
        B = int(rng.integers(1, 5))
        n_splits = int(rng.choice([0, 0, 1, 2, 5]))
        max_pages = int(rng.choice([6, 40]))
        w = synth.scaled(synth.WORKLOADS["c2"], batch=B, n_q_heads=hkv * g, n_kv_heads=hkv, n_boost=nb, context=0,
                         rank_metric=metric, seed=9000 + trial)
        top = (max_pages - 1) * 128
        lengths = [int(x) for x in rng.integers(0, min(top, 20 * 128) + sink, size=B)]
        if trial % 3 == 0:
            lengths[0] = 0
        k, v = H.gen_sequences(w, lengths)
        units = H.unit_oracles(w, lengths, k, v, sink, v_local, v_bits)
        layout, gc = H.gpu_full_cache(w, lengths, k, v, max_pages, sink, v_local, v_bits=v_bits)
        if trial % 2:
            gc.seq_order = torch.from_numpy(rng.permutation(B).astype(np.int32)).cuda()
        # short, peaky sequences are the worst case of the fixed-point images: up to 3.2e-4 with the 20-bit images
        # (measured over all variants); eight-head groups with 4-bit Values keep a two-term image of p*scale (up to
        # 1.4e-3); the stated bar is 2e-3
        tol = 1.6e-3 if (g > 4 and v_bits == 4) else 5e-4
        tag = dict(trial=trial, hkv=hkv, g=g, v_bits=v_bits, nb=nb, sink=sink, v_local=v_local, metric=metric, B=B,
                   n_splits=n_splits, max_pages=max_pages, lengths=lengths)
        q = synth.query(w)
        got = H.gpu_decode(layout, gc, q, w.sm_scale, n_splits, fp32=True)
        err = float(np.abs(got - H.units_attention(w, units, q, w.sm_scale)).max())
        assert np.isfinite(got).all(), tag
        assert err <= tol, (err, str(tag))
        ws = kitty.new_workspace(layout, B, max_pages, n_splits)
        out = torch.empty((B, hkv * g, 128), dtype=torch.float32, device="cuda")
        for step in range(1, 4):
            kn, vn = synth.new_token(w, step)
            q = synth.query(w, step)
            # both sides turn a full window into a page at the start of the next step, so the page about to be
            # written is the one after those the unit holds now
            fresh = np.array([b * max_pages + len(units[(b, 0)].k_pages) for b in range(B)], np.int32)
            for (b, h), u in units.items():
                u.quantize_if_full()
                u.insert(kn[b, h], vn[b, h])
            args = (H.bf16_tensor(kn), H.bf16_tensor(vn), torch.from_numpy(fresh).cuda())
            if (trial + step) % 2:
                kitty.kitty_decode_step(layout, gc, *args, H.bf16_tensor(q), out, w.sm_scale, ws, n_splits)
            else:
                kitty.kitty_append_token(layout, gc, *args)
                kitty.kitty_decode_attention(layout, gc, H.bf16_tensor(q), out, w.sm_scale, ws, n_splits)
            torch.cuda.synchronize()
            got = out.cpu().numpy()
            err = float(np.abs(got - H.units_attention(w, units, q, w.sm_scale)).max())
            assert np.isfinite(got).all(), (step, tag)
            assert err <= tol, (err, step, str(tag))
