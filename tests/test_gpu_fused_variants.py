"""GPU parity of the launch configurations that the small cases of test_gpu_parity.py reach only by chance:
the 36-layer variable-length loop's real shape (batch 128, lengths 1k-32k, longest-first dispatch, 4-wavefront
blocks with several blocks per compute unit, flushes at different steps per sequence), and kitty_decode_step for
eight-head groups, high boost counts and many ranges, each across a flush."""
import numpy as np
import pytest

from oracle import kitty_oracle as ko
from paper_2511_18643_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu

TOL_G4 = 3e-4       # fp32 output, query groups of up to four heads
TOL_G8 = 5e-4       # eight-head groups


def _pair_oracle(w, ksrc, vsrc, sb, h, first_token, n_pages, r, max_pages):
    """Oracle cache of one (sequence, kv-head) rebuilt from the source tokens."""
    g = w.gqa
    oc = ko.KittyCacheOracle(1, 1, g, w.n_boost, 128, max_pages, max_pages, w.rank_metric)
    a = first_token
    if n_pages:
        oc.quantize_pages(ksrc[sb, h, a:a + n_pages * 128].reshape(n_pages, 1, 128, 128),
                          vsrc[sb, h, a:a + n_pages * 128].reshape(n_pages, 1, 128, 128), list(range(n_pages)))
    oc.page_table[0] = np.arange(max_pages)
    oc.n_pages[0] = n_pages
    oc.n_resid[0] = r
    oc.resid_k[0, 0, :r] = ksrc[sb, h, a + n_pages * 128:a + n_pages * 128 + r]
    oc.resid_v[0, 0, :r] = vsrc[sb, h, a + n_pages * 128:a + n_pages * 128 + r]
    return oc


def test_c5_real_shape_two_layers_sampled():
    """Batch 128, seeded lengths uniform in [1024, 32768] (three of them moved so that their windows fill within
    the run), two layers, six kitty_decode_step calls per layer with the longest sequences dispatched first:
    the state of all 128 sequences in closed form, and sampled (sequence, kv-head) pairs (outputs at three steps,
    records written by the flushes, window rows) against the oracle replaying the same tokens."""
    import torch
    from paper_2511_18643_amd import kitty
    w = synth.WORKLOADS["c5"]
    B, hkv, hq, g = w.batch, w.n_kv_heads, w.n_q_heads, w.gqa
    lengths = synth.sequence_lengths(w)
    assert len(lengths) == 128 and min(lengths) >= 1024 and max(lengths) <= 32768
    order_by_len = np.argsort(lengths)
    # three sequences whose windows hold 128, 126 and 123 rows: they flush at steps 1, 3 and 6
    flushers = {int(order_by_len[40]): 128, int(order_by_len[90]): 126, int(order_by_len[120]): 123}
    for b, r in flushers.items():
        lengths[b] = (lengths[b] // 128) * 128 + r if r < 128 else (lengths[b] // 128 + 1) * 128
    n_steps, layers, nsrc = 6, 2, 2
    plan = H.VarLenPlan(lengths, n_steps)
    for b, r in flushers.items():
        assert plan.r0[b] == r
    layout = kitty.make_layout(hq, hkv, w.n_boost, 128, w.rank_metric)
    Ls = max(lengths) + 128 * layers
    ksrc, vsrc = H.varlen_sources(w, nsrc, Ls)
    kt, vt = H.bf16_tensor(ksrc), H.bf16_tensor(vsrc)
    longest, shortest = int(np.argmax(lengths)), int(np.argmin(lengths))
    fl = list(flushers)
    sample = [(longest, 0), (shortest, 7), (fl[0], 3), (fl[1], 0), (fl[2], 7), (int(order_by_len[64]), 5)]
    ns, _ = kitty.kitty_decode_plan(layout, B, plan.max_pages, 0)
    assert ns == 1                                  # 1024 (sequence, kv-head) pairs: one range each, 4 per compute unit
    ws = kitty.new_workspace(layout, B, plan.max_pages)
    base_t = torch.tensor(plan.base[:-1], dtype=torch.int32, device="cuda")
    out = torch.empty((B, hq, 128), dtype=torch.float32, device="cuda")
    for layer in range(layers):
        c = H.varlen_layer_cache(layout, w, plan, kt, vt, layer)
        c.seq_order = torch.argsort(c.n_pages * 128 + c.n_resid, descending=True).to(torch.int32)
        oracles = {(b, h): _pair_oracle(w, ksrc, vsrc, b % nsrc, h, 128 * layer, plan.np0[b], plan.r0[b], plan.max_pages)
                   for b, h in sample}
        for b, h in sample:                         # prefill records of the sampled pairs, a few pages each
            for i in sorted({0, plan.np0[b] // 2, plan.np0[b] - 1}):
                rec = c.pool[int(plan.base[b]) + i, h].cpu().numpy()
                assert np.array_equal(rec, oracles[(b, h)].pool[i, 0]), (layer, b, h, i)
        np_now, r_now = list(plan.np0), list(plan.r0)
        for step in range(1, n_steps + 1):
            kn, vn = synth.new_token(w, 100 * layer + step)
            q = synth.query(w, 100 * layer + step)
            fresh = base_t + c.n_pages
            kitty.kitty_decode_step(layout, c, H.bf16_tensor(kn), H.bf16_tensor(vn), fresh, H.bf16_tensor(q), out,
                                    w.sm_scale, ws)
            for b in range(B):
                if r_now[b] == 128:
                    np_now[b] += 1
                    r_now[b] = 0
                r_now[b] += 1
            for (b, h), oc in oracles.items():
                oc.append_token(kn[b:b + 1, h:h + 1], vn[b:b + 1, h:h + 1], np.array([oc.n_pages[0]]))
            if step in (1, 3, 6):
                torch.cuda.synchronize()
                assert c.n_pages.cpu().tolist() == np_now and c.n_resid.cpu().tolist() == r_now, (layer, step)
                got = out.cpu().numpy()
                assert np.isfinite(got).all()
                for (b, h), oc in oracles.items():
                    want = oc.decode_attention(q[b:b + 1, h * g:(h + 1) * g], w.sm_scale)[0]
                    err = float(np.abs(got[b, h * g:(h + 1) * g] - want).max())
                    assert err <= TOL_G4, (layer, step, b, h, err)
        # a window holding r rows flushes floor((r + n - 1) / 128) times during n appends: the three planned ones
        # and those of the seeded lengths that happen to end within six rows of a page
        assert sum(np_now) - sum(plan.np0) == sum((r + n_steps - 1) // 128 for r in plan.r0) >= 3
        pt = c.page_table.cpu().numpy()
        for (b, h), oc in oracles.items():
            n_p, r = int(oc.n_pages[0]), int(oc.n_resid[0])
            assert n_p == np_now[b] and r == r_now[b]
            if b in flushers:                       # the record the flush wrote, and where the table points
                assert pt[b, n_p - 1] == int(plan.base[b]) + n_p - 1
                rec = c.pool[int(pt[b, n_p - 1]), h].cpu().numpy()
                assert np.array_equal(rec, oc.pool[n_p - 1, 0]), (layer, b, h)
            gk = c.resid_k[b, h, :r].view(torch.int16).cpu().numpy().view(np.uint16)
            gv = c.resid_v[b, h, :r].view(torch.int16).cpu().numpy().view(np.uint16)
            assert np.array_equal(gk, oc.resid_k[0, 0, :r]) and np.array_equal(gv, oc.resid_v[0, 0, :r])
        del c
        torch.cuda.empty_cache()


# (query heads per kv-head, boosted channels, ranges requested, row length of the page table)
#   table of 4 pages: 4-wavefront blocks; 40 pages per range: 8-wavefront blocks; 12 ranges: the merge's loop form
FUSED_CASES = [
    (4, 32, 0, 4), (4, 64, 0, 4), (4, 128, 0, 4), (4, 32, 1, 40), (4, 64, 1, 40), (4, 128, 1, 40),
    (4, 32, 2, 80), (4, 64, 2, 4), (4, 128, 2, 80), (4, 32, 12, 24), (4, 128, 12, 24),
    (8, 0, 0, 4), (8, 16, 1, 40), (8, 32, 0, 4), (8, 32, 1, 40), (8, 32, 2, 80), (8, 32, 2, 4), (8, 32, 12, 24),
    (8, 64, 0, 4), (8, 64, 1, 40), (8, 64, 2, 80), (8, 64, 12, 24), (8, 128, 0, 4), (8, 128, 1, 40), (8, 128, 2, 80),
    (8, 128, 12, 24),
    (4, 48, 0, 4), (4, 96, 2, 80), (8, 48, 0, 4), (8, 48, 2, 80), (8, 80, 1, 40), (8, 96, 12, 24), (8, 112, 0, 4),
    (3, 16, 0, 4), (3, 16, 2, 80), (5, 16, 0, 4), (5, 32, 2, 80), (6, 32, 1, 40), (7, 64, 12, 24),
]


@pytest.mark.parametrize("g,nb,n_splits,max_pages", FUSED_CASES)
def test_decode_step_variants_across_a_flush(g, nb, n_splits, max_pages):
    """kitty_decode_step, five steps: sequences flush at steps 1, 2 and 3, one grows without a flush, one starts
    empty.  State, page table, the records the flushes wrote (bit for bit), window rows and outputs against the
    oracle's append followed by its attention."""
    import torch
    from paper_2511_18643_amd import kitty
    hkv = 2
    w = synth.scaled(synth.WORKLOADS["c4" if g > 4 else "c2"], batch=5, n_q_heads=g * hkv, n_kv_heads=hkv, n_boost=nb,
                     context=0, seed=9000 + 10 * nb + g)
    start = [(20 if max_pages >= 24 else 2) * 128 + 128, 128 + 127, 126, 3 * 128 + 5 if max_pages > 4 else 2 * 128 + 5, 0]
    k0, v0 = H.gen_sequences(w, start)
    oc = H.oracle_cache(w, start, k0, v0, max_pages)
    layout, gc = H.gpu_cache(w, start, k0, v0, max_pages)
    ns, _ = kitty.kitty_decode_plan(layout, 5, max_pages, n_splits)
    assert ns == max(n_splits, 1)
    ws = kitty.new_workspace(layout, 5, max_pages, n_splits)
    ws.fill_(float("nan"))
    out = torch.full((5, g * hkv, 128), float("nan"), dtype=torch.float32, device="cuda")
    tol = TOL_G8 if g > 4 else TOL_G4
    for step in range(1, 6):
        kn, vn = synth.new_token(w, step)
        q = synth.query(w, step)
        fresh = np.array([b * max_pages + int(oc.n_pages[b]) for b in range(5)], np.int32)
        flushed = oc.append_token(kn, vn, fresh)
        assert flushed == (1 if step <= 3 else 0)
        kitty.kitty_decode_step(layout, gc, H.bf16_tensor(kn), H.bf16_tensor(vn), torch.from_numpy(fresh).cuda(),
                                H.bf16_tensor(q), out, w.sm_scale, ws, n_splits)
        torch.cuda.synchronize()
        assert np.array_equal(gc.n_pages.cpu().numpy(), oc.n_pages), step
        assert np.array_equal(gc.n_resid.cpu().numpy(), oc.n_resid), step
        assert np.array_equal(gc.page_table.cpu().numpy()[:, :max_pages], oc.page_table), step
        gp = gc.pool.cpu().numpy()
        for b in range(5):
            for i in range(int(oc.n_pages[b])):
                pid = oc.page_table[b, i]
                assert np.array_equal(gp[pid], oc.pool[pid]), (step, b, i)
            rr = int(oc.n_resid[b])
            gk = gc.resid_k[b, :, :rr].view(torch.int16).cpu().numpy().view(np.uint16)
            gv = gc.resid_v[b, :, :rr].view(torch.int16).cpu().numpy().view(np.uint16)
            assert np.array_equal(gk, oc.resid_k[b, :, :rr]) and np.array_equal(gv, oc.resid_v[b, :, :rr]), (step, b)
        want = oc.decode_attention(q, w.sm_scale)
        got = out.cpu().numpy()
        err = float(np.abs(got - want).max())
        assert np.isfinite(got).all() and err <= tol, (step, err)


@pytest.mark.parametrize("nb", [0, 32])
@pytest.mark.parametrize("n_tokens", [129, 128 + 40, 5 * 128 + 128])
def test_eight_head_groups_with_one_dominant_query_channel(nb, n_tokens):
    """Worst case for the fixed-point image of q*scale: every query head has one element forty times the others',
    on a Key channel that is an outlier (large scale) and, with n_boost 0, not boosted; short contexts, so that
    nothing averages out.  The image's step is set by the largest |q*scale| of a head, so all other channels are
    resolved that much more coarsely.  The stated bound must hold here too."""
    w = synth.scaled(synth.WORKLOADS["c2"], batch=2, n_q_heads=16, n_kv_heads=2, n_boost=nb, context=0, seed=31337)
    lengths = [n_tokens, n_tokens]
    k, v = H.gen_sequences(w, lengths)
    mp = max(w.pages_and_resid(n_tokens)[0], 1)
    oc = H.oracle_cache(w, lengths, k, v, mp)
    layout, gc = H.gpu_cache(w, lengths, k, v, mp)
    qf = ko.bf16_bits_to_f32(synth.query(w)).copy()
    for h in range(2):
        ch = int(synth.outlier_channels(w, h)[0])
        qf[:, 8 * h:8 * (h + 1), ch] = 40.0 * np.sign(qf[:, 8 * h:8 * (h + 1), ch])
    q = ko.f32_to_bf16_bits(qf)
    want = oc.decode_attention(q, w.sm_scale)
    for ns in (0, 2):
        got = H.gpu_decode(layout, gc, q, w.sm_scale, ns, fp32=True)
        err = float(np.abs(got - want).max())
        assert err <= 2e-3, (ns, err)


@pytest.mark.parametrize("n_splits", [0, 2])
def test_decode_step_with_a_full_page_table_drops_the_token_and_attends_over_the_old_state(n_splits):
    """A flush is due but the page table has no free entry (or the fresh id lies outside the pool): that sequence is
    left unchanged, as kitty_append_token leaves it, and attention runs over its old state; the other sequence of
    the batch appends normally.  One launch (n_splits 0) and two (n_splits 2)."""
    import torch
    from paper_2511_18643_amd import kitty
    w = synth.scaled(synth.WORKLOADS["c2"], batch=3, n_q_heads=8, n_kv_heads=2, context=0)
    max_pages = 2
    start = [2 * 128 + 128, 128 + 5, 128 + 128]        # table full and window full; room left; window full, bad fresh id
    k0, v0 = H.gen_sequences(w, start)
    oc = H.oracle_cache(w, start, k0, v0, max_pages)
    layout, gc = H.gpu_cache(w, start, k0, v0, max_pages)
    before = {n: getattr(gc, n).clone() for n in ("n_pages", "n_resid", "page_table", "resid_k", "resid_v", "pool")}
    kn, vn = synth.new_token(w, 1)
    q = synth.query(w, 1)
    fresh = np.array([0, 3, 99], np.int32)             # sequence 2's id is outside the pool of 6 pages
    # the oracle's machine has no refusal: apply the append to sequence 1 only
    oc.resid_k[1, :, 5] = kn[1]; oc.resid_v[1, :, 5] = vn[1]; oc.n_resid[1] = 6
    want = oc.decode_attention(q, w.sm_scale)
    ws = kitty.new_workspace(layout, 3, max_pages, n_splits)
    out = torch.full((3, 8, 128), float("nan"), dtype=torch.float32, device="cuda")
    kitty.kitty_decode_step(layout, gc, H.bf16_tensor(kn), H.bf16_tensor(vn), torch.from_numpy(fresh).cuda(),
                            H.bf16_tensor(q), out, w.sm_scale, ws, n_splits)
    torch.cuda.synchronize()
    assert gc.n_pages.cpu().tolist() == [2, 1, 1] and gc.n_resid.cpu().tolist() == [128, 6, 128]
    assert torch.equal(gc.page_table, before["page_table"]) and torch.equal(gc.pool, before["pool"])
    for b in (0, 2):
        assert torch.equal(gc.resid_k[b], before["resid_k"][b]) and torch.equal(gc.resid_v[b], before["resid_v"][b])
    got = out.cpu().numpy()
    assert np.isfinite(got).all() and float(np.abs(got - want).max()) <= TOL_G4
