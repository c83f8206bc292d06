"""kitty_decode_attention_static (the entry point that allocates nothing: its split partials live in a fixed array
inside the library's device image) against kitty_decode_attention with a caller workspace, through the C ABI, on
two calls in a row, the second on a smaller batch and shorter sequences.  Same kernels, same summation order:
the outputs must be bit-identical, and both within the stated bound of the oracle."""
import ctypes as C

import numpy as np
import pytest

from paper_2511_18643_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _case(w, lengths, max_pages, n_splits, check_oracle):
    import torch
    from paper_2511_18643_amd import kitty
    k, v = H.gen_sequences(w, lengths)
    layout, gc = H.gpu_cache(w, lengths, k, v, max_pages)
    q_bits = synth.query(w)
    q = H.bf16_tensor(q_bits)
    lib = kitty.lib()
    cs = gc.struct()
    stream = torch.cuda.current_stream().cuda_stream
    need = kitty.kitty_decode_workspace_bytes(layout, w.batch, max_pages, n_splits)
    assert 0 < need <= kitty.STATIC_WORKSPACE_BYTES
    for dtype, code in ((torch.float32, 1), (torch.bfloat16, 0)):
        ref = torch.full((w.batch, w.n_q_heads, 128), float("nan"), dtype=dtype, device="cuda")
        got = torch.full_like(ref, float("nan"))
        ws = kitty.new_workspace(layout, w.batch, max_pages, n_splits)
        ws.fill_(float("nan"))
        rc = lib.kitty_decode_attention(C.byref(layout), C.byref(cs), q.data_ptr(), ref.data_ptr(), w.sm_scale, n_splits,
                                        code, ws.data_ptr(), ws.numel() * 4, stream)
        assert rc == 0
        rc = lib.kitty_decode_attention_static(C.byref(layout), C.byref(cs), q.data_ptr(), got.data_ptr(), w.sm_scale,
                                               n_splits, code, stream)
        assert rc == 0
        torch.cuda.synchronize()
        assert torch.isfinite(got.float()).all()
        assert torch.equal(got, ref), (n_splits, dtype)
        if check_oracle and dtype == torch.float32:
            oc = H.oracle_cache(w, lengths, k, v, max_pages)
            want = oc.decode_attention(q_bits, w.sm_scale)
            assert np.abs(got.cpu().numpy() - want).max() <= 3e-4


def test_static_workspace_matches_caller_workspace_two_calls_second_smaller():
    big = synth.scaled(synth.WORKLOADS["c2"], batch=4, n_q_heads=8, n_kv_heads=2, context=0)
    small = synth.scaled(synth.WORKLOADS["c2"], batch=2, n_q_heads=8, n_kv_heads=2, context=0, seed=77)
    for n_splits in (5, 0):
        # first call: 4 sequences of up to 40 pages; second call: 2 shorter ones (its partials cover only the
        # front of the array, the rest still holds the first call's)
        _case(big, [40 * 128 + 128, 17 * 128 + 3, 0, 128 + 1], 40, n_splits, check_oracle=(n_splits == 5))
        _case(small, [6 * 128 + 50, 2 * 128 + 128], 6, n_splits, check_oracle=(n_splits == 5))


def test_static_workspace_refuses_plans_beyond_its_size():
    import torch
    from paper_2511_18643_amd import kitty
    layout = kitty.make_layout(64, 8, 32)
    gc = kitty.Cache(layout, 64, 64, 1)
    n_splits = 8
    assert kitty.kitty_decode_workspace_bytes(layout, 64, 64, n_splits) > kitty.STATIC_WORKSPACE_BYTES
    q = torch.zeros((64, 64, 128), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros_like(q)
    with pytest.raises(kitty.KittyError) as e:
        kitty.kitty_decode_attention_static(layout, gc, q, out, 0.1, n_splits)
    assert e.value.code == kitty.ERR_WORKSPACE
