"""Host-side checks of the C ABI that need no GPU: the library loads, exports every declared
symbol, sizes follow the closed forms, and invalid arguments are rejected before any launch."""
import ctypes as C
import os
import re

import pytest

from paper_2511_18643_amd import kitty

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "kitty.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kitty_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = kitty.lib()
    names = declared_symbols()
    assert set(names) == set(kitty.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_record_sizes():
    for nb, want in ((0, 9344), (16, 9856), (32, 10368), (64, 11392), (128, 13440)):
        lay = kitty.make_layout(32, 8, nb)
        assert kitty.kitty_page_bytes(lay) == want
        assert kitty.kitty_page_payload_bytes(lay) == want - (128 - nb)
        assert want % 128 == 0
    assert kitty.kitty_page_payload_bytes(kitty.make_layout(32, 8, 16)) == 9744
    assert kitty.kitty_page_payload_bytes(kitty.make_layout(32, 8, 32)) == 10272


def test_unsupported_layouts_are_rejected():
    assert kitty.kitty_page_bytes(kitty.make_layout(32, 8, 16, head_dim=64)) == 0
    assert kitty.kitty_page_bytes(kitty.make_layout(32, 8, 16, page_size=64)) == 0
    assert kitty.kitty_page_bytes(kitty.make_layout(32, 8, 16, v_group=32)) == 0
    assert kitty.kitty_page_bytes(kitty.make_layout(32, 8, 24)) == 0           # not a multiple of 16
    assert kitty.kitty_page_bytes(kitty.make_layout(32, 8, 48)) == 9344 + 3 * 512   # every multiple of 16 up to D
    assert kitty.kitty_page_bytes(kitty.make_layout(32, 8, 144)) == 0          # more than D
    assert kitty.kitty_page_bytes(kitty.make_layout(32, 8, 16, residual_window=64)) == 0
    assert kitty.kitty_page_bytes(kitty.make_layout(30, 8, 16)) == 0           # heads do not divide
    assert kitty.kitty_page_bytes(kitty.make_layout(48, 8, 16)) == 9856        # any group of up to eight query heads
    assert kitty.kitty_page_bytes(kitty.make_layout(40, 8, 16)) == 9856
    assert kitty.kitty_page_bytes(kitty.make_layout(72, 8, 16)) == 0           # group of 9
    assert kitty.kitty_page_bytes(kitty.make_layout(32, 8, 16, rank_metric=2)) == 0
    # 4-bit Values: one more 4 KB plane, with any boost count
    assert kitty.kitty_page_bytes(kitty.make_layout(32, 8, 16, v_bits=4)) == 9856 + 4096
    assert kitty.kitty_page_payload_bytes(kitty.make_layout(32, 8, 0, v_bits=4)) == 9216 + 4096
    assert kitty.kitty_page_bytes(kitty.make_layout(32, 8, 16, v_bits=0)) == 9856
    assert kitty.kitty_page_bytes(kitty.make_layout(32, 8, 32, v_bits=4)) == 10368 + 4096
    assert kitty.kitty_page_bytes(kitty.make_layout(32, 8, 128, v_bits=4)) == 13440 + 4096     # 4-bit Keys and Values
    assert kitty.kitty_page_bytes(kitty.make_layout(32, 8, 16, v_bits=3)) == 0
    # Sink up to one page; the Value Local window is one page long and needs the residual window
    assert kitty.kitty_page_bytes(kitty.make_layout(32, 8, 16, sink_tokens=32, v_local=128)) == 9856
    assert kitty.kitty_page_bytes(kitty.make_layout(32, 8, 16, sink_tokens=129)) == 0
    assert kitty.kitty_page_bytes(kitty.make_layout(32, 8, 16, sink_tokens=-1)) == 0
    assert kitty.kitty_page_bytes(kitty.make_layout(32, 8, 16, v_local=64)) == 0
    assert kitty.kitty_page_bytes(kitty.make_layout(32, 8, 16, residual_window=0, v_local=128)) == 0


def test_plan_and_workspace():
    lay = kitty.make_layout(32, 8, 16)
    ns, mp = kitty.kitty_decode_plan(lay, 32, 255, 0)
    assert 1 <= ns <= 255 and mp >= 1 and ns * mp <= 255
    assert kitty.kitty_decode_workspace_bytes(lay, 32, 255, 0) == 32 * 32 * ns * 130 * 4
    for req in (1, 2, 7, 255, 1000):
        ns, mp = kitty.kitty_decode_plan(lay, 32, 255, req)
        assert ns == min(req, 255) and mp == 1
        assert kitty.kitty_decode_workspace_bytes(lay, 32, 255, req) == 32 * 32 * ns * 130 * 4
    lay0 = kitty.make_layout(1, 1, 16, residual_window=0)
    assert kitty.kitty_decode_plan(lay0, 1, 8, 4) == (4, 1)
    assert kitty.kitty_decode_workspace_bytes(lay0, 1, 8, 4) == 4 * 130 * 4
    # a cache with no page table still needs one range for the window
    assert kitty.kitty_decode_plan(lay, 4, 0, 0)[0] == 1


def test_invalid_arguments_return_codes_without_touching_a_gpu():
    lib = kitty.lib()
    lay = kitty.make_layout(32, 8, 16)
    bad = kitty.make_layout(32, 8, 16, head_dim=64)
    assert lib.kitty_quantize_pages(None, None, None, 0, 0, 128, None, None, 1, None, 1, None) == kitty.ERR_INVALID_ARG
    assert lib.kitty_quantize_pages(C.byref(bad), None, None, 0, 0, 128, None, None, 1, None, 1, None) == kitty.ERR_UNSUPPORTED
    assert lib.kitty_quantize_pages(C.byref(lay), None, None, 0, 0, 128, None, None, 1, None, 1, None) == kitty.ERR_INVALID_ARG
    assert lib.kitty_quantize_pages(C.byref(lay), None, None, 0, 0, 128, None, None, 0, None, 1, None) == kitty.KITTY_OK
    # misaligned source, stride not a multiple of 8
    assert lib.kitty_quantize_pages(C.byref(lay), 0x1008, 0x2000, 16384, 16384, 128, None, 0x3000, 1, 0x4000, 1, None) == kitty.ERR_INVALID_ARG
    assert lib.kitty_quantize_pages(C.byref(lay), 0x1000, 0x2000, 16384, 16384, 132, None, 0x3000, 1, 0x4000, 1, None) == kitty.ERR_INVALID_ARG
    cache = kitty.KittyCache(None, None, None, None, None, None, None, None, None, None, 4, 8, 32)
    assert lib.kitty_decode_attention(C.byref(lay), C.byref(cache), None, None, 1.0, 0, 0, None, 0, None) == kitty.ERR_INVALID_ARG
    assert lib.kitty_append_token(C.byref(lay), None, None, None, None, None) == kitty.ERR_INVALID_ARG
    assert lib.kitty_decode_split(C.byref(lay), C.byref(cache), None, 1.0, 0, None, 0, None) == kitty.ERR_INVALID_ARG
    # a complete-looking cache with a workspace that is too small
    cache = kitty.KittyCache(0x10000, 0x20000, 0x30000, 0x40000, 0x50000, 0x60000, None, None, None, None, 4, 8, 32)
    assert lib.kitty_decode_split(C.byref(lay), C.byref(cache), 0x70000, 1.0, 0, 0x80000, 64, None) == kitty.ERR_WORKSPACE
    assert lib.kitty_decode_merge(C.byref(lay), C.byref(cache), 0x70000, 0, 5, 0x80000, 1 << 30, None) == kitty.ERR_INVALID_ARG
    lay0 = kitty.make_layout(32, 8, 16, residual_window=0)
    cache0 = kitty.KittyCache(0x10000, 0x20000, 0x30000, None, None, None, None, None, None, None, 4, 8, 32)
    assert lib.kitty_append_token(C.byref(lay0), C.byref(cache0), 0x1000, 0x2000, 0x3000, None) == kitty.ERR_UNSUPPORTED
    # a Sink in the layout needs the Sink buffers in the cache
    lay_s = kitty.make_layout(32, 8, 16, sink_tokens=32)
    assert lib.kitty_decode_split(C.byref(lay_s), C.byref(cache), 0x70000, 1.0, 0, 0x80000, 1 << 30, None) == kitty.ERR_INVALID_ARG
    assert b"workspace" in lib.kitty_strerror(kitty.ERR_WORKSPACE)
    assert lib.kitty_strerror(12345) == b"unknown error"


def test_build_report_parser_finds_scratch_use():
    """The build refuses kernels that spill to scratch memory; this checks the parser of hipcc's
    kernel-resource-usage remarks that the check relies on."""
    from paper_2511_18643_amd import build
    text = "\n".join([
        "x.h:1:1: remark: Function Name: _ZN5kitty1aEv [-Rpass-analysis=kernel-resource-usage]",
        "x.h:1:1: remark:     VGPRs: 152 [-Rpass-analysis=kernel-resource-usage]",
        "x.h:1:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]",
        "x.h:1:1: remark:     LDS Size [bytes/block]: 74112 [-Rpass-analysis=kernel-resource-usage]",
        "x.h:9:1: remark: Function Name: _ZN5kitty1bEv [-Rpass-analysis=kernel-resource-usage]",
        "x.h:9:1: remark:     VGPRs: 256 [-Rpass-analysis=kernel-resource-usage]",
        "x.h:9:1: remark:     ScratchSize [bytes/lane]: 24 [-Rpass-analysis=kernel-resource-usage]",
    ])
    u = build.kernel_resource_usage(text)
    assert set(u) == {"_ZN5kitty1aEv", "_ZN5kitty1bEv"}
    assert u["_ZN5kitty1aEv"]["VGPRs"] == 152 and u["_ZN5kitty1aEv"]["ScratchSize [bytes/lane]"] == 0
    assert u["_ZN5kitty1aEv"]["LDS Size [bytes/block]"] == 74112
    assert u["_ZN5kitty1bEv"]["ScratchSize [bytes/lane]"] == 24
