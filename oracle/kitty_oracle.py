"""CPU oracle for the Kitty page quantizer and decode attention.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain reference the HIP path is
checked against.  Only tests, the smoke check and the benchmark's cpu_baseline leg may
import it; the product path never does.  It shares no code with the HIP library or its
Python binding and imports nothing but numpy.

What it follows (arXiv 2511.18643):
  * Sec. 2.1            per-channel asymmetric Key quantization, per-token Value quantization
  * Sec. 3.2, Eq. (2)   magnitude score  s_i = (1/T) sum_t |x_{i,t}|  and top-K channel boost
  * Sec. 4.1            page = one quantization group of G tokens; dense 2-bit tensor holding
                        every channel's low two bits, compact 2-bit tensor holding the high
                        two bits of the boosted channels only, channel -> slot index map with
                        a sentinel for non-boosted channels
  * Sec. 4.2, Alg. 1    X = X_low | (X_high << 2);  K = X * scale + zero_point
  * Sec. 3.2, Eq. (1)   attention = softmax(Q K^T / sqrt(d)) (then times V)
  * Sec. 4.3            insert new token -> attention -> quantize+pack when the buffer of G
                        full-precision tokens is full (at most once every G steps); `project_bf16` is the
                        plain linear projection that produces the tokens at prefill
  * Fig. 1, Sec. 3.1,   the full scheme (`KittyUnitOracle`): Sink of S initial tokens kept in full
    Sec. 4.3 step (1)   precision for K and V; Key Q-Buffer; Value Local window of the R newest tokens
                        whose evicted token enters the Value Q-Buffer, so Value pages form R tokens
                        later than Key pages

Readings taken where the paper is silent (each is listed in the design notes too):
  * quantizer formula: asymmetric min/max, scale = fp16((mx-mn)/qmax), zero = fp16(mn),
    code = clamp(rint((x - zero) * inv), 0, qmax) with inv = fp32(1/scale) taken once per
    channel (token), all in IEEE fp32 against the *stored* fp16 values, round-half-even;
    a zero scale gives code 0.
  * ranking: score descending, channel index ascending; boosted channels take slots in
    ascending channel order.  rank_metric 0 = sum_t |x| (Eq. 2 without the rank-irrelevant
    1/T, accumulated in fp64, which is exact under the condition `assert_exact_abs_sum` checks),
    rank_metric 1 = fp32(mx - mn).
  * token set of Eq. (2) = the G tokens of the page being quantized.
  * byte image of a page record: see `RecordLayout` (the layout is this build's own; the
    paper's logical tensors are recovered from it by `to_paper_tensors`).
  * attention runs on the dequantized fp32 values without re-rounding them to 16 bits,
    products in fp64, softmax with max subtraction in fp64.

Nothing here is "parity unpinned" except the end-task accuracy of the method itself, which
needs model weights and datasets and is not reproduced.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

HEAD_DIM = 128      # D, the only head size the paper's models use (Sec. 4.1 footnote: "size per head is 128")
PAGE_SIZE = 128     # G, default group size = page size (Fig. 1 caption, Sec. 4.1)


# --------------------------------------------------------------------------------------
# 16-bit float helpers (inputs and outputs are bf16; metadata is fp16)
# --------------------------------------------------------------------------------------
def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to float32 exactly."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even), return the bit patterns (uint16)."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    r = (u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)
    out = r.astype(np.uint16)
    nan = np.isnan(np.asarray(x, dtype=np.float32))
    if np.any(nan):
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


# --------------------------------------------------------------------------------------
# Quantizer (Sec. 2.1, Sec. 3.2, Sec. 4.1)
# --------------------------------------------------------------------------------------
@dataclass
class KPage:
    codes: np.ndarray      # uint8 [G][D], 0..15 on boosted channels, 0..3 elsewhere
    scale: np.ndarray      # float16 [D]
    zero: np.ndarray       # float16 [D]
    ch: np.ndarray         # uint8 [n_boost], boosted channels, ascending
    score: np.ndarray      # float64 [D], the ranking score that was used

    @property
    def lo(self) -> np.ndarray:     # low two bits of every channel (Sec. 4.1, dense tensor)
        return self.codes & np.uint8(3)

    @property
    def hi(self) -> np.ndarray:     # high two bits (zero on non-boosted channels)
        return self.codes >> np.uint8(2)


@dataclass
class VPage:
    codes: np.ndarray      # uint8 [G][D], 0..3 (0..15 for the 4-bit Value variant)
    scale: np.ndarray      # float16 [G]
    zero: np.ndarray       # float16 [G]
    bits: int = 2          # 2 (the method) or 4 (the K2V4 point of the design-space study, Table 2)


def _asym_quant(x: np.ndarray, mn: np.ndarray, mx: np.ndarray, qmax: np.ndarray):
    """Asymmetric min/max quantization of x against per-row/column (mn, mx, qmax).

    mn/mx/qmax broadcast against x.  Returns (codes uint8, scale fp16, zero fp16) where scale
    and zero have the broadcast shape of mn.  All arithmetic is IEEE fp32.
    """
    x = x.astype(np.float32)
    rng = (mx.astype(np.float32) - mn.astype(np.float32)).astype(np.float32)
    scale_h = (rng / qmax.astype(np.float32)).astype(np.float32).astype(np.float16)
    zero_h = mn.astype(np.float32).astype(np.float16)
    s = scale_h.astype(np.float32)
    z = zero_h.astype(np.float32)
    with np.errstate(divide="ignore", invalid="ignore"):
        inv = np.where(s > 0, (np.float32(1.0) / s).astype(np.float32), np.float32(0.0)).astype(np.float32)
    r = np.rint(((x - z).astype(np.float32) * inv).astype(np.float32))
    r = np.minimum(np.maximum(r, np.float32(0.0)), qmax.astype(np.float32))
    return r.astype(np.uint8), scale_h, zero_h


def assert_exact_abs_sum(x: np.ndarray) -> None:
    """The fp64 sum of a channel's |x| must be exact, so that it does not depend on the order of the additions
    (any reduction tree then gives the same ranking).  bf16 values carry 8 significant bits; the sum of up to
    2^7 of them whose nonzero magnitudes lie within 38 binades of each other needs at most 38 + 8 + 7 = 53 bits,
    which is what fp64 holds.  Pages outside that condition are outside what this oracle defines."""
    a = np.abs(np.asarray(x, dtype=np.float64))
    if a.shape[0] > 128:
        raise ValueError("exactness of the channel score is only shown for up to 128 tokens per page")
    _, e = np.frexp(a)
    big = np.where(a > 0, e, np.iinfo(np.int32).min).max(axis=0)
    small = np.where(a > 0, e, np.iinfo(np.int32).max).min(axis=0)
    span = np.where(big >= small, big.astype(np.int64) - small.astype(np.int64), 0)
    if np.any(span > 38):
        raise ValueError("a channel's nonzero magnitudes span more than 38 binades: its fp64 sum of |x| "
                         "is not guaranteed exact")


def channel_scores(x: np.ndarray, rank_metric: int) -> np.ndarray:
    """Importance score of each channel of a page x[G][D] (Eq. 2; or the range variant)."""
    if rank_metric == 0:
        assert_exact_abs_sum(x)
        return np.abs(x.astype(np.float64)).sum(axis=0)          # sum_t |x|, fp64
    if rank_metric == 1:
        mn = x.min(axis=0).astype(np.float32)
        mx = x.max(axis=0).astype(np.float32)
        return (mx - mn).astype(np.float32).astype(np.float64)
    raise ValueError("rank_metric must be 0 or 1")


def select_boost_channels(score: np.ndarray, n_boost: int) -> np.ndarray:
    """Top-n_boost channels under (score descending, index ascending); returned ascending."""
    d = score.shape[0]
    rank = np.zeros(d, dtype=np.int64)
    for c in range(d):       # rank = number of channels that come strictly before c
        rank[c] = int(np.sum((score > score[c]) | ((score == score[c]) & (np.arange(d) < c))))
    return np.nonzero(rank < n_boost)[0].astype(np.uint8)


def quantize_k_page(x: np.ndarray, n_boost: int, rank_metric: int = 0) -> KPage:
    """Quantize one Key page x[G][D] (float32 holding bf16 values).

    Per channel (Sec. 2.1): min/max over the G tokens; the n_boost highest-scoring channels
    (Sec. 3.2) get 4-bit codes (qmax 15), the rest 2-bit codes (qmax 3).
    """
    x = np.asarray(x, dtype=np.float32)
    g, d = x.shape
    score = channel_scores(x, rank_metric)
    ch = select_boost_channels(score, n_boost)
    qmax = np.full(d, 3.0, dtype=np.float32)
    qmax[ch.astype(np.int64)] = 15.0
    mn = x.min(axis=0)
    mx = x.max(axis=0)
    codes, scale_h, zero_h = _asym_quant(x, mn[None, :], mx[None, :], qmax[None, :])
    return KPage(codes=codes, scale=scale_h[0], zero=zero_h[0], ch=ch, score=score)


def quantize_v_page(x: np.ndarray, bits: int = 2) -> VPage:
    """Quantize one Value page x[G][D]: per token, `bits`-bit, group = the whole head (Sec. 2.1)."""
    assert bits in (2, 4)
    x = np.asarray(x, dtype=np.float32)
    mn = x.min(axis=1)
    mx = x.max(axis=1)
    qmax = np.full((x.shape[0], 1), float(2 ** bits - 1), dtype=np.float32)
    codes, scale_h, zero_h = _asym_quant(x, mn[:, None], mx[:, None], qmax)
    return VPage(codes=codes, scale=scale_h[:, 0], zero=zero_h[:, 0], bits=bits)


def project_bf16(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    """Linear projection of tokens x[T][H] with a weight w[C][H] (one output channel per row, the layout of a linear
    layer), as the producer of the Keys or Values that a page is quantized from (Sec. 4.3: tokens are quantized as
    the engine produces them): y[t][c] = sum_j x[t][j] * w[c][j] in fp64, rounded once to fp32 and once more to bf16
    (nearest even).  Returns bf16 bit patterns (uint16) [T][C].  Inputs are float arrays holding bf16 values."""
    y = np.asarray(x, dtype=np.float64) @ np.asarray(w, dtype=np.float64).T
    return f32_to_bf16_bits(y.astype(np.float32))


def dequant_k(kp: KPage) -> np.ndarray:
    """Alg. 1, last two lines: K = (lo | hi << 2) * scale + zero, in fp32."""
    x = (kp.lo | (kp.hi << np.uint8(2))).astype(np.float32)
    return (x * kp.scale.astype(np.float32)[None, :]).astype(np.float32) + kp.zero.astype(np.float32)[None, :]


def dequant_v(vp: VPage) -> np.ndarray:
    x = vp.codes.astype(np.float32)
    return (x * vp.scale.astype(np.float32)[:, None]).astype(np.float32) + vp.zero.astype(np.float32)[:, None]


# --------------------------------------------------------------------------------------
# Byte image of one (page, kv-head) record
# --------------------------------------------------------------------------------------
class RecordLayout:
    """Formulas for the packed record (D = G = 128).

    All code planes are little-endian 32-bit words of sixteen 2-bit elements; element a of a
    word sits at bit 8*(a % 4) + 2*(a // 4).  Words are placed so that lane l of a 64-wide
    wavefront, reading 16 (or 8) consecutive bytes at l*16 (l*8), receives exactly the words
    of one column of a 16x16x64 matrix-core tile; the formulas below are the definition.

      K dense  (low 2 bits of every channel), word (t, cb) = channels 16cb..16cb+15 of token t
               at  1024*(t//32) + 16*((t%16) + 16*(cb%4)) + 4*(2*((t//16)%2) + cb//4)
      K boost  (high 2 bits of boosted channels), word (t, s) = slots 16s..16s+15 of token t
               with T = t//16, j = t%16: n_boost = 16 at  kb_off + 8*(16*(T%4) + j) + 4*(T//4), otherwise
               at  kb_off + 512*s + 16*(16*(T//4) + j) + 4*(T%4)  (pieces of 2 or 4 words: the words a lane of
               the decode kernel reads together)
      k_scale, k_zero   fp16[128], channel order
      ch       uint8[n_boost] ascending boosted channels, zero-padded to 128 bytes
      V codes, word (d, wv) = positions 16wv..16wv+15 of channel d, where the token at
               position p is 16*(p%8) + p//8
               at  vd_off + 1024*(d//32) + 16*((d%16) + 16*(wv%4)) + 4*(2*((d//16)%2) + wv//4)
      V high   (4-bit Value variant only) the high 2 bits, same word placement, 4096 bytes further
      v_scale, v_zero   fp16[128], position order (entry p belongs to token 16*(p%8) + p//8)
    """

    def __init__(self, n_boost: int, v_bits: int = 2):
        if n_boost % 16 or not (0 <= n_boost <= HEAD_DIM):
            raise ValueError("n_boost must be a multiple of 16 in [0, 128]")
        if v_bits not in (2, 4):
            raise ValueError("v_bits must be 2 or 4")
        self.n_boost = n_boost
        self.v_bits = v_bits
        nb16 = n_boost // 16
        self.kd_off = 0
        self.kb_off = 4096
        self.ks_off = self.kb_off + 512 * nb16
        self.kz_off = self.ks_off + 256
        self.ch_off = self.kz_off + 256
        self.vd_off = self.ch_off + 128
        self.vh_off = self.vd_off + 4096                      # only present with 4-bit Values
        self.vs_off = self.vh_off + (4096 if v_bits == 4 else 0)
        self.vz_off = self.vs_off + 256
        self.record_bytes = self.vz_off + 256
        # bytes the method has to move per page (padding of the channel list excluded)
        self.payload_bytes = self.record_bytes - (128 - n_boost)

    @staticmethod
    def elem_shift(a):
        return 8 * (a % 4) + 2 * (a // 4)

    @staticmethod
    def kd_word_off(t, cb):
        return 1024 * (t // 32) + 16 * ((t % 16) + 16 * (cb % 4)) + 4 * (2 * ((t // 16) % 2) + cb // 4)

    def kb_word_off(self, t, s):
        T, j = t // 16, t % 16
        if self.n_boost == 16:
            return self.kb_off + 512 * s + 8 * (16 * (T % 4) + j) + 4 * (T // 4)      # (s is 0: one slot block)
        return self.kb_off + 512 * s + 16 * (16 * (T // 4) + j) + 4 * (T % 4)

    def vd_word_off(self, d, wv):
        return self.vd_off + 1024 * (d // 32) + 16 * ((d % 16) + 16 * (wv % 4)) + 4 * (2 * ((d // 16) % 2) + wv // 4)

    @staticmethod
    def v_token_at(p):
        return 16 * (p % 8) + p // 8

    @staticmethod
    def v_pos_of(t):
        return 8 * (t % 16) + t // 16


def _put_words(buf32: np.ndarray, byte_off: np.ndarray, elems: np.ndarray) -> None:
    """elems[..., 16] (values 0..3) -> one word each, stored at byte_off[...] (multiple of 4)."""
    a = np.arange(16)
    sh = RecordLayout.elem_shift(a).astype(np.uint32)
    w = (elems.astype(np.uint32) << sh).sum(axis=-1, dtype=np.uint64).astype(np.uint32)
    buf32[(byte_off // 4).ravel()] = w.ravel()


def _get_words(buf32: np.ndarray, byte_off: np.ndarray) -> np.ndarray:
    a = np.arange(16)
    sh = RecordLayout.elem_shift(a).astype(np.uint32)
    w = buf32[(byte_off // 4)]
    return ((w[..., None] >> sh) & np.uint32(3)).astype(np.uint8)


def pack_record(kp: KPage, vp: VPage) -> np.ndarray:
    """Byte image (uint8[record_bytes]) of one page of one kv-head."""
    lay = RecordLayout(len(kp.ch), vp.bits)
    g, d = kp.codes.shape
    assert g == PAGE_SIZE and d == HEAD_DIM
    rec = np.zeros(lay.record_bytes, dtype=np.uint8)
    r32 = rec.view(np.uint32)
    t = np.arange(g)
    # K dense: low bits of every channel
    cb = np.arange(d // 16)
    off = lay.kd_word_off(t[:, None], cb[None, :])
    _put_words(r32, off, kp.lo.reshape(g, d // 16, 16))
    # K boost: high bits of boosted channels, in slot order
    nb16 = lay.n_boost // 16
    if nb16:
        hi_slots = kp.hi[:, kp.ch.astype(np.int64)]                 # [G][n_boost]
        s = np.arange(nb16)
        off = lay.kb_word_off(t[:, None], s[None, :])
        _put_words(r32, off, hi_slots.reshape(g, nb16, 16))
    rec[lay.ks_off:lay.ks_off + 256] = kp.scale.astype(np.float16).view(np.uint8)
    rec[lay.kz_off:lay.kz_off + 256] = kp.zero.astype(np.float16).view(np.uint8)
    rec[lay.ch_off:lay.ch_off + lay.n_boost] = kp.ch
    # V codes: per channel, tokens in position order
    p = np.arange(g)
    tok_at = lay.v_token_at(p)
    vt = vp.codes[tok_at, :].T                                       # [D][position]
    dd = np.arange(d)
    wv = np.arange(g // 16)
    off = lay.vd_word_off(dd[:, None], wv[None, :])
    _put_words(r32, off, (vt & np.uint8(3)).reshape(d, g // 16, 16))
    if vp.bits == 4:
        _put_words(r32, off + (lay.vh_off - lay.vd_off), (vt >> np.uint8(2)).reshape(d, g // 16, 16))
    rec[lay.vs_off:lay.vs_off + 256] = vp.scale[tok_at].astype(np.float16).view(np.uint8)
    rec[lay.vz_off:lay.vz_off + 256] = vp.zero[tok_at].astype(np.float16).view(np.uint8)
    return rec


def unpack_record(rec: np.ndarray, n_boost: int, v_bits: int = 2):
    """Inverse of pack_record: (KPage, VPage) with score left empty."""
    lay = RecordLayout(n_boost, v_bits)
    rec = np.ascontiguousarray(np.asarray(rec, dtype=np.uint8))
    assert rec.shape[0] == lay.record_bytes
    r32 = rec.view(np.uint32)
    g, d = PAGE_SIZE, HEAD_DIM
    t = np.arange(g)
    cb = np.arange(d // 16)
    lo = _get_words(r32, lay.kd_word_off(t[:, None], cb[None, :])).reshape(g, d)
    ch = rec[lay.ch_off:lay.ch_off + n_boost].copy()
    hi = np.zeros((g, d), dtype=np.uint8)
    nb16 = n_boost // 16
    if nb16:
        s = np.arange(nb16)
        hi_slots = _get_words(r32, lay.kb_word_off(t[:, None], s[None, :])).reshape(g, n_boost)
        hi[:, ch.astype(np.int64)] = hi_slots
    k_scale = rec[lay.ks_off:lay.ks_off + 256].view(np.float16).copy()
    k_zero = rec[lay.kz_off:lay.kz_off + 256].view(np.float16).copy()
    kp = KPage(codes=lo | (hi << np.uint8(2)), scale=k_scale, zero=k_zero, ch=ch, score=np.zeros(0))
    dd = np.arange(d)
    wv = np.arange(g // 16)
    vt = _get_words(r32, lay.vd_word_off(dd[:, None], wv[None, :])).reshape(d, g)   # [D][position]
    if v_bits == 4:
        vt = vt | (_get_words(r32, lay.vd_word_off(dd[:, None], wv[None, :]) + (lay.vh_off - lay.vd_off)).reshape(d, g) << np.uint8(2))
    pos_of = lay.v_pos_of(t)
    v_codes = vt[:, pos_of].T
    vs = rec[lay.vs_off:lay.vs_off + 256].view(np.float16)[pos_of].copy()
    vz = rec[lay.vz_off:lay.vz_off + 256].view(np.float16)[pos_of].copy()
    return kp, VPage(codes=v_codes, scale=vs, zero=vz, bits=v_bits)


def to_paper_tensors(rec: np.ndarray, n_boost: int):
    """The paper's logical page tensors (Sec. 4.1, Alg. 1) recovered from a record.

    Returns (tensor_2bits uint8[D][G/4], tensor_high_2bits uint8[n_boost][G/4],
    boost_idx uint8[D]).  Bytes hold four consecutive tokens, token j at bit 2*(j mod 4)
    (the shifts [0,2,4,6,...] of Alg. 1).  boost_idx maps channel -> slot, 0-based, with the
    sentinel n_boost for non-boosted channels (the paper counts from 1 and uses D_boost+1).
    """
    kp, _ = unpack_record(rec, n_boost)
    g, d = kp.codes.shape
    sh = (2 * (np.arange(g) % 4)).astype(np.uint8)

    def bytes_of(plane_dg):      # [rows][G] values 0..3 -> [rows][G/4]
        v = (plane_dg.astype(np.uint16) << sh[None, :]).reshape(plane_dg.shape[0], g // 4, 4)
        return v.sum(axis=-1).astype(np.uint8)

    t2 = bytes_of(kp.lo.T)
    th = bytes_of(kp.hi.T[kp.ch.astype(np.int64), :]) if n_boost else np.zeros((0, g // 4), np.uint8)
    idx = np.full(d, n_boost, dtype=np.uint8)
    idx[kp.ch.astype(np.int64)] = np.arange(n_boost, dtype=np.uint8)
    return t2, th, idx


def dequant_paper_tensors(t2, th, idx, scale, zero, n_boost):
    """K[G][D] (fp32) from the paper's logical page tensors (Sec. 4.1; what Alg. 1 computes).

    Channel by channel: the dense tensor gives every channel's low two bits; a channel whose entry in the index
    map is a real slot (not the sentinel) adds four times the two bits found in that row of the compact tensor;
    the resulting integer is mapped back with the channel's scale and zero-point."""
    d, gb = t2.shape
    k = np.empty((4 * gb, d), dtype=np.float32)

    def fields(row):          # the four 2-bit fields of every byte, lowest bits first: G values in token order
        return ((row[:, None] >> (2 * np.arange(4, dtype=np.uint8))[None, :]) & np.uint8(3)).reshape(-1).astype(np.int32)

    for c in range(d):
        code = fields(t2[c])
        if idx[c] < n_boost:
            code = code + 4 * fields(th[int(idx[c])])
        k[:, c] = (code.astype(np.float32) * np.float32(scale[c])).astype(np.float32) + np.float32(zero[c])
    return k


# --------------------------------------------------------------------------------------
# Attention (Eq. 1) over dequantized pages + full-precision window
# --------------------------------------------------------------------------------------
def softmax_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, sm_scale: float) -> np.ndarray:
    """o = softmax(sm_scale * q k^T) v for one query vector; fp32 inputs, fp64 arithmetic."""
    q64 = q.astype(np.float32).astype(np.float64)
    logits = (k.astype(np.float32).astype(np.float64) @ q64) * np.float64(np.float32(sm_scale))
    m = logits.max()
    e = np.exp(logits - m)
    p = e / e.sum()
    return (p @ v.astype(np.float32).astype(np.float64)).astype(np.float64)


class KittyCacheOracle:
    """Cache of one batch: pool of packed records, page tables, bf16 residual windows.

    State machine of the three-stage pipeline (Sec. 4.3) as seen from the next step: when the
    window of R full-precision tokens is full, the next append first quantizes it into a fresh
    page, then stores the new token; attention therefore always sees the newest token in full
    precision.  With R = 0 there is no window and append is not available.
    """

    def __init__(self, batch, n_kv_heads, n_q_heads, n_boost, residual_window, max_pages,
                 n_pool_pages, rank_metric=0, v_bits=2):
        assert n_q_heads % n_kv_heads == 0
        assert residual_window in (0, PAGE_SIZE)
        self.b, self.hkv, self.hq = batch, n_kv_heads, n_q_heads
        self.n_boost, self.r, self.metric, self.v_bits = n_boost, residual_window, rank_metric, v_bits
        self.lay = RecordLayout(n_boost, v_bits)
        self.pool = np.zeros((n_pool_pages, n_kv_heads, self.lay.record_bytes), dtype=np.uint8)
        self.page_table = np.zeros((batch, max_pages), dtype=np.int32)
        self.n_pages = np.zeros(batch, dtype=np.int32)
        self.resid_k = np.zeros((batch, n_kv_heads, max(residual_window, 1), HEAD_DIM), dtype=np.uint16)
        self.resid_v = np.zeros_like(self.resid_k)
        self.n_resid = np.zeros(batch, dtype=np.int32)

    # -- page quantizer over many pages (prefill path) -------------------------------
    def quantize_pages(self, k_bits, v_bits, page_ids):
        """k_bits/v_bits: uint16 bf16 patterns [n_pages][Hkv][G][D]; writes pool[page_ids]."""
        for i, pid in enumerate(page_ids):
            for h in range(self.hkv):
                kp = quantize_k_page(bf16_bits_to_f32(k_bits[i, h]), self.n_boost, self.metric)
                vp = quantize_v_page(bf16_bits_to_f32(v_bits[i, h]), self.v_bits)
                self.pool[pid, h] = pack_record(kp, vp)

    # -- one decode-step insert (Sec. 4.3 steps 1 and 3) ------------------------------
    def append_token(self, k_new_bits, v_new_bits, fresh_page_ids):
        """k_new_bits/v_new_bits: uint16 [B][Hkv][D]; returns number of sequences that flushed."""
        assert self.r > 0
        flushed = 0
        for b in range(self.b):
            if self.n_resid[b] == self.r:
                pid = int(fresh_page_ids[b])
                for h in range(self.hkv):
                    kp = quantize_k_page(bf16_bits_to_f32(self.resid_k[b, h]), self.n_boost, self.metric)
                    vp = quantize_v_page(bf16_bits_to_f32(self.resid_v[b, h]), self.v_bits)
                    self.pool[pid, h] = pack_record(kp, vp)
                self.page_table[b, self.n_pages[b]] = pid
                self.n_pages[b] += 1
                self.n_resid[b] = 0
                flushed += 1
            self.resid_k[b, :, self.n_resid[b]] = k_new_bits[b]
            self.resid_v[b, :, self.n_resid[b]] = v_new_bits[b]
            self.n_resid[b] += 1
        return flushed

    # -- dequantized view of one (sequence, kv-head) ------------------------------------
    def dequantized(self, b, h):
        ks, vs = [], []
        for i in range(int(self.n_pages[b])):
            kp, vp = unpack_record(self.pool[self.page_table[b, i], h], self.n_boost, self.v_bits)
            ks.append(dequant_k(kp))
            vs.append(dequant_v(vp))
        r = int(self.n_resid[b])
        if r:
            ks.append(bf16_bits_to_f32(self.resid_k[b, h, :r]))
            vs.append(bf16_bits_to_f32(self.resid_v[b, h, :r]))
        if not ks:
            return np.zeros((0, HEAD_DIM), np.float32), np.zeros((0, HEAD_DIM), np.float32)
        return np.concatenate(ks, axis=0), np.concatenate(vs, axis=0)

    # -- decode attention for chosen (b, q-head) pairs ----------------------------------
    def decode_attention(self, q_bits, sm_scale, pairs=None):
        """q_bits: uint16 [B][Hq][D].  Returns float64 [B][Hq][D] (rows not in `pairs` are NaN).

        A sequence with no tokens at all gives zeros.
        """
        out = np.full((self.b, self.hq, HEAD_DIM), np.nan, dtype=np.float64)
        g = self.hq // self.hkv
        if pairs is None:
            pairs = [(b, hq) for b in range(self.b) for hq in range(self.hq)]
        cache = {}
        for b, hq in pairs:
            h = hq // g
            if (b, h) not in cache:
                cache[(b, h)] = self.dequantized(b, h)
            k, v = cache[(b, h)]
            if k.shape[0] == 0:
                out[b, hq] = 0.0
            else:
                out[b, hq] = softmax_attention(bf16_bits_to_f32(q_bits[b, hq]), k, v, sm_scale)
        return out


class KittyUnitOracle:
    """The complete cache of ONE (sequence, kv-head) unit, buffer by buffer as Fig. 1 and Sec. 4.3 name them.

    Key side:   Sink (first S tokens, full precision) | quantized pages | Q-Buffer (< = G tokens, full precision)
    Value side: Sink | quantized pages | Q-Buffer (<= G) | Local (the R newest tokens)
    Step (1) insert:  Sink if it is not full; else K -> Key Q-Buffer, V -> Local, and when Local already
                      holds R tokens its oldest one moves to the Value Q-Buffer first.
    Step (2) attention over everything held, quantized parts dequantized per Alg. 1.
    Step (3) a Q-Buffer holding G tokens is quantized into one page and emptied.
    With S = 0 and R = 0 this is the single-window machine of `KittyCacheOracle` for one unit.
    Pages are kept as KPage / VPage objects: nothing here depends on the byte layout of a record.
    """

    def __init__(self, n_boost, sink=32, local=PAGE_SIZE, rank_metric=0, group=PAGE_SIZE, v_bits=2):
        self.n_boost, self.S, self.R, self.G, self.metric = n_boost, sink, local, group, rank_metric
        self.v_bits = v_bits
        self.sink_k, self.sink_v = [], []          # rows of bf16 bit patterns
        self.k_pages, self.k_qbuf = [], []
        self.v_pages, self.v_qbuf, self.v_local = [], [], []
        self.k_flushes = self.v_flushes = 0

    def insert(self, k_bits, v_bits):              # step (1)
        if len(self.sink_k) < self.S:
            self.sink_k.append(np.array(k_bits, np.uint16))
            self.sink_v.append(np.array(v_bits, np.uint16))
            return
        assert len(self.k_qbuf) < self.G and len(self.v_qbuf) < self.G   # guaranteed by step (3)
        self.k_qbuf.append(np.array(k_bits, np.uint16))
        if self.R == 0:
            self.v_qbuf.append(np.array(v_bits, np.uint16))
            return
        if len(self.v_local) == self.R:            # keep the window at R tokens: oldest one leaves
            self.v_qbuf.append(self.v_local.pop(0))
        self.v_local.append(np.array(v_bits, np.uint16))

    def quantize_if_full(self):                    # step (3)
        if len(self.k_qbuf) == self.G:
            self.k_pages.append(quantize_k_page(bf16_bits_to_f32(np.stack(self.k_qbuf)), self.n_boost, self.metric))
            self.k_qbuf = []
            self.k_flushes += 1
        if len(self.v_qbuf) == self.G:
            self.v_pages.append(quantize_v_page(bf16_bits_to_f32(np.stack(self.v_qbuf)), self.v_bits))
            self.v_qbuf = []
            self.v_flushes += 1

    def n_tokens(self):
        nk = len(self.sink_k) + self.G * len(self.k_pages) + len(self.k_qbuf)
        nv = len(self.sink_v) + self.G * len(self.v_pages) + len(self.v_qbuf) + len(self.v_local)
        assert nk == nv
        return nk

    def keys(self):
        rows = [bf16_bits_to_f32(np.stack(self.sink_k))] if self.sink_k else []
        rows += [dequant_k(kp) for kp in self.k_pages]
        if self.k_qbuf:
            rows.append(bf16_bits_to_f32(np.stack(self.k_qbuf)))
        return np.concatenate(rows, axis=0) if rows else np.zeros((0, HEAD_DIM), np.float32)

    def values(self):
        rows = [bf16_bits_to_f32(np.stack(self.sink_v))] if self.sink_v else []
        rows += [dequant_v(vp) for vp in self.v_pages]
        for part in (self.v_qbuf, self.v_local):
            if part:
                rows.append(bf16_bits_to_f32(np.stack(part)))
        return np.concatenate(rows, axis=0) if rows else np.zeros((0, HEAD_DIM), np.float32)

    def attention(self, q_bits, sm_scale):         # step (2); q_bits: uint16 [g][D] -> float64 [g][D]
        k, v = self.keys(), self.values()
        q_bits = np.atleast_2d(q_bits)
        if k.shape[0] == 0:
            return np.zeros((q_bits.shape[0], HEAD_DIM), np.float64)
        return np.stack([softmax_attention(bf16_bits_to_f32(qr), k, v, sm_scale) for qr in q_bits])

    def step(self, k_bits, v_bits, q_bits, sm_scale):
        self.insert(k_bits, v_bits)
        out = self.attention(q_bits, sm_scale)
        self.quantize_if_full()
        return out

    def prefill(self, k_bits, v_bits):
        """State after the given tokens went through steps (1) and (3) one at a time (no attention)."""
        for kr, vr in zip(k_bits, v_bits):
            self.insert(kr, vr)
            self.quantize_if_full()


def merge_partials(ms, ls, accs):
    """Combine split partials (m_i, l_i, acc_i[D]) of one query (log-sum-exp merge), fp64."""
    ms = np.asarray(ms, dtype=np.float64)
    m = ms.max()
    w = np.exp(ms - m)
    l = float((np.asarray(ls, dtype=np.float64) * w).sum())
    acc = (np.asarray(accs, dtype=np.float64) * w[:, None]).sum(axis=0)
    return acc / l


def partial_attention(q, k, v, sm_scale):
    """(m, l, acc) of one chunk, natural-log domain, fp64 — for the split/merge identity test."""
    q64 = q.astype(np.float64)
    logits = (k.astype(np.float64) @ q64) * np.float64(np.float32(sm_scale))
    m = logits.max()
    e = np.exp(logits - m)
    return m, e.sum(), e @ v.astype(np.float64)
