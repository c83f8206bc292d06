"""Seeded synthetic workloads shaped like the paper's decode-time KV caches.

This module only draws random inputs (and rounds them to bf16, which is the input format of
the library); it holds none of the method's arithmetic, so both the tests' CPU oracle and the
HIP path may be fed from it.  The paper evaluates on Qwen3 / LLaMA3 activations (Sec. 5.1,
Sec. 5.5); no weights or datasets exist here, so Keys are Gaussian with a few persistent
high-magnitude channels (the pattern of Fig. 2a), Values are Gaussian.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

HEAD_DIM = 128
PAGE = 128


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    context: int              # tokens per sequence at attention time (ignored if lengths given)
    n_boost: int              # boosted Key channels per page
    residual_window: int      # 0 or 128
    rank_metric: int          # 0 = mean |x| (Eq. 2), 1 = max - min
    sm_scale: float
    q_scale: float            # q ~ N(0,1) * q_scale
    n_outlier: int            # persistent outlier channels per kv-head
    outlier_gain: float
    token_shift_std: float    # per-token scalar added to every Key channel
    varying_outliers: bool = False   # outlier set and gain redrawn per page (4..12 channels, x4..x16)
    seed: int = 0

    @property
    def gqa(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def pages_and_resid(self, length: int | None = None):
        """(packed pages, residual tokens) of a sequence of `length` tokens."""
        n = self.context if length is None else length
        if self.residual_window == 0:
            assert n % PAGE == 0
            return n // PAGE, 0
        n_pages = (n + PAGE - 1) // PAGE - 1
        return n_pages, n - n_pages * PAGE


INV_SQRT_D = float(1.0 / np.sqrt(128.0))

WORKLOADS = {
    # one head, 8 pages, no window: the small correctness case
    "c1": Workload("c1", 1, 1, 1, 1024, 16, 0, 1, 1.0, INV_SQRT_D, 8, 10.0, 0.0, seed=101),
    # Llama-3-8B-shaped layer, 8k context
    "c2": Workload("c2", 16, 32, 8, 8192, 16, 128, 0, INV_SQRT_D, 1.0, 6, 8.0, 0.1, seed=202),
    # Llama-3-8B-shaped layer, 32k context
    "c3": Workload("c3", 32, 32, 8, 32768, 16, 128, 0, INV_SQRT_D, 1.0, 6, 8.0, 0.1, seed=303),
    # Llama-3-70B-shaped layer, 128k context, 25 % boost, outlier set changes page to page
    "c4": Workload("c4", 8, 64, 8, 131072, 32, 128, 0, INV_SQRT_D, 1.0, 8, 8.0, 0.1,
                   varying_outliers=True, seed=404),
    # Qwen3-8B-shaped decode loop: 36 layers of this shape, variable-length batch (see sequence_lengths)
    "c5": Workload("c5", 128, 32, 8, 0, 16, 128, 0, INV_SQRT_D, 1.0, 6, 8.0, 0.1, seed=505),
}

C5_LAYERS = 36
C5_STEPS = 256


def sequence_lengths(w: Workload, lo: int = 1024, hi: int = 32768) -> list:
    """Seeded context lengths of a variable-length batch, uniform in [lo, hi]."""
    r = _rng(w.seed, 993)
    return [int(x) for x in r.integers(lo, hi + 1, size=w.batch)]


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even (finite inputs)."""
    u = np.array(x, dtype=np.float32, copy=True).view(np.uint32)
    u += np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (u >> np.uint32(16)).astype(np.uint16)


def _rng(seed: int, *stream: int) -> np.random.Generator:
    """Counter-based (Philox) generator keyed by the workload seed and a stream id."""
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, *stream])))


def outlier_channels(w: Workload, h: int) -> np.ndarray:
    """The persistent outlier channels of kv-head h."""
    r = _rng(w.seed, 7, h)
    return np.sort(r.choice(HEAD_DIM, size=w.n_outlier, replace=False))


def kv_block(w: Workload, b: int, h: int, n_tokens: int, first_token: int = 0):
    """bf16 bits (uint16) of K and V for tokens [first_token, first_token + n_tokens) of (b, h).

    Tokens are drawn page by page from a counter-based stream keyed by (seed, b, h, page), so a
    block can be regenerated piecewise and any slice is reproducible on its own.
    """
    assert first_token % PAGE == 0
    k = np.empty((n_tokens, HEAD_DIM), dtype=np.float32)
    v = np.empty((n_tokens, HEAD_DIM), dtype=np.float32)
    fixed = outlier_channels(w, h)
    done = 0
    page = first_token // PAGE
    while done < n_tokens:
        n = min(PAGE, n_tokens - done)
        r = _rng(w.seed, b, h, page)
        kp = r.standard_normal((PAGE, HEAD_DIM), dtype=np.float32)
        vp = r.standard_normal((PAGE, HEAD_DIM), dtype=np.float32)
        shift = r.standard_normal((PAGE, 1), dtype=np.float32) * np.float32(w.token_shift_std)
        if w.varying_outliers:
            cnt = int(r.integers(4, 13))
            chans = r.choice(HEAD_DIM, size=cnt, replace=False)
            gains = r.uniform(4.0, 16.0, size=cnt).astype(np.float32)
            kp[:, chans] *= gains[None, :]
        else:
            kp[:, fixed] *= np.float32(w.outlier_gain)
        kp += shift
        k[done:done + n] = kp[:n]
        v[done:done + n] = vp[:n]
        done += n
        page += 1
    return to_bf16_bits(k), to_bf16_bits(v)


def query(w: Workload, step: int = 0) -> np.ndarray:
    """bf16 bits of q [batch][n_q_heads][D] for decode step `step`."""
    r = _rng(w.seed, 991, step)
    q = r.standard_normal((w.batch, w.n_q_heads, HEAD_DIM), dtype=np.float32) * np.float32(w.q_scale)
    return to_bf16_bits(q)


def new_token(w: Workload, step: int):
    """bf16 bits of (k_new, v_new) [batch][n_kv_heads][D] appended at decode step `step`."""
    r = _rng(w.seed, 992, step)
    k = r.standard_normal((w.batch, w.n_kv_heads, HEAD_DIM), dtype=np.float32)
    v = r.standard_normal((w.batch, w.n_kv_heads, HEAD_DIM), dtype=np.float32)
    shift = r.standard_normal((w.batch, w.n_kv_heads, 1), dtype=np.float32) * np.float32(w.token_shift_std)
    for h in range(w.n_kv_heads):
        k[:, h, outlier_channels(w, h)] *= np.float32(w.outlier_gain)
    k += shift
    return to_bf16_bits(k), to_bf16_bits(v)


def scaled(w: Workload, **kw) -> Workload:
    """A copy of `w` with some fields replaced (used to shrink a workload for tests)."""
    d = {f: getattr(w, f) for f in w.__dataclass_fields__}
    d.update(kw)
    return Workload(**d)
