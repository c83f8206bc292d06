"""How often do the two readings of the quantizer's rounding step give different codes?

TEST INFRASTRUCTURE ONLY (CPU, numpy; calls nothing but the oracle).  The paper fixes the inverse map
(Alg. 1: K = X * scale + zero_point) and names KIVI-style asymmetric quantization (Sec. 2.1, Sec. 3.3) but
prints no rounding formula.  The oracle takes  code = clamp(rint((x - zero) * inv), 0, qmax)  with
inv = fp32(1 / scale)  rounded once per channel (token); the other natural reading divides every element:
code = clamp(rint((x - zero) / scale), 0, qmax).  This script counts, on seeded pages of the 8k-context and
128k-context workloads, the codes on which the two differ, and for each of them whether the exact quotient
(x - zero) / scale is a half-integer, i.e. whether both codes are equally near the input.

Run:  python -m oracle.reading_a5_division_vs_reciprocal [pages per workload]
"""
from __future__ import annotations

import sys
from fractions import Fraction

import numpy as np

from oracle import kitty_oracle as ko
from paper_2511_18643_amd import synth


def division_codes(x, scale_h, zero_h, qmax):
    """The per-element-division reading, IEEE fp32, against the same stored fp16 scale and zero-point."""
    s = scale_h.astype(np.float32)
    z = zero_h.astype(np.float32)
    with np.errstate(divide="ignore", invalid="ignore"):
        r = np.where(s > 0, np.rint(((x - z).astype(np.float32) / s).astype(np.float32)), np.float32(0.0))
    return np.minimum(np.maximum(r, np.float32(0.0)), qmax.astype(np.float32)).astype(np.uint8)


def count(workload: str, n_pages: int):
    w = synth.WORKLOADS[workload]
    total = diff = ties = 0
    off_by = 0
    for h in range(min(w.n_kv_heads, 4)):
        kb, vb = synth.kv_block(w, 0, h, n_pages * 128)
        for p in range(n_pages):
            k = ko.bf16_bits_to_f32(kb[128 * p:128 * (p + 1)])
            v = ko.bf16_bits_to_f32(vb[128 * p:128 * (p + 1)])
            kp = ko.quantize_k_page(k, w.n_boost, w.rank_metric)
            vp = ko.quantize_v_page(v)
            qk = np.full(128, 3.0, np.float32)
            qk[kp.ch.astype(int)] = 15.0
            alt_k = division_codes(k, kp.scale[None, :], kp.zero[None, :], qk[None, :])
            alt_v = division_codes(v, vp.scale[:, None], vp.zero[:, None], np.full((128, 1), 3.0, np.float32))
            for got, alt, x, sc, zr in ((kp.codes, alt_k, k, np.broadcast_to(kp.scale[None, :], k.shape), np.broadcast_to(kp.zero[None, :], k.shape)),
                                       (vp.codes, alt_v, v, np.broadcast_to(vp.scale[:, None], v.shape), np.broadcast_to(vp.zero[:, None], v.shape))):
                total += got.size
                bad = np.nonzero(got != alt)
                diff += len(bad[0])
                for t, c in zip(*bad):
                    quo = (Fraction(float(x[t, c])) - Fraction(float(zr[t, c]))) / Fraction(float(sc[t, c]))
                    ties += int((2 * quo).denominator == 1 and quo.denominator == 2)
                    off_by = max(off_by, abs(int(got[t, c]) - int(alt[t, c])))
    return total, diff, ties, off_by


def main():
    n = int(sys.argv[1]) if len(sys.argv) > 1 else 16
    for name in ("c2", "c4"):
        total, diff, ties, off_by = count(name, n)
        print(f"{name}: {total} codes ({n} pages x {min(synth.WORKLOADS[name].n_kv_heads, 4)} kv-heads, Keys and Values): "
              f"{diff} differ between the two readings ({diff / total:.2e}); {ties} of those are exact ties of "
              f"(x - zero) / scale; largest difference {off_by} code")


if __name__ == "__main__":
    main()
