"""MI355X-native Kitty decode attention over a page-centric 2-bit KV cache (arXiv 2511.18643).

`paper_2511_18643_amd.kitty` is the thin Python binding of the C-ABI library (loaded on first
use; it raises if the HIP library has not been built).  `paper_2511_18643_amd.synth` draws the
seeded synthetic workloads.
"""
