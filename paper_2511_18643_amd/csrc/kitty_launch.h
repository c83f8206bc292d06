// Kernel launches by record variant (number of 16-channel boost blocks, 4-bit Values or not).  The kernels of one
// variant are compiled in a translation unit of their own (kitty_variant.hip, built once per variant), so that the
// variants compile side by side; the host side of the library reaches them through these functions, which are
// declared here and defined and instantiated there.
#pragma once
#include "kitty_decode.h"
#include "kitty_prefill.h"

namespace kitty {

// what the host side has decided about a launch of the streaming kernel
struct SplitLaunch {
  dim3 grid;       // (ranges, kv-heads, sequences)
  bool wide;       // more than four query heads per kv-head: eight head slots per block
  bool big;        // 8-wavefront blocks (else 4)
  bool row_wave;   // a ninth wavefront for the full-precision rows, where the variant has one
  int fused;       // 0 attention only; 1 append first, one range; 2 append first, several ranges
};

template <int NB, bool V4> void launch_quantize_pages(const QuantPagesParams& P, unsigned blocks, hipStream_t st);
template <int NB, bool V4> void launch_project_quantize_pages(const ProjectParams& P, dim3 grid, hipStream_t st);
template <int NB, bool V4> void launch_append_token(const AppendParams& P, dim3 grid, hipStream_t st);
template <int NB, bool V4> void launch_decode_split(const DecodeParams& P, const SplitLaunch& s, hipStream_t st);

}  // namespace kitty
