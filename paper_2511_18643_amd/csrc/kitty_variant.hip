// The kernels of one record variant: compiled once per (KITTY_VARIANT_NB, KITTY_VARIANT_V4), see kitty_launch.h.
#include <type_traits>

#include "kitty_launch.h"

#if !defined(KITTY_VARIANT_NB) || !defined(KITTY_VARIANT_V4)
#error "build with -DKITTY_VARIANT_NB=<0..8> -DKITTY_VARIANT_V4=<0|1>"
#endif

namespace kitty {

template <int NB, bool V4>
void launch_quantize_pages(const QuantPagesParams& P, unsigned blocks, hipStream_t st) {
  hipLaunchKernelGGL((quantize_pages_kernel<NB, V4>), dim3(blocks), dim3(256), 0, st, P);
}

template <int NB, bool V4>
void launch_project_quantize_pages(const ProjectParams& P, dim3 grid, hipStream_t st) {
  hipLaunchKernelGGL((project_quantize_pages_kernel<NB, V4>), grid, dim3(256), 0, st, P);
}

template <int NB, bool V4>
void launch_append_token(const AppendParams& P, dim3 grid, hipStream_t st) {
  hipLaunchKernelGGL((append_token_kernel<NB, V4>), grid, dim3(256), 0, st, P);
}

template <int NB, bool V4>
void launch_decode_split(const DecodeParams& P, const SplitLaunch& s, hipStream_t st) {
  auto go = [&](auto hpl, auto nw, auto fu) {
    constexpr int HPL = decltype(hpl)::value, NW = decltype(nw)::value;
    constexpr int FU = decltype(fu)::value;
    hipLaunchKernelGGL((decode_split_kernel<NB, HPL, NW, FU, V4>), s.grid, dim3(64 * NW), 0, st, P);
  };
  using I1 = std::integral_constant<int, 1>; using I2 = std::integral_constant<int, 2>;
  using I4 = std::integral_constant<int, 4>; using I8 = std::integral_constant<int, 8>;
  // 8-wavefront blocks of the variants that fit 168 registers (2-bit Values with any boost count; 4-bit Values
  // without boosted channels) get a ninth wavefront for the full-precision rows (32k workload -1 to -3 %, 8k
  // workload -12 %); not with the Value Local window, whose rows can only follow the pages (+2 % there)
  constexpr bool ROWW_OK = V4 ? NB == 0 : true;
  auto go_rows = [&](auto fu) {
    constexpr int FU = decltype(fu)::value;
    if constexpr (ROWW_OK) {
      if (s.row_wave) {
        hipLaunchKernelGGL((decode_split_kernel<NB, 1, 8, FU, V4, true>), s.grid, dim3(64 * 9), 0, st, P);
        return;
      }
    }
    go(I1{}, I8{}, fu);
  };
  using F0 = std::integral_constant<int, 0>;   // attention only
  using F1 = std::integral_constant<int, 1>;   // fused step, one range: the kernel also stores the token and advances the state
  using F2 = std::integral_constant<int, 2>;   // fused step, several ranges: the merge launch does that
  auto pick = [&](auto fu) {
    if (s.wide) {
      // (eight-head groups with more than 64 boosted channels: 4-wavefront blocks only, one wavefront per SIMD, because
      // their two-pass contractions need more than 256 registers)
      if constexpr (NB > 4) go(I2{}, I4{}, fu);
      else if (s.big) go(I2{}, I8{}, fu);
      else go(I2{}, I4{}, fu);
    } else {
      if (s.big) go_rows(fu); else go(I1{}, I4{}, fu);
    }
  };
  if (s.fused == 0) pick(F0{});
  else if (s.fused == 1) pick(F1{});
  else pick(F2{});
}

template void launch_quantize_pages<KITTY_VARIANT_NB, KITTY_VARIANT_V4 != 0>(const QuantPagesParams&, unsigned, hipStream_t);
template void launch_project_quantize_pages<KITTY_VARIANT_NB, KITTY_VARIANT_V4 != 0>(const ProjectParams&, dim3, hipStream_t);
template void launch_append_token<KITTY_VARIANT_NB, KITTY_VARIANT_V4 != 0>(const AppendParams&, dim3, hipStream_t);
template void launch_decode_split<KITTY_VARIANT_NB, KITTY_VARIANT_V4 != 0>(const DecodeParams&, const SplitLaunch&, hipStream_t);

}  // namespace kitty
