// Record layout constants and small device helpers shared by the HIP kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kitty {

constexpr int D = 128;   // head_dim
constexpr int G = 128;   // page_size

// Byte offsets inside one (page, kv-head) record; NB16 = n_boost / 16.
//   K dense plane   4096 B   word (t, cb) at 1024*(t/32) + 16*((t%16) + 16*(cb%4)) + 4*(2*((t/16)%2) + cb/4)
//   K boost plane   512*NB16 word (t, s), T = t/16, j = t%16: NB16 == 1 at 8*(16*(T%4) + j) + 4*(T/4); otherwise at
//                   512*s + 16*(16*(T/4) + j) + 4*(T%4): the words a decode lane reads together are contiguous
//   k_scale, k_zero fp16[128] each, channel order
//   ch              uint8[n_boost] ascending, zero-padded to 128 B
//   V plane         4096 B   word (d, wv) at 1024*(d/32) + 16*((d%16) + 16*(wv%4)) + 4*(2*((d/16)%2) + wv/4)
//                   position p of a channel row holds token 16*(p%8) + p/8
//   V high plane    4096 B   only with 4-bit Values (V4): the high two bits, placed like the V plane
//   v_scale, v_zero fp16[128] each, position order
// Every word holds sixteen 2-bit elements, element a at bit 8*(a%4) + 2*(a/4), so that
// (w >> 2v) & 0x03030303 yields elements 4v..4v+3 as four bytes: an int8 matrix-core operand.
template <int NB16, bool V4 = false>
struct Rec {
  static constexpr int kd = 0;
  static constexpr int kb = 4096;
  static constexpr int ks = kb + 512 * NB16;
  static constexpr int kz = ks + 256;
  static constexpr int ch = kz + 256;
  static constexpr int vd = ch + 128;
  static constexpr int vh = vd + 4096;
  static constexpr int vs = vh + (V4 ? 4096 : 0);
  static constexpr int vz = vs + 256;
  static constexpr int bytes = vz + 256;
};

__host__ __device__ constexpr int record_bytes(int nb16, bool v4 = false) { return 9344 + 512 * nb16 + (v4 ? 4096 : 0); }

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

__device__ __forceinline__ float f16_bits_to_f32(uint16_t h) {
  _Float16 x = __builtin_bit_cast(_Float16, h);
  return (float)x;
}

__device__ __forceinline__ uint16_t f32_to_f16_bits(float f) {
  _Float16 x = (_Float16)f;   // v_cvt_f16_f32, round to nearest even
  return __builtin_bit_cast(uint16_t, x);
}

// DPP rotate within each row of 16 lanes; all-reduce over the row by four rotate+op steps.
// Maxima are taken on integers (bit patterns of non-negative floats order like unsigned integers), which
// keeps the float canonicalisation the compiler attaches to fmaxf out of the reduction.
template <int N>
__device__ __forceinline__ int row_ror_i(int v) {
  return __builtin_amdgcn_update_dpp(v, v, 0x120 + N, 0xf, 0xf, true);
}
template <int N>
__device__ __forceinline__ float row_ror(float v) { return __builtin_bit_cast(float, row_ror_i<N>(__builtin_bit_cast(int, v))); }

__device__ __forceinline__ int row_max_i32(int v) {
  v = max(v, row_ror_i<8>(v));
  v = max(v, row_ror_i<4>(v));
  v = max(v, row_ror_i<2>(v));
  v = max(v, row_ror_i<1>(v));
  return v;
}
__device__ __forceinline__ uint32_t row_max_u32(uint32_t v) {
  v = max(v, (uint32_t)row_ror_i<8>((int)v));
  v = max(v, (uint32_t)row_ror_i<4>((int)v));
  v = max(v, (uint32_t)row_ror_i<2>((int)v));
  v = max(v, (uint32_t)row_ror_i<1>((int)v));
  return v;
}
// row maximum of non-negative floats
__device__ __forceinline__ float row_max_nonneg(float v) { return __uint_as_float(row_max_u32(__float_as_uint(v))); }
// row maximum of arbitrary finite floats (or -inf)
__device__ __forceinline__ float row_max(float v) {
  v = fmaxf(v, row_ror<8>(v));
  v = fmaxf(v, row_ror<4>(v));
  v = fmaxf(v, row_ror<2>(v));
  v = fmaxf(v, row_ror<1>(v));
  return v;
}
__device__ __forceinline__ float row_sum(float v) {
  v += row_ror<8>(v);
  v += row_ror<4>(v);
  v += row_ror<2>(v);
  v += row_ror<1>(v);
  return v;
}

}  // namespace kitty
