// Prefill-side fusion: Key/Value projection of a 128-token tile on the bf16 matrix cores, quantized into a page
// record straight from on-chip memory (Sec. 4.3 step 3 applied to the tile that produces the page; Sec. 4.1 record).
// The bf16 K and V of the tile never travel to HBM and back: the projection's output tile is rounded to bf16 in
// LDS, and the page quantizer of kitty_quant.h reads it from there.
//
// One workgroup of 256 threads per (page, kv-head): C[channel][token] = sum_i W[channel][i] * X[token][i] for the
// 128 Key channels and the 128 Value channels of the head (fp32 accumulation in v_mfma_f32_32x32x16_bf16; the
// order of the additions is the matrix core's).  Wavefront w computes matrix w & 1 (0 = Key, 1 = Value) for the
// tokens 64*(w >> 1) .. +63: four row blocks of 32 channels times two column blocks of 32 tokens.  The operand
// chunks (32 input features at a time) are staged in LDS, the next chunk's global loads are in flight while the
// current one is multiplied.
#pragma once
#include "kitty_common.h"
#include "kitty_quant.h"

namespace kitty {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf16 __attribute__((ext_vector_type(8)));

struct ProjectParams {
  const uint16_t* x;        // bf16 [tokens][hidden], row t at x + t * x_token_stride
  const uint16_t* w_k;      // bf16 [n_kv_heads * D][hidden]: row h*D + c produces channel c of kv-head h
  const uint16_t* w_v;
  int64_t x_token_stride;
  const int64_t* src_token_offsets;   // [n_pages] first token of source page i
  const int32_t* dst_page_ids;
  uint8_t* pool;
  int32_t hidden, n_kv_heads, n_pool_pages, rank_metric;
};

#ifndef KITTY_PJ_KC
#define KITTY_PJ_KC 64
#endif
constexpr int PJ_KC = KITTY_PJ_KC;       // input features per staged chunk (a chunk's matrix work has to cover the latency of the next chunk's loads)
constexpr int PJ_PITCH = PJ_KC + 8;       // bf16 elements between staged rows (16 bytes of padding: 16-byte reads of 32 rows spread over all banks)
constexpr int PJ_TILE_PITCH = D + 8;      // bf16 elements between token rows of the projected tile

struct ProjectSmem {
  union {
    struct {
      alignas(16) uint16_t x[G][PJ_PITCH];            // tokens x features
      alignas(16) uint16_t w[2 * D][PJ_PITCH];        // Key channels, then Value channels, x features
    } stage;
    struct {
      alignas(16) uint16_t k[G][PJ_TILE_PITCH];       // projected tile, bf16, [token][channel]
      alignas(16) uint16_t v[G][PJ_TILE_PITCH];
      alignas(16) QuantSmem quant;
    } out;
  };
};

template <int NB16, bool V4>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void project_quantize_pages_kernel(ProjectParams p) {
  __shared__ ProjectSmem smem;
  const int page = blockIdx.x, h = blockIdx.y;
  const int32_t pid = p.dst_page_ids[page];
  if (pid < 0 || pid >= p.n_pool_pages) return;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
  const int mat = w & 1, thalf = w >> 1;
  const uint16_t* xs = p.x + p.src_token_offsets[page] * p.x_token_stride;
  const uint16_t* wk = p.w_k + (size_t)h * D * p.hidden;
  const uint16_t* wv = p.w_v + (size_t)h * D * p.hidden;

  // global -> registers -> LDS in 16-byte pieces; consecutive threads take consecutive pieces of a row, so that a
  // wavefront's load covers whole cache lines (a row of a chunk is PR pieces; X has G rows, W has 2*D rows: Key
  // channels, then Value channels)
  constexpr int PR = PJ_KC / 8, NX = G * PR / 256, NWV = 2 * D * PR / 256;
  static_assert(NX >= 1, "chunk too small for 256 threads");
  uint4 gx[NX], gw[NWV];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < NX; ++i) {
      const int idx = tid + 256 * i, row = idx / PR, pc = idx % PR;
      gx[i] = *reinterpret_cast<const uint4*>(xs + (size_t)row * p.x_token_stride + k0 + 8 * pc);
    }
#pragma unroll
    for (int i = 0; i < NWV; ++i) {
      const int idx = tid + 256 * i, row = idx / PR, pc = idx % PR;
      const uint16_t* wr = row < D ? wk + (size_t)row * p.hidden : wv + (size_t)(row - D) * p.hidden;
      gw[i] = *reinterpret_cast<const uint4*>(wr + k0 + 8 * pc);
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int i = 0; i < NX; ++i) {
      const int idx = tid + 256 * i;
      *reinterpret_cast<uint4*>(&smem.stage.x[idx / PR][8 * (idx % PR)]) = gx[i];
    }
#pragma unroll
    for (int i = 0; i < NWV; ++i) {
      const int idx = tid + 256 * i;
      *reinterpret_cast<uint4*>(&smem.stage.w[idx / PR][8 * (idx % PR)]) = gw[i];
    }
  };

  v16f acc[4][2];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  const int lr = l & 31, lk = l >> 5;      // operand row of this lane and its half of the 16 features of a step
  fetch(0);
  for (int k0 = 0; k0 < p.hidden; k0 += PJ_KC) {
    __syncthreads();                       // the previous chunk has been consumed
    stash();
    __syncthreads();
    if (k0 + PJ_KC < p.hidden) fetch(k0 + PJ_KC);
#pragma unroll
    for (int ks = 0; ks < PJ_KC; ks += 16) {
      v8bf16 a[4], b[2];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        a[i] = __builtin_bit_cast(v8bf16, *reinterpret_cast<const uint4*>(&smem.stage.w[D * mat + 32 * i + lr][ks + 8 * lk]));
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
        b[jb] = __builtin_bit_cast(v8bf16, *reinterpret_cast<const uint4*>(&smem.stage.x[64 * thalf + 32 * jb + lr][ks + 8 * lk]));
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
          acc[i][jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[jb], acc[i][jb], 0, 0, 0);
    }
  }
  __syncthreads();                         // staging memory is reused for the projected tile
  // accumulator register r of a 32x32 block: row (channel) 8*(r/4) + 4*(l/32) + r%4, column (token) l%32.
  // Four consecutive channels of one token are rounded to bf16 (nearest even) and stored as 8 bytes.
  uint16_t (*tile)[PJ_TILE_PITCH] = mat == 0 ? smem.out.k : smem.out.v;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int jb = 0; jb < 2; ++jb)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int tok = 64 * thalf + 32 * jb + lr, ch = 32 * i + 8 * q4 + 4 * lk;
        const uint32_t lo = (uint32_t)f32_to_bf16_rne(acc[i][jb][4 * q4]) | ((uint32_t)f32_to_bf16_rne(acc[i][jb][4 * q4 + 1]) << 16);
        const uint32_t hi = (uint32_t)f32_to_bf16_rne(acc[i][jb][4 * q4 + 2]) | ((uint32_t)f32_to_bf16_rne(acc[i][jb][4 * q4 + 3]) << 16);
        *reinterpret_cast<uint2*>(&tile[tok][ch]) = make_uint2(lo, hi);
      }
  __syncthreads();
  uint8_t* rec = p.pool + ((size_t)pid * p.n_kv_heads + h) * (size_t)Rec<NB16, V4>::bytes;
  quantize_page<NB16, V4, false>(smem.out.quant, &smem.out.k[0][0], &smem.out.v[0][0], PJ_TILE_PITCH, rec, p.rank_metric);
}

}  // namespace kitty
