// Page quantizer: one workgroup of 256 threads turns G=128 tokens of one kv-head into a record.
// Sec. 2.1 (per-channel K / per-token V asymmetric quantization), Sec. 3.2 Eq. (2) (channel
// score and top-K boost), Sec. 4.1 (dense low-bit plane + compact high-bit plane + index list).
#pragma once
#include "kitty_common.h"

namespace kitty {

struct QuantSmem {
  uint32_t tile[G * 65];   // 128 rows of 128 bf16, row stride 65 dwords (bank-conflict-free rows and columns)
  double sum[2][D];
  double score[D];
  float mn[2][D];
  float mx[2][D];
  float inv[D];            // 1 / float(fp16 scale) (0 if the scale is 0), per channel (K phase) or per token (V phase)
  float zr[D];             // float(fp16 zero-point)
  float qm[D];             // 15 or 3
  unsigned long long ballot0;
  uint8_t chl[D];
};

__device__ __forceinline__ float tile_elem(const QuantSmem& s, int t, int c) {
  return bf16_to_f32(reinterpret_cast<const uint16_t*>(s.tile)[t * 130 + c]);
}

// code = clamp(rint((x - zero) * inv), 0, qmax), inv = 1/scale rounded once (IEEE), 0 for a zero scale.
// fp32 subtract and multiply, ties to even; with inv == 0 every code is 0.
// qcode_bits returns the raw bits of clamp((x - zero) * inv, 0, qmax) + 1.5 * 2^23: the addition rounds to
// the nearest integer, ties to even, and leaves that integer in the low byte (clamping first gives the same
// integer as rounding first, because the bounds are integers).
__device__ __forceinline__ uint32_t qcode_bits(float x, float inv, float z, float qmax) {
  const float f = __builtin_amdgcn_fmed3f(__fmul_rn(__fsub_rn(x, z), inv), 0.0f, qmax);
  return __float_as_uint(__fadd_rn(f, 12582912.0f));
}

// Sixteen codes on their way into one packed word.  Register v collects the low bytes of elements 4v..4v+3
// (three byte permutes per four codes); the word takes the low two bits of every byte of register v at bit
// offset 2v (low plane), or bits 2..3 (high plane of 4-bit codes).
struct Pack16 {
  uint32_t u[16];
  __device__ __forceinline__ void put(int a, uint32_t bits) { u[a] = bits; }
  __device__ __forceinline__ uint32_t bytes(int v) const {
    const uint32_t lo = __builtin_amdgcn_perm(u[4 * v + 1], u[4 * v], 0x0c0c0400u);
    const uint32_t hi = __builtin_amdgcn_perm(u[4 * v + 3], u[4 * v + 2], 0x0c0c0400u);
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
  }
  __device__ __forceinline__ uint32_t low() const {
    constexpr uint32_t m = 0x03030303u;
    return (bytes(0) & m) | ((bytes(1) & m) << 2) | ((bytes(2) & m) << 4) | ((bytes(3) & m) << 6);
  }
  __device__ __forceinline__ uint32_t high() const {
    constexpr uint32_t m = 0x0c0c0c0cu;
    return ((bytes(0) & m) >> 2) | (bytes(1) & m) | ((bytes(2) & m) << 2) | ((bytes(3) & m) << 4);
  }
};
__device__ __forceinline__ float inv_scale(float s) { return s > 0.0f ? __fdiv_rn(1.0f, s) : 0.0f; }

// src: bf16 rows of 128 channels, row t at src + t*token_stride (elements), 16-byte aligned.  A thread
// fetches eight 16-byte pieces (fetch_tile) and puts them into the padded LDS tile (store_tile); the two
// halves are separate so that the Value tile can be on its way while the Key tile is being worked on.
struct TileRegs { uint4 v[8]; };
__device__ __forceinline__ void fetch_tile(TileRegs& r, const uint16_t* __restrict__ src, int64_t token_stride, int tid) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int chunk = tid + 256 * i;
    const int t = chunk >> 4, part = chunk & 15;
    r.v[i] = *reinterpret_cast<const uint4*>(src + (int64_t)t * token_stride + part * 8);
  }
}
__device__ __forceinline__ void store_tile(QuantSmem& s, const TileRegs& r, int tid) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int chunk = tid + 256 * i;
    const int t = chunk >> 4, part = chunk & 15;
    uint32_t* d = &s.tile[t * 65 + part * 4];
    d[0] = r.v[i].x; d[1] = r.v[i].y; d[2] = r.v[i].z; d[3] = r.v[i].w;
  }
}

// One block of at least 256 threads; threads 0..255 do the work, every thread takes part in the barriers.
template <int NB16>
__device__ __forceinline__ void quantize_page(QuantSmem& s, const uint16_t* __restrict__ ksrc, const uint16_t* __restrict__ vsrc,
                              int64_t token_stride, uint8_t* __restrict__ rec, int rank_metric) {
  using R = Rec<NB16>;
  const int tid = threadIdx.x;
  const bool act = tid < 256;
  const int c = tid & 127, half = (tid >> 7) & 1;

  // ---------------- Key page ----------------
  TileRegs tr;
  if (act) {
    fetch_tile(tr, ksrc, token_stride, tid);
    store_tile(s, tr, tid);
    fetch_tile(tr, vsrc, token_stride, tid);   // used after the Key page is done
  }
  __syncthreads();
  if (act) {  // per-channel min, max, sum |x| over half of the tokens
    float mn = INFINITY, mx = -INFINITY;
    double sum = 0.0;
    for (int t = half * 64; t < half * 64 + 64; ++t) {
      float x = tile_elem(s, t, c);
      mn = fminf(mn, x);
      mx = fmaxf(mx, x);
      sum += (double)fabsf(x);   // exact for bf16 inputs: the order of the additions does not matter
    }
    s.mn[half][c] = mn; s.mx[half][c] = mx; s.sum[half][c] = sum;
  }
  __syncthreads();
  float mn = 0.f, mx = 0.f;
  if (tid < 128) {
    mn = fminf(s.mn[0][c], s.mn[1][c]);
    mx = fmaxf(s.mx[0][c], s.mx[1][c]);
    s.score[c] = rank_metric == 0 ? s.sum[0][c] + s.sum[1][c] : (double)__fsub_rn(mx, mn);
  }
  __syncthreads();
  bool boosted = false;
  if (tid < 128) {  // rank under (score descending, channel ascending)
    const double my = s.score[c];
    int rank = 0;
    for (int o = 0; o < 128; ++o) {
      double so = s.score[o];
      rank += (so > my) || (so == my && o < c);
    }
    boosted = rank < 16 * NB16;
  }
  unsigned long long bal = __ballot(boosted);
  if (tid == 0) s.ballot0 = bal;
  __syncthreads();
  if (tid < 128) {
    const int lane = tid & 63;
    int slot = __popcll(bal & ((1ull << lane) - 1ull)) + (tid >= 64 ? __popcll(s.ballot0) : 0);
    const float qmax = boosted ? 15.0f : 3.0f;
    const uint16_t sh = f32_to_f16_bits(__fdiv_rn(__fsub_rn(mx, mn), qmax));
    const uint16_t zh = f32_to_f16_bits(mn);
    s.inv[c] = inv_scale(f16_bits_to_f32(sh));
    s.zr[c] = f16_bits_to_f32(zh);
    s.qm[c] = qmax;
    reinterpret_cast<uint16_t*>(rec + R::ks)[c] = sh;
    reinterpret_cast<uint16_t*>(rec + R::kz)[c] = zh;
    if (boosted) { s.chl[slot] = (uint8_t)c; rec[R::ch + slot] = (uint8_t)c; }
    if (c >= 16 * NB16) rec[R::ch + c] = 0;   // pad bytes of the channel list
  }
  __syncthreads();
  if (act) {  // dense plane: thread (q, lane) builds the 16 bytes that lane reads back in the decode kernel
    const int q = tid >> 6, lane = tid & 63;
    uint32_t w[4];
#pragma unroll
    for (int csel = 0; csel < 2; ++csel) {
      const int cb = 4 * csel + (lane >> 4);
      float inv[16], zr[16], qm[16];
#pragma unroll
      for (int a4 = 0; a4 < 4; ++a4) {
        const float4 i4 = *reinterpret_cast<const float4*>(&s.inv[16 * cb + 4 * a4]);
        const float4 z4 = *reinterpret_cast<const float4*>(&s.zr[16 * cb + 4 * a4]);
        const float4 q4 = *reinterpret_cast<const float4*>(&s.qm[16 * cb + 4 * a4]);
        inv[4 * a4] = i4.x; inv[4 * a4 + 1] = i4.y; inv[4 * a4 + 2] = i4.z; inv[4 * a4 + 3] = i4.w;
        zr[4 * a4] = z4.x; zr[4 * a4 + 1] = z4.y; zr[4 * a4 + 2] = z4.z; zr[4 * a4 + 3] = z4.w;
        qm[4 * a4] = q4.x; qm[4 * a4 + 1] = q4.y; qm[4 * a4 + 2] = q4.z; qm[4 * a4 + 3] = q4.w;
      }
#pragma unroll
      for (int tsel = 0; tsel < 2; ++tsel) {
        const int t = 32 * q + 16 * tsel + (lane & 15);
        Pack16 pk;
#pragma unroll
        for (int a2 = 0; a2 < 8; ++a2) {
          const uint32_t two = s.tile[t * 65 + 8 * cb + a2];
          const float x0 = __uint_as_float(two << 16), x1 = __uint_as_float(two & 0xffff0000u);
          pk.put(2 * a2, qcode_bits(x0, inv[2 * a2], zr[2 * a2], qm[2 * a2]));
          pk.put(2 * a2 + 1, qcode_bits(x1, inv[2 * a2 + 1], zr[2 * a2 + 1], qm[2 * a2 + 1]));
        }
        w[2 * tsel + csel] = pk.low();
      }
    }
    reinterpret_cast<uint4*>(rec + R::kd)[64 * q + lane] = make_uint4(w[0], w[1], w[2], w[3]);
  }
  if constexpr (NB16 > 0) {  // boost plane: high two bits of the boosted channels, slot order
    if (act) {
      for (int idx = tid; idx < 128 * NB16; idx += 256) {
        const int sblk = idx >> 7, u = (idx >> 6) & 1, lane = idx & 63;
        const int t = 16 * (4 * u + (lane >> 4)) + (lane & 15);
        Pack16 pk;
#pragma unroll
        for (int a = 0; a < 16; ++a) {
          const int ch = s.chl[16 * sblk + a];
          pk.put(a, qcode_bits(tile_elem(s, t, ch), s.inv[ch], s.zr[ch], 15.0f));
        }
        *reinterpret_cast<uint32_t*>(rec + R::kb + 512 * sblk + 8 * lane + 4 * u) = pk.high();
      }
    }
  }
  __syncthreads();

  // ---------------- Value page ----------------
  if (act) store_tile(s, tr, tid);
  __syncthreads();
  if (act) {  // per-token min, max over half of the channels
    const int t = c;
    float mn2 = INFINITY, mx2 = -INFINITY;
    for (int k = 0; k < 32; ++k) {
      uint32_t two = s.tile[t * 65 + half * 32 + k];
      float a = __uint_as_float(two << 16), b = __uint_as_float(two & 0xffff0000u);
      mn2 = fminf(mn2, fminf(a, b));
      mx2 = fmaxf(mx2, fmaxf(a, b));
    }
    s.mn[half][t] = mn2; s.mx[half][t] = mx2;
  }
  __syncthreads();
  if (tid < 128) {
    const int t = c;
    const float mnv = fminf(s.mn[0][t], s.mn[1][t]);
    const float mxv = fmaxf(s.mx[0][t], s.mx[1][t]);
    const uint16_t sh = f32_to_f16_bits(__fdiv_rn(__fsub_rn(mxv, mnv), 3.0f));
    const uint16_t zh = f32_to_f16_bits(mnv);
    // kept in position order: position p holds token 16*(p%8) + p/8
    const int p = 8 * (t & 15) + (t >> 4);
    s.inv[p] = inv_scale(f16_bits_to_f32(sh));
    s.zr[p] = f16_bits_to_f32(zh);
    reinterpret_cast<uint16_t*>(rec + R::vs)[p] = sh;
    reinterpret_cast<uint16_t*>(rec + R::vz)[p] = zh;
  }
  __syncthreads();
  if (act) {
    const int q = tid >> 6, lane = tid & 63;
    uint32_t w[4];
#pragma unroll
    for (int vsel = 0; vsel < 2; ++vsel) {
      const int wv = 4 * vsel + (lane >> 4);
      float inv[16], zr[16];
#pragma unroll
      for (int a4 = 0; a4 < 4; ++a4) {
        const float4 i4 = *reinterpret_cast<const float4*>(&s.inv[16 * wv + 4 * a4]);
        const float4 z4 = *reinterpret_cast<const float4*>(&s.zr[16 * wv + 4 * a4]);
        inv[4 * a4] = i4.x; inv[4 * a4 + 1] = i4.y; inv[4 * a4 + 2] = i4.z; inv[4 * a4 + 3] = i4.w;
        zr[4 * a4] = z4.x; zr[4 * a4 + 1] = z4.y; zr[4 * a4 + 2] = z4.z; zr[4 * a4 + 3] = z4.w;
      }
#pragma unroll
      for (int dsel = 0; dsel < 2; ++dsel) {
        const int d = 32 * q + 16 * dsel + (lane & 15);
        Pack16 pk;
#pragma unroll
        for (int a = 0; a < 16; ++a) {
          const int p = 16 * wv + a;
          const int t = 16 * (p & 7) + (p >> 3);
          pk.put(a, qcode_bits(tile_elem(s, t, d), inv[a], zr[a], 3.0f));
        }
        w[2 * dsel + vsel] = pk.low();
      }
    }
    reinterpret_cast<uint4*>(rec + R::vd)[64 * q + lane] = make_uint4(w[0], w[1], w[2], w[3]);
  }
  __syncthreads();   // the tile and the window rows may be overwritten by the caller after this
}

struct QuantPagesParams {
  const uint16_t* k_src;
  const uint16_t* v_src;
  int64_t page_stride, head_stride, token_stride;
  const int64_t* src_page_offsets;
  const int32_t* dst_page_ids;
  uint8_t* pool;
  int32_t n_kv_heads, n_pool_pages, rank_metric;
};

template <int NB16>
__global__ __launch_bounds__(256, 4) void quantize_pages_kernel(QuantPagesParams p) {
  __shared__ QuantSmem smem;
  const int i = blockIdx.x, h = blockIdx.y;
  const int32_t pid = p.dst_page_ids[i];
  if (pid < 0 || pid >= p.n_pool_pages) return;
  const int64_t off = (p.src_page_offsets ? p.src_page_offsets[i] : (int64_t)i * p.page_stride) + (int64_t)h * p.head_stride;
  uint8_t* rec = p.pool + ((size_t)pid * p.n_kv_heads + h) * (size_t)Rec<NB16>::bytes;
  quantize_page<NB16>(smem, p.k_src + off, p.v_src + off, p.token_stride, rec, p.rank_metric);
}

struct AppendParams {
  uint8_t* pool;
  int32_t* page_table;
  int32_t* n_pages;
  uint16_t* resid_k;
  uint16_t* resid_v;
  int32_t* n_resid;
  uint16_t* sink_k;
  uint16_t* sink_v;
  int32_t* n_sink;
  const uint16_t* k_new;
  const uint16_t* v_new;
  const int32_t* fresh_page_ids;
  int32_t batch, max_pages, n_pool_pages, n_kv_heads, rank_metric;
  int32_t sink_cap;   // S: tokens the Sink holds (0 = none)
  int32_t v_local;    // 1: Value rows live in two halves of G rows, page i's rows in half i & 1
};

// Value rows of the window of (sequence b, kv-head h).  With the Local window the buffer has two halves of G
// rows: the rows of page i (while they are still needed in full precision) and of the tokens that will form
// page i sit in half i & 1, so the half of the page being filled alternates and the previous one stays readable.
__device__ __forceinline__ size_t resid_v_offset(int b, int h, int n_kv_heads, int v_local, int page) {
  const size_t pair = (size_t)b * n_kv_heads + h;
  return v_local ? (pair * 2 + (size_t)(page & 1)) * (size_t)(G * D) : pair * (size_t)(G * D);
}

// Grid (n_kv_heads, batch).  Reads the sequence state, then either stores the new token in the Sink (while
// it is not full), or flushes a full window into a page and stores the new token in the window.  Every head's
// block must see the old state, so the state is advanced by the block of a sequence that finishes last: blocks
// take a ticket in bits 8.. of n_resid[b] (the row count needs bits 0..7) once they are done, and the holder
// of the last ticket writes the new state, which also clears the tickets.
constexpr int TICKET_SHIFT = 8;

template <int NB16>
__global__ __launch_bounds__(256, 4) void append_token_kernel(AppendParams p) {
  __shared__ QuantSmem smem;
  const int h = blockIdx.x, b = blockIdx.y;
  const int nr = p.n_resid[b] & ((1 << TICKET_SHIFT) - 1);
  const int np = p.n_pages[b];
  const int ns = p.sink_cap ? p.n_sink[b] : 0;
  const bool to_sink = ns < p.sink_cap;
  const int32_t pid = p.fresh_page_ids[b];
  const size_t pair = (size_t)b * p.n_kv_heads + h;
  uint16_t* wk = p.resid_k + pair * (size_t)(G * D);
  const bool flush = !to_sink && nr >= G;
  // a flush that cannot happen (page table full, id outside the pool) leaves the sequence unchanged
  const bool ok = !flush || (np >= 0 && np < p.max_pages && pid >= 0 && pid < p.n_pool_pages);
  const int tid = threadIdx.x;
  if (to_sink) {
    if (tid < 32) {
      const int part = tid & 15;
      const uint16_t* src = (tid < 16 ? p.k_new : p.v_new) + pair * D + part * 8;
      uint16_t* dst = (tid < 16 ? p.sink_k : p.sink_v) + (pair * p.sink_cap + ns) * D + part * 8;
      *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
    }
  } else if (ok) {
    int slot = nr;
    uint16_t* wv = p.resid_v + resid_v_offset(b, h, p.n_kv_heads, p.v_local, np);
    if (flush) {
      uint8_t* rec = p.pool + ((size_t)pid * p.n_kv_heads + h) * (size_t)Rec<NB16>::bytes;
      quantize_page<NB16>(smem, wk, wv, D, rec, p.rank_metric);
      slot = 0;
      wv = p.resid_v + resid_v_offset(b, h, p.n_kv_heads, p.v_local, np + 1);
    }
    if (tid < 32) {
      const int part = tid & 15;
      const uint16_t* src = (tid < 16 ? p.k_new : p.v_new) + pair * D + part * 8;
      uint16_t* dst = (tid < 16 ? wk : wv) + (size_t)slot * D + part * 8;
      *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
    }
  }
  __syncthreads();   // every thread of the block has read the old state
  if (tid == 0) {
    const int old = atomicAdd(&p.n_resid[b], 1 << TICKET_SHIFT);
    if ((old >> TICKET_SHIFT) == p.n_kv_heads - 1) {   // every block of this sequence has read the state
      int new_nr = nr;
      if (to_sink) {
        p.n_sink[b] = ns + 1;
      } else if (ok) {
        if (flush) {
          p.page_table[(size_t)b * p.max_pages + np] = pid;
          p.n_pages[b] = np + 1;
          new_nr = 1;
        } else {
          new_nr = nr + 1;
        }
      }
      atomicExch(&p.n_resid[b], new_nr);
    }
  }
}

}  // namespace kitty
