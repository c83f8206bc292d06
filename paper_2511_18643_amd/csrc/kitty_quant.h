// Page quantizer: one workgroup of 256 threads turns G=128 tokens of one kv-head into a record.
// Sec. 2.1 (per-channel K / per-token V asymmetric quantization), Sec. 3.2 Eq. (2) (channel
// score and top-K boost), Sec. 4.1 (dense low-bit plane + compact high-bit plane + index list).
#pragma once
#include "kitty_common.h"

namespace kitty {

// Work split of the 256 threads: thread (wave, g, part) = (tid >> 6, (tid >> 4) & 3, tid & 15) holds, for both
// the Key and the Value page, the eight channels 8*part..8*part+7 of the eight tokens 4*wave + g + 16*i (i < 8),
// in registers, straight from its eight 16-byte loads.  Per-channel statistics are reduced over i in the thread
// and over the 16 (wave, g) classes through LDS; per-token statistics over the 16 lanes of a row with DPP.  The
// tokens of a thread are the positions 8*(4*wave + g) + i of the Value plane, i.e. half a packed word per
// channel, and its channels are half a packed word of the dense Key plane per token: the other half sits in a
// neighbouring lane (lane ^ 16, lane ^ 1).  Packed words are staged in LDS and stored as one 16-byte piece per
// thread, which is exactly what a decode lane reads back.
struct QuantSmem {
  union {
    struct {                 // per (wave, g) partial statistics of the Key page
      float mn[16][D];
      float mx[16][D];
      double sum[16][D];
    } st;
    struct {
      uint8_t codes[G][D + 4];   // 4-bit Key codes [token][channel] for the boost-plane pass (rows 33 dwords apart:
                                 // the pass reads one channel of 64 tokens at a time)
      uint32_t kout[1024];   // dense Key plane as it goes to memory
      uint32_t vout[1024];   // Value plane as it goes to memory
      uint32_t vout_hi[1024];  // high Value plane (4-bit Values only)
    } pk;
  };
  double score[D];
  float keyf[D];             // score rounded to fp32
  int32_t rk[2][D];          // partial rank counts
  float inv[D];              // per channel: 1 / float(fp16 scale) (0 if the scale is 0)
  float zr[D];               // float(fp16 zero-point)
  float qm[D];               // 15 or 3
  float vinv[G];             // per token, index 8*(4*wave + g) + i
  float vzr[G];
  unsigned long long ballot0, ballot1;
  uint8_t chl[D];
};

// code = clamp(rint((x - zero) * inv), 0, qmax), inv = 1/scale rounded once (IEEE), 0 for a zero scale.
// fp32 subtract and multiply, ties to even; with inv == 0 every code is 0.
// qcode_bits returns the raw bits of clamp((x - zero) * inv, 0, qmax) + 1.5 * 2^23: the addition rounds to
// the nearest integer, ties to even, and leaves that integer in the low byte (clamping first gives the same
// integer as rounding first, because the bounds are integers).
__device__ __forceinline__ uint32_t qcode_bits(float x, float inv, float z, float qmax) {
  const float f = __builtin_amdgcn_fmed3f(__fmul_rn(__fsub_rn(x, z), inv), 0.0f, qmax);
  return __float_as_uint(__fadd_rn(f, 12582912.0f));
}
__device__ __forceinline__ float inv_scale(float s) { return s > 0.0f ? __fdiv_rn(1.0f, s) : 0.0f; }

// low bytes of a, b, c, d -> one word (a in byte 0)
__device__ __forceinline__ uint32_t low_bytes(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  const uint32_t lo = __builtin_amdgcn_perm(b, a, 0x0c0c0400u);
  const uint32_t hi = __builtin_amdgcn_perm(d, c, 0x0c0c0400u);
  return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
}

// Eight bf16 values of a 16-byte piece, widened.
__device__ __forceinline__ void widen8(const uint4& v, float (&x)[8]) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    x[2 * k] = __uint_as_float(w[k] << 16);
    x[2 * k + 1] = __uint_as_float(w[k] & 0xffff0000u);
  }
}

// Dword index inside a 4 KB packed plane of the word with row index r (token for Keys, channel for Values) and
// word index cw (channel block for Keys, position block for Values): byte 1024*(r/32) + 16*((r%16) + 16*(cw%4))
// + 4*(2*((r/16)%2) + cw/4), divided by four.
__device__ __forceinline__ int plane_word(int r, int cw) {
  return 4 * (64 * (r >> 5) + 16 * (cw & 3) + (r & 15)) + 2 * ((r >> 4) & 1) + (cw >> 2);
}

// src: bf16 rows of 128 channels, row t at src + t*token_stride (elements), 16-byte aligned.
// STREAM: the source is read once (batch quantization): non-temporal loads.
struct TileRegs { uint4 v[8]; };
template <bool STREAM>
__device__ __forceinline__ void fetch_tile(TileRegs& r, const uint16_t* __restrict__ src, int64_t token_stride, int tid) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int t = (tid >> 4) + 16 * i, part = tid & 15;
    const uint16_t* at = src + (int64_t)t * token_stride + part * 8;
    if constexpr (STREAM) {
      typedef unsigned int v4u __attribute__((ext_vector_type(4)));
      const v4u x = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(at));
      r.v[i] = make_uint4(x.x, x.y, x.z, x.w);
    } else {
      r.v[i] = *reinterpret_cast<const uint4*>(at);
    }
  }
}

// Stores of the code planes.  STREAM marks them non-temporal: a prefill-sized batch of records is not read again
// soon, and written that way the same traffic is served ~5 % faster (measured on the bare load/store pattern and
// on the kernel); a flush inside a decode step reads its record back at once and keeps ordinary stores.
template <bool STREAM>
__device__ __forceinline__ void plane_store16(uint8_t* dst, const uint4& v) {
  if constexpr (STREAM) {
    typedef unsigned int v4u __attribute__((ext_vector_type(4)));
    const v4u x = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(x, reinterpret_cast<v4u*>(dst));
  } else {
    *reinterpret_cast<uint4*>(dst) = v;
  }
}
template <bool STREAM>
__device__ __forceinline__ void plane_store4(uint8_t* dst, uint32_t v) {
  if constexpr (STREAM) __builtin_nontemporal_store(v, reinterpret_cast<uint32_t*>(dst));
  else *reinterpret_cast<uint32_t*>(dst) = v;
}

// One block of at least 256 threads; threads 0..255 do the work, every thread takes part in the barriers.
// Both source pages are read into registers before the first barrier and never touched again.
template <int NB16, bool V4 = false, bool STREAM = false>
__device__ __forceinline__ void quantize_page(QuantSmem& s, const uint16_t* __restrict__ ksrc, const uint16_t* __restrict__ vsrc,
                                              int64_t token_stride, uint8_t* __restrict__ rec, int rank_metric) {
  using R = Rec<NB16, V4>;
  constexpr float VQMAX = V4 ? 15.0f : 3.0f;
  const int tid = threadIdx.x;
  const bool act = tid < 256;
  const int c = tid & 127;
  const int part = tid & 15, cls = (tid >> 4) & 15;   // cls = 4*wave + g: tokens cls + 16*i, positions 8*cls + i
  TileRegs kq, vq;
  if (act) {
    fetch_tile<STREAM>(kq, ksrc, token_stride, tid);
    fetch_tile<STREAM>(vq, vsrc, token_stride, tid);
  }

  // ---------------- Key page: per-channel min, max, sum |x| ----------------
  if (act) {
    float mn[8], mx[8];
    double sum[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) { mn[k] = INFINITY; mx[k] = -INFINITY; sum[k] = 0.0; }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float x[8];
      widen8(kq.v[i], x);
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        mn[k] = fminf(mn[k], x[k]);
        mx[k] = fmaxf(mx[k], x[k]);
        sum[k] += (double)fabsf(x[k]);   // exact for bf16 inputs: the order of the additions does not matter
      }
    }
    *reinterpret_cast<float4*>(&s.st.mn[cls][8 * part]) = make_float4(mn[0], mn[1], mn[2], mn[3]);
    *reinterpret_cast<float4*>(&s.st.mn[cls][8 * part + 4]) = make_float4(mn[4], mn[5], mn[6], mn[7]);
    *reinterpret_cast<float4*>(&s.st.mx[cls][8 * part]) = make_float4(mx[0], mx[1], mx[2], mx[3]);
    *reinterpret_cast<float4*>(&s.st.mx[cls][8 * part + 4]) = make_float4(mx[4], mx[5], mx[6], mx[7]);
#pragma unroll
    for (int k = 0; k < 8; k += 2) *reinterpret_cast<double2*>(&s.st.sum[cls][8 * part + k]) = make_double2(sum[k], sum[k + 1]);
  }
  __syncthreads();
  float mn = 0.f, mx = 0.f;
  if (tid < 128) {
    mn = INFINITY; mx = -INFINITY;
    double sum = 0.0;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      mn = fminf(mn, s.st.mn[r][c]);
      mx = fmaxf(mx, s.st.mx[r][c]);
      sum += s.st.sum[r][c];
    }
    const double sc = rank_metric == 0 ? sum : (double)__fsub_rn(mx, mn);
    s.score[c] = sc;
    s.keyf[c] = (float)sc;     // round to nearest: monotone
  }
  __syncthreads();
  // Boosted set = the 16*NB16 channels that come first under (score descending, channel ascending).  Fast
  // path: count, per channel, the channels whose score rounded to fp32 is strictly larger (rounding is
  // monotone, so a strictly larger fp32 key means a strictly larger score; both halves of the block take 64
  // candidates each).  Channels with equal fp32 keys get equal counts; membership in the set is still decided
  // correctly unless such a group straddles the boundary, and then more than 16*NB16 channels pass the test:
  // in that case only, the exact comparison on the fp64 scores is run.
  constexpr int KB = 16 * NB16;
  if (act) {
    const float my = s.keyf[c];
    const int o0 = (tid >> 7) * 64;
    int cnt = 0;
    for (int o = o0; o < o0 + 64; ++o) cnt += s.keyf[o] > my;
    s.rk[tid >> 7][c] = cnt;
  }
  __syncthreads();
  bool boosted = false;
  if (tid < 128) boosted = s.rk[0][c] + s.rk[1][c] < KB;
  unsigned long long bal = __ballot(boosted);
  if (tid == 0) s.ballot0 = bal;
  if (tid == 64) s.ballot1 = bal;
  __syncthreads();
  if (__popcll(s.ballot0) + __popcll(s.ballot1) != KB) {   // same for every thread of the block
    __syncthreads();                                       // everybody has read the ballots
    if (tid < 128) {
      const double my = s.score[c];
      int rank = 0;
      for (int o = 0; o < 128; ++o) {
        double so = s.score[o];
        rank += (so > my) || (so == my && o < c);
      }
      boosted = rank < KB;
    }
    bal = __ballot(boosted);
    if (tid == 0) s.ballot0 = bal;
    __syncthreads();
  }
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
  __syncthreads();   // (also: everybody is done with the partial statistics, whose memory the codes reuse)

  // ---------------- Key codes: half a dense word per token and thread ----------------
  if (act) {
    float inv[8], zr[8], qm[8];
    {
      const float4 i0 = *reinterpret_cast<const float4*>(&s.inv[8 * part]), i1 = *reinterpret_cast<const float4*>(&s.inv[8 * part + 4]);
      const float4 z0 = *reinterpret_cast<const float4*>(&s.zr[8 * part]), z1 = *reinterpret_cast<const float4*>(&s.zr[8 * part + 4]);
      const float4 q0 = *reinterpret_cast<const float4*>(&s.qm[8 * part]), q1 = *reinterpret_cast<const float4*>(&s.qm[8 * part + 4]);
      inv[0] = i0.x; inv[1] = i0.y; inv[2] = i0.z; inv[3] = i0.w; inv[4] = i1.x; inv[5] = i1.y; inv[6] = i1.z; inv[7] = i1.w;
      zr[0] = z0.x; zr[1] = z0.y; zr[2] = z0.z; zr[3] = z0.w; zr[4] = z1.x; zr[5] = z1.y; zr[6] = z1.z; zr[7] = z1.w;
      qm[0] = q0.x; qm[1] = q0.y; qm[2] = q0.z; qm[3] = q0.w; qm[4] = q1.x; qm[5] = q1.y; qm[6] = q1.z; qm[7] = q1.w;
    }
    const uint32_t sh0 = 4u * (uint32_t)(part & 1);   // elements 8*(part&1)..+7 of the word: bit offsets 2*(a/4)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int t = cls + 16 * i;
      float x[8];
      widen8(kq.v[i], x);
      uint32_t u[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) u[k] = qcode_bits(x[k], inv[k], zr[k], qm[k]);
      const uint32_t r0 = low_bytes(u[0], u[1], u[2], u[3]), r1 = low_bytes(u[4], u[5], u[6], u[7]);
      if constexpr (NB16 > 0) {
        *reinterpret_cast<uint32_t*>(&s.pk.codes[t][8 * part]) = r0;
        *reinterpret_cast<uint32_t*>(&s.pk.codes[t][8 * part + 4]) = r1;
      }
      const uint32_t half = ((r0 & 0x03030303u) | ((r1 & 0x03030303u) << 2)) << sh0;
      const uint32_t other = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)half, 0xB1, 0xf, 0xf, true);   // lane ^ 1
      if ((part & 1) == 0) s.pk.kout[plane_word(t, part >> 1)] = half | other;
    }
  }

  // ---------------- Value page: per-token min, max over the 16 lanes of a row ----------------
  if (act) {
    float tmn[8], tmx[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float x[8];
      widen8(vq.v[i], x);
      float a = fminf(fminf(fminf(x[0], x[1]), fminf(x[2], x[3])), fminf(fminf(x[4], x[5]), fminf(x[6], x[7])));
      float b = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
      a = fminf(a, row_ror<8>(a)); a = fminf(a, row_ror<4>(a)); a = fminf(a, row_ror<2>(a)); a = fminf(a, row_ror<1>(a));
      b = fmaxf(b, row_ror<8>(b)); b = fmaxf(b, row_ror<4>(b)); b = fmaxf(b, row_ror<2>(b)); b = fmaxf(b, row_ror<1>(b));
      tmn[i] = a; tmx[i] = b;
    }
    // lane `part` < 8 of a row finishes token i = part: fp16 scale and zero-point, reciprocal
    float mnv = tmn[0], mxv = tmx[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) { mnv = part == i ? tmn[i] : mnv; mxv = part == i ? tmx[i] : mxv; }
    if (part < 8) {
      const uint16_t sh = f32_to_f16_bits(__fdiv_rn(__fsub_rn(mxv, mnv), VQMAX));
      const uint16_t zh = f32_to_f16_bits(mnv);
      const int p = 8 * cls + part;        // position of token cls + 16*part
      s.vinv[p] = inv_scale(f16_bits_to_f32(sh));
      s.vzr[p] = f16_bits_to_f32(zh);
      reinterpret_cast<uint16_t*>(rec + R::vs)[p] = sh;
      reinterpret_cast<uint16_t*>(rec + R::vz)[p] = zh;
    }
  }
  __syncthreads();   // Key words and codes staged, per-token metadata in place
  if (act) {
    plane_store16<STREAM>(rec + R::kd + 16 * tid, *reinterpret_cast<const uint4*>(&s.pk.kout[4 * tid]));
    if constexpr (NB16 > 0) {   // boost plane: high two bits of the boosted channels, slot order
      for (int idx = tid; idx < 128 * NB16; idx += 256) {
        // word idx % 128 of slot block idx / 128: the inverse of the plane's placement formula (pieces of W words,
        // W = 2 with one slot block, else 4); a wavefront stores 256 consecutive bytes and reads 64 different tokens
        const int sblk = idx >> 7, wi = idx & 127;
        const int t = NB16 == 1 ? 16 * (4 * (wi & 1) + (wi >> 5)) + ((wi >> 1) & 15)
                                : 16 * (4 * (wi >> 6) + (wi & 3)) + ((wi >> 2) & 15);
        uint32_t word = 0;
#pragma unroll
        for (int a = 0; a < 16; ++a) {
          const uint32_t code = s.pk.codes[t][s.chl[16 * sblk + a]];
          word |= (code >> 2) << (8 * (a & 3) + 2 * (a >> 2));
        }
        plane_store4<STREAM>(rec + R::kb + 512 * sblk + 4 * wi, word);
      }
    }
    // ---------------- Value codes: half a word per channel and thread ----------------
    float inv[8], zr[8];
    {
      const float4 i0 = *reinterpret_cast<const float4*>(&s.vinv[8 * cls]), i1 = *reinterpret_cast<const float4*>(&s.vinv[8 * cls + 4]);
      const float4 z0 = *reinterpret_cast<const float4*>(&s.vzr[8 * cls]), z1 = *reinterpret_cast<const float4*>(&s.vzr[8 * cls + 4]);
      inv[0] = i0.x; inv[1] = i0.y; inv[2] = i0.z; inv[3] = i0.w; inv[4] = i1.x; inv[5] = i1.y; inv[6] = i1.z; inv[7] = i1.w;
      zr[0] = z0.x; zr[1] = z0.y; zr[2] = z0.z; zr[3] = z0.w; zr[4] = z1.x; zr[5] = z1.y; zr[6] = z1.z; zr[7] = z1.w;
    }
    uint32_t r0[8], r1[8];   // per channel k: code bytes of tokens i = 0..3 and 4..7
    {
      uint32_t u[4][8];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float x[8];
        widen8(vq.v[i], x);
#pragma unroll
        for (int k = 0; k < 8; ++k) u[i][k] = qcode_bits(x[k], inv[i], zr[i], VQMAX);
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) r0[k] = low_bytes(u[0][k], u[1][k], u[2][k], u[3][k]);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float x[8];
        widen8(vq.v[4 + i], x);
#pragma unroll
        for (int k = 0; k < 8; ++k) u[i][k] = qcode_bits(x[k], inv[4 + i], zr[4 + i], VQMAX);
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) r1[k] = low_bytes(u[0][k], u[1][k], u[2][k], u[3][k]);
    }
    // positions 8*cls + i are elements 8*(cls&1) + i of word cls/2 of the channel; the other half is in lane ^ 16
    const uint32_t sh0 = 4u * (uint32_t)(cls & 1);
    const int wv = cls >> 1;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const uint32_t half = ((r0[k] & 0x03030303u) | ((r1[k] & 0x03030303u) << 2)) << sh0;
      const uint32_t other = (uint32_t)__shfl_xor((int)half, 16);
      if (((cls & 1) == 0) == (k < 4)) s.pk.vout[plane_word(8 * part + k, wv)] = half | other;   // each lane of the pair stores four
      if constexpr (V4) {
        const uint32_t hh = (((r0[k] & 0x0c0c0c0cu) >> 2) | (r1[k] & 0x0c0c0c0cu)) << sh0;
        const uint32_t ho = (uint32_t)__shfl_xor((int)hh, 16);
        if (((cls & 1) == 0) == (k < 4)) s.pk.vout_hi[plane_word(8 * part + k, wv)] = hh | ho;
      }
    }
  }
  __syncthreads();
  if (act) {
    plane_store16<STREAM>(rec + R::vd + 16 * tid, *reinterpret_cast<const uint4*>(&s.pk.vout[4 * tid]));
    if constexpr (V4) plane_store16<STREAM>(rec + R::vh + 16 * tid, *reinterpret_cast<const uint4*>(&s.pk.vout_hi[4 * tid]));
  }
  __syncthreads();   // the shared memory may be reused by the caller after this
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

template <int NB16, bool V4>
__global__ __launch_bounds__(256, 4) void quantize_pages_kernel(QuantPagesParams p) {
  __shared__ QuantSmem smem;
  // one-dimensional grid, heads fastest: the heads of a page run side by side (a token-major source keeps their rows adjacent)
  const int h = blockIdx.x % p.n_kv_heads, i = blockIdx.x / p.n_kv_heads;
  const int32_t pid = p.dst_page_ids[i];
  if (pid < 0 || pid >= p.n_pool_pages) return;
  const int64_t off = (p.src_page_offsets ? p.src_page_offsets[i] : (int64_t)i * p.page_stride) + (int64_t)h * p.head_stride;
  uint8_t* rec = p.pool + ((size_t)pid * p.n_kv_heads + h) * (size_t)Rec<NB16, V4>::bytes;
  quantize_page<NB16, V4, true>(smem, p.k_src + off, p.v_src + off, p.token_stride, rec, p.rank_metric);
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

template <int NB16, bool V4>
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
      uint8_t* rec = p.pool + ((size_t)pid * p.n_kv_heads + h) * (size_t)Rec<NB16, V4>::bytes;
      quantize_page<NB16, V4>(smem, wk, wv, D, rec, p.rank_metric);
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
