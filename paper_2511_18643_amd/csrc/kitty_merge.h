// The merge launches of plans with several page ranges per (sequence, kv-head).  These kernels do not depend on the
// record variant and are compiled once, with the host side of the library.
#pragma once
#include "kitty_decode.h"

namespace kitty {

// Plans with more than 8 ranges merge their partials a chunk of 16 slots at a time: the loads of a chunk are issued
// together, one memory round trip per chunk (a plan with 32 ranges takes two round trips instead of 64 dependent
// ones: 34 -> 23.5 us for one 128k-token sequence).  Plans with up to 8 ranges fetch every slot at once, below.
template <int MERGE_CHUNK>
struct PartialChunk { float m[MERGE_CHUNK], l[MERGE_CHUNK], a[MERGE_CHUNK]; };
// slots s0 .. s0 + MERGE_CHUNK - 1 of one (sequence, query head) for channel d; slots from n_slots on are not touched
template <int MERGE_CHUNK>
__device__ __forceinline__ void load_partials(PartialChunk<MERGE_CHUNK>& c, const float* base, size_t slot_stride, int d, int s0, int n_slots) {
#pragma unroll
  for (int i = 0; i < MERGE_CHUNK; ++i) {
    const bool in = s0 + i < n_slots;
    c.m[i] = in ? base[(size_t)(s0 + i) * slot_stride + D] : -INFINITY;
    c.l[i] = in ? base[(size_t)(s0 + i) * slot_stride + D + 1] : 0.f;
    c.a[i] = in ? base[(size_t)(s0 + i) * slot_stride + d] : 0.f;
  }
}
// folds the chunk's first n_valid slots (those with a finite maximum) into the running (M, a, L)
template <int MERGE_CHUNK>
__device__ __forceinline__ void fold_partials(const PartialChunk<MERGE_CHUNK>& c, int n_valid, float& M, float& a, float& L) {
  float Mc = M;
#pragma unroll
  for (int i = 0; i < MERGE_CHUNK; ++i) Mc = (i < n_valid) ? fmaxf(Mc, c.m[i]) : Mc;
  if (!(Mc > -INFINITY)) return;                    // nothing so far and nothing here
  const float f0 = __builtin_amdgcn_exp2f(M - Mc);  // exp2(-inf) = 0 while nothing has been folded in yet
  a *= f0;
  L *= f0;
#pragma unroll
  for (int i = 0; i < MERGE_CHUNK; ++i) {
    if (i < n_valid && c.m[i] > -INFINITY) {        // slots beyond n_valid hold stale bytes: select, never multiply
      const float f = __builtin_amdgcn_exp2f(c.m[i] - Mc);
      a = fmaf(c.a[i], f, a);
      L = fmaf(c.l[i], f, L);
    }
  }
  M = Mc;
}

// Log-sum-exp merge of the partials of one (sequence, query head); grid (n_q_heads, batch), 128 threads.
// LONG: the plan has more than 8 ranges (a kernel of its own: with both paths in one kernel the short one, which is
// all latency, measured 2 % slower on the 8k workload's step).
template <bool LONG>
__global__ __launch_bounds__(128) void decode_merge_kernel(DecodeParams p) {
  const int hq = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
  const int g = p.gqa, h = hq / g, hd = hq % g;
  const float* base = p.ws + (((size_t)b * p.n_kv_heads + h) * p.n_splits) * (size_t)g * WS_STRIDE + (size_t)hd * WS_STRIDE;
  const size_t slot_stride = (size_t)g * WS_STRIDE;
  float a = 0.f, L = 0.f;
  if constexpr (!LONG) {
    // few ranges: fetch every slot before the sequence state arrives (one memory round trip), then mask
    float m[8], lv[8], av[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const bool in = s < p.n_splits;
      m[s] = in ? base[s * slot_stride + D] : 0.f;
      lv[s] = in ? base[s * slot_stride + D + 1] : 0.f;
      av[s] = in ? base[s * slot_stride + d] : 0.f;
    }
    const int np = page_count(p, b);
    const int r = (p.has_window ? min(p.n_resid[b], G) : 0) + (p.sink_cap ? min(p.n_sink[b], p.sink_cap) : 0);
    const int sb = active_splits(np, r, p.n_splits, p.min_pages);
    float M = -INFINITY;
#pragma unroll
    for (int s = 0; s < 8; ++s) M = s < sb ? fmaxf(M, m[s]) : M;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      if (s < sb) {   // slots beyond sb hold stale bytes: select, never multiply
        const float f = __builtin_amdgcn_exp2f(m[s] - M);
        a = fmaf(av[s], f, a);
        L = fmaf(lv[s], f, L);
      }
    }
  } else {
    PartialChunk<16> c;
    load_partials(c, base, slot_stride, d, 0, p.n_splits);   // requested before the sequence state arrives
    const int np = page_count(p, b);
    const int r = (p.has_window ? min(p.n_resid[b], G) : 0) + (p.sink_cap ? min(p.n_sink[b], p.sink_cap) : 0);
    const int sb = active_splits(np, r, p.n_splits, p.min_pages);
    float M = -INFINITY;
    for (int s0 = 0;;) {
      fold_partials(c, sb - s0, M, a, L);
      s0 += 16;
      if (s0 >= sb) break;
      load_partials(c, base, slot_stride, d, s0, sb);
    }
  }
  const float o = L > 0.f ? a / L : 0.f;
  const size_t oi = ((size_t)b * p.n_q_heads + hq) * D + d;
  if (p.out_dtype == 0) reinterpret_cast<uint16_t*>(p.out)[oi] = f32_to_bf16_rne(o);
  else reinterpret_cast<float*>(p.out)[oi] = o;
}

// The merge launch of a fused step with several ranges: every slot of the workspace holds a partial (neutral ones
// for ranges a sequence does not use), so the merge does not look at the sequence state, and the block of the
// sequence's first query head then does what is left of kitty_append_token: it stores the new token of every
// kv-head and advances the state (the flush, if one was due, was done by the streaming kernel).
template <bool LONG>
__global__ __launch_bounds__(128) void decode_merge_step_kernel(DecodeParams p) {
  const int hq = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
  const int g = p.gqa, h = hq / g, hd = hq % g;
  // the appending block requests what it needs first (the state before the step, which only it reads, and the new
  // token: up to MAXT 16-byte pieces per thread), so that those round trips overlap the merge
  constexpr int MAXT = 4;                          // 128 threads x 4 pieces = 16 kv-heads per pass
  const bool appender = hq == 0;
  const int pieces = p.n_kv_heads * 32;
  int np_old = 0, nr_old = 0, ns_old = 0;
  int32_t pid = -1;
  uint4 tok[MAXT];
  if (appender) {
    np_old = page_count(p, b);
    nr_old = min(p.n_resid[b], G);
    ns_old = p.sink_cap ? min(p.n_sink[b], p.sink_cap) : 0;
    pid = p.fresh_page_ids[b];
#pragma unroll
    for (int t = 0; t < MAXT; ++t) {
      const int i = d + 128 * t;
      tok[t] = make_uint4(0, 0, 0, 0);
      if (i < pieces) {
        const int hh = i >> 5, part = i & 15, isv = (i >> 4) & 1;
        tok[t] = *reinterpret_cast<const uint4*>((isv ? p.v_new : p.k_new) + ((size_t)b * p.n_kv_heads + hh) * D + part * 8);
      }
    }
  }
  const float* base = p.ws + (((size_t)b * p.n_kv_heads + h) * p.n_splits) * (size_t)g * WS_STRIDE + (size_t)hd * WS_STRIDE;
  const size_t slot_stride = (size_t)g * WS_STRIDE;
  float a = 0.f, L = 0.f;
  if constexpr (!LONG) {     // few ranges: one round trip for every slot
    float m[8], lv[8], av[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const bool in = s < p.n_splits;
      m[s] = in ? base[s * slot_stride + D] : -INFINITY;
      lv[s] = in ? base[s * slot_stride + D + 1] : 0.f;
      av[s] = in ? base[s * slot_stride + d] : 0.f;
    }
    float M = -INFINITY;
#pragma unroll
    for (int s = 0; s < 8; ++s) M = fmaxf(M, m[s]);
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      if (m[s] > -INFINITY) {
        const float f = __builtin_amdgcn_exp2f(m[s] - M);
        a = fmaf(av[s], f, a);
        L = fmaf(lv[s], f, L);
      }
    }
  } else {
    float M = -INFINITY;
    for (int s0 = 0; s0 < p.n_splits; s0 += 16) {
      PartialChunk<16> c;
      load_partials(c, base, slot_stride, d, s0, p.n_splits);
      fold_partials(c, p.n_splits - s0, M, a, L);
    }
  }
  const float o = L > 0.f ? a / L : 0.f;
  const size_t oi = ((size_t)b * p.n_q_heads + hq) * D + d;
  if (p.out_dtype == 0) reinterpret_cast<uint16_t*>(p.out)[oi] = f32_to_bf16_rne(o);
  else reinterpret_cast<float*>(p.out)[oi] = o;

  if (!appender) return;
  const bool to_sink = ns_old < p.sink_cap;
  const bool flush = !to_sink && nr_old >= G;
  const bool ok = !flush || (np_old < p.max_pages && pid >= 0 && pid < p.n_pool_pages);
  __syncthreads();                                 // every thread of the block has read the old state
  if (!to_sink && !ok) return;                     // no page for a full window: the token is dropped, as in kitty_append_token
  const int np_new = np_old + (flush ? 1 : 0);
  const int row = to_sink ? ns_old : (flush ? 0 : nr_old);
  for (int i0 = 0; i0 < pieces; i0 += 128 * MAXT) {
#pragma unroll
    for (int t = 0; t < MAXT; ++t) {
      const int i = i0 + d + 128 * t;
      if (i >= pieces) continue;
      const int hh = i >> 5, part = i & 15, isv = (i >> 4) & 1;
      const size_t pr = (size_t)b * p.n_kv_heads + hh;
      const uint4 val = i0 == 0 ? tok[t] : *reinterpret_cast<const uint4*>((isv ? p.v_new : p.k_new) + pr * D + part * 8);
      uint16_t* dst;
      if (to_sink) dst = (isv ? p.sink_v_w : p.sink_k_w) + (pr * p.sink_cap + row) * D;
      else dst = isv ? p.resid_v_w + resid_v_offset(b, hh, p.n_kv_heads, p.v_local, np_new) + (size_t)row * D
                     : p.resid_k_w + pr * (size_t)(G * D) + (size_t)row * D;
      *reinterpret_cast<uint4*>(dst + part * 8) = val;
    }
  }
  if (d == 0) {
    if (to_sink) {
      p.n_sink_w[b] = ns_old + 1;
    } else {
      if (flush) {
        p.page_table_w[(size_t)b * p.max_pages + np_old] = pid;
        p.n_pages_w[b] = np_old + 1;
      }
      p.n_resid_w[b] = flush ? 1 : nr_old + 1;
    }
  }
}

}  // namespace kitty
