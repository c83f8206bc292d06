// Split-K decode attention read directly from packed records (Sec. 4.3 step 2; Alg. 1; Eq. 1).
//
// One wavefront owns one page at a time and never synchronises with the others inside the loop.
// Dequantization is folded out of the inner products (Alg. 1: K = X*scale + zero):
//     q . K_t      = sum_c (q_c s_c) X[t][c] + sum_c q_c z_c
//     sum_t p_t V_t = sum_t (p_t s_t) X[t][:] + sum_t p_t z_t
// so the 2-bit codes X go to the int8 matrix cores unchanged (mask/shift into bytes), while the
// small vectors q*s and p*s are turned into three signed-byte terms (n = t0 + 256 t1 + 65536 t2)
// occupying separate matrix rows; the integer dot products are exact and are recombined by shifts.
// The high bits of boosted channels are one more short contraction against the same q*s values
// gathered through the channel list (the only gather, and it is of q, never of cache bytes).
#pragma once
#include <climits>
#include <cstddef>
#include <type_traits>

#include "kitty_common.h"
#include "kitty_quant.h"

// Byte terms of the fixed-point images in the kernels for eight-head groups (2 or 3; see PageWorker).
#ifndef KITTY_G8_KEY_TERMS
#define KITTY_G8_KEY_TERMS 3
#endif
#ifndef KITTY_G8_VALUE_TERMS
#define KITTY_G8_VALUE_TERMS 3
#endif

namespace kitty {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

constexpr int WS_STRIDE = D + 2;   // floats per partial: acc[128], running max (log2 domain), weight sum

struct DecodeParams {
  const uint8_t* pool;
  const int32_t* page_table;
  const int32_t* n_pages;
  const uint16_t* resid_k;
  const uint16_t* resid_v;
  const int32_t* n_resid;
  const uint16_t* sink_k;   // bf16 [batch][n_kv_heads][sink_cap][D], the first tokens of every sequence (Fig. 1: Sink)
  const uint16_t* sink_v;
  const int32_t* n_sink;
  const int32_t* seq_order;  // optional permutation: block z serves sequence seq_order[z]
  const uint16_t* q;
  float* ws;
  void* out;
  float qk_scale_log2;   // sm_scale * log2(e)
  int32_t batch, max_pages, n_q_heads, n_kv_heads, gqa;
  int32_t n_splits, min_pages, has_window, out_dtype;
  int32_t direct_out;    // split kernel with n_splits == 1: normalise and store `out` itself, no partials
  int32_t sink_cap;      // S (0 = no Sink)
  int32_t v_local;       // 1: the Values of the newest page are read from the bf16 Local window, not from its record
  // fused step (append, then attention, one launch; only with one range per sequence and kv-head)
  const uint16_t* k_new;
  const uint16_t* v_new;
  const int32_t* fresh_page_ids;
  uint8_t* pool_w;
  int32_t* page_table_w;
  int32_t* n_pages_w;
  uint16_t* resid_k_w;
  uint16_t* resid_v_w;
  int32_t* n_resid_w;
  uint16_t* sink_k_w;
  uint16_t* sink_v_w;
  int32_t* n_sink_w;
  int32_t n_pool_pages, rank_metric;
};

// Packed pages of sequence b as the kernels use it (a count outside [0, max_pages], or pages without a pool,
// can only come from a corrupted state and is folded into the valid range).
__device__ __forceinline__ int page_count(const DecodeParams& p, int b) {
  return p.n_pool_pages > 0 ? max(min(p.n_pages[b], p.max_pages), 0) : 0;
}

// Page ranges of one sequence: with np pages and r full-precision rows (Sink + window), the sequence uses
// Sb = min(n_splits, max(1, np / min_pages)) ranges (one if it only has such rows, none if it is empty);
// range s covers pages [s*np/Sb, (s+1)*np/Sb) and full-precision rows [s*r/Sb, (s+1)*r/Sb).
__device__ __forceinline__ int active_splits(int np, int r, int n_splits, int min_pages) {
  if (np <= 0) return r > 0 ? 1 : 0;
  return min(n_splits, max(1, np / min_pages));
}

// One page's code planes as they sit in a lane's registers.  The four fp16 arrays travel separately: lane
// group 0 fetches k_scale, 1 k_zero, 2 v_scale, 3 v_zero (entries 8j..8j+7 each) and the groups exchange
// them through LDS.
// How the boost plane (16*NB16 slots per token) meets the 64-deep contraction of a matrix instruction.  P slot
// blocks of 16 sit side by side in an operand's four k-blocks; with P < 4 the other k-blocks carry the same slot
// blocks of F - 1 further token tiles, and the tile is chosen by zeroing the query-side operand in the k-blocks of
// the others.  More than 64 slots take KG operands per tile.  Lane (j, k-block kb) holds, per operand, slot block
// kb % P (+ 4 per further operand) of the WPG token tiles WPG * (kb / P) + v (P = 1: tiles kb and 4 + kb): words
// that are contiguous in the record.
template <int NB16>
struct BoostShape {
  static constexpr int P = NB16 <= 1 ? 1 : (NB16 == 2 ? 2 : 4);
  static constexpr int F = 4 / P;
  static constexpr int KG = NB16 > 4 ? 2 : 1;
  static constexpr int WPG = 2 * P;                      // words per lane and operand (8 token tiles / F)
  static constexpr int WORDS = NB16 ? WPG * KG : 1;
  static constexpr int COLS = NB16 == 0 ? 16 : (NB16 <= 2 ? 16 * NB16 : 64 * KG);   // slot columns of the query-side operand
  // token tile of word v of a lane whose k-block belongs to tile class f
  static constexpr int tile(int f, int v) { return P == 1 ? 4 * v + f : WPG * f + v; }
};

template <int NB16, bool V4 = false>
struct PageRegs {
  uint4 kd[4];
  uint32_t kbw[BoostShape<NB16>::WORDS];   // boost plane, see BoostShape
  uint32_t chv[NB16 ? NB16 : 1];
  uint4 vd[4];
  uint4 vh[V4 ? 4 : 1];   // high Value plane (4-bit Values)
};

// Byte offsets of a lane into a record (32-bit, so loads take the scalar record base + one VGPR offset).
struct LaneOffsets {
  uint32_t o16, j, meta;
  uint32_t ob[2];   // the lane's words of the boost plane, per operand; beyond the record (reads as zeros) if it has none
};
template <int NB16, bool V4>
__device__ __forceinline__ LaneOffsets lane_offsets(int l) {
  using R = Rec<NB16, V4>;
  using BS = BoostShape<NB16>;
  const uint32_t j = l & 15, gi = l >> 4;
  const uint32_t base = gi == 0 ? R::ks : (gi == 1 ? R::kz : (gi == 2 ? R::vs : R::vz));
  LaneOffsets o{(uint32_t)l * 16u, j, base + 16u * j, {0u, 0u}};
  constexpr uint32_t NONE = 0x40000000u;
  if constexpr (BS::P == 1) {          // tiles kb and 4 + kb: 8 bytes, lanes in order
    o.ob[0] = R::kb + 8u * (uint32_t)l;
  } else if constexpr (BS::P == 2) {   // slot block kb % 2, tiles 4*(kb/2) .. +3: 16 bytes
    o.ob[0] = R::kb + 512u * (gi & 1u) + 256u * (gi >> 1) + 16u * j;
  } else {                             // slot block 4q + kb, all eight tiles: two pieces of 16 bytes, 256 apart
#pragma unroll
    for (int q = 0; q < BS::KG; ++q) o.ob[q] = (4 * q + (int)gi < NB16) ? R::kb + 512u * (4u * q + gi) + 16u * j : NONE;
  }
  return o;
}

// A page is fetched in three pieces: the lane's 16 bytes of fp16 arrays, the Key planes (+ channel list), the
// Value plane.  Each piece of the next page is requested as soon as the registers of the current one are dead.
// Records are addressed through a buffer resource (base = the record, size = its bytes): the loads take the
// scalar descriptor, one 32-bit lane offset and a constant, so no vector address arithmetic is needed (and an
// offset beyond the record would read zeros instead of foreign memory).
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));
using RecRef = __amdgpu_buffer_rsrc_t;
template <int NB16, bool V4>
__device__ __forceinline__ RecRef rec_ref(const uint8_t* rec) {
  // word 3 of a gfx9-family raw buffer descriptor: 32-bit data format, no swizzle, range-checked by byte offset
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(rec), 0, Rec<NB16, V4>::bytes, 0x00020000);
}
// Records are read once per step: the loads carry the non-temporal hint (cache policy bit 1 of the buffer
// instructions), which alone raises the streaming rate of the 32k workload by 6 % (113 -> 107 us).
#ifndef KITTY_LD_AUX
#define KITTY_LD_AUX 2
#endif
constexpr int REC_LOAD_POLICY = KITTY_LD_AUX;
__device__ __forceinline__ uint4 buf_load16(RecRef r, uint32_t voff, int soff) {
  const v4u v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, REC_LOAD_POLICY);
  return make_uint4(v.x, v.y, v.z, v.w);
}
template <int NB16>
__device__ __forceinline__ uint4 load_meta(RecRef rec, const LaneOffsets& o) {
  return buf_load16(rec, o.meta, 0);
}
template <int NB16, bool V4>
__device__ __forceinline__ void load_k(PageRegs<NB16, V4>& r, RecRef rec, const LaneOffsets& o) {
  using R = Rec<NB16, V4>;
#pragma unroll
  for (int i = 0; i < 4; ++i) r.kd[i] = buf_load16(rec, o.o16, R::kd + 1024 * i);
  using BS = BoostShape<NB16>;
  if constexpr (NB16 > 0) {
    if constexpr (BS::P == 1) {
      const v2u v = __builtin_amdgcn_raw_buffer_load_b64(rec, o.ob[0], 0, REC_LOAD_POLICY);
      r.kbw[0] = v.x; r.kbw[1] = v.y;
    } else if constexpr (BS::P == 2) {
      const uint4 v = buf_load16(rec, o.ob[0], 0);
      r.kbw[0] = v.x; r.kbw[1] = v.y; r.kbw[2] = v.z; r.kbw[3] = v.w;
    } else {
#pragma unroll
      for (int q = 0; q < BS::KG; ++q) {
        const uint4 v0 = buf_load16(rec, o.ob[q], 0), v1 = buf_load16(rec, o.ob[q], 256);
        r.kbw[8 * q + 0] = v0.x; r.kbw[8 * q + 1] = v0.y; r.kbw[8 * q + 2] = v0.z; r.kbw[8 * q + 3] = v0.w;
        r.kbw[8 * q + 4] = v1.x; r.kbw[8 * q + 5] = v1.y; r.kbw[8 * q + 6] = v1.z; r.kbw[8 * q + 7] = v1.w;
      }
    }
  }
#pragma unroll
  for (int s = 0; s < NB16; ++s) r.chv[s] = __builtin_amdgcn_raw_buffer_load_b8(rec, o.j, R::ch + 16 * s, 0);
}
template <int NB16, bool V4>
__device__ __forceinline__ void load_v(PageRegs<NB16, V4>& r, RecRef rec, const LaneOffsets& o) {
  using R = Rec<NB16, V4>;
#pragma unroll
  for (int i = 0; i < 4; ++i) r.vd[i] = buf_load16(rec, o.o16, R::vd + 1024 * i);
  if constexpr (V4) {
#pragma unroll
    for (int i = 0; i < 4; ++i) r.vh[i] = buf_load16(rec, o.o16, R::vh + 1024 * i);
  }
}

// sixteen 2-bit elements -> four registers of four int8 each (elements 4v..4v+3 in register v)
__device__ __forceinline__ v4i unpack16(uint32_t w) {
  v4i r;
  r.x = (int)(w & 0x03030303u);
  r.y = (int)((w >> 2) & 0x03030303u);
  r.z = (int)((w >> 4) & 0x03030303u);
  r.w = (int)((w >> 6) & 0x03030303u);
  return r;
}
// cheaper variant (one shift, four masks): elements 4..7 and 12..15 come out multiplied by 4; the other
// operand carries the inverse weights
__device__ __forceinline__ v4i unpack16_w(uint32_t w) {
  v4i r;
  const uint32_t t = w >> 4;
  r.x = (int)(w & 0x03030303u);
  r.y = (int)(w & 0x0c0c0c0cu);
  r.z = (int)(t & 0x03030303u);
  r.w = (int)(t & 0x0c0c0c0cu);
  return r;
}
// same, each element multiplied by 4 (the weight of the high bits of a 4-bit code)
__device__ __forceinline__ v4i unpack16_x4(uint32_t w) {
  v4i r;
  r.x = (int)((w << 2) & 0x0c0c0c0cu);
  r.y = (int)(w & 0x0c0c0c0cu);
  r.z = (int)((w >> 2) & 0x0c0c0c0cu);
  r.w = (int)((w >> 4) & 0x0c0c0c0cu);
  return r;
}

// byte K of a, b, c, d -> one word (a in byte 0)
template <int K>
__device__ __forceinline__ uint32_t gather_byte(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  constexpr uint32_t sel = 0x0c0c0000u | ((4u + K) << 8) | (uint32_t)K;
  const uint32_t lo = __builtin_amdgcn_perm(b, a, sel);
  const uint32_t hi = __builtin_amdgcn_perm(d, c, sel);
  return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
}

// Integer images are kept as the raw bits of (x + 1.5*2^23): for |x| < 2^22 the low 23 bits hold
// 2^22 + round(x), so byte 0 of the bits is byte 0 of n = round(x), and the carries of the balanced
// byte split (n = t0 + 256 t1 + 65536 t2, each t in [-128,127]) are single adds on the same bits.
constexpr float MAGIC = 12582912.0f;            // 1.5 * 2^23 = 0x4b400000
constexpr uint32_t T1_ADD = 0x80u;              // byte 1 of (bits + 0x80)            = t1
// Three terms: the carries are added in the float domain, for free, by rounding with the constant 1.5*2^23 + 0x8080
// instead: the bits are then v = 0x4b408080 + n, and with |n| < 2^20 - 0x8080
//     t0 = byte 0 of v, top bit flipped        t1 = byte 1 of v, top bit flipped        t2 = byte 2 of v - 0x40.
// Bytes cannot be subtracted without borrows, so the third term is carried as 8 * t2 = (byte 2 << 3) mod 256 (the
// 0x40 becomes 512 and drops out; t2 lies in [-16, 15]) with weight 8192 instead of 65536.
constexpr float MAGIC3 = 12582912.0f + 32896.0f;
constexpr uint32_t MAGIC3_BITS = 0x4b408080u;
constexpr float NLIM3 = 1015000.0f;             // keeps |n| + 0x8080 below 2^20, i.e. t2 within five bits
template <int TR> constexpr float image_magic() { return TR == 3 ? MAGIC3 : MAGIC; }

template <int TR>
__device__ __forceinline__ void split_terms(const uint32_t (&u)[8], uint2 (&w)[TR]) {
  if constexpr (TR == 2) {
    // 16-bit images: the low halves of two values share a register, the carry into the high byte is one packed
    // 16-bit add for both, and each term word is gathered from two such registers
    typedef unsigned short us2 __attribute__((ext_vector_type(2)));
    uint32_t lo[4], up[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      lo[i] = __builtin_amdgcn_perm(u[2 * i + 1], u[2 * i], 0x05040100u);
      const us2 c = __builtin_bit_cast(us2, lo[i]) + (us2){0x80, 0x80};
      up[i] = __builtin_bit_cast(uint32_t, c);
    }
    w[0].x = __builtin_amdgcn_perm(lo[1], lo[0], 0x06040200u);
    w[0].y = __builtin_amdgcn_perm(lo[3], lo[2], 0x06040200u);
    w[1].x = __builtin_amdgcn_perm(up[1], up[0], 0x07050301u);
    w[1].y = __builtin_amdgcn_perm(up[3], up[2], 0x07050301u);
  } else {
    // u holds the bits v (see MAGIC3).  A 4x4 byte transpose per four values: seven byte permutes for the three
    // byte planes, then the fix-ups on whole words.
    uint32_t t[3][2];
#pragma unroll
    for (int hlf = 0; hlf < 2; ++hlf) {
      const uint32_t a = u[4 * hlf], b = u[4 * hlf + 1], c = u[4 * hlf + 2], d = u[4 * hlf + 3];
      const uint32_t lo01 = __builtin_amdgcn_perm(b, a, 0x05010400u);   // a.b0 b.b0 a.b1 b.b1
      const uint32_t lo23 = __builtin_amdgcn_perm(d, c, 0x05010400u);
      const uint32_t hi01 = __builtin_amdgcn_perm(b, a, 0x0c0c0602u);   // a.b2 b.b2 0 0
      const uint32_t hi23 = __builtin_amdgcn_perm(d, c, 0x0c0c0602u);
      t[0][hlf] = __builtin_amdgcn_perm(lo23, lo01, 0x05040100u) ^ 0x80808080u;
      t[1][hlf] = __builtin_amdgcn_perm(lo23, lo01, 0x07060302u) ^ 0x80808080u;
      t[2][hlf] = (__builtin_amdgcn_perm(hi23, hi01, 0x05040100u) << 3) & 0xf8f8f8f8u;
    }
    w[0] = make_uint2(t[0][0], t[0][1]);
    w[1] = make_uint2(t[1][0], t[1][1]);
    w[2] = make_uint2(t[2][0], t[2][1]);
  }
}

// t0 + 256 t1 + 8192 t2x (t2x = 8 t2, see MAGIC3) as two shift-adds (v_lshl_add_u32); the empty asm keeps the
// compiler from re-associating them into two shifts and a three-way add
__device__ __forceinline__ int join_terms(int t0, int t1, int t2x) {
  uint32_t hi = ((uint32_t)t2x << 5) + (uint32_t)t1;
  asm volatile("" : "+v"(hi));
  return (int)((hi << 8) + (uint32_t)t0);
}
__device__ __forceinline__ int join_terms(int t0, int t1) { return (int)(((uint32_t)t1 << 8) + (uint32_t)t0); }

__device__ __forceinline__ void f16x8_to_f32(const uint4& v, float (&f)[8]) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    f[2 * k] = f16_bits_to_f32((uint16_t)(w[k] & 0xffffu));
    f[2 * k + 1] = f16_bits_to_f32((uint16_t)(w[k] >> 16));
  }
}

// x = x * a + b written over x.  The compiler otherwise accumulates into the register of b (the two-operand
// form) and copies the result back for the next loop iteration, one move per running sum and page.  The operands
// must be results of ordinary vector instructions: never of a matrix instruction, of a transcendental one
// (v_exp, v_rcp: a dependent instruction needs a wait state after them) or of a load, because the compiler does
// not track those hazards and waits through inline code.
__device__ __forceinline__ void fma_in_place(float& x, float a, float b) {
  asm("v_fma_f32 %0, %0, %1, %2" : "+v"(x) : "v"(a), "v"(b));
}

__device__ __forceinline__ void wave_lds_fence() {
  // LDS traffic of one wavefront is processed in order; this only stops the compiler from moving
  // a lane's read above another lane's write.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Per-wave LDS scratch.  Rows of the int8 operand matrices are 144 bytes apart so that the
// 16-byte reads of the sixteen rows fall into different banks.
template <int NB16, int HPL>
struct WaveScratch {
  // integer image (raw bits) of q*s per (head, channel), for the boost gather.  The four lane groups gather the same
  // channels from the rows of their own heads at once: the row pitch moves those rows 8 banks apart (a pitch of
  // D words would put all four on the same banks).
  static constexpr int NPITCH = D + (HPL == 1 ? 8 : 4);
  uint32_t nbuf[4 * HPL][NPITCH];
  uint8_t abuf[16 * HPL][144];                         // rows (head, term) x channel; one 16-row matrix per pass
  uint8_t bbuf[16 * HPL][BoostShape<NB16>::COLS + 16];  // rows (head, term) x boost slot (columns of absent slots stay zero)
  uint8_t pbuf[16 * HPL][144];                         // rows (head, term) x position
  float pw[32][8];                               // full-precision rows: softmax weights [row][head]
  float pcorr[8];                                // same path: rescale factor of the running sums per head
  uint8_t meta[4][256];                          // k_scale, k_zero, v_scale, v_zero of the page being processed
  uint8_t zero[16];
};

template <int HPL, int NW>
struct MergeScratch {
  float acc[2 * NW][4 * HPL][D];   // NW wavefronts x {pages, window}
  float m[2 * NW][4 * HPL];
  float l[2 * NW][4 * HPL];
};

template <int NB16, int HPL, int NW, bool FUSED>
union __attribute__((aligned(16))) DecodeSmem {
  WaveScratch<NB16, HPL> w[NW];
  MergeScratch<HPL, NW> mg;
  typename std::conditional<FUSED, QuantSmem, int>::type quant;   // the fused step may flush a window first
};

// Running state of one wavefront on the packed-page path and the work done per page.
// Lane l = (j = l & 15, gi = l >> 4).  In the "compact" role the lane owns channels 8j..8j+7 (K side)
// or positions 8j..8j+7 (V side) of heads gi*HPL + e; in the matrix role it is row/column j of
// k-block gi.  Both roles put head gi*HPL + e in lane group gi, so no cross-group traffic is needed.
//
// With three byte terms the code planes are unpacked with one shift and four masks (unpack16_w), which
// leaves elements 4..7 and 12..15 of a word multiplied by 4.  The compact lane owns elements
// 8*(j&1)..8*(j&1)+7, i.e. its first four values have weight 1 and its last four weight 4; it divides its
// values by that weight before taking the integer image (two bits of the image's precision), and keeps sums
// and maxima of unweighted values by recombining the two halves.
// Groups of eight query heads (HPL == 2): see TRK / TRV below.
template <int NB16, int HPL, bool V4 = false>
struct PageWorker {
  // Byte terms per value of the two fixed-point images: q*scale on the Key side, p*scale on the Value side.
  // Four-head groups carry three terms (20-bit images) in 12 of the 16 matrix rows.  Eight-head groups have room
  // for two terms per head in one matrix (16-bit images); a third term needs 24 rows, i.e. a second MFMA pass over
  // the same code operand.  On the Key side the 16-bit image is not enough: its step is set by the largest
  // |q*scale| of a head, and one dominant query element on an outlier channel coarsens the other 127 channels
  // until the logits are off by 1e-2 (measured: output error up to 1.4e-2 on short contexts, 8e-4 to 1.8e-3 on
  // ordinary data), so both sides carry three terms; KITTY_G8_KEY_TERMS / KITTY_G8_VALUE_TERMS are the compile-time
  // switches the alternatives were measured with.
  static constexpr int TRK = HPL == 1 ? 3 : KITTY_G8_KEY_TERMS;     // byte terms of q*scale
  static constexpr int TRV = HPL == 1 ? 3 : (V4 ? 2 : KITTY_G8_VALUE_TERMS);   // byte terms of p*scale (4-bit Values: no second pass)
  // cheap unpack (one shift, four masks; elements 4..7 and 12..15 of a word come out times 4): relies on the
  // precision of three terms, because the other operand gives up two bits of its image for the inverse weights
  static constexpr bool WEIGHTED_K = TRK == 3, WEIGHTED_V = TRV == 3;
  // weights of the lane's first and last four values (Key side: channels; Value side: tokens) and their log2
  static constexpr float wKA = 1.f, wKB = WEIGHTED_K ? 4.f : 1.f;
  static constexpr float wVA = 1.f, wVB = WEIGHTED_V ? 4.f : 1.f, oVA = 0.f, oVB = WEIGHTED_V ? 2.f : 0.f;
  static constexpr bool TWO_PASS_K = HPL == 2 && TRK == 3, TWO_PASS_V = HPL == 2 && TRV == 3;
  static_assert(!(V4 && TWO_PASS_V), "the high Value plane has no second-pass accumulator");
  static constexpr float NLIM_K = TRK == 3 ? NLIM3 : 32000.0f;   // bound of the integer images
  static constexpr float NLIM_V = TRV == 3 ? NLIM3 : 32000.0f;

  // Matrix row of term t of head hd.  Four heads: rows 4hd + t of one matrix.  Eight heads: terms 0, 1 in
  // rows 2hd + t of the first matrix, term 2 in row 4(hd/2) + hd%2 of a second matrix (rows 16..31) that a
  // second MFMA pass multiplies with the same code operand; either way the terms of heads gi*HPL + e come
  // out in lane group gi.
  static __device__ __forceinline__ int term_row(int hd, int t) {
    if constexpr (HPL == 1) return 4 * hd + t;
    else return t < 2 ? 2 * hd + t : 16 + 4 * (hd >> 1) + (hd & 1);   // t == 2 only with the second pass
  }

  WaveScratch<NB16, HPL>& ws;
  const int j, gi;
  const uint8_t* a_ptr;      // A operand of the logits: row j, k-block gi (second matrix 16 rows further)
  const uint8_t* p_ptr;      // A operand of the Value sum
  const uint8_t* b_own;      // boost operand: row j, the columns of this lane's slot block (k-block gi % P)
  LaneOffsets lo;            // byte offsets of the lane into a record
  float qv[HPL][8];          // q * sm_scale * log2(e) divided by the weight, compact layout
  float m_run[HPL], l_run[HPL], z_run[HPL];
  float acc[HPL][8];         // channel 16*Td + j, in units of acc_unit (the fixed-point step of the last page's p*s)
  float acc_unit[HPL];

  static constexpr int A_PASS = 16 * 144;                           // bytes between the two matrices
  using BS = BoostShape<NB16>;
  static constexpr int B_PASS = 16 * (BS::COLS + 16);

  __device__ __forceinline__ PageWorker(WaveScratch<NB16, HPL>& ws_, int l)
      : ws(ws_), j(l & 15), gi(l >> 4), lo(lane_offsets<NB16, V4>(l)) {
    a_ptr = &ws.abuf[j][16 * gi];
    p_ptr = &ws.pbuf[j][16 * gi];
    b_own = &ws.bbuf[j][16 * (gi % BS::P)];
#pragma unroll
    for (int e = 0; e < HPL; ++e) {
      m_run[e] = -INFINITY; l_run[e] = 0.f; z_run[e] = 0.f; acc_unit[e] = 1.f;
#pragma unroll
      for (int k = 0; k < 8; ++k) acc[e][k] = 0.f;
    }
  }

  // q for head slot e from eight bf16 values (or zeros), scaled by sm_scale*log2(e)
  __device__ __forceinline__ void set_q(int e, const uint4& raw, float scale, bool live) {
    const uint32_t rw[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float inv_w = 1.0f / (2 * k < 4 ? wKA : wKB);
      qv[e][2 * k] = live ? __uint_as_float(rw[k] << 16) * scale * inv_w : 0.f;
      qv[e][2 * k + 1] = live ? __uint_as_float(rw[k] & 0xffff0000u) * scale * inv_w : 0.f;
    }
  }

  __device__ __forceinline__ v4i unpack_k(uint32_t w) const { return WEIGHTED_K ? unpack16_w(w) : unpack16(w); }
  __device__ __forceinline__ v4i unpack_v(uint32_t w) const { return WEIGHTED_V ? unpack16_w(w) : unpack16(w); }

  // stage a page's fp16 arrays in LDS (each lane group holds one of the four)
  __device__ __forceinline__ void stage_meta(const uint4& meta) {
    *reinterpret_cast<uint4*>(&ws.meta[gi][16 * j]) = meta;
  }

  // Phases A-C: integer logits of the 128 tokens of the page in `pg` (k_scale, k_zero staged in LDS).
  // The logit of head gi*HPL + e and token 16T + j is inv_alpha[e] * nl[e][T] + bias[e] (log2 domain).  The byte
  // terms are joined here, tile by tile, so that only one integer per (head, tile) lives on into the softmax.
  __device__ __forceinline__ void logits(const PageRegs<NB16, V4>& pg, int (&nl)[HPL][8],
                                         float (&inv_alpha)[HPL], float (&bias)[HPL]) {
    // ================= A: integer image of q*s, bias q.z =================
    float ks[8], kz[8];
    f16x8_to_f32(*reinterpret_cast<const uint4*>(&ws.meta[0][16 * j]), ks);
    f16x8_to_f32(*reinterpret_cast<const uint4*>(&ws.meta[1][16 * j]), kz);
#pragma unroll
    for (int e = 0; e < HPL; ++e) {
      float qs[8], amaxA = 0.f, amaxB = 0.f, bsA = 0.f, bsB = 0.f;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        qs[k] = qv[e][k] * ks[k];
        qs[k + 4] = qv[e][k + 4] * ks[k + 4];
        amaxA = fmaxf(amaxA, fabsf(qs[k]));
        amaxB = fmaxf(amaxB, fabsf(qs[k + 4]));
        bsA = fmaf(qv[e][k], kz[k], bsA);
        bsB = fmaf(qv[e][k + 4], kz[k + 4], bsB);
      }
      float amax = fmaxf(amaxA * wKA, amaxB * wKB), bsum = fmaf(bsA, wKA, bsB * wKB);   // both weights are 1 with the plain unpack
      amax = fmaxf(row_max_nonneg(amax), 1e-30f);
      bias[e] = row_sum(bsum);
      const float alpha = NLIM_K * __builtin_amdgcn_rcpf(amax);
      inv_alpha[e] = amax * (1.0f / NLIM_K);
      uint32_t u[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) u[k] = __float_as_uint(fmaf(qs[k], alpha, image_magic<TRK>()));
      uint2 tw[TRK];
      split_terms<TRK>(u, tw);
      const int hd = gi * HPL + e;
#pragma unroll
      for (int t = 0; t < TRK; ++t) *reinterpret_cast<uint2*>(&ws.abuf[term_row(hd, t)][8 * j]) = tw[t];
      if constexpr (NB16 > 0) {
        *reinterpret_cast<uint4*>(&ws.nbuf[hd][8 * j]) = make_uint4(u[0], u[1], u[2], u[3]);
        *reinterpret_cast<uint4*>(&ws.nbuf[hd][8 * j + 4]) = make_uint4(u[4], u[5], u[6], u[7]);
      }
    }
    wave_lds_fence();
    // ================= B: same integers gathered through the boosted-channel list =================
    if constexpr (NB16 > 0) {
#pragma unroll
      for (int s = 0; s < NB16; ++s) {
        const uint32_t ch = pg.chv[s];
        // weight the dense plane applies to this channel: 1, 4, 1, 4 for elements 0-3, 4-7, 8-11, 12-15
        const uint32_t sh = WEIGHTED_K ? ((ch >> 1) & 2u) : 0u;
#pragma unroll
        for (int e = 0; e < HPL; ++e) {
          const int hd = gi * HPL + e;
          uint32_t nn = ws.nbuf[hd][ch];
          if constexpr (TRK == 3) {
            // undo the division (an exact multiple, and still within the image's bound: a channel of weight 4
            // was scaled to a quarter of it), then the same three bytes as split_terms
            nn = ((nn - MAGIC3_BITS) << sh) + MAGIC3_BITS;
            ws.bbuf[term_row(hd, 0)][16 * s + j] = (uint8_t)(nn ^ 0x80u);
            ws.bbuf[term_row(hd, 1)][16 * s + j] = (uint8_t)((nn >> 8) ^ 0x80u);
            ws.bbuf[term_row(hd, 2)][16 * s + j] = (uint8_t)((nn >> 16) << 3);
          } else {
            ws.bbuf[term_row(hd, 0)][16 * s + j] = (uint8_t)nn;
            ws.bbuf[term_row(hd, 1)][16 * s + j] = (uint8_t)((nn + T1_ADD) >> 8);
          }
        }
      }
      wave_lds_fence();
    }
    // ================= C: logits for 128 tokens x heads on the int8 matrix cores =================
    // Dense plane, then the boost plane's contribution to the same tiles, then the join of the byte terms.  Eight-head
    // groups (two MFMA passes, twice the accumulators) do this in two halves of four token tiles each, so that at
    // most four tiles' accumulators are alive at a time; four-head groups take all eight tiles at once and read
    // each boost operand once.
    const v4i a0 = *reinterpret_cast<const v4i*>(a_ptr);
    const v4i a1 = *reinterpret_cast<const v4i*>(a_ptr + 64);
    v4i a0x = {0, 0, 0, 0}, a1x = {0, 0, 0, 0};
    if constexpr (TWO_PASS_K) {
      a0x = *reinterpret_cast<const v4i*>(a_ptr + A_PASS);
      a1x = *reinterpret_cast<const v4i*>(a_ptr + A_PASS + 64);
    }
    constexpr int NU = HPL == 2 ? 2 : 1;       // passes over the token tiles
    constexpr int TP = 8 / NU;                 // tiles per pass
#pragma unroll
    for (int uu = 0; uu < NU; ++uu) {
      v4i dq[TP], dqx[TWO_PASS_K ? TP : 1];
#pragma unroll
      for (int t = 0; t < TP; ++t) {
        const int T = TP * uu + t;
        const uint4 ld = pg.kd[T >> 1];
        const uint32_t w0 = (T & 1) ? ld.z : ld.x, w1 = (T & 1) ? ld.w : ld.y;
        const v4i b0 = unpack_k(w0), b1 = unpack_k(w1);
        v4i c = {0, 0, 0, 0};
        c = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0, b0, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1, b1, c, 0, 0, 0);
        dq[t] = c;
        if constexpr (TWO_PASS_K) {
          v4i cx = {0, 0, 0, 0};
          cx = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0x, b0, cx, 0, 0, 0);
          cx = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1x, b1, cx, 0, 0, 0);
          dqx[t] = cx;
        }
      }
      if constexpr (NB16 > 0) {
        // Boost plane: per operand q (64 slots) and tile class f the query-side operand is read with the k-blocks
        // of the other classes zeroed (an LDS address select), then one matrix instruction per tile.
#pragma unroll
        for (int q = 0; q < BS::KG; ++q) {
          v4i ab[BS::F], abx[TWO_PASS_K ? BS::F : 1];
#pragma unroll
          for (int f = 0; f < BS::F; ++f) {
            bool used = false;
#pragma unroll
            for (int v = 0; v < BS::WPG; ++v) used |= (BS::tile(f, v) / TP == uu);
            if (!used) continue;
            const bool mine = (gi / BS::P) == f;
            ab[f] = *reinterpret_cast<const v4i*>(mine ? b_own + 64 * q : ws.zero);
            if constexpr (TWO_PASS_K) abx[f] = *reinterpret_cast<const v4i*>(mine ? b_own + B_PASS + 64 * q : ws.zero);
          }
#pragma unroll
          for (int v = 0; v < BS::WPG; ++v) {
            bool used = false;
#pragma unroll
            for (int f = 0; f < BS::F; ++f) used |= (BS::tile(f, v) / TP == uu);
            if (!used) continue;
            const v4i bb = unpack16_x4(pg.kbw[BS::WPG * q + v]);
#pragma unroll
            for (int f = 0; f < BS::F; ++f) {
              const int T = BS::tile(f, v);
              if (T / TP != uu) continue;
              dq[T % TP] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ab[f], bb, dq[T % TP], 0, 0, 0);
              if constexpr (TWO_PASS_K)
                dqx[T % TP] = __builtin_amdgcn_mfma_i32_16x16x64_i8(abx[f], bb, dqx[T % TP], 0, 0, 0);
            }
          }
        }
      }
#pragma unroll
      for (int t = 0; t < TP; ++t)
#pragma unroll
        for (int e = 0; e < HPL; ++e) nl[e][TP * uu + t] = joined_k(dq[t], dqx[TWO_PASS_K ? t : 0], e);
    }
  }

  __device__ __forceinline__ int joined_k(const v4i& c, const v4i& cx, int e) const {
    if constexpr (HPL == 1) return join_terms(c[0], c[1], c[2]);
    else if constexpr (TWO_PASS_K) return join_terms(c[2 * e], c[2 * e + 1], cx[e]);
    else return join_terms(c[2 * e], c[2 * e + 1]);
  }
  __device__ __forceinline__ int joined_v(const v4i& c, const v4i& cx, int e) const {
    if constexpr (HPL == 1) return join_terms(c[0], c[1], c[2]);
    else if constexpr (TWO_PASS_V) return join_terms(c[2 * e], c[2 * e + 1], cx[e]);
    else return join_terms(c[2 * e], c[2 * e + 1]);
  }

  // Logits only (log2 domain, float) of the page in `pg`, stored as x[token][head]: used for the newest page
  // when its Values are still read in full precision (they are then handled with the other bf16 rows).
  __device__ __forceinline__ void logits_to(const PageRegs<NB16, V4>& pg, float (*x)[4 * HPL]) {
    int nl[HPL][8];
    float inv_alpha[HPL], bias[HPL];
    logits(pg, nl, inv_alpha, bias);
#pragma unroll
    for (int e = 0; e < HPL; ++e)
#pragma unroll
      for (int T = 0; T < 8; ++T)
        x[16 * T + j][gi * HPL + e] = fmaf((float)nl[e][T], inv_alpha[e], bias[e]);
  }

  // Processes the page held in `pg` (its fp16 arrays already staged in LDS).  The pieces of the wavefront's
  // next page (record `rec_nx`; an empty reference if there is none) are requested into the same registers as
  // soon as they are dead.
  __device__ __forceinline__ void process(PageRegs<NB16, V4>& pg, RecRef rec_nx, bool has_nx) {
    uint4 meta_nx = make_uint4(0, 0, 0, 0);
    if (has_nx) meta_nx = load_meta<NB16>(rec_nx, lo);
    int nlg[HPL][8];
    float inv_alpha[HPL], bias[HPL];
    logits(pg, nlg, inv_alpha, bias);
    if (has_nx) load_k<NB16, V4>(pg, rec_nx, lo);   // the Key planes of this page are in the matrix pipeline now
    // ================= D: online softmax; lane (j, gi) owns token 16T + j of heads gi*HPL + e ==========
    float vs[8], vz[8];
    f16x8_to_f32(*reinterpret_cast<const uint4*>(&ws.meta[2][16 * j]), vs);
    f16x8_to_f32(*reinterpret_cast<const uint4*>(&ws.meta[3][16 * j]), vz);
    float corr[HPL], rescale[HPL];
#pragma unroll
    for (int e = 0; e < HPL; ++e) {
      // logits are inv_alpha * nl + bias with inv_alpha > 0: take the maximum on the integers
      int nl[8], mxi = INT_MIN;
#pragma unroll
      for (int T = 0; T < 8; ++T) {
        nl[T] = nlg[e][T];
        mxi = max(mxi, nl[T]);
      }
      mxi = row_max_i32(mxi);
      const float m_new = fmaxf(m_run[e], fmaf((float)mxi, inv_alpha[e], bias[e]));
      corr[e] = __builtin_amdgcn_exp2f(m_run[e] - m_new);
      m_run[e] = m_new;
      // the weights of the Value-side unpack are taken out of p through the exponent
      const float cA = bias[e] - (m_new + oVA), cB = bias[e] - (m_new + oVB);
      float ps[8], psA = 0.f, psB = 0.f, zsA = 0.f, zsB = 0.f, pmA = 0.f, pmB = 0.f;
#pragma unroll
      for (int T = 0; T < 4; ++T) {
        const float pa = __builtin_amdgcn_exp2f(fmaf((float)nl[T], inv_alpha[e], cA));
        const float pb = __builtin_amdgcn_exp2f(fmaf((float)nl[T + 4], inv_alpha[e], cB));
        psA += pa; psB += pb;
        zsA = fmaf(pa, vz[T], zsA); zsB = fmaf(pb, vz[T + 4], zsB);
        ps[T] = pa * vs[T]; ps[T + 4] = pb * vs[T + 4];
        pmA = fmaxf(pmA, ps[T]); pmB = fmaxf(pmB, ps[T + 4]);
      }
      float psum = fmaf(psA, wVA, psB * wVB), zsum = fmaf(zsA, wVA, zsB * wVB), pmax = fmaxf(pmA * wVA, pmB * wVB);
      l_run[e] = fmaf(l_run[e], corr[e], psum);     // (corr comes out of v_exp: not for fma_in_place)
      z_run[e] = fmaf(z_run[e], corr[e], zsum);
      // (the floor keeps the running sums, which are held in units of pmax / NLIM_V, far from overflow; a page
      // whose weights are all below it contributes less than 1e-12 of the total)
      pmax = fmaxf(row_max_nonneg(pmax), 1e-12f);
      const float beta = NLIM_V * __builtin_amdgcn_rcpf(pmax);
      rescale[e] = corr[e] * acc_unit[e] * beta;       // old unit -> new unit, and the softmax correction
      acc_unit[e] = pmax * (1.0f / NLIM_V);
      uint32_t u[8];
#pragma unroll
      for (int T = 0; T < 8; ++T) u[T] = __float_as_uint(fmaf(ps[T], beta, image_magic<TRV>()));
      uint2 tw[TRV];
      split_terms<TRV>(u, tw);
      const int hd = gi * HPL + e;
#pragma unroll
      for (int t = 0; t < TRV; ++t) *reinterpret_cast<uint2*>(&ws.pbuf[term_row(hd, t)][8 * j]) = tw[t];
    }
    wave_lds_fence();
    // ================= E: weighted Value sum on the int8 matrix cores =================
    const v4i pa0 = *reinterpret_cast<const v4i*>(p_ptr);
    const v4i pa1 = *reinterpret_cast<const v4i*>(p_ptr + 64);
    v4i pa0x = {0, 0, 0, 0}, pa1x = {0, 0, 0, 0};
    if constexpr (TWO_PASS_V) {
      pa0x = *reinterpret_cast<const v4i*>(p_ptr + A_PASS);
      pa1x = *reinterpret_cast<const v4i*>(p_ptr + A_PASS + 64);
    }
#pragma unroll
    for (int Td = 0; Td < 8; ++Td) {
      const uint4 ld = pg.vd[Td >> 1];
      const uint32_t w0 = (Td & 1) ? ld.z : ld.x, w1 = (Td & 1) ? ld.w : ld.y;
      const v4i b0 = unpack_v(w0), b1 = unpack_v(w1);
      v4i c = {0, 0, 0, 0}, cx = {0, 0, 0, 0}, chi = {0, 0, 0, 0};
      c = __builtin_amdgcn_mfma_i32_16x16x64_i8(pa0, b0, c, 0, 0, 0);
      c = __builtin_amdgcn_mfma_i32_16x16x64_i8(pa1, b1, c, 0, 0, 0);
      if constexpr (V4) {   // the high two bits of 4-bit Values: same contraction, weight 4
        const uint4 lh = pg.vh[Td >> 1];
        const v4i h0 = unpack_v((Td & 1) ? lh.z : lh.x), h1 = unpack_v((Td & 1) ? lh.w : lh.y);
        chi = __builtin_amdgcn_mfma_i32_16x16x64_i8(pa0, h0, chi, 0, 0, 0);
        chi = __builtin_amdgcn_mfma_i32_16x16x64_i8(pa1, h1, chi, 0, 0, 0);
      }
      if constexpr (TWO_PASS_V) {
        cx = __builtin_amdgcn_mfma_i32_16x16x64_i8(pa0x, b0, cx, 0, 0, 0);
        cx = __builtin_amdgcn_mfma_i32_16x16x64_i8(pa1x, b1, cx, 0, 0, 0);
      }
#pragma unroll
      for (int e = 0; e < HPL; ++e) {
        int ne = joined_v(c, cx, e);
        if constexpr (V4) ne += 4 * joined_v(chi, cx, e);
        fma_in_place(acc[e][Td], rescale[e], (float)ne);
      }
    }
    if (has_nx) {
      load_v<NB16, V4>(pg, rec_nx, lo);
      stage_meta(meta_nx);   // requested at the top of this page
    }
    wave_lds_fence();   // the next page overwrites abuf/pbuf and reads the staged arrays
  }
};

// HPL = query heads per lane: 1 for GQA groups of 1, 2, 4 (three byte terms in one matrix), 2 for groups of 8
// (three byte terms in two matrix passes).  Grid: x = page range (see active_splits), y = kv-head, z = sequence.
// Block = NW wavefronts (4 or 8); wavefront w takes pages p0+w, p0+w+NW, ... of the range and a slice of
// the range's share of the rows held in full precision (Sink, window).
// wavefronts per SIMD the kernel is compiled for (register budget 512 / n)
// (eight-head groups with more than 64 boosted channels need more than 256 registers for their two-pass contractions:
// they run in 4-wavefront blocks with one wavefront per SIMD)
template <int NB16, int HPL>
constexpr int decode_waves_per_simd() { return (HPL == 2 && NB16 > 4) ? 1 : 2; }

// FUSED: the block first performs this (sequence, kv-head)'s share of kitty_append_token (flush a full window
// into the fresh page, store the new token), then attends over the result; needs one range per (sequence,
// kv-head), i.e. grid.x == 1 and direct_out.  The new token's row is taken from k_new / v_new directly, a
// freshly written record is fenced before it is read back, and the sequence state is advanced by the block of
// the sequence that is last to have read the old state (ticket in bits 8.. of n_resid, as in append_token_kernel;
// the ticket is taken right after the state has been read and looked at only at the end).
// ROWW: one more wavefront (index NW) that only does the block's full-precision rows, concurrently with the page
// loop of the others, instead of every wavefront doing a share of them after its pages.  A ninth wavefront puts
// three on one SIMD, so the variant exists where the kernel fits 168 registers.
// FUSED: 0 = attention only; 1 = append first, one range per (sequence, kv-head); 2 = append first, several ranges
// (the merge launch stores the token and advances the state)
template <int NB16, int HPL, int NW, int FUSED, bool V4, bool ROWW = false>
__global__ __launch_bounds__(64 * (NW + (ROWW ? 1 : 0)), (ROWW ? 3 : decode_waves_per_simd<NB16, HPL>())) void decode_split_kernel(DecodeParams p) {
  using R = Rec<NB16, V4>;
  constexpr int RPH = 4 / HPL;
  constexpr int NH = 4 * HPL;              // heads handled by the block
  constexpr int NT = NW + (ROWW ? 1 : 0);  // wavefronts of the block

  constexpr bool DEFER = FUSED == 2;
  __shared__ DecodeSmem<NB16, HPL, NT, FUSED != 0> smem;

  const int slot = blockIdx.x, h = blockIdx.y;
  const int b = p.seq_order ? p.seq_order[blockIdx.z] : (int)blockIdx.z;
  if ((unsigned)b >= (unsigned)p.batch) return;   // not a sequence of this batch (same for the whole block)
  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: page ids stay in scalar registers
  const int l = tid & 63, j = l & 15, gi = l >> 4;
  const bool roww = ROWW && w == NW;       // this wavefront does rows, not pages
  const int g = p.gqa;
  const size_t pair = (size_t)b * p.n_kv_heads + h;

  int np = page_count(p, b);
  int r = p.has_window ? min(p.n_resid[b] & ((1 << TICKET_SHIFT) - 1), G) : 0;
  int ns = p.sink_cap ? min(p.n_sink[b], p.sink_cap) : 0;
  // fused append: state before the step, what the step does to it
  const int nr_old = r, np_old = np, ns_old = ns;
  int newrow = -1;              // window row of the token appended by this step (its data comes from k_new/v_new)
  int newsink = -1;             // or its Sink row
  int32_t fresh_pid = -1;       // page written by this step's flush (not yet in the page table)
  bool ok = true, flush = false;
  const uint16_t* knew_h = nullptr;
  const uint16_t* vnew_h = nullptr;
  // the new token's copy into the cache (threads 0..31 hold 16 bytes each): fetched early, stored at the end of
  // the kernel, so that nobody waits for the round trip; attention reads the token from k_new / v_new itself
  uint4 keep_val = make_uint4(0, 0, 0, 0);
  uint16_t* keep_dst = nullptr;
  // Fused append.  Every block of the sequence works out the state after the step from the state before it.  With
  // one range per (sequence, kv-head) the block also stores the token and takes part in advancing the state; with
  // several ranges (defer_state) the block of the last active range, which alone reads the newest page, flushes a
  // full window into it, and the token and the state are left to the merge launch that follows.
  int32_t pid = -1;
  if constexpr (FUSED) {
    pid = p.fresh_page_ids[b];
    knew_h = p.k_new + pair * D;
    vnew_h = p.v_new + pair * D;
    if (ns_old < p.sink_cap) {    // the Sink is not full: the token goes there and nothing else changes
      newsink = ns_old;
      ns = ns_old + 1;
    } else {
      flush = nr_old >= G;
      ok = !flush || (np_old < p.max_pages && pid >= 0 && pid < p.n_pool_pages);
      if (ok) {
        if (flush) { np = np_old + 1; r = 1; newrow = 0; }
        else { r = nr_old + 1; newrow = nr_old; }
      }
    }
  }
  const int nfp = ns + r;       // rows read in full precision for both Keys and Values: Sink, then window
  const int sb = active_splits(np, nfp, p.n_splits, p.min_pages);
  int ticket = 0;
  if constexpr (FUSED) {
    if (!DEFER || slot == sb - 1) {
      if (newsink >= 0) {
        if (!DEFER && tid < 32)
          keep_dst = (tid < 16 ? p.sink_k_w : p.sink_v_w) + (pair * p.sink_cap + ns_old) * D + (tid & 15) * 8;
      } else if (ok) {
        uint16_t* wkw = p.resid_k_w + pair * (size_t)(G * D);
        if (flush) {
          uint8_t* rec = p.pool_w + ((size_t)pid * p.n_kv_heads + h) * (size_t)R::bytes;
          const uint16_t* wv_old = p.resid_v_w + resid_v_offset(b, h, p.n_kv_heads, p.v_local, np_old);
          quantize_page<NB16, V4>(smem.quant, wkw, wv_old, D, rec, p.rank_metric);
          // The record is read back by this block's wavefronts only, which share the compute unit and its
          // first-level cache: the barrier's workgroup-scope release/acquire is all the ordering needed.  (A
          // device-scope fence here writes the whole second-level cache back: +35 us on a step with a flush.)
          __syncthreads();
          fresh_pid = pid;
        }
        if (!DEFER && tid < 32) {             // keep the token for the following steps
          uint16_t* wvw = p.resid_v_w + resid_v_offset(b, h, p.n_kv_heads, p.v_local, np);
          keep_dst = (tid < 16 ? wkw : wvw) + (size_t)newrow * D + (tid & 15) * 8;
        }
      }
    }
    // Every block of the sequence has to see the old state, so the state is advanced by the block that is last to
    // have read it: a ticket is taken here (its answer is not needed before the end of the kernel, which hides
    // the round trip of the atomic), and the holder of the last ticket stores the new state when it is done.
    if (!DEFER) {
      __syncthreads();            // all wavefronts of this block have read the state (they branched on it above)
      if (tid == 0) ticket = atomicAdd(&p.n_resid_w[b], 1 << TICKET_SHIFT);
      // (fetched behind the barrier, which waits for every outstanding load of the wavefront)
      if (keep_dst) keep_val = *reinterpret_cast<const uint4*>((tid < 16 ? knew_h : vnew_h) + (tid & 15) * 8);
    }
  }
  if (slot >= sb) {   // no share of this sequence for this range
    if (DEFER) {   // the merge that follows does not look at the state: leave a neutral partial
      float* part = p.ws + (((size_t)b * p.n_kv_heads + h) * p.n_splits + slot) * (size_t)g * WS_STRIDE;
      for (int o = tid; o < g * WS_STRIDE; o += 64 * NT) part[o] = (o % WS_STRIDE) == D ? -INFINITY : 0.f;
    }
    if (p.direct_out && slot == 0) {   // empty sequence: the result is defined as zeros
      for (int o = tid; o < g * D; o += 64 * NT) {
        const size_t oi = ((size_t)b * p.n_q_heads + (size_t)h * g) * D + o;
        if (p.out_dtype == 0) reinterpret_cast<uint16_t*>(p.out)[oi] = 0;
        else reinterpret_cast<float*>(p.out)[oi] = 0.f;
      }
    }
    return;
  }
  const int p0 = (int)((long long)slot * np / sb), p1 = (int)((long long)(slot + 1) * np / sb);
  // Local window of the Values (Fig. 1): the newest page's Values are still read from their bf16 rows; its
  // Keys are read from the record, and the logits are handed to the full-precision path below.
  const bool lag_here = p.v_local && np >= 1 && slot == sb - 1;   // the last range holds the newest page
  const int p1q = p1 - (lag_here ? 1 : 0);                        // pages [p0, p1q) are read from records entirely

  WaveScratch<NB16, HPL>& ws = smem.w[w];
  // logits of the newest page, [token][head]: kept in the (by then idle) gather table of the wavefront that
  // computes them, which is the one whose turn the page is
  float (*lagx)[NH] = reinterpret_cast<float (*)[NH]>(&smem.w[lag_here ? (p1q - p0) % NW : 0].nbuf[0][0]);
  static_assert(sizeof(ws.nbuf) >= sizeof(float) * G * NH, "lagx aliases nbuf");
  const size_t qrow = ((size_t)b * p.n_q_heads + (size_t)h * g);
  PageWorker<NB16, HPL, V4> pw(ws, l);

  // ================= rows read in full precision, spread over the ranges and wavefronts =================
  // Range `slot` of `sb` takes rows [slot*nfp/sb, (slot+1)*nfp/sb) of the list (Sink rows, then window rows); the
  // last range also takes the G Value rows of the newest page when the Local window is on (their logits are in
  // lagx).  The block's list is cut into NW near-equal runs, one per wavefront, walked in chunks of 32 rows
  // with an online softmax.  In 4-wavefront blocks (short ranges, or grids with several blocks per compute unit)
  // a wavefront that has pages does its Sink and window rows while its first page is on its way and carries the
  // sums of its own heads through the page loop (+3 % on the variable-length 36-layer loop; in 8-wavefront blocks
  // the same costs 2.5 % on the 32k workload); the newest page's rows always follow the pages.
  float accw[NH][8];        // channels 8j..8j+7 of every head (summed over the lane groups by fp_reduce_own)
  float mw[HPL], lw[HPL];
  auto fp_reset = [&]() {
#pragma unroll
    for (int hh = 0; hh < NH; ++hh)
#pragma unroll
      for (int k = 0; k < 8; ++k) accw[hh][k] = 0.f;
#pragma unroll
    for (int e = 0; e < HPL; ++e) { mw[e] = -INFINITY; lw[e] = 0.f; }
  };
  // sum over the four lane groups (rows 4i + gi: two butterfly steps); every group then holds the full sums and
  // keeps those of its own heads
  auto fp_reduce_own = [&](float (&dst)[HPL][8]) {
#pragma unroll
    for (int hh = 0; hh < NH; ++hh)
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        float v = accw[hh][k];
        v += __shfl_xor(v, 16);
        v += __shfl_xor(v, 32);
        accw[hh][k] = v;
      }
#pragma unroll
    for (int e = 0; e < HPL; ++e) {
      const int hd = gi * HPL + e;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        float v = 0.f;
#pragma unroll
        for (int hh = 0; hh < NH; ++hh) v = (hh == hd) ? accw[hh][k] : v;
        dst[e][k] = v;
      }
    }
  };
  constexpr bool FP_FIRST = !ROWW && NW == 4 && !(HPL == 2 && NB16 >= 4);   // (not where the registers are all taken)
  const int wr0 = (int)((long long)slot * nfp / sb), wr1 = (int)((long long)(slot + 1) * nfp / sb);
  const int nkv = wr1 - wr0;                       // rows of this block with bf16 Keys and Values
  const int nlag = lag_here ? G : 0;               // rows of the newest page (list indices nkv ..)
  // runs of this wavefront: of the whole list, or (rows first) of its two parts
  const int per = (nkv + nlag + NW - 1) / NW;
  const int t0 = w * per, t1 = min(t0 + per, nkv + nlag);
  const int perk = (nkv + NW - 1) / NW, perl = (nlag + NT - 1) / NT;   // (the newest page's rows: every wavefront)
  const int kv0 = w * perk, kv1 = min(kv0 + perk, nkv);
  const int lg0 = nkv + min(w * perl, nlag), lg1 = nkv + min((w + 1) * perl, nlag);
  float kvacc[HPL][8], kvm[HPL], kvl[HPL];         // rows first: what is carried through the page loop
  bool kv_done = false;
  const uint16_t* wk = p.resid_k + pair * (size_t)(G * D);
  const uint16_t* wv = p.resid_v + resid_v_offset(b, h, p.n_kv_heads, p.v_local, np);
  const uint16_t* lagv = p.resid_v + resid_v_offset(b, h, p.n_kv_heads, p.v_local, np - 1);
  const uint16_t* sk = p.sink_k + pair * (size_t)p.sink_cap * D;
  const uint16_t* sv = p.sink_v + pair * (size_t)p.sink_cap * D;
  const uint16_t* qdummy = p.q + qrow * D;       // any readable row: Key operand of rows whose logits come from lagx
  // row i of the block's list -> its Key row, Value row, and index into lagx (or -1)
  auto row_ptrs = [&](int i, const uint16_t*& kp, const uint16_t*& vp, int& li) {
    if (i < nkv) {
      const int f = wr0 + i;
      li = -1;
      if (f < ns) {
        const bool fresh = FUSED && f == newsink;
        kp = fresh ? knew_h : sk + (size_t)f * D;
        vp = fresh ? vnew_h : sv + (size_t)f * D;
      } else {
        const int t = f - ns;
        const bool fresh = FUSED && t == newrow;
        kp = fresh ? knew_h : wk + (size_t)t * D;
        vp = fresh ? vnew_h : wv + (size_t)t * D;
      }
    } else {
      li = i - nkv;
      kp = qdummy;
      vp = lagv + (size_t)li * D;
    }
  };
  auto fp_rows = [&](int t0, int t1) {
    // A operand: query rows; row hd*RPH carries head hd, the other rows are zero
    const int arow_head = j / RPH;
    const bool arow_live = (j % RPH) == 0 && arow_head < g;
    v8bf aq[4];
  #pragma unroll
    for (int mm = 0; mm < 4; ++mm) {
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (arow_live) raw = *reinterpret_cast<const uint4*>(p.q + (qrow + arow_head) * D + 32 * mm + 8 * gi);
      aq[mm] = __builtin_bit_cast(v8bf, raw);
    }
    for (int c0 = t0; c0 < t1; c0 += 32) {
      // Value rows c0 + 4i + gi (i < 8), channels 8j..8j+7: requested first, used last.  Rows past the run are
      // clamped to its last row (their weight is zero; uninitialised rows are never touched).
      uint4 vrow[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint16_t *kp, *vp;
        int li;
        row_ptrs(min(c0 + 4 * i + gi, t1 - 1), kp, vp, li);
        vrow[i] = *reinterpret_cast<const uint4*>(vp + 8 * j);
      }
      float x[HPL][2];
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        const int t = c0 + 16 * tt + j;
        const uint16_t *kr, *vp;
        int li;
        row_ptrs(min(t, t1 - 1), kr, vp, li);
        v4f c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int mm = 0; mm < 4; ++mm) {
          const uint4 raw = *reinterpret_cast<const uint4*>(kr + 32 * mm + 8 * gi);
          c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aq[mm], __builtin_bit_cast(v8bf, raw), c, 0, 0, 0);
        }
#pragma unroll
        for (int e = 0; e < HPL; ++e) {
          const float xl = lagx[max(li, 0)][gi * HPL + e];
          const float xv = li >= 0 ? xl : c[e * RPH] * p.qk_scale_log2;
          x[e][tt] = t < t1 ? xv : -INFINITY;
        }
      }
#pragma unroll
      for (int e = 0; e < HPL; ++e) {
        const float m_new = fmaxf(mw[e], row_max(fmaxf(x[e][0], x[e][1])));   // finite: the chunk has a valid row
        const float corr = __builtin_amdgcn_exp2f(mw[e] - m_new);              // 0 on the first chunk
        mw[e] = m_new;
        const float pa = __builtin_amdgcn_exp2f(x[e][0] - m_new), pb = __builtin_amdgcn_exp2f(x[e][1] - m_new);
        lw[e] = fmaf(lw[e], corr, pa + pb);
        ws.pw[j][gi * HPL + e] = pa;
        ws.pw[16 + j][gi * HPL + e] = pb;
        if (j == 0) ws.pcorr[gi * HPL + e] = corr;
      }
      wave_lds_fence();
      {
        float cr[NH];
#pragma unroll
        for (int q4 = 0; q4 < NH / 4; ++q4) {
          const float4 f = *reinterpret_cast<const float4*>(&ws.pcorr[4 * q4]);
          cr[4 * q4] = f.x; cr[4 * q4 + 1] = f.y; cr[4 * q4 + 2] = f.z; cr[4 * q4 + 3] = f.w;
        }
#pragma unroll
        for (int hh = 0; hh < NH; ++hh)
#pragma unroll
          for (int k = 0; k < 8; ++k) accw[hh][k] *= cr[hh];
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int tl = 4 * i + gi;          // row within the chunk (weight 0 beyond the run)
        float ph[NH];
#pragma unroll
        for (int q4 = 0; q4 < NH / 4; ++q4) {
          const float4 f = *reinterpret_cast<const float4*>(&ws.pw[tl][4 * q4]);
          ph[4 * q4] = f.x; ph[4 * q4 + 1] = f.y; ph[4 * q4 + 2] = f.z; ph[4 * q4 + 3] = f.w;
        }
        const uint32_t vw[4] = {vrow[i].x, vrow[i].y, vrow[i].z, vrow[i].w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const float v0 = __uint_as_float(vw[k] << 16), v1 = __uint_as_float(vw[k] & 0xffff0000u);
#pragma unroll
          for (int hh = 0; hh < NH; ++hh) {
            accw[hh][2 * k] = fmaf(ph[hh], v0, accw[hh][2 * k]);
            accw[hh][2 * k + 1] = fmaf(ph[hh], v1, accw[hh][2 * k + 1]);
          }
        }
      }
      wave_lds_fence();   // the next chunk overwrites pw
    }
  };

  float own[HPL][8];        // the rows' sums for this lane group's heads, channels 8j..8j+7
  if (roww) {                   // (one branch against the other, so that these sums do not live through the page loop)
    fp_reset();
    if (nkv > 0) fp_rows(0, nkv);             // Sink and window rows, while the others stream their pages
    if (lag_here) __syncthreads();            // (the block's other wavefronts meet this barrier below)
    if (lg0 < lg1) fp_rows(lg0, lg1);         // its share of the newest page's rows, now that their logits are there
    fp_reduce_own(own);
  } else {
  if (p0 < p1) {
    const int32_t* pt = p.page_table + (size_t)b * p.max_pages;
    const size_t rec_stride = (size_t)p.n_kv_heads * R::bytes;
    const uint8_t* pool_h = p.pool + (size_t)h * R::bytes;
    // Page ids of this wavefront's pages: lane k of `ids` holds the id of its k-th page (64 at a time), so the
    // loop takes them from a register with v_readlane instead of waiting for a scalar load per page.
    auto load_ids = [&](int first) {
      const int i = p0 + w + NW * (first + l);
      return i < p1 ? pt[i] : 0;
    };
    // (an id outside the pool, which only a corrupted table can hold, is folded onto the pool's last page
    // rather than followed out of bounds: one scalar instruction per page)
    const uint32_t last_page = (uint32_t)(p.n_pool_pages - 1);
    int32_t ids = load_ids(0);
    auto rec_at = [&](int k, int idx) {     // record of the wavefront's k-th page, which is page idx of the sequence
      const int32_t got = (int32_t)min((uint32_t)__builtin_amdgcn_readlane(ids, k & 63), last_page);
      const int32_t id = (FUSED && idx == np_old && fresh_pid >= 0) ? fresh_pid : got;
      return pool_h + (size_t)id * rec_stride;
    };
    // one register buffer: each piece of the next page is requested when the current page no longer needs it.
    PageRegs<NB16, V4> pg{};
    int idx = p0 + w;
    uint4 m0 = make_uint4(0, 0, 0, 0);
    // ---- zero the operand matrices once (rows of absent heads and the unused term row stay zero)
    {
      uint32_t* z32 = reinterpret_cast<uint32_t*>(&ws.abuf[0][0]);
      using WSc = WaveScratch<NB16, HPL>;
      constexpr int nwords = (int)(offsetof(WSc, pw) - offsetof(WSc, abuf)) / 4;   // abuf, bbuf, pbuf are contiguous
      for (int i = l; i < nwords; i += 64) z32[i] = 0u;
      if (l < 4) reinterpret_cast<uint32_t*>(ws.zero)[l] = 0u;
    }
#pragma unroll
    for (int e = 0; e < HPL; ++e) {
      const int hd = gi * HPL + e;
      const bool live = hd < g;
      const uint4 raw = live ? *reinterpret_cast<const uint4*>(p.q + (qrow + hd) * D + 8 * j) : make_uint4(0, 0, 0, 0);
      pw.set_q(e, raw, p.qk_scale_log2, live);
    }
    if (idx < p1) {
      const RecRef rec = rec_ref<NB16, V4>(rec_at(0, idx));
      m0 = load_meta<NB16>(rec, pw.lo);
      load_k<NB16, V4>(pg, rec, pw.lo);
      load_v<NB16, V4>(pg, rec, pw.lo);
      if constexpr (FP_FIRST) {
        if (kv0 < kv1) {
          fp_reset();
          fp_rows(kv0, kv1);
          fp_reduce_own(kvacc);
#pragma unroll
          for (int e = 0; e < HPL; ++e) { kvm[e] = mw[e]; kvl[e] = lw[e]; }
          kv_done = true;
        }
      }
      pw.stage_meta(m0);
      wave_lds_fence();
      // The two wavefronts that share a SIMD take the higher issue priority in turn: with equal priorities the
      // older one (w < 4) wins every conflict and ends its equal share of the pages ~7 % earlier, leaving the block
      // to wait for the younger one.  The younger one gets the higher priority on three pages out of four (plain
      // alternation leaves it 6-7 us behind on the 32k workload; two out of three measures the same, five out of
      // six and more, or always, worse).  4-wavefront blocks share their SIMDs with another block's wavefronts and
      // simply alternate.
      int turn = 0;
      int k = 0;
      // PEEL: every page but the wavefront's last requests the next one; those run in a loop whose loads are
      // unconditional, so that the compiler's waits for them are exact, and the last page follows the loop.
      // Otherwise one loop with the next page's loads behind a branch: the compiler then drains the load queue in
      // the middle of every page, which happens to pace the requests of the 8-wavefront blocks of four-head groups
      // well (32k workload: 97.6 us against 101.5 us peeled); eight-head groups and 4-wavefront blocks stream
      // better peeled (128k workload 137 against 141 us; the 36-layer loop 7.94 against 8.17 ms per step).
      constexpr bool PEEL = HPL == 2 || NW == 4;
      for (; PEEL ? idx + NW < p1 : idx < p1q; idx += NW) {
        const bool has_nx = idx + NW < p1;
        const bool high = NW == 4 ? (turn & 1) != 0 : (w >= 4 ? (turn & 3) != 0 : (turn & 3) == 0);
        if (high) __builtin_amdgcn_s_setprio(1); else __builtin_amdgcn_s_setprio(0);
        ++turn;
        ++k;
        // Where the reloaded ids are first used decides where the compiler waits for them.  Used in this rare
        // branch, the wait sits here; otherwise the loop head has to assume the load may be pending and drains
        // the whole load queue, the current page's Value plane included, before every page (+5 % on the 32k
        // workload).
        if ((k & 63) == 0) ids = max(load_ids(k), 0);
        if constexpr (PEEL) pw.process(pg, rec_ref<NB16, V4>(rec_at(k, idx + NW)), true);   // (a constant: no branches around the loads)
        else pw.process(pg, rec_ref<NB16, V4>(has_nx ? rec_at(k, idx + NW) : pool_h), has_nx);
      }
      if constexpr (PEEL) {
        if (idx < p1q) {
          pw.process(pg, rec_ref<NB16, V4>(pool_h), false);
          idx += NW;
        }
      }
      __builtin_amdgcn_s_setprio(0);
      if (lag_here && idx == p1q) pw.logits_to(pg, lagx);   // this wavefront holds the newest page
    }
  }
  if (lag_here) __syncthreads();   // lagx is complete (the condition is the same for the whole block)

  // ---- the full-precision rows that are still to do, then what was saved is folded in
  if constexpr (ROWW) {
    fp_reset();
    if (lg0 < lg1) fp_rows(lg0, lg1);       // the newest page's rows are shared by all wavefronts of the block
    fp_reduce_own(own);
  } else {
    fp_reset();
    if constexpr (FP_FIRST) {
      if (!kv_done && kv0 < kv1) fp_rows(kv0, kv1);
      if (lg0 < lg1) fp_rows(lg0, lg1);
    } else {
      if (t0 < t1) fp_rows(t0, t1);
    }
    fp_reduce_own(own);
    if constexpr (FP_FIRST) {
      if (kv_done) {
#pragma unroll
        for (int e = 0; e < HPL; ++e) {
          const float M = fmaxf(mw[e], kvm[e]);                       // kvm is finite: the saved part had rows
          const float fa = __builtin_amdgcn_exp2f(mw[e] - M), fb = __builtin_amdgcn_exp2f(kvm[e] - M);
#pragma unroll
          for (int k = 0; k < 8; ++k) own[e][k] = fmaf(own[e][k], fa, kvacc[e][k] * fb);
          lw[e] = fmaf(lw[e], fa, kvl[e] * fb);
          mw[e] = M;
        }
      }
    }
  }

  }   // (wavefronts that do pages)

  // ================= merge the partials (wavefronts x {pages, full-precision rows}), write the result ====
  // slots: pages of wavefront w in slot w, its rows in slot NW + w; with a row wavefront that one's rows in slot
  // NW and, when the newest page's rows are read here, the others' shares of those in slots NW + 1 + w
  float lsum[HPL], zsum[HPL], lwsum[HPL];
#pragma unroll
  for (int e = 0; e < HPL; ++e) { lsum[e] = row_sum(pw.l_run[e]); zsum[e] = row_sum(pw.z_run[e]); lwsum[e] = row_sum(lw[e]); }
  __syncthreads();   // every wavefront is done with its scratch
  MergeScratch<HPL, NT>& mg = smem.mg;
  if (!roww) {
#pragma unroll
    for (int e = 0; e < HPL; ++e) {
      const int hd = gi * HPL + e;
#pragma unroll
      for (int Td = 0; Td < 8; ++Td) mg.acc[w][hd][16 * Td + j] = fmaf(pw.acc[e][Td], pw.acc_unit[e], zsum[e]);
      if (j == 0) { mg.m[w][hd] = pw.m_run[e]; mg.l[w][hd] = lsum[e]; }
    }
  }
  if (!ROWW || roww || lag_here) {
    const int rs = ROWW ? (roww ? NW : NW + 1 + w) : NW + w;
#pragma unroll
    for (int e = 0; e < HPL; ++e) {
      const int hd = gi * HPL + e;
      if (j == 0) { mg.m[rs][hd] = mw[e]; mg.l[rs][hd] = lwsum[e]; }
#pragma unroll
      for (int k = 0; k < 8; ++k) mg.acc[rs][hd][8 * j + k] = own[e][k];
    }
  }
  __syncthreads();
  float* part = p.ws + (((size_t)b * p.n_kv_heads + h) * p.n_splits + slot) * (size_t)g * WS_STRIDE;
  auto merge_out = [&](auto npc) {     // npc: how many partial slots are in use (a compile-time constant)
  constexpr int NPART = decltype(npc)::value;
  for (int o = tid; o < g * D; o += 64 * NT) {
    const int hd = o >> 7, d = o & 127;
    float M = -INFINITY;
#pragma unroll
    for (int ww = 0; ww < NPART; ++ww) M = fmaxf(M, mg.m[ww][hd]);
    float a = 0.f, L = 0.f;
#pragma unroll
    for (int ww = 0; ww < NPART; ++ww) {
      const float f = __builtin_amdgcn_exp2f(mg.m[ww][hd] - M);   // exp2(-inf) = 0 for idle partials
      a = fmaf(mg.acc[ww][hd][d], f, a);
      L = fmaf(mg.l[ww][hd], f, L);
    }
    if (p.direct_out) {   // the only range of this (sequence, kv-head): finish here
      const float v = L > 0.f ? a / L : 0.f;
      const size_t oi = (qrow + hd) * D + d;
      if (p.out_dtype == 0) reinterpret_cast<uint16_t*>(p.out)[oi] = f32_to_bf16_rne(v);
      else reinterpret_cast<float*>(p.out)[oi] = v;
    } else {
      part[hd * WS_STRIDE + d] = a;
      if (d == 0) { part[hd * WS_STRIDE + D] = M; part[hd * WS_STRIDE + D + 1] = L; }
    }
  }
  };
  if constexpr (ROWW) {
    if (lag_here) merge_out(std::integral_constant<int, 2 * NW + 1>{});
    else merge_out(std::integral_constant<int, NW + 1>{});
  } else {
    merge_out(std::integral_constant<int, 2 * NW>{});
  }
  if constexpr (FUSED) {
    if (keep_dst) *reinterpret_cast<uint4*>(keep_dst) = keep_val;
    if (tid == 0 && !DEFER) {
      if ((ticket >> TICKET_SHIFT) == p.n_kv_heads - 1) {   // every block of this sequence has read the old state
        int new_nr = nr_old;
        if (newsink >= 0) {
          p.n_sink_w[b] = ns_old + 1;
        } else if (ok) {
          if (flush) {
            p.page_table_w[(size_t)b * p.max_pages + np_old] = pid;
            p.n_pages_w[b] = np_old + 1;
            new_nr = 1;
          } else {
            new_nr = nr_old + 1;
          }
        }
        atomicExch(&p.n_resid_w[b], new_nr);
      }
    }
  }
}

}  // namespace kitty
