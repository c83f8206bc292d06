// Host-side exercise of libkitty's argument validation and split planning, meant to be built together with the
// library's host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU is touched: every call below
// either is a pure host query or is rejected before anything is enqueued).  Exit status 0 and the line "ok" on
// success; a failed expectation prints the line number.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "../../include/kitty.h"

#define EXPECT(cond)                                              \
  do {                                                            \
    if (!(cond)) {                                                \
      std::printf("failed at line %d: %s\n", __LINE__, #cond);    \
      return 1;                                                   \
    }                                                             \
  } while (0)

static kitty_layout layout_of(int hq, int hkv, int nb) {
  kitty_layout L;
  std::memset(&L, 0, sizeof L);
  L.head_dim = 128; L.page_size = 128; L.v_group = 128; L.n_boost = nb; L.residual_window = 128;
  L.n_q_heads = hq; L.n_kv_heads = hkv; L.rank_metric = 0; L.v_bits = 2;
  return L;
}

int main() {
  // record sizes, every supported boost count, both Value widths
  const int boosts[] = {0, 16, 32, 64, 128};
  for (int nb : boosts) {
    kitty_layout L = layout_of(32, 8, nb);
    EXPECT(kitty_page_bytes(&L) == (size_t)(9344 + 32 * nb));
    EXPECT(kitty_page_payload_bytes(&L) == (size_t)(9344 + 32 * nb - (128 - nb)));
  }
  kitty_layout L = layout_of(32, 8, 16);
  L.v_bits = 4;
  EXPECT(kitty_page_bytes(&L) == 9856 + 4096);
  EXPECT(kitty_page_bytes(nullptr) == 0);
  // every field pushed out of range in turn
  for (int field = 0; field < 11; ++field) {
    kitty_layout B = layout_of(32, 8, 16);
    int32_t* f = reinterpret_cast<int32_t*>(&B);
    static const int32_t bad[11] = {64, 64, 32, 24, 64, 30, 0, 2, 129, 64, 3};
    f[field] = bad[field];
    EXPECT(kitty_page_bytes(&B) == 0);
    int32_t ns = -1, mp = -1;
    EXPECT(kitty_decode_plan(&B, 4, 64, 0, &ns, &mp) < 0);
    EXPECT(kitty_decode_workspace_bytes(&B, 4, 64, 0) == 0);
  }
  // plans over a sweep of sizes: the workspace formula, ranges never empty, extreme arguments
  L = layout_of(64, 8, 32);
  const int32_t batches[] = {1, 2, 7, 32, 128, 65535};
  const int32_t pages[] = {0, 1, 15, 16, 255, 1023, 1 << 20};
  const int32_t reqs[] = {0, 1, 2, 8, 12, 1000, INT32_MAX};
  for (int32_t b : batches)
    for (int32_t p : pages)
      for (int32_t r : reqs) {
        int32_t ns = -1, mp = -1;
        EXPECT(kitty_decode_plan(&L, b, p, r, &ns, &mp) == KITTY_OK);
        EXPECT(ns >= 1 && mp >= 1 && (p == 0 || ns <= p) && (r == 0 || ns <= r));
        EXPECT(kitty_decode_workspace_bytes(&L, b, p, r) == (size_t)b * 64 * (size_t)ns * 130 * 4);
      }
  int32_t ns = 0, mp = 0;
  EXPECT(kitty_decode_plan(&L, 0, 8, 0, &ns, &mp) == KITTY_ERR_INVALID_ARG);
  EXPECT(kitty_decode_plan(&L, 4, -1, 0, &ns, &mp) == KITTY_ERR_INVALID_ARG);
  EXPECT(kitty_decode_plan(&L, 4, 8, -1, &ns, &mp) == KITTY_ERR_INVALID_ARG);
  EXPECT(kitty_decode_plan(&L, 4, 8, 0, nullptr, &mp) == KITTY_ERR_INVALID_ARG);
  EXPECT(kitty_decode_workspace_bytes(&L, -3, 8, 0) == 0);
  // entry points that would launch: every one must refuse these arguments on the host
  std::vector<unsigned char> fake(1 << 16);            // never dereferenced by the library on these paths
  unsigned char* base = fake.data();
  auto at = [&](size_t off) { return (void*)(((uintptr_t)base + 255) / 256 * 256 + off); };
  L = layout_of(32, 8, 16);
  EXPECT(kitty_quantize_pages(nullptr, at(0), at(0), 0, 0, 128, nullptr, (const int32_t*)at(0), 1, at(0), 1, nullptr) == KITTY_ERR_INVALID_ARG);
  EXPECT(kitty_quantize_pages(&L, nullptr, at(0), 0, 0, 128, nullptr, (const int32_t*)at(0), 1, at(0), 1, nullptr) == KITTY_ERR_INVALID_ARG);
  EXPECT(kitty_quantize_pages(&L, at(8), at(0), 16384, 16384, 128, nullptr, (const int32_t*)at(0), 1, at(0), 1, nullptr) == KITTY_ERR_INVALID_ARG);
  EXPECT(kitty_quantize_pages(&L, at(0), at(0), 16384, 16384, 132, nullptr, (const int32_t*)at(0), 1, at(0), 1, nullptr) == KITTY_ERR_INVALID_ARG);
  EXPECT(kitty_quantize_pages(&L, at(0), at(0), 16384, 16384, 64, nullptr, (const int32_t*)at(0), 1, at(0), 1, nullptr) == KITTY_ERR_INVALID_ARG);
  EXPECT(kitty_quantize_pages(&L, at(0), at(0), 16384, 16384, 128, nullptr, (const int32_t*)at(0), -1, at(0), 1, nullptr) == KITTY_ERR_INVALID_ARG);
  EXPECT(kitty_quantize_pages(&L, at(0), at(0), 16384, 16384, 128, nullptr, (const int32_t*)at(0), 0, at(0), 1, nullptr) == KITTY_OK);
  kitty_cache C;
  std::memset(&C, 0, sizeof C);
  C.batch = 4; C.max_pages = 8; C.n_pool_pages = 32;
  EXPECT(kitty_decode_attention(&L, &C, at(0), at(0), 1.f, 0, 0, at(0), 1 << 20, nullptr) == KITTY_ERR_INVALID_ARG);   // no state arrays
  EXPECT(kitty_decode_attention(&L, nullptr, at(0), at(0), 1.f, 0, 0, at(0), 1 << 20, nullptr) == KITTY_ERR_INVALID_ARG);
  C.page_pool = at(0); C.page_table = (int32_t*)at(256); C.n_pages = (int32_t*)at(512);
  C.resid_k = at(1024); C.resid_v = at(2048); C.n_resid = (int32_t*)at(768);
  EXPECT(kitty_decode_split(&L, &C, at(0), 1.f, 0, at(0), 64, nullptr) == KITTY_ERR_WORKSPACE);
  EXPECT(kitty_decode_split(&L, &C, at(0), 1.f, 0, at(4), 1 << 30, nullptr) == KITTY_ERR_INVALID_ARG);               // workspace alignment
  EXPECT(kitty_decode_split(&L, &C, at(0), 1.f, -2, at(0), 1 << 30, nullptr) == KITTY_ERR_INVALID_ARG);
  EXPECT(kitty_decode_split(&L, &C, nullptr, 1.f, 0, at(0), 1 << 30, nullptr) == KITTY_ERR_INVALID_ARG);
  EXPECT(kitty_decode_merge(&L, &C, at(0), 0, 7, at(0), 1 << 30, nullptr) == KITTY_ERR_INVALID_ARG);                  // out_dtype
  EXPECT(kitty_decode_attention(&L, &C, at(0), nullptr, 1.f, 0, 0, at(0), 1 << 30, nullptr) == KITTY_ERR_INVALID_ARG);
  EXPECT(kitty_append_token(&L, &C, nullptr, at(0), (const int32_t*)at(0), nullptr) == KITTY_ERR_INVALID_ARG);
  EXPECT(kitty_append_token(&L, &C, at(8), at(0), (const int32_t*)at(0), nullptr) == KITTY_ERR_INVALID_ARG);
  EXPECT(kitty_decode_step(&L, &C, at(0), at(0), nullptr, at(0), at(0), 1.f, 0, 0, at(0), 1 << 30, nullptr) == KITTY_ERR_INVALID_ARG);
  EXPECT(kitty_decode_step(&L, &C, at(0), at(0), (const int32_t*)at(0), at(0), at(0), 1.f, 0, 0, at(0), 16, nullptr) == KITTY_ERR_WORKSPACE);
  EXPECT(kitty_decode_step(&L, &C, at(0), at(0), (const int32_t*)at(0), at(8), at(0), 1.f, 0, 0, at(0), 1 << 30, nullptr) == KITTY_ERR_INVALID_ARG);
  kitty_layout S = layout_of(32, 8, 16);
  S.sink_tokens = 32;                                   // a Sink in the layout needs the Sink buffers
  EXPECT(kitty_decode_split(&S, &C, at(0), 1.f, 0, at(0), 1 << 30, nullptr) == KITTY_ERR_INVALID_ARG);
  kitty_layout R0 = layout_of(32, 8, 16);
  R0.residual_window = 0;
  EXPECT(kitty_append_token(&R0, &C, at(0), at(0), (const int32_t*)at(0), nullptr) == KITTY_ERR_UNSUPPORTED);
  // the entry point with the library's own workspace: plans beyond its size, bad arguments
  kitty_layout W = layout_of(64, 8, 32);
  kitty_cache CW = C;
  CW.batch = 64; CW.max_pages = 64;
  EXPECT(kitty_decode_workspace_bytes(&W, 64, 64, 8) > (size_t)KITTY_STATIC_WORKSPACE_BYTES);
  EXPECT(kitty_decode_attention_static(&W, &CW, at(0), at(0), 1.f, 8, 0, nullptr) == KITTY_ERR_WORKSPACE);
  EXPECT(kitty_decode_attention_static(&W, &CW, nullptr, at(0), 1.f, 1, 0, nullptr) == KITTY_ERR_INVALID_ARG);
  EXPECT(kitty_decode_attention_static(&W, &CW, at(0), at(0), 1.f, 1, 2, nullptr) == KITTY_ERR_INVALID_ARG);
  for (int code = -6; code <= 1; ++code) EXPECT(std::strlen(kitty_strerror(code)) > 0);
  std::printf("ok\n");
  return 0;
}

// The library's host code is built here without its device code (host pass only).  The references of its translation
// units to their device images are satisfied by empty stand-ins that the test generates (one per unit, named after
// the unit's compilation id); they are never looked at because nothing is launched.
