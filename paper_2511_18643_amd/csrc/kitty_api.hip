// Host side of libkitty: argument validation, split planning and kernel launches (gfx950).
#include "../../include/kitty.h"

#include <mutex>
#include <type_traits>

#include "kitty_launch.h"
#include "kitty_merge.h"

namespace {

using namespace kitty;

int check_layout(const kitty_layout* L) {
  if (!L) return KITTY_ERR_INVALID_ARG;
  if (L->n_q_heads <= 0 || L->n_kv_heads <= 0 || L->n_q_heads % L->n_kv_heads != 0) return KITTY_ERR_INVALID_ARG;
  if (L->n_boost < 0 || L->n_boost > L->head_dim || L->n_boost % 16 != 0) return KITTY_ERR_INVALID_ARG;
  if (L->rank_metric != 0 && L->rank_metric != 1) return KITTY_ERR_INVALID_ARG;
  if (L->head_dim != D || L->page_size != G || L->v_group != D) return KITTY_ERR_UNSUPPORTED;
  if (L->residual_window != 0 && L->residual_window != G) return KITTY_ERR_UNSUPPORTED;
  const int nb16 = L->n_boost / 16;
  const int g = L->n_q_heads / L->n_kv_heads;
  if (g > 8) return KITTY_ERR_UNSUPPORTED;   // a block holds the heads of a group in 4 or 8 slots; unused slots carry a zero query
  if (L->sink_tokens < 0 || L->v_local < 0) return KITTY_ERR_INVALID_ARG;
  if (L->sink_tokens > G) return KITTY_ERR_UNSUPPORTED;
  if (L->v_local != 0 && (L->v_local != G || L->residual_window != G)) return KITTY_ERR_UNSUPPORTED;
  if (L->v_bits != 0 && L->v_bits != 2 && L->v_bits != 4) return KITTY_ERR_INVALID_ARG;
  return KITTY_OK;
}

int check_cache(const kitty_layout* L, const kitty_cache* C) {
  if (!C) return KITTY_ERR_INVALID_ARG;
  if (C->batch <= 0 || C->max_pages < 0 || C->n_pool_pages < 0) return KITTY_ERR_INVALID_ARG;
  if (!C->n_pages) return KITTY_ERR_INVALID_ARG;
  if (C->max_pages > 0 && (!C->page_pool || !C->page_table)) return KITTY_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(C->page_pool) % 128 != 0) return KITTY_ERR_INVALID_ARG;
  if (L->residual_window > 0) {
    if (!C->resid_k || !C->resid_v || !C->n_resid) return KITTY_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(C->resid_k) % 16 != 0 || reinterpret_cast<uintptr_t>(C->resid_v) % 16 != 0)
      return KITTY_ERR_INVALID_ARG;
  }
  if (L->sink_tokens > 0) {
    if (!C->sink_k || !C->sink_v || !C->n_sink) return KITTY_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(C->sink_k) % 16 != 0 || reinterpret_cast<uintptr_t>(C->sink_v) % 16 != 0)
      return KITTY_ERR_INVALID_ARG;
  }
  return KITTY_OK;
}

int num_compute_units() {
  static int cus = 0;   // read once; the value never changes for a device
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      cus = n;
    else
      cus = 256;
  }
  return cus;
}

// Blocks of 8 wavefronts when a range can feed them (>= 4 pages per wavefront), else 4.  A grid with more blocks
// than compute units (a large or variable-length batch) also takes 4: two such blocks share a compute unit, so
// one block's start-up and tail run under the other's streaming, and no compute unit waits for a second round of
// whole 8-wavefront blocks (measured on 32k-token sequences: -14 % at 1.25 blocks per compute unit, -1 % at 2,
// -4 % at 3, -2 % on the variable-length 36-layer loop at 4).
int waves_per_block(int32_t max_pages, int32_t n_splits, int64_t blocks) {
  if (blocks > (int64_t)num_compute_units()) return 4;
  return max_pages / (n_splits > 0 ? n_splits : 1) >= 32 ? 8 : 4;
}

// n_splits page ranges per (sequence, kv-head); a range never covers fewer than min_pages pages
// unless the sequence has fewer (see active_splits in the kernels).
void plan_splits(const kitty_layout* L, int32_t batch, int32_t max_pages, int32_t req, int32_t* n_splits, int32_t* min_pages) {
  int32_t ns, mp;
  if (req > 0) {
    ns = req;
    mp = 1;
  } else {
    // fill the chip once with 8 wavefronts per compute unit (measured: streams best); one range per
    // (sequence, kv-head) whenever there are enough of them, which also makes the merge pass unnecessary
    const int64_t pairs = (int64_t)batch * L->n_kv_heads;
    const int64_t slots = (int64_t)num_compute_units();
    int64_t want = (slots + pairs - 1) / pairs;
    // a range has at least four pages (one per wavefront of a 4-wavefront block): small problems are all latency,
    // and more, shorter ranges shorten it (one 8k-token sequence: 19.4 us with 4 ranges of 16 pages, 14.1 us with 16)
    mp = 4;
    if (want > max_pages / mp) want = max_pages / mp;
    ns = (int32_t)want;
  }
  if (ns > max_pages) ns = max_pages;
  if (ns < 1) ns = 1;
  *n_splits = ns;
  *min_pages = mp;
}

bool v4_of(const kitty_layout* L) { return L->v_bits == 4; }

// f(number of 16-channel boost blocks, 4-bit Values?) with both as compile-time constants
template <typename F>
int dispatch_variant(const kitty_layout* L, F&& f) {
  const int nb16 = L->n_boost / 16;
  if (v4_of(L)) {
    switch (nb16) {
      case 0: return f(std::integral_constant<int, 0>{}, std::true_type{});
      case 1: return f(std::integral_constant<int, 1>{}, std::true_type{});
      case 2: return f(std::integral_constant<int, 2>{}, std::true_type{});
      case 3: return f(std::integral_constant<int, 3>{}, std::true_type{});
      case 4: return f(std::integral_constant<int, 4>{}, std::true_type{});
      case 5: return f(std::integral_constant<int, 5>{}, std::true_type{});
      case 6: return f(std::integral_constant<int, 6>{}, std::true_type{});
      case 7: return f(std::integral_constant<int, 7>{}, std::true_type{});
      case 8: return f(std::integral_constant<int, 8>{}, std::true_type{});
    }
    return KITTY_ERR_UNSUPPORTED;
  }
  switch (nb16) {
    case 0: return f(std::integral_constant<int, 0>{}, std::false_type{});
    case 1: return f(std::integral_constant<int, 1>{}, std::false_type{});
    case 2: return f(std::integral_constant<int, 2>{}, std::false_type{});
    case 3: return f(std::integral_constant<int, 3>{}, std::false_type{});
    case 4: return f(std::integral_constant<int, 4>{}, std::false_type{});
    case 5: return f(std::integral_constant<int, 5>{}, std::false_type{});
    case 6: return f(std::integral_constant<int, 6>{}, std::false_type{});
    case 7: return f(std::integral_constant<int, 7>{}, std::false_type{});
    case 8: return f(std::integral_constant<int, 8>{}, std::false_type{});
  }
  return KITTY_ERR_UNSUPPORTED;
}

int launch_status() { return hipGetLastError() == hipSuccess ? KITTY_OK : KITTY_ERR_HIP; }

int fill_decode_params(const kitty_layout* L, const kitty_cache* C, int32_t n_splits_req, const void* ws,
                       size_t ws_bytes, DecodeParams* P) {
  int rc = check_layout(L);
  if (rc) return rc;
  rc = check_cache(L, C);
  if (rc) return rc;
  if (n_splits_req < 0) return KITTY_ERR_INVALID_ARG;
  if (!ws || reinterpret_cast<uintptr_t>(ws) % 16 != 0) return KITTY_ERR_INVALID_ARG;
  int32_t ns, pps;
  plan_splits(L, C->batch, C->max_pages, n_splits_req, &ns, &pps);
  const size_t need = kitty_decode_workspace_bytes(L, C->batch, C->max_pages, n_splits_req);
  if (ws_bytes < need) return KITTY_ERR_WORKSPACE;
  P->pool = static_cast<const uint8_t*>(C->page_pool);
  P->page_table = C->page_table;
  P->n_pages = C->n_pages;
  P->resid_k = static_cast<const uint16_t*>(C->resid_k);
  P->resid_v = static_cast<const uint16_t*>(C->resid_v);
  P->n_resid = C->n_resid;
  P->sink_k = static_cast<const uint16_t*>(C->sink_k);
  P->sink_v = static_cast<const uint16_t*>(C->sink_v);
  P->n_sink = C->n_sink;
  P->seq_order = C->seq_order;
  P->sink_cap = L->sink_tokens;
  P->v_local = L->v_local ? 1 : 0;
  P->sink_k_w = P->sink_v_w = nullptr;
  P->n_sink_w = nullptr;
  P->q = nullptr;
  P->ws = const_cast<float*>(static_cast<const float*>(ws));
  P->out = nullptr;
  P->qk_scale_log2 = 0.f;
  P->batch = C->batch;
  P->max_pages = C->max_pages;
  P->n_q_heads = L->n_q_heads;
  P->n_kv_heads = L->n_kv_heads;
  P->gqa = L->n_q_heads / L->n_kv_heads;
  P->n_splits = ns;
  P->min_pages = pps;
  P->has_window = L->residual_window > 0 ? 1 : 0;
  P->out_dtype = 0;
  P->direct_out = 0;
  P->k_new = P->v_new = nullptr;
  P->fresh_page_ids = nullptr;
  P->pool_w = nullptr;
  P->page_table_w = nullptr;
  P->n_pages_w = nullptr;
  P->resid_k_w = P->resid_v_w = nullptr;
  P->n_resid_w = nullptr;
  P->n_pool_pages = C->n_pool_pages;
  P->rank_metric = L->rank_metric;
  return KITTY_OK;
}

}  // namespace

// ---- workspace of kitty_decode_attention_static: a fixed array in the library's device image -------------------
// In host code the array's name is only a handle for hipGetSymbolAddress; the address each GPU holds its copy at
// is looked up once per device (with that device current) and kept, and only that pointer is ever given to a
// kernel.
static __device__ __align__(256) float scratch[KITTY_STATIC_WORKSPACE_BYTES / sizeof(float)];

namespace {
constexpr int MAX_DEVICES = 64;
float* scratch_ptr[MAX_DEVICES];   // device address of `scratch` on each GPU, nullptr until first use there
std::mutex scratch_mutex;

int static_workspace(float** ws) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return KITTY_ERR_HIP;
  std::lock_guard<std::mutex> guard(scratch_mutex);
  if (!scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return KITTY_ERR_HIP;
    scratch_ptr[dev] = static_cast<float*>(ptr);
  }
  *ws = scratch_ptr[dev];
  return KITTY_OK;
}
}  // namespace

extern "C" {

size_t kitty_page_bytes(const kitty_layout* L) {
  if (check_layout(L) != KITTY_OK) return 0;
  return (size_t)record_bytes(L->n_boost / 16, v4_of(L));
}

size_t kitty_page_payload_bytes(const kitty_layout* L) {
  if (check_layout(L) != KITTY_OK) return 0;
  return (size_t)record_bytes(L->n_boost / 16, v4_of(L)) - (size_t)(128 - L->n_boost);
}

int kitty_decode_plan(const kitty_layout* L, int32_t batch, int32_t max_pages, int32_t n_splits_req,
                      int32_t* n_splits, int32_t* pages_per_split) {
  int rc = check_layout(L);
  if (rc) return rc;
  if (!n_splits || !pages_per_split || batch <= 0 || max_pages < 0 || n_splits_req < 0) return KITTY_ERR_INVALID_ARG;
  plan_splits(L, batch, max_pages, n_splits_req, n_splits, pages_per_split);
  return KITTY_OK;
}

size_t kitty_decode_workspace_bytes(const kitty_layout* L, int32_t batch, int32_t max_pages, int32_t n_splits_req) {
  if (check_layout(L) != KITTY_OK || batch <= 0 || max_pages < 0 || n_splits_req < 0) return 0;
  int32_t ns, pps;
  plan_splits(L, batch, max_pages, n_splits_req, &ns, &pps);
  return (size_t)batch * L->n_q_heads * (size_t)ns * WS_STRIDE * sizeof(float);
}

int kitty_quantize_pages(const kitty_layout* L, const void* k_src, const void* v_src, int64_t page_stride,
                         int64_t head_stride, int64_t token_stride, const int64_t* src_page_offsets,
                         const int32_t* dst_page_ids, int32_t n_pages, void* page_pool, int32_t n_pool_pages,
                         void* hip_stream) {
  int rc = check_layout(L);
  if (rc) return rc;
  if (n_pages < 0 || n_pool_pages < 0) return KITTY_ERR_INVALID_ARG;
  if (n_pages == 0) return KITTY_OK;
  if (!k_src || !v_src || !dst_page_ids || !page_pool) return KITTY_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(k_src) % 16 || reinterpret_cast<uintptr_t>(v_src) % 16 ||
      reinterpret_cast<uintptr_t>(page_pool) % 128)
    return KITTY_ERR_INVALID_ARG;
  if (token_stride < D || token_stride % 8 || head_stride % 8 || (!src_page_offsets && page_stride % 8))
    return KITTY_ERR_INVALID_ARG;
  if ((int64_t)n_pages * L->n_kv_heads > INT32_MAX) return KITTY_ERR_UNSUPPORTED;
  QuantPagesParams P;
  P.k_src = static_cast<const uint16_t*>(k_src);
  P.v_src = static_cast<const uint16_t*>(v_src);
  P.page_stride = page_stride;
  P.head_stride = head_stride;
  P.token_stride = token_stride;
  P.src_page_offsets = src_page_offsets;
  P.dst_page_ids = dst_page_ids;
  P.pool = static_cast<uint8_t*>(page_pool);
  P.n_kv_heads = L->n_kv_heads;
  P.n_pool_pages = n_pool_pages;
  P.rank_metric = L->rank_metric;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  return dispatch_variant(L, [&](auto nb, auto v4) {
    constexpr int NB = decltype(nb)::value;
    constexpr bool V4 = decltype(v4)::value;
    launch_quantize_pages<NB, V4>(P, (unsigned)((int64_t)n_pages * L->n_kv_heads), st);
    return launch_status();
  });
}

int kitty_project_quantize_pages(const kitty_layout* L, const void* x, int64_t x_token_stride, int32_t hidden,
                                 const void* w_k, const void* w_v, const int64_t* src_token_offsets,
                                 const int32_t* dst_page_ids, int32_t n_pages, void* page_pool, int32_t n_pool_pages,
                                 void* hip_stream) {
  int rc = check_layout(L);
  if (rc) return rc;
  if (n_pages < 0 || n_pool_pages < 0) return KITTY_ERR_INVALID_ARG;
  if (n_pages == 0) return KITTY_OK;
  if (!x || !w_k || !w_v || !src_token_offsets || !dst_page_ids || !page_pool) return KITTY_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(x) % 16 || reinterpret_cast<uintptr_t>(w_k) % 16 || reinterpret_cast<uintptr_t>(w_v) % 16 ||
      reinterpret_cast<uintptr_t>(page_pool) % 128)
    return KITTY_ERR_INVALID_ARG;
  if (hidden <= 0 || x_token_stride < hidden || x_token_stride % 8) return KITTY_ERR_INVALID_ARG;
  if (hidden % PJ_KC) return KITTY_ERR_UNSUPPORTED;
  if (L->n_kv_heads > 65535) return KITTY_ERR_UNSUPPORTED;
  ProjectParams P;
  P.x = static_cast<const uint16_t*>(x);
  P.w_k = static_cast<const uint16_t*>(w_k);
  P.w_v = static_cast<const uint16_t*>(w_v);
  P.x_token_stride = x_token_stride;
  P.src_token_offsets = src_token_offsets;
  P.dst_page_ids = dst_page_ids;
  P.pool = static_cast<uint8_t*>(page_pool);
  P.hidden = hidden;
  P.n_kv_heads = L->n_kv_heads;
  P.n_pool_pages = n_pool_pages;
  P.rank_metric = L->rank_metric;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  return dispatch_variant(L, [&](auto nb, auto v4) {
    constexpr int NB = decltype(nb)::value;
    constexpr bool V4 = decltype(v4)::value;
    launch_project_quantize_pages<NB, V4>(P, dim3(n_pages, L->n_kv_heads), st);
    return launch_status();
  });
}

int kitty_append_token(const kitty_layout* L, const kitty_cache* C, const void* k_new, const void* v_new,
                       const int32_t* fresh_page_ids, void* hip_stream) {
  int rc = check_layout(L);
  if (rc) return rc;
  rc = check_cache(L, C);
  if (rc) return rc;
  if (L->residual_window != G) return KITTY_ERR_UNSUPPORTED;
  if (!k_new || !v_new || !fresh_page_ids || !C->page_pool || !C->page_table) return KITTY_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(k_new) % 16 || reinterpret_cast<uintptr_t>(v_new) % 16) return KITTY_ERR_INVALID_ARG;
  if (L->n_kv_heads > 65535 || C->batch > 65535) return KITTY_ERR_UNSUPPORTED;
  AppendParams P;
  P.pool = static_cast<uint8_t*>(C->page_pool);
  P.page_table = C->page_table;
  P.n_pages = C->n_pages;
  P.resid_k = static_cast<uint16_t*>(C->resid_k);
  P.resid_v = static_cast<uint16_t*>(C->resid_v);
  P.n_resid = C->n_resid;
  P.sink_k = static_cast<uint16_t*>(C->sink_k);
  P.sink_v = static_cast<uint16_t*>(C->sink_v);
  P.n_sink = C->n_sink;
  P.sink_cap = L->sink_tokens;
  P.v_local = L->v_local ? 1 : 0;
  P.k_new = static_cast<const uint16_t*>(k_new);
  P.v_new = static_cast<const uint16_t*>(v_new);
  P.fresh_page_ids = fresh_page_ids;
  P.batch = C->batch;
  P.max_pages = C->max_pages;
  P.n_pool_pages = C->n_pool_pages;
  P.n_kv_heads = L->n_kv_heads;
  P.rank_metric = L->rank_metric;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  return dispatch_variant(L, [&](auto nb, auto v4) {
    constexpr int NB = decltype(nb)::value;
    constexpr bool V4 = decltype(v4)::value;
    launch_append_token<NB, V4>(P, dim3(L->n_kv_heads, C->batch), st);
    return launch_status();
  });
}

namespace {
struct StepArgs {   // the append half of a fused step
  const void* k_new;
  const void* v_new;
  const int32_t* fresh_page_ids;
};

// Launches the streaming kernel.  With `out` non-null and a one-range plan the kernel stores the result itself;
// with `step` non-null it also performs the append first (with several ranges: the flush only; the merge launch
// that follows stores the token and advances the state).
int launch_split(const kitty_layout* L, const kitty_cache* C, const void* q, float sm_scale, int32_t n_splits,
                 void* workspace, size_t workspace_bytes, void* out, int32_t out_dtype, void* hip_stream, bool* merged,
                 const StepArgs* step) {
  DecodeParams P;
  int rc = fill_decode_params(L, C, n_splits, workspace, workspace_bytes, &P);
  if (rc) return rc;
  if (!q || reinterpret_cast<uintptr_t>(q) % 16) return KITTY_ERR_INVALID_ARG;
  if (L->n_kv_heads > 65535 || C->batch > 65535) return KITTY_ERR_UNSUPPORTED;
  P.q = static_cast<const uint16_t*>(q);
  P.qk_scale_log2 = sm_scale * 1.44269504088896340736f;
  P.direct_out = (out && P.n_splits == 1) ? 1 : 0;
  P.out = out;
  P.out_dtype = out_dtype;
  if (merged) *merged = P.direct_out != 0;
  if (step) {
    P.k_new = static_cast<const uint16_t*>(step->k_new);
    P.v_new = static_cast<const uint16_t*>(step->v_new);
    P.fresh_page_ids = step->fresh_page_ids;
    P.pool_w = static_cast<uint8_t*>(C->page_pool);
    P.page_table_w = C->page_table;
    P.n_pages_w = C->n_pages;
    P.resid_k_w = static_cast<uint16_t*>(C->resid_k);
    P.resid_v_w = static_cast<uint16_t*>(C->resid_v);
    P.n_resid_w = C->n_resid;
    P.sink_k_w = static_cast<uint16_t*>(C->sink_k);
    P.sink_v_w = static_cast<uint16_t*>(C->sink_v);
    P.n_sink_w = C->n_sink;
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  SplitLaunch sl;
  sl.grid = dim3(P.n_splits, L->n_kv_heads, C->batch);
  sl.wide = P.gqa > 4;   // more than four query heads per kv-head: eight head slots per block
  sl.big = waves_per_block(C->max_pages, P.n_splits, (int64_t)P.n_splits * L->n_kv_heads * C->batch) == 8;
  sl.row_wave = !L->v_local;
  sl.fused = step == nullptr ? 0 : (P.direct_out ? 1 : 2);
  return dispatch_variant(L, [&](auto nb, auto v4) {
    launch_decode_split<decltype(nb)::value, decltype(v4)::value>(P, sl, st);
    return launch_status();
  });
}
}  // namespace

int kitty_decode_split(const kitty_layout* L, const kitty_cache* C, const void* q, float sm_scale, int32_t n_splits,
                       void* workspace, size_t workspace_bytes, void* hip_stream) {
  return launch_split(L, C, q, sm_scale, n_splits, workspace, workspace_bytes, nullptr, 0, hip_stream, nullptr, nullptr);
}

int kitty_decode_merge(const kitty_layout* L, const kitty_cache* C, void* out, int32_t n_splits, int32_t out_dtype,
                       const void* workspace, size_t workspace_bytes, void* hip_stream) {
  DecodeParams P;
  int rc = fill_decode_params(L, C, n_splits, workspace, workspace_bytes, &P);
  if (rc) return rc;
  if (!out || (out_dtype != 0 && out_dtype != 1)) return KITTY_ERR_INVALID_ARG;
  if (L->n_q_heads > 65535 * 8 || C->batch > 65535) return KITTY_ERR_UNSUPPORTED;
  P.out = out;
  P.out_dtype = out_dtype;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (P.n_splits > 8) hipLaunchKernelGGL(decode_merge_kernel<true>, dim3(L->n_q_heads, C->batch), dim3(128), 0, st, P);
  else hipLaunchKernelGGL(decode_merge_kernel<false>, dim3(L->n_q_heads, C->batch), dim3(128), 0, st, P);
  return launch_status();
}

int kitty_decode_attention(const kitty_layout* L, const kitty_cache* C, const void* q, void* out, float sm_scale,
                           int32_t n_splits, int32_t out_dtype, void* workspace, size_t workspace_bytes,
                           void* hip_stream) {
  if (!out || (out_dtype != 0 && out_dtype != 1)) return KITTY_ERR_INVALID_ARG;
  bool merged = false;
  int rc = launch_split(L, C, q, sm_scale, n_splits, workspace, workspace_bytes, out, out_dtype, hip_stream, &merged, nullptr);
  if (rc || merged) return rc;
  return kitty_decode_merge(L, C, out, n_splits, out_dtype, workspace, workspace_bytes, hip_stream);
}

int kitty_decode_step(const kitty_layout* L, const kitty_cache* C, const void* k_new, const void* v_new,
                      const int32_t* fresh_page_ids, const void* q, void* out, float sm_scale, int32_t n_splits,
                      int32_t out_dtype, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_layout(L);
  if (rc) return rc;
  rc = check_cache(L, C);
  if (rc) return rc;
  if (L->residual_window != G) return KITTY_ERR_UNSUPPORTED;
  if (!k_new || !v_new || !fresh_page_ids || !C->page_pool || !C->page_table) return KITTY_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(k_new) % 16 || reinterpret_cast<uintptr_t>(v_new) % 16) return KITTY_ERR_INVALID_ARG;
  if (!out || (out_dtype != 0 && out_dtype != 1) || n_splits < 0) return KITTY_ERR_INVALID_ARG;
  // Everything either launch could reject is checked here, before the first one: once the streaming kernel is
  // enqueued (it may flush a window into the fresh page) the merge launch that stores the token and advances the
  // state must follow.
  DecodeParams P;
  rc = fill_decode_params(L, C, n_splits, workspace, workspace_bytes, &P);
  if (rc) return rc;
  if (!q || reinterpret_cast<uintptr_t>(q) % 16) return KITTY_ERR_INVALID_ARG;
  if (L->n_kv_heads > 65535 || C->batch > 65535) return KITTY_ERR_UNSUPPORTED;   // grid limits of both launches
  const StepArgs step{k_new, v_new, fresh_page_ids};
  bool merged = false;
  rc = launch_split(L, C, q, sm_scale, n_splits, workspace, workspace_bytes, out, out_dtype, hip_stream, &merged, &step);
  if (rc || merged) return rc;
  // several ranges: the merge launch also stores the token and advances the state
  P.out = out;
  P.out_dtype = out_dtype;
  P.k_new = static_cast<const uint16_t*>(k_new);
  P.v_new = static_cast<const uint16_t*>(v_new);
  P.fresh_page_ids = fresh_page_ids;
  P.page_table_w = C->page_table;
  P.n_pages_w = C->n_pages;
  P.resid_k_w = static_cast<uint16_t*>(C->resid_k);
  P.resid_v_w = static_cast<uint16_t*>(C->resid_v);
  P.n_resid_w = C->n_resid;
  P.sink_k_w = static_cast<uint16_t*>(C->sink_k);
  P.sink_v_w = static_cast<uint16_t*>(C->sink_v);
  P.n_sink_w = C->n_sink;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (P.n_splits > 8) hipLaunchKernelGGL(decode_merge_step_kernel<true>, dim3(L->n_q_heads, C->batch), dim3(128), 0, st, P);
  else hipLaunchKernelGGL(decode_merge_step_kernel<false>, dim3(L->n_q_heads, C->batch), dim3(128), 0, st, P);
  return launch_status();
}

int kitty_decode_attention_static(const kitty_layout* L, const kitty_cache* C, const void* q, void* out, float sm_scale,
                                  int32_t n_splits, int32_t out_dtype, void* hip_stream) {
  int rc = check_layout(L);
  if (rc) return rc;
  rc = check_cache(L, C);
  if (rc) return rc;
  if (n_splits < 0 || !q || reinterpret_cast<uintptr_t>(q) % 16 || !out || (out_dtype != 0 && out_dtype != 1))
    return KITTY_ERR_INVALID_ARG;
  if (L->n_kv_heads > 65535 || C->batch > 65535) return KITTY_ERR_UNSUPPORTED;
  const size_t need = kitty_decode_workspace_bytes(L, C->batch, C->max_pages, n_splits);
  if (need > (size_t)KITTY_STATIC_WORKSPACE_BYTES) return KITTY_ERR_WORKSPACE;
  float* ws = nullptr;
  rc = static_workspace(&ws);
  if (rc) return rc;
  return kitty_decode_attention(L, C, q, out, sm_scale, n_splits, out_dtype, ws, (size_t)KITTY_STATIC_WORKSPACE_BYTES,
                                hip_stream);
}

const char* kitty_strerror(int code) {
  switch (code) {
    case KITTY_OK: return "ok";
    case KITTY_ERR_INVALID_ARG: return "invalid argument (null pointer, bad alignment or inconsistent sizes)";
    case KITTY_ERR_UNSUPPORTED: return "unsupported size (head_dim, page_size, residual window, Sink, Local window, boost count, Value bits or GQA group)";
    case KITTY_ERR_WORKSPACE: return "workspace too small";
    case KITTY_ERR_HIP: return "HIP launch failed";
  }
  return "unknown error";
}

}  // extern "C"
