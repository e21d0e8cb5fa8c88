// C ABI of the Flash-LoRA-Attention library: argument checks, launch planning,
// kernel selection.  Declarations and argument contracts are in lra_attn.h.
#include <cmath>
#include <cstdlib>
#include <mutex>

#include "lra_attn.h"
#include "lra_attn_measure.h"
#include "lra_common.h"
#include "lra_plan.h"

namespace lra {

#ifdef LRA_TIMING
static unsigned long long* g_timing = nullptr;  // instrumented test build only
#endif

static void fill_params(Params& p, const lra_shape* sh, const lra_cache* c, const lra_adapters* ad,
                        const Plan& pl, void* workspace) {
  p.k_base = c->k_base;
  p.v_base = c->v_base;
  p.l = c->l;
  p.b_k = ad->b_k;
  p.b_v = ad->b_v;
  p.n_adapters = ad->n_adapters;
  p.block_table = c->block_table;
  p.seq_lens = c->seq_lens;
  char* ws = static_cast<char*>(workspace);
  p.part_ml = reinterpret_cast<float*>(ws + pl.off_ml);
  p.part_o = reinterpret_cast<float*>(ws + pl.off_o);
  p.part_lr = reinterpret_cast<float*>(ws + pl.off_lr);
  p.part_adapter = reinterpret_cast<int32_t*>(ws + pl.off_adapter);
  p.qt_ws = (pl.qt_bytes > 0 && ad->b_k != nullptr) ? ws + pl.off_qt : nullptr;
  p.kv_token_stride = c->kv_token_stride;
  p.kv_head_stride = c->kv_head_stride;
  p.kv_block_stride = c->kv_block_stride;
  p.l_row_stride = c->l_row_stride ? c->l_row_stride : sh->rank;
  p.l_adapter_stride = c->l_adapter_stride;
  p.l_block = pl.l_block;
  // wide L rows (64 bytes per token and more, or one low-rank cache per adapter): the kv heads of a key share on one XCD
  p.share_major = (sh->rank >= 32 || pl.l_block != 0) ? 1 : 0;
  p.n_q_heads = sh->n_q_heads;
  p.n_kv_heads = sh->n_kv_heads;
  p.group = sh->n_q_heads / sh->n_kv_heads;
  p.head_dim = sh->head_dim;
  p.rank = sh->rank;
  p.block_size = c->block_size;
  p.max_blocks_per_seq = c->max_blocks_per_seq;
  p.num_blocks = c->num_blocks;
  p.n_seqs = c->n_seqs;
  p.max_seq_len = c->max_seq_len;
  p.group_pad = pl.group_pad;
  p.row_groups = pl.row_groups;
  p.split_keys = pl.split_keys;
  p.n_splits = pl.n_splits;
  p.scale = sh->scale > 0.f ? sh->scale : 1.0f / std::sqrt(static_cast<float>(sh->head_dim));
  p.key_rope_theta = sh->key_rope_theta;
#ifdef LRA_TIMING
  p.timing = g_timing;
#endif
}

static lra_status check_workspace(const Plan& pl, void* workspace, size_t workspace_bytes) {
  if (pl.bytes == 0) return LRA_OK;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) || workspace_bytes < pl.bytes)
    return LRA_ERR_WORKSPACE;
  return LRA_OK;
}

// Workspace of lra_attn_decode_static: part of the device image, one copy per GPU.  In host
// code the array's name is only a handle for hipGetSymbolAddress; the address a kernel may use
// is looked up once per device (with that device current) and kept.
static __device__ __align__(256) unsigned char scratch[LRA_STATIC_WORKSPACE_BYTES];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices] = {};

static lra_status scratch_of_current_device(void** ptr) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LRA_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* found = nullptr;
    if (hipGetSymbolAddress(&found, HIP_SYMBOL(scratch)) != hipSuccess || found == nullptr) return LRA_ERR_HIP;
    g_scratch_ptr[dev] = found;
  }
  *ptr = g_scratch_ptr[dev];
  return LRA_OK;
}

}  // namespace lra

using namespace lra;

extern "C" {

size_t lra_workspace_bytes(const lra_shape* shape, const lra_cache* cache, int32_t n_queries,
                           int32_t max_queries_per_seq, int32_t n_new, const lra_tuning* tuning) {
  if (check_common(shape, cache) != LRA_OK) return static_cast<size_t>(-1);
  if (n_new < 0 || n_new > cache->max_seq_len) return static_cast<size_t>(-1);
  if (n_new == 0 && (n_queries < 1 || max_queries_per_seq < 1 || max_queries_per_seq > n_queries))
    return static_cast<size_t>(-1);
  const bool prefill = n_new > 0;
  if (!plan_sizes_fit(shape, cache, prefill ? n_new : n_queries, prefill ? 1 : max_queries_per_seq))
    return static_cast<size_t>(-1);
  return make_plan(shape, cache, prefill ? n_new : n_queries, prefill ? 1 : max_queries_per_seq, prefill,
                   resolve_tuning(tuning)).bytes;
}

// Both decode entry points: checks, plan, then the workspace from the caller or, with
// `use_static`, the library's own per-device buffer.
static lra_status decode_call(const lra_shape* shape, const lra_cache* cache, const lra_adapters* adapters,
                              const void* q, const int32_t* query_adapter, const int32_t* seq_query_start,
                              int32_t n_queries, int32_t max_queries_per_seq, void* out, void* workspace,
                              size_t workspace_bytes, bool use_static, const lra_tuning* tuning, void* stream) {
  lra_status st = check_common(shape, cache);
  if (st != LRA_OK) return st;
  if (!adapters || !q || !query_adapter || !seq_query_start || !out) return LRA_ERR_NULL;
  if (adapters->n_adapters < 1 || n_queries < 1) return LRA_ERR_SHAPE;
  if (max_queries_per_seq < 1 || max_queries_per_seq > n_queries) return LRA_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(out) |
       reinterpret_cast<uintptr_t>(adapters->b_k) | reinterpret_cast<uintptr_t>(adapters->b_v)) & 15)
    return LRA_ERR_SHAPE;
  if (!plan_sizes_fit(shape, cache, n_queries, max_queries_per_seq)) return LRA_ERR_UNSUPPORTED;
  const Tuning tune = resolve_tuning(tuning);
  const Plan pl = make_plan(shape, cache, n_queries, max_queries_per_seq, false, tune);
  if (!pl.launchable) return LRA_ERR_UNSUPPORTED;
  if (use_static) {
    if (pl.bytes > LRA_STATIC_WORKSPACE_BYTES) return LRA_ERR_WORKSPACE;
    st = scratch_of_current_device(&workspace);
    if (st != LRA_OK) return st;
    workspace_bytes = LRA_STATIC_WORKSPACE_BYTES;
  }
  st = check_workspace(pl, workspace, workspace_bytes);
  if (st != LRA_OK) return st;

  Params p{};
  fill_params(p, shape, cache, adapters, pl, workspace);
  p.q = q;
  p.out = out;
  p.query_adapter = query_adapter;
  p.seq_query_start = seq_query_start;
  p.n_queries = n_queries;
  p.max_queries_per_seq = max_queries_per_seq;
  p.n_new = 1;
  p.is_prefill = 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool bf16 = shape->dtype == LRA_BF16;
  if (pl.mfma) {
    if (launch_decode_mfma(p, pl.row_tiles, tune.variant != 2, tune.main_kernel_only, s) != hipSuccess) return LRA_ERR_HIP;
  } else {
    if (launch_generic_partials(p, bf16, pl.rows, s) != hipSuccess) return LRA_ERR_HIP;
  }
  if (tune.main_kernel_only) return LRA_OK;  // measurement: key-streaming kernel alone
  if (launch_merge(p, bf16, pl.rows, s) != hipSuccess) return LRA_ERR_HIP;
  return LRA_OK;
}

lra_status lra_attn_decode(const lra_shape* shape, const lra_cache* cache, const lra_adapters* adapters,
                           const void* q, const int32_t* query_adapter, const int32_t* seq_query_start,
                           int32_t n_queries, int32_t max_queries_per_seq, void* out, void* workspace,
                           size_t workspace_bytes, const lra_tuning* tuning, void* stream) {
  return decode_call(shape, cache, adapters, q, query_adapter, seq_query_start, n_queries, max_queries_per_seq, out,
                     workspace, workspace_bytes, false, tuning, stream);
}

lra_status lra_attn_decode_static(const lra_shape* shape, const lra_cache* cache, const lra_adapters* adapters,
                                  const void* q, const int32_t* query_adapter, const int32_t* seq_query_start,
                                  int32_t n_queries, int32_t max_queries_per_seq, void* out,
                                  const lra_tuning* tuning, void* stream) {
  return decode_call(shape, cache, adapters, q, query_adapter, seq_query_start, n_queries, max_queries_per_seq, out,
                     nullptr, 0, true, tuning, stream);
}

lra_status lra_attn_prefill(const lra_shape* shape, const lra_cache* cache, const lra_adapters* adapters,
                            const void* q, int32_t seq_index, int32_t adapter_index, int32_t n_new,
                            void* out, void* workspace, size_t workspace_bytes, const lra_tuning* tuning,
                            void* stream) {
  lra_status st = check_common(shape, cache);
  if (st != LRA_OK) return st;
  if (!adapters || !q || !out) return LRA_ERR_NULL;
  if (adapters->n_adapters < 1) return LRA_ERR_SHAPE;
  if (seq_index < 0 || seq_index >= cache->n_seqs) return LRA_ERR_SHAPE;
  if (adapter_index < 0 || adapter_index >= adapters->n_adapters) return LRA_ERR_SHAPE;
  if (n_new < 1 || n_new > cache->max_seq_len) return LRA_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(out) |
       reinterpret_cast<uintptr_t>(adapters->b_k) | reinterpret_cast<uintptr_t>(adapters->b_v)) & 15)
    return LRA_ERR_SHAPE;
  if (!plan_sizes_fit(shape, cache, n_new, 1)) return LRA_ERR_UNSUPPORTED;
  const Tuning tune = resolve_tuning(tuning);
  Plan pl = make_plan(shape, cache, n_new, 1, true, tune);
  if (!pl.launchable) return LRA_ERR_UNSUPPORTED;
  // Rotary key side: the completed keys go to the workspace when the call has a key-side adapter and
  // the workspace has room for them; otherwise the kernel completes every key tile itself.
  bool keys_by_prepass = pl.kc_bytes > 0 && adapters->b_k != nullptr;
  if (pl.kc_bytes > 0 && (!keys_by_prepass || check_workspace(pl, workspace, workspace_bytes) != LRA_OK)) {
    keys_by_prepass = false;
    pl.bytes = pl.bytes_without_kc;
    pl.kc_bytes = 0;
  }
  st = check_workspace(pl, workspace, workspace_bytes);
  if (st != LRA_OK) return st;

  Params p{};
  fill_params(p, shape, cache, adapters, pl, workspace);
  p.q = q;
  p.out = out;
  p.n_queries = 1;
  p.max_queries_per_seq = 1;
  p.n_new = n_new;
  p.is_prefill = 1;
  p.seq_index = seq_index;
  p.adapter_index = adapter_index;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool bf16 = shape->dtype == LRA_BF16;
  if (pl.short_prefill) {
    if (launch_decode_mfma(p, pl.row_tiles, tune.variant != 2, tune.main_kernel_only, s) != hipSuccess) return LRA_ERR_HIP;
    if (tune.main_kernel_only) return LRA_OK;
    if (launch_merge(p, bf16, pl.rows, s) != hipSuccess) return LRA_ERR_HIP;
    return LRA_OK;
  }
  if (pl.mfma) {
    if (keys_by_prepass) {
      // K = K_base + RoPE(L B_K) of the call's adapter, once, then the kernel without a key-side
      // adapter on those keys (measurement of the main kernel alone: on the keys an earlier call left)
      void* kc = static_cast<unsigned char*>(workspace) + pl.off_kc;
      if (!tune.main_kernel_only && launch_complete_rope_keys(p, kc, s) != hipSuccess) return LRA_ERR_HIP;
      p.k_base = kc;
      p.b_k = nullptr;
      p.key_rope_theta = 0.f;
      p.keys_f16 = 1;
    }
    if (launch_prefill_mfma(p, s) != hipSuccess) return LRA_ERR_HIP;
    if (pl.n_splits > 1 && !tune.main_kernel_only && launch_merge(p, bf16, pl.rows, s) != hipSuccess)
      return LRA_ERR_HIP;
    return LRA_OK;
  }
  if (launch_generic_partials(p, bf16, pl.rows, s) != hipSuccess) return LRA_ERR_HIP;
  if (tune.main_kernel_only) return LRA_OK;
  if (launch_merge(p, bf16, pl.rows, s) != hipSuccess) return LRA_ERR_HIP;
  return LRA_OK;
}

// Argument checks shared by lra_cache_append and lra_append_workspace_bytes (x may be NULL for the latter).
static lra_status check_append(const lra_shape* shape, const lra_cache* cache, const lra_projection* proj,
                               int32_t seq_index, int32_t n_new) {
  lra_status st = check_common(shape, cache);
  if (st != LRA_OK) return st;
  if (!proj || !proj->w) return LRA_ERR_NULL;
  if (seq_index < 0 || seq_index >= cache->n_seqs) return LRA_ERR_SHAPE;
  if (n_new < 1 || n_new > cache->max_seq_len) return LRA_ERR_SHAPE;
  if (proj->d_model < 64 || !(proj->rope_theta >= 0.f) || std::isinf(proj->rope_theta)) return LRA_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(proj->w) & 15) return LRA_ERR_SHAPE;
  if (shape->dtype != LRA_BF16 || shape->rank % 8 != 0 || proj->d_model % 64 != 0) return LRA_ERR_UNSUPPORTED;
  // x and w are addressed with 32-bit byte offsets inside one buffer resource each
  const int64_t lim = (int64_t{1} << 32) - 4096;
  const int64_t n_feat = 2LL * shape->n_kv_heads * shape->head_dim + shape->rank;
  if (n_feat * proj->d_model * 2 > lim || static_cast<int64_t>(n_new) * proj->d_model * 2 > lim)
    return LRA_ERR_UNSUPPORTED;
  return LRA_OK;
}

size_t lra_append_workspace_bytes(const lra_shape* shape, const lra_cache* cache, const lra_projection* proj,
                                  int32_t n_new, const lra_tuning* tuning) {
  if (check_append(shape, cache, proj, 0, n_new) != LRA_OK) return static_cast<size_t>(-1);
  return plan_append_split(n_new, shape->n_kv_heads, shape->head_dim, shape->rank, proj->d_model, resolve_tuning(tuning)).bytes;
}

lra_status lra_cache_append(const lra_shape* shape, const lra_cache* cache, const lra_projection* proj,
                            const void* x, int32_t seq_index, int32_t n_new, void* workspace,
                            size_t workspace_bytes, const lra_tuning* tuning, void* stream) {
  lra_status st = check_append(shape, cache, proj, seq_index, n_new);
  if (st != LRA_OK) return st;
  if (!x) return LRA_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(x) & 15) return LRA_ERR_SHAPE;
  const Tuning tune = resolve_tuning(tuning);
  AppendParams p{};
  p.x = x;
  p.w = proj->w;
  p.k_base = const_cast<void*>(cache->k_base);
  p.v_base = const_cast<void*>(cache->v_base);
  p.l = const_cast<void*>(cache->l);
  p.block_table = cache->block_table;
  p.seq_lens = cache->seq_lens;
  p.kv_token_stride = cache->kv_token_stride;
  p.kv_head_stride = cache->kv_head_stride;
  p.kv_block_stride = cache->kv_block_stride;
  p.l_row_stride = cache->l_row_stride ? cache->l_row_stride : shape->rank;
  p.d_model = proj->d_model;
  p.n_kv_heads = shape->n_kv_heads;
  p.head_dim = shape->head_dim;
  p.rank = shape->rank;
  p.n_new = n_new;
  p.seq_index = seq_index;
  p.block_size = cache->block_size;
  p.max_blocks_per_seq = cache->max_blocks_per_seq;
  p.max_seq_len = cache->max_seq_len;
  p.rope_theta = proj->rope_theta;
  p.skinny_max = tune.append_skinny;
  p.stages = tune.append_stages;
  p.tile = tune.append_tile;
  // the split over d_model, where the sizes ask for it and the caller brought room for its parts
  const AppendSplit sp = plan_append_split(n_new, shape->n_kv_heads, shape->head_dim, shape->rank, proj->d_model, tune);
  const bool split = sp.k_splits > 1 && workspace != nullptr && !(reinterpret_cast<uintptr_t>(workspace) & 255) &&
                     workspace_bytes >= sp.bytes;
  p.k_splits = split ? sp.k_splits : 1;
  p.split_bt = sp.bt;
  p.split_ws = split ? static_cast<float*>(workspace) : nullptr;
  if (launch_append(p, static_cast<hipStream_t>(stream)) != hipSuccess) return LRA_ERR_HIP;
  return LRA_OK;
}

const char* lra_status_string(lra_status status) {
  switch (status) {
    case LRA_OK: return "ok";
    case LRA_ERR_NULL: return "a required pointer is NULL";
    case LRA_ERR_SHAPE: return "a size, stride or alignment is out of range or inconsistent";
    case LRA_ERR_DTYPE: return "unknown dtype";
    case LRA_ERR_UNSUPPORTED: return "valid arguments outside the supported set";
    case LRA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case LRA_ERR_HIP: return "a HIP launch failed";
  }
  return "unknown status";
}

#ifdef LRA_TIMING
// instrumented test build only
lra_status lra_debug_set_timing(void* buffer) {
  lra::g_timing = static_cast<unsigned long long*>(buffer);
  return LRA_OK;
}
#endif

}  // extern "C"
