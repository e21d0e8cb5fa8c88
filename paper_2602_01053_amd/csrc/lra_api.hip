// C ABI of the Flash-LoRA-Attention library: argument checks, launch planning,
// kernel selection.  Declarations and argument contracts are in lra_attn.h.
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <mutex>

#include "lra_attn.h"
#include "lra_common.h"

namespace lra {

#ifdef LRA_TIMING
static unsigned long long* g_timing = nullptr;  // instrumented test build only
#endif

std::atomic<int32_t> g_variant{0};
std::atomic<int32_t> g_split_keys{0};
std::atomic<int32_t> g_prefill_splits{0};  // 0 = automatic
std::atomic<int32_t> g_append_stages{0};   // LDS stages of the tiled append GEMM (0: chosen from the grid)
std::atomic<int32_t> g_append_tile{0};     // output tile of the append GEMM (0: chosen from the grid, 128, 256)
std::atomic<int32_t> g_append_skinny{64};  // new tokens up to which lra_cache_append streams the weights instead of tiling
std::atomic<int32_t> g_short_prefill{32};  // kShortPrefill: new tokens up to which prefill takes the split-KV path

std::atomic<int32_t> g_profile_mode{0};

constexpr int kCUs = 256;  // MI355X

struct Plan {
  bool mfma;
  bool short_prefill;  // prefill served by the split-KV decode kernels (few new tokens)
  int rows;        // query rows = (queries | new tokens) x Hq
  int split_keys;  // keys per split
  int n_splits;    // splits per sequence at max_seq_len
  int group_pad, row_tiles, row_groups;  // MFMA decode row packing
  size_t off_ml, off_o, off_lr, off_adapter, off_qt, qt_bytes, bytes;
};

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static lra_status check_common(const lra_shape* sh, const lra_cache* c) {
  if (!sh || !c) return LRA_ERR_NULL;
  if (sh->dtype != LRA_BF16 && sh->dtype != LRA_F32) return LRA_ERR_DTYPE;
  if (sh->n_q_heads < 1 || sh->n_kv_heads < 1 || sh->head_dim < 1 || sh->rank < 1) return LRA_ERR_SHAPE;
  if (sh->n_q_heads % sh->n_kv_heads) return LRA_ERR_SHAPE;
  if (!(sh->scale >= 0.f) || std::isinf(sh->scale)) return LRA_ERR_SHAPE;
  if (!(sh->key_rope_theta >= 0.f) || std::isinf(sh->key_rope_theta)) return LRA_ERR_SHAPE;
  if (sh->key_rope_theta > 0.f && (sh->head_dim & 1)) return LRA_ERR_SHAPE;
  if (sh->head_dim != 64 && sh->head_dim != 128) return LRA_ERR_UNSUPPORTED;
  if (sh->rank > 64) return LRA_ERR_UNSUPPORTED;
  if (sh->n_q_heads / sh->n_kv_heads > 16) return LRA_ERR_UNSUPPORTED;
  if (!c->k_base || !c->v_base || !c->l || !c->seq_lens) return LRA_ERR_NULL;
  if (c->n_seqs < 1 || c->max_seq_len < 1) return LRA_ERR_SHAPE;
  if (c->block_size != 0 && c->block_size != 16) return LRA_ERR_UNSUPPORTED;
  if (c->kv_token_stride < sh->head_dim || c->kv_head_stride < sh->head_dim) return LRA_ERR_SHAPE;
  if ((c->kv_token_stride | c->kv_head_stride) & 7) return LRA_ERR_SHAPE;
  if (c->block_size == 0) {
    if (c->n_seqs != 1) return LRA_ERR_SHAPE;
  } else {
    if (!c->block_table) return LRA_ERR_NULL;
    if (c->num_blocks < 1 || c->max_blocks_per_seq < 1) return LRA_ERR_SHAPE;
    if (c->kv_block_stride < 16 * sh->head_dim || (c->kv_block_stride & 7)) return LRA_ERR_SHAPE;
    if (static_cast<int64_t>(c->max_blocks_per_seq) * 16 < c->max_seq_len) return LRA_ERR_SHAPE;
  }
  const uintptr_t bits = reinterpret_cast<uintptr_t>(c->k_base) | reinterpret_cast<uintptr_t>(c->v_base) |
                         reinterpret_cast<uintptr_t>(c->l);
  if (bits & 15) return LRA_ERR_SHAPE;
  return LRA_OK;
}

static Plan make_plan(const lra_shape* sh, const lra_cache* c, int tokens, int max_queries_per_seq, bool prefill) {
  Plan pl{};
  const int G = sh->n_q_heads / sh->n_kv_heads;
  // The MFMA kernels move L in 16-byte pieces: ranks that are not a multiple of 8 take the
  // vector-ALU kernels.
  // The rotary key side: prefill runs on the tile-walking MFMA kernel, which completes a key
  // tile in LDS for its one adapter; decode on the rotary form of the split-KV kernel.
  const bool rope = sh->key_rope_theta > 0.f;
  pl.mfma = sh->dtype == LRA_BF16 && g_variant.load() != 1 && sh->rank % 8 == 0;
  if (prefill && pl.mfma) {
    // the tile-walking kernel addresses a contiguous kv head slice, and L as a whole, with
    // 32-bit byte offsets inside one buffer resource; larger caches take the other kernels
    const int64_t lim = (int64_t{1} << 32) - 4096;
    const int64_t l_rows = c->block_size == 0 ? c->max_seq_len : static_cast<int64_t>(c->num_blocks) * 16;
    if (l_rows * sh->rank * 2 > lim) pl.mfma = false;
    if (c->block_size == 0 && static_cast<int64_t>(c->max_seq_len) * c->kv_token_stride * 2 > lim) pl.mfma = false;
  }
  // A handful of new tokens after a long context gives the tile-walking prefill kernel one
  // workgroup per q head and nothing to split; the split-KV decode kernel, with the new
  // tokens in the place of the agents and a causal limit per row, spreads the context over
  // the chip instead.  (Measured crossover on MI355X: see kShortPrefill.)
  pl.short_prefill = prefill && pl.mfma && tokens <= g_short_prefill.load() &&
                     static_cast<int64_t>(tokens) * 4 <= c->max_seq_len;
  const bool rope_split = rope && pl.mfma && (!prefill || pl.short_prefill);  // rotary form of the split-KV kernel
  if (prefill && pl.mfma && !pl.short_prefill) {
    // Tile-walking kernel: one workgroup per (128-row q tile, q head).  When that is fewer than
    // two workgroups per CU, the key tiles of every q tile are divided among several workgroups
    // (at least eight 64-key tiles each) and the merge kernel finishes the job; otherwise it is
    // one kernel without a workspace.
    pl.rows = tokens * sh->n_q_heads;
    pl.group_pad = pl.row_tiles = pl.row_groups = 1;
    pl.split_keys = c->max_seq_len;
    const int64_t wgs = static_cast<int64_t>((tokens + 127) / 128) * sh->n_q_heads;
    int64_t ns = g_prefill_splits.load();
    if (ns <= 0) {  // automatic: two workgroups per CU, at least eight key tiles per share
      ns = (2 * kCUs + wgs - 1) / wgs;
      const int64_t max_ns = c->max_seq_len / (8 * 64);
      ns = ns > max_ns ? max_ns : ns;
    }
    ns = ns > 32 ? 32 : (ns < 1 ? 1 : ns);
    pl.n_splits = static_cast<int>(ns);
    pl.bytes = 0;
    if (pl.n_splits > 1) {
      const size_t slots = static_cast<size_t>(pl.rows) * pl.n_splits;
      pl.off_ml = 0;
      pl.off_o = align_up(slots * 2 * sizeof(float), 256);
      pl.off_lr = pl.off_o + align_up(slots * sh->head_dim * sizeof(float), 256);
      pl.off_adapter = pl.off_lr + align_up(slots * sh->rank * sizeof(float), 256);
      pl.bytes = pl.off_adapter + align_up(static_cast<size_t>(pl.rows) * sizeof(int32_t), 256);
    }
    return pl;
  }
  pl.rows = tokens * sh->n_q_heads;
  pl.group_pad = G <= 4 ? 4 : (G <= 8 ? 8 : 16);
  pl.row_tiles = 1;
  pl.row_groups = 1;
  int tile = 64;       // keys per wave-step of the vector-ALU kernel
  int64_t work;        // units that want a wave (vector-ALU) or a workgroup share (MFMA)
  int want;
  const int n_seqs_eff = prefill ? 1 : c->n_seqs;
  if (pl.short_prefill) max_queries_per_seq = tokens;
  if (pl.mfma) {
    int rows_needed = max_queries_per_seq * pl.group_pad;
    pl.row_tiles = decode_mfma_row_tiles(rows_needed);
    if (rope_split) {
      // one row tile per workgroup, and (decode) no more agent slots in it than the kernel keeps
      // B_K^T operands for
      const int min_pad = prefill ? 1 : 16 / decode_mfma_rope_slots(sh->rank);
      pl.group_pad = pl.group_pad > min_pad ? pl.group_pad : min_pad;
      pl.row_tiles = 1;
      rows_needed = max_queries_per_seq * pl.group_pad;
    }
    pl.row_groups = (rows_needed + 16 * pl.row_tiles - 1) / (16 * pl.row_tiles);
    tile = 128;        // 4 waves x 32 keys
    work = static_cast<int64_t>(n_seqs_eff) * sh->n_kv_heads * pl.row_groups;
    want = kCUs;
  } else {
    work = pl.rows;
    want = kCUs * 8;
  }
  int split_keys = g_split_keys.load();
  if (split_keys <= 0 && pl.mfma) {
    // Measured on MI355X: one sequence runs best with about one workgroup per CU (the
    // per-workgroup prologue is not amortised otherwise); a ragged batch wants about four
    // times as many, equal-sized pieces so the CUs stay balanced.  A batch is assumed to be
    // half as long on average as its longest sequence.
    const bool batch = n_seqs_eff > 1;
    const int64_t key_heads = work * c->max_seq_len / (batch ? 2 : 1);
    const int64_t wgs = batch ? kCUs * 4 : kCUs;
    split_keys = static_cast<int>((key_heads + wgs - 1) / wgs);
    if (split_keys > c->max_seq_len) split_keys = c->max_seq_len;
  } else if (split_keys <= 0) {
    int64_t ns = (want + work - 1) / work;
    const int64_t max_ns = (c->max_seq_len + tile - 1) / tile;
    ns = ns < 1 ? 1 : (ns > max_ns ? max_ns : ns);
    split_keys = static_cast<int>((c->max_seq_len + ns - 1) / ns);
  }
  split_keys = (split_keys + tile - 1) / tile * tile;
  if (pl.mfma && c->block_size == 0) {
    // the kernel addresses one split of a contiguous cache with 32-bit byte offsets
    const int64_t cap = ((int64_t{1} << 31) - 4096) / (c->kv_token_stride * 2) / tile * tile;
    if (cap < tile) pl.mfma = false;
    else if (split_keys > cap) split_keys = static_cast<int>(cap);
  }
  if (!pl.mfma) pl.short_prefill = false;
  pl.split_keys = split_keys;
  pl.n_splits = (c->max_seq_len + split_keys - 1) / split_keys;
  const size_t slots = static_cast<size_t>(pl.rows) * pl.n_splits;
  pl.off_ml = 0;
  pl.off_o = align_up(slots * 2 * sizeof(float), 256);
  pl.off_lr = pl.off_o + align_up(slots * sh->head_dim * sizeof(float), 256);
  pl.off_adapter = pl.off_lr + align_up(slots * sh->rank * sizeof(float), 256);
  pl.bytes = pl.off_adapter + align_up(static_cast<size_t>(pl.rows) * sizeof(int32_t), 256);
  // room for Qt of the whole call where the streaming form of the split-KV kernel would
  // otherwise reload many B_K rows per workgroup (reserved whether or not the call has a B_K)
  pl.off_qt = pl.bytes;
  pl.qt_bytes = 0;
  if (pl.mfma && c->block_size == 0 && !rope_split && g_variant.load() != 2)
    pl.qt_bytes = decode_stream_qt_bytes(pl.group_pad, sh->rank, pl.row_tiles, pl.row_groups, sh->n_kv_heads);
  pl.bytes += align_up(pl.qt_bytes, 256);
  return pl;
}

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
                           int32_t max_queries_per_seq, int32_t n_new) {
  if (check_common(shape, cache) != LRA_OK) return static_cast<size_t>(-1);
  if (n_new < 0 || n_new > cache->max_seq_len) return static_cast<size_t>(-1);
  if (n_new == 0 && (n_queries < 1 || max_queries_per_seq < 1 || max_queries_per_seq > n_queries))
    return static_cast<size_t>(-1);
  const bool prefill = n_new > 0;
  return make_plan(shape, cache, prefill ? n_new : n_queries, prefill ? 1 : max_queries_per_seq, prefill).bytes;
}

// Both decode entry points: checks, plan, then the workspace from the caller or, with
// `use_static`, the library's own per-device buffer.
static lra_status decode_call(const lra_shape* shape, const lra_cache* cache, const lra_adapters* adapters,
                              const void* q, const int32_t* query_adapter, const int32_t* seq_query_start,
                              int32_t n_queries, int32_t max_queries_per_seq, void* out, void* workspace,
                              size_t workspace_bytes, bool use_static, void* stream) {
  lra_status st = check_common(shape, cache);
  if (st != LRA_OK) return st;
  if (!adapters || !q || !query_adapter || !seq_query_start || !out) return LRA_ERR_NULL;
  if (adapters->n_adapters < 1 || n_queries < 1) return LRA_ERR_SHAPE;
  if (max_queries_per_seq < 1 || max_queries_per_seq > n_queries) return LRA_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(out) |
       reinterpret_cast<uintptr_t>(adapters->b_k) | reinterpret_cast<uintptr_t>(adapters->b_v)) & 15)
    return LRA_ERR_SHAPE;
  const Plan pl = make_plan(shape, cache, n_queries, max_queries_per_seq, false);
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
    if (launch_decode_mfma(p, pl.row_tiles, g_variant.load() != 2, g_profile_mode.load() == 1, s) != hipSuccess) return LRA_ERR_HIP;
  } else {
    if (launch_generic_partials(p, bf16, pl.rows, s) != hipSuccess) return LRA_ERR_HIP;
  }
  if (g_profile_mode.load() == 1) return LRA_OK;  // measurement: key-streaming kernel alone
  if (launch_merge(p, bf16, pl.rows, s) != hipSuccess) return LRA_ERR_HIP;
  return LRA_OK;
}

lra_status lra_attn_decode(const lra_shape* shape, const lra_cache* cache, const lra_adapters* adapters,
                           const void* q, const int32_t* query_adapter, const int32_t* seq_query_start,
                           int32_t n_queries, int32_t max_queries_per_seq, void* out, void* workspace,
                           size_t workspace_bytes, void* stream) {
  return decode_call(shape, cache, adapters, q, query_adapter, seq_query_start, n_queries, max_queries_per_seq, out,
                     workspace, workspace_bytes, false, stream);
}

lra_status lra_attn_decode_static(const lra_shape* shape, const lra_cache* cache, const lra_adapters* adapters,
                                  const void* q, const int32_t* query_adapter, const int32_t* seq_query_start,
                                  int32_t n_queries, int32_t max_queries_per_seq, void* out, void* stream) {
  return decode_call(shape, cache, adapters, q, query_adapter, seq_query_start, n_queries, max_queries_per_seq, out,
                     nullptr, 0, true, stream);
}

lra_status lra_attn_prefill(const lra_shape* shape, const lra_cache* cache, const lra_adapters* adapters,
                            const void* q, int32_t seq_index, int32_t adapter_index, int32_t n_new,
                            void* out, void* workspace, size_t workspace_bytes, void* stream) {
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
  const Plan pl = make_plan(shape, cache, n_new, 1, true);
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
    if (launch_decode_mfma(p, pl.row_tiles, g_variant.load() != 2, g_profile_mode.load() == 1, s) != hipSuccess) return LRA_ERR_HIP;
    if (g_profile_mode.load() == 1) return LRA_OK;
    if (launch_merge(p, bf16, pl.rows, s) != hipSuccess) return LRA_ERR_HIP;
    return LRA_OK;
  }
  if (pl.mfma) {
    if (launch_prefill_mfma(p, s) != hipSuccess) return LRA_ERR_HIP;
    if (pl.n_splits > 1 && g_profile_mode.load() != 1 && launch_merge(p, bf16, pl.rows, s) != hipSuccess)
      return LRA_ERR_HIP;
    return LRA_OK;
  }
  if (launch_generic_partials(p, bf16, pl.rows, s) != hipSuccess) return LRA_ERR_HIP;
  if (g_profile_mode.load() == 1) return LRA_OK;
  if (launch_merge(p, bf16, pl.rows, s) != hipSuccess) return LRA_ERR_HIP;
  return LRA_OK;
}

lra_status lra_cache_append(const lra_shape* shape, const lra_cache* cache, const lra_projection* proj,
                            const void* x, int32_t seq_index, int32_t n_new, void* stream) {
  lra_status st = check_common(shape, cache);
  if (st != LRA_OK) return st;
  if (!proj || !proj->w || !x) return LRA_ERR_NULL;
  if (seq_index < 0 || seq_index >= cache->n_seqs) return LRA_ERR_SHAPE;
  if (n_new < 1 || n_new > cache->max_seq_len) return LRA_ERR_SHAPE;
  if (proj->d_model < 64 || !(proj->rope_theta >= 0.f)) return LRA_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(proj->w)) & 15) return LRA_ERR_SHAPE;
  if (shape->dtype != LRA_BF16 || shape->rank % 8 != 0 || proj->d_model % 64 != 0) return LRA_ERR_UNSUPPORTED;
  // x and w are addressed with 32-bit byte offsets inside one buffer resource each
  const int64_t lim = (int64_t{1} << 32) - 4096;
  const int64_t n_feat = 2LL * shape->n_kv_heads * shape->head_dim + shape->rank;
  if (n_feat * proj->d_model * 2 > lim || static_cast<int64_t>(n_new) * proj->d_model * 2 > lim)
    return LRA_ERR_UNSUPPORTED;
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
  p.skinny_max = g_append_skinny.load();
  p.stages = g_append_stages.load();
  p.tile = g_append_tile.load();
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

int32_t lra_set_kernel_variant(int32_t variant) { return g_variant.exchange(variant == 1 || variant == 2 ? variant : 0); }

int32_t lra_set_prefill_splits(int32_t splits) { return g_prefill_splits.exchange(splits < 0 ? 0 : splits); }

int32_t lra_set_append_stages(int32_t stages) {
  return g_append_stages.exchange(stages < 2 || stages > 4 ? 0 : stages);
}

int32_t lra_set_append_tile(int32_t tile) {
  return g_append_tile.exchange(tile == 64 || tile == 128 || tile == 256 ? tile : 0);
}

int32_t lra_set_append_skinny(int32_t tokens) { return g_append_skinny.exchange(tokens < 0 ? 0 : tokens); }

int32_t lra_set_short_prefill(int32_t tokens) { return g_short_prefill.exchange(tokens < 0 ? 0 : tokens); }

int32_t lra_set_decode_split_keys(int32_t keys) { return g_split_keys.exchange(keys < 0 ? 0 : keys); }


int32_t lra_set_profile_mode(int32_t mode) { return g_profile_mode.exchange(mode == 1 ? 1 : 0); }

#ifdef LRA_TIMING
// instrumented test build only
lra_status lra_debug_set_timing(void* buffer) {
  lra::g_timing = static_cast<unsigned long long*>(buffer);
  return LRA_OK;
}
#endif

}  // extern "C"
