// Launch planning (host only; see lra_plan.h).
#include "lra_plan.h"

#include <cmath>

namespace lra {

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

Tuning resolve_tuning(const lra_tuning* t) {
  Tuning r;
  if (!t) return r;
  r.variant = (t->kernel_variant == 1 || t->kernel_variant == 2) ? t->kernel_variant : 0;
  r.split_keys = t->decode_split_keys > 0 ? t->decode_split_keys : 0;
  if (t->short_prefill != 0) r.short_prefill = t->short_prefill < 0 ? 0 : t->short_prefill;
  r.prefill_splits = t->prefill_splits > 0 ? t->prefill_splits : 0;
  r.rope_key_prepass = t->rope_key_prepass >= 0;
  if (t->append_skinny != 0) r.append_skinny = t->append_skinny < 0 ? 0 : t->append_skinny;
  r.append_stages = (t->append_stages >= 2 && t->append_stages <= 4) ? t->append_stages : 0;
  r.append_tile = (t->append_tile == 64 || t->append_tile == 128 || t->append_tile == 256) ? t->append_tile : 0;
  r.append_k_splits = (t->append_k_splits >= 1 && t->append_k_splits <= 16) ? t->append_k_splits : 0;
  r.main_kernel_only = t->measure_main_kernel_only == 1;
  return r;
}

// Caps that keep the planner's and the kernels' 32-bit arithmetic in range: query rows
// (tokens x Hq) and the padded rows of one sequence (queries x 16) below 2^30.
bool plan_sizes_fit(const lra_shape* sh, const lra_cache* c, int32_t tokens, int32_t max_queries_per_seq) {
  (void)c;
  if (tokens < 1 || max_queries_per_seq < 1) return false;
  if (static_cast<int64_t>(tokens) * sh->n_q_heads > (int64_t{1} << 30)) return false;
  if (static_cast<int64_t>(max_queries_per_seq) * 16 > (int64_t{1} << 30)) return false;
  return true;
}

// A chunk whose 128-feature output tiles occupy about half of the chip or less walks all of d_model in
// each of them, one 64-wide step after the other, at what one compute unit can pull from L2.  Such
// chunks divide d_model among several workgroups per tile (a power of two of parts, at least four
// steps each, about one workgroup per compute unit in all) and add the parts in a second kernel.
// Measured on the Llama-3-8B projection: 64 tokens 14 against 21 us, 128 tokens 13 against 23 us; up to
// 32 tokens the weight-streaming kernel is as fast and stays.  Forced tile or stage choices keep the
// unsplit kernels.
AppendSplit plan_append_split(int n_new, int n_kv_heads, int head_dim, int rank, int d_model, const Tuning& tune) {
  AppendSplit none{1, 128, 0};
  if (tune.append_k_splits == 1 || tune.append_tile != 0 || tune.append_stages != 0) return none;
  if (n_new < 1 || n_new > (1 << 20) || d_model < 64) return none;  // (keeps the byte count below 2^48)
  const int n_steps = d_model / 64;
  const int64_t hd = static_cast<int64_t>(n_kv_heads) * head_dim;
  const int64_t tile_rows = 2 * ((hd + 127) / 128) + 1;
  const int64_t tiles128 = (static_cast<int64_t>(n_new) + 127) / 128 * tile_rows;
  if (tune.append_k_splits == 0 && (n_new <= 32 || tiles128 * 2 > kCUs))
    return none;
  AppendSplit sp{1, tiles128 <= 100 ? 64 : 128, 0};
  const int64_t tiles = (static_cast<int64_t>(n_new) + sp.bt - 1) / sp.bt * tile_rows;
  if (tune.append_k_splits > 1) {
    if (n_steps % tune.append_k_splits != 0 || tiles * tune.append_k_splits > 65535 * 16) return none;
    sp.k_splits = tune.append_k_splits;
  } else {
    for (int ks = 16; ks >= 2; ks /= 2)
      if (n_steps % ks == 0 && n_steps / ks >= 4 && tiles * ks <= kCUs) {  // one workgroup per compute unit at most
        sp.k_splits = ks;
        break;
      }
  }
  if (sp.k_splits < 2) return none;
  const int64_t n_feat = 2 * hd + rank;
  sp.bytes = align_up(static_cast<size_t>(sp.k_splits) * static_cast<size_t>(n_new) * static_cast<size_t>(n_feat) * sizeof(float), 256);
  return sp;
}

int decode_mfma_row_tiles(int rows_needed) { return rows_needed <= 16 ? 1 : 2; }

// (the B_K^T operands of a tile's slots stay in registers: 4 slots at ranks up to 16, 2 up to 32, 4
// again above, where the kernel has a compute unit to itself)
int decode_mfma_rope_slots(int rank) { return rank <= 16 ? 4 : (rank <= 32 ? 2 : 4); }

// The pre-pass pays (one more launch) once a workgroup of the streaming kernel would have to load
// more than eight 16-row blocks of B_K.
size_t decode_stream_qt_bytes(int group_pad, int rank, int row_tiles, int row_groups, int n_kv_heads) {
  const int slots = 16 / group_pad, ncb = (rank + 15) / 16;
  if (slots * ncb * row_tiles <= 8) return 0;
  const int rks = rank > 32 ? 2 : 1;
  return static_cast<size_t>(row_groups) * n_kv_heads * row_tiles * rks * 1024;
}

lra_status check_common(const lra_shape* sh, const lra_cache* c) {
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
  if (sh->n_q_heads > 4096) return LRA_ERR_UNSUPPORTED;
  if (!c->k_base || !c->v_base || !c->l || !c->seq_lens) return LRA_ERR_NULL;
  if (c->n_seqs < 1 || c->max_seq_len < 1) return LRA_ERR_SHAPE;
  if (c->n_seqs > (1 << 20) || c->max_seq_len > (1 << 30)) return LRA_ERR_UNSUPPORTED;
  if (c->block_size != 0 && c->block_size != 16) return LRA_ERR_UNSUPPORTED;
  if (c->kv_token_stride < sh->head_dim || c->kv_head_stride < sh->head_dim) return LRA_ERR_SHAPE;
  if ((c->kv_token_stride | c->kv_head_stride) & 7) return LRA_ERR_SHAPE;
  // extents stay far inside 64-bit element offsets (and the planner's products inside int64)
  if (c->kv_token_stride > (int64_t{1} << 31) || c->kv_head_stride > (int64_t{1} << 40)) return LRA_ERR_UNSUPPORTED;
  if (c->block_size == 0) {
    if (c->n_seqs != 1) return LRA_ERR_SHAPE;
  } else {
    if (!c->block_table) return LRA_ERR_NULL;
    if (c->num_blocks < 1 || c->max_blocks_per_seq < 1) return LRA_ERR_SHAPE;
    if (c->kv_block_stride < 16 * sh->head_dim || (c->kv_block_stride & 7)) return LRA_ERR_SHAPE;
    if (c->kv_block_stride > (int64_t{1} << 40) || c->num_blocks > (int64_t{1} << 60) / c->kv_block_stride)
      return LRA_ERR_UNSUPPORTED;
    if (static_cast<int64_t>(c->max_blocks_per_seq) * 16 < c->max_seq_len) return LRA_ERR_SHAPE;
  }
  if (c->l_row_stride < 0 || c->l_adapter_stride < 0 || (c->l_adapter_stride & 7)) return LRA_ERR_SHAPE;
  if (c->l_row_stride != sh->rank && (c->l_row_stride & 7)) return LRA_ERR_SHAPE;  // (dense rows of any rank are fine)
  if (c->l_row_stride != 0 && c->l_row_stride < sh->rank) return LRA_ERR_SHAPE;
  if (c->l_row_stride > (int64_t{1} << 31) || c->l_adapter_stride > (int64_t{1} << 40)) return LRA_ERR_UNSUPPORTED;
  if (c->block_size != 0 && c->num_blocks > 0 &&
      (c->l_row_stride ? c->l_row_stride : sh->rank) > (int64_t{1} << 56) / c->num_blocks)
    return LRA_ERR_UNSUPPORTED;
  const uintptr_t bits = reinterpret_cast<uintptr_t>(c->k_base) | reinterpret_cast<uintptr_t>(c->v_base) |
                         reinterpret_cast<uintptr_t>(c->l);
  if (bits & 15) return LRA_ERR_SHAPE;
  return LRA_OK;
}

Plan make_plan(const lra_shape* sh, const lra_cache* c, int tokens, int max_queries_per_seq, bool prefill,
               const Tuning& tune) {
  Plan pl{};
  const int G = sh->n_q_heads / sh->n_kv_heads;
  // The MFMA kernels move L in 16-byte pieces: ranks that are not a multiple of 8 take the
  // vector-ALU kernels.
  // The rotary key side: prefill runs on the tile-walking MFMA kernel, which completes a key
  // tile in LDS for its one adapter; decode on the rotary form of the split-KV kernel.
  const bool rope = sh->key_rope_theta > 0.f;
  pl.mfma = sh->dtype == LRA_BF16 && tune.variant != 1 && sh->rank % 8 == 0;
  // Low-rank rows with a stride of their own, or one low-rank cache per adapter (BaseShared): the
  // tile-walking prefill kernel and the streaming form of the split-KV kernel read them; that form
  // needs a contiguous cache and no rotary key side, everything else takes the vector-ALU kernels.
  const int64_t l_pitch = c->l_row_stride ? c->l_row_stride : sh->rank;
  const bool custom_l = c->l_adapter_stride > 0 || l_pitch != sh->rank;
  const bool stream_ok = c->block_size == 0 && !(sh->key_rope_theta > 0.f) && tune.variant != 2;
  // ... except that the older split-KV kernel reads such rows too when every row tile of a workgroup belongs to
  // ONE low-rank cache: paged caches and batches then give each agent a row tile (and a workgroup) of its own,
  // which streams K_base / V_base once per agent of a sequence instead of once per sequence (the other agents'
  // workgroups find the tiles in L2), still on the matrix cores.  The rotary form of that kernel likewise (its
  // tiles then hold one agent slot each).
  const bool tile_per_agent = custom_l && !stream_ok;
  // Plain decode with one low-rank cache per adapter does better: the split-KV kernel has the same column-block L
  // tile as the streaming form (one block per agent slot of a row tile), so K_base / V_base are requested once for
  // the agents of a tile.  It addresses a paged pool of low-rank rows with 32-bit byte offsets inside one resource.
  const bool block_per_slot =
      tile_per_agent && !prefill && !rope && c->l_adapter_stride > 0 &&
      (c->block_size == 0 || static_cast<int64_t>(c->num_blocks) * 16 * l_pitch * 2 <= (int64_t{1} << 31) - 4096);
  const bool stream_only = custom_l && !tile_per_agent;
  if (prefill && pl.mfma) {
    // the tile-walking kernel addresses a contiguous kv head slice, and L as a whole, with
    // 32-bit byte offsets inside one buffer resource; larger caches take the other kernels
    const int64_t lim = (int64_t{1} << 32) - 4096;
    const int64_t l_rows = c->block_size == 0 ? c->max_seq_len : static_cast<int64_t>(c->num_blocks) * 16;
    if (l_rows * l_pitch * 2 > lim) pl.mfma = false;
    if (c->block_size == 0 && static_cast<int64_t>(c->max_seq_len) * c->kv_token_stride * 2 > lim) pl.mfma = false;
  }
  // A handful of new tokens after a long context gives the tile-walking prefill kernel one
  // workgroup per q head and nothing to split; the split-KV decode kernel, with the new
  // tokens in the place of the agents and a causal limit per row, spreads the context over
  // the chip instead.  (Measured crossover on MI355X: see kShortPrefill.)
  pl.short_prefill = prefill && pl.mfma && tokens <= tune.short_prefill &&
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
    int64_t ns = tune.prefill_splits;
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
    pl.off_qt = pl.bytes;
    pl.bytes_without_kc = pl.bytes;
    if (rope && tune.rope_key_prepass) {
      // room for the completed keys of the call's adapter, in the layout of K_base (whether or
      // not the call has a B_K); caches beyond 4 GB keep completing tiles inside the kernel.
      // Paged caches: the blocks of the call's sequence in logical order, with the strides of the pool.
      int64_t span = -1;  // elements; -1: no pre-pass
      if (c->block_size == 0)
        span = (static_cast<int64_t>(c->max_seq_len) - 1) * c->kv_token_stride +
               (static_cast<int64_t>(sh->n_kv_heads) - 1) * c->kv_head_stride + sh->head_dim;
      else if (c->kv_block_stride <= (int64_t{1} << 31))  // (keeps the product below inside int64)
        span = (static_cast<int64_t>(c->max_seq_len) - 1) / 16 * c->kv_block_stride +
               (static_cast<int64_t>(sh->n_kv_heads) - 1) * c->kv_head_stride + 15 * c->kv_token_stride + sh->head_dim;
      if (span >= 0 && span <= (int64_t{1} << 31)) {
        pl.off_kc = pl.bytes;
        pl.kc_bytes = align_up(static_cast<size_t>(span) * 2, 256);
        pl.bytes += pl.kc_bytes;
      }
    }
    pl.launchable = true;  // at most 32 shares in y
    return pl;
  }
  pl.rows = tokens * sh->n_q_heads;
  pl.group_pad = G <= 4 ? 4 : (G <= 8 ? 8 : 16);
  pl.l_block = 0;
  if (tile_per_agent && !block_per_slot && !prefill && c->l_adapter_stride > 0) pl.group_pad = 16;  // one agent per 16-row tile
  if (pl.mfma && !prefill && c->l_adapter_stride > 0 && (!tile_per_agent || block_per_slot)) {
    // every agent slot of a row tile brings its own column block of the L tile: 64 columns per tile
    pl.l_block = sh->rank <= 16 ? 16 : (sh->rank <= 32 ? 32 : 64);
    const int min_pad = 16 / (64 / pl.l_block);
    pl.group_pad = pl.group_pad > min_pad ? pl.group_pad : min_pad;
  }
  pl.row_tiles = 1;
  pl.row_groups = 1;
  int tile = 64;       // keys per wave-step of the vector-ALU kernel
  int64_t work;        // units that want a wave (vector-ALU) or a workgroup share (MFMA)
  int want;
  const int n_seqs_eff = prefill ? 1 : c->n_seqs;
  if (pl.short_prefill) max_queries_per_seq = tokens;
  if (pl.mfma) {
    int rows_needed = max_queries_per_seq * pl.group_pad;
    pl.row_tiles = (pl.l_block || (tile_per_agent && !prefill && c->l_adapter_stride > 0)) ? 1 : decode_mfma_row_tiles(rows_needed);  // (an L tile holds the column blocks, or the one cache, of one row tile's agents)
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
  int split_keys = tune.split_keys;
  if (split_keys <= 0 && pl.mfma) {
    // Measured on MI355X: one sequence runs best with about one workgroup per CU (the
    // per-workgroup prologue is not amortised otherwise); a ragged batch wants about four
    // times as many, equal-sized pieces so the CUs stay balanced.  A batch is assumed to be
    // half as long on average as its longest sequence.
    const bool batch = n_seqs_eff > 1;
    int64_t wgs = batch ? kCUs * 4 : kCUs;
    // ... and one long sequence in a paged cache (the split-KV kernel, two workgroups per compute unit) with two,
    // as long as a share then still has 512 keys (32768 tokens x 8 kv heads: 35.7 against 38.6 us, 65536: 49.2
    // against 53.7; at 256 keys per share the doubling loses)
    if (!batch && !prefill && c->block_size != 0 && !rope && work * c->max_seq_len >= int64_t{2} * kCUs * 512) wgs = 2 * kCUs;
    if (work >= 2 * wgs) {
      split_keys = c->max_seq_len;  // more units than workgroups wanted: one share per sequence
    } else {
      const int64_t key_heads = work * c->max_seq_len / (batch ? 2 : 1);
      const int64_t sk = (key_heads + wgs - 1) / wgs;
      split_keys = sk > c->max_seq_len ? c->max_seq_len : static_cast<int>(sk);
    }
  } else if (split_keys <= 0) {
    int64_t ns = (want + work - 1) / work;
    const int64_t max_ns = (c->max_seq_len + tile - 1) / tile;
    ns = ns < 1 ? 1 : (ns > max_ns ? max_ns : ns);
    split_keys = static_cast<int>((c->max_seq_len + ns - 1) / ns);
  }
  if (split_keys > (1 << 30)) split_keys = 1 << 30;  // (a tuning value; max_seq_len itself is capped there)
  split_keys = (split_keys + tile - 1) / tile * tile;
  if (tune.split_keys <= 0 && pl.mfma && !prefill && c->n_seqs > 1 && c->seq_lens_host != nullptr && c->n_seqs <= 16384) {
    // The lengths are known.  A batch of sequences of about the same length runs best when the workgroups that find
    // keys are all resident at once, two per compute unit, and equal in size (measured on MI355X, 16 sequences of
    // 32768 tokens: 5.7 TB/s at 512 workgroups, 5.0 at 2048, 4.9 at 704): the smallest share size that keeps them
    // within that; never smaller than the choice above, so the workspace of a call without the lengths is large
    // enough for any call with them.  A ragged batch (shortest sequence below three quarters of the longest) does
    // best in two rounds - its shares are unequal, and twice as many workgroups as there are places level that out
    // (16 sequences of 6.5 k to 65 k tokens: 173-175 us at 840 to 960 workgroups, 199 us at 512) - but not in two
    // rounds and a bit: the time jumps by a tenth between 960 and 1020 workgroups (a second batch, 24 sequences of
    // 2 k to 40 k tokens: 190 us at 916, 206 us at 1036).  There the bound is 940.
    const int64_t units = static_cast<int64_t>(sh->n_kv_heads) * pl.row_groups;
    int64_t shortest = c->max_seq_len, longest = 0;
    for (int t = 0; t < c->n_seqs; ++t) {
      int64_t len = c->seq_lens_host[t];
      len = len < 0 ? 0 : (len > c->max_seq_len ? c->max_seq_len : len);
      shortest = len < shortest ? len : shortest;
      longest = len > longest ? len : longest;
    }
    const bool even_lengths = shortest * 4 >= longest * 3 && longest > 0;
    auto workgroups = [&](int64_t share) {
      int64_t n = 0;
      for (int t = 0; t < c->n_seqs; ++t) {
        int64_t len = c->seq_lens_host[t];
        len = len < 0 ? 0 : (len > c->max_seq_len ? c->max_seq_len : len);
        n += (len + share - 1) / share;
      }
      return n * units;
    };
    int64_t lo = split_keys / tile, hi = (static_cast<int64_t>(c->max_seq_len) + tile - 1) / tile;  // in tiles
    if (hi < lo) hi = lo;
    const int64_t bound = even_lengths ? 2 * kCUs : 940;
    if (longest > 0 && workgroups(lo * tile) > bound) {
      while (lo < hi) {  // smallest share in (lo, hi] within the bound, else hi
        const int64_t mid = lo + (hi - lo) / 2;
        if (workgroups(mid * tile) <= bound) hi = mid;
        else lo = mid + 1;
      }
      split_keys = static_cast<int>(hi * tile);
    }
  }
  if (pl.mfma && c->block_size == 0) {
    // the kernel addresses one split of a contiguous cache with 32-bit byte offsets
    const int64_t cap = ((int64_t{1} << 31) - 4096) / (c->kv_token_stride * 2) / tile * tile;
    if (cap < tile) pl.mfma = false;
    else if (split_keys > cap) split_keys = static_cast<int>(cap);
  }
  if (pl.mfma && tile_per_agent && c->block_size == 0) {
    // a wave addresses the L rows of its keys with 32-bit byte offsets
    const int64_t cap_l = ((int64_t{1} << 31) - 4096) / (l_pitch * 2) * 4 / tile * tile;
    if (cap_l < tile) pl.mfma = false;
    else if (split_keys > cap_l) split_keys = static_cast<int>(cap_l);
  }
  if (!pl.mfma) pl.short_prefill = false;
  if (pl.mfma && stream_only) {
    // These calls want the streaming form: at most one workgroup per compute unit, and a wave's L rows inside 32-bit
    // byte offsets.  Where that does not fit (more (kv head, row group) units than compute units, a very wide row
    // pitch) the split-KV kernel reads the same layouts, a wave addressing a quarter of a key share.
    const int64_t max_shares = kCUs / work;
    const int64_t cap_l = ((int64_t{1} << 31) - 4096) / (l_pitch * 2) / tile * tile;
    int64_t sk = split_keys;
    bool fits = max_shares >= 1 && cap_l >= tile;
    if (fits) {
      const int64_t need = ((c->max_seq_len + max_shares - 1) / max_shares + tile - 1) / tile * tile;
      if (sk < need) sk = need;
      fits = sk <= cap_l && sk <= ((int64_t{1} << 31) - 4096) / (c->kv_token_stride * 2) / tile * tile;
    }
    if (fits) {
      split_keys = static_cast<int>(sk);
    } else {
      const int64_t cap4 = ((int64_t{1} << 31) - 4096) / (l_pitch * 2) * 4 / tile * tile;
      if (cap4 < tile) pl.mfma = false;
      else if (split_keys > cap4) split_keys = static_cast<int>(cap4);
    }
  }
  if (!pl.mfma) pl.l_block = 0;
  pl.split_keys = split_keys;
  pl.n_splits = static_cast<int>((static_cast<int64_t>(c->max_seq_len) + split_keys - 1) / split_keys);
  // grids: (kv head, share, sequence x row group) for the MFMA kernels, (row, share) otherwise
  pl.launchable = pl.n_splits <= 65535 &&
                  (!pl.mfma || static_cast<int64_t>(n_seqs_eff) * pl.row_groups <= 65535);
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
  if (pl.mfma && c->block_size == 0 && !rope_split && tune.variant != 2 && pl.l_block == 0)
    pl.qt_bytes = decode_stream_qt_bytes(pl.group_pad, sh->rank, pl.row_tiles, pl.row_groups, sh->n_kv_heads);
  pl.bytes += align_up(pl.qt_bytes, 256);
  pl.bytes_without_kc = pl.bytes;
  return pl;
}

}  // namespace lra
