// Fuzz driver for the host-side launch planning (csrc/lra_plan.cpp), built for the CPU alone with
// -fsanitize=address,undefined by tests/test_plan_sanitized.py: random and extreme shapes, strides
// and sizes go through the argument checks and, where those accept them, through the planner; every
// plan must keep its invariants, and the sanitizers must stay silent (signed overflow in the 32-bit
// offset caps and workspace sizes is what this is after).
#include <vector>
#include <cinttypes>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <initializer_list>

#include "lra_plan.h"

using namespace lra;

static uint64_t state = 0x9e3779b97f4a7c15ull;
static uint64_t rnd() {
  state ^= state << 13;
  state ^= state >> 7;
  state ^= state << 17;
  return state;
}
static int64_t pick(std::initializer_list<int64_t> v) { return *(v.begin() + rnd() % v.size()); }

#define CHECK(cond)                                                                     \
  do {                                                                                  \
    if (!(cond)) {                                                                      \
      std::fprintf(stderr, "plan_fuzz: %s failed at case %d (line %d)\n", #cond, it, __LINE__); \
      return 1;                                                                         \
    }                                                                                   \
  } while (0)

int main(int argc, char** argv) {
  const int cases = argc > 1 ? std::atoi(argv[1]) : 200000;
  static char dummy[64];
  int accepted = 0;
  for (int it = 0; it < cases; ++it) {
    // every field: usually from the values the library supports, now and then a bad one
    auto pv = [&](std::initializer_list<int64_t> good, std::initializer_list<int64_t> bad) { return rnd() % 12 ? pick(good) : pick(bad); };
    lra_shape sh{};
    sh.n_kv_heads = static_cast<int32_t>(pv({1, 2, 4, 8, 3}, {0, -1, 1 << 20}));
    sh.n_q_heads = sh.n_kv_heads > 0 && rnd() % 12 ? sh.n_kv_heads * static_cast<int32_t>(pv({1, 2, 4, 7, 8, 16}, {17}))
                                                   : static_cast<int32_t>(pick({0, 5, 32, INT32_MAX}));
    sh.head_dim = static_cast<int32_t>(pv({64, 128}, {96, 0, 256}));
    sh.rank = static_cast<int32_t>(pv({1, 4, 8, 12, 16, 24, 32, 40, 64}, {65, 0, -3}));
    sh.dtype = static_cast<int32_t>(pv({0, 0, 0, 1}, {2, -1}));
    sh.scale = rnd() % 6 ? 0.f : static_cast<float>(pick({1, -1})) * 0.125f;
    sh.key_rope_theta = rnd() % 4 ? 0.f : 500000.f;
    lra_cache c{};
    c.k_base = c.v_base = c.l = dummy;
    c.seq_lens = reinterpret_cast<const int32_t*>(dummy);
    const bool paged = rnd() % 2;
    c.block_size = paged ? 16 : static_cast<int32_t>(pv({0}, {8}));
    c.n_seqs = paged ? static_cast<int32_t>(pv({1, 2, 16, 1000, 1 << 20}, {0, (1 << 20) + 1})) : static_cast<int32_t>(pv({1}, {2}));
    c.max_seq_len = static_cast<int32_t>(pv({1, 2, 31, 32, 33, 127, 128, 129, 1000, 8192, 65536, 1 << 20, 1 << 27, 1 << 30},
                                            {INT32_MAX, 0, -1}));
    const int64_t d = sh.head_dim > 0 ? sh.head_dim : 8;
    c.kv_token_stride = pv({d, d * 8, d * 8 + 8, d * 1024, int64_t{1} << 33}, {d - 8, 0, d + 4});
    c.kv_head_stride = pv({d, d * 16, static_cast<int64_t>(c.max_seq_len > 0 ? c.max_seq_len : 1) * d, int64_t{1} << 40}, {0});
    c.kv_block_stride = paged ? pv({16 * d, 16 * d * 8, int64_t{1} << 36}, {8, 0}) : 0;
    c.max_blocks_per_seq = paged ? static_cast<int32_t>(pv({(static_cast<int64_t>(c.max_seq_len > 0 ? c.max_seq_len : 1) + 15) / 16, INT32_MAX}, {1, 4})) : 0;
    c.num_blocks = paged ? static_cast<int32_t>(pv({1, 100, 1 << 20, INT32_MAX}, {0})) : 0;
    c.block_table = paged && rnd() % 16 ? reinterpret_cast<const int32_t*>(dummy) : nullptr;
    const int64_t rk = sh.rank > 0 ? sh.rank : 8;
    c.l_row_stride = pv({0, 0, (rk + 7) / 8 * 8, rk * 4 / 8 * 8 + 8, 4096, int64_t{1} << 31}, {rk - 1 > 0 ? (rk - 1) / 8 * 8 : 8, 12, -8, (int64_t{1} << 31) + 8});
    c.l_adapter_stride = pv({0, 0, 0, 16, 64, int64_t{1} << 30, int64_t{1} << 40}, {-8, 4, (int64_t{1} << 40) + 8});
    lra_tuning t{};
    t.kernel_variant = static_cast<int32_t>(pick({0, 0, 1, 2, 7}));
    t.decode_split_keys = static_cast<int32_t>(pick({0, 0, 1, 64, 100, 1 << 20, INT32_MAX, -5}));
    t.short_prefill = static_cast<int32_t>(pick({0, -1, 1, 64, INT32_MAX}));
    t.prefill_splits = static_cast<int32_t>(pick({0, 1, 5, 32, 1000, -1}));
    t.rope_key_prepass = static_cast<int32_t>(pick({0, 0, -1, 1}));
    const Tuning tune = resolve_tuning(rnd() % 4 ? &t : nullptr);
    if (check_common(&sh, &c) != LRA_OK) continue;
    ++accepted;
    const int G = sh.n_q_heads / sh.n_kv_heads;
    for (int prefill = 0; prefill < 2; ++prefill) {
      int64_t tokens = pick({1, 2, 3, 4, 8, 16, 17, 33, 64, 1000, 4096, 1 << 20, 1 << 26, INT32_MAX});
      if (prefill && tokens > c.max_seq_len) tokens = c.max_seq_len;
      int64_t mq = prefill ? 1 : pick({1, 1, 2, 4, 5, 9, 64, tokens});
      if (mq > tokens) mq = tokens;
      if (!plan_sizes_fit(&sh, &c, static_cast<int32_t>(tokens), static_cast<int32_t>(mq))) continue;
      const Plan pl = make_plan(&sh, &c, static_cast<int>(tokens), static_cast<int>(mq), prefill != 0, tune);
      CHECK(pl.rows == tokens * sh.n_q_heads);
      CHECK(pl.n_splits >= 1 && pl.split_keys >= 1);
      CHECK(static_cast<int64_t>(pl.n_splits) * pl.split_keys >= c.max_seq_len || (prefill && pl.mfma && !pl.short_prefill));
      CHECK(pl.off_ml % 256 == 0 && pl.off_o % 256 == 0 && pl.off_lr % 256 == 0 && pl.off_adapter % 256 == 0 && pl.off_qt % 256 == 0);
      CHECK(pl.bytes % 256 == 0);
      CHECK(pl.bytes == pl.bytes_without_kc + pl.kc_bytes && pl.off_kc % 256 == 0 && pl.kc_bytes % 256 == 0);
      if (pl.kc_bytes) {  // completed keys of a rotary prefill: a copy of the K_base extent behind everything else
        CHECK(prefill && pl.mfma && !pl.short_prefill && sh.key_rope_theta > 0.f);
        CHECK(pl.off_kc >= pl.bytes_without_kc);
        // contiguous: the extent of K_base; paged: the sequence's blocks in logical order at the strides of the pool
        const int64_t span = c.block_size == 0
            ? (static_cast<int64_t>(c.max_seq_len) - 1) * c.kv_token_stride +
                  (static_cast<int64_t>(sh.n_kv_heads) - 1) * c.kv_head_stride + sh.head_dim
            : (static_cast<int64_t>(c.max_seq_len) - 1) / 16 * c.kv_block_stride +
                  (static_cast<int64_t>(sh.n_kv_heads) - 1) * c.kv_head_stride + 15 * c.kv_token_stride + sh.head_dim;
        CHECK(pl.kc_bytes >= static_cast<size_t>(span) * 2 && pl.kc_bytes <= (size_t{1} << 32) + 256);
      }
      if (pl.bytes_without_kc) {
        const size_t slots = static_cast<size_t>(pl.rows) * pl.n_splits;
        CHECK(pl.off_o >= slots * 8 && pl.off_lr >= pl.off_o + slots * sh.head_dim * 4);
        CHECK(pl.off_adapter >= pl.off_lr + slots * sh.rank * 4 && pl.off_qt >= pl.off_adapter + static_cast<size_t>(pl.rows) * 4);
        CHECK(pl.bytes_without_kc >= pl.off_qt + pl.qt_bytes);
      }
      if (pl.l_block) {  // per-adapter low-rank caches on the MFMA decode path, one column block of the L tile per agent slot
        CHECK(!prefill && pl.mfma && c.l_adapter_stride > 0 && pl.row_tiles == 1 && !(sh.key_rope_theta > 0.f));
        CHECK(pl.l_block * (16 / pl.group_pad) <= 64 && pl.l_block >= sh.rank && pl.qt_bytes == 0);
        const int64_t pitch = c.l_row_stride ? c.l_row_stride : sh.rank;
        if (c.block_size == 0) {
          // contiguous cache (streaming form with at most one workgroup per compute unit, else split-KV form): a
          // wave's L rows inside 32-bit byte offsets
          CHECK(static_cast<int64_t>(pl.split_keys) / 4 * pitch * 2 < (int64_t{1} << 31));
        } else {
          // split-KV form on a paged cache: the whole pool of an adapter's L rows inside them
          CHECK(static_cast<int64_t>(c.num_blocks) * 16 * pitch * 2 < (int64_t{1} << 31));
        }
      }
      if (!prefill && c.n_seqs > 1 && c.n_seqs <= 2000) {
        // with a host copy of the lengths (any values: they are clamped) the key shares only grow, the workspace
        // only shrinks, and nothing else of the plan moves
        std::vector<int32_t> lens(static_cast<size_t>(c.n_seqs));
        for (auto& v : lens) v = static_cast<int32_t>(pick({-3, 0, 1, 17, c.max_seq_len / 2, c.max_seq_len, c.max_seq_len, INT32_MAX}));
        lra_cache cm = c;
        cm.seq_lens_host = lens.data();
        const Plan pm = make_plan(&sh, &cm, static_cast<int>(tokens), static_cast<int>(mq), false, tune);
        CHECK(pm.mfma == pl.mfma && pm.group_pad == pl.group_pad && pm.row_groups == pl.row_groups && pm.l_block == pl.l_block);
        CHECK(pm.split_keys >= pl.split_keys && pm.n_splits <= pl.n_splits && pm.bytes <= pl.bytes);
        CHECK(pm.split_keys % (pm.mfma ? 128 : 64) == 0);
        if (c.block_size == 0 && pm.mfma) CHECK(static_cast<int64_t>(pm.split_keys) * c.kv_token_stride * 2 < (int64_t{1} << 31));
      }
      const bool split_path = !prefill || pl.short_prefill || !pl.mfma;
      if (split_path && pl.mfma) {
        CHECK(pl.split_keys % 128 == 0);
        CHECK(pl.group_pad == 4 || pl.group_pad == 8 || pl.group_pad == 16);
        CHECK(pl.group_pad >= G && (pl.row_tiles == 1 || pl.row_tiles == 2));
        CHECK(static_cast<int64_t>(pl.row_groups) * pl.row_tiles * 16 >= (prefill ? tokens : mq) * pl.group_pad);
        if (c.block_size == 0) CHECK(static_cast<int64_t>(pl.split_keys) * c.kv_token_stride * 2 < (int64_t{1} << 31));
        CHECK(!pl.launchable || (pl.n_splits <= 65535 && static_cast<int64_t>(pl.row_groups) * (prefill ? 1 : c.n_seqs) <= 65535));
      } else if (split_path) {
        CHECK(pl.split_keys % 64 == 0);
      }
    }
  }
  // the split of lra_cache_append over d_model
  for (int it = 0; it < cases; ++it) {
    const int64_t n_new = pick({1, 16, 32, 33, 64, 100, 128, 129, 512, 1000, 1024, 4096, 1 << 20, (1 << 20) + 1, INT32_MAX});
    const int hkv = static_cast<int>(pick({1, 2, 3, 8, 64, 4096}));
    const int d = static_cast<int>(pick({64, 128}));
    const int r = static_cast<int>(pick({8, 16, 24, 64}));
    const int dm = static_cast<int>(pick({64, 128, 704, 768, 1024, 4096, 8192, 1 << 20}));
    lra_tuning t{};
    t.append_k_splits = static_cast<int32_t>(pick({0, 0, 1, 2, 3, 8, 16, 17, -1}));
    t.append_tile = static_cast<int32_t>(pick({0, 0, 0, 64, 128}));
    t.append_stages = static_cast<int32_t>(pick({0, 0, 0, 3}));
    const Tuning tune = resolve_tuning(&t);
    const AppendSplit sp = plan_append_split(static_cast<int>(n_new), hkv, d, r, dm, tune);
    CHECK(sp.k_splits >= 1 && sp.k_splits <= 16 && (sp.bt == 64 || sp.bt == 128));
    CHECK((sp.k_splits == 1) == (sp.bytes == 0));
    if (sp.k_splits > 1) {
      const int64_t n_feat = 2LL * hkv * d + r;
      CHECK((dm / 64) % sp.k_splits == 0 && n_new <= (1 << 20));
      CHECK(sp.bytes >= static_cast<size_t>(sp.k_splits) * n_new * n_feat * 4 && sp.bytes % 256 == 0);
      CHECK(tune.append_tile == 0 && tune.append_stages == 0 && tune.append_k_splits != 1);
      if (tune.append_k_splits == 0) {
        const int64_t tiles = (n_new + sp.bt - 1) / sp.bt * (2 * ((static_cast<int64_t>(hkv) * d + 127) / 128) + 1);
        CHECK(tiles * sp.k_splits <= kCUs && dm / 64 / sp.k_splits >= 4 && n_new > 32);
      }
    }
  }
  std::printf("plan_fuzz: %d cases, %d accepted by the argument checks, all plans consistent\n", cases, accepted);
  return accepted > cases / 10 ? 0 : 2;
}
