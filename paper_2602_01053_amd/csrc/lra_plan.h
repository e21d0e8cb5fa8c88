// Host-side launch planning of the Flash-LoRA-Attention library: argument checks and the choice
// of kernel family, key shares, row packing and workspace layout.  Plain C++ with no HIP
// dependency, so that the arithmetic (32-bit offset caps, workspace sizes) can also be compiled
// for the CPU alone and run under the address and undefined-behaviour sanitizers.
#pragma once

#include <stddef.h>
#include <stdint.h>

#include "lra_attn.h"

namespace lra {

constexpr int kCUs = 256;  // MI355X

// lra_tuning with every "0 = automatic" resolved.
struct Tuning {
  int variant = 0;          // 0 automatic, 1 vector-ALU kernels, 2 MFMA kernels without the streaming form
  int split_keys = 0;       // keys per workgroup in decode, 0 = automatic
  int short_prefill = 32;   // new tokens up to which a prefill takes the split-KV path (0 = never)
  int prefill_splits = 0;   // workgroups sharing the key tiles of a q tile, 0 = automatic
  bool rope_key_prepass = true;  // rotary prefill on contiguous caches: completed keys by a pre-pass
  int append_skinny = 64;   // new tokens up to which lra_cache_append streams the weights (0 = never)
  int append_stages = 0;    // LDS stages of the tiled append GEMM, 0 = chosen from the grid
  int append_tile = 0;      // output tile of the append GEMM, 0 = chosen from the grid
  int append_k_splits = 0;  // parts of d_model in the append GEMM: 0 = chosen from the grid, 1 = never split
  bool main_kernel_only = false;  // measurement: enqueue only the dominant kernel of a call
};
Tuning resolve_tuning(const lra_tuning* t);

struct Plan {
  bool mfma;
  bool short_prefill;  // prefill served by the split-KV decode kernels (few new tokens)
  int rows;        // query rows = (queries | new tokens) x Hq
  int split_keys;  // keys per split
  int n_splits;    // splits per sequence at max_seq_len
  int group_pad, row_tiles, row_groups;  // MFMA decode row packing
  int l_block;     // split-KV MFMA kernels with per-adapter low-rank caches: padded rank of one slot's column block, else 0
  bool launchable;  // false: a grid dimension would exceed the limit of 65535 in y or z (LRA_ERR_UNSUPPORTED)
  size_t off_ml, off_o, off_lr, off_adapter, off_qt, qt_bytes, bytes;
  // rotary prefill with the completed keys in the workspace: their offset and size (0: none), and
  // the size the plan has without them
  size_t off_kc, kc_bytes, bytes_without_kc;
};

lra_status check_common(const lra_shape* sh, const lra_cache* c);
// false: the call is too large for the planner's 32-bit row arithmetic (LRA_ERR_UNSUPPORTED)
bool plan_sizes_fit(const lra_shape* sh, const lra_cache* c, int32_t tokens, int32_t max_queries_per_seq);
Plan make_plan(const lra_shape* sh, const lra_cache* c, int tokens, int max_queries_per_seq, bool prefill,
               const Tuning& tune);

// lra_cache_append: parts of d_model the tiled GEMM is divided into (1: none), the token side of its
// tile, and the fp32 workspace the parts need.
struct AppendSplit {
  int k_splits, bt;
  size_t bytes;
};
AppendSplit plan_append_split(int n_new, int n_kv_heads, int head_dim, int rank, int d_model, const Tuning& tune);

// Row tiles per workgroup the split-KV MFMA kernels are built for.
int decode_mfma_row_tiles(int rows_needed);
// Agent slots a 16-row tile may hold in the rotary form of the split-KV kernel.
int decode_mfma_rope_slots(int rank);
// Bytes of workspace the Qt pre-pass of the streaming form takes (0: Qt is formed per workgroup).
size_t decode_stream_qt_bytes(int group_pad, int rank, int row_tiles, int row_groups, int n_kv_heads);

}  // namespace lra
