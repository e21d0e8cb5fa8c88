// Shared declarations of the Flash-LoRA-Attention HIP library (gfx950 only).
// Kernel parameter block, element conversion and wavefront (64 lanes) helpers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lra {

constexpr int kWave = 64;

// One parameter block for every kernel of the library.  Pointers are device
// pointers; strides are in elements.
struct Params {
  const void* q;
  const void* k_base;
  const void* v_base;
  const void* l;
  const void* b_k;  // may be null: B_K = 0
  const void* b_v;  // may be null: B_V = 0
  void* out;
  const int32_t* block_table;
  const int32_t* seq_lens;
  const int32_t* query_adapter;
  const int32_t* seq_query_start;
  // split-KV partial state, fp32 (Alg. 1's m, l, O, O_lr per query row and split)
  float* part_ml;  // [rows][n_splits][2]
  float* part_o;   // [rows][n_splits][d]
  float* part_lr;  // [rows][n_splits][r]
  int32_t* part_adapter;  // [rows]: adapter of the row's query, left by the first kernel for the merge
  void* qt_ws;            // Qt = Q B_K^T of the whole call in MFMA operand order, or null (formed per workgroup)
  int64_t kv_token_stride, kv_head_stride, kv_block_stride;
  int64_t l_row_stride;      // elements between L rows (>= rank)
  int64_t l_adapter_stride;  // elements between the L rows of consecutive adapters; 0: one L for all
  int32_t l_block;           // split-KV MFMA kernels, per-adapter L: padded rank of one agent slot's column block (16, 32, 64); 0: one L
  int32_t n_q_heads, n_kv_heads, group, head_dim, rank;
  int32_t group_pad;   // rows reserved per agent in the MFMA row tiles: 4, 8 or 16 (>= group)
  int32_t row_groups;  // workgroups along the query-row axis per (sequence, kv head)
  int32_t block_size, max_blocks_per_seq, num_blocks, n_seqs, max_seq_len;
  int32_t n_queries, max_queries_per_seq;
  int32_t n_adapters;
  int32_t n_new;          // query tokens of the prefill call, 1 in decode
  int32_t is_prefill;     // 0: decode (rows = queries x Hq), 1: prefill (rows = new tokens x Hq)
  int32_t seq_index, adapter_index;  // prefill only
  int32_t split_keys, n_splits;
  float scale;
  float key_rope_theta;  // > 0: the key-side adapter contribution is rotated by its token's position
  int32_t share_major;       // decode_stream_kernel: workgroup index laid out so that all kv heads of a key share run on one XCD
  int32_t keys_f16;          // prefill_mfma_kernel: k_base holds completed keys K_base + RoPE(L B_K) as fp16 (left by the key pre-pass)
  int32_t rg_interleave;     // decode_mfma_kernel with several row groups: 0, or the power of two m of the grid layout that
                             // puts the row groups of a (sequence, kv head, key share) on one XCD, next to each other in time
#ifdef LRA_TIMING
  unsigned long long* timing;  // instrumented test build only: per-wave phase stamps
#endif
};

typedef uint16_t bf16_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t x) {
  return __uint_as_float(static_cast<uint32_t>(x) << 16);
}

// round to nearest even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<bf16_t>((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<bf16_t>(u >> 16);
}

template <typename T> __device__ __forceinline__ float to_f32(T x);
template <> __device__ __forceinline__ float to_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t x) { return bf16_to_f32(x); }

template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float x) { return f32_to_bf16(x); }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
  return v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// Element offset of (sequence t, token j, kv head h) in K_base / V_base.
__device__ __forceinline__ int64_t kv_offset(const Params& p, int t, int j, int h) {
  if (p.block_size == 0) return static_cast<int64_t>(j) * p.kv_token_stride + static_cast<int64_t>(h) * p.kv_head_stride;
  const int blk = p.block_table[static_cast<int64_t>(t) * p.max_blocks_per_seq + (j >> 4)];
  return static_cast<int64_t>(blk) * p.kv_block_stride + static_cast<int64_t>(h) * p.kv_head_stride +
         static_cast<int64_t>(j & 15) * p.kv_token_stride;
}

// Element offset of (sequence t, token j) in the L rows of adapter a.
__device__ __forceinline__ int64_t l_offset(const Params& p, int t, int j, int a) {
  const int64_t base = static_cast<int64_t>(a) * p.l_adapter_stride;
  if (p.block_size == 0) return base + static_cast<int64_t>(j) * p.l_row_stride;
  const int blk = p.block_table[static_cast<int64_t>(t) * p.max_blocks_per_seq + (j >> 4)];
  return base + (static_cast<int64_t>(blk) * 16 + (j & 15)) * p.l_row_stride;
}

// Launchers (defined next to their kernels).
hipError_t launch_generic_partials(const Params& p, bool is_bf16, int rows, hipStream_t s);
hipError_t launch_merge(const Params& p, bool is_bf16, int rows, hipStream_t s);
hipError_t launch_decode_mfma(const Params& p, int row_tiles, bool allow_stream_form, bool main_kernel_only, hipStream_t s);
bool decode_stream_applies(const Params& p, int row_tiles, int n_cus);
hipError_t launch_decode_stream(const Params& p, int row_tiles, bool main_kernel_only, hipStream_t s);
hipError_t launch_prefill_mfma(const Params& p, hipStream_t s);
// rotary key side, contiguous cache: the completed keys of the call's adapter, in K_base's layout, into kc
hipError_t launch_complete_rope_keys(const Params& p, void* kc, hipStream_t s);

// Arguments of the cache-append producer kernel.
struct AppendParams {
  const void* x;   // [n_new][d_model]
  const void* w;   // [2*Hkv*d + rank][d_model]
  void* k_base;
  void* v_base;
  void* l;
  const int32_t* block_table;
  const int32_t* seq_lens;
  int64_t kv_token_stride, kv_head_stride, kv_block_stride;
  int64_t l_row_stride;  // elements between L rows (>= rank); the rows of adapter 0 are written
  int32_t d_model, n_kv_heads, head_dim, rank, n_new, seq_index;
  int32_t block_size, max_blocks_per_seq, max_seq_len;
  float rope_theta;
  int stages;      // LDS stages of the tiled GEMM: 0 = chosen from the grid, else 2, 3 or 4
  int tile;        // output tile of the GEMM kernels: 0 = chosen from the grid, 128 or 256
  int skinny_max;  // up to this many new tokens the weight-streaming kernel runs instead of the tiled GEMM
  // split over d_model: parts (1 = none), token side of the tile (64 or 128), fp32 partial sums [part][token][feature]
  int k_splits, split_bt;
  float* split_ws;
};
hipError_t launch_append(const AppendParams& p, hipStream_t s);

}  // namespace lra
