/*
 * lra_attn.h - C ABI of the Flash-LoRA-Attention library for MI355X (gfx950).
 *
 * Method: LRAgent (arxiv 2602.01053), Sec. 3.3 and Alg. 1 ("Flash-LoRA-Attention
 * forward"), App. B (reordering by associativity), App. D.1 (the same
 * decomposition on the key side).
 *
 * Every agent of a multi-LoRA system attends over ONE shared base cache
 * (K_base, V_base) and ONE shared low-rank cache L (n x r, the activations right
 * after the shared LoRA down-projection; Sec. 3.2 "BaseLRShared").  Agent a's own
 * keys and values are, by definition,
 *
 *     K^a = K_base + L . B_K^a        V^a = V_base + L . B_V^a
 *
 * and are never formed.  The library evaluates O = softmax(scale . Q K^a^T) V^a as
 *
 *     S = scale . ( Q K_base^T + (Q B_K^T) L^T )        (App. D.1 reordering)
 *     O = ( P V_base + (P L) B_V ) / rowsum             (Sec. 3.3, Alg. 1)
 *
 * inside an online-softmax loop over key tiles, with the rank-r accumulator P.L
 * carried next to the head-dimension accumulator and B_V applied once at the end.
 *
 * Conventions that hold for every entry point
 *   - Pointers marked DEVICE point to memory of the current HIP device, pointers
 *     marked HOST to ordinary host memory.  Nothing is copied across.
 *   - Ownership: every buffer belongs to the caller.  The library allocates and
 *     frees nothing and keeps no pointer after a call returns.
 *   - Asynchronous: kernels are enqueued on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream).  No call synchronises.  Outputs are valid
 *     once the stream has reached the end of the enqueued work.
 *   - Errors: a status code is returned; nothing is thrown and nothing aborts.
 *     All argument checks run before the first launch, so a status other than
 *     LRA_OK (except LRA_ERR_HIP) means nothing was enqueued.  Inputs are never
 *     written.
 *   - Deterministic: equal arguments give bitwise equal outputs.
 *   - Re-entrant: the library holds no mutable state apart from the one-time, per-device
 *     lookup of lra_attn_decode_static's buffer; calls from several threads need no lock.
 *   - The caches already contain the rows of the new query tokens: a sequence of
 *     n tokens holds L_p old and L_c new ones, n = L_p + L_c (Alg. 1, first line).
 *   - Element type `dtype` applies to Q, K_base, V_base, L, B_K, B_V and the
 *     output alike.  Accumulation is always fp32.
 *   - Alignment: all DEVICE tensor pointers 16-byte aligned; the cache strides
 *     multiples of 8 elements.
 *
 * Supported: head_dim in {64, 128}; 1 <= rank <= 64; n_q_heads a multiple of
 * n_kv_heads with a group of at most 16; q head g reads kv head g / (Hq/Hkv);
 * block_size 0 (contiguous) or 16; dtype bf16 (MFMA kernels) or fp32 (vector-ALU
 * kernels; bf16 ranks that are not a multiple of 8 take those as well - padding L with zero
 * columns and B_K, B_V with zero rows to the next multiple of 8 gives the same outputs on the
 * MFMA kernels).  Size caps: n_q_heads <= 4096, n_seqs <= 2^20, max_seq_len <= 2^30,
 * query rows (queries or new tokens times n_q_heads) <= 2^30, kv_token_stride <= 2^31,
 * kv_head_stride and kv_block_stride <= 2^40 elements, num_blocks * kv_block_stride <= 2^60,
 * at most 65535 key shares per sequence and 65535 (sequence, row group) pairs per call.
 * Anything else returns LRA_ERR_UNSUPPORTED.
 */
#ifndef LRA_ATTN_H
#define LRA_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LRA_OK = 0,
  LRA_ERR_NULL = 1,        /* a required pointer is NULL */
  LRA_ERR_SHAPE = 2,       /* a size or stride is out of range or inconsistent */
  LRA_ERR_DTYPE = 3,       /* dtype is not one of lra_dtype */
  LRA_ERR_UNSUPPORTED = 4, /* valid, but outside the supported set above */
  LRA_ERR_WORKSPACE = 5,   /* workspace NULL, misaligned or smaller than required */
  LRA_ERR_HIP = 6          /* a HIP launch reported an error */
} lra_status;

typedef enum { LRA_BF16 = 0, LRA_F32 = 1 } lra_dtype;

/* Attention shape of one layer. */
typedef struct {
  int32_t n_q_heads;  /* Hq */
  int32_t n_kv_heads; /* Hkv */
  int32_t head_dim;   /* d = d_head of Alg. 1 */
  int32_t rank;       /* r, columns of the LR cache and rows of every B */
  int32_t dtype;      /* lra_dtype */
  float scale;        /* softmax scale; 0.0f selects 1/sqrt(head_dim) (the score step of Alg. 1).
                         The rank never enters the scale. */
  float key_rope_theta; /* 0: the key-side adapter is added as it is, K = K_base + L B_K, and
                         the scores are reordered (App. D.1 without a rotation).
                         > 0: the rotary setting of App. D.1 (LoRA on the key projection of a
                         model with rotary embeddings, the qkvo ablation): K_base holds rotated
                         keys, and the adapter's contribution, reconstructed in the head
                         dimension, is rotated by its token's position before the score,
                           K_j = K_base,j + RoPE_j(L_j B_K),
                         rotate-half pairs (i, i + d/2), angle j * theta^(-2i/d), position j =
                         the token's index in its sequence.  Q is the caller's (rotated) query.
                         The value side is unchanged.  bf16 with rank % 8 == 0 runs on MFMA
                         kernels (decode and prefills of a few tokens: the split-KV kernel
                         rotates L B_K per key tile in registers, once for every agent of the
                         tile; other prefills complete each key tile in LDS), everything else
                         on the vector-ALU kernels.  Those other prefills hold the completed
                         keys as fp16 (a second rounding to bf16 would cost more accuracy than
                         the rest of the call): key magnitudes must stay below 65504 there. */
} lra_shape;

/*
 * Shared base cache + shared LR cache (Sec. 3.2: one copy for all agents).
 *
 * Contiguous form (block_size == 0), exactly one sequence:
 *   token j, kv head h of K_base is the d elements at
 *       k_base + j*kv_token_stride + h*kv_head_stride        (units: elements)
 *   token-major [n][Hkv][d] is token_stride = Hkv*d, head_stride = d;
 *   head-major  [Hkv][n][d] is token_stride = d,     head_stride = n*d.
 *   L is dense [n][rank].
 *
 * Paged form (block_size == 16): token j of sequence t lives in physical block
 *   b = block_table[t*max_blocks_per_seq + j/16], slot j%16, at
 *       k_base + b*kv_block_stride + h*kv_head_stride + (j%16)*kv_token_stride
 *   ([num_blocks][Hkv][16][d] is block_stride = Hkv*16*d, head_stride = 16*d,
 *   token_stride = d).  L is dense [num_blocks][16][rank].
 *   Block-table entries past a sequence's last block are never read.  Entries that
 *   are read must lie in [0, num_blocks); they are not checked on the device.
 *   Slots past seq_lens[t] inside the last block may hold anything, NaN included.
 *
 * v_base uses the same strides as k_base.
 *
 * Low-rank cache.  Row (token j) of adapter a is the `rank` elements at
 *       l + a*l_adapter_stride + row_index*l_row_stride
 *   with row_index = j (contiguous) or b*16 + j%16 (paged), l_row_stride = 0 meaning rank.
 *   l_adapter_stride = 0 is the paper's final scheme, BaseLRShared: one L for every agent
 *   (the shared down-projection), all agents' keys and values are K_base + L B_K^a,
 *   V_base + L B_V^a.  l_adapter_stride > 0 is BaseShared: agent a attends over
 *   K_base + L_a B_K^a, V_base + L_a B_V^a with its own L_a; [n][A][r] storage is
 *   row stride A*r, adapter stride r; [A][n][r] storage is row stride r, adapter stride n*r.
 *   Both strides are multiples of 8 elements (a row stride equal to the rank is always accepted).
 *   The byte model changes with it: a decode call
 *   streams the L rows of every agent on the sequence (A*r instead of r elements per token).
 *   Kernels: bf16 with rank % 8 == 0 runs on the MFMA kernels.  Decode without the rotary
 *   key side reads K_base / V_base once for the agents of a row tile (each brings its own
 *   column block of the L tile, so a tile holds 4 agents at rank <= 16, 2 at rank <= 32, 1
 *   above; on a paged cache the low-rank rows of one adapter, num_blocks * 16 rows at the row
 *   stride, must then lie within 2 GB); decode with the rotary key side, or beyond that
 *   size, gives every agent a row tile and a workgroup of its own, which requests K_base /
 *   V_base once per agent (the later requests are served by L2); prefill reads the one
 *   agent's rows with their stride.  Other dtypes and ranks run on the vector-ALU
 *   kernels.  lra_cache_append fills adapter 0's rows only (BaseLRShared is the scheme with
 *   one producer call per token).
 */
typedef struct {
  const void* k_base;          /* DEVICE */
  const void* v_base;          /* DEVICE */
  const void* l;               /* DEVICE */
  int64_t kv_token_stride;
  int64_t kv_head_stride;
  int64_t kv_block_stride;     /* paged only */
  int32_t block_size;          /* 0 or 16 */
  int32_t max_blocks_per_seq;  /* paged only: row length of block_table */
  int32_t num_blocks;          /* paged only */
  int32_t n_seqs;              /* 1 when contiguous */
  int64_t l_row_stride;        /* elements between consecutive L rows; 0 = dense (rank) */
  int64_t l_adapter_stride;    /* 0: ONE low-rank cache for all agents (BaseLRShared).
                                  > 0: BaseShared (Sec. 3.2) - every adapter a has its own
                                  low-rank cache L_a = X A_a, whose row of a token starts
                                  a * l_adapter_stride elements after that token's row of
                                  adapter 0 (see below) */
  const int32_t* block_table;  /* DEVICE int32 [n_seqs][max_blocks_per_seq]; NULL when contiguous */
  const int32_t* seq_lens;     /* DEVICE int32 [n_seqs]: cached tokens n_t of each sequence, >= 1 */
  int32_t max_seq_len;         /* HOST-known upper bound of every seq_lens[t]; sizes the launch.
                                  The attention calls treat a longer sequence as if it ended
                                  there (decode: its first max_seq_len tokens; prefill: the new
                                  tokens are taken to be the last of those).  lra_cache_append
                                  writes nothing for a sequence whose device-side length
                                  exceeds it. */
  const int32_t* seq_lens_host; /* HOST int32 [n_seqs], optional (NULL: unknown): what the caller
                                  believes seq_lens holds.  Read during the call, never after it
                                  returns, and used for launch planning only: the decode of a
                                  batch sizes its key shares so that the workgroups that find
                                  keys fill the compute units once (sequences of about equal
                                  length) or just under twice (ragged lengths); without it a
                                  batch is taken to be half as long on average as max_seq_len.
                                  The results do
                                  not depend on it; entries outside [0, max_seq_len] are clamped.
                                  Key shares only grow with it, so a workspace sized with NULL
                                  here serves every call on the same shapes. */
} lra_cache;

/*
 * Per-agent adapter table (Sec. 3.2: every agent turns the shared caches into its own
 * keys and values through its own up-projection B_i).
 * Adapter ids (query_adapter) are device data the host cannot check: the kernels clamp them
 * into [0, n_adapters), so a bad id selects a wrong adapter but never reads outside the tables.
 * b_k / b_v: DEVICE [n_adapters][rank][Hkv*head_dim], row-major; kv head h owns
 * columns h*d .. (h+1)*d-1 (Eq. 1: B is r x d_out).  Any LoRA scaling alpha/r is
 * folded into B by the caller.  b_k == NULL means B_K = 0 for every adapter (the
 * paper's main setting: keys fully shared); b_v == NULL means B_V = 0.  With b_k == NULL
 * the bf16 kernels skip the key-side adapter work altogether (no Q B_K^T, no L term in the
 * scores) instead of computing it with zeros.
 */
typedef struct {
  const void* b_k;
  const void* b_v;
  int32_t n_adapters;
} lra_adapters;

/*
 * Optional per-call tuning, passed by pointer to every entry point (NULL, or a zero-filled
 * struct, selects the automatic choice everywhere).  The library keeps no tuning state of
 * its own: the same struct must be given to lra_workspace_bytes and to the call it sizes.
 * None of the fields changes a result beyond rounding.
 *   kernel_variant     0 automatic (MFMA kernels for bf16, vector-ALU kernels for fp32; among the
 *                      MFMA kernels, decode calls on a contiguous cache that give every compute
 *                      unit at most one workgroup take the form with two tile stages per wave and
 *                      separate prologue waves); 1 vector-ALU kernels for every dtype; 2 automatic
 *                      without that form
 *   decode_split_keys  keys per workgroup in decode (the flash-decoding split size), rounded up
 *                      to the kernel's key tile; 0 automatic
 *   short_prefill      bf16 prefill calls with at most this many new tokens (and a context at
 *                      least four times as long) run on the split-KV decode kernels, the new
 *                      tokens standing in for the agents; 0 automatic (32, the measured
 *                      crossover), negative: never
 *   prefill_splits     workgroups that share the key tiles of one q tile in the tile-walking
 *                      prefill kernel (1..32; more than one ends with the merge kernel);
 *                      0 automatic (two workgroups per CU, at least eight 64-key tiles each)
 *   rope_key_prepass   prefill calls of the tile-walking kernel with the rotary key side
 *                      (key_rope_theta > 0 and a b_k): 0 automatic (the completed keys
 *                      K_base + RoPE(L B_K) of the call's adapter and sequence are written once
 *                      into the workspace by a pre-pass and the call runs on them: the workspace
 *                      then holds a copy of the K_base extent, (max_seq_len - 1) * kv_token_stride
 *                      + (Hkv - 1) * kv_head_stride + head_dim elements, or for a paged cache the
 *                      blocks of one sequence in logical order at the strides of the pool,
 *                      ((max_seq_len - 1) / 16) * kv_block_stride + (Hkv - 1) * kv_head_stride +
 *                      15 * kv_token_stride + head_dim elements; up to 4 GB; a call whose
 *                      workspace is too small for that but large enough otherwise completes the
 *                      key tiles inside the kernel instead, at a cost in time); negative: never
 *   append_skinny      lra_cache_append calls with at most this many new tokens stream the
 *                      weights instead of tiling; 0 automatic (64), negative: never
 *   append_stages      LDS stages of lra_cache_append's tiled GEMM: 2, 3 or 4; 0 automatic
 *   append_tile        output tile of that GEMM: 64, 128 or 256; 0 automatic
 *   append_k_splits    parts d_model is divided into when lra_cache_append is given a workspace:
 *                      0 automatic (from the sizes), 1 never, 2..16 that many where d_model / 64
 *                      is a multiple of it
 *   measure_main_kernel_only  1: the call enqueues only its dominant kernel (the key-streaming
 *                      kernel) so that a benchmark can time it alone; `out` is NOT produced.
 *                      For measurement only (see lra_attn_measure.h).
 */
typedef struct {
  int32_t kernel_variant;
  int32_t decode_split_keys;
  int32_t short_prefill;
  int32_t prefill_splits;
  int32_t rope_key_prepass;
  int32_t append_skinny;
  int32_t append_stages;
  int32_t append_tile;
  int32_t append_k_splits;
  int32_t measure_main_kernel_only;
} lra_tuning;

/*
 * Bytes of DEVICE workspace a call needs; 0 is a valid answer.
 *   n_new == 0 : for lra_attn_decode with these n_queries / max_queries_per_seq
 *   n_new >= 1 : for lra_attn_prefill with this n_new (the two query counts are ignored)
 * Returns (size_t)-1 when the arguments themselves would be rejected.  The answer
 * depends on `tuning`: pass the struct the call itself will get.
 */
size_t lra_workspace_bytes(const lra_shape* shape, const lra_cache* cache, int32_t n_queries,
                           int32_t max_queries_per_seq, int32_t n_new, const lra_tuning* tuning);

/*
 * Decode step for many agents at once (Alg. 1 with L_c = 1 per query, the
 * flash-decoding split over keys the paper builds on, and the adapter table).
 *
 * Query i is one new token of one agent.  It attends over all seq_lens[t] cached
 * tokens of its sequence t (no mask) with adapter query_adapter[i].  Queries are
 * grouped by sequence: sequence t owns queries seq_query_start[t] ..
 * seq_query_start[t+1]-1, so all agents working on one sequence share a single
 * pass over that sequence's K_base, V_base and L.
 *
 *   q                DEVICE [n_queries][Hq][d]
 *   query_adapter    DEVICE int32 [n_queries], values in [0, n_adapters)
 *   seq_query_start  DEVICE int32 [n_seqs+1], non-decreasing, [0] = 0, [n_seqs] = n_queries
 *   max_queries_per_seq  HOST-known upper bound of the per-sequence query count
 *   out              DEVICE [n_queries][Hq][d], same dtype as q
 *   workspace        DEVICE, 256-byte aligned, >= lra_workspace_bytes(...); contents
 *                    undefined afterwards.  Calls that overlap in time need
 *                    separate workspaces.
 */
lra_status lra_attn_decode(const lra_shape* shape, const lra_cache* cache,
                           const lra_adapters* adapters, const void* q,
                           const int32_t* query_adapter, const int32_t* seq_query_start,
                           int32_t n_queries, int32_t max_queries_per_seq, void* out,
                           void* workspace, size_t workspace_bytes, const lra_tuning* tuning,
                           void* stream);

/*
 * lra_attn_decode for callers that cannot allocate or size a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels
 * and bit for bit the same output as lra_attn_decode, but the split-KV partial states go to
 * a buffer of LRA_STATIC_WORKSPACE_BYTES that is part of the library's device image (every GPU
 * the library runs on holds one copy until the process ends).  The call allocates and frees
 * nothing.  The first call on a device looks up that device's copy of the buffer (one HIP
 * query, no allocation); make that first call outside graph capture.
 *   - LRA_ERR_WORKSPACE, with nothing enqueued, when the call would need more than
 *     LRA_STATIC_WORKSPACE_BYTES (lra_workspace_bytes gives the need).
 *   - All calls on one GPU share that GPU's buffer: calls that overlap in time on one GPU
 *     (different streams, or threads) race on it and must be serialised by the caller.
 *     Nothing in the buffer has to survive from one call to the next.
 */
#define LRA_STATIC_WORKSPACE_BYTES ((size_t)64 << 20)
lra_status lra_attn_decode_static(const lra_shape* shape, const lra_cache* cache,
                                  const lra_adapters* adapters, const void* q,
                                  const int32_t* query_adapter, const int32_t* seq_query_start,
                                  int32_t n_queries, int32_t max_queries_per_seq, void* out,
                                  const lra_tuning* tuning, void* stream);

/*
 * Causal prefill of one agent (Alg. 1 as printed: L_c = n_new query tokens after
 * L_p cached ones).  The n_new query tokens are the LAST n_new tokens of sequence
 * seq_index, whose cache rows are already in place; new token i sees keys
 * 0 .. n_t - n_new + i ("Mask" in the score step of Alg. 1, aligned to the end).
 *
 *   q    DEVICE [n_new][Hq][d]        out  DEVICE [n_new][Hq][d]
 *   seq_index in [0, n_seqs), adapter_index in [0, n_adapters)
 *   1 <= n_new <= max_seq_len; the device-side seq_lens[seq_index] must be >= n_new.
 */
lra_status lra_attn_prefill(const lra_shape* shape, const lra_cache* cache,
                            const lra_adapters* adapters, const void* q, int32_t seq_index,
                            int32_t adapter_index, int32_t n_new, void* out, void* workspace,
                            size_t workspace_bytes, const lra_tuning* tuning, void* stream);

/*
 * Projection weights of one attention layer for lra_cache_append.
 * w: DEVICE [2*Hkv*head_dim + rank][d_model], row-major, one output feature per row (the
 * layout of a linear layer's weight): first W_K (kv head h owns rows h*d .. (h+1)*d-1), then
 * W_V, then the shared LoRA down-projection A (Eq. 1: Delta W = A B, A is d_model x r), one
 * rank per row.  16-byte aligned; d_model a multiple of 64.
 * rope_theta > 0 rotates the keys by the rotary position embedding in its rotate-half form
 * (pair (i, i + d/2) of the token at position j by the angle j * rope_theta^(-2i/d)) before
 * they are cached - the cached keys are the rotated ones (App. D.1); 0 stores them unrotated.
 */
typedef struct {
  const void* w;
  int32_t d_model;
  float rope_theta;
} lra_projection;

/*
 * The step before the attention path (Sec. 3.2 and the diagram of base and LR cache
 * computation): for the LAST n_new tokens of sequence seq_index, whose length seq_lens
 * already counts them, compute from their hidden states x
 *     K_base rows = rope(x W_K^T),   V_base rows = x W_V^T,   L rows = x A
 * (fp32 accumulation, one rounding to bf16) and write them into the caches described by
 * `cache`, whose k_base / v_base / l are WRITTEN by this call although declared const in
 * the struct.  Only BaseLRShared needs this once per appended token, for all agents.
 *
 *   x  DEVICE [n_new][d_model], dense, 16-byte aligned
 * bf16 only; head_dim in {64, 128}; rank a multiple of 8.  Asynchronous on `stream` like the
 * other calls.
 *   workspace  DEVICE, 256-byte aligned, optional (NULL, 0): with at least
 *              lra_append_workspace_bytes(...) bytes, chunks whose output would occupy a fraction
 *              of the chip (some tens to about a thousand tokens) divide d_model among several
 *              workgroups per output tile and finish in a second kernel; without it every size
 *              runs as one kernel.  Contents undefined afterwards; calls that overlap in time
 *              need separate workspaces.
 */
lra_status lra_cache_append(const lra_shape* shape, const lra_cache* cache, const lra_projection* proj,
                            const void* x, int32_t seq_index, int32_t n_new, void* workspace,
                            size_t workspace_bytes, const lra_tuning* tuning, void* stream);

/*
 * Bytes of DEVICE workspace with which lra_cache_append takes its fastest path for this n_new;
 * 0 when the call has no use for one.  (size_t)-1 when the arguments would be rejected.
 */
size_t lra_append_workspace_bytes(const lra_shape* shape, const lra_cache* cache,
                                  const lra_projection* proj, int32_t n_new, const lra_tuning* tuning);

/* Static, NUL-terminated description of a status code. */
const char* lra_status_string(lra_status status);

#ifdef __cplusplus
}
#endif
#endif /* LRA_ATTN_H */
