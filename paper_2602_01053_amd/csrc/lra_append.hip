// Cache-append producer of the Flash-LoRA-Attention library (bf16, gfx950): the step before
// the attention path.  For the new tokens of one sequence it forms
//     [K' | V | L] = X . [W_K | W_V | A]          (LRAgent Sec. 3.2: base cache from the
//                                                  pretrained projections, LR cache from the
//                                                  shared LoRA down-projection)
// rotates the keys by the model's rotary position embedding (the cached keys are the rotated
// ones, App. D.1) and writes the rows into K_base, V_base and L, contiguous or paged.
//
// Four kernels, chosen by the number of new tokens (launch_append at the end of the file): a
// matrix-vector kernel (1-2 tokens), a weight-streaming MFMA kernel (up to 64), and two tiled
// GEMM kernels (128 features x 128 or 64 tokens per workgroup; 256 x 256 for chunks whose tiles
// fill whole rounds of the chip).
//
// The tiled GEMM takes the weights one output feature per row (the usual layout of a linear
// layer) and computes transposed, Y^T[feature][token] = W[feature][:] . X[token][:], so
// that both operands are rows of 16-byte chunks along d_model (ds_read_b128, no transposed
// reads) and every lane ends up with four consecutive features of one token: an 8-byte
// store into a cache row.  A workgroup walks d_model in steps of 64; the W and X tiles go
// from HBM straight into a ring of 2 to 4 LDS stages (buffer_load ... lds, swizzled by
// choosing which chunk a lane fetches).  The four waves form a 2 x 2 grid; a wave's two
// 32-feature blocks are chosen d/2 apart, so the two halves of every rotary pair sit in the
// same lane and register of its two accumulators and the rotation needs no data movement.
// The rotation rate of every pair is tabulated once per workgroup in double precision
// (revolutions per position); angle = fractional part of position * rate, so positions in
// the tens of thousands lose nothing.
#include "lra_prefill_util.h"

namespace lra {

// Length of the sequence the new rows are appended to.  max_seq_len is exact for this call: it
// sizes the caches, so a device-side length beyond it cannot be honoured - such a call writes
// nothing (every row index comes out negative and is skipped) rather than overwrite live rows.
__device__ __forceinline__ int append_length(int len, int max_seq_len) { return len <= max_seq_len ? len : 0; }


// BT = 64 halves the token side of the tile (a wave then owns 64 features x 32 tokens): twice the
// workgroups and three quarters of the bytes per step for chunks too small to fill the chip.
// SPLITK: blockIdx.z takes one of p.k_splits equal parts of d_model and leaves its fp32 sums in the
// workspace, [part][token][feature] (feature = row of w); append_finish_kernel adds the parts,
// rotates, casts and stores.  For chunks whose output tiles would occupy a fraction of the chip
// and walk all of d_model one step after the other.
template <int D, bool PAGED, int NS, int BT = 128, bool SPLITK = false>
__global__ __launch_bounds__(256, NS == 2 ? 2 : 1) void append_kernel(AppendParams p) {
  constexpr int BF = 128, BK = 64;  // features, d_model step (BT tokens)
  constexpr bool ONE_TB = BT == 64;  // one 32-token block per wave
  constexpr int REQ = ONE_TB ? 6 : 8;  // requests per step and wave
  constexpr int TILE_BYTES = BF * BK * 2;      // the W tile: 128 rows of 128 bytes
  constexpr int STAGE = TILE_BYTES + BT * BK * 2;  // [W tile][X tile]
  constexpr int HALF = D / 2;

  __shared__ __align__(16) unsigned char smem[NS * STAGE];
  __shared__ double rope_rate[D / 2];  // revolutions per position of every rotary pair

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, g2 = lane >> 5;
  const int wr = wave >> 1, wc = wave & 1;  // position in the 2 x 2 grid of waves: features, tokens
  const int HD = p.n_kv_heads * D;
  const int n_ct_kv = (HD + BF - 1) / BF;   // feature tiles of the K (and of the V) region
  // The L tiles (little matrix work) come first in the grid, so they run beside the first full
  // tiles instead of as a round of their own at the end.
  const int ct = static_cast<int>(blockIdx.y) - 1;
  const int kind = ct < 0 ? 2 : (ct < n_ct_kv ? 0 : 1);  // 0 K, 1 V, 2 L
  const int ct_in = kind == 0 ? ct : (kind == 1 ? ct - n_ct_kv : 0);
  const int feat0 = ct_in * BF;                                 // first feature of the tile inside its region
  const int w_row0 = (kind == 0 ? 0 : (kind == 1 ? HD : 2 * HD)) + feat0;  // its row of w
  const int tok0 = blockIdx.x * BT;
  const int n_new = p.n_new;
  const int n_t = append_length(PF_CONST_I32(p.seq_lens)[p.seq_index], p.max_seq_len);
  const int pos0 = n_t - n_new;  // cache row (= position) of new token 0

  // ---------------- tile traffic ----------------
  // A wave-wide load moves 8 rows of 128 bytes.  Load i fills rows 8i ..; lane l lands at row
  // 8i + l/8, physical chunk l%8, and fetches logical chunk (l%8) ^ ((row >> 1) & 7).  Wave w
  // issues loads i = w, w+4, w+8, w+12 of either tile: the swizzle of its rows does not
  // depend on the load, so one offset per lane serves all of them.  Rows past the end of w
  // (the L tile holds fewer than 128 features) or of x read as zero.
  const uint32_t ldw2 = static_cast<uint32_t>(p.d_model) * 2u;
  const uint32_t n_w_rows = static_cast<uint32_t>(2 * HD + p.rank);
  const pf_u32x4 rs_w = pf_rsrc(p.w, (n_w_rows - 1) * ldw2 + ldw2);
  const pf_u32x4 rs_x = pf_rsrc(p.x, static_cast<uint32_t>(n_new - 1) * ldw2 + ldw2);
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(PF_LDS_AS(unsigned char, smem)));
  const uint32_t voff = static_cast<uint32_t>(lane >> 3) * ldw2 +
                        (((lane & 7) ^ ((4 * wave + (lane >> 4)) & 7)) << 4);
  // request number part (0..7) of this wave for the step at k0: W and X alternate
  auto issue_part = [&](int k0, int st, int part) __attribute__((always_inline)) {
    const int i = wave + 4 * (part >> 1);
    const uint32_t dst = lds0 + st * STAGE + i * 1024;
    if ((part & 1) == 0) pf_load16_to_lds(rs_w, dst, voff, static_cast<uint32_t>(w_row0 + 8 * i) * ldw2 + k0 * 2);
    else if (8 * i < BT) pf_load16_to_lds(rs_x, dst + TILE_BYTES, voff, static_cast<uint32_t>(tok0 + 8 * i) * ldw2 + k0 * 2);
  };
  auto issue_step = [&](int k0, int st) __attribute__((always_inline)) {
#pragma unroll
    for (int part = 0; part < 8; ++part) issue_part(k0, st, part);
  };
  const int n_steps = SPLITK ? p.d_model / BK / p.k_splits : p.d_model / BK;
  const int k_first = SPLITK ? static_cast<int>(blockIdx.z) * n_steps * BK : 0;  // first d_model index of this part
#pragma unroll
  for (int st = 0; st < NS - 1; ++st)
    if (st < n_steps) issue_step(k_first + st * BK, st);
  if constexpr (!SPLITK)  // (the finishing kernel rotates)
    if (tid < D / 2 && p.rope_theta > 0.f) rope_rate[tid] = rope_rate_rev(tid, D, p.rope_theta);  // read after the loop's barriers

  // ---------------- operands ----------------
  // A operand: W rows (features), B operand: X rows (tokens); lane (row l32 of a 32-row block,
  // k = 16ks + 8g2 + e): the 16-byte chunk 2ks + g2 of its row, at chunk ^ ((row >> 1) & 7).
  const int pre = l32 * (BK * 2) + (((l32 >> 1) & 7) << 4);
  // the wave's two feature blocks are half a head apart: rotary pairs meet in one lane
  // The L tile holds at most 64 features (blocks 0 and 1): there every wave takes both and
  // one token block, half the matrix work of a K or V tile.
  const bool lr_tile = kind == 2;
  const int fb0 = lr_tile ? 0 : (D == 128 ? wr : 2 * wr);
  const int fb1 = lr_tile ? 1 : (D == 128 ? wr + 2 : 2 * wr + 1);
  // (BT = 64: one token block per wave, wc or, in the L tile, wave % 2 with waves 2 and 3 repeating 0 and 1)
  const int tb0 = ONE_TB ? (lr_tile ? (wave & 1) : wc) : (lr_tile ? wave : 2 * wc);
  const int tb1 = 2 * wc + 1;  // unused by the L tile and with BT = 64
  const bool stores = !(ONE_TB && lr_tile && wave >= 2);

  pf_f32x16 acc[2][2];  // [feature block fb0 / fb1][token block tb0 / tb1]
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  // Step s computes on stage s % NS while the tiles of the next NS - 2 steps are in flight and
  // the one after them is requested: a wave waits until only the loads younger than step s
  // (8 per step and wave) are outstanding, the barrier makes every wave's share visible and
  // retires stage (s - 1) % NS, which the new requests then overwrite.
  // A wave issues in order and a wave-wide request holds it for as long as the memory pipe of
  // the compute unit (shared by the four waves) needs to take it.  With one workgroup per
  // compute unit the eight requests therefore go out two per k-slice between the MFMAs, next
  // to the LDS reads of the following slice (operand registers double-buffered; sched_barrier
  // keeps the compiler from regrouping them).
  auto k_step = [&](int step, auto st_c, auto lr_c) __attribute__((always_inline)) {
    constexpr int ST = decltype(st_c)::value;
    constexpr bool LR = decltype(lr_c)::value;
    constexpr int KS = BK / 16;
    if (step + NS - 2 < n_steps) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(REQ * (NS - 2)));
    else pf_wait_vm0();
    __syncthreads();
    const bool more = step + NS - 1 < n_steps;
    const int k_next = k_first + (step + NS - 1) * BK;
    const unsigned char* wt = smem + ST * STAGE;
    const unsigned char* xt = wt + TILE_BYTES;
    if (NS == 2) {
      // Two workgroups per compute unit: the other one's MFMAs cover this one's requests, and
      // what pays is reading far ahead.  All requests first, then the sixteen operand reads of
      // the step ordered against its sixteen MFMAs: two k-slices of reads, one read per MFMA.
      if (more) issue_step(k_next, (ST + NS - 1) % NS);
      pf_bf16x8 a0[KS], a1[KS], b0[KS], b1[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const int off = pre ^ ((2 * ks + g2) << 4);
        a0[ks] = pf_as_bf16x8(*reinterpret_cast<const uint4*>(wt + off + fb0 * 32 * (BK * 2)));
        b0[ks] = pf_as_bf16x8(*reinterpret_cast<const uint4*>(xt + off + tb0 * 32 * (BK * 2)));
        a1[ks] = pf_as_bf16x8(*reinterpret_cast<const uint4*>(wt + off + fb1 * 32 * (BK * 2)));
        if (!LR) b1[ks] = pf_as_bf16x8(*reinterpret_cast<const uint4*>(xt + off + tb1 * 32 * (BK * 2)));
      }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[ks], b0[ks], acc[0][0], 0, 0, 0);
        acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[ks], b0[ks], acc[1][0], 0, 0, 0);
        if (!LR) {
          acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[ks], b1[ks], acc[0][1], 0, 0, 0);
          acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[ks], b1[ks], acc[1][1], 0, 0, 0);
        }
      }
      constexpr int READS = LR ? 12 : 16, MFMAS = LR ? 8 : 16, AHEAD = READS / 2;
      __builtin_amdgcn_sched_group_barrier(0x100, AHEAD, 0);
#pragma unroll
      for (int i = 0; i < READS - AHEAD; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, MFMAS - (READS - AHEAD), 0);
      return;
    }
    // One workgroup per compute unit (the deeper rings): nothing else covers the requests.
    pf_bf16x8 a0[2], a1[2], b0[2], b1[2];
    auto read_slice = [&](int ks, int buf) __attribute__((always_inline)) {
      const int off = pre ^ ((2 * ks + g2) << 4);
      a0[buf] = pf_as_bf16x8(*reinterpret_cast<const uint4*>(wt + off + fb0 * 32 * (BK * 2)));
      b0[buf] = pf_as_bf16x8(*reinterpret_cast<const uint4*>(xt + off + tb0 * 32 * (BK * 2)));
      a1[buf] = pf_as_bf16x8(*reinterpret_cast<const uint4*>(wt + off + fb1 * 32 * (BK * 2)));
      if (!LR) b1[buf] = pf_as_bf16x8(*reinterpret_cast<const uint4*>(xt + off + tb1 * 32 * (BK * 2)));
    };
    read_slice(0, 0);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int cur = ks & 1;
      __builtin_amdgcn_sched_barrier(0);
      if (more) {
        issue_part(k_next, (ST + NS - 1) % NS, 2 * ks);
        issue_part(k_next, (ST + NS - 1) % NS, 2 * ks + 1);
      }
      if (ks + 1 < KS) read_slice(ks + 1, cur ^ 1);
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[cur], b0[cur], acc[0][0], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[cur], b0[cur], acc[1][0], 0, 0, 0);
      if (!LR) {
        acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[cur], b1[cur], acc[0][1], 0, 0, 0);
        acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[cur], b1[cur], acc[1][1], 0, 0, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  auto k_loop = [&](auto lr_c) __attribute__((always_inline)) {
    for (int step = 0; step < n_steps; step += NS) {
      k_step(step, std::integral_constant<int, 0>{}, lr_c);
      if (step + 1 < n_steps) k_step(step + 1, std::integral_constant<int, 1>{}, lr_c);
      if (NS > 2 && step + 2 < n_steps) k_step(step + 2, std::integral_constant<int, 2 % NS>{}, lr_c);
      if (NS > 3 && step + 3 < n_steps) k_step(step + 3, std::integral_constant<int, 3 % NS>{}, lr_c);
    }
  };
  if (lr_tile || ONE_TB) k_loop(std::true_type{});  // one token block per wave
  else k_loop(std::false_type{});

  // ---------------- epilogue: rotate the keys, cast, store into the cache rows ----------------
  // acc[a][b], register i, lane (l32, g2): feature 32*fb_a + 8(i/4) + 4g2 + i%4 of the tile,
  // token 32*tb_b + l32 of the tile.
  if constexpr (SPLITK) {
    // the sums of this part of d_model as they are, four consecutive features per 16-byte store
    const int n_feat = 2 * HD + p.rank;
    const int region = kind == 2 ? p.rank : HD;   // features of this tile's region
    float* part = p.split_ws + static_cast<int64_t>(blockIdx.z) * p.n_new * n_feat;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      if ((b == 1 && (lr_tile || ONE_TB)) || !stores) continue;
      const int tok = tok0 + 32 * (b == 0 ? tb0 : tb1) + l32;
      if (tok >= n_new) continue;
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int f = feat0 + 32 * (a == 0 ? fb0 : fb1) + 8 * q + 4 * g2;  // inside the region: all four or none
          if (f < region)
            *reinterpret_cast<float4*>(part + static_cast<int64_t>(tok) * n_feat + (w_row0 - feat0) + f) =
                make_float4(acc[a][b][4 * q + 0], acc[a][b][4 * q + 1], acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]);
        }
    }
    return;
  }
  bf16_t* kcache = static_cast<bf16_t*>(kind == 0 ? p.k_base : p.v_base);
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    if ((b == 1 && (lr_tile || ONE_TB)) || !stores) continue;
    const int tok = tok0 + 32 * (b == 0 ? tb0 : tb1) + l32;
    const int j = pos0 + tok;  // cache row of this token, and its position
    if (tok >= n_new || j < 0) continue;  // (a sequence length below n_new breaks the contract: nothing is written)
    int64_t row_off;           // element offset of (token j, kv head 0) in K_base / V_base, or of row j in L
    if (PAGED) {
      const int blk = p.block_table[static_cast<int64_t>(p.seq_index) * p.max_blocks_per_seq + (j >> 4)];
      row_off = kind == 2 ? (static_cast<int64_t>(blk) * 16 + (j & 15)) * p.l_row_stride
                          : static_cast<int64_t>(blk) * p.kv_block_stride + static_cast<int64_t>(j & 15) * p.kv_token_stride;
    } else {
      row_off = kind == 2 ? static_cast<int64_t>(j) * p.l_row_stride : static_cast<int64_t>(j) * p.kv_token_stride;
    }
    if (kind == 2) {
      bf16_t* lrow = static_cast<bf16_t*>(p.l) + row_off;
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int f = 32 * (a == 0 ? fb0 : fb1) + 8 * q + 4 * g2;  // the rank is a multiple of 8: all four or none
          if (f < p.rank)
            *reinterpret_cast<uint2*>(lrow + f) =
                make_uint2(pf_pack2(acc[a][b][4 * q + 0], acc[a][b][4 * q + 1]), pf_pack2(acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]));
        }
      continue;
    }
    if (kind == 0 && p.rope_theta > 0.f) {
      // pair (feature dd, dd + d/2) of a head: acc[0] holds the first half, acc[1] the second
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int dd = (32 * fb0 + 8 * (i >> 2) + 4 * g2 + (i & 3)) % D;  // < d/2 by construction
        float sn, cs;
        rope_sincos(rope_rate[dd], j, sn, cs);
        const float lo = acc[0][b][i], hi = acc[1][b][i];
        acc[0][b][i] = lo * cs - hi * sn;
        acc[1][b][i] = hi * cs + lo * sn;
      }
    }
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int f = feat0 + 32 * (a == 0 ? fb0 : fb1) + 8 * q + 4 * g2;  // feature inside the K (V) region
        if (f < HD) {
          const int head = f / D, dd = f - head * D;
          *reinterpret_cast<uint2*>(kcache + row_off + static_cast<int64_t>(head) * p.kv_head_stride + dd) =
              make_uint2(pf_pack2(acc[a][b][4 * q + 0], acc[a][b][4 * q + 1]), pf_pack2(acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]));
        }
      }
  }
  (void)HALF;
}

// ---------------------------------------------------------------------------------------
// 256 features x 256 tokens per workgroup (for chunks whose tiles fill whole rounds of the chip).  At
// 128 x 128 a step moves 32 KB into LDS for 2.1 MFLOP and every MFMA costs one 1 KB LDS read:
// with two workgroups per compute unit the LDS is busier than the matrix pipes.  Here a wave
// owns 128 x 128 of the output (sixteen 32 x 32 accumulators, kept in the accumulation
// registers), reads eight operands for sixteen MFMAs, and a step moves 64 KB for 8.4 MFLOP.
// Same LDS layout, DMA and epilogue as append_kernel; two stages of 64 KB, one workgroup per
// compute unit.  The wave's four feature blocks are one head (d = 128: pairs (0,2), (1,3)) or
// two (d = 64: pairs (0,1), (2,3)).  Measured: about 1.45 us per step against 0.9 us of MFMA
// work; ahead of append_kernel when its tiles fill whole rounds of the chip (16384 tokens:
// 277 us against 302 us), behind it otherwise (the grid of 256-wide tiles quantises worse).
// ---------------------------------------------------------------------------------------
template <int D, bool PAGED>
__global__ __launch_bounds__(256, 1) void append_wide_kernel(AppendParams p) {
  constexpr int BF = 256, BT = 256, BK = 64;
  constexpr int TILE_BYTES = BF * BK * 2;  // 256 rows of 128 bytes
  constexpr int STAGE = 2 * TILE_BYTES;    // [W tile][X tile]
  __shared__ __align__(16) unsigned char smem[2 * STAGE];
  __shared__ double rope_rate[D / 2];  // revolutions per position of every rotary pair

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, g2 = lane >> 5;
  const int wr = wave >> 1, wc = wave & 1;
  const int HD = p.n_kv_heads * D;
  const int n_ct_kv = (HD + BF - 1) / BF;
  // The L tiles (little matrix work) come first in the grid, so they run beside the first full
  // tiles instead of as a round of their own at the end.
  const int ct = static_cast<int>(blockIdx.y) - 1;
  const int kind = ct < 0 ? 2 : (ct < n_ct_kv ? 0 : 1);  // 0 K, 1 V, 2 L
  const int ct_in = kind == 0 ? ct : (kind == 1 ? ct - n_ct_kv : 0);
  const int feat0 = ct_in * BF;
  const int w_row0 = (kind == 0 ? 0 : (kind == 1 ? HD : 2 * HD)) + feat0;
  const int tok0 = blockIdx.x * BT;
  const int n_new = p.n_new;
  const int n_t = append_length(PF_CONST_I32(p.seq_lens)[p.seq_index], p.max_seq_len);
  const int pos0 = n_t - n_new;

  // tile traffic: as in append_kernel, 32 wave-wide loads per tile, wave w issues i = w + 4q
  const uint32_t ldw2 = static_cast<uint32_t>(p.d_model) * 2u;
  const uint32_t n_w_rows = static_cast<uint32_t>(2 * HD + p.rank);
  const pf_u32x4 rs_w = pf_rsrc(p.w, (n_w_rows - 1) * ldw2 + ldw2);
  const pf_u32x4 rs_x = pf_rsrc(p.x, static_cast<uint32_t>(n_new - 1) * ldw2 + ldw2);
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(PF_LDS_AS(unsigned char, smem)));
  const uint32_t voff = static_cast<uint32_t>(lane >> 3) * ldw2 +
                        (((lane & 7) ^ ((4 * wave + (lane >> 4)) & 7)) << 4);
  // request number part (0..15) of this wave for the step at k0: W loads first, then X
  auto issue_part = [&](int k0, int st, int part) __attribute__((always_inline)) {
    const int i = wave + 4 * (part & 7);
    const uint32_t dst = lds0 + st * STAGE + i * 1024;
    if (part < 8) pf_load16_to_lds(rs_w, dst, voff, static_cast<uint32_t>(w_row0 + 8 * i) * ldw2 + k0 * 2);
    else pf_load16_to_lds(rs_x, dst + TILE_BYTES, voff, static_cast<uint32_t>(tok0 + 8 * i) * ldw2 + k0 * 2);
  };
  auto issue_step = [&](int k0, int st) __attribute__((always_inline)) {
#pragma unroll
    for (int part = 0; part < 16; ++part) issue_part(k0, st, part);
  };
  const int n_steps = p.d_model / BK;
  issue_step(0, 0);
  if (tid < D / 2 && p.rope_theta > 0.f) rope_rate[tid] = rope_rate_rev(tid, D, p.rope_theta);  // read after the loop's barriers

  const int pre = l32 * (BK * 2) + (((l32 >> 1) & 7) << 4);
  const bool lr_tile = kind == 2;
  // K, V tiles: feature blocks 4 wr + i, token blocks 4 wc + j (i, j < 4).
  // L tile (at most 64 features): feature blocks 0, 1 and token blocks 2 wave + j (j < 2).
  const int fbase = lr_tile ? 0 : 4 * wr;
  const int tbase = lr_tile ? 2 * wave : 4 * wc;


  // One step.  A wave issues instructions in order, and a wave-wide request occupies the
  // memory pipe of the compute unit for some sixteen cycles (all four waves share it): sixteen
  // requests issued in a row keep the wave off the matrix pipe for as long as the pipe needs
  // to take them, and the two times add up.  So the requests for the next step go out two at a
  // time between the groups of four MFMAs of the first half of the step, next to the LDS reads of the next k-slice
  // (registers double-buffered); sched_barrier keeps the compiler from regrouping them.
  auto k_step = [&](auto& acc, int step, auto st_c, auto lr_c, auto more_c) __attribute__((always_inline)) {
    constexpr int ST = decltype(st_c)::value;
    constexpr bool LR = decltype(lr_c)::value;
    const bool MORE = more_c;                       // another step follows: request its tiles (uniform)
    constexpr int NA = LR ? 2 : 4, NB = LR ? 2 : 4;
    constexpr int KS = BK / 16;
    constexpr int GROUPS = KS * NA;          // groups of NB MFMAs in a step
    constexpr int PARTS = 2 * 16 / GROUPS;   // requests per group: all sixteen go out in the first half of the
                                             // step, so that the last one has the other half to land
    pf_wait_vm0();
    __syncthreads();
    const unsigned char* wt = smem + ST * STAGE + fbase * 32 * (BK * 2);
    const unsigned char* xt = smem + ST * STAGE + TILE_BYTES + tbase * 32 * (BK * 2);
    pf_bf16x8 a[2][NA], b[2][NB];
    {
      const int off = pre ^ (g2 << 4);
#pragma unroll
      for (int i = 0; i < NA; ++i) a[0][i] = pf_as_bf16x8(*reinterpret_cast<const uint4*>(wt + off + i * 32 * (BK * 2)));
#pragma unroll
      for (int j = 0; j < NB; ++j) b[0][j] = pf_as_bf16x8(*reinterpret_cast<const uint4*>(xt + off + j * 32 * (BK * 2)));
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int cur = ks & 1, nxt = cur ^ 1;
      const int off = pre ^ ((2 * (ks + 1) + g2) << 4);
#pragma unroll
      for (int i = 0; i < NA; ++i) {
        __builtin_amdgcn_sched_barrier(0);
        if (MORE && (ks * NA + i) * PARTS < 16) {
#pragma unroll
          for (int q = 0; q < PARTS; ++q) issue_part((step + 1) * BK, ST ^ 1, (ks * NA + i) * PARTS + q);
        }
        if (ks + 1 < KS) {
          // two operands of the next k-slice per group, in the order its groups need them: its
          // first group takes every b and a[0], so the b's go first (NA == NB)
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            const int o = 2 * i + q;  // 0 .. NA + NB - 1
            if (o < NB) b[nxt][o] = pf_as_bf16x8(*reinterpret_cast<const uint4*>(xt + off + o * 32 * (BK * 2)));
            else a[nxt][o - NB] = pf_as_bf16x8(*reinterpret_cast<const uint4*>(wt + off + (o - NB) * 32 * (BK * 2)));
          }
        }
#pragma unroll
        for (int j = 0; j < NB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cur][i], b[cur][j], acc[i][j], 0, 0, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  auto k_loop = [&](auto& acc, auto lr_c) __attribute__((always_inline)) {
    constexpr int N = decltype(lr_c)::value ? 2 : 4;
#pragma unroll
    for (int a = 0; a < N; ++a)
#pragma unroll
      for (int b = 0; b < N; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
    // (one loop body for every step: peeled first or last steps make the compiler move the sixteen accumulator
    // tuples between the copies of the body, through scratch memory)
    for (int step = 0; step < n_steps; step += 2) {
      k_step(acc, step, std::integral_constant<int, 0>{}, lr_c, step + 1 < n_steps);
      if (step + 1 < n_steps) k_step(acc, step + 1, std::integral_constant<int, 1>{}, lr_c, step + 2 < n_steps);
    }
    pf_wait_vm0();
  };

  // epilogue.  acc[a][b], register i, lane (l32, g2): feature 32 (fbase + a) + 8 (i/4) + 4 g2 + i%4
  // of the tile, token 32 (tbase + b) + l32 of the tile.
  bf16_t* kcache = static_cast<bf16_t*>(kind == 0 ? p.k_base : p.v_base);
  auto store_block = [&](auto& acc, auto lr_c, auto b_c) __attribute__((always_inline)) {
    constexpr int b = decltype(b_c)::value;
    constexpr bool LR = decltype(lr_c)::value;
    const int tok = tok0 + 32 * (tbase + b) + l32;
    const int j = pos0 + tok;
    if (tok >= n_new || j < 0) return;
    int64_t row_off;
    if (PAGED) {
      const int blk = p.block_table[static_cast<int64_t>(p.seq_index) * p.max_blocks_per_seq + (j >> 4)];
      row_off = kind == 2 ? (static_cast<int64_t>(blk) * 16 + (j & 15)) * p.l_row_stride
                          : static_cast<int64_t>(blk) * p.kv_block_stride + static_cast<int64_t>(j & 15) * p.kv_token_stride;
    } else {
      row_off = kind == 2 ? static_cast<int64_t>(j) * p.l_row_stride : static_cast<int64_t>(j) * p.kv_token_stride;
    }
    if constexpr (LR) {
      bf16_t* lrow = static_cast<bf16_t*>(p.l) + row_off;
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int f = 32 * a + 8 * q + 4 * g2;
          if (f < p.rank)
            *reinterpret_cast<uint2*>(lrow + f) =
                make_uint2(pf_pack2(acc[a][b][4 * q + 0], acc[a][b][4 * q + 1]), pf_pack2(acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]));
        }
    } else {
    if (kind == 0 && p.rope_theta > 0.f) {
      // rotates the pair of blocks (lo, hi); block_lo = position of lo among the wave's four
      auto rotate = [&](pf_f32x16& lo_v, pf_f32x16& hi_v, int block_lo) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int dd = (32 * block_lo + 8 * (i >> 2) + 4 * g2 + (i & 3)) % D;  // < d/2 by construction
          float sn, cs;
          rope_sincos(rope_rate[dd], j, sn, cs);
          const float lo = lo_v[i], hi = hi_v[i];
          lo_v[i] = lo * cs - hi * sn;
          hi_v[i] = hi * cs + lo * sn;
        }
      };
      if (D == 128) {
        rotate(acc[0][b], acc[2][b], 0);
        rotate(acc[1][b], acc[3][b], 1);
      } else {
        rotate(acc[0][b], acc[1][b], 0);
        rotate(acc[2][b], acc[3][b], 2);
      }
    }
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int f = feat0 + 32 * (fbase + a) + 8 * q + 4 * g2;
        if (f < HD) {
          const int head = f / D, dd = f - head * D;
          *reinterpret_cast<uint2*>(kcache + row_off + static_cast<int64_t>(head) * p.kv_head_stride + dd) =
              make_uint2(pf_pack2(acc[a][b][4 * q + 0], acc[a][b][4 * q + 1]), pf_pack2(acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]));
        }
      }
    }
  };
  // (the two kinds of tile keep accumulators of their own: sixteen 16-register tuples leave no room for a copy)
  if (lr_tile) {
    pf_f32x16 acc[2][2];  // [feature block][token block]
    k_loop(acc, std::true_type{});
    store_block(acc, std::true_type{}, std::integral_constant<int, 0>{});
    store_block(acc, std::true_type{}, std::integral_constant<int, 1>{});
  } else {
    pf_f32x16 acc[4][4];
    k_loop(acc, std::false_type{});
    store_block(acc, std::false_type{}, std::integral_constant<int, 0>{});
    store_block(acc, std::false_type{}, std::integral_constant<int, 1>{});
    store_block(acc, std::false_type{}, std::integral_constant<int, 2>{});
    store_block(acc, std::false_type{}, std::integral_constant<int, 3>{});
  }
}

// ---------------------------------------------------------------------------------------
// Few new tokens (a decode step appends one): the projection is one pass over the weights,
// bound by HBM, and a 128 x 128 tile grid would put a handful of workgroups on the chip.
// Here a workgroup owns 16 output features and 16 * NT tokens; its 8 waves split d_model
// (wave w takes the 64-wide steps w, w+8, ...), feed v_mfma_f32_16x16x32_bf16 straight from
// global loads (every weight element is used once: nothing to stage) and add their partial
// tiles through LDS.  The 16 features are 8 + the 8 half a head further on, so the rotary
// pairs meet in one thread of the epilogue.  blockIdx.y walks chunks of 16 * NT tokens.
// ---------------------------------------------------------------------------------------
template <int D, int NT, bool PAGED>
__global__ __launch_bounds__(512) void append_skinny_kernel(AppendParams p) {
  constexpr int NW = 8;
  __shared__ __align__(16) float red[NW][NT][256];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, g4 = lane >> 4;
  const int HD = p.n_kv_heads * D;
  const int groups_kv = HD / 16;  // feature groups of the K (and of the V) region
  const int fg = blockIdx.x;
  const int kind = fg < groups_kv ? 0 : (fg < 2 * groups_kv ? 1 : 2);
  const int fg_in = kind == 0 ? fg : (kind == 1 ? fg - groups_kv : fg - 2 * groups_kv);
  const int head = fg_in / (D / 16), sub = fg_in - head * (D / 16);
  // feature (inside its region) of tile row i: K/V  head*D + 8 sub + i  (i < 8),  + d/2 - 8 beyond;  L  16 fg_in + i
  auto feature_of = [&](int i) __attribute__((always_inline)) {
    return kind == 2 ? 16 * fg_in + i : head * D + 8 * sub + (i < 8 ? i : i - 8 + D / 2);
  };
  const int n_new = p.n_new;
  const int tok0 = blockIdx.y * (16 * NT);
  const int n_t = append_length(PF_CONST_I32(p.seq_lens)[p.seq_index], p.max_seq_len);
  const int pos0 = n_t - n_new;

  // operand rows of this lane (clamped into the tensors; what a clamped row produces is never stored)
  const int w_row = (kind == 0 ? 0 : (kind == 1 ? HD : 2 * HD)) +
                    (kind == 2 ? min(feature_of(l16), p.rank - 1) : feature_of(l16));
  const int64_t ld = p.d_model;
  const bf16_t* wp = static_cast<const bf16_t*>(p.w) + static_cast<int64_t>(w_row) * ld + 8 * g4;
  const bf16_t* xp[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
    xp[t] = static_cast<const bf16_t*>(p.x) + static_cast<int64_t>(min(tok0 + 16 * t + l16, n_new - 1)) * ld + 8 * g4;

  pf_f32x4 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) acc[t] = pf_f32x4{0.f, 0.f, 0.f, 0.f};

  // A step covers 64 values of d_model with two MFMAs: lane (l16, g4) holds k = 64 s + 16 g4 .. + 16
  // of its W row (A) and of its token (B), the first eight for one MFMA, the rest for the other
  // (any assignment of k to lanes is right as long as A and B share it); four lanes read one
  // 128-byte line of a row.
  const int n_steps = p.d_model / 64;
  constexpr int U = 8 / NT;  // steps in flight per wave (64 operand registers of x)
  const bf16_t* wq = wp + 8 * g4;  // wp and xp already carry 8 g4
  int s = wave;
  for (; s + (U - 1) * NW < n_steps; s += U * NW) {
    pf_u32x4 a[U][2], b[U][NT][2];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      a[u][0] = *reinterpret_cast<const pf_u32x4*>(wq + (s + u * NW) * 64);
      a[u][1] = *reinterpret_cast<const pf_u32x4*>(wq + (s + u * NW) * 64 + 8);
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        b[u][t][0] = *reinterpret_cast<const pf_u32x4*>(xp[t] + 8 * g4 + (s + u * NW) * 64);
        b[u][t][1] = *reinterpret_cast<const pf_u32x4*>(xp[t] + 8 * g4 + (s + u * NW) * 64 + 8);
      }
    }
    // every request of the batch is out before the first result is used (left alone the
    // compiler recycles a few registers and the loads trickle out a handful at a time)
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(pf_bf16x8, a[u][0]), __builtin_bit_cast(pf_bf16x8, b[u][t][0]), acc[t], 0, 0, 0);
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(pf_bf16x8, a[u][1]), __builtin_bit_cast(pf_bf16x8, b[u][t][1]), acc[t], 0, 0, 0);
      }
  }
  for (; s < n_steps; s += NW) {
    const uint4 a0 = *reinterpret_cast<const uint4*>(wq + s * 64);
    const uint4 a1 = *reinterpret_cast<const uint4*>(wq + s * 64 + 8);
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const uint4 b0 = *reinterpret_cast<const uint4*>(xp[t] + 8 * g4 + s * 64);
      const uint4 b1 = *reinterpret_cast<const uint4*>(xp[t] + 8 * g4 + s * 64 + 8);
      acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf_as_bf16x8(a0), pf_as_bf16x8(b0), acc[t], 0, 0, 0);
      acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf_as_bf16x8(a1), pf_as_bf16x8(b1), acc[t], 0, 0, 0);
    }
  }
  // acc[t], register e, lane (l16, g4): tile row (feature) 4 g4 + e, token 16 t + l16
#pragma unroll
  for (int t = 0; t < NT; ++t) *reinterpret_cast<pf_f32x4*>(&red[wave][t][lane * 4]) = acc[t];
  __syncthreads();

  // thread (t, i < 8, token): sums the 8 partial tiles for rows i and i + 8, rotates, stores
  if (tid >= NT * 128) return;
  const int t = tid >> 7, i = (tid >> 4) & 7, tk = tid & 15;
  const int tok = tok0 + 16 * t + tk;
  if (tok >= n_new || pos0 + tok < 0) return;
  const int at_lo = (tk + 16 * (i >> 2)) * 4 + (i & 3);  // row i      -> lane tk + 16 (i/4), register i%4
  const int at_hi = at_lo + 128;                         // row i + 8  -> two lane groups further
  float lo = 0.f, hi = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    lo += red[w][t][at_lo];
    hi += red[w][t][at_hi];
  }
  const int j = pos0 + tok;
  if (kind == 2) {
    int64_t row_off;
    if (PAGED) {
      const int blk = p.block_table[static_cast<int64_t>(p.seq_index) * p.max_blocks_per_seq + (j >> 4)];
      row_off = (static_cast<int64_t>(blk) * 16 + (j & 15)) * p.l_row_stride;
    } else {
      row_off = static_cast<int64_t>(j) * p.l_row_stride;
    }
    bf16_t* lrow = static_cast<bf16_t*>(p.l) + row_off;
    const int f = 16 * fg_in + i;
    if (f < p.rank) lrow[f] = f32_to_bf16(lo);
    if (f + 8 < p.rank) lrow[f + 8] = f32_to_bf16(hi);
    return;
  }
  const int dd = 8 * sub + i;  // < d/2
  if (kind == 0 && p.rope_theta > 0.f) {
    float sn, cs;
    rope_sincos(rope_rate_rev(dd, D, p.rope_theta), j, sn, cs);
    const float a = lo, b = hi;
    lo = a * cs - b * sn;
    hi = b * cs + a * sn;
  }
  int64_t row_off;
  if (PAGED) {
    const int blk = p.block_table[static_cast<int64_t>(p.seq_index) * p.max_blocks_per_seq + (j >> 4)];
    row_off = static_cast<int64_t>(blk) * p.kv_block_stride + static_cast<int64_t>(j & 15) * p.kv_token_stride;
  } else {
    row_off = static_cast<int64_t>(j) * p.kv_token_stride;
  }
  bf16_t* dst = static_cast<bf16_t*>(kind == 0 ? p.k_base : p.v_base) + row_off + static_cast<int64_t>(head) * p.kv_head_stride + dd;
  dst[0] = f32_to_bf16(lo);
  dst[D / 2] = f32_to_bf16(hi);
}

// ---------------------------------------------------------------------------------------
// One to four new tokens (every decode step appends one): a matrix-vector product.  One wave
// per weight row reads it in fully coalesced 1 KB pieces, all in flight at once, and forms
// the dot products with v_dot2c_f32_bf16; the 2 * Hkv * d + r rows make several hundred
// workgroups, enough outstanding loads to run at HBM speed.  A workgroup's four rows are two
// rotary pairs (features f, f+1 and f + d/2, f+1 + d/2).
// ---------------------------------------------------------------------------------------
typedef __bf16 ap_bf16x2 __attribute__((ext_vector_type(2)));

template <int D, int NT, bool PAGED>
__global__ __launch_bounds__(256) void append_gemv_kernel(AppendParams p) {
  __shared__ float red[4][NT];
  // A call of this kernel is one round of requests and a handful of dependent latencies; each is
  // kept off the others' path: the parameter block comes in one round trip, the sequence length
  // (needed only by the last step) is requested first and by hand, the weight requests (the bytes
  // that take long) leave before the activations and unconditionally (pieces beyond the row are
  // fetched from its last piece and multiplied by zero: a load under a condition makes the
  // compiler wait for earlier loads on the spot), and the rotation rate of the pair (double
  // precision exp2 and log2) is worked out while the requests are in flight.
  asm volatile("" ::"s"(p.w), "s"(p.x), "s"(p.seq_lens), "s"(p.k_base), "s"(p.v_base), "s"(p.l));
  asm volatile("" ::"s"(p.d_model), "s"(p.n_kv_heads), "s"(p.rank), "s"(p.n_new), "s"(p.seq_index), "s"(p.max_seq_len),
               "s"(p.rope_theta), "s"(p.kv_token_stride), "s"(p.kv_head_stride), "s"(p.l_row_stride));
  int len_raw;
  asm volatile("s_load_dword %0, %1, 0x0" : "=s"(len_raw) : "s"(p.seq_lens + p.seq_index));
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int HD = p.n_kv_heads * D;
  const int groups_kv = HD / 4;
  const int fg = blockIdx.x;
  const int kind = fg < groups_kv ? 0 : (fg < 2 * groups_kv ? 1 : 2);
  const int fg_in = kind == 0 ? fg : (kind == 1 ? fg - groups_kv : fg - 2 * groups_kv);
  const int head = fg_in / (D / 4), sub = fg_in - head * (D / 4);  // K, V: pairs 2 sub, 2 sub + 1 of this head
  const int pr = wave & 1, half = wave >> 1;
  // row of this wave: K/V  head*D + 2 sub + pr (+ d/2 for the second half);  L  4 fg_in + pr + 2 half
  const int feat = kind == 2 ? 4 * fg_in + pr + 2 * half : head * D + 2 * sub + pr + half * (D / 2);
  const int w_row = kind == 2 ? 2 * HD + min(feat, p.rank - 1) : (kind == 1 ? HD : 0) + feat;
  const int n_new = p.n_new;
  const int64_t ld = p.d_model;
  const uint4* wp = reinterpret_cast<const uint4*>(static_cast<const bf16_t*>(p.w) + static_cast<int64_t>(w_row) * ld);
  const uint4* xp[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
    xp[t] = reinterpret_cast<const uint4*>(static_cast<const bf16_t*>(p.x) + static_cast<int64_t>(min(t, n_new - 1)) * ld);

  float acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) acc[t] = 0.f;
  const int n_chunks = p.d_model / 8;  // 16-byte pieces of a row; lane l takes l, l + 64, ...
  constexpr int U = 8;
  double rate = 0.0;  // revolutions per position of this thread's rotary pair (threads of the last step)
  for (int c0 = lane; c0 < n_chunks; c0 += 64 * U) {
    uint4 wv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      // (non-temporal: a weight row is read once per call, by this wave)
      const pf_u32x4 t4 = __builtin_nontemporal_load(reinterpret_cast<const pf_u32x4*>(wp + min(c0 + 64 * u, n_chunks - 1)));
      wv[u] = make_uint4(t4[0], t4[1], t4[2], t4[3]);
    }
    // all weight requests out before anything else.  (The operands stay HIP's uint4 structs on purpose:
    // with native 4-vectors this compiler selected element 0 for all four dot products.)
    __builtin_amdgcn_sched_barrier(0);
    uint4 xv[NT][U];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int u = 0; u < U; ++u) xv[t][u] = xp[t][min(c0 + 64 * u, n_chunks - 1)];
    __builtin_amdgcn_sched_barrier(0);
    if (c0 == lane && tid < 2 * NT && kind == 0 && p.rope_theta > 0.f) {
      rate = rope_rate_rev(2 * sub + (tid & 1), D, p.rope_theta);
      asm volatile("" ::"v"(rate));  // (here, under the requests, not after the reduction)
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        uint4 x4 = xv[t][u];
        if (c0 + 64 * u >= n_chunks) x4 = make_uint4(0u, 0u, 0u, 0u);  // (a piece beyond the row)
        acc[t] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(ap_bf16x2, wv[u].x), __builtin_bit_cast(ap_bf16x2, x4.x), acc[t], false);
        acc[t] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(ap_bf16x2, wv[u].y), __builtin_bit_cast(ap_bf16x2, x4.y), acc[t], false);
        acc[t] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(ap_bf16x2, wv[u].z), __builtin_bit_cast(ap_bf16x2, x4.z), acc[t], false);
        acc[t] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(ap_bf16x2, wv[u].w), __builtin_bit_cast(ap_bf16x2, x4.w), acc[t], false);
      }
    }
  }
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    float v = acc[t];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    if (lane == 0) red[wave][t] = v;
  }
  __syncthreads();

  // thread (pair, token): both halves of a rotary pair (K), two independent features (V, L)
  if (tid >= 2 * NT) return;
  const int q = tid & 1, t = tid >> 1;
  asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(len_raw));
  const int n_t = append_length(len_raw, p.max_seq_len);
  const int j = n_t - n_new + t;
  if (t >= n_new || j < 0) return;
  float lo = red[q][t], hi = red[2 + q][t];
  if (kind == 2) {
    int64_t row_off;
    if (PAGED) {
      const int blk = p.block_table[static_cast<int64_t>(p.seq_index) * p.max_blocks_per_seq + (j >> 4)];
      row_off = (static_cast<int64_t>(blk) * 16 + (j & 15)) * p.l_row_stride;
    } else {
      row_off = static_cast<int64_t>(j) * p.l_row_stride;
    }
    bf16_t* lrow = static_cast<bf16_t*>(p.l) + row_off;
    const int f = 4 * fg_in + q;
    if (f < p.rank) lrow[f] = f32_to_bf16(lo);
    if (f + 2 < p.rank) lrow[f + 2] = f32_to_bf16(hi);
    return;
  }
  const int dd = 2 * sub + q;  // < d/2
  if (kind == 0 && p.rope_theta > 0.f) {
    float sn, cs;
    rope_sincos(rate, j, sn, cs);
    const float a = lo, b = hi;
    lo = a * cs - b * sn;
    hi = b * cs + a * sn;
  }
  int64_t row_off;
  if (PAGED) {
    const int blk = p.block_table[static_cast<int64_t>(p.seq_index) * p.max_blocks_per_seq + (j >> 4)];
    row_off = static_cast<int64_t>(blk) * p.kv_block_stride + static_cast<int64_t>(j & 15) * p.kv_token_stride;
  } else {
    row_off = static_cast<int64_t>(j) * p.kv_token_stride;
  }
  bf16_t* dst = static_cast<bf16_t*>(kind == 0 ? p.k_base : p.v_base) + row_off + static_cast<int64_t>(head) * p.kv_head_stride + dd;
  dst[0] = f32_to_bf16(lo);
  dst[D / 2] = f32_to_bf16(hi);
}

// Second half of the split over d_model: adds the parts append_kernel<..., SPLITK> left in the
// workspace, rotates the keys, casts and writes the cache rows.  Grid (new token, chunk of 256
// items); a thread takes one item, four consecutive features: of V or L as they are, of K together with their
// rotary partners half a head further on.
template <int D, bool PAGED, int MAXP>  // MAXP: 2, 4, 8 or 16, at least the number of parts
__global__ __launch_bounds__(256) void append_finish_kernel(AppendParams p) {
  // A chain of latencies like the other small kernels here: the parameter block in one round trip,
  // the sequence length requested first and by hand, the loads of ALL parts issued at once (from
  // clamped part indices: a part beyond the count is fetched again and not added), and the rotation
  // rates of the pairs worked out while they are in flight.
  asm volatile("" ::"s"(p.split_ws), "s"(p.seq_lens), "s"(p.k_base), "s"(p.v_base), "s"(p.l), "s"(p.block_table));
  asm volatile("" ::"s"(p.n_kv_heads), "s"(p.rank), "s"(p.n_new), "s"(p.seq_index), "s"(p.max_seq_len), "s"(p.k_splits),
               "s"(p.rope_theta), "s"(p.kv_token_stride), "s"(p.kv_head_stride), "s"(p.l_row_stride));
  int len_raw;
  asm volatile("s_load_dword %0, %1, 0x0" : "=s"(len_raw) : "s"(p.seq_lens + p.seq_index));
  const int tid = threadIdx.x;
  const int tok = blockIdx.x;
  const int HD = p.n_kv_heads * D;
  const int n_feat = 2 * HD + p.rank;
  const int k_items = HD / 8, v_items = HD / 4, l_items = p.rank / 4;
  const int it_raw = blockIdx.y * 256 + tid;
  const bool has_item = it_raw < k_items + v_items + l_items;
  const int it = has_item ? it_raw : 0;  // (threads beyond the items repeat item 0 and store nothing)
  const int ks = p.k_splits;
  const float* row = p.split_ws + static_cast<int64_t>(tok) * n_feat;
  const int64_t part_stride = static_cast<int64_t>(p.n_new) * n_feat;
  // first feature of the item's four, and of their rotary partners (key items only)
  const bool is_k = it < k_items, is_v = !is_k && it < k_items + v_items;
  const int head = is_k ? it / (D / 8) : 0, dd = is_k ? (it - head * (D / 8)) * 4 : 0;
  const int f0 = is_k ? head * D + dd : (is_v ? HD + (it - k_items) * 4 : 2 * HD + (it - k_items - v_items) * 4);
  const int f1 = is_k ? f0 + D / 2 : f0;
  float4 x0[MAXP], x1[MAXP];
#pragma unroll
  for (int z = 0; z < MAXP; ++z) {
    const int64_t off = min(z, ks - 1) * part_stride;
    x0[z] = *reinterpret_cast<const float4*>(row + off + f0);
    x1[z] = *reinterpret_cast<const float4*>(row + off + f1);
  }
  __builtin_amdgcn_sched_barrier(0);
  // rotation rates of the pairs, for the workgroups that hold key items (under the loads)
  __shared__ double rope_rate[D / 2];
  if (static_cast<int>(blockIdx.y) * 256 < k_items && p.rope_theta > 0.f) {
    if (tid < D / 2) rope_rate[tid] = rope_rate_rev(tid, D, p.rope_theta);
    __syncthreads();
  }
  if (!has_item) return;
  asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(len_raw));
  const int n_t = append_length(len_raw, p.max_seq_len);
  const int j = n_t - p.n_new + tok;  // cache row of this token, and its position
  if (j < 0) return;
  int64_t kv_off, l_off;  // element offsets of (token j, kv head 0) in K_base / V_base and of row j in L
  if (PAGED) {
    const int blk = p.block_table[static_cast<int64_t>(p.seq_index) * p.max_blocks_per_seq + (j >> 4)];
    kv_off = static_cast<int64_t>(blk) * p.kv_block_stride + static_cast<int64_t>(j & 15) * p.kv_token_stride;
    l_off = (static_cast<int64_t>(blk) * 16 + (j & 15)) * p.l_row_stride;
  } else {
    kv_off = static_cast<int64_t>(j) * p.kv_token_stride;
    l_off = static_cast<int64_t>(j) * p.l_row_stride;
  }
  // the parts in order: the same sum every run
  float4 lo = make_float4(0.f, 0.f, 0.f, 0.f), hi = lo;
#pragma unroll
  for (int z = 0; z < MAXP; ++z)
    if (z < ks) {
      lo.x += x0[z].x; lo.y += x0[z].y; lo.z += x0[z].z; lo.w += x0[z].w;
      hi.x += x1[z].x; hi.y += x1[z].y; hi.z += x1[z].z; hi.w += x1[z].w;
    }
  auto store4 = [&](bf16_t* dst, float4 v) {
    *reinterpret_cast<uint2*>(dst) = make_uint2(pf_pack2(v.x, v.y), pf_pack2(v.z, v.w));
  };
  if (is_k) {
    if (p.rope_theta > 0.f) {
      float l4[4] = {lo.x, lo.y, lo.z, lo.w}, h4[4] = {hi.x, hi.y, hi.z, hi.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float sn, cs;
        rope_sincos(rope_rate[dd + e], j, sn, cs);
        const float a = l4[e], b = h4[e];
        l4[e] = a * cs - b * sn;
        h4[e] = b * cs + a * sn;
      }
      lo = make_float4(l4[0], l4[1], l4[2], l4[3]);
      hi = make_float4(h4[0], h4[1], h4[2], h4[3]);
    }
    bf16_t* dst = static_cast<bf16_t*>(p.k_base) + kv_off + static_cast<int64_t>(head) * p.kv_head_stride + dd;
    store4(dst, lo);
    store4(dst + D / 2, hi);
  } else if (is_v) {
    const int f = f0 - HD, vh = f / D, vd = f - vh * D;
    store4(static_cast<bf16_t*>(p.v_base) + kv_off + static_cast<int64_t>(vh) * p.kv_head_stride + vd, lo);
  } else {
    store4(static_cast<bf16_t*>(p.l) + l_off + (f0 - 2 * HD), lo);
  }
}

template <int D, int NT>
static void launch_gemv(const AppendParams& p, hipStream_t s) {
  const int hd = p.n_kv_heads * p.head_dim;
  dim3 grid(2 * (hd / 4) + (p.rank + 3) / 4);
  if (p.block_size != 0) hipLaunchKernelGGL((append_gemv_kernel<D, NT, true>), grid, dim3(256), 0, s, p);
  else hipLaunchKernelGGL((append_gemv_kernel<D, NT, false>), grid, dim3(256), 0, s, p);
}

template <int D, int NT>
static void launch_skinny(const AppendParams& p, hipStream_t s) {
  const int hd = p.n_kv_heads * p.head_dim;
  dim3 grid(2 * (hd / 16) + (p.rank + 15) / 16, (p.n_new + 16 * NT - 1) / (16 * NT));
  if (p.block_size != 0) hipLaunchKernelGGL((append_skinny_kernel<D, NT, true>), grid, dim3(512), 0, s, p);
  else hipLaunchKernelGGL((append_skinny_kernel<D, NT, false>), grid, dim3(512), 0, s, p);
}

hipError_t launch_append(const AppendParams& p, hipStream_t s) {
  const int hd = p.n_kv_heads * p.head_dim;
  const bool paged = p.block_size != 0;
  if (p.k_splits > 1) {
    // Split over d_model (chosen by the host from the sizes, with a workspace): tiles of 128 features
    // x 64 or 128 tokens, four LDS stages, p.k_splits parts in z, then the finishing kernel.
    const int bt = p.split_bt;
    dim3 grid((p.n_new + bt - 1) / bt, 2 * ((hd + 127) / 128) + 1, p.k_splits);
#define LRA_APPEND_SPLIT(DD, PG)                                                                                        \
  do {                                                                                                                  \
    if (bt == 64) hipLaunchKernelGGL((append_kernel<DD, PG, 4, 64, true>), grid, dim3(256), 0, s, p);                   \
    else hipLaunchKernelGGL((append_kernel<DD, PG, 4, 128, true>), grid, dim3(256), 0, s, p);                           \
    if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;                                                   \
    const dim3 fgrid(p.n_new, (hd / 8 + hd / 4 + p.rank / 4 + 255) / 256);                                              \
    if (p.k_splits <= 2) hipLaunchKernelGGL((append_finish_kernel<DD, PG, 2>), fgrid, dim3(256), 0, s, p);              \
    else if (p.k_splits <= 4) hipLaunchKernelGGL((append_finish_kernel<DD, PG, 4>), fgrid, dim3(256), 0, s, p);         \
    else if (p.k_splits <= 8) hipLaunchKernelGGL((append_finish_kernel<DD, PG, 8>), fgrid, dim3(256), 0, s, p);         \
    else hipLaunchKernelGGL((append_finish_kernel<DD, PG, 16>), fgrid, dim3(256), 0, s, p);                             \
  } while (0)
    if (p.head_dim == 128) {
      if (paged) LRA_APPEND_SPLIT(128, true);
      else LRA_APPEND_SPLIT(128, false);
    } else {
      if (paged) LRA_APPEND_SPLIT(64, true);
      else LRA_APPEND_SPLIT(64, false);
    }
#undef LRA_APPEND_SPLIT
    return hipGetLastError();
  }
  if (p.n_new <= 2 && p.n_new <= p.skinny_max) {
    if (p.head_dim == 128) {
      if (p.n_new == 1) launch_gemv<128, 1>(p, s);
      else launch_gemv<128, 2>(p, s);
    } else {
      if (p.n_new == 1) launch_gemv<64, 1>(p, s);
      else launch_gemv<64, 2>(p, s);
    }
    return hipGetLastError();
  }
  if (p.n_new <= p.skinny_max) {
    const int nt = p.n_new <= 16 ? 1 : (p.n_new <= 32 ? 2 : 4);
    if (p.head_dim == 128) {
      if (nt == 1) launch_skinny<128, 1>(p, s);
      else if (nt == 2) launch_skinny<128, 2>(p, s);
      else launch_skinny<128, 4>(p, s);
    } else {
      if (nt == 1) launch_skinny<64, 1>(p, s);
      else if (nt == 2) launch_skinny<64, 2>(p, s);
      else launch_skinny<64, 4>(p, s);
    }
    return hipGetLastError();
  }
  // 256 x 256 tiles, one workgroup per CU: on request, or when their full tiles fill whole rounds of
  // the chip's 256 CUs (at most a tenth of the last round idle) and there are at least two rounds.
  // Measured on the Llama-3-8B projection: 277 us against 302 us at 16384 new tokens (512 tiles, two
  // rounds), but 165 against 158 at 8192 and worse wherever a round stays half empty.
  const int wide_full = ((p.n_new + 255) / 256) * 2 * (hd / 256);
  const int wide_rounds = (wide_full + 255) / 256;
  const bool wide_fits = wide_full >= 448 && wide_rounds * 256 * 10 <= wide_full * 11;
  if (p.tile == 256 || (p.tile == 0 && p.stages == 0 && wide_fits)) {
    dim3 wgrid((p.n_new + 255) / 256, 2 * ((hd + 255) / 256) + 1);
    if (p.head_dim == 128) {
      if (paged) hipLaunchKernelGGL((append_wide_kernel<128, true>), wgrid, dim3(256), 0, s, p);
      else hipLaunchKernelGGL((append_wide_kernel<128, false>), wgrid, dim3(256), 0, s, p);
    } else {
      if (paged) hipLaunchKernelGGL((append_wide_kernel<64, true>), wgrid, dim3(256), 0, s, p);
      else hipLaunchKernelGGL((append_wide_kernel<64, false>), wgrid, dim3(256), 0, s, p);
    }
    return hipGetLastError();
  }
  dim3 grid((p.n_new + 127) / 128, 2 * ((hd + 127) / 128) + 1);
  // One workgroup per compute unit or fewer: nothing shares the LDS, so a deeper ring of
  // stages (more requests in flight per workgroup) is free; beyond that two workgroups per
  // unit with two stages each hide each other's waits.
  const int stages = p.stages != 0 ? p.stages : (static_cast<int>(grid.x * grid.y) <= 256 ? 4 : 2);
  // half-size token tiles while even those leave CUs idle, or when asked for (Llama-3-8B projection:
  // 22-24 us against 33-34 us up to 512 new tokens, level at 1024)
  if (p.tile == 64 || (p.tile == 0 && p.stages == 0 && static_cast<int>(grid.x * grid.y) <= 100)) {
    dim3 g64((p.n_new + 63) / 64, grid.y);
    if (p.head_dim == 128) {
      if (paged) hipLaunchKernelGGL((append_kernel<128, true, 4, 64>), g64, dim3(256), 0, s, p);
      else hipLaunchKernelGGL((append_kernel<128, false, 4, 64>), g64, dim3(256), 0, s, p);
    } else {
      if (paged) hipLaunchKernelGGL((append_kernel<64, true, 4, 64>), g64, dim3(256), 0, s, p);
      else hipLaunchKernelGGL((append_kernel<64, false, 4, 64>), g64, dim3(256), 0, s, p);
    }
    return hipGetLastError();
  }
#define LRA_APPEND_LAUNCH(DD, PG, NS_) hipLaunchKernelGGL((append_kernel<DD, PG, NS_>), grid, dim3(256), 0, s, p)
#define LRA_APPEND_STAGES(DD, PG)            \
  do {                                       \
    if (stages == 2) LRA_APPEND_LAUNCH(DD, PG, 2);      \
    else if (stages == 3) LRA_APPEND_LAUNCH(DD, PG, 3); \
    else LRA_APPEND_LAUNCH(DD, PG, 4);                  \
  } while (0)
  if (p.head_dim == 128) {
    if (paged) LRA_APPEND_STAGES(128, true);
    else LRA_APPEND_STAGES(128, false);
  } else {
    if (paged) LRA_APPEND_STAGES(64, true);
    else LRA_APPEND_STAGES(64, false);
  }
#undef LRA_APPEND_STAGES
#undef LRA_APPEND_LAUNCH
  return hipGetLastError();
}

}  // namespace lra
