// Cache-append producer of the Flash-LoRA-Attention library (bf16, gfx950): the step before
// the attention path.  For the new tokens of one sequence it forms
//     [K' | V | L] = X . [W_K | W_V | A]          (LRAgent Sec. 3.2: base cache from the
//                                                  pretrained projections, LR cache from the
//                                                  shared LoRA down-projection)
// rotates the keys by the model's rotary position embedding (the cached keys are the rotated
// ones, App. D.1) and writes the rows into K_base, V_base and L, contiguous or paged.
//
// One MFMA GEMM with the weights stored one output feature per row (the usual layout of a
// linear layer), computed transposed, Y^T[feature][token] = W[feature][:] . X[token][:], so
// that both operands are rows of 16-byte chunks along d_model (ds_read_b128, no transposed
// reads) and every lane ends up with four consecutive features of one token: an 8-byte
// store into a cache row.  A workgroup owns 128 features x 128 tokens and walks d_model in
// steps of 64; the W and X tiles go from HBM straight into a double-buffered LDS stage
// (buffer_load ... lds, swizzled by choosing which chunk a lane fetches).  The four waves
// form a 2 x 2 grid; a wave's two 32-feature blocks are chosen d/2 apart, so the two halves
// of every rotary pair sit in the same lane and register of its two accumulators and the
// rotation needs no data movement.  Angles are formed in double precision and reduced
// before the single-precision sine and cosine, so positions in the tens of thousands lose
// nothing.
#include "lra_prefill_util.h"

namespace lra {

template <int D, bool PAGED>
__global__ __launch_bounds__(256, 2) void append_kernel(AppendParams p) {
  constexpr int BF = 128, BT = 128, BK = 64;  // features, tokens, d_model step
  constexpr int TILE_BYTES = BF * BK * 2;      // one operand tile: 128 rows of 128 bytes
  constexpr int STAGE = 2 * TILE_BYTES;        // [W tile][X tile]
  constexpr int HALF = D / 2;

  __shared__ __align__(16) unsigned char smem[2 * STAGE];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, g2 = lane >> 5;
  const int wr = wave >> 1, wc = wave & 1;  // position in the 2 x 2 grid of waves: features, tokens
  const int HD = p.n_kv_heads * D;
  const int n_ct_kv = (HD + BF - 1) / BF;   // feature tiles of the K (and of the V) region
  const int ct = blockIdx.y;
  const int kind = ct < n_ct_kv ? 0 : (ct < 2 * n_ct_kv ? 1 : 2);  // 0 K, 1 V, 2 L
  const int ct_in = kind == 0 ? ct : (kind == 1 ? ct - n_ct_kv : 0);
  const int feat0 = ct_in * BF;                                 // first feature of the tile inside its region
  const int w_row0 = (kind == 0 ? 0 : (kind == 1 ? HD : 2 * HD)) + feat0;  // its row of w
  const int tok0 = blockIdx.x * BT;
  const int n_new = p.n_new;
  const int n_t = min(PF_CONST_I32(p.seq_lens)[p.seq_index], p.max_seq_len);
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
  auto issue_step = [&](int k0, int st) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int i = wave + 4 * q;
      const uint32_t dst = lds0 + st * STAGE + i * 1024;
      pf_load16_to_lds(rs_w, dst, voff, static_cast<uint32_t>(w_row0 + 8 * i) * ldw2 + k0 * 2);
      pf_load16_to_lds(rs_x, dst + TILE_BYTES, voff, static_cast<uint32_t>(tok0 + 8 * i) * ldw2 + k0 * 2);
    }
  };
  issue_step(0, 0);

  // ---------------- operands ----------------
  // A operand: W rows (features), B operand: X rows (tokens); lane (row l32 of a 32-row block,
  // k = 16ks + 8g2 + e): the 16-byte chunk 2ks + g2 of its row, at chunk ^ ((row >> 1) & 7).
  const int pre = l32 * (BK * 2) + (((l32 >> 1) & 7) << 4);
  // the wave's two feature blocks are half a head apart: rotary pairs meet in one lane
  const int fb0 = D == 128 ? wr : 2 * wr;
  const int fb1 = D == 128 ? wr + 2 : 2 * wr + 1;

  pf_f32x16 acc[2][2];  // [feature block 0/1][token block 2wc / 2wc+1]
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  pf_wait_vm0();
  __syncthreads();
  const int n_steps = p.d_model / BK;
  auto k_step = [&](int step, auto st_c) {
    constexpr int ST = decltype(st_c)::value;
    if (step + 1 < n_steps) issue_step((step + 1) * BK, ST ^ 1);
    const unsigned char* wt = smem + ST * STAGE;
    const unsigned char* xt = wt + TILE_BYTES;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const int off = pre ^ ((2 * ks + g2) << 4);
      const pf_bf16x8 a0 = pf_as_bf16x8(*reinterpret_cast<const uint4*>(wt + off + fb0 * 32 * (BK * 2)));
      const pf_bf16x8 a1 = pf_as_bf16x8(*reinterpret_cast<const uint4*>(wt + off + fb1 * 32 * (BK * 2)));
      const pf_bf16x8 b0 = pf_as_bf16x8(*reinterpret_cast<const uint4*>(xt + off + (2 * wc) * 32 * (BK * 2)));
      const pf_bf16x8 b1 = pf_as_bf16x8(*reinterpret_cast<const uint4*>(xt + off + (2 * wc + 1) * 32 * (BK * 2)));
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b0, acc[0][0], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b0, acc[1][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, acc[1][1], 0, 0, 0);
    }
    // the next step's tiles have landed (this wave's share) and everybody is done with these
    pf_wait_vm0();
    __syncthreads();
  };
  for (int step = 0; step < n_steps; step += 2) {
    k_step(step, std::integral_constant<int, 0>{});
    if (step + 1 < n_steps) k_step(step + 1, std::integral_constant<int, 1>{});
  }

  // ---------------- epilogue: rotate the keys, cast, store into the cache rows ----------------
  // acc[a][b], register i, lane (l32, g2): feature 32*fb_a + 8(i/4) + 4g2 + i%4 of the tile,
  // token 32*(2wc + b) + l32 of the tile.
  bf16_t* kcache = static_cast<bf16_t*>(kind == 0 ? p.k_base : p.v_base);
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const int tok = tok0 + 32 * (2 * wc + b) + l32;
    if (tok >= n_new) continue;
    const int j = pos0 + tok;  // cache row of this token, and its position
    int64_t row_off;           // element offset of (token j, kv head 0) in K_base / V_base, or of row j in L
    if (PAGED) {
      const int blk = p.block_table[static_cast<int64_t>(p.seq_index) * p.max_blocks_per_seq + (j >> 4)];
      row_off = kind == 2 ? (static_cast<int64_t>(blk) * 16 + (j & 15)) * p.rank
                          : static_cast<int64_t>(blk) * p.kv_block_stride + static_cast<int64_t>(j & 15) * p.kv_token_stride;
    } else {
      row_off = kind == 2 ? static_cast<int64_t>(j) * p.rank : static_cast<int64_t>(j) * p.kv_token_stride;
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
      const double log2_theta = log2(static_cast<double>(p.rope_theta));
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int dd = (32 * fb0 + 8 * (i >> 2) + 4 * g2 + (i & 3)) % D;  // < d/2 by construction
        const double inv_freq = exp2(-2.0 * dd / D * log2_theta);
        double ang = static_cast<double>(j) * inv_freq;
        ang -= 6.283185307179586476925 * floor(ang * 0.15915494309189533577);
        float sn, cs;
        sincosf(static_cast<float>(ang), &sn, &cs);
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

hipError_t launch_append(const AppendParams& p, hipStream_t s) {
  const int hd = p.n_kv_heads * p.head_dim;
  dim3 grid((p.n_new + 127) / 128, 2 * ((hd + 127) / 128) + 1);
  const bool paged = p.block_size != 0;
  if (p.head_dim == 128) {
    if (paged) hipLaunchKernelGGL((append_kernel<128, true>), grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL((append_kernel<128, false>), grid, dim3(256), 0, s, p);
  } else {
    if (paged) hipLaunchKernelGGL((append_kernel<64, true>), grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL((append_kernel<64, false>), grid, dim3(256), 0, s, p);
  }
  return hipGetLastError();
}

}  // namespace lra
