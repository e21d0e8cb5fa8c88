// MFMA decode kernel of the Flash-LoRA-Attention library (bf16, gfx950).
//
// One workgroup streams one range of keys of one (sequence, kv head) for ALL
// query rows that share that stream: every agent decoding on the sequence times
// the q heads of the GQA group.  Those rows form the 16-wide N dimension of
// v_mfma_f32_16x16x32_bf16, so K_base, V_base and L are read from HBM once for
// all agents (LRAgent Sec. 3.2, one base cache and one LR cache for the system).
//
// Per 32-key step (Alg. 1 lines 9-17 with the App. D.1 key-side reordering):
//   S^T[key][row]  = K_base[key][:] . Q[row][:]  +  L[key][:] . Qt[row][:]     (MFMA)
//   online softmax along keys (per row = per lane column)
//   O^T[d][row]   += V_base^T[d][key] . P^T[key][row]                          (MFMA)
//   Olr^T[p][row] += L^T[p][key]      . P^T[key][row]                          (MFMA)
// with Qt = Q B_K^T computed once per workgroup in the prologue (MFMA).
// Computing S transposed makes the C-layout of the score tile coincide with the
// B-operand layout of the second product, so P never moves between lanes.
//
// Data path: coalesced 16-byte global loads into registers (one or two steps
// ahead), a swizzled copy into wave-private LDS, ds_read_b128 for the K/L
// A-operands and ds_read_b64_tr_b16 for the transposed V/L A-operands.  The
// waves of a workgroup own disjoint key ranges and never synchronise inside the
// loop; their states are merged through LDS at the end (flash-decoding rule) and
// one partial (m, l, O, O_lr) per workgroup goes to the workspace.
#include "lra_common.h"

namespace lra {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ uint4 lds_read16(const unsigned char* base, int byte_off) {
  return *reinterpret_cast<const uint4*>(base + byte_off);
}

__device__ __forceinline__ void lds_write16(unsigned char* base, int byte_off, uint4 v) {
  *reinterpret_cast<uint4*>(base + byte_off) = v;
}

// ds_read_b64_tr_b16: inside every group of 16 lanes, lane i receives for e = 0..3
// element (i % 4) of the 8 bytes addressed by lane 4e + i/4.
__device__ __forceinline__ s16x4 lds_read_tr16(const unsigned char* base, int byte_off) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, base + byte_off));
}

__device__ __forceinline__ bf16x8 join_tr(s16x4 lo, s16x4 hi) {
  s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  return static_cast<uint32_t>(f32_to_bf16(a)) | (static_cast<uint32_t>(f32_to_bf16(b)) << 16);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int D, int RT, int RP, int NW, int PF>
__global__ __launch_bounds__(NW * 64) void decode_mfma_kernel(Params p) {
  constexpr int KS = D / 32;    // MFMA k-steps over the head dimension
  constexpr int RKS = RP / 32;  // MFMA k-steps over the (padded) rank
  constexpr int DB = D / 16;    // 16-wide output blocks over d
  constexpr int RB = RP / 16;   // 16-wide output blocks over the rank
  constexpr int KCH = D / 8;    // 16-byte chunks per K/V row
  constexpr int RCH = RP / 8;   // 16-byte chunks per L row in LDS
  constexpr int KVL = D / 16;   // wave-wide 16-byte loads per 32-key K (or V) tile
  constexpr int LL = RP / 16;   // wave-wide 16-byte loads per 32-key L tile
  constexpr int KV_BYTES = 32 * D * 2;
  constexpr int L_BYTES = 32 * RP * 2;
  constexpr int WAVE_BYTES = 2 * KV_BYTES + L_BYTES;
  constexpr int QT_BYTES = RT * 16 * RP * 2;
  constexpr int NACC = RT * (DB + RB) * 4 + RT;
  constexpr int MERGE_SLOT = NACC * 64 * 4;
  constexpr int STAGE_TOTAL = NW * WAVE_BYTES + QT_BYTES;
  constexpr int MERGE_TOTAL = (NW / 2) * MERGE_SLOT;
  constexpr int SMEM = STAGE_TOTAL > MERGE_TOTAL ? STAGE_TOTAL : MERGE_TOTAL;
  constexpr int LSW_SHIFT = (RP == 32) ? 1 : 0;

  __shared__ __align__(16) unsigned char smem[SMEM];
  __shared__ float m_sh[NW][RT][16];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ln = lane & 15, lg = lane >> 4;
  const int split = blockIdx.x, h = blockIdx.y;
  const int t = blockIdx.z / p.row_groups;
  const int rg = blockIdx.z - t * p.row_groups;
  const int n_t = min(p.seq_lens[t], p.max_seq_len);
  const int j0 = split * p.split_keys;
  if (j0 >= n_t) return;
  const int q_begin = p.seq_query_start[t];
  const int n_q = p.seq_query_start[t + 1] - q_begin;
  const int GP = p.group_pad, G = p.group, r = p.rank;
  const int row0 = rg * RT * 16;
  if (row0 >= n_q * GP) return;

  const int j1 = min(j0 + p.split_keys, n_t);
  const int kpw = p.split_keys / NW;  // multiple of 32
  const int jw0 = j0 + wave * kpw;
  const int jw1 = min(jw0 + kpw, j1);

  unsigned char* ks_lds = smem + wave * WAVE_BYTES;
  unsigned char* vs_lds = ks_lds + KV_BYTES;
  unsigned char* ls_lds = vs_lds + KV_BYTES;
  unsigned char* qt_lds = smem + NW * WAVE_BYTES;

  const bf16_t* kb = static_cast<const bf16_t*>(p.k_base);
  const bf16_t* vb = static_cast<const bf16_t*>(p.v_base);
  const bf16_t* lr = static_cast<const bf16_t*>(p.l);
  const int32_t* bt = p.block_table + static_cast<int64_t>(t) * p.max_blocks_per_seq;
  const bool paged = p.block_size != 0;
  const bool l_fast = (r & 7) == 0;

  struct Stage {
    uint4 k[KVL], v[KVL], l[LL];
  };

  // ---- global -> register loads of one 32-key step starting at token j ----
  auto load_stage = [&](Stage& st, int j) {
    int blk0 = 0, blk1 = 0;
    if (paged) {
      blk0 = bt[j >> 4];
      blk1 = (j + 16 < n_t) ? bt[(j >> 4) + 1] : blk0;
    }
#pragma unroll
    for (int i = 0; i < KVL; ++i) {
      const int f = i * 64 + lane;
      const int key = f / KCH, ch = f % KCH;
      const int tok = min(j + key, n_t - 1);
      int64_t off;
      if (paged) {
        const int blk = ((tok >> 4) == (j >> 4)) ? blk0 : blk1;
        off = static_cast<int64_t>(blk) * p.kv_block_stride + static_cast<int64_t>(tok & 15) * p.kv_token_stride;
      } else {
        off = static_cast<int64_t>(tok) * p.kv_token_stride;
      }
      off += static_cast<int64_t>(h) * p.kv_head_stride + ch * 8;
      st.k[i] = *reinterpret_cast<const uint4*>(kb + off);
      st.v[i] = *reinterpret_cast<const uint4*>(vb + off);
    }
#pragma unroll
    for (int i = 0; i < LL; ++i) {
      const int f = i * 64 + lane;
      const int key = f / RCH, ch = f % RCH;
      const int tok = min(j + key, n_t - 1);
      int64_t row;
      if (paged) {
        const int blk = ((tok >> 4) == (j >> 4)) ? blk0 : blk1;
        row = static_cast<int64_t>(blk) * 16 + (tok & 15);
      } else {
        row = tok;
      }
      const bf16_t* src = lr + row * r + ch * 8;
      uint4 val = make_uint4(0, 0, 0, 0);
      if (l_fast) {
        if (ch * 8 < r) val = *reinterpret_cast<const uint4*>(src);
      } else {
        uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (ch * 8 + e < r) w[e >> 1] |= static_cast<uint32_t>(src[e]) << ((e & 1) * 16);
        val = make_uint4(w[0], w[1], w[2], w[3]);
      }
      st.l[i] = val;
    }
  };

  // ---- registers -> wave-private LDS, swizzled on 16-byte chunks ----
  auto store_stage = [&](const Stage& st) {
#pragma unroll
    for (int i = 0; i < KVL; ++i) {
      const int f = i * 64 + lane;
      const int key = f / KCH, ch = f % KCH;
      lds_write16(ks_lds, key * (D * 2) + ((ch ^ (key & 7)) << 4), st.k[i]);
      lds_write16(vs_lds, key * (D * 2) + ((ch ^ ((key & 3) << 1)) << 4), st.v[i]);
    }
#pragma unroll
    for (int i = 0; i < LL; ++i) {
      const int f = i * 64 + lane;
      const int key = f / RCH, ch = f % RCH;
      lds_write16(ls_lds, key * (RP * 2) + ((ch ^ ((key >> LSW_SHIFT) & (RCH - 1))) << 4), st.l[i]);
    }
  };

  Stage st0, st1;
  const bool has_keys = jw0 < jw1;
  if (has_keys) load_stage(st0, jw0);
  if (PF == 2 && jw0 + 32 < jw1) load_stage(st1, jw0 + 32);

  // ---- prologue: Q rows as MFMA operands, Qt = Q B_K^T through LDS ----
  bf16x8 qb[RT][KS];   // B operand of S^T: lane (row ln, k = 32ks + 8lg + e)
  bf16x8 qtb[RT][RKS];
  const bf16_t* qg = static_cast<const bf16_t*>(p.q);
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int R = row0 + rt * 16 + ln;
    const int slot = R / GP, gg = R - slot * GP;
    const bool valid = slot < n_q && gg < G;
    const bf16_t* qrow = qg + (static_cast<int64_t>(q_begin + slot) * p.n_q_heads + h * G + gg) * D;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (valid) v = *reinterpret_cast<const uint4*>(qrow + ks * 32 + lg * 8);
      qb[rt][ks] = as_bf16x8(v);
    }
  }
  {
    const int S = 16 / GP;  // agent slots per 16-row tile
    const bf16_t* bkg = static_cast<const bf16_t*>(p.b_k);
    const int64_t ldb = static_cast<int64_t>(p.n_kv_heads) * D;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      for (int idx = wave; idx < S * RB; idx += NW) {
        const int si = idx / RB, cb = idx - si * RB;
        const int slot = (row0 + rt * 16) / GP + si;
        const int rho = cb * 16 + ln;
        const bool live = bkg != nullptr && slot < n_q && rho < r;
        int a = 0;
        if (slot < n_q) a = p.query_adapter[q_begin + slot];
        const bf16_t* brow = bkg + (static_cast<int64_t>(a) * r + rho) * ldb + h * D + lg * 8;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          uint4 v = make_uint4(0, 0, 0, 0);
          if (live) v = *reinterpret_cast<const uint4*>(brow + ks * 32);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qb[rt][ks], as_bf16x8(v), acc, 0, 0, 0);
        }
        // C layout: rows 4lg + j, column rho.  Rows 4lg..4lg+3 belong to slot (4lg)/GP.
        if ((4 * lg) / GP == si) {
          bf16_t* dst = reinterpret_cast<bf16_t*>(qt_lds) + (rt * 16 + 4 * lg) * RP + rho;
#pragma unroll
          for (int j = 0; j < 4; ++j) dst[j * RP] = f32_to_bf16(acc[j]);
        }
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int ks = 0; ks < RKS; ++ks)
      qtb[rt][ks] = as_bf16x8(lds_read16(qt_lds, ((rt * 16 + ln) * RP + ks * 32 + lg * 8) * 2));

  // ---- main loop ----
  f32x4 o_acc[RT][DB], lr_acc[RT][RB];
  float m_run[RT], l_run[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    m_run[rt] = -INFINITY;
    l_run[rt] = 0.f;
#pragma unroll
    for (int b = 0; b < DB; ++b) o_acc[rt][b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int b = 0; b < RB; ++b) lr_acc[rt][b] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  const float sc = p.scale * 1.44269504088896340736f;  // scores in base-2 units

  auto compute_step = [&](int j) {
    // S^T for two 16-key tiles
    f32x4 s[2][RT];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int key = tt * 16 + ln;
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) s[tt][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 a = as_bf16x8(lds_read16(ks_lds, key * (D * 2) + (((ks * 4 + lg) ^ (key & 7)) << 4)));
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
          s[tt][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qb[rt][ks], s[tt][rt], 0, 0, 0);
      }
#pragma unroll
      for (int ks = 0; ks < RKS; ++ks) {
        const bf16x8 a = as_bf16x8(
            lds_read16(ls_lds, key * (RP * 2) + (((ks * 4 + lg) ^ ((key >> LSW_SHIFT) & (RCH - 1))) << 4)));
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
          s[tt][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qtb[rt][ks], s[tt][rt], 0, 0, 0);
      }
    }
    // online softmax; element (tt, jj) of this lane is key j + 16tt + 4lg + jj of row ln
    bf16x8 pb[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      float mx = -INFINITY;
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int key = j + tt * 16 + lg * 4 + jj;
          const float v = key < n_t ? s[tt][rt][jj] * sc : -INFINITY;
          s[tt][rt][jj] = v;
          mx = fmaxf(mx, v);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run[rt], mx);
      const float alpha = fast_exp2(m_run[rt] - m_new);
      m_run[rt] = m_new;
      float pe[8];
      float sum = 0.f;
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const float e = fast_exp2(s[tt][rt][jj] - m_new);
          pe[tt * 4 + jj] = e;
          sum += e;
        }
      l_run[rt] = l_run[rt] * alpha + sum;
      uint4 pk = make_uint4(pack_bf16x2(pe[0], pe[1]), pack_bf16x2(pe[2], pe[3]), pack_bf16x2(pe[4], pe[5]),
                            pack_bf16x2(pe[6], pe[7]));
      pb[rt] = as_bf16x8(pk);
#pragma unroll
      for (int b = 0; b < DB; ++b) o_acc[rt][b] *= alpha;
#pragma unroll
      for (int b = 0; b < RB; ++b) lr_acc[rt][b] *= alpha;
    }
    // O^T += V^T P^T ; Olr^T += L^T P^T
    const int ka = 4 * lg + (ln >> 2);  // key (within a 16-key tile) this lane addresses for the transpose read
#pragma unroll
    for (int b = 0; b < DB; ++b) {
      const int ch = 2 * b + ((ln & 3) >> 1);
      const int sub = (ln & 1) * 8;
      const s16x4 lo = lds_read_tr16(vs_lds, ka * (D * 2) + ((ch ^ ((ka & 3) << 1)) << 4) + sub);
      const s16x4 hi = lds_read_tr16(vs_lds, (16 + ka) * (D * 2) + ((ch ^ ((ka & 3) << 1)) << 4) + sub);
      const bf16x8 a = join_tr(lo, hi);
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
        o_acc[rt][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pb[rt], o_acc[rt][b], 0, 0, 0);
    }
#pragma unroll
    for (int b = 0; b < RB; ++b) {
      const int ch = 2 * b + ((ln & 3) >> 1);
      const int sub = (ln & 1) * 8;
      const int k0 = ka, k1 = 16 + ka;
      const s16x4 lo = lds_read_tr16(ls_lds, k0 * (RP * 2) + ((ch ^ ((k0 >> LSW_SHIFT) & (RCH - 1))) << 4) + sub);
      const s16x4 hi = lds_read_tr16(ls_lds, k1 * (RP * 2) + ((ch ^ ((k1 >> LSW_SHIFT) & (RCH - 1))) << 4) + sub);
      const bf16x8 a = join_tr(lo, hi);
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
        lr_acc[rt][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pb[rt], lr_acc[rt][b], 0, 0, 0);
    }
  };

  if (PF == 2) {
    for (int j = jw0; j < jw1; j += 64) {
      store_stage(st0);
      if (j + 64 < jw1) load_stage(st0, j + 64);
      __builtin_amdgcn_wave_barrier();
      compute_step(j);
      __builtin_amdgcn_wave_barrier();
      if (j + 32 < jw1) {
        store_stage(st1);
        if (j + 96 < jw1) load_stage(st1, j + 96);
        __builtin_amdgcn_wave_barrier();
        compute_step(j + 32);
        __builtin_amdgcn_wave_barrier();
      }
    }
  } else {
    for (int j = jw0; j < jw1; j += 32) {
      store_stage(st0);
      if (j + 32 < jw1) load_stage(st0, j + 32);
      __builtin_amdgcn_wave_barrier();
      compute_step(j);
      __builtin_amdgcn_wave_barrier();
    }
  }

  // ---- merge the waves of this workgroup (flash-decoding rule), base-2 units ----
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    l_run[rt] += __shfl_xor(l_run[rt], 16, 64);
    l_run[rt] += __shfl_xor(l_run[rt], 32, 64);
    if (lg == 0) m_sh[wave][rt][ln] = m_run[rt];
  }
  __syncthreads();
  float m_all[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    float mm = m_sh[0][rt][ln];
#pragma unroll
    for (int w = 1; w < NW; ++w) mm = fmaxf(mm, m_sh[w][rt][ln]);
    m_all[rt] = mm;  // finite: wave 0 always owns at least one key
    const float wgt = fast_exp2(m_run[rt] - mm);
    l_run[rt] *= wgt;
#pragma unroll
    for (int b = 0; b < DB; ++b) o_acc[rt][b] *= wgt;
#pragma unroll
    for (int b = 0; b < RB; ++b) lr_acc[rt][b] *= wgt;
  }
  float* mslots = reinterpret_cast<float*>(smem);
#pragma unroll
  for (int stride = NW / 2; stride >= 1; stride >>= 1) {
    if (wave >= stride && wave < 2 * stride) {
      float* dst = mslots + (wave - stride) * (NACC * 64) + lane;
      int x = 0;
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) dst[(x++) * 64] = o_acc[rt][b][jj];
#pragma unroll
        for (int b = 0; b < RB; ++b)
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) dst[(x++) * 64] = lr_acc[rt][b][jj];
        dst[(x++) * 64] = l_run[rt];
      }
    }
    __syncthreads();
    if (wave < stride) {
      const float* src = mslots + wave * (NACC * 64) + lane;
      int x = 0;
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) o_acc[rt][b][jj] += src[(x++) * 64];
#pragma unroll
        for (int b = 0; b < RB; ++b)
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) lr_acc[rt][b][jj] += src[(x++) * 64];
        l_run[rt] += src[(x++) * 64];
      }
    }
    __syncthreads();
  }

  // ---- wave 0 writes the workgroup's partial state ----
  if (wave == 0) {
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const int R = row0 + rt * 16 + ln;
      const int slot_q = R / GP, gg = R - slot_q * GP;
      if (!(slot_q < n_q && gg < G)) continue;
      const int64_t row = static_cast<int64_t>(q_begin + slot_q) * p.n_q_heads + h * G + gg;
      const int64_t slot = row * p.n_splits + split;
      if (lg == 0) {
        p.part_ml[slot * 2 + 0] = m_all[rt] * 0.69314718055994530942f;  // natural-log units
        p.part_ml[slot * 2 + 1] = l_run[rt];
      }
#pragma unroll
      for (int b = 0; b < DB; ++b)
        *reinterpret_cast<f32x4*>(p.part_o + slot * D + b * 16 + lg * 4) = o_acc[rt][b];
#pragma unroll
      for (int b = 0; b < RB; ++b)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int rho = b * 16 + lg * 4 + jj;
          if (rho < r) p.part_lr[slot * r + rho] = lr_acc[rt][b][jj];
        }
    }
  }
}

template <int D, int RT, int RP>
static hipError_t launch_cfg(const Params& p, dim3 grid, hipStream_t s, int pf) {
  constexpr int NW = 4;
  if (pf == 2)
    hipLaunchKernelGGL((decode_mfma_kernel<D, RT, RP, NW, 2>), grid, dim3(NW * 64), 0, s, p);
  else
    hipLaunchKernelGGL((decode_mfma_kernel<D, RT, RP, NW, 1>), grid, dim3(NW * 64), 0, s, p);
  return hipGetLastError();
}

// Row tiles per workgroup the kernel is built for.
int decode_mfma_row_tiles(int rows_needed) { return rows_needed <= 16 ? 1 : 2; }

hipError_t launch_decode_mfma(const Params& p, int row_tiles, int prefetch, hipStream_t s) {
  dim3 grid(p.n_splits, p.n_kv_heads, p.n_seqs * p.row_groups);
  const int rp = p.rank <= 32 ? 32 : 64;
  const int key = (p.head_dim == 128 ? 4 : 0) | (row_tiles == 2 ? 2 : 0) | (rp == 64 ? 1 : 0);
  switch (key) {
    case 0: return launch_cfg<64, 1, 32>(p, grid, s, prefetch);
    case 1: return launch_cfg<64, 1, 64>(p, grid, s, prefetch);
    case 2: return launch_cfg<64, 2, 32>(p, grid, s, prefetch);
    case 3: return launch_cfg<64, 2, 64>(p, grid, s, prefetch);
    case 4: return launch_cfg<128, 1, 32>(p, grid, s, prefetch);
    case 5: return launch_cfg<128, 1, 64>(p, grid, s, prefetch);
    case 6: return launch_cfg<128, 2, 32>(p, grid, s, prefetch);
    default: return launch_cfg<128, 2, 64>(p, grid, s, prefetch);
  }
}

}  // namespace lra
