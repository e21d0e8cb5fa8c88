// MFMA causal prefill kernel of the Flash-LoRA-Attention library (bf16, gfx950).
//
// Alg. 1 of LRAgent (Sec. 3.3) for L_c new tokens of one agent after L_p cached
// ones, with the key side reordered as in App. D.1: per 64-key tile
//   S^T[key][row]  = K_base[key][:] . Q[row][:] + L[key][:] . Qt[row][:]   (MFMA, k = d + r)
//   online softmax along keys, causal mask aligned to the end of the sequence
//   O^T[d][row]   += V_base^T[d][key] . P^T[key][row]                      (MFMA)
//   Olr^T[p][row] += L^T[p][key]      . P^T[key][row]                      (MFMA)
// and after the last tile O^T += B_V^T . Olr^T (one more MFMA k-step per 16 ranks),
// O /= l.  Qt = Q B_K^T is formed once per wave before the loop (MFMA).
//
// A workgroup owns 128 query rows of one q head (4 waves x 32 rows) and walks the
// key tiles up to its causal limit.  v_mfma_f32_32x32x16_bf16 throughout; the
// transposed score tile leaves P^T in the lanes that need it as the B operand of
// the second product.  K_base / V_base / L tiles are shared by the four waves:
// global loads one tile ahead into registers, swizzled stores into a double
// buffered LDS tile, one barrier per tile.  ds_read_b128 feeds the K operand,
// ds_read_b64_tr_b16 the transposed V and L operands.  Workgroups are numbered so
// that all q heads of a kv head run on the same XCD and share its L2.
#include "lra_common.h"

namespace lra {

typedef __bf16 pf_bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 pf_bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 pf_bf16x2 __attribute__((ext_vector_type(2)));
typedef float pf_f32x16 __attribute__((ext_vector_type(16)));
typedef float pf_f32x4 __attribute__((ext_vector_type(4)));
typedef float pf_f32x2 __attribute__((ext_vector_type(2)));
typedef short pf_s16x4 __attribute__((ext_vector_type(4)));
typedef short pf_s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int pf_u32x4 __attribute__((ext_vector_type(4)));  // native vector: stays in registers
typedef unsigned int pf_u32x2 __attribute__((ext_vector_type(2)));

#define PF_LDS_AS(T, p) ((__attribute__((address_space(3))) T*)(p))

__device__ __forceinline__ pf_bf16x8 pf_as_bf16x8(uint4 v) { return __builtin_bit_cast(pf_bf16x8, v); }

__device__ __forceinline__ pf_s16x4 pf_read_tr16(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(PF_LDS_AS(pf_s16x4, p));
}

__device__ __forceinline__ pf_bf16x8 pf_join(pf_s16x4 lo, pf_s16x4 hi) {
  pf_s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(pf_bf16x8, v);
}

__device__ __forceinline__ uint32_t pf_pack2(float a, float b) {  // one v_cvt_pk_bf16_f32
  const pf_f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, pf_bf16x2));
}

// value of the partner lane l ^ 32 (inline assembly: the compiler's builtin for
// v_permlane32_swap treats its two results as one value)
__device__ __forceinline__ float pf_partner32(float v) {
  float x = v, y = v;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(x), "+v"(y));
  // lanes 0-31: x = own, y = partner ; lanes 32-63: x = partner, y = own
  return (threadIdx.x & 32) ? x : y;
}

// LDS swizzles (XOR on the 16-byte chunk index of a row).  The LDS of this chip serves
// 256 bytes per clock (64 banks): a ds_read_b128 is conflict-free when 16 consecutive
// lanes cover 16 different chunk positions of that 256-byte window, a ds_read_b64_tr_b16
// when the eight 32-byte pieces of 32 consecutive lanes do.
template <int D> __device__ __forceinline__ int pf_swz_k(int key) { return D == 128 ? (key & 15) : ((key >> 1) & 7); }
template <int D> __device__ __forceinline__ int pf_swz_v(int key) {
  return D == 128 ? ((key & 3) << 2) : (((key >> 1) & 1) << 2);
}

template <int D, int RP, bool PAGED>
__global__ __launch_bounds__(256, 2) void prefill_mfma_kernel(Params p) {
  constexpr int BM = 128, BN = 64;
  constexpr int KS = D / 16;   // k-steps of S^T over the head dimension
  constexpr int RKS = RP / 16; // k-steps over the padded rank
  constexpr int DB = D / 32;   // 32-row blocks of O^T
  constexpr int RB = (RP + 31) / 32;  // 32-row blocks of Olr^T
  constexpr int KCH = D / 8;   // 16-byte chunks per K/V row
  constexpr int KV_LOADS = BN * KCH / 256;  // per-thread 16-byte loads per K (or V) tile
  constexpr int LCH = RP / 8;               // 16-byte chunks per L row
  constexpr int L_LOADS = (BN * LCH + 255) / 256;
  constexpr int LS = RP * 2 + 8;            // L row stride in LDS (bytes): odd multiple of 8 spreads banks
  constexpr int K_BYTES = BN * D * 2;
  constexpr int L_BYTES = (BN * LS + 15) / 16 * 16;
  constexpr int STAGE = 2 * K_BYTES + L_BYTES;
  // With a half-empty last 32-row block of Olr^T (rank 16 or 48 after padding), one of its
  // idle rows carries a column of ones appended to the L tile, so the matrix core also
  // accumulates the softmax row sums.
  constexpr bool ONES_ROW = (RP % 32) != 0;

  __shared__ __align__(16) unsigned char smem[2 * STAGE];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, g2 = lane >> 5;
  const int Hq = p.n_q_heads, Hkv = p.n_kv_heads, G = p.group, r = p.rank;

  // workgroup -> (kv head, q head in group, q tile); consecutive ids go to consecutive XCDs
  const int lin = blockIdx.x;
  const int hk = lin % Hkv;
  const int rest = lin / Hkv;
  const int gq = rest % G;
  const int qt = rest / G;
  const int head = hk * G + gq;
  const int t = p.seq_index;
  const int n_t = min(p.seq_lens[t], p.max_seq_len);
  const int n_new = p.n_new;
  const int q0 = qt * BM;
  if (q0 >= n_new) return;
  const int base_vis = n_t - n_new;  // new token i sees keys 0 .. base_vis + i
  const int row = q0 + wave * 32 + l32;           // this lane's query row (new-token index)
  const int row_c = min(row, n_new - 1);          // clamped for loads; rows past the end are never stored
  const int limit = base_vis + row_c;             // last visible key of this lane's row
  const int wg_last = base_vis + min(q0 + BM, n_new) - 1;  // last key any row of the workgroup sees
  const int n_tiles = wg_last / BN + 1;

  const bf16_t* kb = static_cast<const bf16_t*>(p.k_base);
  const bf16_t* vb = static_cast<const bf16_t*>(p.v_base);
  const bf16_t* lr = static_cast<const bf16_t*>(p.l);
  const int32_t* bt = p.block_table + static_cast<int64_t>(t) * p.max_blocks_per_seq;

  // ---------------- tile staging: global -> registers -> LDS ----------------
  pf_u32x4 st_k[KV_LOADS], st_v[KV_LOADS], st_l[L_LOADS];  // one tile ahead, in registers
  // Contiguous cache: raw buffer resources over this kv head's rows; the per-thread byte
  // offsets are loop invariant and the tile offset travels in a scalar register, so a
  // tile costs no address arithmetic.  Rows past the sequence read as zero (they are
  // masked anyway).
  __amdgpu_buffer_rsrc_t rs_k, rs_v, rs_l;
  uint32_t kv_voff[KV_LOADS], l_voff[L_LOADS];
  const uint32_t ts2 = static_cast<uint32_t>(p.kv_token_stride) * 2u, r2 = static_cast<uint32_t>(r) * 2u;
  if (!PAGED) {
    const uint32_t kv_bytes = static_cast<uint32_t>(n_t - 1) * ts2 + D * 2;
    rs_k = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(kb) + static_cast<int64_t>(hk) * p.kv_head_stride, 0,
                                            static_cast<int>(kv_bytes), 0x00020000);
    rs_v = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(vb) + static_cast<int64_t>(hk) * p.kv_head_stride, 0,
                                            static_cast<int>(kv_bytes), 0x00020000);
    rs_l = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(lr), 0, static_cast<int>(static_cast<uint32_t>(n_t) * r2),
                                            0x00020000);
#pragma unroll
    for (int i = 0; i < KV_LOADS; ++i) {
      const int f = i * 256 + tid;
      kv_voff[i] = static_cast<uint32_t>(f / KCH) * ts2 + (f % KCH) * 16;
    }
#pragma unroll
    for (int i = 0; i < L_LOADS; ++i) {
      const int f = min(i * 256 + tid, BN * LCH - 1);
      l_voff[i] = static_cast<uint32_t>(f / LCH) * r2 + min(f % LCH, (r - 1) >> 3) * 16;
    }
  }
  // part q of 4 of the next tile's loads (contiguous cache): spread over the tile's
  // phases so that the eight waves of a CU do not hit the vector memory queue together
  auto load_part = [&](int j, int q) {
#pragma unroll
    for (int i = 0; i < KV_LOADS; ++i)
      if (i * 4 / KV_LOADS == q) {
        st_k[i] = __builtin_amdgcn_raw_buffer_load_b128(rs_k, kv_voff[i], static_cast<uint32_t>(j) * ts2, 0);
        st_v[i] = __builtin_amdgcn_raw_buffer_load_b128(rs_v, kv_voff[i], static_cast<uint32_t>(j) * ts2, 0);
      }
    if (q == 3) {
#pragma unroll
      for (int i = 0; i < L_LOADS; ++i)
        st_l[i] = __builtin_amdgcn_raw_buffer_load_b128(rs_l, l_voff[i], static_cast<uint32_t>(j) * r2, 0);
    }
  };
  auto load_tile = [&](int j) {
    if (!PAGED) {
#pragma unroll
      for (int q = 0; q < 4; ++q) load_part(j, q);
      return;
    }
#pragma unroll
    for (int i = 0; i < KV_LOADS; ++i) {
      const int f = i * 256 + tid;
      const int key = f / KCH, ch = f % KCH;
      const int tok = min(j + key, n_t - 1);  // clamped: masked later, never out of the sequence
      const int blk = bt[tok >> 4];
      const int64_t off = static_cast<int64_t>(blk) * p.kv_block_stride + static_cast<int64_t>(tok & 15) * p.kv_token_stride +
                          static_cast<int64_t>(hk) * p.kv_head_stride + ch * 8;
      st_k[i] = *reinterpret_cast<const pf_u32x4*>(kb + off);
      st_v[i] = *reinterpret_cast<const pf_u32x4*>(vb + off);
    }
#pragma unroll
    for (int i = 0; i < L_LOADS; ++i) {
      // every thread loads something valid (no branch around a load: a conditional load
      // would force the compiler to wait for it on the spot); store_tile drops or zeroes
      // what lies outside the tile or beyond the rank
      const int f = min(i * 256 + tid, BN * LCH - 1);
      const int key = f / LCH;
      const int ch = min(f % LCH, (r - 1) >> 3);
      const int tok = min(j + key, n_t - 1);
      const int64_t lrow = static_cast<int64_t>(bt[tok >> 4]) * 16 + (tok & 15);
      st_l[i] = *reinterpret_cast<const pf_u32x4*>(lr + lrow * r + ch * 8);
    }
  };
  auto store_tile = [&](unsigned char* buf) {
    unsigned char* ks = buf;
    unsigned char* vs = buf + K_BYTES;
    unsigned char* ls = buf + 2 * K_BYTES;
#pragma unroll
    for (int i = 0; i < KV_LOADS; ++i) {
      const int f = i * 256 + tid;
      const int key = f / KCH, ch = f % KCH;
      *reinterpret_cast<pf_u32x4*>(ks + key * (D * 2) + ((ch ^ pf_swz_k<D>(key)) << 4)) = st_k[i];
      *reinterpret_cast<pf_u32x4*>(vs + key * (D * 2) + ((ch ^ pf_swz_v<D>(key)) << 4)) = st_v[i];
    }
#pragma unroll
    for (int i = 0; i < L_LOADS; ++i) {
      const int f = i * 256 + tid;
      const int key = f / LCH, ch = f % LCH;
      if (f < BN * LCH) {
        const bool live = ch * 8 < r;  // chunks beyond the rank are zero
        unsigned char* dst = ls + key * LS + ch * 16;  // rows are 8-byte aligned only
        const pf_u32x4 v = live ? st_l[i] : pf_u32x4{0u, 0u, 0u, 0u};
        *reinterpret_cast<pf_u32x2*>(dst) = pf_u32x2{v[0], v[1]};
        *reinterpret_cast<pf_u32x2*>(dst + 8) = pf_u32x2{v[2], v[3]};
      }
    }
  };

  load_tile(0);

  // ---------------- prologue: Q operands, Qt = Q B_K^T ----------------
  // qb[ks]: B operand of S^T: lane (row l32, k = 16ks + 8g2 + e)
  pf_bf16x8 qb[KS];
  {
    const bf16_t* qrow = static_cast<const bf16_t*>(p.q) + (static_cast<int64_t>(row_c) * Hq + head) * D + g2 * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qb[ks] = pf_as_bf16x8(*reinterpret_cast<const uint4*>(qrow + ks * 16));
  }
  // Qt^T[rho][row] = B_K[rho][:] . Q[row][:]: C layout lane (row l32; reg i <-> rho = 32b + 8(i/4) + 4g2 + i%4).
  // As B operand of the rank k-steps of S^T, k-step ks' takes registers 8ks'..8ks'+7 of
  // block b = ks'/2, i.e. element e <-> rho = 16ks' + 8(e/4) + 4g2 + e%4; the L operand
  // below is read in the same order.
  pf_bf16x8 qtb[RKS];
  {
    const int64_t ldb = static_cast<int64_t>(Hkv) * D;
    const bf16_t* bkg = static_cast<const bf16_t*>(p.b_k);
#pragma unroll
    for (int b = 0; b < RB; ++b) {
      pf_f32x16 acc;
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] = 0.f;
      const int rho = b * 32 + l32;
      const bool live = bkg != nullptr && rho < r;
      const bf16_t* brow = bkg + (static_cast<int64_t>(p.adapter_index) * r + (live ? rho : 0)) * ldb + hk * D + g2 * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (live) v = *reinterpret_cast<const uint4*>(brow + ks * 16);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf_as_bf16x8(v), qb[ks], acc, 0, 0, 0);
      }
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int ks2 = b * 2 + half;
        if (ks2 < RKS) {
          const int o = half * 8;
          qtb[ks2] = pf_as_bf16x8(make_uint4(pf_pack2(acc[o + 0], acc[o + 1]), pf_pack2(acc[o + 2], acc[o + 3]),
                                             pf_pack2(acc[o + 4], acc[o + 5]), pf_pack2(acc[o + 6], acc[o + 7])));
        }
      }
    }
  }

  // ---------------- per-lane LDS read offsets ----------------
  // K rows as A operand of S^T (ds_read_b128): key = 32kt + l32, logical chunk c = 2ks + g2
  // lives at chunk c ^ swizzle(key); row offset and swizzle occupy disjoint address bits,
  // so the address is k_pre ^ (c << 4) (+ kt * 32 rows)
  const int k_pre = l32 * (D * 2) + (pf_swz_k<D>(l32) << 4);
  // V^T as A operand of O^T (ds_read_b64_tr_b16): lane a of a 16-lane group addresses
  // row 4*g2 + a/4 (+ 8 for the second read) of the 16-key k-step, 8 bytes at
  // d = 32b + 16dsel + 4(a%4): chunk 4b + 2dsel + c0, half sub; the swizzle flips chunk
  // bits 2..3, so the address is v_pre ^ (b << 6) (+ row offsets)
  const int a16 = lane & 15;
  const int dsel = (lane >> 4) & 1;   // which 16 of the 32 output rows this 16-lane group produces
  const int vrow = 4 * g2 + (a16 >> 2);
  const int v_pre = vrow * (D * 2) + ((((a16 & 3) >> 1) + 2 * dsel + pf_swz_v<D>(vrow)) << 4) + (a16 & 1) * 8;
  // L rows as A operand of S^T: two 8-byte pieces per k-step; L^T as A operand of Olr^T
  const int l_rd = l32 * LS + g2 * 8;           // + ks'*32 (+16 for the second piece) + kt*32*LS

  // ---------------- main loop ----------------
  pf_f32x16 o_acc[DB], lr_acc[RB];
#pragma unroll
  for (int b = 0; b < DB; ++b)
#pragma unroll
    for (int i = 0; i < 16; ++i) o_acc[b][i] = 0.f;
#pragma unroll
  for (int b = 0; b < RB; ++b)
#pragma unroll
    for (int i = 0; i < 16; ++i) lr_acc[b][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float sc = p.scale * 1.44269504088896340736f;

  if (ONES_ROW && tid < 2 * BN) {  // pad of every L row of both buffers: bf16 [1, 0, 0, 0]
    unsigned char* dst = smem + (tid / BN) * STAGE + 2 * K_BYTES + (tid % BN) * LS + RP * 2;
    *reinterpret_cast<pf_u32x2*>(dst) = pf_u32x2{0x00003f80u, 0u};
  }
  store_tile(smem);
  __syncthreads();

#ifdef LRA_PF_TIMING
  long long tph[6] = {0, 0, 0, 0, 0, 0};
  long long tprev = __builtin_readcyclecounter();
#define PF_MARK(i) { const long long tn = __builtin_readcyclecounter(); tph[i] += tn - tprev; tprev = tn; }
#else
#define PF_MARK(i)
#endif
  for (int tile = 0; tile < n_tiles; ++tile) {
    const int j = tile * BN;
    unsigned char* buf = smem + (tile & 1) * STAGE;
    const unsigned char* ks_l = buf;
    const unsigned char* vs_l = buf + K_BYTES;
    const unsigned char* ls_l = buf + 2 * K_BYTES;
    const bool more = tile + 1 < n_tiles;
    // unconditional: after the last tile this re-reads it (a conditional load would be
    // waited for right where it is issued)
    const int jn = more ? j + BN : j;
    if (PAGED) load_tile(jn); else load_part(jn, 0);
    PF_MARK(0)

    // S^T for the two 32-key halves of the tile
    pf_f32x16 s[2];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
      for (int i = 0; i < 16; ++i) s[kt][i] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const pf_bf16x8 a = pf_as_bf16x8(
            *reinterpret_cast<const uint4*>(ks_l + (k_pre ^ ((2 * ks + g2) << 4)) + kt * 32 * D * 2));
        s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qb[ks], s[kt], 0, 0, 0);
      }
#pragma unroll
      for (int ks = 0; ks < RKS; ++ks) {
        const unsigned char* src = ls_l + l_rd + ks * 32 + kt * 32 * LS;
        const uint2 lo = *reinterpret_cast<const uint2*>(src);
        const uint2 hi = *reinterpret_cast<const uint2*>(src + 16);
        s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf_as_bf16x8(make_uint4(lo.x, lo.y, hi.x, hi.y)), qtb[ks],
                                                        s[kt], 0, 0, 0);
      }
    }
    if (!PAGED) load_part(jn, 1);
    PF_MARK(1)
    // causal mask + online softmax.  Element (kt, i) of this lane is key
    // j + 32kt + 8(i/4) + 4g2 + i%4 of row l32.
    if (j + BN - 1 > base_vis + q0 + wave * 32) {  // some row of this wave does not see the whole tile
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = j + 32 * kt + 8 * (i >> 2) + 4 * g2 + (i & 3);
          if (key > limit) s[kt][i] = -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[kt][i]);
    mx = fmaxf(mx, pf_partner32(mx)) * sc;
    if (__builtin_amdgcn_ballot_w64(mx > m_run) != 0) {
      const float m_new = fmaxf(m_run, mx);
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int b = 0; b < DB; ++b) o_acc[b] *= alpha;
#pragma unroll
      for (int b = 0; b < RB; ++b) lr_acc[b] *= alpha;
    }
    const float nm = -m_run;  // finite from the first tile on: key 0 is visible to every row
    pf_bf16x8 pb[2][2];       // [kt][16-key k-step]
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      float e[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        e[i] = __builtin_amdgcn_exp2f(fmaf(s[kt][i], sc, nm));
        if (!ONES_ROW) l_run += e[i];
      }
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2)
        pb[kt][h2] = pf_as_bf16x8(make_uint4(pf_pack2(e[8 * h2 + 0], e[8 * h2 + 1]), pf_pack2(e[8 * h2 + 2], e[8 * h2 + 3]),
                                             pf_pack2(e[8 * h2 + 4], e[8 * h2 + 5]), pf_pack2(e[8 * h2 + 6], e[8 * h2 + 7])));
    }
    if (!PAGED) load_part(jn, 2);
    PF_MARK(2)
    // O^T += V^T P^T ; Olr^T += L^T P^T, one 16-key k-step at a time.
    // k-step (kt, h2), element e <-> key 32kt + 16h2 + 8(e/4) + 4g2 + e%4.
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        if (!PAGED && kt == 1 && h2 == 0) load_part(jn, 3);
        const int rowoff = (32 * kt + 16 * h2) * (D * 2);
#pragma unroll
        for (int b = 0; b < DB; ++b) {
          const unsigned char* src = vs_l + (v_pre ^ (b << 6)) + rowoff;
          const pf_bf16x8 a = pf_join(pf_read_tr16(src), pf_read_tr16(src + 8 * (D * 2)));
          o_acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[kt][h2], o_acc[b], 0, 0, 0);
        }
#pragma unroll
        for (int b = 0; b < RB; ++b) {
          // rows rho = 32b + 16dsel + a16 of L^T.  In a half-empty last block the upper 16
          // lanes read the pad of the row instead ([1, 0, 0, 0]): output row 32b + 16 then
          // accumulates the row sums; the rows after it are never used.
          const bool upper_idle = ONES_ROW && b == RB - 1;
          const int col = (upper_idle && dsel) ? RP * 2 : b * 64 + dsel * 32 + (a16 & 3) * 8;
          const unsigned char* src = ls_l + vrow * LS + col + (32 * kt + 16 * h2) * LS;
          const pf_bf16x8 a = pf_join(pf_read_tr16(src), pf_read_tr16(src + 8 * LS));
          lr_acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[kt][h2], lr_acc[b], 0, 0, 0);
        }
      }

    PF_MARK(3)
    if (more) store_tile(smem + ((tile + 1) & 1) * STAGE);
    PF_MARK(4)
    __syncthreads();
    PF_MARK(5)
  }
#ifdef LRA_PF_TIMING
  if (blockIdx.x == 300 && lane == 0) {
    for (int i = 0; i < 6; ++i) p.part_ml[wave * 8 + i] = static_cast<float>(tph[i]);
    p.part_ml[wave * 8 + 6] = static_cast<float>(n_tiles);
  }
#endif

  // ---------------- epilogue: O^T += B_V^T Olr^T, O /= l, store ----------------
  if (ONES_ROW) {
    // row sums sit in register 8 (rho = 32(RB-1) + 16) of the lanes with g2 == 0
    const float mine = lr_acc[RB - 1][8];
    const float other = pf_partner32(mine);
    l_run = g2 == 0 ? mine : other;
  } else {
    l_run += pf_partner32(l_run);
  }
  if (p.b_v != nullptr) {
    const int64_t ldb = static_cast<int64_t>(Hkv) * D;
    const bf16_t* bv = static_cast<const bf16_t*>(p.b_v) + static_cast<int64_t>(p.adapter_index) * r * ldb + hk * D;
#pragma unroll
    for (int ks = 0; ks < RKS; ++ks) {
      // B operand: Olr^T registers 8(ks&1)..+7 of block ks/2: element e <-> rho = 16ks + 8(e/4) + 4g2 + e%4
      const int o = (ks & 1) * 8;
      const pf_f32x16& src = lr_acc[ks >> 1];
      const pf_bf16x8 bop =
          pf_as_bf16x8(make_uint4(pf_pack2(src[o + 0], src[o + 1]), pf_pack2(src[o + 2], src[o + 3]),
                                  pf_pack2(src[o + 4], src[o + 5]), pf_pack2(src[o + 6], src[o + 7])));
#pragma unroll
      for (int b = 0; b < DB; ++b) {
        // A operand: B_V^T: lane (d = 32b + l32, element e <-> rho as above)
        uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int rho = 16 * ks + 8 * (e >> 2) + 4 * g2 + (e & 3);
          const uint32_t val = rho < r ? static_cast<uint32_t>(bv[rho * ldb + 32 * b + l32]) : 0u;
          w[e >> 1] |= val << ((e & 1) * 16);
        }
        o_acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf_as_bf16x8(make_uint4(w[0], w[1], w[2], w[3])), bop,
                                                           o_acc[b], 0, 0, 0);
      }
    }
  }
  if (row < n_new) {
    const float inv = 1.0f / l_run;
    bf16_t* orow = static_cast<bf16_t*>(p.out) + (static_cast<int64_t>(row) * Hq + head) * D;
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        // registers 4q..4q+3 are d = 32b + 8q + 4g2 + 0..3
        const uint2 pk = make_uint2(pf_pack2(o_acc[b][4 * q + 0] * inv, o_acc[b][4 * q + 1] * inv),
                                    pf_pack2(o_acc[b][4 * q + 2] * inv, o_acc[b][4 * q + 3] * inv));
        *reinterpret_cast<uint2*>(orow + 32 * b + 8 * q + 4 * g2) = pk;
      }
  }
}

template <int D, int RP>
static hipError_t launch_pf(const Params& p, dim3 grid, hipStream_t s) {
  if (p.block_size != 0)
    hipLaunchKernelGGL((prefill_mfma_kernel<D, RP, true>), grid, dim3(256), 0, s, p);
  else
    hipLaunchKernelGGL((prefill_mfma_kernel<D, RP, false>), grid, dim3(256), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_prefill_mfma(const Params& p, hipStream_t s) {
  const int q_tiles = (p.n_new + 127) / 128;
  dim3 grid(q_tiles * p.n_q_heads);
  const int rp = p.rank <= 16 ? 16 : (p.rank <= 32 ? 32 : 64);
  if (p.head_dim == 128) {
    if (rp == 16) return launch_pf<128, 16>(p, grid, s);
    if (rp == 32) return launch_pf<128, 32>(p, grid, s);
    return launch_pf<128, 64>(p, grid, s);
  }
  if (rp == 16) return launch_pf<64, 16>(p, grid, s);
  if (rp == 32) return launch_pf<64, 32>(p, grid, s);
  return launch_pf<64, 64>(p, grid, s);
}

}  // namespace lra
