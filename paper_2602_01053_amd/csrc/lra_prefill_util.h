// Device helpers shared by the MFMA prefill kernels of the Flash-LoRA-Attention library
// (bf16, gfx950): vector types, LDS transpose reads, bf16 packing, hand-issued
// HBM -> LDS loads and the LDS swizzles of the K, V and L tiles.
#pragma once
#include <type_traits>

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

typedef _Float16 pf_f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 pf_f16x2 __attribute__((ext_vector_type(2)));
// two floats rounded to fp16 (nearest even), packed
__device__ __forceinline__ uint32_t pf_pack2_f16(float a, float b) {
  const pf_f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, pf_f16x2));
}
// eight bf16 values as fp16: exact for magnitudes from 2^-14 (6.1e-5) to 65504; smaller ones lose
// bits they barely had (below 6e-8 they become zero), larger ones become infinite
__device__ __forceinline__ pf_f16x8 pf_bf16x8_to_f16x8(pf_bf16x8 v) {
  const uint4 u = __builtin_bit_cast(uint4, v);
  const uint32_t w[4] = {u.x, u.y, u.z, u.w};
  uint32_t o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) o[i] = pf_pack2_f16(__uint_as_float(w[i] << 16), __uint_as_float(w[i] & 0xffff0000u));
  return __builtin_bit_cast(pf_f16x8, make_uint4(o[0], o[1], o[2], o[3]));
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

// Raw buffer resource over [base, base + bytes) as four scalar words: loads past the end
// return zero and touch no memory.  The words are wave-uniform by construction;
// readfirstlane pins them to scalar registers.
__device__ __forceinline__ pf_u32x4 pf_rsrc(const void* base, uint32_t bytes) {
  auto uni = [](uint32_t v) { return static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(v))); };
  const uint64_t a = reinterpret_cast<uint64_t>(base);
  return pf_u32x4{uni(static_cast<uint32_t>(a)), uni(static_cast<uint32_t>(a >> 32) & 0xffffu), uni(bytes), 0x00020000u};
}

// buffer_load_dwordx4 ... lds: 16 bytes per lane from the buffer straight into LDS at
// lds_addr + lane*16 (the LDS base travels in M0; one wait state between the write of M0
// and the load).  Inline assembly on purpose: the compiler does not track these loads, so
// it neither parks their data in registers nor drains them before unrelated LDS reads.
// The waits are placed by hand (pf_wait_vm0) and LDS ordering comes from the barriers.
__device__ __forceinline__ void pf_load16_to_lds(pf_u32x4 rs, uint32_t lds_addr, uint32_t voff, uint32_t soff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(__builtin_amdgcn_readfirstlane(static_cast<int>(lds_addr))), "v"(voff), "s"(rs),
                 "s"(__builtin_amdgcn_readfirstlane(static_cast<int>(soff)))  // wave-uniform by construction
               : "m0");
}
__device__ __forceinline__ void pf_wait_vm0() { asm volatile("s_waitcnt vmcnt(0)"); }

// Read-only int32 tables addressed as constant memory, so that wave-uniform reads stay
// scalar loads although the kernel contains assembly statements the compiler cannot see
// through.
typedef const __attribute__((address_space(4))) int32_t* pf_const_i32;
#define PF_CONST_I32(p) ((pf_const_i32)(p))

constexpr uint32_t kPfOob = 0x80000000u;  // beyond any resource this kernel builds

// Rotary angles.  Pair dd of a head turns by pos * theta^(-2 dd / d) radians; the kernels keep
// that rate in revolutions (divided by 2 pi) in double precision, so that the product with a
// position in the tens of thousands can be reduced to its fractional part without loss, and
// take sine and cosine of the fraction with v_sin_f32 / v_cos_f32 (argument in revolutions,
// absolute error around 1e-6: far below the bf16 rounding of the result).
__device__ __forceinline__ double rope_rate_rev(int dd, int head_dim, float theta) {
  return exp2(-2.0 * dd / head_dim * log2(static_cast<double>(theta))) * 0.15915494309189533577;
}
__device__ __forceinline__ void rope_sincos(double rate_rev, int pos, float& sn, float& cs) {
  double rev = static_cast<double>(pos) * rate_rev;
  rev -= floor(rev);
  const float fr = static_cast<float>(rev);
  sn = __builtin_amdgcn_sinf(fr);
  cs = __builtin_amdgcn_cosf(fr);
}

// LDS swizzles (XOR on the 16-byte chunk index of a row).  The LDS of this chip serves
// 256 bytes per clock (64 banks): a ds_read_b128 is conflict-free when 16 consecutive
// lanes cover 16 different chunk positions of that 256-byte window, a ds_read_b64_tr_b16
// when the eight 32-byte pieces of 32 consecutive lanes do.
template <int D> __device__ __forceinline__ int pf_swz_k(int key) { return D == 128 ? (key & 15) : ((key >> 1) & 7); }
template <int D> __device__ __forceinline__ int pf_swz_v(int key) {
  return D == 128 ? ((key & 3) << 2) : (((key >> 1) & 1) << 2);
}
// L rows are dense (2, 4 or 8 chunks): as many consecutive rows as fill 256 bytes share a
// swizzle value, the next group takes the next one.
template <int LCH> __device__ __forceinline__ int pf_swz_l(int key) {
  return LCH == 2 ? ((key >> 3) & 1) : (LCH == 4 ? ((key >> 2) & 3) : ((key >> 1) & 7));
}


// Tile traffic of the prefill kernels: HBM -> LDS with no registers in between.
//
// A tile is 64 keys: K rows, V rows (d bf16 each) and L rows (RP bf16, dense).  A wave-wide
// load moves 1 KB: KROWS rows of K or V, LROWS rows of L.  Load i of a tile fills LDS rows
// i*ROWS ..; lane l lands at row i*ROWS + l/CH, physical chunk l%CH, and therefore fetches
// logical chunk (l%CH) ^ swizzle(row).  Wave w of the four issues loads i = w + 4q, for
// which the swizzle of its rows does not depend on q: one K, one V offset per lane.
// Rows past the sequence (and chunks past the rank) lie outside the resource: they read as
// zero and touch no memory; such keys are masked anyway.  A stage is laid out as
// [K tile][V tile][L tile].
template <int D, int RP, bool PAGED>
struct PfTileLoader {
  static constexpr int BN = 64;
  static constexpr int KCH = D / 8;              // 16-byte chunks per K/V row
  static constexpr int KROWS = 64 / KCH;         // K/V rows one wave-wide load moves (4 or 8)
  static constexpr int KV_DMA = BN / KROWS / 4;  // wave-wide loads per wave and K (or V) tile (4 or 2)
  static constexpr int LCH = RP / 8;             // 16-byte chunks per L row (2, 4 or 8)
  static constexpr int LROWS = 64 / LCH;         // L rows one wave-wide load moves (32, 16 or 8)
  static constexpr int L_DMA = (LCH + 3) / 4;    // the tile takes LCH loads; wave w issues i = w + 4q < LCH
  static constexpr int K_BYTES = BN * D * 2;

  const Params& p;
  const bf16_t *kb, *vb;
  pf_const_i32 bt;
  pf_u32x4 rs_k, rs_v, rs_l;
  uint32_t ts2, r2, lp2, lds0, k_voff, v_voff, l_voff[L_DMA];  // lp2: bytes between L rows
  int wave, lane, hk, n_t, nb_last;

  __device__ __forceinline__ PfTileLoader(const Params& p_, unsigned char* smem, int wave_, int lane_, int hk_, int t,
                                          int n_t_)
      : p(p_), wave(wave_), lane(lane_), hk(hk_), n_t(n_t_) {
    kb = static_cast<const bf16_t*>(p.k_base);
    vb = static_cast<const bf16_t*>(p.v_base);
    // the rows of the call's one adapter (BaseShared: its own low-rank cache), with their own stride
    const bf16_t* lr = static_cast<const bf16_t*>(p.l) + static_cast<int64_t>(p.adapter_index) * p.l_adapter_stride;
    bt = PF_CONST_I32(p.block_table) + static_cast<int64_t>(t) * p.max_blocks_per_seq;
    const int r = p.rank;
    ts2 = static_cast<uint32_t>(p.kv_token_stride) * 2u;
    r2 = static_cast<uint32_t>(r) * 2u;
    lp2 = static_cast<uint32_t>(p.l_row_stride) * 2u;
    lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(PF_LDS_AS(unsigned char, smem)));
    nb_last = (n_t - 1) >> 4;
    const int rr = lane / KCH, pc = lane % KCH;
    const int krow = wave * KROWS + rr;  // LDS row of load i = w (loads w + 4q: + 4q*KROWS, same swizzle)
    k_voff = static_cast<uint32_t>(rr) * ts2 + ((pc ^ pf_swz_k<D>(krow)) << 4);
    v_voff = static_cast<uint32_t>(rr) * ts2 + ((pc ^ pf_swz_v<D>(krow)) << 4);
    rs_k = rs_v = rs_l = pf_u32x4{0u, 0u, 0u, 0u};
#pragma unroll
    for (int q = 0; q < L_DMA; ++q) l_voff[q] = kPfOob;
    if (!PAGED) {
      const uint32_t kv_bytes = static_cast<uint32_t>(n_t - 1) * ts2 + D * 2;
      rs_k = pf_rsrc(kb + static_cast<int64_t>(hk) * p.kv_head_stride, kv_bytes);
      rs_v = pf_rsrc(vb + static_cast<int64_t>(hk) * p.kv_head_stride, kv_bytes);
      rs_l = pf_rsrc(lr, static_cast<uint32_t>(n_t - 1) * lp2 + r2);
#pragma unroll
      for (int q = 0; q < L_DMA; ++q) {
        const int lrow = (wave + 4 * q) * LROWS + lane / LCH;
        const int lch = (lane % LCH) ^ pf_swz_l<LCH>(lrow);
        l_voff[q] = (lch * 8 < r) ? static_cast<uint32_t>(lane / LCH) * lp2 + (lch << 4) : kPfOob;
      }
    } else {
      // paged L: one resource over the whole array; the lane's physical row is chosen per tile
      rs_l = pf_rsrc(lr, (static_cast<uint32_t>(p.num_blocks) * 16u - 1u) * lp2 + r2);
    }
  }

  // K and V loads number q (of KV_DMA) of this wave for the tile starting at key j
  __device__ __forceinline__ void issue_kv(int j, uint32_t stage_off, int q) const {
    const int i = wave + 4 * q;
    const uint32_t dst = lds0 + stage_off + i * 1024;
    if (!PAGED) {
      const uint32_t soff = static_cast<uint32_t>(j + i * KROWS) * ts2;
      pf_load16_to_lds(rs_k, dst, k_voff, soff);
      pf_load16_to_lds(rs_v, dst + K_BYTES, v_voff, soff);
    } else {
      // the KROWS rows of one load lie in one 16-token block
      const int tok = j + i * KROWS;
      const int blk = bt[min(tok >> 4, nb_last)];
      const int nv = max(0, min(KROWS, n_t - tok));  // rows of this load inside the sequence
      const uint32_t bytes = nv > 0 ? static_cast<uint32_t>(nv - 1) * ts2 + D * 2 : 0u;
      const int64_t off = static_cast<int64_t>(blk) * p.kv_block_stride + static_cast<int64_t>(hk) * p.kv_head_stride +
                          static_cast<int64_t>(tok & 15) * p.kv_token_stride;
      // completed keys left by the pre-pass lie at the block's logical index, with the strides of the pool
      const int64_t off_k = p.keys_f16 ? off + (static_cast<int64_t>(min(tok >> 4, nb_last)) - blk) * p.kv_block_stride : off;
      pf_load16_to_lds(pf_rsrc(kb + off_k, bytes), dst, k_voff, 0);
      pf_load16_to_lds(pf_rsrc(vb + off, bytes), dst + K_BYTES, v_voff, 0);
    }
  }

  __device__ __forceinline__ void issue_l(int j, uint32_t stage_off) const {
    const int r = p.rank;
#pragma unroll
    for (int q = 0; q < L_DMA; ++q) {
      const int i = wave + 4 * q;
      if (i < LCH) {
        const uint32_t dst = lds0 + stage_off + 2 * K_BYTES + i * 1024;
        if (!PAGED) {
          pf_load16_to_lds(rs_l, dst, l_voff[q], static_cast<uint32_t>(j + i * LROWS) * lp2);
        } else {
          // LROWS rows span at most two blocks; their ids are wave-uniform (scalar loads)
          const int tok0 = j + i * LROWS;
          const int blk_a = bt[min(tok0 >> 4, nb_last)];
          const int blk_b = bt[min((tok0 >> 4) + 1, nb_last)];
          const int lrow = i * LROWS + lane / LCH;
          const int tok = tok0 + lane / LCH;
          const int blk = ((tok >> 4) == (tok0 >> 4)) ? blk_a : blk_b;
          const int lch = (lane % LCH) ^ pf_swz_l<LCH>(lrow);
          const uint32_t voff = (tok < n_t && lch * 8 < r)
                                    ? (static_cast<uint32_t>(blk) * 16u + static_cast<uint32_t>(tok & 15)) * lp2 + (lch << 4)
                                    : kPfOob;
          pf_load16_to_lds(rs_l, dst, voff, 0);
        }
      }
    }
  }

  // this wave's share of the tile starting at key j, into the stage at byte offset stage_off
  __device__ __forceinline__ void issue_tile(int j, uint32_t stage_off) const {
#pragma unroll
    for (int q = 0; q < KV_DMA; ++q) issue_kv(j, stage_off, q);
    issue_l(j, stage_off);
  }
};

}  // namespace lra
