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
// every wave requests its quarter of the next tile straight from HBM into the
// other LDS stage (buffer_load ... lds, swizzled by choosing which chunk each lane
// fetches) at the top of the current tile; one wait and one barrier per tile.
// ds_read_b128 feeds the K operand, ds_read_b64_tr_b16 the transposed V and L
// operands, both scheduled several products ahead.  Two workgroups share a CU, so
// the softmax arithmetic of one overlaps the matrix work of the other.
// Workgroups are numbered so that all q heads of a kv head run on the same XCD and
// share its L2.
#include "lra_prefill_util.h"

namespace lra {

// HAS_BK = false is the value-only setting (b_k == NULL, keys fully shared): no Qt and no
// L term in the scores; L is still staged for P.L.
// SPLIT = true: the key tiles of a q tile are shared by gridDim.y workgroups; each leaves its
// softmax state (m, l, O, O_lr per row) in the workspace and the merge kernel combines
// them, applies B_V and normalises (for calls with too few q tiles to fill the chip).
// ROPE_K = true (with HAS_BK = false) is the rotary key side of App. D.1: the cached keys are
// rotated ones and the adapter's contribution has to be rotated by its key's position before
// the score, so it cannot ride on Qt.  Instead every key tile is completed in LDS before the
// scores are taken: E^T = B_K^T . L^T for the tile's 64 keys (two MFMAs per wave and 16
// ranks: a wave owns 32 keys and the two 32-feature blocks that hold the halves of its rotary
// pairs, so both halves of a pair sit in the same lane and register), rotated, and added to
// the K_base rows of the tile (8-byte read-modify-writes in bf16).  One more barrier per
// tile; the score loop is the value-only one.
template <int D, int RP, bool PAGED, bool HAS_BK, bool SPLIT, bool ROPE_K = false, bool KC16 = false>
__global__ __launch_bounds__(256, 2) void prefill_mfma_kernel(Params p) {
  static_assert(!(ROPE_K && HAS_BK), "the rotary key side replaces the Qt term");
  // Completed keys K_base + RoPE(L B_K) are held as fp16, whether the key pre-pass left them in the workspace
  // (KC16) or this kernel completes the tiles in LDS (ROPE_K): rounding the sum to bf16 a second time costs
  // 2.5e-3 to 4e-3 of relative error in the output on its own, fp16 (three more bits) a quarter of that.
  // The scores are then an fp16 product, with Q converted once in the prologue (exact for a bf16 Q of
  // ordinary magnitudes); V, L and the probabilities stay bf16.
  constexpr bool KF16 = ROPE_K || KC16;
  static_assert(!(KC16 && (HAS_BK || ROPE_K)), "pre-pass keys: nothing left to add");
  constexpr int BM = 128, BN = 64;
  constexpr int KS = D / 16;   // k-steps of S^T over the head dimension
  constexpr int RKS = RP / 16; // k-steps over the padded rank
  constexpr int DB = D / 32;   // 32-row blocks of O^T
  constexpr int RB = (RP + 31) / 32;  // 32-row blocks of Olr^T
  constexpr int KCH = D / 8;          // 16-byte chunks per K/V row
  constexpr int LCH = RP / 8;         // 16-byte chunks per L row (2, 4 or 8)
  constexpr int K_BYTES = BN * D * 2;
  constexpr int L_BYTES = BN * RP * 2;
  constexpr int STAGE = 2 * K_BYTES + L_BYTES;
  // With a half-empty last 32-row block of Olr^T (rank 16 or 48 after padding), its idle
  // upper lanes read a constant [1, 0, 0, 0] instead of L, so the matrix core also
  // accumulates the softmax row sums.
  constexpr bool ONES_ROW = (RP % 32) != 0;
  constexpr int ONES_AT = 2 * STAGE;

  __shared__ __align__(16) unsigned char smem[2 * STAGE + (ONES_ROW ? 16 : 0)];
  // rotary key side: revolutions per position of every rotary pair (double, and rounded to float for
  // the offsets inside a tile), and the angle of the first key of a tile (fraction of a revolution),
  // double-buffered like the stages
  __shared__ double rope_rate[ROPE_K ? D / 2 : 1];
  __shared__ __align__(16) float rope_rate_f[ROPE_K ? D / 2 : 4];
  __shared__ __align__(16) float rope_fr0[2][ROPE_K ? D / 2 : 4];

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
  int qt = rest / G;
  {
    // Causal q tiles differ in length (tile i walks the keys up to its diagonal).  The 256 compute units take
    // workgroups in rounds of 256; a unit that holds two workgroups holds number k and number k + 256.  Every other
    // round walks its q tiles backwards, so the long tiles of one round sit next to the short tiles of the next
    // and the units finish together.
    const int q_tiles = (p.n_new + BM - 1) / BM;
    const int tpr = max(1, 256 / Hq);              // q tiles per round
    const int round = qt / tpr, pos = qt - round * tpr;
    const int cnt = min(tpr, q_tiles - round * tpr);
    if ((round & 1)) qt = round * tpr + (cnt - 1 - pos);
  }
  const int t = p.seq_index;
  const int a_idx = p.adapter_index;
  const int n_t = min(PF_CONST_I32(p.seq_lens)[t], p.max_seq_len);
  const int n_new = p.n_new;
  const int q0 = qt * BM;
  if (q0 >= n_new) return;
  const int base_vis = n_t - n_new;  // new token i sees keys 0 .. base_vis + i
  const int row = q0 + wave * 32 + l32;           // this lane's query row (new-token index)
  const int n_live = n_new;                       // live rows of the tile
  const int row_c = min(row, n_live - 1);         // clamped for loads; rows past the end are never stored
  // token and q head of this lane's row: where its q, out and workspace rows are
  const int grow = row, grow_c = row_c;
  const int head = hk * G + gq;
  const int limit = base_vis + row_c;             // last visible key of this lane's row
  const int wg_last = base_vis + min(q0 + BM, n_new) - 1;  // last key any row of the workgroup sees
  const int n_tiles = wg_last / BN + 1;
  // this workgroup's share of the q tile's key tiles: [tile_begin, tile_end)
  const int split = SPLIT ? blockIdx.y : 0;
  const int tile_begin = SPLIT ? static_cast<int>(static_cast<int64_t>(n_tiles) * split / p.n_splits) : 0;
  const int tile_end = SPLIT ? static_cast<int>(static_cast<int64_t>(n_tiles) * (split + 1) / p.n_splits) : n_tiles;
  if (SPLIT && tile_begin >= tile_end) {
    // more workgroups than key tiles: leave an empty state (zero row sum), all the merge
    // kernel looks at
    if (row < n_live && g2 == 0) {
      const int64_t slot = (static_cast<int64_t>(grow) * Hq + head) * p.n_splits + split;
      p.part_ml[slot * 2 + 0] = -INFINITY;
      p.part_ml[slot * 2 + 1] = 0.f;
      if (split == 0) p.part_adapter[static_cast<int64_t>(grow) * Hq + head] = a_idx;
    }
    return;
  }

  // ---------------- tile traffic: HBM -> LDS, no registers in between ----------------
  const PfTileLoader<D, RP, PAGED> loader(p, smem, wave, lane, hk, t, n_t);
  auto issue_tile = [&](int j, int st) { loader.issue_tile(j, st * STAGE); };

  issue_tile(tile_begin * BN, 0);
  if (ONES_ROW && tid == 0) *reinterpret_cast<pf_u32x4*>(smem + ONES_AT) = pf_u32x4{0x00003f80u, 0u, 0u, 0u};

  // ---------------- rotary key side: B_K^T operands of E^T, rotation rates ----------------
  // Wave (pair set ps = wave / 2, key half kt_e = wave % 2); d = 128: feature blocks ps and ps + 2,
  // d = 64: blocks 0 and 1 (waves 2, 3 have nothing to do).  A operand of E^T = B_K^T . L^T: lane
  // (feature l32 of the block, half g2), element e <-> rho = 16ks + 8(e/4) + 4g2 + e%4, the order in
  // which the L operand is read below.
  constexpr int E_WAVES = ROPE_K ? 2 * (D / 64) : 0;
  const int fb_lo = D == 128 ? (wave >> 1) : 0, fb_hi = D == 128 ? (wave >> 1) + 2 : 1;
  const int kt_e = wave & 1;
  pf_bf16x8 bkt[2][ROPE_K ? RKS : 1];
  if (ROPE_K) {
    if (tid < D / 2) {  // read after the barrier that precedes the loop
      const double rate = rope_rate_rev(tid, D, p.key_rope_theta);
      rope_rate[tid] = rate;
      rope_rate_f[tid] = static_cast<float>(rate);
      double rev = static_cast<double>(tile_begin * BN) * rate;
      rev -= floor(rev);
      rope_fr0[0][tid] = static_cast<float>(rev);
    }
    if (wave < E_WAVES) {
      const int64_t ldb = static_cast<int64_t>(Hkv) * D;
      const bf16_t* bkg = static_cast<const bf16_t*>(p.b_k) + static_cast<int64_t>(a_idx) * r * ldb + hk * D;
      const bool has_b = p.b_k != nullptr;  // (a decode call may come without key-side adapters: nothing to add)
#pragma unroll
      for (int sel = 0; sel < 2; ++sel)
#pragma unroll
        for (int ks = 0; ks < RKS; ++ks) {
          uint32_t w4[4];
#pragma unroll
          for (int e2 = 0; e2 < 4; ++e2) {
            uint32_t pair = 0;
#pragma unroll
            for (int x = 0; x < 2; ++x) {
              const int e = 2 * e2 + x;
              const int rho = 16 * ks + 8 * (e >> 2) + 4 * g2 + (e & 3);
              const uint32_t v = (has_b && rho < r) ? bkg[rho * ldb + 32 * (sel == 0 ? fb_lo : fb_hi) + l32] : 0u;
              pair |= v << (16 * x);
            }
            w4[e2] = pair;
          }
          bkt[sel][ks] = pf_as_bf16x8(make_uint4(w4[0], w4[1], w4[2], w4[3]));
        }
    }
  }

  // ---------------- prologue: Q operands, Qt = Q B_K^T ----------------
  // qb[ks]: B operand of S^T: lane (row l32, k = 16ks + 8g2 + e)
  pf_bf16x8 qb[KS];
  {
    const bf16_t* qrow = static_cast<const bf16_t*>(p.q) + (static_cast<int64_t>(grow_c) * Hq + head) * D + g2 * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qb[ks] = pf_as_bf16x8(*reinterpret_cast<const uint4*>(qrow + ks * 16));
  }
  pf_f16x8 qh[KF16 ? KS : 1];  // the same operands as fp16, for scores against fp16 keys
  if constexpr (KF16) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qh[ks] = pf_bf16x8_to_f16x8(qb[ks]);
  }
  // Qt^T[rho][row] = B_K[rho][:] . Q[row][:]: C layout lane (row l32; reg i <-> rho = 32b + 8(i/4) + 4g2 + i%4).
  // As B operand of the rank k-steps of S^T, k-step ks' takes registers 8ks'..8ks'+7 of
  // block b = ks'/2, i.e. element e <-> rho = 16ks' + 8(e/4) + 4g2 + e%4; the L operand
  // below is read in the same order.
  pf_bf16x8 qtb[RKS];
  if (HAS_BK) {
    const int64_t ldb = static_cast<int64_t>(Hkv) * D;
    const bf16_t* bkg = static_cast<const bf16_t*>(p.b_k);
    // rows of this adapter's B_K for kv head hk; rows past the rank (and everything when
    // there is no B_K) lie outside the resource and read as zero
    const __amdgpu_buffer_rsrc_t rs_b = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t*>(bkg) + (bkg != nullptr ? static_cast<int64_t>(a_idx) * r * ldb + hk * D : 0), 0,
        bkg != nullptr ? static_cast<int>((static_cast<int64_t>(r - 1) * ldb + D) * 2) : 0, 0x00020000);
#pragma unroll
    for (int b = 0; b < RB; ++b) {
      pf_f32x16 acc;
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] = 0.f;
      const int rho = b * 32 + l32;
      const uint32_t boff = rho < r ? static_cast<uint32_t>(rho * ldb * 2 + g2 * 16) : kPfOob;
      pf_u32x4 bk[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) bk[ks] = __builtin_amdgcn_raw_buffer_load_b128(rs_b, boff, ks * 32, 0);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(pf_bf16x8, bk[ks]), qb[ks], acc, 0, 0, 0);
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

  // ---------------- per-lane LDS read offsets (stage 0; stage 1 is STAGE further) ----------------
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
  const int v_pre = K_BYTES + vrow * (D * 2) + ((((a16 & 3) >> 1) + 2 * dsel + pf_swz_v<D>(vrow)) << 4) + (a16 & 1) * 8;
  // L rows as A operand of S^T: two 8-byte pieces per k-step (chunks 2ks' and 2ks' + 1, half
  // g2); the swizzle of row 32kt + l32 does not depend on kt
  int l_rd[RKS][2];
#pragma unroll
  for (int ks = 0; ks < RKS; ++ks)
#pragma unroll
    for (int pc = 0; pc < 2; ++pc)
      l_rd[ks][pc] = 2 * K_BYTES + l32 * (RP * 2) + (((2 * ks + pc) ^ pf_swz_l<LCH>(l32)) << 4) + g2 * 8;
  // L^T as A operand of Olr^T: rows rho = 32b + 16dsel + 4(a%4) .. +3 of key vrow (+8 for the
  // second read; +16 per k-step does not change the swizzle).  In a half-empty last block
  // the upper 16 lanes read the constant [1, 0, 0, 0] instead: output row 32b + 16 then
  // accumulates the row sums; the rows after it are never used.
  int lt_rd[RB][2];
#pragma unroll
  for (int b = 0; b < RB; ++b)
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      const int key = vrow + 8 * hh;
      const int ch = 4 * b + 2 * dsel + ((a16 & 3) >> 1);
      lt_rd[b][hh] = 2 * K_BYTES + key * (RP * 2) + (((ch & (LCH - 1)) ^ pf_swz_l<LCH>(key)) << 4) + (a16 & 1) * 8;
    }
  const bool ones_lane = ONES_ROW && dsel == 1;  // in block RB - 1

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
  // The running maximum is only raised when some row's tile maximum exceeds it by more than
  // kSlack (base-2 units): until then probabilities up to 2^kSlack are accumulated, which
  // fp32 sums and bf16 probabilities hold without loss, and the final division by the row
  // sum (taken with the same reference) cancels the factor exactly.
  constexpr float kSlack = 8.0f;
  constexpr int kReadAheadS = 8, kReadAheadPV = 6;

  pf_wait_vm0();
  __syncthreads();

  auto tile_step = [&](int tile, auto st_c) {
    constexpr int ST = decltype(st_c)::value;
    const int j = tile * BN;
    const unsigned char* ks_l = smem + ST * STAGE;  // K region; the V and L offsets are part of v_pre, l_rd, lt_rd
    const bool more = tile + 1 < tile_end;
    // the other stage was last read before the barrier that ended the previous tile; where
    // in the tile the requests are placed makes no measurable difference
    if (more) issue_tile(j + BN, ST ^ 1);

    if (ROPE_K) {
      if (wave < E_WAVES) {
        pf_f32x16 e_lo, e_hi;
#pragma unroll
        for (int i = 0; i < 16; ++i) e_lo[i] = e_hi[i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < RKS; ++ks) {
          const uint2 lo = *reinterpret_cast<const uint2*>(ks_l + l_rd[ks][0] + kt_e * 32 * RP * 2);
          const uint2 hi = *reinterpret_cast<const uint2*>(ks_l + l_rd[ks][1] + kt_e * 32 * RP * 2);
          const pf_bf16x8 lop = pf_as_bf16x8(make_uint4(lo.x, lo.y, hi.x, hi.y));
          e_lo = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bkt[0][ks], lop, e_lo, 0, 0, 0);
          e_hi = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bkt[1][ks], lop, e_hi, 0, 0, 0);
        }
        // register i of this lane: key 32 kt_e + l32 of the tile (position j + that), features
        // 32 fb + 8 (i/4) + 4 g2 + i%4 of blocks fb_lo, fb_hi: pair index = the fb_lo feature
        // Angle of (key, pair) in revolutions: that of the tile's first key, kept in double precision
        // by the table threads, plus the key's offset in the tile times the rate (at most 63 x 0.16
        // revolutions: single precision holds it to 1e-6).
        const int key = 32 * kt_e + l32;
        const float key_f = static_cast<float>(key);
        unsigned char* krow = smem + ST * STAGE + key * (D * 2) + 8 * g2;
        const int swz = pf_swz_k<D>(key);
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int dd0 = 32 * fb_lo + 8 * q4 + 4 * g2;
          const pf_f32x4 fr0 = *reinterpret_cast<const pf_f32x4*>(&rope_fr0[ST][dd0]);
          const pf_f32x4 rt = *reinterpret_cast<const pf_f32x4*>(&rope_rate_f[dd0]);
          float lo4[4], hi4[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int i = 4 * q4 + e;
            const float fr = fmaf(key_f, rt[e], fr0[e]);
            const float sn = __builtin_amdgcn_sinf(fr), cs = __builtin_amdgcn_cosf(fr);
            lo4[e] = e_lo[i] * cs - e_hi[i] * sn;
            hi4[e] = e_hi[i] * cs + e_lo[i] * sn;
          }
#pragma unroll
          for (int sel = 0; sel < 2; ++sel) {
            const float* add = sel == 0 ? lo4 : hi4;
            uint2* at = reinterpret_cast<uint2*>(krow + (((4 * (sel == 0 ? fb_lo : fb_hi) + q4) ^ swz) << 4));
            const uint2 old = *at;
            *at = make_uint2(pf_pack2_f16(__uint_as_float(old.x << 16) + add[0], __uint_as_float(old.x & 0xffff0000u) + add[1]),
                             pf_pack2_f16(__uint_as_float(old.y << 16) + add[2], __uint_as_float(old.y & 0xffff0000u) + add[3]));
          }
        }
      }
      __syncthreads();  // the completed keys are visible to the score loop of every wave
      if (more && tid < D / 2) {  // the next tile's first angle, for the expansion after the barrier that ends this tile
        double rev = static_cast<double>(j + BN) * rope_rate[tid];
        rev -= floor(rev);
        rope_fr0[ST ^ 1][tid] = static_cast<float>(rev);
      }
    }

    // S^T for the two 32-key halves of the tile.  The halves alternate, so consecutive
    // matrix instructions never wait for each other's result, and the LDS reads run
    // kReadAheadS operands ahead of the products that consume them.
    pf_f32x16 s[2];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int i = 0; i < 16; ++i) s[kt][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        const uint4 a4 = *reinterpret_cast<const uint4*>(ks_l + (k_pre ^ ((2 * ks + g2) << 4)) + kt * 32 * D * 2);
        if constexpr (KF16)
          s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(pf_f16x8, a4), qh[ks], s[kt], 0, 0, 0);
        else
          s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf_as_bf16x8(a4), qb[ks], s[kt], 0, 0, 0);
      }
    if (HAS_BK) {
#pragma unroll
      for (int ks = 0; ks < RKS; ++ks)
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
          const uint2 lo = *reinterpret_cast<const uint2*>(ks_l + l_rd[ks][0] + kt * 32 * RP * 2);
          const uint2 hi = *reinterpret_cast<const uint2*>(ks_l + l_rd[ks][1] + kt * 32 * RP * 2);
          s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf_as_bf16x8(make_uint4(lo.x, lo.y, hi.x, hi.y)), qtb[ks],
                                                          s[kt], 0, 0, 0);
        }
    }
    // instruction order for the scheduler: kReadAheadS LDS reads, then one product per read
    __builtin_amdgcn_sched_group_barrier(0x100, kReadAheadS, 0);
#pragma unroll
    for (int i = 0; i < 2 * KS; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    if (HAS_BK) {
#pragma unroll
      for (int i = 0; i < 2 * RKS; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      }
    }
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
    if (__builtin_amdgcn_ballot_w64(mx > m_run + kSlack) != 0) {  // always on the first tile (m_run = -inf)
      const float m_new = fmaxf(m_run, mx);
      // a share that does not start at key 0 may hold rows that have seen nothing yet
      const float alpha = (SPLIT && m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(m_run - m_new);
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int b = 0; b < DB; ++b) o_acc[b] *= alpha;
#pragma unroll
      for (int b = 0; b < RB; ++b) lr_acc[b] *= alpha;
    }
    // finite from the first tile on (key 0 is visible to every row) unless the share starts later
    const float nm = (SPLIT && m_run == -INFINITY) ? 0.f : -m_run;
    pf_bf16x8 pb[2][2];       // [kt][16-key k-step]
    auto exp_half = [&](int kt) __attribute__((always_inline)) {
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
    };
    // The exponentials of the second 32-key half run under the products of the first: a matrix instruction
    // occupies its pipe for 32 cycles, and the wave is free to issue vector work meanwhile.
    exp_half(0);
    __builtin_amdgcn_sched_barrier(0);
    exp_half(1);
    // O^T += V^T P^T ; Olr^T += L^T P^T, one 16-key k-step at a time.
    // k-step (kt, h2), element e <-> key 32kt + 16h2 + 8(e/4) + 4g2 + e%4.
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        const int rowoff = (32 * kt + 16 * h2) * (D * 2);
#pragma unroll
        for (int b = 0; b < DB; ++b) {
          const unsigned char* src = ks_l + (v_pre ^ (b << 6)) + rowoff;
          const pf_bf16x8 a = pf_join(pf_read_tr16(src), pf_read_tr16(src + 8 * (D * 2)));
          o_acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[kt][h2], o_acc[b], 0, 0, 0);
        }
#pragma unroll
        for (int b = 0; b < RB; ++b) {
          const int koff = (32 * kt + 16 * h2) * (RP * 2);
          const unsigned char* src0 = ks_l + lt_rd[b][0] + koff;
          const unsigned char* src1 = ks_l + lt_rd[b][1] + koff;
          if (ONES_ROW && b == RB - 1) {
            src0 = ones_lane ? smem + ONES_AT : src0;
            src1 = ones_lane ? smem + ONES_AT : src1;
          }
          const pf_bf16x8 a = pf_join(pf_read_tr16(src0), pf_read_tr16(src1));
          lr_acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[kt][h2], lr_acc[b], 0, 0, 0);
        }
      }
    // the transposed reads (two per operand) run kReadAheadPV operands ahead
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * kReadAheadPV, 0);
#pragma unroll
    for (int i = 0; i < 2 * (DB + RB); ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, ONES_ROW ? 3 : 5, 0);
    }
#pragma unroll
    for (int i = 0; i < 2 * (DB + RB); ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    }
    // the next tile has landed (this wave's share) and everybody is done reading this one
    pf_wait_vm0();
    __syncthreads();
  };
  for (int tile = tile_begin; tile < tile_end; tile += 2) {
    tile_step(tile, std::integral_constant<int, 0>{});
    if (tile + 1 < tile_end) tile_step(tile + 1, std::integral_constant<int, 1>{});
  }

  // ---------------- epilogue: O^T += B_V^T Olr^T, O /= l, store ----------------
  if (ONES_ROW) {
    // row sums sit in register 8 (rho = 32(RB-1) + 16) of the lanes with g2 == 0
    const float mine = lr_acc[RB - 1][8];
    const float other = pf_partner32(mine);
    l_run = g2 == 0 ? mine : other;
  } else {
    l_run += pf_partner32(l_run);
  }
  if (SPLIT) {
    // this share's state for the merge kernel: m in natural-log units, l, O^T and Olr^T as
    // fp32 rows [slot][d] and [slot][rank]; registers 4q..4q+3 are d (rho) = 32b + 8q + 4g2 + 0..3
    if (row < n_live) {
      const int64_t slot = (static_cast<int64_t>(grow) * Hq + head) * p.n_splits + split;
      if (g2 == 0) {
        p.part_ml[slot * 2 + 0] = m_run * 0.69314718055994530942f;
        p.part_ml[slot * 2 + 1] = l_run;
        if (split == 0) p.part_adapter[static_cast<int64_t>(grow) * Hq + head] = a_idx;
      }
#pragma unroll
      for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int q = 0; q < 4; ++q)
          *reinterpret_cast<pf_f32x4*>(p.part_o + slot * D + 32 * b + 8 * q + 4 * g2) =
              pf_f32x4{o_acc[b][4 * q + 0], o_acc[b][4 * q + 1], o_acc[b][4 * q + 2], o_acc[b][4 * q + 3]};
#pragma unroll
      for (int b = 0; b < RB; ++b)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int rho = 32 * b + 8 * q + 4 * g2;  // the rank is a multiple of 8: all four or none
          if (rho < r)
            *reinterpret_cast<pf_f32x4*>(p.part_lr + slot * r + rho) =
                pf_f32x4{lr_acc[b][4 * q + 0], lr_acc[b][4 * q + 1], lr_acc[b][4 * q + 2], lr_acc[b][4 * q + 3]};
        }
    }
    return;
  }
  if (p.b_v != nullptr) {
    const int64_t ldb = static_cast<int64_t>(Hkv) * D;
    const bf16_t* bv = static_cast<const bf16_t*>(p.b_v) + static_cast<int64_t>(a_idx) * r * ldb + hk * D;
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
  if (row < n_live) {
    const float inv = 1.0f / l_run;
    bf16_t* orow = static_cast<bf16_t*>(p.out) + (static_cast<int64_t>(grow) * Hq + head) * D;
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

template <int D, int RP, bool SPLIT>
static hipError_t launch_pf2(const Params& p, dim3 grid, hipStream_t s) {
  const bool paged = p.block_size != 0, has_bk = p.b_k != nullptr;
  if (has_bk && p.key_rope_theta > 0.f) {
    if (paged) hipLaunchKernelGGL((prefill_mfma_kernel<D, RP, true, false, SPLIT, true>), grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL((prefill_mfma_kernel<D, RP, false, false, SPLIT, true>), grid, dim3(256), 0, s, p);
    return hipGetLastError();
  }
  if (p.keys_f16) {  // (set by the host only where the pre-pass has completed the keys)
    if (has_bk) return hipErrorInvalidValue;
    if (paged) hipLaunchKernelGGL((prefill_mfma_kernel<D, RP, true, false, SPLIT, false, true>), grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL((prefill_mfma_kernel<D, RP, false, false, SPLIT, false, true>), grid, dim3(256), 0, s, p);
    return hipGetLastError();
  }
  if (paged && has_bk)
    hipLaunchKernelGGL((prefill_mfma_kernel<D, RP, true, true, SPLIT>), grid, dim3(256), 0, s, p);
  else if (paged)
    hipLaunchKernelGGL((prefill_mfma_kernel<D, RP, true, false, SPLIT>), grid, dim3(256), 0, s, p);
  else if (has_bk)
    hipLaunchKernelGGL((prefill_mfma_kernel<D, RP, false, true, SPLIT>), grid, dim3(256), 0, s, p);
  else
    hipLaunchKernelGGL((prefill_mfma_kernel<D, RP, false, false, SPLIT>), grid, dim3(256), 0, s, p);
  return hipGetLastError();
}

template <int D, int RP>
static hipError_t launch_pf(const Params& p, dim3 grid, hipStream_t s) {
  return p.n_splits > 1 ? launch_pf2<D, RP, true>(p, grid, s) : launch_pf2<D, RP, false>(p, grid, s);
}

hipError_t launch_prefill_mfma(const Params& p, hipStream_t s) {
  const int q_tiles = (p.n_new + 127) / 128;
  dim3 grid(q_tiles * p.n_q_heads, p.n_splits);
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

// ---------------------------------------------------------------------------------------
// Rotary key side, contiguous caches: the keys of the call's one adapter, formed once.
//   K_j = K_base,j + RoPE_j(L_j B_K^a)             (App. D.1: with LoRA on the key projection the
//                                                   adapter's part is rebuilt in the head dimension
//                                                   before the rotation)
// The tile-walking kernel can complete every key tile in LDS itself, but a call of many q tiles
// then repeats that work in every workgroup that walks the tile (q tiles x q heads of the kv head:
// 64 times at 2048 new tokens and a group of 4).  This pre-pass writes the completed keys of all
// visible tokens into the workspace, in the layout of K_base (same strides), and the call then
// runs the plain kernel without a key-side adapter on them.  HBM bound: K_base read and written
// once (+ L); rank x d multiply-adds per key and head on the vector ALU.
// One workgroup per (16 keys, kv head); lane (key, group g of 16): the pairs (dd, dd + d/2),
// dd = PPL g .. PPL g + PPL - 1, PPL = d/32.  E in fp32, angle = fractional part of position x rate
// in double precision, as in the producer of the caches.
// ---------------------------------------------------------------------------------------
template <int D, bool PAGED>
__global__ __launch_bounds__(256) void complete_rope_keys_kernel(Params p, unsigned short* kc) {
  constexpr int PPL = D / 32;              // rotary pairs per lane
  __shared__ __align__(16) unsigned short b_lds[64 * D];  // B_K^a rows of this kv head, [rho][d]
  __shared__ double rate[D / 2];
  const int tid = threadIdx.x;
  const int h = blockIdx.y;
  const int r = p.rank;
  const int n_t = min(PF_CONST_I32(p.seq_lens)[p.seq_index], p.max_seq_len);
  const int j = blockIdx.x * 16 + (tid >> 4);
  if (blockIdx.x * 16 >= n_t) return;
  const int a = min(max(p.adapter_index, 0), p.n_adapters - 1);
  const unsigned short* bk = static_cast<const unsigned short*>(p.b_k) +
                             (static_cast<int64_t>(a) * r * p.n_kv_heads + h) * D;
  for (int i = tid; i < r * (D / 8); i += 256) {
    const int rho = i / (D / 8), c = i - rho * (D / 8);
    *reinterpret_cast<uint4*>(b_lds + rho * D + c * 8) =
        *reinterpret_cast<const uint4*>(bk + static_cast<int64_t>(rho) * p.n_kv_heads * D + c * 8);
  }
  if (tid < D / 2) rate[tid] = rope_rate_rev(tid, D, p.key_rope_theta);
  __syncthreads();
  if (j >= n_t) return;
  const int g = tid & 15;
  // paged: the key's block comes from the sequence's row of the block table; the completed keys are written at
  // the block's LOGICAL index (the kernel that reads them needs no table for them)
  const int blk = PAGED ? PF_CONST_I32(p.block_table)[static_cast<int64_t>(p.seq_index) * p.max_blocks_per_seq + (j >> 4)] : 0;
  const int64_t l_index = PAGED ? static_cast<int64_t>(blk) * 16 + (j & 15) : j;
  const unsigned short* lrow = static_cast<const unsigned short*>(p.l) + static_cast<int64_t>(a) * p.l_adapter_stride +
                               l_index * p.l_row_stride;
  float lo[PPL], hi[PPL];
#pragma unroll
  for (int i = 0; i < PPL; ++i) lo[i] = hi[i] = 0.f;
  for (int r0 = 0; r0 < r; r0 += 8) {  // the rank is a multiple of 8
    const uint4 lv = *reinterpret_cast<const uint4*>(lrow + r0);
    const uint32_t lw[4] = {lv.x, lv.y, lv.z, lv.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float lf = __uint_as_float((e & 1) ? (lw[e >> 1] & 0xffff0000u) : (lw[e >> 1] << 16));
      const unsigned short* brow = b_lds + (r0 + e) * D + PPL * g;
#pragma unroll
      for (int i = 0; i < PPL; ++i) {
        lo[i] = fmaf(lf, __uint_as_float(static_cast<uint32_t>(brow[i]) << 16), lo[i]);
        hi[i] = fmaf(lf, __uint_as_float(static_cast<uint32_t>(brow[D / 2 + i]) << 16), hi[i]);
      }
    }
  }
  const int64_t in_blk = static_cast<int64_t>(PAGED ? (j & 15) : j) * p.kv_token_stride + static_cast<int64_t>(h) * p.kv_head_stride + PPL * g;
  const int64_t off_src = in_blk + (PAGED ? static_cast<int64_t>(blk) * p.kv_block_stride : 0);
  const int64_t off_dst = in_blk + (PAGED ? static_cast<int64_t>(j >> 4) * p.kv_block_stride : 0);
  // the lane's PPL consecutive features of either half: one 8-byte (d = 128) or 4-byte (d = 64) piece
  struct alignas(PPL * 2) Piece { unsigned short v[PPL]; };
  const unsigned short* ksrc = static_cast<const unsigned short*>(p.k_base) + off_src;
  unsigned short* kdst = kc + off_dst;
  const Piece klo = *reinterpret_cast<const Piece*>(ksrc), khi = *reinterpret_cast<const Piece*>(ksrc + D / 2);
  Piece olo, ohi;
#pragma unroll
  for (int i = 0; i < PPL; ++i) {
    float sn, cs;
    rope_sincos(rate[PPL * g + i], j, sn, cs);
    // (as fp16: see prefill_mfma_kernel)
    olo.v[i] = __builtin_bit_cast(unsigned short, static_cast<_Float16>(__uint_as_float(static_cast<uint32_t>(klo.v[i]) << 16) + (lo[i] * cs - hi[i] * sn)));
    ohi.v[i] = __builtin_bit_cast(unsigned short, static_cast<_Float16>(__uint_as_float(static_cast<uint32_t>(khi.v[i]) << 16) + (hi[i] * cs + lo[i] * sn)));
  }
  *reinterpret_cast<Piece*>(kdst) = olo;
  *reinterpret_cast<Piece*>(kdst + D / 2) = ohi;
}

hipError_t launch_complete_rope_keys(const Params& p, void* kc, hipStream_t s) {
  const dim3 grid((p.max_seq_len + 15) / 16, p.n_kv_heads);
  unsigned short* dst = static_cast<unsigned short*>(kc);
  if (p.block_size != 0) {
    if (p.head_dim == 128) hipLaunchKernelGGL((complete_rope_keys_kernel<128, true>), grid, dim3(256), 0, s, p, dst);
    else hipLaunchKernelGGL((complete_rope_keys_kernel<64, true>), grid, dim3(256), 0, s, p, dst);
  } else {
    if (p.head_dim == 128) hipLaunchKernelGGL((complete_rope_keys_kernel<128, false>), grid, dim3(256), 0, s, p, dst);
    else hipLaunchKernelGGL((complete_rope_keys_kernel<64, false>), grid, dim3(256), 0, s, p, dst);
  }
  return hipGetLastError();
}

}  // namespace lra
