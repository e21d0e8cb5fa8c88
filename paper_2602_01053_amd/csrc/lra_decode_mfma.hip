// MFMA decode kernel of the Flash-LoRA-Attention library (bf16, gfx950).
//
// One workgroup streams one range of keys of one (sequence, kv head) for ALL
// query rows that share that stream: every agent decoding on the sequence times
// the q heads of the GQA group.  Those rows form the 16-wide N dimension of
// v_mfma_f32_16x16x32_bf16, so K_base, V_base and L are read from HBM once for
// all agents (LRAgent Sec. 3.2: one base cache and one LR cache for the system).
//
// Per 32-key step (the inner loop of Alg. 1 with the App. D.1 key-side reordering):
//   S^T[key][row]  = K_base[key][:] . Q[row][:]  +  L[key][:] . Qt[row][:]     (MFMA)
//   online softmax along keys (per row = per lane column)
//   O^T[d][row]   += V_base^T[d][key] . P^T[key][row]                          (MFMA)
//   Olr^T[p][row] += L^T[p][key]      . P^T[key][row]                          (MFMA)
// with Qt = Q B_K^T computed once per workgroup in the prologue (MFMA, shared
// through LDS).  Computing S transposed makes the C-layout of the score tile
// coincide with the B-operand layout of the second product, so P never moves
// between lanes.
//
// Data path: buffer_load ... lds (16 bytes per lane, straight from HBM into
// wave-private LDS, no staging registers; K_base and V_base non-temporal, since
// nobody reads them twice, L cached for the workgroups of the other kv heads).  Each lane fetches the 16-byte chunk
// that belongs at ITS LDS slot under an XOR swizzle, so the later ds_read_b128
// (K operand), ds_read_b64 (L operand) and ds_read_b64_tr_b16 (transposed V and
// L operands) avoid bank conflicts.  Keys past the end of a wave's range are
// outside the buffer resource: the hardware returns zeros for them and touches
// no memory, so there is no tail branch on the load side.  A wave holds one
// tile; latency is hidden by the eight waves a CU holds, not by a software
// pipeline inside the wave.  The waves of a workgroup own disjoint key ranges
// and never synchronise inside the loop; their states are merged through LDS at
// the end (flash-decoding rule) and one partial (m, l, O, O_lr) per workgroup
// goes to the workspace.
#include "lra_common.h"
#include "lra_decode_util.h"
#include "lra_plan.h"
#include "lra_prefill_util.h"

namespace lra {

// Agent slots per tile of the rotary form at ranks above 32: that kernel has a CU to itself
// (its LDS leaves no room for a second workgroup), hence 512 registers per wave.
constexpr int kRopeSlots64 = 4;

// HAS_BK = false is the value-only setting (b_k == NULL, keys fully shared): no Qt, no
// adapter lookup on the key side, no L term in the scores; L is still streamed for P.L.
// CAUSAL = true serves lra_attn_prefill with a handful of new tokens: the new tokens of the
// one sequence take the place of the agents (same adapter for all), and row i only sees the
// keys up to n - n_new + i (the mask of Alg. 1); a long context is then split over the whole chip
// like any decode call instead of being walked by one workgroup per q head.
//
// RPE > 0 is the rotary key side, K_j = K_base,j + RoPE_j(L_j B_K) (what App. D.1 leaves to the
// key cache because the rotation stands between L_j and B_K): the L.Qt term of the scores is
// replaced, per 16-key tile and agent slot, by
//   E^T[f][key]   = B_K^T[f][:] . L^T[:][key]                 (MFMA, C layout: lane = key)
//   rotate the pairs (f, f + D/2) of E^T by the key's angle   (registers, sine/cosine shared by the slots)
//   S^T[key][row] += rot(E)[key][f] . Q[row][f]                (MFMA; the C layout of E^T is the
//                                                              A layout of this product)
// with Q masked to the rows of the slot.  The B_K^T operands of NS agent slots stay in
// registers (RPE = padded rank of that product: 16, 32 or 64, for 4, 2 or 4 slots per tile - at
// 64 the LDS leaves room for one workgroup per CU only, whose waves then have 512 registers);
// in the causal form all rows belong to the one adapter of the call.
//
// PA = true is the decode form for one low-rank cache per adapter (BaseShared, Sec. 3.2) outside the rotary key
// side: the L tile is a row of column blocks [agent slot][32 keys][l_block ranks], block s requested from the cache
// of the adapter of agent slot s; Qt of a row stands in the block of its slot and is zero elsewhere, so the same
// products give Qt_a . L_a^T and P . L_a per agent, and a row keeps only its own block of O_lr.  K_base and V_base are
// then read once for all agents of a tile, and no zero padding is streamed.
// RGI = false leaves out the grid layout for several row groups (below).  The rotary forms sit at the edge of their
// register file, and the few instructions of that layout at the top of the kernel were enough to move their
// allocation (config 2 with the rotary key side: 21.9 -> 23.3 us per call): they are built both ways and take the
// layout only when a call has several row groups.
template <int D, int RT, int RP, bool PAGED, bool HAS_BK, bool CAUSAL, int RPE = 0, bool PA = false, bool RGI = true>
__global__ __launch_bounds__(256, RPE == 64 ? 1 : 2) void decode_mfma_kernel(Params p) {
  constexpr int NW = 4;
  constexpr bool ROPE = RPE > 0;
  static_assert(!PA || (!ROPE && !CAUSAL && RT == 1), "per-adapter low-rank caches: plain decode form, one row tile");
  constexpr int NS = !ROPE ? 1 : (RPE == 16 ? 4 : (RPE == 32 ? 2 : kRopeSlots64));  // agent slots with operands in registers
  constexpr int EK = RPE == 64 ? 2 : 1;                                    // 32-wide k-steps of the E product
  static_assert(!ROPE || (RT == 1 && HAS_BK && (RPE == 64) == (RP == 64)), "rotary form: one row tile");
  constexpr int NSL = CAUSAL ? 1 : NS;  // the causal form has one adapter for all rows: one slot
  constexpr int KS = D / 32;       // MFMA k-steps over the head dimension
  constexpr int RKS = RP / 32;     // MFMA k-steps over the (padded) rank
  constexpr int DB = D / 16;       // 16-wide output blocks over d
  constexpr int RB = RP / 16;      // 16-wide output blocks over the rank
  constexpr int KCH = D / 8;       // 16-byte chunks per K/V row
  constexpr int RCH = RP / 8;      // 16-byte chunks per L row in LDS
  constexpr int KROWS = 64 / KCH;  // K/V rows one wave-wide load moves
  constexpr int KVL = 32 / KROWS;  // wave-wide loads per 32-key K (or V) tile
  constexpr int LROWS = 64 / RCH;
  constexpr int LL = 32 / LROWS;
  constexpr int KV_BYTES = 32 * D * 2;
  constexpr int L_BYTES = 32 * RP * 2;
  constexpr int WAVE_BYTES = 2 * KV_BYTES + L_BYTES;
  constexpr int NACC = RT * (DB + RB) * 4 + RT;
  constexpr int MERGE_SLOT = NACC * 64 * 4;
  constexpr int STAGE_TOTAL = NW * WAVE_BYTES;
  constexpr int MERGE_TOTAL = (NW / 2) * MERGE_SLOT;
  constexpr int SMEM = STAGE_TOTAL > MERGE_TOTAL ? STAGE_TOTAL : MERGE_TOTAL;
  constexpr int LSW_SHIFT = (RP == 32) ? 1 : 0;
  constexpr int QT_BYTES = RT * RKS * 1024;
  constexpr int M_BYTES = NW * RT * 16 * 4;
  // Two workgroups per CU need 2 * LDS <= 160 KB.  Where the tile regions alone
  // leave no room, the Qt exchange area and the per-wave maxima live inside the
  // tile regions and the first tile is requested only after the prologue.
  constexpr int ROPE_FLOATS = ROPE ? NW * 128 : 4;  // per wave: 64 rates, 64 phases of the current step
  constexpr bool ALIAS = 2 * (SMEM + QT_BYTES + M_BYTES + (ROPE ? ROPE_FLOATS * 4 : 0)) > 160 * 1024;
  constexpr int EXTRA = ALIAS ? 16 : QT_BYTES + M_BYTES;
  static_assert(QT_BYTES <= WAVE_BYTES && RT * 64 <= WAVE_BYTES, "aliased areas must fit one wave's region");

  __shared__ __align__(16) unsigned char smem[SMEM];
  __shared__ __align__(16) unsigned char extra_lds[EXTRA];
  __shared__ __align__(16) float rope_tab[ROPE_FLOATS];
  unsigned char* qt_lds = ALIAS ? smem : extra_lds;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ln = lane & 15, lg = lane >> 4;
  LRA_STAMP_DECL;
  LRA_STAMP(0);
  // kv head is the fastest grid index: workgroups go round-robin over the XCDs, so with 8 kv
  // heads all workgroups of a head run on one XCD and share Q and B_K in its L2
  const int h = blockIdx.x;
  int split = blockIdx.y;
  int t = CAUSAL ? p.seq_index : blockIdx.z / p.row_groups;
  int rg = CAUSAL ? blockIdx.z : blockIdx.z - t * p.row_groups;
  if constexpr (RGI) if (p.rg_interleave > 0) {
    // Several row groups share the keys of a (sequence, kv head, key share): only the first to ask reads them from
    // HBM if the others ask the same L2 soon after.  Workgroups go round-robin over the 8 XCDs in the order of
    // their linear index x + Hkv * y, so with m = lcm(8, Hkv) / Hkv and y = (share mod m) + m * (row group +
    // row_groups * (share / m)) the row groups of a share are lcm(8, Hkv) workgroups apart: the same XCD, the next
    // round of the dispatcher.  (Key shares are padded to a multiple of m; z is the sequence.)
    const int m = p.rg_interleave, y = blockIdx.y;
    const int hi = y >> __builtin_ctz(m);
    const int q = hi / p.row_groups;
    rg = hi - q * p.row_groups;
    split = (y & (m - 1)) + m * q;
    t = CAUSAL ? p.seq_index : blockIdx.z;
    if (split >= p.n_splits) return;
  }
  // The first and the last entry of seq_query_start are fixed by the contract (0 and
  // n_queries): a single sequence needs no table read at all, and the adapter ids can be
  // requested at once instead of one memory round trip later.
  const int32_t len_t = CONST_I32(p.seq_lens)[t];
  int q_begin = 0, q_end = CAUSAL ? p.n_new : p.n_queries;
  if (!CAUSAL) {
    if (t > 0) q_begin = CONST_I32(p.seq_query_start)[t];
    if (t + 1 < p.n_seqs) q_end = CONST_I32(p.seq_query_start)[t + 1];
  }
  const int n_t = min(len_t, p.max_seq_len);
  const int j0 = split * p.split_keys;
  const int n_q = q_end - q_begin;
  const int GP = p.group_pad, G = p.group, r = p.rank;
  const int row0 = rg * RT * 16;
  if (row0 >= n_q * GP) return;
  asm volatile("" ::"s"(n_t));
  LRA_STAMP(1);
  // workspace slot of the row this lane stands for in row tile rt (-1: padding row)
  auto row_slot = [&](int rt) -> int64_t {
    const int R = row0 + rt * 16 + ln;
    const int slot_q = R / GP, gg = R - slot_q * GP;
    if (!(slot_q < n_q && gg < G)) return -1;
    return (static_cast<int64_t>(q_begin + slot_q) * p.n_q_heads + h * G + gg) * p.n_splits + split;
  };
  if (j0 >= n_t) {
    // a split past the end of this sequence: leave an empty state (zero row sum), which is
    // all the merge kernel looks at; the O and O_lr rows of the slot stay unwritten
    if (wave == 0 && lg == 0) {
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        const int64_t slot = row_slot(rt);
        if (slot >= 0) {
          p.part_ml[slot * 2 + 0] = -INFINITY;
          p.part_ml[slot * 2 + 1] = 0.f;
        }
      }
    }
    return;
  }
  // The merge kernel takes each row's adapter from the workspace: the workgroups of split 0
  // copy it there (requested now, stored with the state at the end).
  int my_adapter[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int R = row0 + rt * 16 + ln;
    const int slot_q = min(R / GP, n_q - 1);
    my_adapter[rt] = CAUSAL ? p.adapter_index : (split == 0 ? p.query_adapter[q_begin + slot_q] : 0);
  }
  // last key each of this lane's rows may see (causal form only)
  int lim[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) lim[rt] = n_t - n_q + min((row0 + rt * 16 + ln) / GP, n_q - 1);
  const int lim_first = n_t - n_q + row0 / GP;  // the smallest of them in this workgroup

  // adapter of every agent slot of every row tile: wave-uniform loads, requested before
  // anything else so that the B_K rows they select can follow one round trip earlier
  // (only in the one-row-tile kernels: in the two-tile ones the extra registers and the wait
  // cost the streaming kernel more than the merge kernel gains)
  const bool warm_bv = RT == 1 && p.b_v != nullptr && split == min(1, p.n_splits - 1);
  int a_slot[RT][4];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int si = 0; si < 4; ++si) {
      const int slot = (row0 + rt * 16) / GP + si;
      if (CAUSAL)
        a_slot[rt][si] = (si < 16 / GP && slot < n_q) ? p.adapter_index : -1;
      else
        a_slot[rt][si] = ((HAS_BK || warm_bv || p.l_adapter_stride > 0) && si < 16 / GP && slot < n_q)
                             ? min(max(CONST_I32(p.query_adapter)[q_begin + slot], 0), p.n_adapters - 1)  // device data: kept inside the table
                             : -1;
    }
  const int j1 = min(j0 + p.split_keys, n_t);
  const int kpw = p.split_keys / NW;  // multiple of 32
  const int jw0 = j0 + wave * kpw;
  const int jw1 = max(jw0, min(jw0 + kpw, j1));  // == jw0 for a wave without keys

  unsigned char* ks_lds = smem + wave * WAVE_BYTES;
  unsigned char* vs_lds = ks_lds + KV_BYTES;
  unsigned char* ls_lds = vs_lds + KV_BYTES;

  const bf16_t* kb = static_cast<const bf16_t*>(p.k_base);
  const bf16_t* vb = static_cast<const bf16_t*>(p.v_base);
  // Low-rank rows: dense, or with a pitch of their own; with one low-rank cache per adapter the host gives every
  // agent a row tile (and this kernel one row tile per workgroup), so the tile's first slot names the cache
  const int64_t lp = p.l_row_stride;
  const bf16_t* lr = static_cast<const bf16_t*>(p.l) +
                     (!PA && p.l_adapter_stride > 0 ? static_cast<int64_t>(max(a_slot[0][0], 0)) * p.l_adapter_stride : 0);
  // PA: ranks per column block (16, 32 or 64), 16-byte chunks per row of a block, bytes per row of a block; the
  // XOR swizzle of the chunk index inside a block row (none for 32-byte rows: 16 rows fill two clocks densely).
  // Without PA the tile is one block of RP ranks and all of this folds to the constants of that layout.
  const int lb = PA ? p.l_block : RP;
  const int lcpr = lb >> 3, lcs = __builtin_ctz(lcpr), lb2 = lb * 2;
  auto swz_l = [&](int row) { return lcpr == 8 ? (row & 7) : (lcpr == 4 ? ((row >> 1) & 3) : 0); };
  const int gps = __builtin_ctz(GP);  // GP is 4, 8 or 16
  const uint32_t ts2 = static_cast<uint32_t>(p.kv_token_stride) * 2u;  // token stride in bytes
  const uint32_t r2 = static_cast<uint32_t>(r) * 2u;                     // L row in bytes
  const uint32_t lp2 = static_cast<uint32_t>(lp) * 2u;                   // bytes between L rows

  // ===================== per-lane constants of the tile traffic =====================
  // The LDS of this chip serves 256 bytes per clock (64 banks): a ds_read_b128 is free of
  // conflicts when 16 consecutive lanes hit 16 different 16-byte positions of that window,
  // a ds_read_b64_tr_b16 when the eight 32-byte pieces of 32 consecutive lanes do.  Rows of
  // 256 bytes (d = 128) all start at position 0, rows of 128 bytes alternate halves; the XOR
  // swizzles below (on the 16-byte chunk index of a row) spread them accordingly:
  //   K (b128, 16 rows per clock)      chunk ^ (row & 15)            | chunk ^ ((row >> 1) & 7)
  //   V (tr_b64, 8 rows per clock)     chunk ^ ((row & 7) << 1)      | chunk ^ (((row >> 1) & 3) << 1)
  auto swz_k = [](int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); };
  auto swz_v = [](int row) { return D == 128 ? ((row & 7) << 1) : (((row >> 1) & 3) << 1); };
  // global -> LDS: lane l of load i lands at LDS row i*ROWS + l/CH, physical chunk l%CH,
  // and therefore fetches logical chunk (l%CH) ^ swizzle(row).  The swizzle of row
  // i*ROWS + l/CH repeats with period 16/KROWS (K) and 8/KROWS (V) in i.
  constexpr int KPER = KROWS == 4 ? 4 : 2, VPER = KROWS == 4 ? 2 : 1;
  uint32_t k_voff[KPER], v_voff[VPER], l_voff;
  uint32_t l_in_row = 0;  // PA: byte offset of the lane's chunk inside an L row
  bool l_ok = true;       // PA: that chunk lies inside the rank
  {
    const int rr = lane / KCH, pc = lane % KCH;
#pragma unroll
    for (int q = 0; q < KPER; ++q) k_voff[q] = static_cast<uint32_t>(rr) * ts2 + ((pc ^ swz_k(q * KROWS + rr)) << 4);
#pragma unroll
    for (int q = 0; q < VPER; ++q) v_voff[q] = static_cast<uint32_t>(rr) * ts2 + ((pc ^ swz_v(q * KROWS + rr)) << 4);
    if constexpr (PA) {
      // lane -> (row inside a request, chunk of the block row): the swizzle repeats from request to request
      const int lrow = lane >> lcs, lpc = lane & (lcpr - 1);
      const int lch = lpc ^ swz_l(lrow);
      l_ok = lch * 8 < r;
      l_in_row = static_cast<uint32_t>(lch) << 4;
      l_voff = l_ok ? static_cast<uint32_t>(lrow) * lp2 + l_in_row : kOob;
    } else {
      const int lrow = lane / RCH, lpc = lane % RCH;
      const int lch = lpc ^ ((lrow >> LSW_SHIFT) & (RCH - 1));
      l_voff = (lch * 8 < r) ? static_cast<uint32_t>(lrow) * lp2 + (lch << 4) : kOob;
    }
  }
  // LDS -> MFMA operands (byte offsets inside the tile regions).
  // K rows as A operand of S^T: key = 16tt + ln, logical chunk 4ks + lg at chunk ^ swz_k(key):
  // row offset, swizzle and lg sit in disjoint address bits, so the address is
  // k_pre ^ (ks << 6) + tt * 16 rows.
  const int k_pre = ln * (2 * D) + ((swz_k(ln) ^ lg) << 4);
  // V^T as A operand of O^T: this lane addresses row ka (+16tt) of the tile, logical chunk
  // 2b + c0 (+ half sub): address v_pre ^ (b << 5) + tt * 16 rows.
  const int ka = 4 * lg + (ln >> 2);  // row (within a 16-key tile) this lane addresses in transpose reads
  const int v_pre = ka * (2 * D) + ((swz_v(ka) + ((ln & 3) >> 1)) << 4) + (ln & 1) * 8;
  int l_rd[RKS][2];  // L rows as A operand of S^T: two 8-byte pieces per k-step
  int lt_rd[RB];     // L^T as A operand of Olr^T
  if constexpr (PA) {
    // column chunk ch of the tile (8 ranks) lies in block ch / lcpr, chunk ch % lcpr of a row there
    auto chunk_addr = [&](int ch, int row) {
      const int blk = ch >> lcs, cc = ch & (lcpr - 1);
      return blk * (32 * lb2) + row * lb2 + ((cc ^ swz_l(row)) << 4);
    };
#pragma unroll
    for (int ks = 0; ks < RKS; ++ks)
#pragma unroll
      for (int pc = 0; pc < 2; ++pc) l_rd[ks][pc] = chunk_addr(4 * ks + 2 * pc + (lg >> 1), ln) + (lg & 1) * 8;
#pragma unroll
    for (int b = 0; b < RB; ++b) lt_rd[b] = chunk_addr(2 * b + ((ln & 3) >> 1), ka) + (ln & 1) * 8;
  } else {
    const int swz_s = (ln >> LSW_SHIFT) & (RCH - 1);
#pragma unroll
    for (int ks = 0; ks < RKS; ++ks)
#pragma unroll
      for (int pc = 0; pc < 2; ++pc) {
        const int ch = 4 * ks + 2 * pc + (lg >> 1);
        l_rd[ks][pc] = ln * (2 * RP) + ((ch ^ swz_s) << 4) + (lg & 1) * 8;
      }
    const int swz_t = (ka >> LSW_SHIFT) & (RCH - 1);
#pragma unroll
    for (int b = 0; b < RB; ++b) {
      const int ch = 2 * b + ((ln & 3) >> 1);
      lt_rd[b] = ka * (2 * RP) + ((ch ^ swz_t) << 4) + (ln & 1) * 8;
    }
  }

  // Contiguous cache: one resource per wave covering exactly its keys [jw0, jw1).
  u32x4 rs_k = {0u, 0u, 0u, 0u}, rs_v = rs_k, rs_l = rs_k;
  if (!PAGED) {
    const int nk = jw1 - jw0;
    const int64_t base = static_cast<int64_t>(h) * p.kv_head_stride + static_cast<int64_t>(jw0) * p.kv_token_stride;
    const uint32_t bytes = nk > 0 ? static_cast<uint32_t>(nk - 1) * ts2 + D * 2 : 0u;
    rs_k = make_rsrc_words(kb + base, bytes);
    rs_v = make_rsrc_words(vb + base, bytes);
    rs_l = make_rsrc_words(lr + static_cast<int64_t>(jw0) * lp, nk > 0 ? static_cast<uint32_t>(nk - 1) * lp2 + r2 : 0u);
  }
  // PA: one L resource per request of 1 KB - the requests of a column block read the cache of that block's agent
  // slot (a block beyond the tile's slots, or of an empty slot, reads nothing).  Contiguous cache: the rows of the
  // wave's keys, as above.  Paged cache: the adapter's whole pool (the host has checked that it fits 32-bit byte
  // offsets); a lane then addresses its row through the physical block and masks the keys past the wave's range itself.
  constexpr int LREQ = PA ? LL : 1;
  u32x4 rs_la[LREQ];
  uint32_t l_row0[LREQ];  // first tile row of the request
  if constexpr (PA) {
    const int rows_per_req = 64 >> lcs;  // 1 KB of rows of lb ranks
    const int rpb_shift = lcs - 1;       // lb/16 requests per block
    const int nk = jw1 - jw0;
    const uint32_t bytes = PAGED ? (static_cast<uint32_t>(p.num_blocks) * 16u - 1u) * lp2 + r2
                                 : (nk > 0 ? static_cast<uint32_t>(nk - 1) * lp2 + r2 : 0u);
#pragma unroll
    for (int i = 0; i < LL; ++i) {
      const int blk = i >> rpb_shift, qq = i - (blk << rpb_shift);
      const int a = blk == 0 ? a_slot[0][0] : (blk == 1 ? a_slot[0][1] : (blk == 2 ? a_slot[0][2] : a_slot[0][3]));
      const bool live = blk < (16 >> gps) && a >= 0;
      rs_la[i] = make_rsrc_words(static_cast<const bf16_t*>(p.l) + static_cast<int64_t>(live ? a : 0) * p.l_adapter_stride +
                                     (PAGED ? 0 : static_cast<int64_t>(jw0) * lp),
                                 live ? bytes : 0u);
      l_row0[i] = static_cast<uint32_t>(qq * rows_per_req);
    }
  }
  const const_i32_ptr bt = CONST_I32(p.block_table) + static_cast<int64_t>(t) * p.max_blocks_per_seq;

  // Paged cache: the two physical block ids of a step are fetched one step ahead (scalar
  // loads), so the table lookup is off the path that requests the tile.
  int blk_next[2] = {0, 0};
  auto fetch_block_ids = [&](int j) {
    if (PAGED) {
      const int nb_last = (n_t - 1) >> 4;
      blk_next[0] = bt[min(j >> 4, nb_last)];
      blk_next[1] = bt[min((j >> 4) + 1, nb_last)];
    }
  };
  fetch_block_ids(jw0);

  // K_base / V_base requests: non-temporal when this workgroup is the only reader of its keys; with
  // several row groups per (sequence, kv head) the others find the tiles in L2
  const bool stream_kv = p.row_groups == 1;
  auto kv_load = [&](u32x4 rs, unsigned char* lds, uint32_t voff, uint32_t soff) __attribute__((always_inline)) {
    if (stream_kv) buf_load16_to_lds<true>(rs, lds, voff, soff);
    else buf_load16_to_lds<false>(rs, lds, voff, soff);
  };
  // ---- HBM -> LDS for the 32-key step starting at token j ----
  auto issue_tile = [&](int j) {
    if (PAGED) {
      const int64_t hoff = static_cast<int64_t>(h) * p.kv_head_stride;
      const int blk_cur[2] = {blk_next[0], blk_next[1]};
      fetch_block_ids(j + 32);
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int jb = j + 16 * half;
        const int blk = blk_cur[half];
        const int nv = max(0, min(16, jw1 - jb));  // slots of this block inside the wave's range
        const uint32_t kv_bytes = nv > 0 ? static_cast<uint32_t>(nv - 1) * ts2 + D * 2 : 0u;
        const u32x4 pk = make_rsrc_words(kb + static_cast<int64_t>(blk) * p.kv_block_stride + hoff, kv_bytes);
        const u32x4 pv = make_rsrc_words(vb + static_cast<int64_t>(blk) * p.kv_block_stride + hoff, kv_bytes);
        const u32x4 pl = make_rsrc_words(lr + static_cast<int64_t>(blk) * 16 * lp, nv > 0 ? static_cast<uint32_t>(nv - 1) * lp2 + r2 : 0u);
#pragma unroll
        for (int i = 0; i < KVL / 2; ++i) {
          const int ii = half * (KVL / 2) + i;
          kv_load(pk, ks_lds + ii * 1024, k_voff[ii % KPER], i * KROWS * ts2);
          kv_load(pv, vs_lds + ii * 1024, v_voff[ii % VPER], i * KROWS * ts2);
        }
        if constexpr (!PA) {
#pragma unroll
          for (int i = 0; i < LL / 2; ++i) {
            const int ii = half * (LL / 2) + i;
            buf_load16_to_lds(pl, ls_lds + ii * 1024, l_voff, i * LROWS * lp2);
          }
        }
      }
      if constexpr (PA) {
        // tile row of this lane in request i: l_row0[i] + lane / lcpr; its physical block is the first or the
        // second of the step; rows at or past the end of the wave's range read nothing (zeros)
        const uint32_t lrow = static_cast<uint32_t>(lane >> lcs);
        const uint32_t pg0 = static_cast<uint32_t>(blk_cur[0]) * 16u * lp2, pg1 = static_cast<uint32_t>(blk_cur[1]) * 16u * lp2;
#pragma unroll
        for (int i = 0; i < LL; ++i) {
          const uint32_t row = l_row0[i] + lrow;
          const bool ok = l_ok && j + static_cast<int>(row) < jw1;
          const uint32_t voff = ok ? (row < 16u ? pg0 : pg1) + (row & 15u) * lp2 + l_in_row : kOob;
          buf_load16_to_lds(rs_la[i], ls_lds + i * 1024, voff, 0u);
        }
      }
    } else {
      const uint32_t s0 = static_cast<uint32_t>(j - jw0);
#pragma unroll
      for (int i = 0; i < KVL; ++i) {
        kv_load(rs_k, ks_lds + i * 1024, k_voff[i % KPER], (s0 + i * KROWS) * ts2);
        kv_load(rs_v, vs_lds + i * 1024, v_voff[i % VPER], (s0 + i * KROWS) * ts2);
      }
      if constexpr (PA) {
#pragma unroll
        for (int i = 0; i < LL; ++i) buf_load16_to_lds(rs_la[i], ls_lds + i * 1024, l_voff, (s0 + l_row0[i]) * lp2);
      } else {
#pragma unroll
        for (int i = 0; i < LL; ++i) buf_load16_to_lds(rs_l, ls_lds + i * 1024, l_voff, (s0 + i * LROWS) * lp2);
      }
    }
  };

  // The first tile is on its way before the prologue touches Q and B_K.
  if (!ROPE && (!ALIAS || !HAS_BK) && jw0 < jw1) issue_tile(jw0);
  LRA_STAMP(2);

  // ===================== prologue: Q operands and Qt = Q B_K^T =====================
  // qb[rt][ks]: lane (row ln of tile rt, k = 32ks + 8lg + e), e = 0..7.  Used as the
  // B operand of S^T and as the B operand of Qt^T = B_K Q^T below.
  bf16x8 qb[RT][KS];
  // rotary form: the same rows once more in the order the rotated E^T blocks come out of
  // their product: qp[fb] = Q[row ln][16fb + 4lg + 0..3]
  s16x4 qp[ROPE ? DB : 1];
  {
    const __amdgpu_buffer_rsrc_t rs_q =
        make_rsrc(static_cast<const bf16_t*>(p.q) + static_cast<int64_t>(q_begin) * p.n_q_heads * D,
                  static_cast<uint32_t>(n_q) * p.n_q_heads * D * 2);
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const int R = row0 + rt * 16 + ln;
      const int slot = R / GP, gg = R - slot * GP;
      const bool valid = slot < n_q && gg < G;
      const uint32_t off = valid ? static_cast<uint32_t>((slot * p.n_q_heads + h * G + gg) * D * 2 + lg * 16) : kOob;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) qb[rt][ks] = as_bf16x8(buf_load16(rs_q, off, ks * 64));
      if constexpr (ROPE) {
        const uint32_t offp = valid ? off - lg * 8 : kOob;
#pragma unroll
        for (int fb = 0; fb < DB; ++fb)
          qp[fb] = __builtin_bit_cast(s16x4, __builtin_amdgcn_raw_buffer_load_b64(rs_q, offp, fb * 32, 0));
      }
    }
  }
  // Qt^T block (rho block cb, tile rt) = B_K^a[16cb..16cb+15][:] . Q_tile^T : C layout
  // lane (rho = 16cb + 4lg + j, row ln).  Rows of a tile belong to 16/GP agents; each
  // agent's product is kept only in its own rows (lanes).  The items are spread over
  // the waves and exchanged through LDS in operand-ready form: operand (rt, ks') of
  // lane l is the 16 bytes at ((rt*RKS + ks')*64 + l)*16, elements
  // e -> rho = 32ks' + 16(e/4) + 4lg + e%4.  The L operand below uses the same order.
  bf16x8 qtb[RT][RKS];
  // ===================== rotary form: B_K^T operands and rotation rates =====================
  using e_op = typename std::conditional<RPE == 16, s16x4, bf16x8>::type;
  e_op bkt[NSL][ROPE ? DB : 1][EK];
  float* rope_w = rope_tab + (ROPE ? wave * 128 : 0);
  double rate_d = 0.0;
  if constexpr (ROPE) {
    // The slices B_K[a][:, h*D .. h*D+D) of the tile's agents go through this wave's K and V
    // regions in the layout of a V tile (rows = rank index) and come back transposed, which is
    // the A operand of E^T.  Rows beyond the rank, and the slices of empty slots, are outside
    // the resource and arrive as zeros.
    const int64_t ldb = static_cast<int64_t>(p.n_kv_heads) * D;
    const uint32_t ldb2 = static_cast<uint32_t>(ldb) * 2u;
    constexpr int SLOT_BYTES = RPE * D * 2;
    constexpr int SPP = NSL * SLOT_BYTES <= 2 * KV_BYTES ? NSL : 2 * KV_BYTES / SLOT_BYTES;  // slots per pass through the regions
    static_assert(SPP >= 1 && NSL % SPP == 0, "a slice must fit the K and V regions");
    uint32_t bk_voff[VPER];
    {
      const int rr = lane / KCH, pc = lane % KCH;
#pragma unroll
      for (int q = 0; q < VPER; ++q) bk_voff[q] = static_cast<uint32_t>(rr) * ldb2 + ((pc ^ swz_v(q * KROWS + rr)) << 4);
    }
    const bf16_t* bkg = static_cast<const bf16_t*>(p.b_k);
    rate_d = rope_rate_rev(lane & (D / 2 - 1), D, p.key_rope_theta);
    rope_w[lane] = static_cast<float>(rate_d);
#pragma unroll
    for (int s0 = 0; s0 < NSL; s0 += SPP) {
#pragma unroll
      for (int sp = 0; sp < SPP; ++sp) {
        const int a = min(a_slot[0][s0 + sp], p.n_adapters - 1);
        const uint32_t bytes = a >= 0 ? static_cast<uint32_t>((r - 1) * ldb + D) * 2u : 0u;
        const u32x4 rs_b = make_rsrc_words(bkg + static_cast<int64_t>(a >= 0 ? a : 0) * r * ldb + h * D, bytes);
#pragma unroll
        for (int i = 0; i < RPE / KROWS; ++i)
          buf_load16_to_lds(rs_b, ks_lds + sp * SLOT_BYTES + i * 1024, bk_voff[i % VPER], i * KROWS * ldb2);
      }
      wait_vm0();
      lds_fence();
#pragma unroll
      for (int sp = 0; sp < SPP; ++sp)
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
          for (int ek = 0; ek < EK; ++ek) {
            const unsigned char* src = ks_lds + sp * SLOT_BYTES + ek * (64 * D) + (v_pre ^ (b << 5));
            if constexpr (RPE == 16)
              bkt[s0 + sp][b][ek] = lds_read_tr16(src);
            else
              bkt[s0 + sp][b][ek] = join_tr(lds_read_tr16(src), lds_read_tr16(src + 32 * D));
          }
      __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the regions are about to be written again
      lds_fence();
    }
    if (jw0 < jw1) issue_tile(jw0);
  }
  if (HAS_BK && !ROPE) {
    if constexpr (PA) {
      // every piece of the exchange area starts as zero: blocks beyond a slot's rank, the other slots' blocks
      if (wave < RT * RKS) *reinterpret_cast<uint4*>(qt_lds + (wave * 64 + lane) * 16) = make_uint4(0u, 0u, 0u, 0u);
      static_assert(!PA || RT * RKS <= NW, "one piece per wave");
      __syncthreads();
    }
    const int S = 16 / GP;         // agent slots per 16-row tile
    const int ncb = (r + 15) >> 4;
    const int64_t ldb = static_cast<int64_t>(p.n_kv_heads) * D;
    const bf16_t* bkg = static_cast<const bf16_t*>(p.b_k);
    constexpr int MAXIT = 4;  // at most 4 slots x 4 rho blocks per tile over 4 waves
    const int n_items = S * ncb;
    // every B_K tile of this wave's items is requested before the first product starts
    uint4 bt4[RT][MAXIT][KS];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int it = 0; it < MAXIT; ++it) {
        const int idx = wave + it * NW;
        const int si = idx / ncb, cb = idx - si * ncb;
        const int a = si == 0 ? a_slot[rt][0] : (si == 1 ? a_slot[rt][1] : (si == 2 ? a_slot[rt][2] : a_slot[rt][3]));
        const bool live = idx < n_items && a >= 0;
        const uint32_t bytes = live ? static_cast<uint32_t>((r - 1) * ldb + D) * 2u : 0u;
        const __amdgpu_buffer_rsrc_t rs_b = make_rsrc(bkg + static_cast<int64_t>(live ? a : 0) * r * ldb + h * D, bytes);
        const uint32_t off = static_cast<uint32_t>((cb * 16 + ln) * ldb * 2 + lg * 16);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) bt4[rt][it][ks] = buf_load16(rs_b, off, ks * 64);
      }
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int it = 0; it < MAXIT; ++it) {
        const int idx = wave + it * NW;
        if (idx < n_items) {
          const int si = idx / ncb, cb = idx - si * ncb;
          f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < KS; ++ks)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(bt4[rt][it][ks]), qb[rt][ks], acc, 0, 0, 0);
          if (ln / GP == si) {
            const int kb = PA ? si * (lb >> 4) + cb : cb;  // 16-rank block along the L tile's columns
            unsigned char* dst = qt_lds + ((rt * RKS + (kb >> 1)) * 64 + lane) * 16;
            const uint2 pk = make_uint2(pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3]));
            if constexpr (PA)
              *reinterpret_cast<uint2*>(dst + (kb & 1) * 8) = pk;
            else if (!(cb & 1) && cb + 1 >= ncb)  // the odd block next to it lies beyond the rank: zeros
              *reinterpret_cast<uint4*>(dst) = make_uint4(pk.x, pk.y, 0u, 0u);
            else
              *reinterpret_cast<uint2*>(dst + (cb & 1) * 8) = pk;
          }
        }
      }
    __syncthreads();
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int ks = 0; ks < RKS; ++ks) {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);  // k-steps entirely beyond the rank were never written
        if (PA || ks * 32 < r) v = lds_read16(qt_lds + ((rt * RKS + ks) * 64 + lane) * 16);
        qtb[rt][ks] = as_bf16x8(v);
      }
  }
  if (ALIAS && HAS_BK && !ROPE) {
    __syncthreads();  // the exchange area is about to be overwritten by tiles
    if (jw0 < jw1) issue_tile(jw0);
  }

  LRA_STAMP(3);
  // ===================== main loop =====================
  f32x4 o_acc[RT][DB], lr_acc[RT][RB];
  float m_run[RT], l_run[RT];  // m_run in base-2 units of the scaled score
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    m_run[rt] = -INFINITY;
    l_run[rt] = 0.f;
#pragma unroll
    for (int b = 0; b < DB; ++b) o_acc[rt][b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int b = 0; b < RB; ++b) lr_acc[rt][b] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  const float sc = p.scale * 1.44269504088896340736f;

  for (int j = jw0; j < jw1; j += 32) {
    // the tile requested one step earlier (or before the prologue) has landed
    wait_vm0();
    lds_fence();
    if (j == jw0) LRA_STAMP(4);
    f32x4 s[2][RT];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) s[tt][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 a = as_bf16x8(lds_read16(ks_lds + (k_pre ^ (ks << 6)) + tt * 32 * D));
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
          s[tt][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qb[rt][ks], s[tt][rt], 0, 0, 0);
      }
      if (HAS_BK && !ROPE) {
#pragma unroll
        for (int ks = 0; ks < RKS; ++ks) {
          const uint2 lo = lds_read8(ls_lds + l_rd[ks][0] + tt * 16 * lb2);  // (16 rows of a block further)
          const uint2 hi = lds_read8(ls_lds + l_rd[ks][1] + tt * 16 * lb2);
          const bf16x8 a = as_bf16x8(make_uint4(lo.x, lo.y, hi.x, hi.y));
#pragma unroll
          for (int rt = 0; rt < RT; ++rt)
            s[tt][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qtb[rt][ks], s[tt][rt], 0, 0, 0);
        }
      }
    }
    if constexpr (ROPE) {
      // phase (in revolutions) of every rotary pair at position j: lane = pair, in double so
      // that positions in the tens of thousands lose nothing; the lanes below add the key's
      // own offset in single precision
      {
        double rev = static_cast<double>(j) * rate_d;
        rev -= floor(rev);
        rope_w[64 + lane] = static_cast<float>(rev);
      }
      e_op lop[2][EK];  // L^T as B operand of E^T: the register contents of the L operand of S^T
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int ek = 0; ek < EK; ++ek) {
          const uint2 lo = lds_read8(ls_lds + l_rd[ek][0] + tt * 32 * RP);
          if constexpr (RPE == 16) {
            lop[tt][ek] = __builtin_bit_cast(s16x4, lo);
          } else {
            const uint2 hi = lds_read8(ls_lds + l_rd[ek][1] + tt * 32 * RP);
            lop[tt][ek] = as_bf16x8(make_uint4(lo.x, lo.y, hi.x, hi.y));
          }
        }
      const int n_slots = CAUSAL ? 1 : 16 / GP;
      const int my_slot = CAUSAL ? 0 : ln / GP;
      const float keyf[2] = {static_cast<float>(ln), static_cast<float>(16 + ln)};
#pragma unroll
      for (int fbl = 0; fbl < DB / 2; ++fbl) {
        const f32x4 rt4 = *reinterpret_cast<const f32x4*>(rope_w + 16 * fbl + 4 * lg);
        const f32x4 f04 = *reinterpret_cast<const f32x4*>(rope_w + 64 + 16 * fbl + 4 * lg);
        float cs[2][4], sn[2][4];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            const float fr = fmaf(keyf[tt], rt4[jj], f04[jj]);
            sn[tt][jj] = __builtin_amdgcn_sinf(fr);
            cs[tt][jj] = __builtin_amdgcn_cosf(fr);
          }
#pragma unroll
        for (int si = 0; si < NSL; ++si) {
          if (si >= n_slots) continue;
          const bool mine = my_slot == si;
          const s16x4 zero4 = {0, 0, 0, 0};
          const s16x4 q_lo = mine ? qp[fbl] : zero4;
          const s16x4 q_hi = mine ? qp[fbl + DB / 2] : zero4;
#pragma unroll
          for (int tt = 0; tt < 2; ++tt) {
            f32x4 e_lo = {0.f, 0.f, 0.f, 0.f}, e_hi = e_lo;
            if constexpr (RPE == 16) {
              e_lo = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(bkt[si][fbl][0], lop[tt][0], e_lo, 0, 0, 0);
              e_hi = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(bkt[si][fbl + DB / 2][0], lop[tt][0], e_hi, 0, 0, 0);
            } else {
#pragma unroll
              for (int ek = 0; ek < EK; ++ek) {
                e_lo = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bkt[si][fbl][ek], lop[tt][ek], e_lo, 0, 0, 0);
                e_hi = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bkt[si][fbl + DB / 2][ek], lop[tt][ek], e_hi, 0, 0, 0);
              }
            }
            float r_lo[4], r_hi[4];
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
              r_lo[jj] = e_lo[jj] * cs[tt][jj] - e_hi[jj] * sn[tt][jj];
              r_hi[jj] = e_hi[jj] * cs[tt][jj] + e_lo[jj] * sn[tt][jj];
            }
            const s16x4 a_lo = __builtin_bit_cast(s16x4, make_uint2(pack_bf16x2(r_lo[0], r_lo[1]), pack_bf16x2(r_lo[2], r_lo[3])));
            const s16x4 a_hi = __builtin_bit_cast(s16x4, make_uint2(pack_bf16x2(r_hi[0], r_hi[1]), pack_bf16x2(r_hi[2], r_hi[3])));
            s[tt][0] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_lo, q_lo, s[tt][0], 0, 0, 0);
            s[tt][0] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_hi, q_hi, s[tt][0], 0, 0, 0);
          }
        }
      }
    }
    // online softmax; element (tt, jj) of this lane is key j + 16tt + 4lg + jj of row ln
    const bool tail = j + 32 > jw1 || (CAUSAL && j + 31 > lim_first);
    bf16x8 pb[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      if (tail) {
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            const int key = j + tt * 16 + lg * 4 + jj;
            if (key >= jw1 || (CAUSAL && key > lim[rt])) s[tt][rt][jj] = -INFINITY;
          }
      }
      float mx = fmaxf(fmaxf(fmaxf(s[0][rt][0], s[0][rt][1]), fmaxf(s[0][rt][2], s[0][rt][3])),
                       fmaxf(fmaxf(s[1][rt][0], s[1][rt][1]), fmaxf(s[1][rt][2], s[1][rt][3])));
      mx = max_over_lane_groups(mx) * sc;  // sc > 0
      if (__builtin_amdgcn_ballot_w64(mx > m_run[rt]) != 0) {
        const float m_new = fmaxf(m_run[rt], mx);
        // causal form: a row may have seen no key yet (both maxima -inf)
        const float alpha = (CAUSAL && m_new == -INFINITY) ? 1.f : fast_exp2(m_run[rt] - m_new);
        m_run[rt] = m_new;
        l_run[rt] *= alpha;
#pragma unroll
        for (int b = 0; b < DB; ++b) o_acc[rt][b] *= alpha;
#pragma unroll
        for (int b = 0; b < RB; ++b) lr_acc[rt][b] *= alpha;
      }
      const float nm = (CAUSAL && m_run[rt] == -INFINITY) ? 0.f : -m_run[rt];
      float pe[8];
      float sum = 0.f;
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const float e = fast_exp2(fmaf(s[tt][rt][jj], sc, nm));
          pe[tt * 4 + jj] = e;
          sum += e;
        }
      l_run[rt] += sum;
      pb[rt] = as_bf16x8(make_uint4(pack_bf16x2(pe[0], pe[1]), pack_bf16x2(pe[2], pe[3]), pack_bf16x2(pe[4], pe[5]),
                                    pack_bf16x2(pe[6], pe[7])));
    }
    // O^T += V^T P^T ; Olr^T += L^T P^T
#pragma unroll
    for (int b = 0; b < DB; ++b) {
      const unsigned char* src = vs_lds + (v_pre ^ (b << 5));
      const bf16x8 a = join_tr(lds_read_tr16(src), lds_read_tr16(src + 32 * D));
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
        o_acc[rt][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pb[rt], o_acc[rt][b], 0, 0, 0);
    }
#pragma unroll
    for (int b = 0; b < RB; ++b) {
      const unsigned char* src = ls_lds + lt_rd[b];
      const bf16x8 a = join_tr(lds_read_tr16(src), lds_read_tr16(src + 16 * lb2));
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
        lr_acc[rt][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pb[rt], lr_acc[rt][b], 0, 0, 0);
    }
    // the next tile overwrites this one: every LDS read above must have returned
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
    lds_fence();
    if (j == jw0) LRA_STAMP(5);
    if (j + 32 < jw1) issue_tile(j + 32);
  }
  LRA_STAMP(6);

  // One workgroup per (sequence, kv head, row group) touches the B_V rows the merge kernel
  // will need (one 4-byte read per 128-byte line) once its keys are done, so that they wait
  // in this XCD's L2 instead of in HBM: wave w takes agent slot w of every row tile.  The
  // values are only looked at by an empty statement at the very end.
  int warm[RT][2];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    warm[rt][0] = warm[rt][1] = 0;
    const int a = wave == 0 ? a_slot[rt][0] : (wave == 1 ? a_slot[rt][1] : (wave == 2 ? a_slot[rt][2] : a_slot[rt][3]));
    if (warm_bv && a >= 0) {
      constexpr int LPR = D * 2 / 128;  // 128-byte lines per B_V row of one kv head
      const int n_lines = r * LPR;      // <= 128
      const char* bv = static_cast<const char*>(p.b_v) +
                       (static_cast<int64_t>(a) * r * p.n_kv_heads * D + static_cast<int64_t>(h) * D) * 2;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int li = i * 64 + lane;
        if (li < n_lines)
          warm[rt][i] = *reinterpret_cast<const int*>(bv + static_cast<int64_t>(li / LPR) * p.n_kv_heads * D * 2 + (li % LPR) * 128);
      }
    }
  }

  // ===================== merge the waves of this workgroup =====================
  // per-wave maxima: in a wave's own tile region when aliased (nobody else touches it
  // before the barrier), else in their own area
  float* m_mine = reinterpret_cast<float*>(ALIAS ? smem + wave * WAVE_BYTES : extra_lds + QT_BYTES + wave * RT * 64);
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    l_run[rt] = sum_over_lane_groups(l_run[rt]);
    if (lg == 0) m_mine[rt * 16 + ln] = m_run[rt];
  }
  __syncthreads();
  float m_all[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    float mm = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float* m_w = reinterpret_cast<const float*>(ALIAS ? smem + w * WAVE_BYTES : extra_lds + QT_BYTES + w * RT * 64);
      mm = fmaxf(mm, m_w[rt * 16 + ln]);
    }
    m_all[rt] = mm;  // finite (wave 0 always owns a key) unless a causal row sees none of this split
    const float wgt = (CAUSAL && mm == -INFINITY) ? 0.f : fast_exp2(m_run[rt] - mm);
    l_run[rt] *= wgt;
#pragma unroll
    for (int b = 0; b < DB; ++b) o_acc[rt][b] *= wgt;
#pragma unroll
    for (int b = 0; b < RB; ++b) lr_acc[rt][b] *= wgt;
  }
  if (ALIAS) __syncthreads();  // the maxima are about to be overwritten by merge slots
  float* mslots = reinterpret_cast<float*>(smem);
  constexpr int PER_RT = (DB + RB) * 4 + 1;  // floats per lane and row tile: O^T, Olr^T, l
  // Where four slots fit, every wave deposits its state once and then sums and stores a
  // quarter of it (one barrier, four waves writing); otherwise a two-level tree through two
  // slots with wave 0 writing.
  constexpr bool FLAT = NW * MERGE_SLOT <= SMEM;
  if (FLAT) {
    float* dst = mslots + wave * (NACC * 64) + lane;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
      for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) dst[(rt * PER_RT + b * 4 + jj) * 64] = o_acc[rt][b][jj];
#pragma unroll
      for (int b = 0; b < RB; ++b)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) dst[(rt * PER_RT + (DB + b) * 4 + jj) * 64] = lr_acc[rt][b][jj];
      dst[(rt * PER_RT + (DB + RB) * 4) * 64] = l_run[rt];
    }
    __syncthreads();
    LRA_STAMP(7);
    auto total = [&](int x) {
      float v = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) v += mslots[w * (NACC * 64) + x * 64 + lane];
      return v;
    };
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const int64_t slot = row_slot(rt);
      if (slot < 0) continue;
      // blocks are dealt round robin: O^T block b to wave b % 4, Olr^T block b to wave
      // (DB + b) % 4, the row sum to wave 3 (wave-uniform branches)
#pragma unroll
      for (int b = 0; b < DB; ++b)
        if ((b & (NW - 1)) == wave) {
          f32x4 v;
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) v[jj] = total(rt * PER_RT + b * 4 + jj);
          *reinterpret_cast<f32x4*>(p.part_o + slot * D + b * 16 + lg * 4) = v;
        }
#pragma unroll
      for (int b = 0; b < RB; ++b)
        if (((DB + b) & (NW - 1)) == wave) {
          // PA: a row keeps the column block of its own agent slot only, as ranks 0 .. r-1 of its state
          const int cblk = PA ? b >> (lcs - 1) : 0;
          const bool mine = !PA || cblk == (ln >> gps);
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            const int rho = b * 16 + lg * 4 + jj - cblk * lb;
            const float v = total(rt * PER_RT + (DB + b) * 4 + jj);
            if (mine && rho < r) p.part_lr[slot * r + rho] = v;
          }
        }
      if (wave == NW - 1 && lg == 0) {
        p.part_ml[slot * 2 + 0] = m_all[rt] * 0.69314718055994530942f;  // natural-log units
        p.part_ml[slot * 2 + 1] = total(rt * PER_RT + (DB + RB) * 4);
        if (split == 0) p.part_adapter[slot / p.n_splits] = my_adapter[rt];
      }
    }
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) asm volatile("" ::"v"(warm[rt][0]), "v"(warm[rt][1]));
    LRA_STAMP(8);
#ifdef LRA_TIMING
    asm volatile("s_waitcnt vmcnt(0)");
#endif
    LRA_STAMP(9);
    LRA_STAMP_FLUSH();
    return;
  }
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

  LRA_STAMP(7);
  // ===================== wave 0 writes the workgroup's partial state =====================
  if (wave == 0) {
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const int64_t slot = row_slot(rt);
      if (slot < 0) continue;
      if (lg == 0) {
        p.part_ml[slot * 2 + 0] = m_all[rt] * 0.69314718055994530942f;  // natural-log units
        p.part_ml[slot * 2 + 1] = l_run[rt];
        if (split == 0) p.part_adapter[slot / p.n_splits] = my_adapter[rt];
      }
#pragma unroll
      for (int b = 0; b < DB; ++b)
        *reinterpret_cast<f32x4*>(p.part_o + slot * D + b * 16 + lg * 4) = o_acc[rt][b];
#pragma unroll
      for (int b = 0; b < RB; ++b) {
        const int cblk = PA ? b >> (lcs - 1) : 0;
        const bool mine = !PA || cblk == (ln >> gps);
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int rho = b * 16 + lg * 4 + jj - cblk * lb;
          if (mine && rho < r) p.part_lr[slot * r + rho] = lr_acc[rt][b][jj];
        }
      }
    }
  }
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) asm volatile("" ::"v"(warm[rt][0]), "v"(warm[rt][1]));
  LRA_STAMP(8);
  LRA_STAMP_FLUSH();
}

template <int D, int RT, int RP, bool CAUSAL>
static hipError_t launch_cfg2(const Params& p, dim3 grid, hipStream_t s) {
  const dim3 block(256);
  const bool paged = p.block_size != 0, has_bk = p.b_k != nullptr;
  if (p.l_block != 0) {
    // per-adapter low-rank caches, one column block of the L tile per agent slot: decode, one row tile
    if constexpr (RT == 1 && !CAUSAL) {
      if (paged && has_bk) hipLaunchKernelGGL((decode_mfma_kernel<D, 1, RP, true, true, false, 0, true>), grid, block, 0, s, p);
      else if (paged) hipLaunchKernelGGL((decode_mfma_kernel<D, 1, RP, true, false, false, 0, true>), grid, block, 0, s, p);
      else if (has_bk) hipLaunchKernelGGL((decode_mfma_kernel<D, 1, RP, false, true, false, 0, true>), grid, block, 0, s, p);
      else hipLaunchKernelGGL((decode_mfma_kernel<D, 1, RP, false, false, false, 0, true>), grid, block, 0, s, p);
      return hipGetLastError();
    } else {
      return hipErrorInvalidValue;
    }
  }
  if (paged && has_bk)
    hipLaunchKernelGGL((decode_mfma_kernel<D, RT, RP, true, true, CAUSAL>), grid, block, 0, s, p);
  else if (paged)
    hipLaunchKernelGGL((decode_mfma_kernel<D, RT, RP, true, false, CAUSAL>), grid, block, 0, s, p);
  else if (has_bk)
    hipLaunchKernelGGL((decode_mfma_kernel<D, RT, RP, false, true, CAUSAL>), grid, block, 0, s, p);
  else
    hipLaunchKernelGGL((decode_mfma_kernel<D, RT, RP, false, false, CAUSAL>), grid, block, 0, s, p);
  return hipGetLastError();
}

template <int D, int RT, int RP>
static hipError_t launch_cfg(const Params& p, dim3 grid, hipStream_t s) {
  return p.is_prefill ? launch_cfg2<D, RT, RP, true>(p, grid, s) : launch_cfg2<D, RT, RP, false>(p, grid, s);
}

template <int D, int RP, int RPE>
static hipError_t launch_rope(const Params& p, dim3 grid, hipStream_t s) {
  const bool paged = p.block_size != 0;
  if (p.is_prefill) {
    // (launch_decode_mfma keeps the plain grid for these)
    if (paged) hipLaunchKernelGGL((decode_mfma_kernel<D, 1, RP, true, true, true, RPE, false, false>), grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL((decode_mfma_kernel<D, 1, RP, false, true, true, RPE, false, false>), grid, dim3(256), 0, s, p);
  } else if (p.rg_interleave > 0) {
    if (paged) hipLaunchKernelGGL((decode_mfma_kernel<D, 1, RP, true, true, false, RPE, false, true>), grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL((decode_mfma_kernel<D, 1, RP, false, true, false, RPE, false, true>), grid, dim3(256), 0, s, p);
  } else {
    if (paged) hipLaunchKernelGGL((decode_mfma_kernel<D, 1, RP, true, true, false, RPE, false, false>), grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL((decode_mfma_kernel<D, 1, RP, false, true, false, RPE, false, false>), grid, dim3(256), 0, s, p);
  }
  return hipGetLastError();
}

static hipError_t launch_decode_mfma_grid(const Params& p, int row_tiles, dim3 grid, hipStream_t s);

hipError_t launch_decode_mfma(const Params& p, int row_tiles, bool allow_stream_form, bool main_kernel_only, hipStream_t s) {
  // calls that give a compute unit at most one workgroup: the form with two tile stages per wave
  if (allow_stream_form && decode_stream_applies(p, row_tiles, 256)) return launch_decode_stream(p, row_tiles, main_kernel_only, s);
  dim3 grid(p.n_kv_heads, p.n_splits, (p.is_prefill ? 1 : p.n_seqs) * p.row_groups);
  Params pi = p;
  pi.rg_interleave = 0;
  const bool rope_prefill = p.is_prefill && p.key_rope_theta > 0.f && p.b_k != nullptr;  // (built without that layout)
  if (p.row_groups > 1 && !rope_prefill) {
    // (see the kernel: row groups of a key share next to each other on one XCD)
    int g = p.n_kv_heads, e = 8;
    while (e) { const int tmp = g % e; g = e; e = tmp; }  // g = gcd(Hkv, 8)
    const int m = 8 / g;
    const int64_t gy = static_cast<int64_t>((p.n_splits + m - 1) / m) * m * p.row_groups;
    if (gy <= 65535) {
      pi.rg_interleave = m;
      grid = dim3(p.n_kv_heads, static_cast<unsigned>(gy), p.is_prefill ? 1 : p.n_seqs);
    }
  }
  return launch_decode_mfma_grid(pi, row_tiles, grid, s);
}

static hipError_t launch_decode_mfma_grid(const Params& p, int row_tiles, dim3 grid, hipStream_t s) {
  if (p.key_rope_theta > 0.f && p.b_k != nullptr) {
    if (row_tiles != 1 || (!p.is_prefill && 16 / p.group_pad > decode_mfma_rope_slots(p.rank))) return hipErrorInvalidValue;
    const int sel = (p.head_dim == 128 ? 3 : 0) + (p.rank <= 16 ? 0 : (p.rank <= 32 ? 1 : 2));
    switch (sel) {
      case 0: return launch_rope<64, 32, 16>(p, grid, s);
      case 1: return launch_rope<64, 32, 32>(p, grid, s);
      case 2: return launch_rope<64, 64, 64>(p, grid, s);
      case 3: return launch_rope<128, 32, 16>(p, grid, s);
      case 4: return launch_rope<128, 32, 32>(p, grid, s);
      default: return launch_rope<128, 64, 64>(p, grid, s);
    }
  }
  // columns of the L tile: the rank, or with per-adapter low-rank caches one block per agent slot of a row tile
  const int tile_rank = (p.l_block != 0 && !p.is_prefill) ? (16 / p.group_pad) * p.l_block : p.rank;
  const int rp = tile_rank <= 32 ? 32 : 64;
  const int key = (p.head_dim == 128 ? 4 : 0) | (row_tiles == 2 ? 2 : 0) | (rp == 64 ? 1 : 0);
  switch (key) {
    case 0: return launch_cfg<64, 1, 32>(p, grid, s);
    case 1: return launch_cfg<64, 1, 64>(p, grid, s);
    case 2: return launch_cfg<64, 2, 32>(p, grid, s);
    case 3: return launch_cfg<64, 2, 64>(p, grid, s);
    case 4: return launch_cfg<128, 1, 32>(p, grid, s);
    case 5: return launch_cfg<128, 1, 64>(p, grid, s);
    case 6: return launch_cfg<128, 2, 32>(p, grid, s);
    default: return launch_cfg<128, 2, 64>(p, grid, s);
  }
}

}  // namespace lra
