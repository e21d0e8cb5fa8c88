// Split-KV decode kernel for calls that give every compute unit at most one workgroup
// (bf16, gfx950): one sequence in a contiguous cache, no rotary key side.
//
// Same arithmetic and data layout as decode_mfma_kernel (the inner loop of Alg. 1 with the
// App. D.1 key-side reordering, scores computed transposed, all agents x GQA rows of a kv
// head in the N dimension of v_mfma_f32_16x16x32_bf16); what differs is the schedule.  A call
// of this size (tens of MB) is a chain of latencies, not a stream, so the kernel is built
// around one rule: every byte of K_base / V_base / L is requested as early as the LDS can
// take it, and nothing stands between the kernel's first instruction and its first request
// that the request does not need.
//   - A workgroup owns the whole LDS of its CU.  Waves 0-3 stream: each has TWO tile stages
//     (2 x 32 keys) and requests both before it does anything else; the requests are
//     hand-issued buffer_load ... lds, retire in order, and are waited for by hand-placed
//     s_waitcnt vmcnt(N) with the number of younger requests - K and L of a tile before its V,
//     so the scores and the softmax of a tile run while its V rows are still on their way.
//   - Waves 4-7 are the prologue: they load Q and the B_K rows of the workgroup's agents
//     into registers with ordinary loads (their own request counters: nothing of theirs
//     queues in front of a tile), form Qt = Q B_K^T by MFMA and leave Q and Qt in LDS in
//     operand-ready order - in a hand-over area of their own where the LDS has room for one
//     next to the tile stages, else (head dimension 128 with 64 ranks) in the second stage of
//     the last streaming wave, which that wave fills only after everybody has picked them up.
//     Their loads are issued before the streaming waves' first requests (a bare barrier orders
//     the two): the memory path of a compute unit serves requests in order, so a load issued
//     behind 80 KB of tile requests comes back after them.  With many agent slots and large
//     ranks Qt comes from a pre-pass kernel instead and is only copied.  The prologue waves
//     then touch the B_V rows the merge kernel will need and wait at the final barrier.
//   - With one low-rank cache per adapter (BaseShared) the L tile is a row of column blocks,
//     one per agent slot of the row tile, each requested from that slot's cache; Qt of a row
//     is zero outside the block of its slot, so the products are unchanged (template form PA).
//   - All divisions by the row padding (a power of two) are shifts; the addresses of the
//     LDS reads are formed after the requests have left.
//   - The four streaming waves merge their states with one barrier (each deposits its
//     unscaled state and its maxima, then sums a quarter of the blocks with the
//     flash-decoding weights, in wave order).
#include "lra_common.h"
#include "lra_decode_util.h"

namespace lra {

#ifdef LRA_TIMING
#define LRA_STAMP(k) do { unsigned long long t_; asm volatile("s_waitcnt lgkmcnt(0)\n\ts_memrealtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(t_)); tt[k] = t_; } while (0)
#define LRA_STAMP_DECL unsigned long long tt[12] = {0,0,0,0,0,0,0,0,0,0,0,0}
#define LRA_STAMP_FLUSH() do { if (p.timing && lane == 0) { \
    unsigned long long* o_ = p.timing + ((static_cast<size_t>(blockIdx.z) * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * 128 + wave * 16; \
    for (int i_ = 0; i_ < 12; ++i_) o_[i_] = tt[i_]; \
    o_[12] = __builtin_amdgcn_s_getreg((20) | (0 << 6) | ((4 - 1) << 11)); \
    o_[13] = __builtin_amdgcn_s_getreg((4) | (0 << 6) | ((32 - 1) << 11)); } } while (0)
#else
#define LRA_STAMP(k)
#define LRA_STAMP_DECL
#define LRA_STAMP_FLUSH()
#endif

// LDS bytes of one workgroup of decode_stream_kernel<D, RT, RP>: the tile stages and nothing else.
constexpr int decode_stream_lds_bytes(int D, int RP) { return 4 * 2 * (2 * 32 * D * 2 + 32 * RP * 2); }

template <int D, int RT, int RP, bool HAS_BK, bool CAUSAL, bool PA, bool SI = false>
__global__ __launch_bounds__(512, 2) void decode_stream_kernel(Params p) {
  static_assert(!PA || (!CAUSAL && RT == 1), "per-adapter low-rank caches: decode form, one row tile");
  constexpr int NW = 4;            // streaming waves; waves NW .. 2 NW - 1 are the prologue waves
  constexpr int KS = D / 32;       // MFMA k-steps over the head dimension
  constexpr int RKS = RP / 32;     // MFMA k-steps over the (padded) rank
  constexpr int DB = D / 16;       // 16-wide output blocks over d
  constexpr int RB = RP / 16;      // 16-wide output blocks over the rank
  constexpr int KCH = D / 8;       // 16-byte chunks per K/V row
  constexpr int RCH = RP / 8;      // 16-byte chunks per L row in LDS
  constexpr int KROWS = 64 / KCH;  // K/V rows one wave-wide request moves
  constexpr int KVL = 32 / KROWS;  // requests per 32-key K (or V) tile
  constexpr int LROWS = 64 / RCH;
  constexpr int LL = 32 / LROWS;
  constexpr int TL = 2 * KVL + LL; // requests of one tile, in the order K, L, V
  constexpr int KV_BYTES = 32 * D * 2;
  constexpr int L_BYTES = 32 * RP * 2;
  constexpr int STAGE_BYTES = 2 * KV_BYTES + L_BYTES;
  constexpr int WAVE_BYTES = 2 * STAGE_BYTES;
  constexpr int ROW_BYTES = D * 2;
  constexpr int MAXIT = RP / 16;               // Qt items per prologue wave and row tile: 4 slots x RP/16 rho blocks over 4 waves
  constexpr int Q_BYTES = RT * KS * 1024;      // Q as B operands: 16 bytes per lane, k-step and row tile
  constexpr int QT_BYTES = RT * RKS * 1024;
  constexpr int NBLK = DB + RB;                                // f32x4 blocks per lane and row tile
  constexpr int SLOT_BYTES = RT * (NBLK * 1024 + 512);         // merge slot of a wave: blocks, then (m, l) pairs
  static_assert(SLOT_BYTES <= WAVE_BYTES, "a wave's merge slot lives in its own tile region");
  // Q and Qt are handed from the prologue waves to the streaming waves through an area of their own
  // where the LDS has room for it next to the tile stages; otherwise (head dimension 128 with 64
  // ranks) through the second stage of the last streaming wave, which then gets its second tile
  // only after everybody has picked them up.
  constexpr bool HANDOVER_IN_STAGE = NW * WAVE_BYTES + Q_BYTES + QT_BYTES > 160 * 1024;
  static_assert(Q_BYTES + QT_BYTES <= STAGE_BYTES, "Q and Qt fit one tile stage");
  // SI ("split issue", for key ranges of at most two tiles per wave): a streaming wave requests its
  // first tile only; its second tile is requested, and waited for, by the prologue wave of the
  // same number, which has nothing else left to do.  A wave issues in order, and the memory path
  // accepts requests only as fast as data returns: a wave that requests both tiles itself sits in
  // the issue of the second one for microseconds after its first tile has landed, and starts
  // computing only then.
  static_assert(!SI || !HANDOVER_IN_STAGE, "split issue needs the second stage from the start");
  static_assert(NW * WAVE_BYTES == decode_stream_lds_bytes(D, RP), "LDS accounting");
  static_assert(NW * WAVE_BYTES <= 160 * 1024, "LDS of one CU");

  __shared__ __align__(16) unsigned char smem[NW * WAVE_BYTES];
  __shared__ __align__(16) unsigned char handover[HANDOVER_IN_STAGE ? 16 : Q_BYTES + QT_BYTES];
  unsigned char* q_lds = HANDOVER_IN_STAGE ? smem + (NW - 1) * WAVE_BYTES + STAGE_BYTES : handover;
  unsigned char* qt_lds = q_lds + Q_BYTES;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ln = lane & 15, lg = lane >> 4;
  const bool helper = wave >= NW;
  LRA_STAMP_DECL;
  LRA_STAMP(0);
  // Everything of the parameter block that stands before the first request is asked for at once:
  // left to itself the compiler fetches it piece by piece, each piece a round trip of its own
  // behind the branch that needs it.
  asm volatile("" ::"s"(p.k_base), "s"(p.v_base), "s"(p.l), "s"(p.seq_lens), "s"(p.query_adapter));
  asm volatile("" ::"s"(p.kv_token_stride), "s"(p.kv_head_stride), "s"(p.l_row_stride), "s"(p.l_adapter_stride));
  asm volatile("" ::"s"(p.rank), "s"(p.group_pad), "s"(p.row_groups), "s"(p.max_seq_len), "s"(p.n_queries), "s"(p.n_adapters),
               "s"(p.split_keys), "s"(p.l_block), "s"(p.share_major), "s"(p.n_splits));
  // Workgroups go round-robin over the 8 XCDs in the order of their linear index, and every XCD
  // has an L2 of its own.  Two layouts of that index, chosen by the host:
  //  - kv head fastest (grid (Hkv, key shares, row groups)): with 8 kv heads all workgroups of a
  //    head run on one XCD, share Q and B_K there, and leave the B_V rows the merge kernel will
  //    ask for in the L2 it will ask from.  Every XCD then reads all of L.
  //  - share_major (grid (8 Hkv, key shares / 8, row groups), x = (key share mod 8) + 8 kv head):
  //    all kv heads of one key share run on ONE XCD, at the same time, and read that share's L rows
  //    once instead of once per head.  For wide L rows (8 heads, r = 64: 8 x 4.2 MB of a 141 MB call).
  const int bx = blockIdx.x, by = blockIdx.y;
  const int h = p.share_major ? bx >> 3 : bx;
  const int split = p.share_major ? by * 8 + (bx & 7) : by;
  const int rg = blockIdx.z;
  if (split >= p.n_splits) return;  // (share_major pads the key shares to a multiple of 8)
  const int t = CAUSAL ? p.seq_index : 0;                      // contiguous caches hold one sequence
  const int32_t len_t = CONST_I32(p.seq_lens)[t];
  const int n_q = CAUSAL ? p.n_new : p.n_queries;
  const int GP = p.group_pad, G = p.group, r = p.rank;
  const int gps = __builtin_ctz(GP);                           // GP is 4, 8 or 16
  const int row0 = rg * RT * 16;
  // adapters of the agent slots of the row tiles (wave-uniform), -1 for an empty slot.  All ids are
  // requested before any is looked at (unconditional loads from a clamped index: one round trip
  // for the lot); being device data, they are then kept inside the table, as the merge kernel does.
  int a_slot[RT][4];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int si = 0; si < 4; ++si) {
      const int slot = ((row0 + rt * 16) >> gps) + si;
      a_slot[rt][si] = CAUSAL ? p.adapter_index : CONST_I32(p.query_adapter)[min(slot, n_q - 1)];
    }
  asm volatile("" ::"s"(len_t), "s"(a_slot[0][0]), "s"(a_slot[0][1]), "s"(a_slot[0][2]), "s"(a_slot[0][3]));  // one wait for all of them
  if (row0 >= (n_q << gps)) return;
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int si = 0; si < 4; ++si) {
      const int slot = ((row0 + rt * 16) >> gps) + si;
      const bool live = si < (16 >> gps) && slot < n_q;
      a_slot[rt][si] = live ? min(max(a_slot[rt][si], 0), p.n_adapters - 1) : -1;
    }
  auto slot_adapter = [&](int rt, int si) {
    return si == 0 ? a_slot[rt][0] : (si == 1 ? a_slot[rt][1] : (si == 2 ? a_slot[rt][2] : a_slot[rt][3]));
  };
  const int n_t = min(len_t, p.max_seq_len);
  const int j0 = split * p.split_keys;
  // output row (query x Hq + q head) this lane stands for in row tile rt (-1: padding row);
  // its workspace slot is row * n_splits + split
  auto row_index = [&](int rt) -> int {
    const int R = row0 + rt * 16 + ln;
    const int slot_q = R >> gps, gg = R & (GP - 1);
    if (!(slot_q < n_q && gg < G)) return -1;
    return slot_q * p.n_q_heads + h * G + gg;
  };
  if (j0 >= n_t) {
    // a split past the end of the sequence: leave an empty state (zero row sum), which is
    // all the merge kernel looks at; the O and O_lr rows of the slot stay unwritten
    if (wave == 0 && lg == 0) {
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        const int row = row_index(rt);
        if (row >= 0) {
          const int64_t slot = static_cast<int64_t>(row) * p.n_splits + split;
          p.part_ml[slot * 2 + 0] = -INFINITY;
          p.part_ml[slot * 2 + 1] = 0.f;
        }
      }
    }
    return;
  }
  LRA_STAMP(1);

  // ===================== tile requests (of streaming wave sw) =====================
  const int j1 = min(j0 + p.split_keys, n_t);
  const int kpw = p.split_keys / NW;  // multiple of 32
  const uint32_t ts2 = static_cast<uint32_t>(p.kv_token_stride) * 2u;  // token stride in bytes
  const uint32_t r2 = static_cast<uint32_t>(r) * 2u;                     // L row in bytes
  const uint32_t lp2 = static_cast<uint32_t>(p.l_row_stride) * 2u;       // bytes between L rows
  // The L tile in LDS is a row of column blocks, [block][32 keys][lb ranks]: one block of RP ranks
  // with one low-rank cache for all agents, one block of l_block ranks per agent slot with
  // per-adapter caches (BaseShared).  A block takes lb/16 requests of 1 KB.
  constexpr bool per_agent = PA;
  const int lb = per_agent ? p.l_block : RP;   // ranks per block: 16, 32 or 64
  const int lcpr = lb >> 3;                    // 16-byte chunks per row of a block: 2, 4 or 8
  const int lcs = __builtin_ctz(lcpr);         // (all powers of two: shifts, no divisions)
  const int lb2 = lb * 2;                      // bytes per row of a block
  // XOR swizzle of the chunk index inside a block row (none for 32-byte rows: 16 rows fill two clocks densely)
  auto swz_l = [&](int row) { return lcpr == 8 ? (row & 7) : (lcpr == 4 ? ((row >> 1) & 3) : 0); };
  // LDS swizzles (XOR on the 16-byte chunk index of a row; the LDS serves 256 bytes per clock):
  //   K (ds_read_b128, 16 rows per clock)           chunk ^ (row & 15)        | chunk ^ ((row >> 1) & 7)
  //   V (ds_read_b64_tr_b16, 8 rows per clock)      chunk ^ ((row & 7) << 1)  | chunk ^ (((row >> 1) & 3) << 1)
  // Lane l of request i lands at LDS row i*KROWS + l/KCH, physical chunk l%KCH, and therefore
  // fetches the logical chunk (l%KCH) ^ swizzle(row); the swizzle repeats with period
  // 16/KROWS (K) and 8/KROWS (V) in i.
  auto swz_k = [](int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); };
  auto swz_v = [](int row) { return D == 128 ? ((row & 7) << 1) : (((row >> 1) & 3) << 1); };
  constexpr int KPER = KROWS == 4 ? 4 : 2, VPER = KROWS == 4 ? 2 : 1;
  // K_base / V_base requests are non-temporal when this workgroup is the only reader of its
  // keys; with several row groups per kv head the others find the tiles in L2
  const bool stream_kv = p.row_groups == 1;
  struct TileRequests {
    int jw0, jw1;               // keys of the wave
    unsigned char* wave_lds;    // its tile stages
    uint32_t k_voff[KPER], v_voff[VPER], l_voff;
    u32x4 rs_k, rs_v, rs_l[LL];  // one resource per wave covering exactly its keys; one L resource per request: the requests of a block read that block's adapter
    uint32_t l_soff[LL];        // first row of the request inside its block, in bytes of the source
  };
  auto tile_requests = [&](int sw) __attribute__((always_inline)) {
    TileRequests q;
    q.jw0 = j0 + sw * kpw;
    q.jw1 = max(q.jw0, min(q.jw0 + kpw, j1));  // == jw0 for a wave without keys
    q.wave_lds = smem + sw * WAVE_BYTES;
    const int rr = lane / KCH, pc = lane % KCH;
#pragma unroll
    for (int i = 0; i < KPER; ++i) q.k_voff[i] = static_cast<uint32_t>(rr) * ts2 + ((pc ^ swz_k(i * KROWS + rr)) << 4);
#pragma unroll
    for (int i = 0; i < VPER; ++i) q.v_voff[i] = static_cast<uint32_t>(rr) * ts2 + ((pc ^ swz_v(i * KROWS + rr)) << 4);
    {
      const int lrow = lane >> lcs, lpc = lane & (lcpr - 1);  // row inside a request: the swizzle repeats from request to request
      const int lch = lpc ^ swz_l(lrow);
      q.l_voff = (lch * 8 < r) ? static_cast<uint32_t>(lrow) * lp2 + (lch << 4) : kOob;
    }
    const int nk = q.jw1 - q.jw0;
    const int64_t base = static_cast<int64_t>(h) * p.kv_head_stride + static_cast<int64_t>(q.jw0) * p.kv_token_stride;
    const uint32_t bytes = nk > 0 ? static_cast<uint32_t>(nk - 1) * ts2 + D * 2 : 0u;
    q.rs_k = make_rsrc_words(static_cast<const bf16_t*>(p.k_base) + base, bytes);
    q.rs_v = make_rsrc_words(static_cast<const bf16_t*>(p.v_base) + base, bytes);
    const int rows_per_req = 64 >> lcs;  // 1 KB of rows of lb ranks
    const int rpb_shift = lcs - 1;       // lb/16 requests per block
    const uint32_t l_bytes = nk > 0 ? static_cast<uint32_t>(nk - 1) * lp2 + r2 : 0u;
#pragma unroll
    for (int i = 0; i < LL; ++i) {
      const int blk = i >> rpb_shift, qq = i - (blk << rpb_shift);
      // block = agent slot of the row tile (per-adapter caches), or the one cache (of the call's adapter in
      // the causal form); a block beyond the tile's slots reads nothing
      int a = CAUSAL ? p.adapter_index : 0;
      bool live = blk == 0;
      if (per_agent) {
        a = slot_adapter(0, blk);
        live = blk < (16 >> gps) && a >= 0;
      }
      q.rs_l[i] = make_rsrc_words(static_cast<const bf16_t*>(p.l) + static_cast<int64_t>(live ? a : 0) * p.l_adapter_stride +
                                      static_cast<int64_t>(q.jw0) * p.l_row_stride,
                                  live ? l_bytes : 0u);
      q.l_soff[i] = static_cast<uint32_t>(qq * rows_per_req) * lp2;
    }
    return q;
  };
  // HBM -> LDS for the 32-key step starting at token j of the sequence, into stage st of the
  // wave: K rows, then L rows, then V rows
  // (parts: 1 = the K rows, 2 = the L and V rows, 3 = all, always in this order)
  auto issue_tile_of = [&](const TileRequests& q, int j, int st, int parts) __attribute__((always_inline)) {
    unsigned char* ks = q.wave_lds + st * STAGE_BYTES;
    unsigned char* vs = ks + KV_BYTES;
    unsigned char* ls = vs + KV_BYTES;
    const uint32_t s0 = static_cast<uint32_t>(j - q.jw0);
    if (parts & 1) {
      if (stream_kv) {
#pragma unroll
        for (int i = 0; i < KVL; ++i) buf_load16_to_lds<true>(q.rs_k, ks + i * 1024, q.k_voff[i % KPER], (s0 + i * KROWS) * ts2);
      } else {
#pragma unroll
        for (int i = 0; i < KVL; ++i) buf_load16_to_lds<false>(q.rs_k, ks + i * 1024, q.k_voff[i % KPER], (s0 + i * KROWS) * ts2);
      }
    }
    if (parts & 2) {
#pragma unroll
      for (int i = 0; i < LL; ++i) buf_load16_to_lds(q.rs_l[i], ls + i * 1024, q.l_voff, s0 * lp2 + q.l_soff[i]);
      if (stream_kv) {
#pragma unroll
        for (int i = 0; i < KVL; ++i) buf_load16_to_lds<true>(q.rs_v, vs + i * 1024, q.v_voff[i % VPER], (s0 + i * KROWS) * ts2);
      } else {
#pragma unroll
        for (int i = 0; i < KVL; ++i) buf_load16_to_lds<false>(q.rs_v, vs + i * 1024, q.v_voff[i % VPER], (s0 + i * KROWS) * ts2);
      }
    }
  };

  if (helper) {
    // ===================== prologue waves: Q operands and Qt = Q B_K^T =====================
    const int hw = wave - NW;
    // qb[rt][ks]: lane (row ln of tile rt, k = 32ks + 8lg + e), e = 0..7: the B operand of S^T
    // and of Qt^T = B_K Q^T
    bf16x8 qb[RT][KS];
    {
      const __amdgpu_buffer_rsrc_t rs_q = make_rsrc(p.q, static_cast<uint32_t>(n_q) * p.n_q_heads * D * 2);
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        const int R = row0 + rt * 16 + ln;
        const int slot = R >> gps, gg = R & (GP - 1);
        const bool valid = slot < n_q && gg < G;
        const uint32_t off = valid ? static_cast<uint32_t>((slot * p.n_q_heads + h * G + gg) * ROW_BYTES + lg * 16) : kOob;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qb[rt][ks] = as_bf16x8(buf_load16(rs_q, off, ks * 64));
      }
    }
    const bool qt_ready = HAS_BK && p.qt_ws != nullptr;  // a pre-pass has formed Qt for the whole call
    if (qt_ready) {
      // operand-ready Qt of this (kv head, row group): RT*RKS pieces of 1 KB; prologue wave hw copies
      // pieces hw, hw + NW, ...
      const uint4* src = reinterpret_cast<const uint4*>(p.qt_ws) + (static_cast<size_t>(rg) * p.n_kv_heads + h) * (RT * RKS * 64);
      uint4 piece[(RT * RKS + NW - 1) / NW];
#pragma unroll
      for (int i = 0; i < (RT * RKS + NW - 1) / NW; ++i) {
        const int idx = hw + i * NW;
        piece[i] = idx < RT * RKS ? src[idx * 64 + lane] : make_uint4(0u, 0u, 0u, 0u);
      }
      __builtin_amdgcn_s_barrier();  // these loads have left (see below)
#pragma unroll
      for (int i = 0; i < (RT * RKS + NW - 1) / NW; ++i) {
        const int idx = hw + i * NW;
        if (idx < RT * RKS) *reinterpret_cast<uint4*>(qt_lds + (idx * 64 + lane) * 16) = piece[i];
      }
    }
    // Per-adapter low-rank caches (BaseShared): the L tile holds one column block of lb ranks per
    // agent slot, so Qt of a row lives in the block of its slot and is zero elsewhere.
    const int lb16 = per_agent ? p.l_block >> 4 : 0;  // 16-rank blocks per slot
    if (HAS_BK && !qt_ready) {
      // every lane of the hand-over area starts as zero (blocks beyond the rank, other slots' blocks)
#pragma unroll
      for (int i = 0; i < (RT * RKS + NW - 1) / NW; ++i) {
        const int idx = hw + i * NW;
        if (idx < RT * RKS) *reinterpret_cast<uint4*>(qt_lds + (idx * 64 + lane) * 16) = make_uint4(0u, 0u, 0u, 0u);
      }
      __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): written before the barrier below lets the products follow
      // Item idx = hw + it*NW of row tile rt is (agent slot si, rho block cb); this lane holds row
      // rho = 16cb + ln of B_K^a, columns h*D + 32ks + 8lg ..: the A operand of Qt^T.  Rows beyond
      // the rank and the rows of empty slots lie outside the resource and arrive as zeros.
      const int S = 16 >> gps;         // agent slots per 16-row tile
      const int ncb = (r + 15) >> 4;   // rho blocks: 1 .. RP/16
      const int n_items = S * ncb;
      // idx -> (slot, rho block): idx / ncb without a division (idx < 16, ncb <= 4)
      const int inv_ncb = ncb == 1 ? 257 : (ncb == 2 ? 129 : (ncb == 3 ? 86 : 65));  // 256 / ncb + 1
      auto item_slot = [&](int idx) { return (idx * inv_ncb) >> 8; };
      const int64_t ldb = static_cast<int64_t>(p.n_kv_heads) * D;
      const bf16_t* bkg = static_cast<const bf16_t*>(p.b_k);
      uint4 bt4[RT][MAXIT][KS];
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int it = 0; it < MAXIT; ++it) {
          const int idx = hw + it * NW;
          const int si = item_slot(idx), cb = idx - si * ncb;
          const int a = slot_adapter(rt, si);
          const bool live = idx < n_items && a >= 0;
          const uint32_t bytes = live ? static_cast<uint32_t>((r - 1) * ldb + D) * 2u : 0u;
          const __amdgpu_buffer_rsrc_t rs_b = make_rsrc(bkg + static_cast<int64_t>(live ? a : 0) * r * ldb + h * D, bytes);
          const uint32_t off = static_cast<uint32_t>((cb * 16 + ln) * ldb * 2 + lg * 16);
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) bt4[rt][it][ks] = buf_load16(rs_b, off, ks * 64);
        }
      // The streaming waves hold their requests back until these loads have left: the memory
      // path of a CU takes requests in order, and behind 144 KB of tile requests Q and B_K would
      // arrive last.  (A bare barrier: nothing is exchanged yet, it only orders the issue.)
      __builtin_amdgcn_s_barrier();
      // Qt^T block (rho block cb, tile rt) in C layout: lane (rho = 16cb + 4lg + j, row ln).  Rows
      // of a tile belong to 16/GP agents; each agent's product is kept only in its own rows
      // (lanes).  Left in LDS in operand-ready form: operand (rt, ks') of lane l is the 16 bytes
      // at ((rt*RKS + ks')*64 + l)*16, elements e -> rho = 32ks' + 16(e/4) + 4lg + e%4 (the L
      // operand of the loop uses the same order).
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int it = 0; it < MAXIT; ++it) {
          const int idx = hw + it * NW;
          if (idx < n_items) {
            const int si = item_slot(idx), cb = idx - si * ncb;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
              acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(bt4[rt][it][ks]), qb[rt][ks], acc, 0, 0, 0);
            if ((ln >> gps) == si) {
              const int kb = si * lb16 + cb;  // 16-rank block along the L tile's columns
              unsigned char* dst = qt_lds + ((rt * RKS + (kb >> 1)) * 64 + lane) * 16;
              *reinterpret_cast<uint2*>(dst + (kb & 1) * 8) = make_uint2(pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3]));
            }
          }
        }
    }
    if constexpr (!HAS_BK) __builtin_amdgcn_s_barrier();  // the Q loads have left (see above)
    if (hw == 0) {
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          *reinterpret_cast<uint4*>(q_lds + ((rt * KS + ks) * 64 + lane) * 16) = __builtin_bit_cast(uint4, qb[rt][ks]);
    }
    LRA_STAMP(2);
    // One workgroup per (kv head, row group) touches the B_V rows the merge kernel will need
    // (one 4-byte read per 128-byte line), so that they wait in this XCD's L2 instead of in
    // HBM: prologue wave w takes agent slot w of every row tile.
    int warm[RT];
    // (the merge kernel's rows of kv head h run on XCD h mod 8: under share_major that is where key share h mod 8 runs)
    const int warm_split = p.share_major ? min(h & 7, p.n_splits - 1) : min(1, p.n_splits - 1);
    auto warm_b_v = [&]() __attribute__((always_inline)) {
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        warm[rt] = 0;
        const int a = slot_adapter(rt, hw);
        if (p.b_v != nullptr && split == warm_split && a >= 0) {
          constexpr int LPR = D * 2 / 128;  // 128-byte lines per B_V row of one kv head
          const int n_lines = r * LPR;      // <= 128
          const char* bv = static_cast<const char*>(p.b_v) +
                           (static_cast<int64_t>(a) * r * p.n_kv_heads * D + static_cast<int64_t>(h) * D) * 2;
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            const int li = i * 64 + lane;
            if (li < n_lines)
              warm[rt] += *reinterpret_cast<const int*>(bv + static_cast<int64_t>(li / LPR) * p.n_kv_heads * D * 2 + (li % LPR) * 128);
          }
        }
      }
    };
    if constexpr (SI) {
      // the second tile of streaming wave hw: requested here, so that wave can start on its first.
      // (Before the barrier that hands Q and Qt over: the streaming waves arrive there only when
      // their own requests have been taken, and need Q and Qt only when their tile has landed.)
      warm_b_v();
      const TileRequests q = tile_requests(hw);
      if (q.jw0 + 32 < q.jw1) issue_tile_of(q, q.jw0 + 32, 1, 3);
      __syncthreads();  // Q and Qt are in LDS
      // Requests retire in order: with at most the KVL requests of the V rows outstanding (anything
      // issued after them only makes this later), the K and L rows of the tile have landed.
      wait_vm<KVL>();
      lds_fence();
      __syncthreads();  // the streaming waves may read K and L of their second tile
      wait_vm0();
      lds_fence();
      __syncthreads();  // ... and its V rows
    } else {
      __syncthreads();  // Q and Qt are in LDS
      if constexpr (HANDOVER_IN_STAGE) __syncthreads();  // ... and have been picked up
      warm_b_v();
    }
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) asm volatile("" ::"v"(warm[rt]));
    __syncthreads();  // the streaming waves' merge barrier
    LRA_STAMP(11);
    LRA_STAMP_FLUSH();
    return;
  }

  // ===================== streaming waves =====================
  const TileRequests treq = tile_requests(wave);
  const int jw0 = treq.jw0, jw1 = treq.jw1;
  unsigned char* wave_lds = treq.wave_lds;
  auto issue_tile = [&](int j, int st) __attribute__((always_inline)) { issue_tile_of(treq, j, st, 3); };
  // (Letting the K rows of the first tile leave before this barrier starts the stream 0.3 us earlier
  // and makes the call slower: Q and B_K then queue behind 32 KB and Qt is late.)
  __builtin_amdgcn_s_barrier();  // the prologue waves' loads have left: theirs go first
  if (jw0 < jw1) issue_tile(jw0, 0);
  if constexpr (!HANDOVER_IN_STAGE && !SI)
    if (jw0 + 32 < jw1) issue_tile(jw0 + 32, 1);
  LRA_STAMP(2);
  __builtin_amdgcn_sched_barrier(0);

  // ---- addresses of the LDS reads ----
  // K rows as A operand of S^T: key = 16tt + ln, logical chunk 4ks + lg at chunk ^ swz_k(key):
  // row offset, swizzle and lg sit in disjoint address bits: k_pre ^ (ks << 6) + tt * 16 rows.
  const int k_pre = ln * ROW_BYTES + ((swz_k(ln) ^ lg) << 4);
  // V^T as A operand of O^T: this lane addresses row ka (+16tt) of the tile, logical chunk
  // 2b + c0 (+ half sub): address v_pre ^ (b << 5) + tt * 16 rows.
  const int ka = 4 * lg + (ln >> 2);
  const int v_pre = ka * ROW_BYTES + ((swz_v(ka) + ((ln & 3) >> 1)) << 4) + (ln & 1) * 8;
  int l_rd[RKS][2];  // L rows as A operand of S^T: two 8-byte pieces per k-step
  int lt_rd[RB];     // L^T as A operand of Olr^T
  {
    // column chunk ch of the tile (8 ranks) lies in block ch / lcpr, chunk ch % lcpr of a row there
    auto chunk_addr = [&](int ch, int row) {
      const int blk = ch >> lcs, cc = ch & (lcpr - 1);
      return blk * (32 * lb2) + row * lb2 + ((cc ^ swz_l(row)) << 4);
    };
#pragma unroll
    for (int ks = 0; ks < RKS; ++ks)
#pragma unroll
      for (int pcs = 0; pcs < 2; ++pcs) l_rd[ks][pcs] = chunk_addr(4 * ks + 2 * pcs + (lg >> 1), ln) + (lg & 1) * 8;
#pragma unroll
    for (int b = 0; b < RB; ++b) lt_rd[b] = chunk_addr(2 * b + ((ln & 3) >> 1), ka) + (ln & 1) * 8;
  }
  // last key each of this lane's rows may see (causal form only)
  int lim[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) lim[rt] = n_t - n_q + min((row0 + rt * 16 + ln) >> gps, n_q - 1);
  const int lim_first = n_t - n_q + (row0 >> gps);  // the smallest of them in this workgroup
  int out_row[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) out_row[rt] = row_index(rt);

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

  __syncthreads();  // the prologue waves have left Q and Qt in LDS
  bf16x8 qb[RT][KS], qtb[RT][RKS];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qb[rt][ks] = as_bf16x8(lds_read16(q_lds + ((rt * KS + ks) * 64 + lane) * 16));
#pragma unroll
    for (int ks = 0; ks < RKS; ++ks) {
      uint4 v = make_uint4(0u, 0u, 0u, 0u);  // k-steps entirely beyond the rank were never written
      if (HAS_BK && (per_agent || ks * 32 < r)) v = lds_read16(qt_lds + ((rt * RKS + ks) * 64 + lane) * 16);
      qtb[rt][ks] = as_bf16x8(v);
    }
  }
  if constexpr (HANDOVER_IN_STAGE) {
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the reads have returned
    lds_fence();
    __syncthreads();  // everybody has picked them up: the hand-over area is a tile stage again
    if (jw0 + 32 < jw1) issue_tile(jw0 + 32, 1);
  }
  LRA_STAMP(3);

  // ===================== main loop =====================
  // One 32-key step on the tile in stage st.  `younger` = the tile of the other stage has been
  // requested after this one (TL requests that may stay outstanding).
  // `by_barrier` (split issue): the tile was requested by the prologue wave, which announces K and
  // L, then V, with a workgroup barrier each.
  auto step = [&](int j, int st, bool younger, bool by_barrier) __attribute__((always_inline)) {
    const unsigned char* ks_lds = wave_lds + st * STAGE_BYTES;
    const unsigned char* vs_lds = ks_lds + KV_BYTES;
    const unsigned char* ls_lds = vs_lds + KV_BYTES;
    // K and L rows of the tile have landed when only its V requests (and the younger tile's) are out
    if (by_barrier) __syncthreads();
    else if (younger) wait_vm<TL + KVL>();
    else wait_vm<KVL>();
    lds_fence();
    f32x4 s[2][RT];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) s[tt][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 a = as_bf16x8(lds_read16(ks_lds + (k_pre ^ (ks << 6)) + tt * 16 * ROW_BYTES));
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
          s[tt][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qb[rt][ks], s[tt][rt], 0, 0, 0);
      }
      if constexpr (HAS_BK) {
#pragma unroll
        for (int ks = 0; ks < RKS; ++ks) {
          const uint2 lo = lds_read8(ls_lds + l_rd[ks][0] + tt * 16 * lb2);
          const uint2 hi = lds_read8(ls_lds + l_rd[ks][1] + tt * 16 * lb2);
          const bf16x8 a = as_bf16x8(make_uint4(lo.x, lo.y, hi.x, hi.y));
#pragma unroll
          for (int rt = 0; rt < RT; ++rt)
            s[tt][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qtb[rt][ks], s[tt][rt], 0, 0, 0);
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
    // Olr^T += L^T P^T (L has landed with K), then the V rows: O^T += V^T P^T
#pragma unroll
    for (int b = 0; b < RB; ++b) {
      const unsigned char* src = ls_lds + lt_rd[b];
      const bf16x8 a = join_tr(lds_read_tr16(src), lds_read_tr16(src + 16 * lb2));
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
        lr_acc[rt][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pb[rt], lr_acc[rt][b], 0, 0, 0);
    }
    if (by_barrier) __syncthreads();
    else if (younger) wait_vm<TL>();
    else wait_vm0();
    lds_fence();
#pragma unroll
    for (int b = 0; b < DB; ++b) {
      const unsigned char* src = vs_lds + (v_pre ^ (b << 5));
      const bf16x8 a = join_tr(lds_read_tr16(src), lds_read_tr16(src + 16 * ROW_BYTES));
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
        o_acc[rt][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pb[rt], o_acc[rt][b], 0, 0, 0);
    }
    // the next tile of this stage overwrites this one: every LDS read above must have returned
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
    lds_fence();
  };

  // Stage 0 holds tile j, stage 1 tile j + 32 (where the wave has that many keys); after a step
  // the tile two steps ahead, if there is one, is requested into the stage it frees.
  if constexpr (SI) {
    // at most two tiles: the first requested by this wave, the second by its prologue wave
    if (jw0 < jw1) step(jw0, 0, false, false);
    LRA_STAMP(4);
    if (jw0 + 32 < jw1) {
      step(jw0 + 32, 1, false, true);
    } else {
      __syncthreads();  // the two barriers of the second tiles
      __syncthreads();
    }
  } else if (jw0 < jw1) {
    int j = jw0;
    while (true) {
      const bool has1 = j + 32 < jw1;
      step(j, 0, has1, false);
      if (j == jw0) LRA_STAMP(4);
      const bool has2 = j + 64 < jw1;
      if (has2) issue_tile(j + 64, 0);
      if (!has1) break;
      step(j + 32, 1, has2, false);
      if (j + 96 < jw1) issue_tile(j + 96, 1);
      if (!has2) break;
      j += 64;
    }
  }
  LRA_STAMP(5);

  // ===================== merge the streaming waves (one barrier) =====================
  // Every wave deposits its state as it stands - blocks as 16 bytes per lane, then (m, l) per
  // lane - in its own tile region (nothing of its own is outstanding any more); after the
  // barrier wave w sums blocks w, w + 4, ... of all four states with the weights
  // 2^(m_w' - max m), in wave order, and stores them.
  {
    unsigned char* mine = wave_lds;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      unsigned char* base = mine + rt * (NBLK * 1024 + 512);
#pragma unroll
      for (int b = 0; b < DB; ++b) *reinterpret_cast<f32x4*>(base + b * 1024 + lane * 16) = o_acc[rt][b];
#pragma unroll
      for (int b = 0; b < RB; ++b) *reinterpret_cast<f32x4*>(base + (DB + b) * 1024 + lane * 16) = lr_acc[rt][b];
      const float lsum = sum_over_lane_groups(l_run[rt]);
      *reinterpret_cast<f32x2*>(base + NBLK * 1024 + lane * 8) = f32x2{m_run[rt], lsum};
    }
  }
  __syncthreads();
  LRA_STAMP(6);
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    float wgt[NW], m_all = -INFINITY, l_all = 0.f;
    f32x2 ml[NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      ml[w] = *reinterpret_cast<const f32x2*>(smem + w * WAVE_BYTES + rt * (NBLK * 1024 + 512) + NBLK * 1024 + lane * 8);
      m_all = fmaxf(m_all, ml[w][0]);
    }
    // m_all is finite (wave 0 always owns a key) unless a causal row sees none of this split
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      wgt[w] = ml[w][0] == -INFINITY ? 0.f : fast_exp2(ml[w][0] - m_all);
      l_all = fmaf(wgt[w], ml[w][1], l_all);
    }
    if (out_row[rt] < 0) continue;
    const int64_t slot = static_cast<int64_t>(out_row[rt]) * p.n_splits + split;
#pragma unroll
    for (int x = 0; x < NBLK; ++x) {
      if ((x & (NW - 1)) != wave) continue;  // wave-uniform
      f32x4 v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const f32x4 part = *reinterpret_cast<const f32x4*>(smem + w * WAVE_BYTES + rt * (NBLK * 1024 + 512) + x * 1024 + lane * 16);
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) v[jj] = fmaf(wgt[w], part[jj], v[jj]);
      }
      if (x < DB) {
        *reinterpret_cast<f32x4*>(p.part_o + slot * D + x * 16 + lg * 4) = v;
      } else {
        // the rank is a multiple of 8: four entries are inside or outside together.  With per-adapter
        // caches a row keeps the block of its own agent slot only.
        int rho = (x - DB) * 16 + lg * 4;
        bool mine = true;
        if (per_agent) {
          const int blk = (x - DB) >> (lcs - 1);
          mine = blk == (ln >> gps);
          rho -= blk * lb;
        }
        if (mine && rho < r) *reinterpret_cast<f32x4*>(p.part_lr + slot * r + rho) = v;
      }
    }
    if (wave == NW - 1 && lg == 0) {
      p.part_ml[slot * 2 + 0] = m_all * 0.69314718055994530942f;  // natural-log units
      p.part_ml[slot * 2 + 1] = l_all;
      if (split == 0) p.part_adapter[out_row[rt]] = max(slot_adapter(rt, ln >> gps), 0);
    }
  }
  LRA_STAMP(11);
  LRA_STAMP_FLUSH();
}

// Qt = Q B_K^T for every row of a decode call, once per call instead of once per workgroup of
// the streaming kernel (App. D.1: the query-side projection of the key-side reordering).  With
// many agents and a large rank every key share of a kv head would otherwise reload the B_K rows of
// all its agents (config "8 agents, r = 64": 128 KB per workgroup, 32 workgroups per head).
// One workgroup per (kv head, row tile, agent slot); wave = rho block.  Output: the operand-ready
// layout the streaming kernel keeps in LDS, [row group][kv head][row tile][k-step][lane] 16 bytes,
// elements e -> rho = 32ks' + 16(e/4) + 4lg + e%4.
template <int D, int RP, bool CAUSAL>
__global__ __launch_bounds__(256) void decode_qt_prepass_kernel(Params p, int row_tiles) {
  constexpr int KS = D / 32, RKS = RP / 32, ROW_BYTES = D * 2;
  const int lane = threadIdx.x & 63;
  const int cb = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // rho block of this wave
  const int ln = lane & 15, lg = lane >> 4;
  // (the parameter block in one round trip; row_tiles is 1 or 2: no division)
  asm volatile("" ::"s"(p.q), "s"(p.b_k), "s"(p.query_adapter), "s"(p.qt_ws));
  asm volatile("" ::"s"(p.n_q_heads), "s"(p.n_kv_heads), "s"(p.group), "s"(p.rank), "s"(p.group_pad), "s"(p.n_queries),
               "s"(p.n_new), "s"(p.n_adapters), "s"(p.adapter_index), "s"(row_tiles));
  const int h = blockIdx.x, si = blockIdx.z;
  const int by = blockIdx.y;
  const int rg = row_tiles == 2 ? by >> 1 : by, rt = row_tiles == 2 ? by & 1 : 0;
  const int n_q = CAUSAL ? p.n_new : p.n_queries;
  const int GP = p.group_pad, G = p.group, r = p.rank;
  const int gps = __builtin_ctz(GP);
  const int ncb = (r + 15) >> 4;
  const int tile_row0 = (rg * row_tiles + rt) * 16;
  const int slot = (tile_row0 >> gps) + si;
  if (si >= (16 >> gps) || cb >= ncb) return;
  int a = -1;
  if (slot < n_q) a = min(max(CAUSAL ? p.adapter_index : CONST_I32(p.query_adapter)[slot], 0), p.n_adapters - 1);
  const bool live = a >= 0;
  const int64_t ldb = static_cast<int64_t>(p.n_kv_heads) * D;
  const __amdgpu_buffer_rsrc_t rs_q = make_rsrc(p.q, static_cast<uint32_t>(n_q) * p.n_q_heads * D * 2);
  const __amdgpu_buffer_rsrc_t rs_b =
      make_rsrc(static_cast<const bf16_t*>(p.b_k) + static_cast<int64_t>(live ? a : 0) * r * ldb + h * D,
                live ? static_cast<uint32_t>((r - 1) * ldb + D) * 2u : 0u);
  const int R = tile_row0 + ln;
  const int sq = R >> gps, gg = R & (GP - 1);
  const uint32_t qoff = (sq < n_q && gg < G) ? static_cast<uint32_t>((sq * p.n_q_heads + h * G + gg) * ROW_BYTES + lg * 16) : kOob;
  const uint32_t boff = static_cast<uint32_t>((cb * 16 + ln) * ldb * 2 + lg * 16);
  bf16x8 qv[KS], bv[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    qv[ks] = as_bf16x8(buf_load16(rs_q, qoff, ks * 64));
    bv[ks] = as_bf16x8(buf_load16(rs_b, boff, ks * 64));
  }
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bv[ks], qv[ks], acc, 0, 0, 0);
  if ((ln >> gps) == si) {
    unsigned char* dst = static_cast<unsigned char*>(p.qt_ws) +
                         ((((static_cast<size_t>(rg) * p.n_kv_heads + h) * row_tiles + rt) * RKS + (cb >> 1)) * 64 + lane) * 16;
    const uint2 pk = make_uint2(pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3]));
    if (!(cb & 1) && cb + 1 >= ncb)  // the odd block next to it lies beyond the rank: zeros
      *reinterpret_cast<uint4*>(dst) = make_uint4(pk.x, pk.y, 0u, 0u);
    else
      *reinterpret_cast<uint2*>(dst + (cb & 1) * 8) = pk;
  }
}

template <int D, int RP>
static void launch_prepass2(const Params& p, int row_tiles, hipStream_t s) {
  const dim3 grid(p.n_kv_heads, p.row_groups * row_tiles, 16 / p.group_pad), block(256);
  if (p.is_prefill) hipLaunchKernelGGL((decode_qt_prepass_kernel<D, RP, true>), grid, block, 0, s, p, row_tiles);
  else hipLaunchKernelGGL((decode_qt_prepass_kernel<D, RP, false>), grid, block, 0, s, p, row_tiles);
}

// Whether a decode launch can take decode_stream_kernel: contiguous cache, no rotary key side, at
// most one workgroup per compute unit.
bool decode_stream_applies(const Params& p, int row_tiles, int n_cus) {
  if (p.block_size != 0 || (p.key_rope_theta > 0.f && p.b_k != nullptr)) return false;
  if (row_tiles < 1 || row_tiles > 2) return false;
  const int64_t wgs = static_cast<int64_t>(p.n_kv_heads) * p.n_splits * p.row_groups;
  return wgs <= n_cus;
}

template <int D, int RT, int RP, bool SI>
static hipError_t launch_stream3(const Params& p, dim3 grid, hipStream_t s) {
  const dim3 block(512);
  const bool has_bk = p.b_k != nullptr;
  if (p.is_prefill) {
    if (has_bk) hipLaunchKernelGGL((decode_stream_kernel<D, RT, RP, true, true, false, SI>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((decode_stream_kernel<D, RT, RP, false, true, false, SI>), grid, block, 0, s, p);
  } else if (p.l_block != 0) {
    // per-adapter low-rank caches: one column block of the L tile per agent slot (one row tile only)
    if constexpr (RT == 1) {
      if (has_bk) hipLaunchKernelGGL((decode_stream_kernel<D, 1, RP, true, false, true, SI>), grid, block, 0, s, p);
      else hipLaunchKernelGGL((decode_stream_kernel<D, 1, RP, false, false, true, SI>), grid, block, 0, s, p);
    } else {
      return hipErrorInvalidValue;
    }
  } else {
    if (has_bk) hipLaunchKernelGGL((decode_stream_kernel<D, RT, RP, true, false, false, SI>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((decode_stream_kernel<D, RT, RP, false, false, false, SI>), grid, block, 0, s, p);
  }
  return hipGetLastError();
}

// Key ranges of at most two 32-key tiles per streaming wave take the split-issue form (where the
// LDS has room for the hand-over area next to the tile stages).
template <int D, int RT, int RP>
static hipError_t launch_stream2(const Params& p, dim3 grid, hipStream_t s) {
  constexpr bool can_split_issue = !(D == 128 && RP == 64);
  if constexpr (can_split_issue) {
    if (p.split_keys <= 256) return launch_stream3<D, RT, RP, true>(p, grid, s);
  }
  return launch_stream3<D, RT, RP, false>(p, grid, s);
}

// main_kernel_only (measurement): the streaming kernel alone, on whatever Qt an earlier call left
hipError_t launch_decode_stream(const Params& p, int row_tiles, bool main_kernel_only, hipStream_t s) {
  const dim3 grid = p.share_major ? dim3(8 * p.n_kv_heads, (p.n_splits + 7) / 8, p.row_groups)
                                  : dim3(p.n_kv_heads, p.n_splits, p.row_groups);  // (see the index layouts in the kernel)
  if (p.qt_ws != nullptr && !main_kernel_only) {
    if (p.head_dim == 128) { if (p.rank > 32) launch_prepass2<128, 64>(p, row_tiles, s); else launch_prepass2<128, 32>(p, row_tiles, s); }
    else { if (p.rank > 32) launch_prepass2<64, 64>(p, row_tiles, s); else launch_prepass2<64, 32>(p, row_tiles, s); }
    if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
  }
  // columns of the L tile: the rank, or with per-adapter low-rank caches one block per agent slot of a row tile
  const int tile_rank = (p.l_block != 0 && !p.is_prefill) ? (16 / p.group_pad) * p.l_block : p.rank;
  const int key = (p.head_dim == 128 ? 4 : 0) | (row_tiles == 2 ? 2 : 0) | (tile_rank > 32 ? 1 : 0);
  switch (key) {
    case 0: return launch_stream2<64, 1, 32>(p, grid, s);
    case 1: return launch_stream2<64, 1, 64>(p, grid, s);
    case 2: return launch_stream2<64, 2, 32>(p, grid, s);
    case 3: return launch_stream2<64, 2, 64>(p, grid, s);
    case 4: return launch_stream2<128, 1, 32>(p, grid, s);
    case 5: return launch_stream2<128, 1, 64>(p, grid, s);
    case 6: return launch_stream2<128, 2, 32>(p, grid, s);
    default: return launch_stream2<128, 2, 64>(p, grid, s);
  }
}

}  // namespace lra
