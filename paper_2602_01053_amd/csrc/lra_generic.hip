// Vector-ALU kernels of the Flash-LoRA-Attention library: a straightforward
// wave-per-row partial-attention kernel for any dtype, and the split merge +
// epilogue kernel every decode path ends with.
//
// Partial kernel: Alg. 1 (LRAgent, Sec. 3.3) for one query row and one range of
// keys, with the key-side reordering of App. D.1:
//     s_j  = scale * ( q . K_base[j] + (q B_K^T) . L[j] )
//     m, l = online softmax statistics,  O += p_j V_base[j],  O_lr += p_j L[j]
// The epilogue O += O_lr B_V and the division by l (the last two steps of Alg. 1) happen in
// the merge kernel, after the per-split states are combined.
#include "lra_common.h"

namespace lra {

// row . vec, the row read in 16-byte pieces where its length and address allow (every lane of these kernels walks
// a row of its own, so a piece is one cache-line touch instead of four or eight)
template <typename T>
__device__ __forceinline__ float dot_row(const T* __restrict__ row, const float* __restrict__ vec, int len) {
  constexpr int PER = 16 / static_cast<int>(sizeof(T));  // elements per piece: 4 (fp32) or 8 (bf16)
  float acc = 0.f;
  if (len % PER == 0 && (reinterpret_cast<uintptr_t>(row) & 15) == 0) {
    for (int c = 0; c < len; c += PER) {
      const uint4 piece = *reinterpret_cast<const uint4*>(row + c);
      const uint32_t w[4] = {piece.x, piece.y, piece.z, piece.w};
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        float x;
        if constexpr (sizeof(T) == 4) x = __uint_as_float(w[e]);
        else x = __uint_as_float((e & 1) ? (w[e >> 1] & 0xffff0000u) : (w[e >> 1] << 16));
        acc = fmaf(x, vec[c + e], acc);
      }
    }
    return acc;
  }
  for (int c = 0; c < len; ++c) acc = fmaf(to_f32<T>(row[c]), vec[c], acc);
  return acc;
}

template <typename T>
__global__ __launch_bounds__(kWave) void generic_partial_kernel(Params p) {
  const int row = blockIdx.x;
  const int split = blockIdx.y;
  const int lane = threadIdx.x;
  const int Hq = p.n_q_heads, d = p.head_dim, r = p.rank;
  const int tok = row / Hq;
  const int g = row - tok * Hq;
  const int h = g / p.group;

  int t, a, n_vis;
  if (p.is_prefill) {
    t = p.seq_index;
    a = p.adapter_index;
    const int n_t = min(p.seq_lens[t], p.max_seq_len);
    n_vis = n_t - p.n_new + tok + 1;
  } else {
    t = 0;
    while (t + 1 < p.n_seqs && p.seq_query_start[t + 1] <= tok) ++t;
    a = min(max(p.query_adapter[tok], 0), p.n_adapters - 1);  // ids are device data: kept inside the table
    n_vis = min(p.seq_lens[t], p.max_seq_len);
  }
  const int j0 = split * p.split_keys;
  const int j1 = min(j0 + p.split_keys, n_vis);

  __shared__ float q_s[128];
  __shared__ float qt_s[64];
  const T* q = static_cast<const T*>(p.q) + static_cast<int64_t>(row) * d;
  for (int c = lane; c < d; c += kWave) q_s[c] = to_f32<T>(q[c]);
  __syncthreads();
  if (lane < r) {
    float acc = 0.f;
    if (p.b_k != nullptr) {
      const T* bk = static_cast<const T*>(p.b_k) +
                    (static_cast<int64_t>(a) * r + lane) * (static_cast<int64_t>(p.n_kv_heads) * d) + h * d;
      acc = dot_row<T>(bk, q_s, d);
    }
    qt_s[lane] = acc;
  }
  __syncthreads();

  const T* kb = static_cast<const T*>(p.k_base);
  const T* vb = static_cast<const T*>(p.v_base);
  const T* lr = static_cast<const T*>(p.l);

  float m = -INFINITY, ell = 0.f, o0 = 0.f, o1 = 0.f, olr = 0.f;
  for (int jb = j0; jb < j1; jb += kWave) {
    const int j = jb + lane;
    const bool valid = j < j1;
    float s = -INFINITY;
    if (valid) {
      const float sk = dot_row<T>(kb + kv_offset(p, t, j, h), q_s, d);
      const float sl = dot_row<T>(lr + l_offset(p, t, j, a), qt_s, r);
      s = p.scale * (sk + sl);
    }
    const float m_new = fmaxf(m, wave_max(s));  // finite: lane 0 is always valid here
    const float alpha = (m == -INFINITY) ? 0.f : expf(m - m_new);
    const float pj = valid ? expf(s - m_new) : 0.f;
    ell = alpha * ell + wave_sum(pj);
    o0 *= alpha;
    o1 *= alpha;
    olr *= alpha;
    // O += p_j V_j, O_lr += p_j L_j: lane = column.  Eight keys' rows are requested before the first is used (one
    // row per trip would pay a memory round trip per key); every load is unconditional from a clamped index, what
    // it fetched in vain is not added.
    const int cnt = min(kWave, j1 - jb);
    const int c0 = min(lane, d - 1), c1 = min(lane + kWave, d - 1), cl = min(lane, r - 1);
    for (int jj0 = 0; jj0 < cnt; jj0 += 8) {
      float v0[8], v1[8], vl[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int jk = jb + min(jj0 + u, cnt - 1);
        const T* v = vb + kv_offset(p, t, jk, h);
        v0[u] = to_f32<T>(v[c0]);
        v1[u] = to_f32<T>(v[c1]);
        vl[u] = to_f32<T>(lr[l_offset(p, t, jk, a) + cl]);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (jj0 + u < cnt) {  // (uniform)
          const float pjj = __shfl(pj, jj0 + u, kWave);
          o0 = fmaf(pjj, v0[u], o0);
          o1 = fmaf(pjj, v1[u], o1);
          olr = fmaf(pjj, vl[u], olr);
        }
      }
    }
    m = m_new;
  }

  const int64_t slot = static_cast<int64_t>(row) * p.n_splits + split;
  if (lane == 0) {
    p.part_ml[slot * 2 + 0] = m;  // a split past the row's last visible key leaves (-inf, 0)
    p.part_ml[slot * 2 + 1] = ell;
    if (split == 0) p.part_adapter[row] = a;
  }
  if (lane < d) p.part_o[slot * d + lane] = o0;
  if (lane + kWave < d) p.part_o[slot * d + lane + kWave] = o1;
  if (lane < r) p.part_lr[slot * r + lane] = olr;
}

// The same for the rotary key side (App. D.1 with the rotation in place: LoRA on the key
// projection of a model with rotary embeddings).  K_j = K_base,j + RoPE_j(L_j B_K): the
// rotation sits between L_j B_K and the score, so (q B_K^T) . L_j no longer applies.  With
// rotate-half pairs (i, i + h), h = d/2, and c_i, s_i the cosine and sine of j * theta^(-2i/d),
//     q . RoPE_j(L_j B) = sum_i  c_i (L_j . U_i) + s_i (L_j . W_i),
//     U_i[rho] = q_i B[rho][i] + q_{i+h} B[rho][i+h],   W_i[rho] = q_{i+h} B[rho][i] - q_i B[rho][i+h],
// r-vectors per pair that depend on the query row only.  The wave forms U and W once in LDS,
// stages the L rows of its 64 keys there as well, and every lane (one key) sums over the
// pairs.  r * d multiply-adds per (row, key) instead of d + r: the price of the rotation
// without materialising the keys.  Angles as in the cache-append producer: rates in double
// precision and revolutions, fractional part, v_sin_f32 / v_cos_f32.
template <typename T>
__global__ __launch_bounds__(kWave) void generic_partial_rope_kernel(Params p) {
  const int row = blockIdx.x;
  const int split = blockIdx.y;
  const int lane = threadIdx.x;
  const int Hq = p.n_q_heads, d = p.head_dim, r = p.rank, half = d / 2;
  const int tok = row / Hq;
  const int g = row - tok * Hq;
  const int h = g / p.group;

  int t, a, n_vis;
  if (p.is_prefill) {
    t = p.seq_index;
    a = p.adapter_index;
    const int n_t = min(p.seq_lens[t], p.max_seq_len);
    n_vis = n_t - p.n_new + tok + 1;
  } else {
    t = 0;
    while (t + 1 < p.n_seqs && p.seq_query_start[t + 1] <= tok) ++t;
    a = min(max(p.query_adapter[tok], 0), p.n_adapters - 1);  // ids are device data: kept inside the table
    n_vis = min(p.seq_lens[t], p.max_seq_len);
  }
  const int j0 = split * p.split_keys;
  const int j1 = min(j0 + p.split_keys, n_vis);

  __shared__ float q_s[128];
  __shared__ float u_s[64 * 64];   // [rho][i], i < d/2
  __shared__ float w_s[64 * 64];
  __shared__ float l_s[64 * 65];   // [key of the step][rho], rows padded to 65 floats
  __shared__ double rate_s[64];    // revolutions per position of pair i
  const T* q = static_cast<const T*>(p.q) + static_cast<int64_t>(row) * d;
  for (int c = lane; c < d; c += kWave) q_s[c] = to_f32<T>(q[c]);
  if (lane < half)
    rate_s[lane] = exp2(-2.0 * lane / d * log2(static_cast<double>(p.key_rope_theta))) * 0.15915494309189533577;
  __syncthreads();
  {
    const T* bk = static_cast<const T*>(p.b_k) + static_cast<int64_t>(a) * r * (static_cast<int64_t>(p.n_kv_heads) * d) + h * d;
    for (int e = lane; e < r * half; e += kWave) {
      const int rho = e / half, i = e - rho * half;
      const float b_lo = to_f32<T>(bk[static_cast<int64_t>(rho) * p.n_kv_heads * d + i]);
      const float b_hi = to_f32<T>(bk[static_cast<int64_t>(rho) * p.n_kv_heads * d + i + half]);
      u_s[rho * 64 + i] = q_s[i] * b_lo + q_s[i + half] * b_hi;
      w_s[rho * 64 + i] = q_s[i + half] * b_lo - q_s[i] * b_hi;
    }
  }
  __syncthreads();

  const T* kb = static_cast<const T*>(p.k_base);
  const T* vb = static_cast<const T*>(p.v_base);
  const T* lr = static_cast<const T*>(p.l);

  float m = -INFINITY, ell = 0.f, o0 = 0.f, o1 = 0.f, olr = 0.f;
  for (int jb = j0; jb < j1; jb += kWave) {
    const int j = jb + lane;
    const bool valid = j < j1;
    // this lane's L row, as floats, where the lane can index it with a loop variable
    if (valid) {
      const T* lrow = lr + l_offset(p, t, j, a);
      for (int rho = 0; rho < r; ++rho) l_s[lane * 65 + rho] = to_f32<T>(lrow[rho]);
    }
    __syncthreads();  // one wave: orders the staging against the other lanes' reads below
    float s = -INFINITY;
    if (valid) {
      const float sk = dot_row<T>(kb + kv_offset(p, t, j, h), q_s, d);
      float sl = 0.f;
      for (int i = 0; i < half; ++i) {
        float u = 0.f, w = 0.f;
        for (int rho = 0; rho < r; ++rho) {
          const float lv = l_s[lane * 65 + rho];
          u = fmaf(lv, u_s[rho * 64 + i], u);
          w = fmaf(lv, w_s[rho * 64 + i], w);
        }
        double rev = static_cast<double>(j) * rate_s[i];
        rev -= floor(rev);
        const float fr = static_cast<float>(rev);
        sl = fmaf(__builtin_amdgcn_cosf(fr), u, fmaf(__builtin_amdgcn_sinf(fr), w, sl));
      }
      s = p.scale * (sk + sl);
    }
    const float m_new = fmaxf(m, wave_max(s));  // finite: lane 0 is always valid here
    const float alpha = (m == -INFINITY) ? 0.f : expf(m - m_new);
    const float pj = valid ? expf(s - m_new) : 0.f;
    ell = alpha * ell + wave_sum(pj);
    o0 *= alpha;
    o1 *= alpha;
    olr *= alpha;
    // (as in generic_partial_kernel: the V rows of eight keys requested before the first is used)
    const int cnt = min(kWave, j1 - jb);
    const int c0 = min(lane, d - 1), c1 = min(lane + kWave, d - 1);
    for (int jj0 = 0; jj0 < cnt; jj0 += 8) {
      float v0[8], v1[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const T* v = vb + kv_offset(p, t, jb + min(jj0 + u, cnt - 1), h);
        v0[u] = to_f32<T>(v[c0]);
        v1[u] = to_f32<T>(v[c1]);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (jj0 + u < cnt) {  // (uniform)
          const float pjj = __shfl(pj, jj0 + u, kWave);
          o0 = fmaf(pjj, v0[u], o0);
          o1 = fmaf(pjj, v1[u], o1);
          if (lane < r) olr = fmaf(pjj, l_s[(jj0 + u) * 65 + lane], olr);
        }
      }
    }
    m = m_new;
    __syncthreads();  // before the next step overwrites the staged rows
  }

  const int64_t slot = static_cast<int64_t>(row) * p.n_splits + split;
  if (lane == 0) {
    p.part_ml[slot * 2 + 0] = m;  // a split past the row's last visible key leaves (-inf, 0)
    p.part_ml[slot * 2 + 1] = ell;
    if (split == 0) p.part_adapter[row] = a;
  }
  if (lane < d) p.part_o[slot * d + lane] = o0;
  if (lane + kWave < d) p.part_o[slot * d + lane + kWave] = o1;
  if (lane < r) p.part_lr[slot * r + lane] = olr;
}

// Flash-decoding merge of the per-split states followed by Alg. 1's epilogue:
//   M = max_s m_s, w_s = exp(m_s - M), l = sum w_s l_s, O = sum w_s O_s,
//   O_lr = sum w_s O_lr,s ;  out = (O + O_lr B_V) / l.
// One workgroup of 128 x kMergeGroups threads per query row.  Thread (c, g) owns
// column c of the splits s = g, g + kMergeGroups, ... and, for the epilogue, the
// B_V rows rho = g, g + kMergeGroups, ...  All of a thread's global loads (split
// statistics, partial rows, B_V) are issued before the first one is consumed, so
// the kernel costs about two memory round trips.  Groups are added in a fixed
// order: the result does not depend on which workgroup of the first kernel
// finished first.
constexpr int kMergeUnroll = 8;  // splits per thread and pass
// Rows from which the wave-per-row form of the merge runs (measured on MI355X: 1792 rows of config
// 5 take 12.7 us against 20.5 us; 256 rows of config 4 take 10.4 us against 9.3 us).
constexpr int kMergeWaveRows = 1024;

#ifdef LRA_TIMING
#define LRA_MSTAMP(k) do { unsigned long long t_; asm volatile("s_waitcnt lgkmcnt(0)\n\ts_memrealtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(t_)); mt[k] = t_; } while (0)
#else
#define LRA_MSTAMP(k)
#endif

template <typename T, int kMergeGroups>
__global__ __launch_bounds__(128 * kMergeGroups) void merge_kernel(Params p) {
#ifdef LRA_TIMING
  unsigned long long mt[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#endif
  LRA_MSTAMP(0);
  // Workgroups go round-robin over the XCDs; numbering them kv head first puts the rows of
  // kv head h on the XCD(s) where the streaming kernel wrote that head's partial states.
  const int Hq = p.n_q_heads, d = p.head_dim, r = p.rank;
  const int h = blockIdx.x % p.n_kv_heads;
  const int rest = blockIdx.x / p.n_kv_heads;
  const int tok = rest / p.group;
  const int g = h * p.group + rest % p.group;
  const int row = tok * Hq + g;
  const int c = threadIdx.x, gq = threadIdx.y;
  const int tid = gq * 128 + c;
  // Everything this kernel needs was left in the workspace by the first kernel: the row's
  // adapter, and a zero row sum in every split that had no visible key (its O and O_lr rows
  // were never written and are ignored below).  No sequence table is read here.
  const int ns = p.n_splits;
  // (clamped: whatever the workspace holds, the B_V rows read below exist)
  const int a = min(max(p.part_adapter[row], 0), p.n_adapters - 1);
#ifdef LRA_TIMING
  asm volatile("" ::"v"(a));
#endif
  LRA_MSTAMP(1);
  const int64_t slot0 = static_cast<int64_t>(row) * p.n_splits;
  const float2* ml = reinterpret_cast<const float2*>(p.part_ml) + slot0;
  const float* po = p.part_o + slot0 * d + c;
  const float* pl = p.part_lr + slot0 * r + c;
  const bool col_o = c < d, col_l = c < r;

  __shared__ float red[2 * kMergeGroups];
  __shared__ float o_sh[kMergeGroups][128];
  __shared__ float olr_sh[kMergeGroups][64];
  __shared__ float ell_sh[kMergeGroups];

  // ---- issue: statistics for the row maximum, first pass of partial rows, B_V rows ----
  float big = -INFINITY;
  for (int s = tid; s < ns; s += 128 * kMergeGroups) {
    const float2 v = ml[s];
    if (v.y > 0.f) big = fmaxf(big, v.x);
  }
  float2 st[kMergeUnroll];
  float xo[kMergeUnroll], xl[kMergeUnroll];
#pragma unroll
  for (int i = 0; i < kMergeUnroll; ++i) {
    const int s = i * kMergeGroups + gq;
    const bool ok = s < ns;
    st[i] = ok ? ml[s] : make_float2(0.f, 0.f);
    xo[i] = (ok && col_o) ? po[static_cast<int64_t>(s) * d] : 0.f;
    xl[i] = (ok && col_l) ? pl[static_cast<int64_t>(s) * r] : 0.f;
  }
  float bvv[64 / kMergeGroups];
  {
    const int64_t ld = static_cast<int64_t>(p.n_kv_heads) * d;
    const T* bv = static_cast<const T*>(p.b_v) + static_cast<int64_t>(a) * r * ld + h * d + c;
#pragma unroll
    for (int i = 0; i < 64 / kMergeGroups; ++i) {
      const int rho = i * kMergeGroups + gq;
      bvv[i] = (p.b_v != nullptr && col_o && rho < r) ? to_f32<T>(bv[rho * ld]) : 0.f;
    }
  }

  LRA_MSTAMP(2);
  big = wave_max(big);
  if ((tid & 63) == 0) red[tid >> 6] = big;
  __syncthreads();
  LRA_MSTAMP(3);
  big = red[0];
#pragma unroll
  for (int i = 1; i < 2 * kMergeGroups; ++i) big = fmaxf(big, red[i]);

  float ell = 0.f, o = 0.f, olr = 0.f;
#pragma unroll
  for (int i = 0; i < kMergeUnroll; ++i) {
    const bool live = st[i].y > 0.f;
    const float w = live ? expf(st[i].x - big) : 0.f;
    ell = fmaf(w, st[i].y, ell);
    o = fmaf(w, live ? xo[i] : 0.f, o);
    olr = fmaf(w, live ? xl[i] : 0.f, olr);
  }
  // further passes, only for more than kMergeGroups * kMergeUnroll splits
  for (int s = kMergeGroups * kMergeUnroll + gq; s < ns; s += kMergeGroups) {
    const float2 v = ml[s];
    const float x = col_o ? po[static_cast<int64_t>(s) * d] : 0.f;
    const float y = col_l ? pl[static_cast<int64_t>(s) * r] : 0.f;
    const bool live = v.y > 0.f;
    const float w = live ? expf(v.x - big) : 0.f;
    ell = fmaf(w, v.y, ell);
    o = fmaf(w, live ? x : 0.f, o);
    olr = fmaf(w, live ? y : 0.f, olr);
  }
  if (c < 64) olr_sh[gq][c] = olr;
  if (c == 0) ell_sh[gq] = ell;
  LRA_MSTAMP(4);
  __syncthreads();
  // epilogue O += O_lr B_V: group g contributes its rows rho = g, g + kMergeGroups, ...
#pragma unroll
  for (int i = 0; i < 64 / kMergeGroups; ++i) {
    const int rho = i * kMergeGroups + gq;
    if (rho < r) {
      float x = olr_sh[0][rho];
#pragma unroll
      for (int k = 1; k < kMergeGroups; ++k) x += olr_sh[k][rho];
      o = fmaf(x, bvv[i], o);
    }
  }
  o_sh[gq][c] = o;
  __syncthreads();
  if (gq == 0 && col_o) {
    o = o_sh[0][c];
    ell = ell_sh[0];
#pragma unroll
    for (int k = 1; k < kMergeGroups; ++k) {
      o += o_sh[k][c];
      ell += ell_sh[k];
    }
    static_cast<T*>(p.out)[static_cast<int64_t>(row) * d + c] = from_f32<T>(o / ell);
  }
  LRA_MSTAMP(5);
#ifdef LRA_TIMING
  if (p.timing && (tid & 63) == 0) {
    unsigned long long* o_ = p.timing + 4096 * 128 + static_cast<size_t>(blockIdx.x) * 64 + (tid >> 6) * 8;
    for (int i_ = 0; i_ < 6; ++i_) o_[i_] = mt[i_];
  }
#endif
}

// The same merge with wide loads, for the common case (head dimension 64 or 128, rank a multiple of
// 4, at most 64 splits): one workgroup of 256 threads per query row.
//   - lane = split for the statistics: every wave forms the flash-decoding weights w_s on its own
//     (one 8-byte load per lane), so no barrier stands before the partial rows can be weighted;
//   - O rows as float4: thread (split group sg, column quad cq) sums splits sg, sg + SG, ...;
//   - O_lr rows as float4: thread (split group of 16, quad q < r/4);
//   - the B_V slice of the row's adapter and kv head ([r][d] elements) travels to LDS in 16-byte
//     pieces; the epilogue O += O_lr B_V reads it from there.
// Three barriers; every sum runs in a fixed order (splits ascending inside a thread, groups
// ascending across threads), so the result does not depend on which workgroup of the first
// kernel finished first.  All loads of a thread are issued before the first is consumed.
template <typename T, int D>
__global__ __launch_bounds__(256) void merge_rows_kernel(Params p) {
  constexpr int CQ = D / 4;        // column quads of an O row
  constexpr int SG = 256 / CQ;     // split groups for the O rows
  constexpr int OP = 64 / SG;      // passes over at most 64 splits
  constexpr int BV_PIECES = 64 * D * static_cast<int>(sizeof(T)) / 16 / 256;  // 16-byte pieces of B_V per thread at r = 64
  // This kernel is a chain of latencies (launch, parameter block, the row's adapter id, the loads,
  // two barriers), so nothing may stand between them: the parameter block is fetched in one round
  // trip (left alone the compiler fetches it piece by piece behind each use), the grid is (kv head,
  // q head of the group, query) so that no index needs a division, and every load is unconditional
  // from a clamped index (a load under a condition, with zero as the other value, makes the compiler
  // wait for it on the spot: both write the same register); what a clamped index fetched in vain
  // gets weight zero below.
  asm volatile("" ::"s"(p.part_adapter), "s"(p.part_ml), "s"(p.part_o), "s"(p.part_lr), "s"(p.b_v), "s"(p.out));
  asm volatile("" ::"s"(p.n_q_heads), "s"(p.n_kv_heads), "s"(p.group), "s"(p.head_dim), "s"(p.rank), "s"(p.n_splits),
               "s"(p.n_adapters));
  const int Hq = p.n_q_heads, r = p.rank, ns = p.n_splits;
  const int h = blockIdx.x;
  const int row = static_cast<int>(blockIdx.z) * Hq + h * p.group + static_cast<int>(blockIdx.y);
  const int tid = threadIdx.x, lane = tid & 63;
  const int64_t slot0 = static_cast<int64_t>(row) * ns;

  __shared__ __align__(16) float o_sh[SG][D];
  __shared__ __align__(16) float lr_sh[16][64];
  __shared__ __align__(16) float olr_tot[64];
  __shared__ __align__(16) unsigned char bv_sh[64 * D * sizeof(T)];

  // the row's adapter first: the B_V rows depend on it (clamped: whatever the workspace holds, the
  // B_V rows read below exist)
  // (requested here by hand and waited for where the B_V addresses are formed: left to the compiler
  // the request sinks below the vector loads, and its round trip is then paid after theirs)
  int a_raw;
  asm volatile("s_load_dword %0, %1, 0x0" : "=s"(a_raw) : "s"(p.part_adapter + row));

  // ---- issue everything ----
  const float2 st_raw = reinterpret_cast<const float2*>(p.part_ml)[slot0 + min(lane, ns - 1)];
  const int sg = tid / CQ, cq = tid % CQ;
  float4 xo[OP];
#pragma unroll
  for (int k = 0; k < OP; ++k)
    xo[k] = *reinterpret_cast<const float4*>(p.part_o + (slot0 + min(sg + SG * k, ns - 1)) * D + cq * 4);
  const int lg16 = tid >> 4, q = tid & 15;
  const bool q_live = q * 4 < r;
  float4 xl[4];
#pragma unroll
  for (int k = 0; k < 4; ++k)
    xl[k] = *reinterpret_cast<const float4*>(p.part_lr + (slot0 + min(lg16 + 16 * k, ns - 1)) * r + (q_live ? q * 4 : 0));
  constexpr int ROW_PIECES = D * static_cast<int>(sizeof(T)) / 16;  // 16-byte pieces per B_V row of one kv head
  uint4 bvp[BV_PIECES];
  asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(a_raw));
  const int a = min(max(a_raw, 0), p.n_adapters - 1);
  // (Requesting the slices of all adapters of a small table next to the partial rows, to pick the row's
  // own when its id arrives, takes one dependent round trip off the path and was measured 0.8 us slower.)
  if (p.b_v != nullptr) {  // (uniform)
    const int64_t ld = static_cast<int64_t>(p.n_kv_heads) * D;
    const T* bv = static_cast<const T*>(p.b_v) + static_cast<int64_t>(a) * r * ld + h * D;
#pragma unroll
    for (int k = 0; k < BV_PIECES; ++k) {
      const int e = tid + 256 * k;
      const int rho = min(e / ROW_PIECES, r - 1), pc = e % ROW_PIECES;  // (rows beyond the rank: fetched again, never read)
      bvp[k] = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(bv + rho * ld) + pc * 16);
    }
  } else {
#pragma unroll
    for (int k = 0; k < BV_PIECES; ++k) bvp[k] = make_uint4(0u, 0u, 0u, 0u);
  }
  const float2 st = lane < ns ? st_raw : make_float2(0.f, 0.f);

  // ---- weights (per wave, lane = split) ----
  const bool live = st.y > 0.f;  // a share without a visible key left a zero row sum; its rows were never written
  const float big = wave_max(live ? st.x : -INFINITY);
  const float w = live ? expf(st.x - big) : 0.f;
  const float ell = wave_sum(w * st.y);

  // ---- weighted sums of this thread's splits ----
  float4 o = make_float4(0.f, 0.f, 0.f, 0.f), olr = o;
#pragma unroll
  for (int k = 0; k < OP; ++k) {
    const float wk = __shfl(w, min(sg + SG * k, 63), kWave);
    if (sg + SG * k < ns && wk > 0.f) {  // also keeps whatever an unwritten row holds out of the sums
      o.x = fmaf(wk, xo[k].x, o.x);
      o.y = fmaf(wk, xo[k].y, o.y);
      o.z = fmaf(wk, xo[k].z, o.z);
      o.w = fmaf(wk, xo[k].w, o.w);
    }
  }
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const float wk = __shfl(w, lg16 + 16 * k, kWave);
    if (lg16 + 16 * k < ns && wk > 0.f && q_live) {
      olr.x = fmaf(wk, xl[k].x, olr.x);
      olr.y = fmaf(wk, xl[k].y, olr.y);
      olr.z = fmaf(wk, xl[k].z, olr.z);
      olr.w = fmaf(wk, xl[k].w, olr.w);
    }
  }
  *reinterpret_cast<float4*>(&o_sh[sg][cq * 4]) = o;
  *reinterpret_cast<float4*>(&lr_sh[lg16][q * 4]) = olr;
#pragma unroll
  for (int k = 0; k < BV_PIECES; ++k) *reinterpret_cast<uint4*>(bv_sh + (tid + 256 * k) * 16) = bvp[k];
  __syncthreads();
  if (tid < 64) {
    float x = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) x += lr_sh[k][tid];
    olr_tot[tid] = x;
  }
  __syncthreads();
  if (tid < D) {
    float x = 0.f;
#pragma unroll
    for (int k = 0; k < SG; ++k) x += o_sh[k][tid];
    const T* bcol = reinterpret_cast<const T*>(bv_sh) + tid;
    for (int rho = 0; rho < r; ++rho) x = fmaf(olr_tot[rho], to_f32<T>(bcol[rho * D]), x);
    static_cast<T*>(p.out)[static_cast<int64_t>(row) * D + tid] = from_f32<T>(x / ell);
  }
}

// The same merge for calls with many rows: one wave per row (four rows, q heads of one kv
// head, per workgroup), no LDS and no barrier, so that a CU holds twenty rows' worth of loads
// in flight instead of four.  Lane = split for the statistics (at most 64 splits), lane =
// column (pair of columns at d = 128) for the rows; the weight of a split and the entries of
// O_lr travel by v_readlane.  Splits are added in index order.
template <typename T, int D>
__global__ __launch_bounds__(256) void merge_wave_kernel(Params p) {
  constexpr int CPL = D / 64;  // columns per lane: c = CPL * lane + k
  // (as in merge_rows_kernel: the parameter block in one round trip, a grid (kv head, group of four q
  // heads, query) without divisions, the adapter id requested by hand ahead of the vector loads, and
  // unconditional loads from clamped indices)
  asm volatile("" ::"s"(p.part_adapter), "s"(p.part_ml), "s"(p.part_o), "s"(p.part_lr), "s"(p.b_v), "s"(p.out));
  asm volatile("" ::"s"(p.n_q_heads), "s"(p.n_kv_heads), "s"(p.group), "s"(p.head_dim), "s"(p.rank), "s"(p.n_splits),
               "s"(p.n_adapters));
  const int Hq = p.n_q_heads, r = p.rank, G = p.group;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int h = blockIdx.x;
  const int gq = static_cast<int>(blockIdx.y) * 4 + wave;
  if (gq >= G) return;
  const int row = static_cast<int>(blockIdx.z) * Hq + h * G + gq;
  const int ns = p.n_splits;
  const int64_t slot0 = static_cast<int64_t>(row) * ns;
  int a_raw;
  asm volatile("s_load_dword %0, %1, 0x0" : "=s"(a_raw) : "s"(p.part_adapter + row));

  const float2 st_raw = reinterpret_cast<const float2*>(p.part_ml)[slot0 + min(lane, ns - 1)];
  const float2 st = lane < ns ? st_raw : make_float2(0.f, 0.f);
  const bool live = st.y > 0.f;  // a share without a visible key left a zero row sum; its rows were never written
  const float big = wave_max(live ? st.x : -INFINITY);
  const float w = live ? expf(st.x - big) : 0.f;
  const float ell = wave_sum(w * st.y);

  const float* po = p.part_o + slot0 * D + CPL * lane;
  const float* pl = p.part_lr + slot0 * r + (lane < r ? lane : 0);
  float o[CPL], olr = 0.f;
#pragma unroll
  for (int k = 0; k < CPL; ++k) o[k] = 0.f;
  constexpr int U = 8;
  for (int s0 = 0; s0 < ns; s0 += U) {
    float x[U][CPL], y[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int sidx = min(s0 + u, ns - 1);
      if (CPL == 2) {
        const float2 v = *reinterpret_cast<const float2*>(po + static_cast<int64_t>(sidx) * D);
        x[u][0] = v.x;
        x[u][CPL - 1] = v.y;
      } else {
        x[u][0] = po[static_cast<int64_t>(sidx) * D];
      }
      y[u] = pl[static_cast<int64_t>(sidx) * r];  // (lanes beyond the rank read column 0; their sums are never used)
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float wu = (s0 + u < ns) ? __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, w), (s0 + u) & 63)) : 0.f;
      if (wu > 0.f) {  // wave-uniform; also keeps whatever an unwritten row holds out of the sums
#pragma unroll
        for (int k = 0; k < CPL; ++k) o[k] = fmaf(wu, x[u][k], o[k]);
        olr = fmaf(wu, y[u], olr);
      }
    }
  }
  // epilogue O += O_lr B_V, sixteen B_V rows requested at a time
  asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(a_raw));
  const int a = min(max(a_raw, 0), p.n_adapters - 1);
  if (p.b_v != nullptr) {
    const int64_t ld = static_cast<int64_t>(p.n_kv_heads) * D;
    const T* bv = static_cast<const T*>(p.b_v) + static_cast<int64_t>(a) * r * ld + h * D + CPL * lane;
    for (int r0 = 0; r0 < r; r0 += 16) {
      float b[16][CPL];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int rho = min(r0 + i, r - 1);
#pragma unroll
        for (int k = 0; k < CPL; ++k) b[i][k] = to_f32<T>(bv[rho * ld + k]);
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        if (r0 + i < r) {
          const float xr = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, olr), (r0 + i) & 63));
#pragma unroll
          for (int k = 0; k < CPL; ++k) o[k] = fmaf(xr, b[i][k], o[k]);
        }
      }
    }
  }
  T* out = static_cast<T*>(p.out) + static_cast<int64_t>(row) * D + CPL * lane;
#pragma unroll
  for (int k = 0; k < CPL; ++k) out[k] = from_f32<T>(o[k] / ell);
}

template <typename T>
static bool launch_merge_wave(const Params& p, int rows, hipStream_t s) {
  // worth it from a few hundred rows on; the statistics need one lane per split
  if (rows < kMergeWaveRows || p.n_splits > 64 || (p.head_dim != 64 && p.head_dim != 128)) return false;
  const int tokens = rows / p.n_q_heads;
  if (tokens > 65535) return false;  // (the query index is the grid's z)
  dim3 grid(p.n_kv_heads, (p.group + 3) / 4, tokens);
  if (p.head_dim == 128) hipLaunchKernelGGL((merge_wave_kernel<T, 128>), grid, dim3(256), 0, s, p);
  else hipLaunchKernelGGL((merge_wave_kernel<T, 64>), grid, dim3(256), 0, s, p);
  return true;
}

hipError_t launch_generic_partials(const Params& p, bool is_bf16, int rows, hipStream_t s) {
  dim3 grid(rows, p.n_splits), block(kWave);
  if (p.key_rope_theta > 0.f && p.b_k != nullptr) {
    if (is_bf16) hipLaunchKernelGGL(generic_partial_rope_kernel<bf16_t>, grid, block, 0, s, p);
    else hipLaunchKernelGGL(generic_partial_rope_kernel<float>, grid, block, 0, s, p);
    return hipGetLastError();
  }
  if (is_bf16)
    hipLaunchKernelGGL(generic_partial_kernel<bf16_t>, grid, block, 0, s, p);
  else
    hipLaunchKernelGGL(generic_partial_kernel<float>, grid, block, 0, s, p);
  return hipGetLastError();
}

template <typename T>
static void launch_merge_t(const Params& p, int rows, hipStream_t s) {
  if (launch_merge_wave<T>(p, rows, s)) return;
  if (p.rank % 4 == 0 && p.n_splits <= 64 && (p.head_dim == 64 || p.head_dim == 128) && rows / p.n_q_heads <= 65535) {
    // (kv head, q head of the group, query): workgroups go round-robin over the XCDs, so with 8 kv heads
    // the rows of a head are merged on one XCD
    const dim3 grid(p.n_kv_heads, p.group, rows / p.n_q_heads);
    if (p.head_dim == 128) hipLaunchKernelGGL((merge_rows_kernel<T, 128>), grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL((merge_rows_kernel<T, 64>), grid, dim3(256), 0, s, p);
    return;
  }
  // enough 128-thread groups that one pass of kMergeUnroll splits per thread covers the splits
  const int groups = (p.n_splits + kMergeUnroll - 1) / kMergeUnroll;
  dim3 grid(rows);
  if (groups <= 1)
    hipLaunchKernelGGL((merge_kernel<T, 1>), grid, dim3(128, 1), 0, s, p);
  else if (groups <= 2)
    hipLaunchKernelGGL((merge_kernel<T, 2>), grid, dim3(128, 2), 0, s, p);
  else if (groups <= 4)
    hipLaunchKernelGGL((merge_kernel<T, 4>), grid, dim3(128, 4), 0, s, p);
  else
    hipLaunchKernelGGL((merge_kernel<T, 8>), grid, dim3(128, 8), 0, s, p);
}

hipError_t launch_merge(const Params& p, bool is_bf16, int rows, hipStream_t s) {
  if (is_bf16)
    launch_merge_t<bf16_t>(p, rows, s);
  else
    launch_merge_t<float>(p, rows, s);
  return hipGetLastError();
}

}  // namespace lra
