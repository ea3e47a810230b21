// Decode step with a caller-supplied top-k set (the paper's pred-top-index hook, Section 4.1: any approximate
// top-k method may supply I_t): no pass over the whole K cache.  Scores exist only for the tokens that are
// attended:
//
//   sparse_score_kernel   s_i = sm_scale * <K[i], q> for the tokens of I_f and I_bs, written next to their
//                         places in the index lists
//   given_gather_kernel   the N and D sums of Section 4.1 over [I_f, I_dyn]: scores of I_f from the sparse
//                         list, scores of I_dyn computed here from their K rows (with nested samples the
//                         base-sample part of I_dyn has its scores in the list already); V rows gathered as
//                         in the dense-scored path.  No head maximum is known in advance, so every lane group keeps a
//                         running maximum and rescales (online softmax), and the merge combines the splits'
//                         (max, D, N) partials the same way.
//
// grid = (query heads, splits, sequences) for both, head fastest and in head_of_block order: the splits of a
// head, and the heads of a KV head, then share an XCD and its L2 (index lists, and the K and V rows they have in
// common); d/8 adjacent lanes read one K or V row with one 16-byte load each.
#include <type_traits>

#include "vatt_internal.h"

namespace vatt {
namespace {

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), acc,
                                         false);
}

struct GivenArgs {
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  KVLayout Lk, Lv;
  const HeadRec* head_rec;
  const int32_t* idx;
  float* sparse;      // [B*Hq][idx_cap]: score of the token at the same place of the index lists
  float* part;        // [B*Hq][splits][d + 4]: N[d], D, running maximum
  float* vstat;       // [B*Hq][splits][2d + 4]: N_f[d], R1[d], R2, maximum (numerator statistics, targets N / SDPA)
  float* out_o;
  float* out_lse;
  int64_t seg_sink, seg_win, seg_topk, seg_base, seg_dyn, idx_cap;
  int Hq, group, splits;
  int group_major;  // see head_of_block (the KV head count is Hq / group)
  int q_len;  // query tokens per sequence: blockIdx.z = sequence * q_len + query token
  float sm_scale;
  // random cache of base-sample rows: heads whose HeadRec.base_cached is set read their base sample's rows from it
  const void* rcache;
  CacheLayout rc;
  const int32_t* base_slot;  // [B*Hq][b0_max]
  int b0_max;
};

template <int D>
__device__ __forceinline__ void load_q(const GivenArgs& A, int bh, int sub, uint32_t (&qw)[4]) {
  const uint4 t = *reinterpret_cast<const uint4*>(A.q + (int64_t)bh * D + sub * 8);
  qw[0] = t.x;
  qw[1] = t.y;
  qw[2] = t.z;
  qw[3] = t.w;
}

template <int LPR>
__device__ __forceinline__ float row_score(const uint4& kv, const uint32_t (&qw)[4], float sm_scale) {
  float a = 0.f;
  a = dot2_bf16(kv.x, qw[0], a);
  a = dot2_bf16(kv.y, qw[1], a);
  a = dot2_bf16(kv.z, qw[2], a);
  a = dot2_bf16(kv.w, qw[3], a);
  return group_sum<LPR>(a) * sm_scale + 0.0f;
}

// Scores of the tokens of I_f and I_bs (HeadRec.b holds |I_bs| at this point).  With STATS (targets N and
// SDPA) the V rows of the same tokens are read as well and the numerator statistics of Algorithm 2 are
// accumulated on the way: N_f = sum_{I_f} w V, R1 = sum_{I_bs} w V, R2 = sum_{I_bs} ||w V||^2 with
// w = exp(s - max); no maximum is known yet, so every lane group keeps a running one and rescales.
template <int D, bool PAGED, bool STATS>
__global__ __launch_bounds__(kGatherThreads) void sparse_score_kernel(GivenArgs A) {
  constexpr int LPR = D / 8;
  constexpr int RPW = kWave / LPR;
  constexpr int WAVES = kGatherThreads / kWave;
  constexpr int RPB = RPW * WAVES;
  constexpr int GROUPS = RPB;
  constexpr int U = 8;
  const int h = head_of_block((int)blockIdx.x, A.Hq, A.Hq / A.group, A.group_major), split = blockIdx.y, b = blockIdx.z;
  const int bh = b * A.Hq + h;
  const int kvh = h / A.group;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = lane % LPR, rsub = lane / LPR;
  const HeadRec r = A.head_rec[bh];
  const int32_t* idx = A.idx + (int64_t)bh * A.idx_cap;
  float* sp = A.sparse + (int64_t)bh * A.idx_cap;
  const int total = r.n_sink + r.n_win + r.k + r.b;
  const int per = (total + A.splits - 1) / A.splits;
  const int p_lo = split * per, p_hi = min(p_lo + per, total);
  const unsigned char* cache_rec = r.base_cached ? cache_record(A.rcache, A.rc, b / A.q_len, A.Hq / A.group, kvh) : nullptr;
  const int32_t* slots_of = A.base_slot + (int64_t)bh * A.b0_max;
  uint32_t qw[4];
  load_q<D>(A, bh, sub, qw);
  float acc_f[8], acc_b[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) acc_f[c] = acc_b[c] = 0.f;
  float r2 = 0.f, m_run = -INFINITY;
  // U rows per lane group at a time, without a branch per row: places in the lists (arithmetic), tokens (one
  // load each; for a base sample that came from the random cache also its slots), rows (one or two loads each),
  // then the arithmetic.  A slot beyond the range repeats the range's last row and writes nothing.  The base
  // sample has its own walk: its rows may come from the cache, and its statistics go to sums of their own.
  const int n_fix = r.n_sink + r.n_win + r.k;
  const bool cached = r.base_cached != 0;
  auto walk = [&](int lo, int hi, auto tail_tag) {
    constexpr bool kTail = decltype(tail_tag)::value;
    for (int p0 = lo + wave * RPW + rsub; p0 < hi; p0 += RPB * U) {
      int64_t place[U];
      bool valid[U];
      int tok[U], slot[U];
      uint4 kv[U], vv[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int p = p0 + u * RPB;
        valid[u] = p < hi;
        const int pc = min(p, hi - 1);
        place[u] = kTail ? A.seg_base + (pc - n_fix)
                         : fixed_place(pc, r.n_sink, r.n_win, A.seg_sink, A.seg_win, A.seg_topk);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        tok[u] = idx[place[u]];
        slot[u] = 0;
        vv[u] = make_uint4(0u, 0u, 0u, 0u);
      }
      if (kTail && cached) {
        // the copies of the rows in the cache: rows of neighbouring slots, shared by the group's heads
#pragma unroll
        for (int u = 0; u < U; ++u) slot[u] = slots_of[place[u] - A.seg_base];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int64_t so = (int64_t)min(max(slot[u], 0), A.rc.slots - 1) * D + sub * 8;
          kv[u] = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(cache_rec + A.rc.off_k) + so);
          if (STATS) vv[u] = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(cache_rec + A.rc.off_v) + so);
        }
      } else {
        int blk[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          tok[u] = min(max(tok[u], 0), r.n - 1);
          blk[u] = kv_block<PAGED>(A.Lk, b / A.q_len, tok[u]);  // (K and V share the block table)
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          kv[u] = load_stream_16(A.k + kv_row_offset_in<PAGED>(A.Lk, b / A.q_len, kvh, tok[u], blk[u]) + sub * 8);
          if (STATS) vv[u] = load_stream_16(A.v + kv_row_offset_in<PAGED>(A.Lv, b / A.q_len, kvh, tok[u], blk[u]) + sub * 8);
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float s = row_score<LPR>(kv[u], qw, A.sm_scale);
        if (valid[u] && sub == 0) sp[place[u]] = s;
        if (STATS && valid[u]) {
          if (s > m_run) {
            const float f = __expf(m_run - s);  // 0 when m_run is -inf
#pragma unroll
            for (int c = 0; c < 8; ++c) {
              acc_f[c] *= f;
              acc_b[c] *= f;
            }
            r2 *= f * f;
            m_run = s;
          }
          const float wt = __expf(s - m_run);
          const uint32_t ww[4] = {vv[u].x, vv[u].y, vv[u].z, vv[u].w};
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const float x = wt * bf16_lo(ww[c]), y = wt * bf16_hi(ww[c]);
            if constexpr (kTail) {
              acc_b[2 * c] += x;
              acc_b[2 * c + 1] += y;
              r2 += x * x + y * y;
            } else {
              acc_f[2 * c] += x;
              acc_f[2 * c + 1] += y;
            }
          }
        }
      }
    }
  };
  walk(p_lo, min(p_hi, n_fix), std::false_type{});
  walk(max(p_lo, n_fix), p_hi, std::true_type{});
  if (!STATS) return;
  // every lane group has its own (maximum, N_f, R1, R2 share): bring them to the workgroup's maximum and add
  __shared__ float s_f[STATS ? GROUPS : 1][STATS ? D : 1], s_b[STATS ? GROUPS : 1][STATS ? D : 1];
  __shared__ float s_r2[GROUPS][LPR], s_m[GROUPS];
  const int g = wave * RPW + rsub;
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    s_f[g][sub * 8 + c] = acc_f[c];
    s_b[g][sub * 8 + c] = acc_b[c];
  }
  s_r2[g][sub] = r2;
  if (sub == 0) s_m[g] = m_run;
  __syncthreads();
  float M = -INFINITY;
#pragma unroll
  for (int j = 0; j < GROUPS; ++j) M = fmaxf(M, s_m[j]);
  float* out = A.vstat + ((int64_t)bh * A.splits + split) * (2 * D + 4);
  if (tid < D) {
    float a = 0.f, c2 = 0.f;
#pragma unroll
    for (int j = 0; j < GROUPS; ++j) {
      const float f = s_m[j] > -INFINITY ? __expf(s_m[j] - M) : 0.f;
      a += s_f[j][tid] * f;
      c2 += s_b[j][tid] * f;
    }
    out[tid] = a;
    out[D + tid] = c2;
  }
  if (tid == 0) {
    float t = 0.f;
#pragma unroll
    for (int j = 0; j < GROUPS; ++j) {
      const float f = s_m[j] > -INFINITY ? __expf(s_m[j] - M) : 0.f;
      float q2 = 0.f;
#pragma unroll
      for (int c = 0; c < LPR; ++c) q2 += s_r2[j][c];
      t += q2 * f * f;
    }
    out[2 * D] = t;
    out[2 * D + 1] = M;
  }
}

template <int D, bool PAGED>
__global__ __launch_bounds__(kGatherThreads) void given_gather_kernel(GivenArgs A) {
  constexpr int LPR = D / 8;
  constexpr int RPW = kWave / LPR;
  constexpr int WAVES = kGatherThreads / kWave;
  constexpr int RPB = RPW * WAVES;
  constexpr int GROUPS = RPB;  // lane groups of a workgroup, each with its own running maximum
  constexpr int U = 8;
  const int h = head_of_block((int)blockIdx.x, A.Hq, A.Hq / A.group, A.group_major), split = blockIdx.y, b = blockIdx.z;
  const int bh = b * A.Hq + h;
  const int kvh = h / A.group;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = lane % LPR, rsub = lane / LPR;
  const HeadRec r = A.head_rec[bh];
  const int32_t* idx = A.idx + (int64_t)bh * A.idx_cap;
  const float* sp = A.sparse + (int64_t)bh * A.idx_cap;
  const int total = r.n_sink + r.n_win + r.k + r.b;
  const int per = (total + A.splits - 1) / A.splits;
  const int p_lo = split * per, p_hi = min(p_lo + per, total);
  const float tail_bias = r.scale > 0.f ? __logf(r.scale) : 0.f;  // ln(n_s / b): sampled tokens weigh n_s / b
  uint32_t qw[4];
  load_q<D>(A, bh, sub, qw);

  float acc[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) acc[c] = 0.f;
  float dsum = 0.f, m_run = -INFINITY;

  // U rows per lane group at a time, without a branch per row (places, then tokens and known scores, then
  // rows, then the arithmetic); a slot beyond the range repeats the range's last row and adds nothing.  Three
  // walks: I_f (scores in the sparse list), the leading entries of the final sample that repeat the base
  // sample (nested samples: scores in the base sample's places of the sparse list), and the rest of the final
  // sample, whose scores are computed here from their K rows.
  const int n_fix = r.n_sink + r.n_win + r.k;
  auto walk = [&](int lo, int hi, auto kind_tag) {
    constexpr int kKind = decltype(kind_tag)::value;  // 0: I_f, 1: kept base-sample entries, 2: newly drawn
    constexpr bool kTail = kKind != 0;
    for (int p0 = lo + wave * RPW + rsub; p0 < hi; p0 += RPB * U) {
      int64_t place[U];
      bool valid[U];
      int tok[U];
      float s[U];
      uint4 kv[U], vv[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int p = p0 + u * RPB;
        valid[u] = p < hi;
        const int pc = min(p, hi - 1);
        place[u] = kTail ? A.seg_dyn + (pc - n_fix)
                         : fixed_place(pc, r.n_sink, r.n_win, A.seg_sink, A.seg_win, A.seg_topk);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        tok[u] = idx[place[u]];
        s[u] = kKind == 2 ? 0.f : sp[kKind == 1 ? A.seg_base + (place[u] - A.seg_dyn) : place[u]];
        kv[u] = make_uint4(0u, 0u, 0u, 0u);
      }
      int blk[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        tok[u] = min(max(tok[u], 0), r.n - 1);
        blk[u] = kv_block<PAGED>(A.Lv, b / A.q_len, tok[u]);  // (K and V share the block table)
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (kKind == 2) kv[u] = load_stream_16(A.k + kv_row_offset_in<PAGED>(A.Lk, b / A.q_len, kvh, tok[u], blk[u]) + sub * 8);
        vv[u] = load_stream_16(A.v + kv_row_offset_in<PAGED>(A.Lv, b / A.q_len, kvh, tok[u], blk[u]) + sub * 8);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        // (the lanes of a group stay together: every lane of the group computes the row's score)
        if (kKind == 2) s[u] = row_score<LPR>(kv[u], qw, A.sm_scale);
        if (valid[u]) {
          const float e = s[u] + (kTail ? tail_bias : 0.f);
          if (e > m_run) {
            const float f = __expf(m_run - e);  // 0 when m_run is -inf
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[c] *= f;
            dsum *= f;
            m_run = e;
          }
          const float wt = __expf(e - m_run);
          const uint32_t ww[4] = {vv[u].x, vv[u].y, vv[u].z, vv[u].w};
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            acc[2 * c] += wt * bf16_lo(ww[c]);
            acc[2 * c + 1] += wt * bf16_hi(ww[c]);
          }
          dsum += wt;
        }
      }
    }
  };
  const int n_kept = n_fix + min(max(r.b_keep, 0), r.b);
  walk(p_lo, min(p_hi, n_fix), std::integral_constant<int, 0>{});
  walk(max(p_lo, n_fix), min(p_hi, n_kept), std::integral_constant<int, 1>{});
  walk(max(p_lo, n_kept), p_hi, std::integral_constant<int, 2>{});

  // every lane group has its own (maximum, D, N): bring them to the workgroup's maximum and add
  __shared__ float s_acc[GROUPS][D];
  __shared__ float s_d[GROUPS], s_m[GROUPS];
  const int g = wave * RPW + rsub;
#pragma unroll
  for (int c = 0; c < 8; ++c) s_acc[g][sub * 8 + c] = acc[c];
  if (sub == 0) {
    s_d[g] = dsum;
    s_m[g] = m_run;
  }
  __syncthreads();
  float M = -INFINITY;
#pragma unroll
  for (int j = 0; j < GROUPS; ++j) M = fmaxf(M, s_m[j]);
  float* part = A.part + ((int64_t)bh * A.splits + split) * (D + 4);
  if (tid < D) {
    float a = 0.f;
#pragma unroll
    for (int j = 0; j < GROUPS; ++j) a += s_acc[j][tid] * (s_m[j] > -INFINITY ? __expf(s_m[j] - M) : 0.f);
    part[tid] = a;
  }
  if (tid == 0) {
    float d = 0.f;
#pragma unroll
    for (int j = 0; j < GROUPS; ++j) d += s_d[j] * (s_m[j] > -INFINITY ? __expf(s_m[j] - M) : 0.f);
    part[D] = d;
    part[D + 1] = M;
  }
}

// Combines the per-split (maximum, D, N) partials of a head in split order: O = N / D, lse = M + ln D.
template <int D>
__global__ __launch_bounds__(D) void given_merge_kernel(const float* __restrict__ part, int splits, int Hq,
                                                        float* __restrict__ out_o, float* __restrict__ out_lse,
                                                        int group_major, int Hkv) {
  const int h = head_of_block((int)blockIdx.x, Hq, Hkv, group_major), b = blockIdx.y, bh = b * Hq + h;
  const int c = threadIdx.x;
  const float* p = part + (int64_t)bh * splits * (D + 4);
  float M = -INFINITY;
#pragma unroll 8
  for (int s = 0; s < splits; ++s) M = fmaxf(M, p[s * (D + 4) + D + 1]);
  float a = 0.f, dtot = 0.f;
#pragma unroll 8
  for (int s = 0; s < splits; ++s) {
    const float ms = p[s * (D + 4) + D + 1];
    const float f = ms > -INFINITY ? __expf(ms - M) : 0.f;
    a += p[s * (D + 4) + c] * f;
    dtot += p[s * (D + 4) + D] * f;
  }
  out_o[(int64_t)bh * D + c] = a / dtot;
  if (c == 0 && out_lse) out_lse[bh] = M + logf(dtot);
}

template <int D>
hipError_t launch_given_d(const Plan& pl, int stage, const void* q, const void* k, const void* v,
                          const int32_t* block_table, const void* rcache, void* ws, const int32_t* out_idx,
                          float* out_o, float* out_lse, hipStream_t st) {
  const vatt_params& p = pl.p;
  char* w = static_cast<char*>(ws);
  GivenArgs A;
  A.q = static_cast<const uint16_t*>(q);
  A.k = static_cast<const uint16_t*>(k);
  A.v = static_cast<const uint16_t*>(v);
  A.Lk = pl.kv_k;
  A.Lk.block_table = block_table;
  A.Lv = pl.kv_v;
  A.Lv.block_table = block_table;
  A.head_rec = reinterpret_cast<const HeadRec*>(w + pl.off_head_rec);
  A.idx = out_idx;
  A.sparse = reinterpret_cast<float*>(w + pl.off_sparse);
  A.part = reinterpret_cast<float*>(w + pl.off_gather_part);
  A.vstat = reinterpret_cast<float*>(w + pl.off_vstat_part);
  A.out_o = out_o;
  A.out_lse = out_lse;
  A.seg_sink = pl.seg_off[0];
  A.seg_win = pl.seg_off[1];
  A.seg_topk = pl.seg_off[2];
  A.seg_base = pl.seg_off[3];
  A.seg_dyn = pl.seg_off[4];
  A.idx_cap = (int64_t)pl.idx_cap;
  A.Hq = p.n_q_heads;
  A.group = pl.group;
  A.splits = pl.given_splits;
  A.q_len = pl.q_len;
  A.group_major = pl.group_major;
  A.sm_scale = pl.sm_scale;
  A.rcache = rcache;
  A.rc = cache_layout(pl);
  A.base_slot = reinterpret_cast<const int32_t*>(w + pl.off_base_slot);
  A.b0_max = pl.b0_max;
  const bool paged = p.kv_layout == VATT_LAYOUT_PAGED;
  const bool stats = p.target != VATT_TARGET_D;
  if (stage == 0 && !stats) A.splits = pl.sparse_splits;  // scores only: no partial sums, any number of workgroups
  dim3 grid(p.n_q_heads, A.splits, pl.vbatch);
  if (stage == 0) {
    if (paged && stats) hipLaunchKernelGGL((sparse_score_kernel<D, true, true>), grid, dim3(kGatherThreads), 0, st, A);
    else if (paged) hipLaunchKernelGGL((sparse_score_kernel<D, true, false>), grid, dim3(kGatherThreads), 0, st, A);
    else if (stats) hipLaunchKernelGGL((sparse_score_kernel<D, false, true>), grid, dim3(kGatherThreads), 0, st, A);
    else hipLaunchKernelGGL((sparse_score_kernel<D, false, false>), grid, dim3(kGatherThreads), 0, st, A);
    return hipGetLastError();
  }
  if (paged) hipLaunchKernelGGL((given_gather_kernel<D, true>), grid, dim3(kGatherThreads), 0, st, A);
  else hipLaunchKernelGGL((given_gather_kernel<D, false>), grid, dim3(kGatherThreads), 0, st, A);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((given_merge_kernel<D>), dim3(p.n_q_heads, pl.vbatch), dim3(D), 0, st, A.part, A.splits,
                     p.n_q_heads, out_o, out_lse, pl.group_major, p.n_kv_heads);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_sparse_score(const Plan& pl, const void* q, const void* k, const void* v,
                               const int32_t* block_table, const void* rcache, void* ws, const int32_t* out_idx,
                               hipStream_t st) {
  if (pl.p.head_dim == 128) return launch_given_d<128>(pl, 0, q, k, v, block_table, rcache, ws, out_idx, nullptr, nullptr, st);
  if (pl.p.head_dim == 64) return launch_given_d<64>(pl, 0, q, k, v, block_table, rcache, ws, out_idx, nullptr, nullptr, st);
  return hipErrorInvalidValue;
}

hipError_t launch_given_merge(const Plan& pl, void* ws, int splits, float* out_o, float* out_lse, hipStream_t st) {
  const vatt_params& p = pl.p;
  const float* part = reinterpret_cast<const float*>(static_cast<char*>(ws) + pl.off_gather_part);
  if (p.head_dim == 128)
    hipLaunchKernelGGL((given_merge_kernel<128>), dim3(p.n_q_heads, pl.vbatch), dim3(128), 0, st, part, splits,
                       p.n_q_heads, out_o, out_lse, pl.group_major, p.n_kv_heads);
  else if (p.head_dim == 64)
    hipLaunchKernelGGL((given_merge_kernel<64>), dim3(p.n_q_heads, pl.vbatch), dim3(64), 0, st, part, splits,
                       p.n_q_heads, out_o, out_lse, pl.group_major, p.n_kv_heads);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_given_gather(const Plan& pl, const void* q, const void* k, const void* v,
                               const int32_t* block_table, void* ws, const int32_t* out_idx, float* out_o,
                               float* out_lse, hipStream_t st) {
  if (pl.p.head_dim == 128) return launch_given_d<128>(pl, 1, q, k, v, block_table, nullptr, ws, out_idx, out_o, out_lse, st);
  if (pl.p.head_dim == 64) return launch_given_d<64>(pl, 1, q, k, v, block_table, nullptr, ws, out_idx, out_o, out_lse, st);
  return hipErrorInvalidValue;
}

}  // namespace vatt
