// Sparse attention over the selected tokens: SDPA_{S,p} of Eq. 3 with S = [I_f, I_dyn], p = [1, b/n_s],
// computed as the N and D sums of Section 4.1:
//   N = sum_{I_f} w_i V[i] + (n_s/b) sum_{I_dyn} w_i V[i],   D likewise without V,   O = N / D,
// with w_i = exp(s_i - m), m the head's largest score (so every weight is <= 1 and partial sums of
// different workgroups add directly).  Also the V-side statistics of Algorithm 2 for the numerator and
// SDPA targets (N_f, sum r_i and sum ||r_i||^2 over the base sample, r_i = w_i V[i]).
//
// grid = (query heads, splits, sequences).  A workgroup walks its slice of the head's token list 16 rows
// (d = 128) at a time: d/8 adjacent lanes read one 256-byte V row with one 16-byte load each.  With more
// than one split per head a small second kernel adds the per-split partials in split order and writes
// O and ln D (a kernel boundary is the cheapest device-wide ordering point on this chip).
// The head index is the fastest grid dimension on purpose: workgroups go to the chip's eight XCDs round-robin
// in launch order, so with a head count that is a multiple of eight all splits of a head run on one XCD and
// share its L2 for the head record, the index list and the lines of the score row (measured: 46.4 -> 45.1 us
// per call at batch 1).  With head_of_block the heads of one KV head share an XCD as well: they read the same
// sink and window rows of V and many of the same heavy tokens (L2 hits of this kernel at 32K tokens and batch
// 1: 42 K -> 63 K of 194 K requests).
#include "vatt_internal.h"

namespace vatt {
namespace {

struct GatherArgs {
  const uint16_t* v;
  KVLayout L;
  const float* scores;
  const float* place_sc;  // [B*Hq][idx_cap]: scores of listed tokens at their list places (selection kernel)
  const HeadRec* head_rec;
  const int32_t* idx;
  float* part;        // [B*Hq][splits][d + 4]
  double* vpart;      // [B*Hq][splits][2d + 2]
  float* out_o;
  float* out_lse;
  int64_t seg_sink, seg_win, seg_topk, seg_base, seg_dyn, idx_cap;
  int n_pad, Hq, group, splits;
  int group_major, Hkv;  // see head_of_block
  int q_len;  // query tokens per sequence: blockIdx.z = sequence * q_len + query token
};

// A head's list is walked by position: [sink | window | top-k | tail) where the tail is the final sample
// (scaled by n_s/b) or, for the statistics pass, the base sample (unscaled).
template <int D, bool PAGED, bool STATS>
__global__ __launch_bounds__(kGatherThreads) void gather_kernel(GatherArgs A) {
  constexpr int LPR = D / 8;
  constexpr int RPW = kWave / LPR;
  constexpr int WAVES = kGatherThreads / kWave;
  constexpr int RPB = RPW * WAVES;  // rows per workgroup step
  constexpr int U = 8;              // independent rows in flight per lane

  const int h = head_of_block((int)blockIdx.x, A.Hq, A.Hkv, A.group_major), split = blockIdx.y, b = blockIdx.z;
  const int bh = b * A.Hq + h;
  const int kvh = h / A.group;
  const int seq = b / A.q_len;  // the sequence whose cache this (sequence, query token) pair reads
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = lane % LPR, rsub = lane / LPR;

  const HeadRec r = A.head_rec[bh];
  // (pointers that are the same for the whole workgroup, indexed with 32-bit offsets: address arithmetic in 64
  // bits for every row was most of this kernel's instructions, and the kernel was bound by issuing them)
  const int32_t* idx = A.idx + (int64_t)bh * A.idx_cap;
  const float* placed = A.place_sc + (int64_t)bh * A.idx_cap;  // scores by list place
  const float* row = A.scores + (int64_t)bh * A.n_pad;          // scores by token
  const bool tail_by_token = r.tail_by_token != 0;               // (the same for the whole workgroup)
  const uint16_t* v_head = PAGED ? A.v : A.v + (int64_t)seq * A.L.seq_stride + (int64_t)kvh * A.L.head_stride;
  const int total = r.n_sink + r.n_win + r.k + r.b;
  const int per = (total + A.splits - 1) / A.splits;
  const int p_lo = split * per, p_hi = min(p_lo + per, total);
  const uint32_t seg_sink = (uint32_t)A.seg_sink, seg_win = (uint32_t)A.seg_win, seg_topk = (uint32_t)A.seg_topk;
  const uint32_t seg_tail = (uint32_t)(STATS ? A.seg_base : A.seg_dyn), last_place = (uint32_t)A.idx_cap - 1u;
  const float tail_scale = STATS ? 1.0f : r.scale;

  float acc[8], acc2[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) acc[c] = acc2[c] = 0.f;
  float dsum = 0.f, r2 = 0.f;

  // A wave takes RPW * U rows per step: RPW lane groups of LPR lanes, U rows in flight per group.  The work
  // that belongs to a row, not to a column, is done once per row by the row's own lane (lane L of the wave for row
  // L of the step) instead of by every lane of the group that reads the row: list place, list entry and score
  // (sink and window tokens follow from the place by arithmetic; their list load is issued all the same), the
  // token and the weight.  Token and weight then reach the group's lanes through a wave shuffle, which leaves
  // the vector ALU free: with all of it done per lane this kernel was bound by issuing instructions, not by
  // memory.  Then, in stages without a branch per row, so that the loads of a stage go out together:
  // block-table entries on a paged cache, the V rows, the sums.  A place beyond the range carries weight 0.
  constexpr int ROWS_W = RPW * U;   // rows of a wave per step (32 at d = 128, 64 at d = 64)
  static_assert(ROWS_W <= kWave, "one lane per row of a step");
  const int n_sw = r.n_sink + r.n_win;
  const int win_shift = r.n - r.n_win - r.n_sink;  // window token = list position + this
  const int u_mine = lane / RPW, g_mine = lane % RPW;   // the row this lane prepares: slot u_mine of lane group g_mine
  // (the list entry and the score of the next step's row are requested one step ahead, so that a step starts
  // with them at hand: one dependent round trip per step instead of two)
  auto place_of = [&](int p0) {
    const int pc = min(p0 + u_mine * RPB + wave * RPW + g_mine, p_hi - 1);
    const int t2 = pc - n_sw, t3 = t2 - r.k;
    const uint32_t edge = pc < r.n_sink ? seg_sink + (uint32_t)pc : seg_win + (uint32_t)(pc - r.n_sink);
    return min(t3 >= 0 ? seg_tail + (uint32_t)t3 : t2 >= 0 ? seg_topk + (uint32_t)t2 : edge, last_place);
  };
  int listed_next = 0;
  float sc_next = 0.f;
  if (p_lo < p_hi) {
    const uint32_t place0 = place_of(p_lo);
    listed_next = idx[place0];
    sc_next = placed[place0];
  }
  for (int p0 = p_lo; p0 < p_hi; p0 += RPB * U) {
    const int p = p0 + u_mine * RPB + wave * RPW + g_mine;
    const bool valid = lane < ROWS_W && p < p_hi;
    const int pc = min(p, p_hi - 1);
    const int t2 = pc - n_sw, t3 = t2 - r.k;
    const bool is_tail = t3 >= 0;
    const int listed = listed_next;
    float sc = sc_next;
    {
      const uint32_t place_n = place_of(p0 + RPB * U);  // (beyond the range: the range's last place once more)
      listed_next = idx[place_n];
      sc_next = placed[place_n];
    }
    const int by_rule = pc < r.n_sink ? pc : pc + win_shift;
    const int tok_mine = min(max(t2 >= 0 ? listed : by_rule, 0), r.n - 1);
    if (tail_by_token) {  // a sample whose scores were not at hand when its list was written
      const float by_token = row[tok_mine];
      sc = is_tail ? by_token : sc;
    }
    const float wt_mine = valid ? __expf(sc - r.m) * (is_tail ? tail_scale : 1.0f) : 0.f;
    if (!(STATS && is_tail)) dsum += wt_mine;

    int tok[U], blk[U];
    float wt[U];
    bool tail[U];
    uint4 vv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int src = u * RPW + rsub;
      tok[u] = __shfl(tok_mine, src);
      wt[u] = __shfl(wt_mine, src);
      tail[u] = STATS ? (__shfl((int)is_tail, src) != 0) : false;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) blk[u] = kv_block<PAGED>(A.L, seq, tok[u]);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if constexpr (PAGED) vv[u] = load_stream_16(A.v + kv_row_offset_in<true>(A.L, seq, kvh, tok[u], blk[u]) + sub * 8);
      else vv[u] = load_stream_16(v_head + ((uint32_t)tok[u] * (uint32_t)D + (uint32_t)(sub * 8)));  // (n_max * d < 2^32)
    }
    // (all U rows are requested before the first is used: left to itself the scheduler waits for the first rows
    // in order to reuse their registers for the later ones)
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t ww[4] = {vv[u].x, vv[u].y, vv[u].z, vv[u].w};
      if (STATS && tail[u]) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const float a = wt[u] * bf16_lo(ww[c]), bb = wt[u] * bf16_hi(ww[c]);
          acc2[2 * c] += a;
          acc2[2 * c + 1] += bb;
          r2 += a * a + bb * bb;
        }
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          acc[2 * c] += wt[u] * bf16_lo(ww[c]);
          acc[2 * c + 1] += wt[u] * bf16_hi(ww[c]);
        }
      }
    }
  }

  // rows of one wave sit in lane groups rsub = 0 .. RPW-1: add them, then add the waves through LDS
#pragma unroll
  for (int o = LPR; o < kWave; o <<= 1) {
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      acc[c] += __shfl_xor(acc[c], o);
      if (STATS) acc2[c] += __shfl_xor(acc2[c], o);
    }
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    dsum += __shfl_xor(dsum, o);
    if (STATS) r2 += __shfl_xor(r2, o);
  }
  __shared__ float s_acc[WAVES][D];
  __shared__ float s_acc2[STATS ? WAVES : 1][STATS ? D : 1];
  __shared__ float s_d[WAVES], s_r2[WAVES];
  if (rsub == 0) {
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      s_acc[wave][sub * 8 + c] = acc[c];
      if (STATS) s_acc2[wave][sub * 8 + c] = acc2[c];
    }
  }
  if (lane == 0) {
    s_d[wave] = dsum;
    s_r2[wave] = r2;
  }
  __syncthreads();

  if (STATS) {
    double* out = A.vpart + ((int64_t)bh * A.splits + split) * (2 * D + 2);
    if (tid < D) {
      double a = 0.0, a2 = 0.0;
#pragma unroll
      for (int w2 = 0; w2 < WAVES; ++w2) {
        a += (double)s_acc[w2][tid];
        a2 += (double)s_acc2[w2][tid];
      }
      out[tid] = a;
      out[D + tid] = a2;
    }
    if (tid == 0) {
      double t = 0.0;
#pragma unroll
      for (int w2 = 0; w2 < WAVES; ++w2) t += (double)s_r2[w2];
      out[2 * D] = t;
      out[2 * D + 1] = 0.0;
    }
    return;
  }

  float* part = A.part + ((int64_t)bh * A.splits + split) * (D + 4);
  float dtot = 0.f;
#pragma unroll
  for (int w2 = 0; w2 < WAVES; ++w2) dtot += s_d[w2];
  if (tid < D) {
    float a = 0.f;
#pragma unroll
    for (int w2 = 0; w2 < WAVES; ++w2) a += s_acc[w2][tid];
    if (A.splits == 1) {
      A.out_o[(int64_t)bh * D + tid] = a / dtot;  // one workgroup per head: finished here
    } else {
      part[tid] = a;
    }
  }
  if (tid == 0) {
    if (A.splits == 1) {
      if (A.out_lse) A.out_lse[bh] = r.m + logf(dtot);
    } else {
      part[D] = dtot;
    }
  }
}

// Adds the per-split partial sums of a head in split order: O = N / D, lse = m + ln D.
template <int D>
__global__ __launch_bounds__(D) void gather_merge_kernel(const float* __restrict__ part,
                                                         const HeadRec* __restrict__ head_rec, int splits, int Hq,
                                                         float* __restrict__ out_o, float* __restrict__ out_lse,
                                                         int group_major, int Hkv) {
  const int h = head_of_block((int)blockIdx.x, Hq, Hkv, group_major), b = blockIdx.y, bh = b * Hq + h;
  const int c = threadIdx.x;
  const float* p = part + (int64_t)bh * splits * (D + 4);
  float a = 0.f, dtot = 0.f;
#pragma unroll 8
  for (int s = 0; s < splits; ++s) {
    a += p[s * (D + 4) + c];
    dtot += p[s * (D + 4) + D];
  }
  out_o[(int64_t)bh * D + c] = a / dtot;
  if (c == 0 && out_lse) out_lse[bh] = head_rec[bh].m + logf(dtot);
}

template <int D, bool STATS>
hipError_t launch_gather_d(const Plan& pl, const void* v, const int32_t* block_table, void* ws,
                           const int32_t* out_idx, float* out_o, float* out_lse, hipStream_t st) {
  const vatt_params& p = pl.p;
  char* w = static_cast<char*>(ws);
  GatherArgs A;
  A.v = static_cast<const uint16_t*>(v);
  A.L = pl.kv_v;
  A.L.block_table = block_table;
  A.scores = reinterpret_cast<const float*>(w + pl.off_scores);
  A.place_sc = reinterpret_cast<const float*>(w + pl.off_sparse);
  A.head_rec = reinterpret_cast<const HeadRec*>(w + pl.off_head_rec);
  A.idx = out_idx;
  A.part = reinterpret_cast<float*>(w + pl.off_gather_part);
  A.vpart = reinterpret_cast<double*>(w + pl.off_vstat_part);
  A.out_o = out_o;
  A.out_lse = out_lse;
  A.seg_sink = pl.seg_off[0];
  A.seg_win = pl.seg_off[1];
  A.seg_topk = pl.seg_off[2];
  A.seg_base = pl.seg_off[3];
  A.seg_dyn = pl.seg_off[4];
  A.idx_cap = (int64_t)pl.idx_cap;
  A.n_pad = pl.n_pad;
  A.Hq = p.n_q_heads;
  A.group = pl.group;
  A.splits = STATS ? pl.vstat_splits : pl.gather_splits;
  A.q_len = pl.q_len;
  A.group_major = pl.group_major;
  A.Hkv = p.n_kv_heads;
  dim3 grid(p.n_q_heads, A.splits, pl.vbatch);
  if (p.kv_layout == VATT_LAYOUT_PAGED)
    hipLaunchKernelGGL((gather_kernel<D, true, STATS>), grid, dim3(kGatherThreads), 0, st, A);
  else
    hipLaunchKernelGGL((gather_kernel<D, false, STATS>), grid, dim3(kGatherThreads), 0, st, A);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || STATS || A.splits == 1) return e;
  hipLaunchKernelGGL((gather_merge_kernel<D>), dim3(p.n_q_heads, pl.vbatch), dim3(D), 0, st, A.part, A.head_rec,
                     A.splits, p.n_q_heads, out_o, out_lse, pl.group_major, p.n_kv_heads);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gather(const Plan& pl, const void* v, const int32_t* block_table, void* ws,
                         const int32_t* out_idx, float* out_o, float* out_lse, hipStream_t st) {
  if (pl.p.head_dim == 128) return launch_gather_d<128, false>(pl, v, block_table, ws, out_idx, out_o, out_lse, st);
  if (pl.p.head_dim == 64) return launch_gather_d<64, false>(pl, v, block_table, ws, out_idx, out_o, out_lse, st);
  return hipErrorInvalidValue;
}

hipError_t launch_gather_merge(const Plan& pl, void* ws, int splits, float* out_o, float* out_lse, hipStream_t st) {
  const vatt_params& p = pl.p;
  char* w = static_cast<char*>(ws);
  const float* part = reinterpret_cast<const float*>(w + pl.off_gather_part);
  const HeadRec* rec = reinterpret_cast<const HeadRec*>(w + pl.off_head_rec);
  if (p.head_dim == 128)
    hipLaunchKernelGGL((gather_merge_kernel<128>), dim3(p.n_q_heads, pl.vbatch), dim3(128), 0, st, part, rec, splits,
                       p.n_q_heads, out_o, out_lse, pl.group_major, p.n_kv_heads);
  else if (p.head_dim == 64)
    hipLaunchKernelGGL((gather_merge_kernel<64>), dim3(p.n_q_heads, pl.vbatch), dim3(64), 0, st, part, rec, splits,
                       p.n_q_heads, out_o, out_lse, pl.group_major, p.n_kv_heads);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_vstats(const Plan& pl, const void* v, const int32_t* block_table, void* ws,
                         const int32_t* out_idx, hipStream_t st) {
  if (pl.p.head_dim == 128) return launch_gather_d<128, true>(pl, v, block_table, ws, out_idx, nullptr, nullptr, st);
  if (pl.p.head_dim == 64) return launch_gather_d<64, true>(pl, v, block_table, ws, out_idx, nullptr, nullptr, st);
  return hipErrorInvalidValue;
}

}  // namespace vatt
