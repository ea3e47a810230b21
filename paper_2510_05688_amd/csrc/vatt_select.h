// What the two selection kernels share (vatt_select.hip: scores at hand; vatt_select_given.hip: top-k set
// supplied by the caller): the argument block, the views of a score row, the exact top-k selection on LDS
// histograms, the budget of Algorithm 2 and the row accumulation of the fused gathers.  Everything here is
// device code that is inlined into those kernels, or host code that fills their arguments.
#pragma once
#include <type_traits>

#include "vatt_internal.h"
#include "vatt_sampler.h"

namespace vatt {
namespace {

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;

// ---------------------------------------------------------------------------
// Per-head kernel.
// ---------------------------------------------------------------------------
struct HeadArgs {
  const float* scores;
  const float* sub_max;  // [B*Hq][n_sub]: largest score of every kSubTile keys
  const int32_t* given_idx;  // [B*Hq][k_max]: caller-supplied top-k tokens (given-top-k path)
  const int32_t* given_cnt;  // [B*Hq]
  const float* sparse;       // [B*Hq][idx_cap]: scores at the places of the index lists (given-top-k path)
  float* place_sc;           // the same region on the scored path: the selection-only kernel leaves there the
                             // score of every listed token, for the gather kernel
  const int32_t* seq_lens;
  const uint64_t* seq_seeds;
  HeadRec* head_rec;
  const double* vstat_part;  // [B*Hq][vstat_splits][2d+2] (targets N, SDPA)
  const float* given_vstat;  // [B*Hq][given_splits][2d+4]: N_f[d], R1[d], R2, maximum (given-top-k path)
  int given_splits;
  int32_t* out_idx;
  int32_t* out_counts;
  double* out_budget_raw;
  float* out_stats;
  SelectParams sp;
  double z_half, z_quarter, eps, cap_frac;
  double range_factor;  // > 0: range-based Hoeffding budget for the denominator, ln(2 / delta) / 2
  int64_t seg_topk, seg_base, seg_dyn, seg_sink, seg_win;
  int64_t idx_cap;
  int n_pad, n_max, Hq, n_sub;
  int target, phase, small_batches, topk_general, vstat_splits, head_dim;
  int k_max, b0_max, b_max;
  int q_len;  // query tokens per sequence: blockIdx.y = sequence * q_len + query token
  int group_major, Hkv;  // see head_of_block
  int nested; // the final sample keeps the base sample and adds b - b0 tokens drawn outside it
  int b_multiple;  // b is rounded up to a multiple of this (1: the paper's rule)
  int ascending;   // the two samples' lists are written in ascending token order (else in acceptance order)
  uint32_t draw_cap;  // 0: the default 64 L + 4096
  unsigned long long* dbg;
  // fused gather (head_kernel with FD > 0): every head has `splits` workgroups, each of which repeats the
  // selection and then gathers every splits-th row of the head's token list
  const uint16_t* v;
  KVLayout L;
  float* part;       // [B*Hq][splits][d + 4]: partial (sum w V, sum w) of every workgroup
  int splits, split_shift, group;
  int glist_cap, dlist_cap;  // LDS entries for a workgroup's share of I_f and of the final sample
  // first batches of both sampler streams made ahead by prework_kernel (nullptr: made here)
  const uint4* pre_tok;       // [B*Hq][kHeadThreads]: the four proposed tokens of every thread
  const uint32_t* pre_flags;  // [B*Hq][kHeadThreads]: ok | first << 4 | (made ? 256 : 0)
  // random cache of base-sample rows (nullptr: the base sample is drawn)
  const void* rcache;
  CacheLayout rc;
  int32_t* base_slot;         // [B*Hq][b0_max]: cache slot of every base-sample entry taken from the cache
  // caller-supplied top-k, second selection phase with the gather fused in (given_topk_kernel<NT, FD>)
  const uint16_t* gq;         // queries [B*Hq][d]
  const uint16_t* gk;         // K cache
  KVLayout Lk;
  float sm_scale;
};


// ---------------------------------------------------------------------------
// The head's score row as the threads of the workgroup see it (general top-k path): thread t owns tokens
// t, t + NT, t + 2 NT, ...; every pass streams the row from global memory (it stays in the L2 cache), kTile
// scores per thread at a time.
//
// A pass visits the row in groups of kGroup scores per thread (kGroup * NT consecutive tokens per workgroup).
// Groups beyond the sequence are skipped; a group that lies entirely in the middle region is handed over with
// the tag InsideTag, so that the pass spends no instructions on the region test there.  The bodies are free of
// per-score branches: the compiler interleaves the work of neighbouring scores only then.
// ---------------------------------------------------------------------------
struct InsideTag { static constexpr bool value = true; };
struct EdgeTag { static constexpr bool value = false; };

template <int NT>
struct RowView {
  static constexpr int kTile = 16;
  static constexpr int kGroup = 8;
  const float* row;
  int n;

  template <class G>
  __device__ __forceinline__ void dispatch(const HeadSizes& hs, const float (&s)[kGroup], int g_lo, int t0, G&& g) {
    if (g_lo >= hs.mid_lo && g_lo + kGroup * NT <= hs.mid_hi) g(s, g_lo + t0, InsideTag{});
    else g(s, g_lo + t0, EdgeTag{});
  }

  // g(scores[kGroup], token of scores[0], tag): slot u of the group is token i0 + u * NT; under EdgeTag a slot
  // may lie outside the middle region or at or beyond n (it then carries a copy of the last score).
  template <class G>
  __device__ __forceinline__ void for_each_group(const HeadSizes& hs, G&& g) {
    for (int base = 0; base < n; base += NT * kTile) {
      float v[kTile];
#pragma unroll
      for (int u = 0; u < kTile; ++u) v[u] = row[min(base + u * NT + (int)threadIdx.x, n - 1)];
#pragma unroll
      for (int q = 0; q < kTile; q += kGroup) {
        if (base + q * NT < n) {
          float s[kGroup];
#pragma unroll
          for (int u = 0; u < kGroup; ++u) s[u] = v[q + u];
          dispatch(hs, s, base + q * NT, (int)threadIdx.x, g);
        }
      }
    }
  }
  // act(score, token) for the middle-region scores that pred(score) selects, when those are few: the test
  // runs branch-free over a group, and only a group with a hit anywhere in the wave walks its slots.
  template <class P, class A>
  __device__ __forceinline__ void for_each_rare(const HeadSizes& hs, P&& pred, A&& act) {
    for_each_group(hs, [&](const float (&s)[kGroup], int i0, auto tag) {
      uint32_t hit = 0;
#pragma unroll
      for (int u = 0; u < kGroup; ++u) {
        const int i = i0 + u * NT;
        const bool mid = decltype(tag)::value || (i >= hs.mid_lo && i < hs.mid_hi);
        hit |= ((mid && pred(s[u])) ? 1u : 0u) << u;
      }
      if (__ballot(hit != 0u)) {
#pragma unroll
        for (int u = 0; u < kGroup; ++u)
          if ((hit >> u) & 1u) act(s[u], i0 + u * NT);
      }
    });
  }
  // f(score, token, in the middle region) for every slot of the groups visited.
  template <class F>
  __device__ __forceinline__ void for_each(const HeadSizes& hs, F&& f) {
    for_each_group(hs, [&](const float (&s)[kGroup], int i0, auto tag) {
#pragma unroll
      for (int u = 0; u < kGroup; ++u) {
        const int i = i0 + u * NT;
        f(s[u], i, decltype(tag)::value || (i >= hs.mid_lo && i < hs.mid_hi));
      }
    });
  }
};

// The candidates for the top-k set as a list of composites in LDS: the same interface as RowView.
constexpr int kCandCap = 2048;
template <int NT>
struct CandView {
  const uint64_t* list;
  uint32_t count;
  template <class F>
  __device__ __forceinline__ void for_each(const HeadSizes&, F&& f) {
    for (uint32_t t = threadIdx.x; t < count; t += NT) {
      const uint64_t c = list[t];
      f(float_from_order_key(~(uint32_t)(c >> 32)), (int)(uint32_t)c, true);
    }
  }
  template <class P, class A>
  __device__ __forceinline__ void for_each_rare(const HeadSizes&, P&& pred, A&& act) {
    for (uint32_t t = threadIdx.x; t < count; t += NT) {
      const uint64_t c = list[t];
      const float sc = float_from_order_key(~(uint32_t)(c >> 32));
      if (pred(sc)) act(sc, (int)(uint32_t)c);
    }
  }
};

constexpr int kBins = 2048;   // histogram bins of one pass
constexpr int kSmall = 256;   // scores of one bin that are ranked directly

struct TopkSmem {
  uint32_t hist[kBins + 1];  // the last bin takes what is out of play
  uint64_t slist[kSmall];
  uint32_t slist_n;
  uint32_t j, below, inbin;
  uint64_t result;
  float wf[2][16];
  uint32_t wu[2][16];
  uint64_t wq[16];
  uint32_t cand_n, qual_n;
};

template <int NT, class View>
struct TopkOps {
  static constexpr int SW = NT / kWave;
  using Row = View;
  using HeadSmem = typename HeadOps<NT>::HeadSmem;

  // The bin that holds rank r (1-based) of the histogram: ts.j, with ts.below scores in the bins before it
  // and ts.inbin in it.
  static __device__ void locate(uint32_t r, TopkSmem& ts, HeadSmem& sm) {
    constexpr int BPT = kBins / NT;
    const int tid = threadIdx.x;
    uint32_t v[BPT], sum = 0;
#pragma unroll
    for (int q = 0; q < BPT; ++q) {
      v[q] = ts.hist[tid * BPT + q];
      sum += v[q];
    }
    uint32_t total;
    uint32_t excl = block_exclusive_scan<NT>(sum, &total, sm.scan);
    if (excl < r && r <= excl + sum) {
      uint32_t cum = excl;
      bool found = false;
#pragma unroll
      for (int q = 0; q < BPT; ++q) {
        if (!found && cum + v[q] >= r) {
          found = true;
          ts.j = (uint32_t)(tid * BPT + q);
          ts.below = cum;
          ts.inbin = v[q];
        }
        cum += v[q];
      }
    }
    __syncthreads();
  }

  static __device__ void zero_hist(TopkSmem& ts) {
    __syncthreads();  // earlier readers of the histogram are done
    for (int q = threadIdx.x; q <= kBins; q += NT) ts.hist[q] = 0;
    if (threadIdx.x == 0) ts.slist_n = 0;
    __syncthreads();
  }

  // Rank r (1-based) among the composites of the middle region that pred selects (at most kSmall): ts.result.
  template <class P>
  static __device__ __forceinline__ void rank_small(Row& rv, const HeadSizes& hs, uint32_t r, P&& pred, TopkSmem& ts) {
    const int tid = threadIdx.x;
    rv.for_each_rare(hs, pred, [&](float sc, int i) {
      const uint32_t pos = atomicAdd(&ts.slist_n, 1u);
      if (pos < (uint32_t)kSmall) ts.slist[pos] = ((uint64_t)(~float_order_key(sc)) << 32) | (uint32_t)i;
    });
    __syncthreads();
    const uint32_t cnt = min(ts.slist_n, (uint32_t)kSmall);
    if ((uint32_t)tid < cnt) {
      const uint64_t mine = ts.slist[tid];
      uint32_t below = 0;
      for (uint32_t q = 0; q < cnt; ++q) below += (ts.slist[q] < mine) ? 1u : 0u;
      if (below == r - 1u) ts.result = mine;
    }
    __syncthreads();
  }

  // Threshold composite of the k smallest composites among the `count` middle-region scores of the view,
  // 0 < k < count.  [smin, smax]: a range that holds every one of them.  scratch: all-zero bitmap, left all zero.
  static __device__ __forceinline__ uint64_t threshold(Row& rv, const HeadSizes& hs, uint32_t k, uint32_t count,
                                                       float smin, float smax, uint32_t* scratch, uint32_t* wpre,
                                                       TopkSmem& ts, HeadSmem& sm, unsigned long long* dbg) {
    const int tid = threadIdx.x;
    uint32_t r = k;
    uint32_t lo = ~float_order_key(smax), hi = ~float_order_key(smin);  // key range in play
    uint32_t m = count;
    // ---- first pass: bins of equal width in the score; (smax - s) * scale stays below kBins ----
    const float scale = (float)(kBins - 1) / (smax - smin);
    if (smax > smin && scale < 1e30f) {
      zero_hist(ts);
      rv.for_each(hs, [&](float s, int, bool mid) {
        const uint32_t b = (uint32_t)((smax - s) * scale);
        atomicAdd(&ts.hist[mid ? b : (uint32_t)kBins], 1u);
      });
      __syncthreads();
      VATT_STAMP(dbg, 20);
      locate(r, ts, sm);
      const uint32_t j = ts.j;
      r -= ts.below;
      m = ts.inbin;
      VATT_NOTE(dbg, 25, m);
      auto in_bin = [&](float s) { return (uint32_t)((smax - s) * scale) == j; };
      if (m <= (uint32_t)kSmall) {
        rank_small(rv, hs, r, in_bin, ts);
        VATT_STAMP(dbg, 21);
        return ts.result;
      }
      // many scores in one bin: go on with the integer keys of that bin
      uint32_t kmin = kInv32, kmax = 0u;
      rv.for_each(hs, [&](float s, int, bool mid) {
        const bool in = mid && in_bin(s);
        const uint32_t key = ~float_order_key(s);
        kmin = in ? min(kmin, key) : kmin;
        kmax = in ? max(kmax, key) : kmax;
      });
      kmin = wave_min_u32(kmin);
      kmax = wave_max_u32(kmax);
      __syncthreads();
      if ((tid & 63) == 0) {
        ts.wu[0][tid >> 6] = kmin;
        ts.wu[1][tid >> 6] = kmax;
      }
      __syncthreads();
      lo = kInv32;
      hi = 0u;
#pragma unroll
      for (int w = 0; w < SW; ++w) {
        lo = min(lo, ts.wu[0][w]);
        hi = max(hi, ts.wu[1][w]);
      }
    }
    // ---- further passes: bins of equal width in the integer key ----
    for (int pass = 0; pass < 4; ++pass) {
      if (r == m) return ((uint64_t)hi << 32) | kInv32;  // everything up to hi
      if (lo == hi) break;
      const uint32_t span = hi - lo;
      const int s = max(0, (32 - (int)__clz(span)) - 11);  // (span >> s) < kBins
      zero_hist(ts);
      rv.for_each(hs, [&](float sc, int, bool mid) {
        const uint32_t d = ~float_order_key(sc) - lo;
        atomicAdd(&ts.hist[(mid && d <= span) ? (d >> s) : (uint32_t)kBins], 1u);
      });
      __syncthreads();
      locate(r, ts, sm);
      const uint32_t lo_new = lo + (ts.j << s);
      hi = min(hi, lo_new + ((1u << s) - 1u));
      lo = lo_new;
      r -= ts.below;
      m = ts.inbin;
      if (m <= (uint32_t)kSmall) {
        const uint32_t lo_c = lo, span_c = hi - lo;
        rank_small(rv, hs, r, [&](float sc) { return ~float_order_key(sc) - lo_c <= span_c; }, ts);
        return ts.result;
      }
    }
    if (r == m) return ((uint64_t)hi << 32) | kInv32;
    // ---- more than kSmall equal scores around the threshold: the r lowest tokens among them ----
    const int words = (hs.n + 31) >> 5;
    const uint32_t key_eq = lo;
    rv.for_each(hs, [&](float sc, int i, bool mid) {
      const bool eq = mid && ~float_order_key(sc) == key_eq;
      atomicOr(&scratch[min(i, hs.n - 1) >> 5], eq ? (1u << (i & 31)) : 0u);
    });
    __syncthreads();
    HeadOps<NT>::word_prefix(scratch, words, wpre, sm);
    for (int w = tid; w < words; w += NT) {
      const uint32_t bits = scratch[w], before = wpre[w];
      if (before < r && r <= before + (uint32_t)__popc(bits)) {
        uint32_t b = bits;
        for (uint32_t q = before + 1; q < r; ++q) b &= b - 1u;
        ts.result = ((uint64_t)key_eq << 32) | (uint32_t)((w << 5) + (__ffs(b) - 1));
      }
    }
    __syncthreads();
    for (int w = tid; w < words; w += NT) scratch[w] = 0;
    __syncthreads();
    return ts.result;
  }
};


// ---------------------------------------------------------------------------
// Algorithm 2 from the sums over I_f and the base sample (shared by the scored path and the path with a
// caller-supplied top-k set): unbiased variance, D^, rho_D = n_s sigma / D^; the numerator's
// rho_N = n_s sqrt(Tr Sigma) / ||N^|| from its own sums; b* of the target (Corollaries for D and N, Theorem 4.3
// with delta' = delta / 2); then b = min(n_s, max(b0, min(ceil(b*), ceil(cap n_s)))), optionally rounded up to
// a multiple.  Everything in double; every thread of the workgroup computes the same values.
// ---------------------------------------------------------------------------
struct Budget {
  double sigma2, D_hat, b_star;
  int b;
};
__device__ __forceinline__ double numerator_rho(int n_s, int b0, double sum_r_sq, double sum_r2, double nhat_sq,
                                                double* tr_sigma) {
  const double b0d = (double)b0, ns = (double)n_s;
  *tr_sigma = b0 > 1 ? fmax(sum_r2 - sum_r_sq / b0d, 0.0) / (b0d - 1.0) : 0.0;
  const double num = ns * sqrt(*tr_sigma), nn = sqrt(nhat_sq);
  return nn > 0.0 ? num / nn : (num > 0.0 ? INFINITY : 0.0);
}
// w_range: an interval length that holds every residual weight (only read for the range-based Hoeffding budget).
__device__ __forceinline__ Budget algorithm2_budget(const HeadArgs& A, int n_s, int b0, double D_f, double sum_w,
                                                    double sum_w2, double rho_N, double w_range) {
  Budget B;
  const double b0d = (double)b0, ns = (double)n_s;
  const double w_bar = sum_w / b0d;
  // unbiased variance from the two sums; the scores are shifted so that the largest weight is 1
  B.sigma2 = b0 > 1 ? fmax(sum_w2 - sum_w * w_bar, 0.0) / (b0d - 1.0) : 0.0;
  B.D_hat = D_f + ns * w_bar;
  const double rho_D = ns * sqrt(B.sigma2) / B.D_hat;
  if (A.target == VATT_TARGET_D && A.range_factor > 0.0) {
    // Hoeffding's inequality proper: b* = (ln(2 / delta) / 2) (n_s R / (eps D))^2, no variance involved
    const double t = ns * w_range / (A.eps * B.D_hat);
    B.b_star = A.range_factor * t * t;
  } else if (A.target == VATT_TARGET_D) {
    const double t = A.z_half * rho_D / A.eps;
    B.b_star = t * t;
  } else if (A.target == VATT_TARGET_N) {
    const double t = A.z_half * rho_N / A.eps;
    B.b_star = t * t;
  } else {
    const double t = 2.0 * A.z_quarter * (rho_D + rho_N) / A.eps;
    B.b_star = t * t;
  }
  const int cap = (int)ceil(A.cap_frac * ns);
  int want = n_s;
  if (B.b_star == B.b_star && B.b_star < ns) want = (int)ceil(B.b_star);
  int b = min(n_s, max(b0, min(want, cap)));
  // (optional) rounded up to a multiple, not beyond the largest value the rule above can give
  if (A.b_multiple > 1) b = min(min(n_s, max(b0, cap)), (b + A.b_multiple - 1) / A.b_multiple * A.b_multiple);
  B.b = min(b, A.b_max);
  return B;
}

// Accumulates weight * (8 bf16 values of a V row) into acc.
__device__ __forceinline__ void add_weighted_row(float (&acc)[8], float wt, const uint4& vv) {
  const uint32_t ww[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    acc[2 * c] += wt * bf16_lo(ww[c]);
    acc[2 * c + 1] += wt * bf16_hi(ww[c]);
  }
}

// The arguments every launch of the two kernels starts from.
inline void fill_head_args(HeadArgs& A, const Plan& pl, int phase, const int32_t* seq_lens, const uint64_t* seq_seeds,
                           void* ws, int32_t* out_idx, int32_t* out_counts, double* out_budget_raw,
                           float* out_stats) {
  const vatt_params& p = pl.p;
  char* w = static_cast<char*>(ws);
  A.scores = reinterpret_cast<const float*>(w + pl.off_scores);
  A.sub_max = reinterpret_cast<const float*>(w + pl.off_sub_max);
  A.n_sub = pl.n_sub;
  A.seq_lens = seq_lens;
  A.seq_seeds = seq_seeds;
  A.head_rec = reinterpret_cast<HeadRec*>(w + pl.off_head_rec);
  A.vstat_part = reinterpret_cast<const double*>(w + pl.off_vstat_part);
  A.out_idx = out_idx;
  A.out_counts = out_counts;
  A.out_budget_raw = out_budget_raw;
  A.out_stats = out_stats;
  A.sp = pl.sel;
  A.z_half = pl.z_half;
  A.range_factor = pl.range_factor;
  A.z_quarter = pl.z_quarter;
  A.eps = pl.eps;
  A.cap_frac = pl.cap_frac;
  A.seg_sink = pl.seg_off[0];
  A.seg_win = pl.seg_off[1];
  A.seg_topk = pl.seg_off[2];
  A.seg_base = pl.seg_off[3];
  A.seg_dyn = pl.seg_off[4];
  A.idx_cap = (int64_t)pl.idx_cap;
  A.n_pad = pl.n_pad;
  A.n_max = p.n_max;
  A.Hq = p.n_q_heads;
  A.target = p.target;
  A.phase = phase;
  A.small_batches = pl.sampler_small_batches;
  A.topk_general = pl.topk_general_path;
  A.draw_cap = pl.sampler_draw_cap;
  A.vstat_splits = pl.vstat_splits;
  A.head_dim = p.head_dim;
  A.k_max = pl.k_max;
  A.b0_max = pl.b0_max;
  A.b_max = pl.b_max;
  A.q_len = pl.q_len;
  A.nested = pl.nested_samples;
  A.group_major = pl.group_major;
  A.Hkv = p.n_kv_heads;
  A.b_multiple = pl.budget_multiple;
  A.ascending = pl.ascending_samples;
  A.dbg = reinterpret_cast<unsigned long long*>(w + pl.off_debug) + 64;
  A.given_idx = nullptr;
  A.given_cnt = nullptr;
  A.given_vstat = reinterpret_cast<const float*>(w + pl.off_vstat_part);
  A.given_splits = pl.given_splits;
  A.sparse = reinterpret_cast<const float*>(w + pl.off_sparse);
  A.place_sc = reinterpret_cast<float*>(w + pl.off_sparse);
  A.v = nullptr;
  A.L = pl.kv_v;
  A.part = nullptr;
  A.splits = 1;
  A.split_shift = 0;
  A.group = pl.group;
  A.glist_cap = 0;
  A.dlist_cap = 0;
  A.pre_tok = nullptr;
  A.pre_flags = nullptr;
  A.gq = nullptr;
  A.gk = nullptr;
  A.Lk = pl.kv_k;
  A.sm_scale = pl.sm_scale;
  A.rcache = nullptr;
  A.rc = CacheLayout{};
  A.base_slot = reinterpret_cast<int32_t*>(w + pl.off_base_slot);
}

}  // namespace
}  // namespace vatt
