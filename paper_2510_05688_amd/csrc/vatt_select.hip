// Index selection and budget: Algorithm 1 up to the final sample and all of Algorithm 2, per (sequence, query head),
// in one kernel with one workgroup per head.
//
// Top-k: the k largest scores of the middle region, ties to the lower token, i.e. the k smallest composites
// (~order_key(score), token).  Usual path: the score kernel leaves the largest score of every 8 keys; the k-th
// largest of those maxima is a lower bound of the k-th largest score (located to one bin of a 2048-bin LDS
// histogram), the 8-key sub-tiles that reach it are listed, their scores loaded, and the scores at or above the
// bound are the candidates, a few more than k.  The exact threshold among them: histogram over 2048
// equal-width score bins, the bin that holds rank k located by a workgroup scan, its few scores ranked as
// composites.  General path (short rows, very large k, long runs of equal scores): the same histogram selection
// streamed over the whole row, refined by further histograms over the integer keys when a bin holds many
// scores, and by token order inside a run of equal scores, so the result is exact for any data.
//
// Samples: sequential uniform draws from the middle region (Philox4x32-10 words, unbiased multiply-and-reject
// mapping), skipping top-k members and tokens drawn before; the first c accepted tokens are the sample (for
// c > n_s / 2 they are the tokens left out).  The kernel processes the draw sequence in batches: all draws of
// a batch are generated at once, repeated tokens are resolved to their earliest draw, and a prefix count in
// draw order finds where the sample is complete; the result equals the sequential procedure bit for bit.
//
// Floating-point sums are taken in a fixed order, or as fixed-point integers where the order depends on
// scheduling, so the statistics and the budget are reproducible too.
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

// NT = workgroup size.  FD = 0: selection only (the gather is a kernel of its own).  FD = head dimension: fused
// gather for small batches, where one workgroup per head would leave most of the chip idle and every kernel
// boundary is a visible part of the step: every head gets A.splits workgroups (blockIdx.z), each of which runs
// the whole selection (identical results in all of them: nothing is exchanged), keeps every A.splits-th token
// of the head's list in LDS, gathers those V rows and leaves a partial (sum w V, sum w) for the merge kernel.
// Only workgroup 0 of a head writes the index lists, counts, statistics and budget.  The rows of I_f are
// requested as soon as the top-k set is known and are added after the samplers have run.
template <int NT, int FD, bool PAGED>
__global__ __launch_bounds__(NT, FD > 0 ? 1 : 4) void head_kernel(HeadArgs A) {
  constexpr bool kFused = FD > 0;
  using O = HeadOps<NT>;
  using TKR = TopkOps<NT, RowView<NT>>;
  using TKC = TopkOps<NT, CandView<NT>>;
  using HeadSmem = typename O::HeadSmem;
  using Sampler = typename O::Sampler;
  constexpr int SW = NT / kWave;
  extern __shared__ __align__(16) unsigned char dyn_smem[];
  __shared__ TopkSmem ts;
  const int h = head_of_block((int)blockIdx.x, A.Hq, A.Hkv, A.group_major), b = blockIdx.y;
  const int bh = b * A.Hq + h;
  const int tid = threadIdx.x;
  const uint32_t split = kFused ? blockIdx.z : 0u, shift = kFused ? (uint32_t)A.split_shift : 0u;
  const uint32_t smask = (1u << shift) - 1u;
  const bool writer = split == 0u;  // this workgroup writes the head's outputs
  // The sub-tile maxima the score kernel left are requested first of all, before even the sequence length is
  // known (what lies beyond the row's own sub-tiles is masked once it is): the kernel starts with a chain of
  // dependent loads, and this takes one link out of it.  Rows of up to 8 * NT sub-tiles keep the maxima in
  // registers for the three passes below, longer rows stream them in every pass.
  constexpr int SU = NT >= 1024 ? 16 : 8;  // sub-tile maxima a thread has in flight (rows up to 131072 / 32768 tokens)
  const float* sub_max = A.sub_max + (int64_t)bh * A.n_sub;
  float sub_reg[SU];
#pragma unroll
  for (int u = 0; u < SU; ++u) {
    const int t = u * NT + tid;
    sub_reg[u] = t < A.n_sub ? sub_max[t] : -INFINITY;
  }
  uint4 pre_t = make_uint4(0u, 0u, 0u, 0u);
  uint32_t pre_f = 0u;
  bool pre_made = false;
  if (NT == kHeadThreads && A.pre_tok) {
    pre_t = A.pre_tok[(int64_t)bh * NT + tid];
    pre_f = A.pre_flags[(int64_t)bh * NT + tid];
    pre_made = (A.pre_flags[(int64_t)bh * NT] & 256u) != 0u;  // one word for the whole workgroup: uniform
  }
  // In a multi-query step b stands for (sequence, query token); query token t of q_len sees the sequence up to
  // and including itself, which leaves out the q_len - 1 - t newer tokens.
  const int seq = b / A.q_len, qtok = b - seq * A.q_len;
  const int n = max(min(max(A.seq_lens[seq], 1), A.n_max) - (A.q_len - 1 - qtok), 1);  // clamp, then the causal cut
  const HeadSizes hs = head_sizes(n, A.sp);
  const int words_max = ((A.n_max + 63) >> 6) << 1;  // an even number of words: bitmaps are also written 64 bits at a time
  const int words = (n + 31) >> 5;

  HeadSmem& sm = *reinterpret_cast<HeadSmem*>(dyn_smem);
  uint64_t* cand = reinterpret_cast<uint64_t*>(dyn_smem + ((sizeof(HeadSmem) + 15) & ~size_t(15)));
  uint32_t* qual = reinterpret_cast<uint32_t*>(cand + kCandCap);
  uint32_t* bm_f = qual + kCandCap;
  uint32_t* taken0 = bm_f + words_max;
  uint32_t* taken1 = taken0 + words_max;
  uint32_t* scratch = taken1 + words_max;
  uint32_t* wpre = scratch + words_max;
  uint32_t* mail = wpre + words_max;
  // (the 512-thread kernel can generate the first batches of both streams at once: the final sample's stream
  // then needs a scratch bitmap and mail slots of its own)
  constexpr bool kTwoStreams = NT == kHeadThreads;
  uint32_t* scratch1 = kTwoStreams ? mail + words_max : scratch;
  uint32_t* mail1 = kTwoStreams ? scratch1 + words_max : mail;
  // fused gather: this workgroup's share of I_f and of the final sample, and the cross-wave sums
  uint32_t* glist = mail1 + words_max;
  uint32_t* dlist = glist + (kFused ? A.glist_cap : 0);
  // (the scores of the listed tokens, so that the gather requests V rows only)
  float* glist_sc = reinterpret_cast<float*>(dlist + (kFused ? A.dlist_cap : 0));
  float* dlist_sc = glist_sc + (kFused ? A.glist_cap : 0);
  float* g_red = dlist_sc + (kFused ? A.dlist_cap : 0);
  // (I_f is dealt out in runs of consecutive list places: its top-k part is in ascending token order, so a
  // workgroup's rows then lie close together in the cache)
  uint32_t g_lo = 0, g_hi = 0;
  if (kFused) {
    const uint32_t n_f = (uint32_t)(hs.n_sink + hs.n_win + hs.k);
    const uint32_t run = min((n_f + smask) >> shift, (uint32_t)A.glist_cap);  // ceil(n_f / splits)
    g_lo = min(split * run, n_f);
    g_hi = min(g_lo + run, n_f);
  }
  auto to_glist = [&](uint32_t p, uint32_t tok, float sc) {
    if (kFused && p >= g_lo && p < g_hi) {
      glist[p - g_lo] = tok;
      glist_sc[p - g_lo] = sc;
    }
  };

  const float* row = A.scores + (int64_t)bh * A.n_pad;
  int32_t* idx = A.out_idx + (int64_t)bh * A.idx_cap;
  const uint64_t seed = A.seq_seeds[seq];

  VATT_STAMP(A.dbg, 0);
  // The score row is requested first (when it is kept in registers), so that its latency overlaps the
  // sampler work below.
  RowView<NT> rv;
  rv.row = row;
  rv.n = n;
  const float edge0 = (A.phase != 2 && tid < hs.n_sink) ? row[tid] : -INFINITY;
  const float edge1 = (A.phase != 2 && tid < hs.n_win) ? row[hs.mid_hi + tid] : -INFINITY;
  for (int w = tid; w < words; w += NT) {
    bm_f[w] = 0;
    taken0[w] = 0;
    taken1[w] = 0;
    scratch[w] = 0;
    mail[w] = kInv32;
    if (kTwoStreams) {
      scratch1[w] = 0;
      mail1[w] = kInv32;
    }
  }
  __syncthreads();

  // The draw sequences do not depend on the scores: the first batch of each stream is generated, and the
  // scores of the base-sample proposals are requested, before the top-k set is known.
  const uint32_t L = (uint32_t)max(hs.mid_hi - hs.mid_lo, 1);
  Sampler S0, S1;
  S0.taken = taken0;
  S0.scratch = scratch;
  S0.mail = mail;
  S0.bm_f = bm_f;
  S0.wpre = wpre;
  S0.row = row;
  S0.seed = seed;
  S0.stream = 0u;
  S0.head = (uint32_t)h;
  S0.query = (uint32_t)qtok;
  S0.L = L;
  S0.thr = (uint32_t)((0x100000000ull - (uint64_t)L) % (uint64_t)L);
  {
    const uint64_t dflt = 64ull * (uint64_t)L + 4096ull;
    S0.cap = (uint32_t)min(A.draw_cap ? (uint64_t)A.draw_cap : dflt, 0x80000000ull);
  }
  S0.m = 0.f;
  S0.dbg = A.dbg ? A.dbg + 200 : nullptr;
  S1 = S0;
  S1.taken = taken1;
  S1.scratch = scratch1;
  S1.mail = mail1;
  S1.stream = 1u;
  S1.dbg = A.dbg ? A.dbg + 300 : nullptr;
  DrawBatch spec0 = {}, spec1 = {};
  const bool want0 = hs.n_s > 0 && A.phase != 2 && hs.b0 < hs.n_s;
  const bool want1 = hs.n_s > 0 && A.phase != 1 && !A.nested;  // (a nested final sample rarely draws at all)
  const int n_sub = (n + kSubTile - 1) / kSubTile;
  const int sub_lo = (hs.mid_lo + kSubTile - 1) / kSubTile, sub_hi = hs.mid_hi / kSubTile;  // whole middle sub-tiles
  const bool sub_resident = n_sub <= SU * NT;
#pragma unroll
  for (int u = 0; u < SU; ++u) {
    const int t = u * NT + tid;
    sub_reg[u] = (sub_resident && t < n_sub) ? sub_reg[u] : -INFINITY;
  }
  // g(maxima[SU], first sub-tile of the batch): slot u is sub-tile first + u * NT + tid, -inf beyond the row
  auto each_sub_batch = [&](auto&& g) {
    if (sub_resident) {
      g(sub_reg, 0);
    } else {
      for (int base = 0; base < n_sub; base += NT * SU) {
        float v[SU];
#pragma unroll
        for (int u = 0; u < SU; ++u) {
          const int t = base + u * NT + tid;
          v[u] = t < n_sub ? sub_max[t] : -INFINITY;
        }
        g(v, base);
      }
    }
  };
  bool spec1_made = false, pair_made = false;
  if (kTwoStreams && want0 && want1 && 2 * ahead_blocks<NT>(A.small_batches) <= NT) {
    // both streams at once: the lower half of the workgroup generates the first batch of the base sample,
    // the upper half that of the final sample
    const int half = tid >= NT / 2 ? 1 : 0;
    const int blocks = ahead_blocks<NT>(A.small_batches);
    DrawBatch mine = {};
    if (pre_made) {
      // made ahead, while the scores were computed: the proposals are marked as drawn, and the scores of the
      // base sample's proposals are requested
      const uint32_t tk[4] = {pre_t.x, pre_t.y, pre_t.z, pre_t.w};
      uint32_t* tk_bm = half ? taken1 : taken0;
      mine.ok = pre_f & 15u;
      mine.first = (pre_f >> 4) & 15u;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        mine.tok[e] = min(max(tk[e], (uint32_t)hs.mid_lo), (uint32_t)max(hs.mid_hi - 1, hs.mid_lo));
        mine.sc[e] = row[mine.tok[e]];
        if ((mine.ok >> e) & 1u) atomicOr(&tk_bm[mine.tok[e] >> 5], 1u << (mine.tok[e] & 31));
      }
      mine.blocks = blocks;
      mine.have_sc = true;
    } else {
      O::make_batch(mine, half ? S1 : S0, hs, 0u, blocks, false, true, sm, tid - half * (NT / 2));
    }
    spec0.blocks = spec1.blocks = blocks;
    spec0.have_sc = true;
    if (half) spec1 = mine; else spec0 = mine;
    spec1_made = true;
    pair_made = true;
  } else if (want0) {
    O::make_batch(spec0, S0, hs, 0u, ahead_blocks<NT>(A.small_batches), false, true, sm, tid);
  }
  VATT_STAMP(A.dbg, 1);

  // ---- the head maximum m ----
  float m, lo_sub;  // lo_sub: the smallest maximum of a whole middle sub-tile
  {
    float v_max = -INFINITY, v_min = INFINITY;
    each_sub_batch([&](const float (&v)[SU], int base) {
#pragma unroll
      for (int u = 0; u < SU; ++u) {
        const int t = base + u * NT + tid;
        v_max = fmaxf(v_max, v[u]);
        v_min = (t >= sub_lo && t < sub_hi) ? fminf(v_min, v[u]) : v_min;
      }
    });
    v_max = wave_max(v_max);
    v_min = -wave_max(-v_min);
    if ((tid & 63) == 0) {
      ts.wf[0][tid >> 6] = v_max;
      ts.wf[1][tid >> 6] = v_min;
    }
    __syncthreads();
    m = ts.wf[0][0];
    lo_sub = ts.wf[1][0];
#pragma unroll
    for (int w = 1; w < SW; ++w) {
      m = fmaxf(m, ts.wf[0][w]);
      lo_sub = fminf(lo_sub, ts.wf[1][w]);
    }
  }
  S0.m = m;
  S1.m = m;
  VATT_STAMP(A.dbg, 2);

  int topk_flag = 0;
  uint32_t tau_key = 0u;  // largest composite key (~order key: the smallest score) among this thread's top-k members
  float acc_f32 = 0.f;  // this thread's share of D_f = sum over I_f of exp(s_i - m), kept in fp32 per thread
  double acc_f = 0.0;
  // ---- I_t (Algorithm 1, top-k step) ----
  if (A.phase != 2) {
    const int mid_len = hs.mid_hi - hs.mid_lo;
    if (hs.k > 0) {
      float sT = -INFINITY;
      uint32_t Tidx = kInv32;
      bool marked = false;
      uint64_t T_cand = ~0ull;   // fast path: members are the candidates with composite <= T_cand
      uint32_t n_cand_used = 0;
      if (hs.k < mid_len) {
        // Fast path.  A lower bound of the k-th largest score: the k-th largest of the sub-tile maxima (of
        // the sub-tiles that lie entirely in the middle region) has at least k middle scores at or above it.
        // Found to one histogram bin, it leaves a few more than k candidates, which are listed in LDS and
        // selected among exactly.
        bool have_T = false;
        if (sub_hi - sub_lo >= hs.k && !A.topk_general) {
          float bound = lo_sub;  // every middle sub-tile maximum is at or above this
          const float scale = (float)(kBins - 1) / (m - lo_sub);
          if (m > lo_sub && scale < 1e30f) {
            TKR::zero_hist(ts);
            each_sub_batch([&](const float (&v)[SU], int base) {
#pragma unroll
              for (int u = 0; u < SU; ++u) {
                const int t = base + u * NT + tid;
                const bool in = t >= sub_lo && t < sub_hi;
                atomicAdd(&ts.hist[in ? (uint32_t)((m - v[u]) * scale) : (uint32_t)kBins], 1u);
              }
            });
            __syncthreads();
            TKR::locate((uint32_t)hs.k, ts, sm);
            // the lower edge of the bin of the k-th largest maximum, a little further down for rounding
            bound = fmaxf(lo_sub, m - ((float)ts.j + 1.02f) / scale);
          }
          VATT_STAMP(A.dbg, 22);
          // sub-tiles that may hold a candidate: those that touch the middle region with a maximum at or
          // above the bound (order in the list does not matter)
          if (tid == 0) {
            ts.cand_n = 0;
            ts.qual_n = 0;
          }
          __syncthreads();
          const int sub_first = hs.mid_lo / kSubTile, sub_last = (hs.mid_hi + kSubTile - 1) / kSubTile;
          each_sub_batch([&](const float (&v)[SU], int base) {
            uint32_t hit = 0;
#pragma unroll
            for (int u = 0; u < SU; ++u) {
              const int t = base + u * NT + tid;
              hit |= ((t >= sub_first && t < sub_last && v[u] >= bound) ? 1u : 0u) << u;
            }
            const uint32_t mine = (uint32_t)__popc(hit);
            const uint32_t incl = wave_inclusive_scan_u32(mine);
            const uint32_t wave_tot = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
            if (wave_tot) {
              uint32_t at = 0;
              if ((tid & 63) == 0) at = atomicAdd(&ts.qual_n, wave_tot);
              at = (uint32_t)__builtin_amdgcn_readfirstlane((int)at);
              uint32_t pos = at + incl - mine;
#pragma unroll
              for (int u = 0; u < SU; ++u) {
                if ((hit >> u) & 1u) {
                  if (pos < (uint32_t)kCandCap) qual[pos] = (uint32_t)(base + u * NT + tid);
                  ++pos;
                }
              }
            }
          });
          __syncthreads();
          const uint32_t n_qual = ts.qual_n;
          VATT_STAMP(A.dbg, 23);
          VATT_NOTE(A.dbg, 27, n_qual);
          if (n_qual <= (uint32_t)kCandCap) {
            // candidates: the middle scores of those sub-tiles that are at or above the bound
            static_assert(kSubTile == 8, "two 16-byte loads per sub-tile");
            constexpr int Q = 2;  // sub-tiles a thread has in flight
            for (uint32_t q0 = 0; q0 < n_qual; q0 += NT * Q) {
              float sv[Q][kSubTile];
              int tok0[Q];
#pragma unroll
              for (int u = 0; u < Q; ++u) {
                const uint32_t q = q0 + u * NT + tid;
                const bool ok = q < n_qual;
                tok0[u] = ok ? (int)min(qual[min(q, (uint32_t)(kCandCap - 1))], (uint32_t)(sub_last - 1)) * kSubTile : -1;
                const float4* src = reinterpret_cast<const float4*>(row + max(tok0[u], 0));
                const float4 x = ok ? src[0] : make_float4(0.f, 0.f, 0.f, 0.f);
                const float4 y = ok ? src[1] : make_float4(0.f, 0.f, 0.f, 0.f);
                sv[u][0] = x.x; sv[u][1] = x.y; sv[u][2] = x.z; sv[u][3] = x.w;
                sv[u][4] = y.x; sv[u][5] = y.y; sv[u][6] = y.z; sv[u][7] = y.w;
              }
              if (q0 == 0 && want1 && !spec1_made) {
                // the final sample's first batch of draws is generated while these loads are in flight
                O::make_batch(spec1, S1, hs, 0u, ahead_blocks<NT>(A.small_batches), false, false, sm, tid);
                spec1_made = true;
              }
              uint32_t hit = 0;
#pragma unroll
              for (int u = 0; u < Q; ++u) {
#pragma unroll
                for (int e = 0; e < kSubTile; ++e) {
                  const int i = tok0[u] + e;
                  hit |= ((tok0[u] >= 0 && i >= hs.mid_lo && i < hs.mid_hi && sv[u][e] >= bound) ? 1u : 0u)
                         << (u * kSubTile + e);
                }
              }
              const uint32_t mine = (uint32_t)__popc(hit);
              const uint32_t incl = wave_inclusive_scan_u32(mine);
              const uint32_t wave_tot = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
              if (wave_tot) {
                uint32_t at = 0;
                if ((tid & 63) == 0) at = atomicAdd(&ts.cand_n, wave_tot);
                at = (uint32_t)__builtin_amdgcn_readfirstlane((int)at);
                uint32_t pos = at + incl - mine;
#pragma unroll
                for (int u = 0; u < Q; ++u) {
#pragma unroll
                  for (int e = 0; e < kSubTile; ++e) {
                    if ((hit >> (u * kSubTile + e)) & 1u) {
                      if (pos < (uint32_t)kCandCap)
                        cand[pos] = ((uint64_t)(~float_order_key(sv[u][e])) << 32) | (uint32_t)(tok0[u] + e);
                      ++pos;
                    }
                  }
                }
              }
            }
            __syncthreads();
          }
          const uint32_t n_cand = n_qual <= (uint32_t)kCandCap ? ts.cand_n : 0u;
          VATT_STAMP(A.dbg, 24);
          VATT_NOTE(A.dbg, 26, n_cand);
          if (n_cand <= (uint32_t)kCandCap && n_cand >= (uint32_t)hs.k) {
            CandView<NT> cv;
            cv.list = cand;
            cv.count = n_cand;
            uint64_t T = ~0ull;
            if (n_cand > (uint32_t)hs.k)
              T = TKC::threshold(cv, hs, (uint32_t)hs.k, n_cand, bound, m, scratch, wpre, ts, sm, A.dbg);
            // (the list order depends on scheduling: the members' weights are summed as 40-bit fixed-point
            // integers, whose sum does not depend on the order; every weight is at most 1)
            uint64_t fixed_sum = 0;
            for (uint32_t t = tid; t < n_cand; t += NT) {
              const uint64_t c = cand[t];
              if (c <= T) {
                const uint32_t i = min((uint32_t)c, (uint32_t)(n - 1));
                atomicOr(&bm_f[i >> 5], 1u << (i & 31));
                tau_key = max(tau_key, (uint32_t)(c >> 32));
                fixed_sum += (uint64_t)(__expf(float_from_order_key(~(uint32_t)(c >> 32)) - m) * 1099511627776.0f);
              }
            }
            fixed_sum = wave_sum(fixed_sum);
            __syncthreads();
            if ((tid & 63) == 0) ts.wq[tid >> 6] = fixed_sum;
            __syncthreads();
            if (tid == 0) {
              uint64_t tot = 0;
              for (int w = 0; w < SW; ++w) tot += ts.wq[w];
              acc_f += (double)tot * (1.0 / 1099511627776.0);
            }
            have_T = true;
            marked = true;
            T_cand = T;
            n_cand_used = n_cand;
          }
        }
        if (!have_T) {
          topk_flag = kFlagTopkGeneral;
          // General path: histogram over the whole row.  It needs the smallest score of the middle region.
          float v_min = INFINITY, v_max = -INFINITY;
          rv.for_each(hs, [&](float s, int, bool mid) {
            v_min = mid ? fminf(v_min, s) : v_min;
            v_max = mid ? fmaxf(v_max, s) : v_max;
          });
          v_min = -wave_max(-v_min);
          v_max = wave_max(v_max);
          __syncthreads();
          if ((tid & 63) == 0) {
            ts.wf[0][tid >> 6] = v_max;
            ts.wf[1][tid >> 6] = v_min;
          }
          __syncthreads();
          float smax = ts.wf[0][0], smin = ts.wf[1][0];
#pragma unroll
          for (int w = 1; w < SW; ++w) {
            smax = fmaxf(smax, ts.wf[0][w]);
            smin = fminf(smin, ts.wf[1][w]);
          }
          const uint64_t T = TKR::threshold(rv, hs, (uint32_t)hs.k, (uint32_t)mid_len, smin, smax, scratch, wpre, ts,
                                            sm, A.dbg);
          sT = float_from_order_key(~(uint32_t)(T >> 32));
          Tidx = (uint32_t)T;
        }
      }
      VATT_STAMP(A.dbg, 3);
      if (!marked) {
        // Members of the top-k set go into the bitmap: slot u of a wave holds 64 consecutive tokens, so the
        // wave's compare mask is two whole bitmap words, stored by one lane.  A score equal to the threshold
        // score is rare and sends its group through the full comparison.  The weights of the members are
        // added on the way.
        uint64_t* bm64 = reinterpret_cast<uint64_t*>(bm_f);
        rv.for_each_group(hs, [&](const float (&s)[RowView<NT>::kGroup], int i0, auto tag) {
          constexpr int G = RowView<NT>::kGroup;
          constexpr bool kInside = decltype(tag)::value;
          const int first0 = i0 - (tid & 63);  // token of lane 0 in slot 0: a multiple of 64
#pragma unroll
          for (int u = 0; u < G; ++u) {
            const int i = i0 + u * NT;
            const bool mid = kInside || (i >= hs.mid_lo && i < hs.mid_hi);
            const bool take = mid && (s[u] > sT || (s[u] == sT && (uint32_t)i <= Tidx));
            const uint64_t mask = __ballot(take);
            if ((tid & 63) == 0 && (kInside || first0 + u * NT < n)) bm64[(first0 + u * NT) >> 6] = mask;
            if (mask) acc_f32 += take ? __expf(s[u] - m) : 0.f;
            tau_key = take ? max(tau_key, ~float_order_key(s[u])) : tau_key;
          }
        });
        __syncthreads();
      }
      // ascending token list from the bitmap
      O::word_prefix(bm_f, words, wpre, sm);
      if (marked) {
        // every member sits in the candidate list: its place in the ascending list is the number of members
        // below it, from the word prefix and the bits below its own (no thread walks a crowded word)
        for (uint32_t t = tid; t < n_cand_used; t += NT) {
          const uint64_t c = cand[t];
          if (c <= T_cand) {
            const uint32_t i = min((uint32_t)c, (uint32_t)(n - 1));
            const uint32_t pos = wpre[i >> 5] + (uint32_t)__popc(bm_f[i >> 5] & ((1u << (i & 31)) - 1u));
            if (writer && pos < (uint32_t)A.k_max) idx[A.seg_topk + pos] = (int32_t)i;
            to_glist((uint32_t)(hs.n_sink + hs.n_win) + pos, i, float_from_order_key(~(uint32_t)(c >> 32)));
          }
        }
      } else {
        const int wpt = (words + NT - 1) / NT;
        const int w0 = tid * wpt;
        for (int w = w0; w < min(w0 + wpt, words); ++w) {
          uint32_t bits = bm_f[w];
          uint32_t pos = wpre[w];
          while (bits) {
            const int i = (w << 5) + (__ffs(bits) - 1);
            bits &= bits - 1u;
            if (writer && pos < (uint32_t)A.k_max) idx[A.seg_topk + pos] = i;
            if (kFused) to_glist((uint32_t)(hs.n_sink + hs.n_win) + pos, (uint32_t)i, row[i]);
            ++pos;
          }
        }
      }
      VATT_STAMP(A.dbg, 4);
    }
    // weights of the sink and window tokens (their scores were requested at the start)
    acc_f32 += __expf(edge0 - m) + __expf(edge1 - m);  // exp(-inf) = 0 for threads without a token
    for (int i = tid + NT; i < hs.n_sink; i += NT) acc_f32 += __expf(row[i] - m);
    for (int i = tid + NT; i < hs.n_win; i += NT) acc_f32 += __expf(row[hs.mid_hi + i] - m);
    for (int i = tid; i < hs.n_sink; i += NT) {
      if (writer) idx[A.seg_sink + i] = i;
      if (kFused) to_glist((uint32_t)i, (uint32_t)i, i == tid ? edge0 : row[i]);
    }
    for (int i = tid; i < hs.n_win; i += NT) {
      if (writer) idx[A.seg_win + i] = hs.mid_hi + i;
      if (kFused) to_glist((uint32_t)(hs.n_sink + i), (uint32_t)(hs.mid_hi + i), i == tid ? edge1 : row[hs.mid_hi + i]);
    }
  } else {
    // phase 2: rebuild the top-k bitmap from the list written in phase 1
    for (int t = tid; t < hs.k; t += NT) {
      const int i = O::list_tok(idx, A.seg_topk + t, n);
      O::mark_bit(bm_f, (uint32_t)i);
      acc_f += (double)__expf(row[i] - m);
    }
    for (int i = tid; i < hs.n_sink; i += NT) acc_f += (double)__expf(row[i] - m);
    for (int i = tid; i < hs.n_win; i += NT) acc_f += (double)__expf(row[hs.mid_hi + i] - m);
  }
  VATT_STAMP(A.dbg, 30);
  __syncthreads();
  VATT_STAMP(A.dbg, 31);

  // Fused gather, first part: the V rows (and scores) of this workgroup's share of I_f are requested now and
  // added after the samplers have run.  LPR adjacent lanes read one row; NG rows per round, UF rounds in flight.
  constexpr int LPR = kFused ? FD / 8 : 16;
  constexpr int NG = NT / LPR;
  constexpr int UF = 8;
  const int g_sub = tid % LPR, g_grp = tid / LPR;
  const int kvh = kFused ? h / A.group : 0;
  float gacc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float gdsum = 0.f;
  uint4 fv[UF];
  float fs[UF];
  int my_nf = 0;
  // contiguous cache: this lane's 8 columns of row 0 of the head's V slice
  const uint16_t* v_head = (kFused && !PAGED)
                               ? A.v + (int64_t)seq * A.L.seq_stride + (int64_t)kvh * A.L.head_stride + g_sub * 8
                               : nullptr;
  // UF rows of a list at once, without branches: all list entries (and their scores) are read from LDS first,
  // then all rows are requested.  The lists are padded to whole calls, so the LDS reads need no bound; a slot
  // beyond the list reads row 0 and gets the score -inf (weight exp(-inf - m) = 0).  (Written with a per-slot
  // condition, every slot became a branch of its own with an LDS wait inside: sixteen serial LDS round trips.)
  // HaveSc: the scores of the listed tokens are in LDS (list_sc), else they are read from the score row.
  auto load_rows = [&](const uint32_t* list, const float* list_sc, int j0, int count, float (&sc)[UF], uint4 (&vv)[UF],
                       auto have_sc) {
    constexpr bool HaveSc = decltype(have_sc)::value;
    uint32_t t[UF];
    const int jb = j0 + g_grp;
#pragma unroll
    for (int u = 0; u < UF; ++u) {
      t[u] = list[jb + u * NG];
      sc[u] = HaveSc ? list_sc[jb + u * NG] : 0.f;
    }
    int blk[UF];
    bool valid[UF];
#pragma unroll
    for (int u = 0; u < UF; ++u) {
      valid[u] = jb + u * NG < count;
      t[u] = valid[u] ? min(t[u], (uint32_t)(n - 1)) : 0u;
      blk[u] = kv_block<PAGED>(A.L, seq, (int)t[u]);  // (paged cache: all block-table entries before any row)
    }
#pragma unroll
    for (int u = 0; u < UF; ++u) {
      if constexpr (!HaveSc) sc[u] = row[t[u]];
      if constexpr (PAGED) vv[u] = load_stream_16(A.v + kv_row_offset_in<true>(A.L, seq, kvh, (int)t[u], blk[u]) + g_sub * 8);
      else vv[u] = load_stream_16(v_head + t[u] * (uint32_t)(kFused ? FD : 1));  // (n_max * d < 2^32)
    }
#pragma unroll
    for (int u = 0; u < UF; ++u) sc[u] = valid[u] ? sc[u] : -INFINITY;
  };
  using ScInLds = std::true_type;
  using ScInRow = std::false_type;
  if constexpr (kFused) my_nf = (int)(g_hi - g_lo);

  VATT_STAMP(A.dbg, 32);
  if (want1 && !spec1_made) O::make_batch(spec1, S1, hs, 0u, ahead_blocks<NT>(A.small_batches), false, false, sm, tid);

  // ---- I_bs (Algorithm 2, base sample) and the sums over it ----
  int flags = topk_flag;
  double acc_w = 0.0, acc_w2 = 0.0;
  // Fused gather, usual case (both first batches at hand, base sample neither the whole residual nor taken as a
  // complement): the draws of both streams are tested against the top-k set and counted in draw order by ONE
  // workgroup scan (the lower half of the workgroup holds the base sample's stream, the upper half the final
  // sample's; the two counts travel in the halves of one word).  The base sample is complete if its first
  // batch holds b0 accepted draws.  And since the budget is never below b0, the first b0 accepted draws of the
  // other stream belong to the final sample whatever the budget turns out to be (unless it asks for so much
  // that the sample is taken as a complement): their V rows are requested now, with those of I_f, and
  // are in when the budget is known.
  bool fast_base = false, spec_dyn = false;
  uint32_t acc_bits = 0, acc_pos = 0, tot1 = 0;
  const int half = tid >= NT / 2 ? 1 : 0;
  float dacc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};  // final-sample rows, before the factor n_s / b
  float ddsum = 0.f;
  uint4 dv[UF];
  float ds[UF];
  int my_spec = 0;
  // Without the fused gather the same shortcut saves the second scan and the samplers' own passes; the sorted
  // and the nested forms of the lists are made by the general path only.
  if (kTwoStreams && A.phase == 0 && (kFused || (!A.ascending && !A.nested))) {
    const uint32_t ns = (uint32_t)hs.n_s, c0 = (uint32_t)hs.b0;
    if (pair_made && hs.n_s > 0 && c0 < ns && 2u * c0 <= ns) {
      const DrawBatch& B = half ? spec1 : spec0;
      acc_bits = B.first & ~O::test_bits4(bm_f, B.tok);
      uint32_t total;
      const uint32_t excl = block_exclusive_scan<NT>((uint32_t)__popc(acc_bits) << (half ? 16 : 0), &total, sm.scan);
      const uint32_t tot0 = total & 0xffffu;
      tot1 = total >> 16;
      acc_pos = half ? excl >> 16 : excl & 0xffffu;
      fast_base = tot0 >= c0;
      spec_dyn = fast_base && tot1 >= c0;
    }
    if (fast_base) {
      uint32_t pos = acc_pos;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool a = (acc_bits >> e) & 1u;
        const bool take = a && pos < (uint32_t)hs.b0;
        if (!half) {
          if (take && writer && pos < (uint32_t)A.b0_max) idx[A.seg_base + pos] = (int32_t)spec0.tok[e];
          const double w = take ? (double)__expf(spec0.sc[e] - m) : 0.0;
          acc_w += w;
          acc_w2 += w * w;
        } else if (kFused && spec_dyn && take && (pos & smask) == split && (pos >> shift) < (uint32_t)A.dlist_cap) {
          dlist[pos >> shift] = spec1.tok[e];
          dlist_sc[pos >> shift] = spec1.sc[e];
        }
        pos += a ? 1u : 0u;
      }
      if constexpr (kFused) {
        __syncthreads();
        VATT_STAMP(A.dbg, 5);
        load_rows(glist, glist_sc, 0, my_nf, fs, fv, ScInLds{});
        if (spec_dyn) {
          my_spec = hs.b0 > (int)split ? (int)(((uint32_t)hs.b0 - split + smask) >> shift) : 0;
          my_spec = min(my_spec, A.dlist_cap);
          load_rows(dlist, dlist_sc, 0, my_spec, ds, dv, ScInLds{});
        }
      }
    }
  }
  if (hs.n_s > 0 && !fast_base) {
    if (A.phase != 2) {
      Emit E0 = emit_to(idx + A.seg_base, (uint32_t)A.b0_max);
      E0.global = writer;
      const int f = O::draw_sample(S0, hs, (uint32_t)hs.b0, spec0, want0, A.small_batches, E0, &acc_w, &acc_w2, sm);
      flags |= ((f & 1) ? kFlagBaseComplement : 0) | ((f & 2) ? kFlagBaseBatches : 0) | ((f & 4) ? kFlagDrawCap : 0);
      if (A.ascending && !(f & 1))
        O::sort_ascending(idx + A.seg_base, (uint32_t)min(hs.b0, A.b0_max), scratch, wpre, n, sm);
      VATT_STAMP(A.dbg, 5);
    } else {
      for (int t = tid; t < hs.b0; t += NT) {
        const double wgt = (double)__expf(row[O::list_tok(idx, A.seg_base + t, n)] - m);
        acc_w += wgt;
        acc_w2 += wgt * wgt;
      }
    }
  }
  acc_f += (double)acc_f32;
  if (A.phase == 1) {
    if (tid == 0) {
      HeadRec r;
      r.m = m;
      r.scale = 0.f;
      r.n = n;
      r.n_sink = hs.n_sink;
      r.n_win = hs.n_win;
      r.k = hs.k;
      r.b = hs.n_s > 0 ? hs.b0 : 0;  // the statistics pass walks the base sample
      r.n_s = hs.n_s;
      r.b_keep = 0;
      r.base_cached = 0;
      A.head_rec[bh] = r;
      A.out_counts[(int64_t)bh * 8 + 7] = flags;
    }
    return;
  }

  // ---- statistics (Algorithm 2, get-stats): w_i = exp(s_i - m) ----
  // For the range-based Hoeffding budget: every residual token scores at most the weakest top-k member, so the
  // residual weights lie in [0, exp(min_{I_t} s - m)]; without a top-k set only w <= 1 is known.
  double w_range = 1.0;
  if (A.range_factor > 0.0 && hs.k > 0) {
    const uint32_t wk = wave_max_u32(tau_key);
    if ((tid & 63) == 0) ts.wu[0][tid >> 6] = wk;
    __syncthreads();
    uint32_t key = 0u;
#pragma unroll
    for (int w = 0; w < SW; ++w) key = max(key, ts.wu[0][w]);
    w_range = exp((double)float_from_order_key(~key) - (double)m);
  }
  double sums[3] = {acc_f, acc_w, acc_w2};
  O::block_sum(sums, sm);
  VATT_STAMP(A.dbg, 6);
  const double D_f = sums[0];
  double sigma2 = 0.0, b_star = 0.0, tr_sigma = 0.0, nhat_sq = 0.0;
  int bfin = 0;
  if (hs.n_s > 0) {
    const double b0d = (double)hs.b0, ns = (double)hs.n_s;
    double rho_N = 0.0;
    if (A.target != VATT_TARGET_D) {
      // numerator statistics from the V pass: per split {N_f[d], R1[d], R2, pad}
      const int d = A.head_dim;
      const int stride = 2 * d + 2;
      const double* vp = A.vstat_part + (int64_t)bh * A.vstat_splits * stride;
      double t3[3] = {0.0, 0.0, 0.0};
      if (tid < d) {
        double nf = 0.0, r1 = 0.0;
        for (int s = 0; s < A.vstat_splits; ++s) {
          nf += vp[s * stride + tid];
          r1 += vp[s * stride + d + tid];
        }
        const double nh = nf + ns * r1 / b0d;
        t3[0] = nh * nh;
        t3[1] = r1 * r1;
      }
      if (tid == 0)
        for (int s = 0; s < A.vstat_splits; ++s) t3[2] += vp[s * stride + 2 * d];
      O::block_sum(t3, sm);
      nhat_sq = t3[0];
      rho_N = numerator_rho(hs.n_s, hs.b0, t3[1], t3[2], nhat_sq, &tr_sigma);
    }
    const Budget bud = algorithm2_budget(A, hs.n_s, hs.b0, D_f, sums[1], sums[2], rho_N, w_range);
    sigma2 = bud.sigma2;
    b_star = bud.b_star;
    bfin = bud.b;
    const double D_hat = bud.D_hat;
    if (tid == 0 && writer && A.out_stats) {
      float* st = A.out_stats + (int64_t)bh * 4;
      st[0] = (float)D_hat;
      st[1] = (float)sigma2;
      st[2] = (float)tr_sigma;
      st[3] = (float)nhat_sq;
    }
  } else if (tid == 0 && writer && A.out_stats) {
    float* st = A.out_stats + (int64_t)bh * 4;
    st[0] = (float)D_f;
    st[1] = st[2] = st[3] = 0.f;
  }

  VATT_STAMP(A.dbg, 7);
  // ---- I_dyn (Algorithm 1, final sample) ----
  bool fast_dyn = false;
  {
    if constexpr (kFused) {
      if (!fast_base) load_rows(glist, glist_sc, 0, my_nf, fs, fv, ScInLds{});
    }
    // the first batch of draws holds the whole final sample, and it is not taken as a complement: its members
    // are the accepted draws counted above, up to the budget
    fast_dyn = spec_dyn && (uint32_t)bfin <= tot1 && 2u * (uint32_t)bfin <= (uint32_t)hs.n_s;
    if (fast_dyn) {
      uint32_t pos = acc_pos;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool a = (acc_bits >> e) & 1u;
        if (half && a && pos < (uint32_t)bfin) {
          if (writer && pos < (uint32_t)A.b_max) idx[A.seg_dyn + pos] = (int32_t)spec1.tok[e];
          if (kFused && pos >= (uint32_t)hs.b0 && (pos & smask) == split && (pos >> shift) < (uint32_t)A.dlist_cap) {
            dlist[pos >> shift] = spec1.tok[e];
            dlist_sc[pos >> shift] = spec1.sc[e];
          }
        }
        pos += a ? 1u : 0u;
      }
      if (kFused) __syncthreads();
    }
  }
  if (bfin > 0 && !fast_dyn) {
    Emit E1 = emit_to(idx + A.seg_dyn, (uint32_t)A.b_max);
    E1.global = writer;
    if (kFused) {
      E1.lds = dlist;
      E1.lds_cap = (uint32_t)A.dlist_cap;
      E1.shift = shift;
      E1.split = split;
    }
    const int f = (!kFused && A.nested)
                      ? O::draw_nested(S1, hs, (uint32_t)hs.b0, (uint32_t)bfin, bm_f, idx + A.seg_base,
                                       idx + A.seg_dyn, (uint32_t)A.b_max, A.small_batches, sm)
                      : O::draw_sample(S1, hs, (uint32_t)bfin, spec1, want1, A.small_batches, E1, nullptr, nullptr, sm);
    flags |= ((f & 1) ? kFlagDynComplement : 0) | ((f & 2) ? kFlagDynBatches : 0) | ((f & 4) ? kFlagDrawCap : 0);
    if (!kFused && A.ascending && !A.nested && !(f & 1))
      O::sort_ascending(idx + A.seg_dyn, (uint32_t)min(bfin, A.b_max), scratch, wpre, n, sm);
    VATT_STAMP(A.dbg, 8);
  }
  if (tid == 0 && writer) {
    int32_t* c = A.out_counts + (int64_t)bh * 8;
    const int prev = (A.phase == 2) ? c[7] : 0;
    c[0] = hs.n_sink;
    c[1] = hs.n_win;
    c[2] = hs.k;
    c[3] = hs.n_s > 0 ? hs.b0 : 0;
    c[4] = bfin;
    c[5] = hs.n_s;
    c[6] = n;
    c[7] = prev | flags;
    if (A.out_budget_raw) A.out_budget_raw[bh] = b_star;
    HeadRec r;
    r.m = m;
    r.scale = bfin > 0 ? (float)((double)hs.n_s / (double)bfin) : 0.f;
    r.n = n;
    r.n_sink = hs.n_sink;
    r.n_win = hs.n_win;
    r.k = hs.k;
    r.b = bfin;
    r.n_s = hs.n_s;
    r.b_keep = (A.nested && bfin > 0) ? hs.b0 : 0;
    r.base_cached = 0;
    A.head_rec[bh] = r;
  }
  VATT_STAMP(A.dbg, 9);

  // Fused gather, second part: add the rows of I_f that were requested above, then the rest of I_f (only long
  // lists have one), then this workgroup's share of the final sample with the weight factor n_s / b.
  if constexpr (kFused) {
    auto add_rows = [&](float (&acc)[8], float& dsum, const float (&sc)[UF], const uint4 (&vv)[UF]) {
#pragma unroll
      for (int u = 0; u < UF; ++u) {
        const float wt = __expf(sc[u] - m);
        add_weighted_row(acc, wt, vv[u]);
        dsum += g_sub == 0 ? wt : 0.f;
      }
    };
    add_rows(gacc, gdsum, fs, fv);
    for (int j0 = UF * NG; j0 < my_nf; j0 += UF * NG) {
      load_rows(glist, glist_sc, j0, my_nf, fs, fv, ScInLds{});
      add_rows(gacc, gdsum, fs, fv);
    }
    int my_nd = bfin > (int)split ? (int)(((uint32_t)bfin - split + smask) >> shift) : 0;
    my_nd = min(my_nd, A.dlist_cap);
    int j_done = 0;  // entries of this workgroup's share of the final sample that are already requested
    if (fast_dyn) {
      add_rows(dacc, ddsum, ds, dv);  // (slots beyond the list carry weight 0)
      j_done = min(UF * NG, my_spec);
      // rows requested ahead cover the first b0 tokens; what the budget adds comes after them in the list
    }
    for (int j0 = j_done; j0 < my_nd; j0 += UF * NG) {
      if (fast_dyn) load_rows(dlist, dlist_sc, j0, my_nd, ds, dv, ScInLds{});
      else load_rows(dlist, dlist_sc, j0, my_nd, ds, dv, ScInRow{});
      add_rows(dacc, ddsum, ds, dv);
    }
    const float tail_scale = bfin > 0 ? (float)((double)hs.n_s / (double)bfin) : 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) gacc[c] += tail_scale * dacc[c];
    gdsum += tail_scale * ddsum;
    VATT_STAMP(A.dbg, 10);
    // lane groups of a wave hold different rows: add them, then the waves through LDS
#pragma unroll
    for (int o = LPR; o < kWave; o <<= 1) {
#pragma unroll
      for (int c = 0; c < 8; ++c) gacc[c] += __shfl_xor(gacc[c], o);
    }
    gdsum = wave_sum_f32(gdsum);
    const int lane = tid & 63, wave = tid >> 6;
    float* g_d = g_red + SW * FD;
    if (lane < LPR) {
#pragma unroll
      for (int c = 0; c < 8; ++c) g_red[wave * FD + lane * 8 + c] = gacc[c];
    }
    if (lane == 0) g_d[wave] = gdsum;
    __syncthreads();
    float dtot = 0.f;
#pragma unroll
    for (int w2 = 0; w2 < SW; ++w2) dtot += g_d[w2];
    float* part = A.part + ((int64_t)bh * A.splits + split) * (FD + 4);
    if (tid < FD) {
      float a = 0.f;
#pragma unroll
      for (int w2 = 0; w2 < SW; ++w2) a += g_red[w2 * FD + tid];
      part[tid] = a;
    }
    if (tid == 0) part[FD] = dtot;
    VATT_STAMP(A.dbg, 11);
  }
}


// ---------------------------------------------------------------------------
// Selection with a caller-supplied top-k set (no score row exists).
//   phase 0: I_t = the supplied tokens that lie in the middle region, without repeats; ascending list;
//            sizes of Algorithm 1 from |I_t|; base sample drawn (its weights are not known yet).
//   phase 1: with the scores of I_f and I_bs at hand (sparse list): maximum, D_f, base-sample sums, budget of
//            Algorithm 2 for the denominator target, final sample.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int base_count_of(int n_s, const SelectParams& p) {
  int b0 = p.base_abs > 0 ? p.base_abs : (int)floor(p.base_frac * (double)n_s);
  b0 = b0 < 2 ? 2 : b0;
  return b0 > n_s ? n_s : b0;
}

// FD = 0: selection only.  FD = head dimension (phase 1 only): the gather is fused in for small batches, as in
// head_kernel: every head gets A.splits workgroups (blockIdx.z), each of which runs the whole second phase
// (identical results in all of them), keeps every A.splits-th token of the final sample in LDS, and gathers
// that share and a contiguous run of I_f: scores of I_f from the sparse list, scores of the sampled tokens from
// their K rows, V rows, running maximum per lane group (no head maximum bounds the sampled scores); one partial
// (N, D, maximum) per workgroup for given_merge_kernel.
template <int NT, int FD, bool PAGED>
__global__ __launch_bounds__(NT) void given_topk_kernel(HeadArgs A) {
  using O = HeadOps<NT>;
  using HeadSmem = typename O::HeadSmem;
  using Sampler = typename O::Sampler;
  constexpr int SW = NT / kWave;
  constexpr bool kFused = FD > 0;
  extern __shared__ __align__(16) unsigned char dyn_smem[];
  __shared__ float s_wf[16];
  const uint32_t split = kFused ? blockIdx.z : 0u, shift = kFused ? (uint32_t)A.split_shift : 0u;
  const bool writer = split == 0u;
  const int h = head_of_block((int)blockIdx.x, A.Hq, A.Hkv, A.group_major), b = blockIdx.y;
  const int bh = b * A.Hq + h;
  const int tid = threadIdx.x;
  const int seq = b / A.q_len, qtok = b - seq * A.q_len;  // (sequence, query token) of a multi-query step
  const int n = max(min(max(A.seq_lens[seq], 1), A.n_max) - (A.q_len - 1 - qtok), 1);  // clamp, then the causal cut
  HeadSizes hs = head_sizes(n, A.sp);
  const int words_max = ((A.n_max + 63) >> 6) << 1;
  const int words = (n + 31) >> 5;
  HeadSmem& sm = *reinterpret_cast<HeadSmem*>(dyn_smem);
  uint64_t* cand = reinterpret_cast<uint64_t*>(dyn_smem + ((sizeof(HeadSmem) + 15) & ~size_t(15)));
  uint32_t* bm_f = reinterpret_cast<uint32_t*>(cand + kCandCap) + kCandCap;
  uint32_t* taken = bm_f + words_max;
  uint32_t* scratch = taken + 2 * words_max;
  uint32_t* wpre = scratch + words_max;
  uint32_t* mail = wpre + words_max;
  // fused gather (second phase): this workgroup's share of the final sample, and the cross-wave sums
  uint32_t* dlist = mail + words_max;
  float* g_red = reinterpret_cast<float*>(dlist + (kFused ? A.dlist_cap : 0));
  // fused scores (first phase): this workgroup's run of I_f, its share of the base sample and, for a base sample
  // from the random cache, the slots of that share
  uint32_t* glist = mail + words_max;
  uint32_t* blist = glist + (kFused ? A.glist_cap : 0);
  uint32_t* bslot = blist + (kFused ? A.dlist_cap : 0);
  const int n_fix0 = 0;
  (void)n_fix0;
  int32_t* idx = A.out_idx + (int64_t)bh * A.idx_cap;
  const int mid_len = hs.mid_hi - hs.mid_lo;

  for (int w = tid; w < words; w += NT) {
    bm_f[w] = 0;
    taken[w] = 0;
    scratch[w] = 0;
    mail[w] = kInv32;
  }
  __syncthreads();
  if (A.phase == 0) {
    const int cnt = min(max(A.given_cnt[bh], 0), A.k_max);
    const int32_t* given = A.given_idx + (int64_t)bh * A.k_max;
    // (four entries per thread are read before any is used: a read behind a condition waits for the one before)
    for (int t0 = 0; t0 < cnt; t0 += 4 * NT) {
      int g[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) g[u] = given[min(t0 + u * NT + tid, cnt - 1)];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (t0 + u * NT + tid < cnt && g[u] >= hs.mid_lo && g[u] < hs.mid_hi) O::mark_bit(bm_f, (uint32_t)g[u]);
    }
  } else {
    const HeadRec r = A.head_rec[bh];
    for (int t0 = 0; t0 < r.k; t0 += 4 * NT) {  // (four list entries per thread read together)
      int g[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) g[u] = O::list_tok(idx, A.seg_topk + min(t0 + u * NT + tid, r.k - 1), n);
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (t0 + u * NT + tid < r.k) O::mark_bit(bm_f, (uint32_t)g[u]);
    }
  }
  __syncthreads();
  const int k_eff = A.phase == 0 ? (int)O::word_prefix(bm_f, words, wpre, sm) : A.head_rec[bh].k;
  hs.k = k_eff;
  hs.n_s = mid_len - k_eff;
  hs.b0 = hs.n_s > 0 ? base_count_of(hs.n_s, A.sp) : 0;

  Sampler S;
  S.taken = taken;
  S.scratch = scratch;
  S.mail = mail;
  S.bm_f = bm_f;
  S.wpre = wpre;
  S.row = nullptr;
  S.seed = A.seq_seeds[seq];
  S.stream = A.phase == 0 ? 0u : 1u;
  S.head = (uint32_t)h;
  S.query = (uint32_t)qtok;
  S.L = (uint32_t)max(mid_len, 1);
  S.thr = (uint32_t)((0x100000000ull - (uint64_t)S.L) % (uint64_t)S.L);
  {
    const uint64_t dflt = 64ull * (uint64_t)S.L + 4096ull;
    S.cap = (uint32_t)min(A.draw_cap ? (uint64_t)A.draw_cap : dflt, 0x80000000ull);
  }
  S.m = 0.f;
  S.dbg = nullptr;
  const DrawBatch none = {};
  // (first phase fused with the scores: the run of [sink | window | top-k) this workgroup scores)
  int f0_lo = 0, f0_hi = 0;
  if (kFused && A.phase == 0) {
    const int n_f = hs.n_sink + hs.n_win + k_eff;
    const int run = min((n_f + (int)A.splits - 1) >> shift, A.glist_cap);
    f0_lo = min((int)split * run, n_f);
    f0_hi = min(f0_lo + run, n_f);
  }

  if (A.phase == 0) {
    {
      const int wpt = (words + NT - 1) / NT;
      const int w0 = tid * wpt;
      for (int w = w0; w < min(w0 + wpt, words); ++w) {
        uint32_t bits = bm_f[w];
        uint32_t pos = wpre[w];
        while (bits) {
          const int i = (w << 5) + (__ffs(bits) - 1);
          bits &= bits - 1u;
          if (writer && pos < (uint32_t)A.k_max) idx[A.seg_topk + pos] = i;
          if (kFused) {
            const int p = hs.n_sink + hs.n_win + (int)pos;  // place in [sink | window | top-k)
            if (p >= f0_lo && p < f0_hi) glist[p - f0_lo] = (uint32_t)i;
          }
          ++pos;
        }
      }
    }
    for (int i = tid; i < hs.n_sink; i += NT) {
      if (writer) idx[A.seg_sink + i] = i;
      if (kFused && i >= f0_lo && i < f0_hi) glist[i - f0_lo] = (uint32_t)i;
    }
    for (int i = tid; i < hs.n_win; i += NT) {
      if (writer) idx[A.seg_win + i] = hs.mid_hi + i;
      const int p = hs.n_sink + i;
      if (kFused && p >= f0_lo && p < f0_hi) glist[p - f0_lo] = (uint32_t)(hs.mid_hi + i);
    }
    __syncthreads();
    int flags = 0;
    bool cached = false;
    if (hs.n_s > 0 && A.rcache) {
      // base sample = the first b0 cached tokens, in slot order, that are residual tokens of this head; the
      // cache is used only when it holds that many
      const unsigned char* rec = cache_record(A.rcache, A.rc, seq, A.Hkv, h / A.group);
      const int cnt = min(max(*reinterpret_cast<const int32_t*>(rec), 0), A.rc.slots);
      const int32_t* ctok = reinterpret_cast<const int32_t*>(rec + 16);
      const int per = (cnt + NT - 1) / NT;
      const int s0 = min(tid * per, cnt), s1 = min(s0 + per, cnt);
      // a thread's slots four at a time: their tokens are read together, then their bitmap words together
      // (bit j of the result: slot sb + j holds a residual token; the token comes back in tk[j])
      auto residual4 = [&](int sb, int (&tk)[4]) -> uint32_t {
        uint32_t w[4], r4 = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) tk[j] = ctok[min(sb + j, cnt - 1)];
#pragma unroll
        for (int j = 0; j < 4; ++j) w[j] = bm_f[min(max(tk[j], 0), n - 1) >> 5];  // (a token outside the sequence fails the range test below)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          r4 |= ((sb + j < s1 && tk[j] >= hs.mid_lo && tk[j] < hs.mid_hi && !((w[j] >> (tk[j] & 31)) & 1u)) ? 1u : 0u) << j;
        return r4;
      };
      uint32_t mine = 0;
      for (int sb = s0; sb < s1; sb += 4) {
        int tk[4];
        mine += (uint32_t)__popc(residual4(sb, tk));
      }
      uint32_t total;
      uint32_t pos = block_exclusive_scan<NT>(mine, &total, sm.scan);
      cached = total >= (uint32_t)hs.b0;
      if (cached) {
        int32_t* slot_of = A.base_slot + (int64_t)bh * A.b0_max;
        const uint32_t lim = (uint32_t)min(hs.b0, A.b0_max);
        for (int sb = s0; sb < s1 && pos < lim; sb += 4) {
          int tk[4];
          const uint32_t r4 = residual4(sb, tk);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            if (((r4 >> j) & 1u) && pos < lim) {
              if (writer) {
                idx[A.seg_base + pos] = tk[j];
                slot_of[pos] = sb + j;
              }
              if (kFused && (pos & ((1u << shift) - 1u)) == split && (pos >> shift) < (uint32_t)A.dlist_cap) {
                blist[pos >> shift] = (uint32_t)tk[j];
                bslot[pos >> shift] = (uint32_t)(sb + j);
              }
              ++pos;
            }
          }
        }
        flags |= kFlagBaseFromCache;
      }
    }
    if (hs.n_s > 0 && !cached) {
      Emit E0 = emit_to(idx + A.seg_base, (uint32_t)A.b0_max);
      if (kFused) {
        E0.global = writer;
        E0.lds = blist;
        E0.lds_cap = (uint32_t)A.dlist_cap;
        E0.shift = shift;
        E0.split = split;
      }
      const int f = O::draw_sample(S, hs, (uint32_t)hs.b0, none, false, A.small_batches, E0, nullptr, nullptr, sm);
      flags |= ((f & 1) ? kFlagBaseComplement : 0) | ((f & 2) ? kFlagBaseBatches : 0) | ((f & 4) ? kFlagDrawCap : 0);
      if (!kFused && A.ascending && !(f & 1))
        O::sort_ascending(idx + A.seg_base, (uint32_t)min(hs.b0, A.b0_max), scratch, wpre, n, sm);
    }
    if (tid == 0 && writer) {
      HeadRec r;
      r.m = 0.f;
      r.scale = 0.f;
      r.n = n;
      r.n_sink = hs.n_sink;
      r.n_win = hs.n_win;
      r.k = k_eff;
      r.b = hs.b0;  // the score pass walks the base sample
      r.n_s = hs.n_s;
      r.b_keep = 0;
      r.base_cached = cached ? 1 : 0;
      A.head_rec[bh] = r;
      A.out_counts[(int64_t)bh * 8 + 7] = flags;
    }
    if constexpr (kFused) {
      // ---- the scores of this workgroup's share of I_f and of the base sample (denominator target) ----
      // s_i = sm_scale <K[i], q>, written to the tokens' places of the sparse list; rows as in the gather below:
      // tokens, block-table entries and rows each in a loop of their own over the slots in flight
      constexpr int LPR = FD / 8;
      constexpr int NG = NT / LPR;
      constexpr int UF = 8;
      const int g_sub = tid % LPR, g_grp = tid / LPR;
      const int kvh = h / A.group;
      __syncthreads();  // the lists of this workgroup's share are complete
      float* spw = const_cast<float*>(A.sparse) + (int64_t)bh * A.idx_cap;
      uint32_t qw[4];
      {
        const uint4 t = *reinterpret_cast<const uint4*>(A.gq + (int64_t)bh * FD + g_sub * 8);
        qw[0] = t.x;
        qw[1] = t.y;
        qw[2] = t.z;
        qw[3] = t.w;
      }
      auto score_of = [&](const uint4& kv) -> float {
        float a = 0.f;
        a = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, kv.x), __builtin_bit_cast(bf16x2_t, qw[0]), a, false);
        a = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, kv.y), __builtin_bit_cast(bf16x2_t, qw[1]), a, false);
        a = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, kv.z), __builtin_bit_cast(bf16x2_t, qw[2]), a, false);
        a = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, kv.w), __builtin_bit_cast(bf16x2_t, qw[3]), a, false);
        return group_sum<LPR>(a) * A.sm_scale + 0.0f;
      };
      const int my_nf = f0_hi - f0_lo;
      for (int j0 = g_grp; j0 < my_nf; j0 += NG * UF) {
        int tok[UF], blk[UF];
        uint4 kv[UF];
#pragma unroll
        for (int u = 0; u < UF; ++u) tok[u] = (int)min(glist[min(j0 + u * NG, my_nf - 1)], (uint32_t)(n - 1));
#pragma unroll
        for (int u = 0; u < UF; ++u) blk[u] = kv_block<PAGED>(A.Lk, seq, tok[u]);
#pragma unroll
        for (int u = 0; u < UF; ++u)
          kv[u] = load_stream_16(A.gk + kv_row_offset_in<PAGED>(A.Lk, seq, kvh, tok[u], blk[u]) + g_sub * 8);
#pragma unroll
        for (int u = 0; u < UF; ++u) {
          const float sc = score_of(kv[u]);
          const int j = j0 + u * NG;
          if (j < my_nf && g_sub == 0)
            spw[fixed_place(f0_lo + j, hs.n_sink, hs.n_win, A.seg_sink, A.seg_win, A.seg_topk)] = sc;
        }
      }
      int my_nb = hs.n_s > 0 && hs.b0 > (int)split ? (int)(((uint32_t)hs.b0 - split + ((1u << shift) - 1u)) >> shift) : 0;
      my_nb = min(my_nb, A.dlist_cap);
      const unsigned char* crec = cached ? cache_record(A.rcache, A.rc, seq, A.Hkv, kvh) : nullptr;
      for (int j0 = g_grp; j0 < my_nb; j0 += NG * UF) {
        int tok[UF], blk[UF];
        uint4 kv[UF];
        if (cached) {
          // the copies of the rows in the cache: rows of neighbouring slots, shared by the group's heads
#pragma unroll
          for (int u = 0; u < UF; ++u) tok[u] = (int)min(bslot[min(j0 + u * NG, my_nb - 1)], (uint32_t)(A.rc.slots - 1));
#pragma unroll
          for (int u = 0; u < UF; ++u)
            kv[u] = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(crec + A.rc.off_k) +
                                                    (int64_t)tok[u] * FD + g_sub * 8);
        } else {
#pragma unroll
          for (int u = 0; u < UF; ++u) tok[u] = (int)min(blist[min(j0 + u * NG, my_nb - 1)], (uint32_t)(n - 1));
#pragma unroll
          for (int u = 0; u < UF; ++u) blk[u] = kv_block<PAGED>(A.Lk, seq, tok[u]);
#pragma unroll
          for (int u = 0; u < UF; ++u)
            kv[u] = load_stream_16(A.gk + kv_row_offset_in<PAGED>(A.Lk, seq, kvh, tok[u], blk[u]) + g_sub * 8);
        }
#pragma unroll
        for (int u = 0; u < UF; ++u) {
          const float sc = score_of(kv[u]);
          const int j = j0 + u * NG;
          if (j < my_nb && g_sub == 0) spw[A.seg_base + (((int64_t)j << shift) | split)] = sc;
        }
      }
    }
    return;
  }

  // ---- phase 1 ----
  // scores of [sink | window | top-k | base sample], a few per thread, requested together
  const float* sp = A.sparse + (int64_t)bh * A.idx_cap;
  const int n_fix = hs.n_sink + hs.n_win + k_eff, n_all = n_fix + hs.b0;
  // (places by arithmetic and loads without a condition around them, so that a thread's loads go out together;
  // a slot beyond the list repeats the last entry and then counts as -inf)
  auto place_of = [&](int p) -> int64_t {
    const int64_t fixed = fixed_place(p, hs.n_sink, hs.n_win, A.seg_sink, A.seg_win, A.seg_topk);
    return p < n_fix ? fixed : A.seg_base + (p - n_fix);
  };
  constexpr int U = 4;
  auto load_batch = [&](int base, float (&v)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = sp[place_of(min(base + u * NT + tid, n_all - 1))];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = base + u * NT + tid < n_all ? v[u] : -INFINITY;
  };
  float v_max = -INFINITY;
  float v_first[U] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};  // the first batch stays in registers for the second pass
  for (int base = 0; base < n_all; base += NT * U) {
    float v[U];
    load_batch(base, v);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      v_max = fmaxf(v_max, v[u]);
      if (base == 0) v_first[u] = v[u];
    }
  }
  v_max = wave_max(v_max);
  if ((tid & 63) == 0) s_wf[tid >> 6] = v_max;
  __syncthreads();
  float m = s_wf[0];
#pragma unroll
  for (int w = 1; w < SW; ++w) m = fmaxf(m, s_wf[w]);
  double acc_f = 0.0, acc_w = 0.0, acc_w2 = 0.0;
  for (int base = 0; base < n_all; base += NT * U) {
    float v[U];
    if (base == 0) {
#pragma unroll
      for (int u = 0; u < U; ++u) v[u] = v_first[u];
    } else {
      load_batch(base, v);  // (a second read of a few values, only for lists beyond 2048 entries)
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int p = base + u * NT + tid;
      const double w = (double)__expf(v[u] - m);  // 0 for the slots beyond the list
      acc_f += p < n_fix ? w : 0.0;
      acc_w += p < n_fix ? 0.0 : w;
      acc_w2 += p < n_fix ? 0.0 : w * w;
    }
  }
  double sums[3] = {acc_f, acc_w, acc_w2};
  O::block_sum(sums, sm);
  const double D_f = sums[0];
  double sigma2 = 0.0, b_star = 0.0, D_hat = D_f, tr_sigma = 0.0, nhat_sq = 0.0;
  int bfin = 0;
  if (hs.n_s > 0) {
    const double b0d = (double)hs.b0, ns = (double)hs.n_s;
    double rho_N = 0.0;
    if (A.target != VATT_TARGET_D) {
      // numerator statistics left by the score kernel of the listed tokens, one partial per split, each in
      // units of its own maximum: brought to the head's maximum m (the largest of them) and added
      const int d = A.head_dim;
      const int stride = 2 * d + 4;
      const float* vp = A.given_vstat + (int64_t)bh * A.given_splits * stride;
      double t3[3] = {0.0, 0.0, 0.0};
      if (tid < d) {
        double nf = 0.0, r1 = 0.0;
        for (int s2 = 0; s2 < A.given_splits; ++s2) {
          const float ms = vp[s2 * stride + 2 * d + 1];
          const double f = ms > -INFINITY ? exp((double)ms - (double)m) : 0.0;
          nf += (double)vp[s2 * stride + tid] * f;
          r1 += (double)vp[s2 * stride + d + tid] * f;
        }
        const double nh = nf + ns * r1 / b0d;
        t3[0] = nh * nh;
        t3[1] = r1 * r1;
      }
      if (tid == 0) {
        for (int s2 = 0; s2 < A.given_splits; ++s2) {
          const float ms = vp[s2 * stride + 2 * d + 1];
          const double f = ms > -INFINITY ? exp((double)ms - (double)m) : 0.0;
          t3[2] += (double)vp[s2 * stride + 2 * d] * f * f;
        }
      }
      O::block_sum(t3, sm);
      nhat_sq = t3[0];
      rho_N = numerator_rho(hs.n_s, hs.b0, t3[1], t3[2], nhat_sq, &tr_sigma);
    }
    const Budget bud = algorithm2_budget(A, hs.n_s, hs.b0, D_f, sums[1], sums[2], rho_N, 0.0);
    sigma2 = bud.sigma2;
    b_star = bud.b_star;
    bfin = bud.b;
    D_hat = bud.D_hat;
  }
  int flags = 0;
  if (bfin > 0) {
    Emit E1 = emit_to(idx + A.seg_dyn, (uint32_t)A.b_max);
    if (kFused) {
      E1.global = writer;
      E1.lds = dlist;
      E1.lds_cap = (uint32_t)A.dlist_cap;
      E1.shift = shift;
      E1.split = split;
    }
    const int f = (!kFused && A.nested)
                      ? O::draw_nested(S, hs, (uint32_t)hs.b0, (uint32_t)bfin, bm_f, idx + A.seg_base,
                                       idx + A.seg_dyn, (uint32_t)A.b_max, A.small_batches, sm)
                      : O::draw_sample(S, hs, (uint32_t)bfin, none, false, A.small_batches, E1, nullptr, nullptr, sm);
    flags |= ((f & 1) ? kFlagDynComplement : 0) | ((f & 2) ? kFlagDynBatches : 0) | ((f & 4) ? kFlagDrawCap : 0);
    if (!kFused && A.ascending && !A.nested && !(f & 1))
      O::sort_ascending(idx + A.seg_dyn, (uint32_t)min(bfin, A.b_max), scratch, wpre, n, sm);
  }
  if (tid == 0 && writer) {
    int32_t* c = A.out_counts + (int64_t)bh * 8;
    c[0] = hs.n_sink;
    c[1] = hs.n_win;
    c[2] = k_eff;
    c[3] = hs.b0;
    c[4] = bfin;
    c[5] = hs.n_s;
    c[6] = n;
    c[7] = c[7] | flags;
    if (A.out_budget_raw) A.out_budget_raw[bh] = b_star;
    if (A.out_stats) {
      float* st = A.out_stats + (int64_t)bh * 4;
      st[0] = (float)D_hat;
      st[1] = (float)sigma2;
      st[2] = (float)tr_sigma;
      st[3] = (float)nhat_sq;
      // (in units of exp(-m) with m the largest score among I_f and I_bs, which is HeadRec.m and out_lse's shift)
    }
    HeadRec r;
    r.m = m;
    r.scale = bfin > 0 ? (float)((double)hs.n_s / (double)bfin) : 0.f;
    r.n = n;
    r.n_sink = hs.n_sink;
    r.n_win = hs.n_win;
    r.k = k_eff;
    r.b = bfin;
    r.n_s = hs.n_s;
    r.b_keep = (A.nested && bfin > 0) ? hs.b0 : 0;
    r.base_cached = 0;
    // (with the gather fused in nothing reads the record again, and the head's other workgroups may still be
    // reading the first phase's)
    if (!kFused) A.head_rec[bh] = r;
  }

  if constexpr (kFused) {
    // ---- the gather of this workgroup's share ----
    // LPR adjacent lanes hold one row, NG rows per round, UF rounds in flight; places, tokens, block-table
    // entries and rows each in a loop of their own over the UF slots (no branch per row); a slot beyond a list
    // repeats its last entry and adds nothing.
    constexpr int LPR = FD / 8;
    constexpr int NG = NT / LPR;
    constexpr int UF = 8;
    const int g_sub = tid % LPR, g_grp = tid / LPR;
    const int kvh = h / A.group;
    __syncthreads();  // the final sample's share is complete in dlist
    uint32_t qw[4];
    {
      const uint4 t = *reinterpret_cast<const uint4*>(A.gq + (int64_t)bh * FD + g_sub * 8);
      qw[0] = t.x;
      qw[1] = t.y;
      qw[2] = t.z;
      qw[3] = t.w;
    }
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float dsum = 0.f, m_run = -INFINITY;
    auto add_row = [&](float e, const uint4& vv) {
      if (e > m_run) {
        const float f = __expf(m_run - e);  // 0 when m_run is -inf
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c] *= f;
        dsum *= f;
        m_run = e;
      }
      const float wt = __expf(e - m_run);
      add_weighted_row(acc, wt, vv);
      dsum += wt;
    };
    // I_f: a contiguous run of [sink | window | top-k) per workgroup (the top-k part is in ascending token order)
    const int n_fix2 = hs.n_sink + hs.n_win + k_eff;
    const int run = (n_fix2 + (int)A.splits - 1) >> shift;
    const int f_lo = min((int)split * run, n_fix2), f_hi = min(f_lo + run, n_fix2);
    for (int j0 = f_lo + g_grp; j0 < f_hi; j0 += NG * UF) {
      int64_t place[UF];
      int tok[UF], blk[UF];
      float sc[UF];
      uint4 vv[UF];
#pragma unroll
      for (int u = 0; u < UF; ++u)
        place[u] = fixed_place(min(j0 + u * NG, f_hi - 1), hs.n_sink, hs.n_win, A.seg_sink, A.seg_win, A.seg_topk);
#pragma unroll
      for (int u = 0; u < UF; ++u) {
        tok[u] = min(max(idx[place[u]], 0), n - 1);
        sc[u] = sp[place[u]];
      }
#pragma unroll
      for (int u = 0; u < UF; ++u) blk[u] = kv_block<PAGED>(A.L, seq, tok[u]);
#pragma unroll
      for (int u = 0; u < UF; ++u)
        vv[u] = load_stream_16(A.v + kv_row_offset_in<PAGED>(A.L, seq, kvh, tok[u], blk[u]) + g_sub * 8);
#pragma unroll
      for (int u = 0; u < UF; ++u)
        if (j0 + u * NG < f_hi) add_row(sc[u], vv[u]);
    }
    // the final sample: every A.splits-th token, scores from the K rows, weights carry n_s / b
    int my_nd = bfin > (int)split ? (int)(((uint32_t)bfin - split + ((1u << shift) - 1u)) >> shift) : 0;
    my_nd = min(my_nd, A.dlist_cap);
    const float tail_bias = bfin > 0 ? __logf((float)((double)hs.n_s / (double)bfin)) : 0.f;
    for (int j0 = g_grp; j0 < my_nd; j0 += NG * UF) {
      int tok[UF], blk[UF];
      uint4 kv[UF], vv[UF];
#pragma unroll
      for (int u = 0; u < UF; ++u) tok[u] = (int)min(dlist[min(j0 + u * NG, my_nd - 1)], (uint32_t)(n - 1));
#pragma unroll
      for (int u = 0; u < UF; ++u) blk[u] = kv_block<PAGED>(A.L, seq, tok[u]);  // (K and V share the block table)
#pragma unroll
      for (int u = 0; u < UF; ++u) {
        kv[u] = load_stream_16(A.gk + kv_row_offset_in<PAGED>(A.Lk, seq, kvh, tok[u], blk[u]) + g_sub * 8);
        vv[u] = load_stream_16(A.v + kv_row_offset_in<PAGED>(A.L, seq, kvh, tok[u], blk[u]) + g_sub * 8);
      }
#pragma unroll
      for (int u = 0; u < UF; ++u) {
        // (the lanes of a group stay together: every lane of the group computes the row's score)
        float a = 0.f;
        a = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, kv[u].x), __builtin_bit_cast(bf16x2_t, qw[0]), a, false);
        a = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, kv[u].y), __builtin_bit_cast(bf16x2_t, qw[1]), a, false);
        a = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, kv[u].z), __builtin_bit_cast(bf16x2_t, qw[2]), a, false);
        a = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, kv[u].w), __builtin_bit_cast(bf16x2_t, qw[3]), a, false);
        const float s_row = group_sum<LPR>(a) * A.sm_scale + 0.0f;
        if (j0 + u * NG < my_nd) add_row(s_row + tail_bias, vv[u]);
      }
    }
    // the lane groups of a wave to their common maximum and added, then the waves through LDS
    float M = m_run;
#pragma unroll
    for (int o = LPR; o < kWave; o <<= 1) M = fmaxf(M, __shfl_xor(M, o));
    {
      const float f = m_run > -INFINITY ? __expf(m_run - M) : 0.f;
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[c] *= f;
      dsum *= f;
    }
#pragma unroll
    for (int o = LPR; o < kWave; o <<= 1) {
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[c] += __shfl_xor(acc[c], o);
      dsum += __shfl_xor(dsum, o);
    }
    const int lane = tid & 63, wave = tid >> 6;
    float* g_d = g_red + SW * FD;
    float* g_m = g_d + SW;
    if (lane < LPR) {
#pragma unroll
      for (int c = 0; c < 8; ++c) g_red[wave * FD + lane * 8 + c] = acc[c];
    }
    if (lane == 0) {
      g_d[wave] = dsum;
      g_m[wave] = M;
    }
    __syncthreads();
    float Mall = -INFINITY;
#pragma unroll
    for (int w2 = 0; w2 < SW; ++w2) Mall = fmaxf(Mall, g_m[w2]);
    float* part = A.part + ((int64_t)bh * A.splits + split) * (FD + 4);
    if (tid < FD) {
      float a = 0.f;
#pragma unroll
      for (int w2 = 0; w2 < SW; ++w2) a += g_red[w2 * FD + tid] * (g_m[w2] > -INFINITY ? __expf(g_m[w2] - Mall) : 0.f);
      part[tid] = a;
    }
    if (tid == 0) {
      float dt = 0.f;
#pragma unroll
      for (int w2 = 0; w2 < SW; ++w2) dt += g_d[w2] * (g_m[w2] > -INFINITY ? __expf(g_m[w2] - Mall) : 0.f);
      part[FD] = dt;
      part[FD + 1] = Mall;
    }
  }
}

typedef void (*HeadKernel)(HeadArgs);
// The instantiation for a plan: workgroup size; with the fused gather also head dimension and cache layout.
HeadKernel head_kernel_for(const Plan& pl, bool fused) {
  if (fused) {
    const bool paged = pl.p.kv_layout == VATT_LAYOUT_PAGED;
    if (pl.p.head_dim == 128) return paged ? head_kernel<kHeadThreads, 128, true> : head_kernel<kHeadThreads, 128, false>;
    return paged ? head_kernel<kHeadThreads, 64, true> : head_kernel<kHeadThreads, 64, false>;
  }
  return pl.head_threads == kHeadThreadsLong ? head_kernel<kHeadThreadsLong, 0, false> : head_kernel<kHeadThreads, 0, false>;
}

}  // namespace

size_t head_kernel_static_lds_bytes();

hipError_t set_kernel_attributes(const Plan& pl) {
  // The limit on dynamic LDS belongs to the kernel, not to the plan: it is raised to all a CU has (less the
  // kernels' static part), so that plans of different capacities can be used in any order.
  (void)pl;
  const int cap = 160 * 1024 - (int)head_kernel_static_lds_bytes();
  const void* fused_given[4] = {reinterpret_cast<const void*>(given_topk_kernel<kHeadThreads, 128, false>),
                                reinterpret_cast<const void*>(given_topk_kernel<kHeadThreads, 128, true>),
                                reinterpret_cast<const void*>(given_topk_kernel<kHeadThreads, 64, false>),
                                reinterpret_cast<const void*>(given_topk_kernel<kHeadThreads, 64, true>)};
  for (const void* f : fused_given) {
    const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, cap);
    if (e != hipSuccess) return e;
  }
  const void* kernels[7] = {reinterpret_cast<const void*>(head_kernel<kHeadThreads, 0, false>),
                            reinterpret_cast<const void*>(head_kernel<kHeadThreadsLong, 0, false>),
                            reinterpret_cast<const void*>(head_kernel<kHeadThreads, 128, false>),
                            reinterpret_cast<const void*>(head_kernel<kHeadThreads, 128, true>),
                            reinterpret_cast<const void*>(head_kernel<kHeadThreads, 64, false>),
                            reinterpret_cast<const void*>(head_kernel<kHeadThreads, 64, true>),
                            reinterpret_cast<const void*>(given_topk_kernel<kHeadThreads, 0, false>)};
  for (const void* f : kernels) {
    const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, cap);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

size_t head_kernel_lds_bytes(int n_max, int head_threads) {
  const size_t words_max = ((size_t)(n_max + 63) >> 6) << 1;
  const size_t fixed = head_threads == kHeadThreadsLong ? sizeof(HeadOps<kHeadThreadsLong>::HeadSmem)
                                                        : sizeof(HeadOps<kHeadThreads>::HeadSmem);
  return ((fixed + 15) & ~size_t(15)) + (size_t)kCandCap * (sizeof(uint64_t) + sizeof(uint32_t)) +
         (head_threads == kHeadThreads ? 8 : 6) * words_max * sizeof(uint32_t);
}

// LDS entries of a workgroup's share of I_f and of the final sample when `splits` workgroups share a head.
// (padded to whole calls of the row loader: 8 rounds of NT / (d / 8) rows, 512 entries at d = 64,
// and one call more, since the final sample's list is also walked from a start that is not a multiple of a call)
int fused_glist_cap(const Plan& pl, int splits) { return ((pl.p.sink + pl.p.window + pl.k_max) / splits + 2 + 1023) & ~511; }
int fused_dlist_cap(const Plan& pl, int splits) { return (pl.b_max / splits + 2 + 1023) & ~511; }
// Dynamic LDS of the selection kernel with the fused gather (512 threads).
size_t fused_head_lds_bytes(const Plan& pl, int splits) {
  return head_kernel_lds_bytes(pl.p.n_max, kHeadThreads) +
         ((size_t)fused_glist_cap(pl, splits) + (size_t)fused_dlist_cap(pl, splits)) * (sizeof(uint32_t) + sizeof(float)) +
         (size_t)(kHeadThreads / kWave) * (pl.p.head_dim + 1) * sizeof(float) + 64;
}

size_t head_kernel_static_lds_bytes() { return sizeof(TopkSmem) + 64; }

static void fill_head_args(HeadArgs& A, const Plan& pl, int phase, const int32_t* seq_lens, const uint64_t* seq_seeds,
                           void* ws, int32_t* out_idx, int32_t* out_counts, double* out_budget_raw,
                           float* out_stats);

hipError_t launch_given_select(const Plan& pl, int phase, const int32_t* seq_lens, const uint64_t* seq_seeds,
                               const int32_t* given_idx, const int32_t* given_cnt, const void* rcache, void* ws,
                               int32_t* out_idx, int32_t* out_counts, double* out_budget_raw, float* out_stats,
                               hipStream_t st) {
  HeadArgs A;
  fill_head_args(A, pl, phase, seq_lens, seq_seeds, ws, out_idx, out_counts, out_budget_raw, out_stats);
  A.given_idx = given_idx;
  A.given_cnt = given_cnt;
  A.rcache = rcache;
  A.rc = cache_layout(pl);
  hipLaunchKernelGGL((given_topk_kernel<kHeadThreads, 0, false>), dim3(pl.p.n_q_heads, pl.vbatch), dim3(kHeadThreads),
                     pl.head_lds_bytes, st, A);
  return hipGetLastError();
}

// Dynamic LDS of the selection phases of the caller-supplied-top-k path with scores / gather fused in: the first
// phase keeps its run of I_f and its share of the base sample (tokens and cache slots), the second its share of
// the final sample and the cross-wave sums.
int given_glist_cap(const Plan& pl, int splits) { return (pl.p.sink + pl.p.window + pl.k_max) / splits + 2; }
size_t given_fused_lds_bytes(const Plan& pl, int splits) {
  const size_t dl = (size_t)fused_dlist_cap(pl, splits);
  const size_t first = ((size_t)given_glist_cap(pl, splits) + 2 * dl) * sizeof(uint32_t);
  const size_t second = dl * sizeof(uint32_t) + (size_t)(kHeadThreads / kWave) * (pl.p.head_dim + 2) * sizeof(float);
  return head_kernel_lds_bytes(pl.p.n_max, kHeadThreads) + std::max(first, second);
}

bool given_fused_fits(const Plan& pl, int splits) {
  if (splits < 1 || splits > 16 || (splits & (splits - 1)) != 0) return false;
  if (pl.p.target != VATT_TARGET_D || (pl.p.head_dim != 64 && pl.p.head_dim != 128)) return false;
  return given_fused_lds_bytes(pl, splits) + head_kernel_static_lds_bytes() <= 160 * 1024;
}

// The plan's own choice: as for the scored path, when there are at most half as many heads as compute units.
int given_fused_splits_for(const Plan& pl) {
  const int heads = pl.vbatch * pl.p.n_q_heads;
  if (heads * 2 > pl.num_cus) return 0;
  int s2 = 1;
  while (s2 * 2 * heads <= pl.num_cus && s2 < 16) s2 *= 2;
  while (s2 >= 1 && !given_fused_fits(pl, s2)) s2 /= 2;  // (fewer workgroups per head need longer LDS lists)
  return given_fused_fits(pl, s2) ? s2 : 0;
}

hipError_t launch_given_fused(const Plan& pl, int phase, const void* q, const void* k, const void* v,
                              const int32_t* block_table, const int32_t* seq_lens, const uint64_t* seq_seeds,
                              const int32_t* given_idx, const int32_t* given_cnt, const void* rcache, void* ws,
                              int32_t* out_idx, int32_t* out_counts, double* out_budget_raw, float* out_stats,
                              hipStream_t st) {
  HeadArgs A;
  fill_head_args(A, pl, phase, seq_lens, seq_seeds, ws, out_idx, out_counts, out_budget_raw, out_stats);
  const int S = pl.given_fuse_splits;
  A.given_idx = given_idx;
  A.given_cnt = given_cnt;
  A.rcache = rcache;
  A.rc = cache_layout(pl);
  A.glist_cap = given_glist_cap(pl, S);
  A.v = static_cast<const uint16_t*>(v);
  A.L = pl.kv_v;
  A.L.block_table = block_table;
  A.gq = static_cast<const uint16_t*>(q);
  A.gk = static_cast<const uint16_t*>(k);
  A.Lk = pl.kv_k;
  A.Lk.block_table = block_table;
  A.sm_scale = pl.sm_scale;
  A.part = reinterpret_cast<float*>(static_cast<char*>(ws) + pl.off_gather_part);
  A.splits = S;
  A.split_shift = 0;
  while ((1 << A.split_shift) < S) ++A.split_shift;
  A.dlist_cap = fused_dlist_cap(pl, S);
  const dim3 grid(pl.p.n_q_heads, pl.vbatch, S);
  const size_t lds = given_fused_lds_bytes(pl, S);  // (the larger of the two phases' needs)
  const bool paged = pl.p.kv_layout == VATT_LAYOUT_PAGED;
  if (pl.p.head_dim == 128) {
    if (paged) hipLaunchKernelGGL((given_topk_kernel<kHeadThreads, 128, true>), grid, dim3(kHeadThreads), lds, st, A);
    else hipLaunchKernelGGL((given_topk_kernel<kHeadThreads, 128, false>), grid, dim3(kHeadThreads), lds, st, A);
  } else {
    if (paged) hipLaunchKernelGGL((given_topk_kernel<kHeadThreads, 64, true>), grid, dim3(kHeadThreads), lds, st, A);
    else hipLaunchKernelGGL((given_topk_kernel<kHeadThreads, 64, false>), grid, dim3(kHeadThreads), lds, st, A);
  }
  return hipGetLastError();
}

hipError_t launch_head(const Plan& pl, int phase, const int32_t* seq_lens, const uint64_t* seq_seeds, void* ws,
                       int32_t* out_idx, int32_t* out_counts, double* out_budget_raw, float* out_stats,
                       hipStream_t st) {
  HeadArgs A;
  fill_head_args(A, pl, phase, seq_lens, seq_seeds, ws, out_idx, out_counts, out_budget_raw, out_stats);
  const vatt_params& p = pl.p;
  hipLaunchKernelGGL(head_kernel_for(pl, false), dim3(p.n_q_heads, pl.vbatch), dim3(pl.head_threads), pl.head_lds_bytes, st, A);
  return hipGetLastError();
}

bool fused_splits_fit(const Plan& pl, int splits) {
  if (splits < 1 || splits > 16 || (splits & (splits - 1)) != 0) return false;
  if (pl.head_threads != kHeadThreads || pl.p.target != VATT_TARGET_D) return false;
  return fused_head_lds_bytes(pl, splits) + head_kernel_static_lds_bytes() <= 160 * 1024;
}

// Small batches only: with fewer heads than half the compute units, every head gets the largest power of two
// of workgroups (at most 16) that the chip can run at once, one per compute unit.
int fused_splits_for(const Plan& pl) {
  const int heads = pl.vbatch * pl.p.n_q_heads;
  if (2 * heads > pl.num_cus) return 0;
  int s = 1;
  while (2 * s * heads <= pl.num_cus && s < 16) s *= 2;
  while (s >= 2 && !fused_splits_fit(pl, s)) s /= 2;
  return s >= 2 ? s : 0;
}

// Selection with the fused gather (denominator target, fresh final sample): pl.fuse_splits workgroups per head.
hipError_t launch_head_fused(const Plan& pl, const void* v, const int32_t* block_table, const int32_t* seq_lens,
                             const uint64_t* seq_seeds, void* ws, int32_t* out_idx, int32_t* out_counts,
                             double* out_budget_raw, float* out_stats, bool pre_made, hipStream_t st) {
  HeadArgs A;
  fill_head_args(A, pl, 0, seq_lens, seq_seeds, ws, out_idx, out_counts, out_budget_raw, out_stats);
  const vatt_params& p = pl.p;
  if (pre_made) {  // launch_prework ran for this call
    A.pre_tok = reinterpret_cast<const uint4*>(static_cast<char*>(ws) + pl.off_pre_tok);
    A.pre_flags = reinterpret_cast<const uint32_t*>(static_cast<char*>(ws) + pl.off_pre_flags);
  }
  A.v = static_cast<const uint16_t*>(v);
  A.L = pl.kv_v;
  A.L.block_table = block_table;
  A.part = reinterpret_cast<float*>(static_cast<char*>(ws) + pl.off_gather_part);
  A.splits = pl.fuse_splits;
  A.split_shift = 0;
  while ((1 << A.split_shift) < pl.fuse_splits) ++A.split_shift;
  A.group = pl.group;
  A.glist_cap = fused_glist_cap(pl, pl.fuse_splits);
  A.dlist_cap = fused_dlist_cap(pl, pl.fuse_splits);
  hipLaunchKernelGGL(head_kernel_for(pl, true), dim3(p.n_q_heads, pl.vbatch, pl.fuse_splits), dim3(kHeadThreads),
                     fused_head_lds_bytes(pl, pl.fuse_splits), st, A);
  return hipGetLastError();
}

static void fill_head_args(HeadArgs& A, const Plan& pl, int phase, const int32_t* seq_lens, const uint64_t* seq_seeds,
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

}  // namespace vatt
