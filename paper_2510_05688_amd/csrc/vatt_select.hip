// Index selection and budget: lines 1-8 of Algorithm 1 and all of Algorithm 2, per (sequence, query head).
//
// Every selection here is "the c smallest of a set of distinct 64-bit composites":
//   top-k     composite = (~order_key(score) << 32) | token     (largest score first, ties to the lower token)
//   samples   composite = (philox_key(token) << 32) | token     (smallest key first, ties to the lower token)
// Distinct composites make every selection a pure set operation: the result does not depend on
// the order in which lanes, waves or workgroups contribute, so index sets and budgets are
// reproducible bit for bit.
//
// Two kernels:
//   stage1_kernel  even workgroups: one chunk of a head's score row each; the chunk is kept in registers,
//                  its own top-k is radix-selected and written as candidates (any member of the global top-k
//                  is in its chunk's top-k), plus the chunk maximum.
//                  odd workgroups: Philox keys of one slice of tokens for both sampler streams; tokens whose
//                  key lies under a conservative bound of the threshold that the base sample (stream 0) and
//                  a final sample of up to twice that size (stream 1) will need are appended to per-head
//                  candidate lists.  This is integer work that does not depend on the scores, spread over
//                  the whole chip instead of the one workgroup a head gets in the next kernel.
//   head_kernel    one workgroup per head: merges the top-k candidates into the exact top-k, builds the
//                  membership bitmap, selects the base sample from its candidate list, computes the
//                  statistics and the budget of Algorithm 2, selects the final sample, and writes every
//                  index list in ascending token order.  When a candidate list cannot serve (budget above
//                  the bound, list overflow) the sample is drawn by an exact in-kernel sweep instead.
#include "vatt_internal.h"

namespace vatt {
namespace {

constexpr uint32_t kInv32 = 0xffffffffu;
constexpr uint64_t kInvalid = ~0ull;

// ---------------------------------------------------------------------------
// Workgroup-wide exclusive scan of one uint32 per thread.
// ---------------------------------------------------------------------------
template <int NT>
struct BlockScanSmem {
  uint32_t wave_total[NT / kWave];
};
// Returns the exclusive prefix of v; *total gets the workgroup sum.
template <int NT>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* total, BlockScanSmem<NT>& sm) {
  constexpr int SW = NT / kWave;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t incl = v;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const uint32_t t = __shfl_up(incl, o);
    if (lane >= o) incl += t;
  }
  __syncthreads();  // protects wave_total against a previous use
  if (lane == kWave - 1) sm.wave_total[wave] = incl;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < SW; ++w) {
    const uint32_t t = sm.wave_total[w];
    if (w < wave) base += t;
    tot += t;
  }
  *total = tot;
  return base + incl - v;
}

// ---------------------------------------------------------------------------
// Workgroup select: a threshold T such that the number of valid composites <= T lies in [c, cap]
// (exactly c when cap == c).  Composites sit in registers (hi word, lo word; E per thread; all-ones =
// absent).  Requires 1 <= c <= number of valid composites.
//
// Radix descent with 256 buckets per pass, counted by LDS atomics.  The bucket of an element is its offset
// inside the current value range shifted down so that the range spans at most 256 buckets: the first pass
// starts from the minimum and maximum of the data, so the buckets are spread over the values that actually
// occur (scores of a head's best tokens share sign and exponent; sampler keys under a bound share their
// leading zeros).  The 256 counts are prefix-summed by 256 threads, the bucket that holds the c-th element
// becomes the next range, and once it holds at most 64 elements one wave ranks them directly.
// ---------------------------------------------------------------------------
template <int NT>
struct SelectSmem {
  static constexpr int SMALL = 64;
  uint32_t hist[256];
  uint32_t wave_a[NT / kWave], wave_b[NT / kWave];
  uint32_t sel_bucket, sel_excl, sel_count;
  uint64_t slist[SMALL];
  uint32_t slist_n;
  uint64_t result;
};

template <int NT, int E>
struct BlockSelect {
  static constexpr int SW = NT / kWave;
  static constexpr int SMALL = SelectSmem<NT>::SMALL;
  static_assert(NT >= 256, "the bucket scan uses 256 threads");

  __device__ static uint64_t run(const uint32_t (&xh)[E], const uint32_t (&xl)[E], uint32_t c, uint32_t cap,
                                 SelectSmem<NT>& sm, unsigned long long* dbg = nullptr) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    VATT_STAMP(dbg, 10);
    // range of the high words present
    uint32_t mn = kInv32, mx = 0u;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const bool valid = (xh[e] & xl[e]) != kInv32;
      mn = valid ? min(mn, xh[e]) : mn;
      mx = valid ? max(mx, xh[e]) : mx;
    }
    mn = wave_min_u32(mn);
    mx = wave_max_u32(mx);
    __syncthreads();  // the caller may still be reading a previous result out of this scratch
    if (lane == 0) {
      sm.wave_a[wave] = mn;
      sm.wave_b[wave] = mx;
    }
    if (tid < 256) sm.hist[tid] = 0;
    if (tid < SMALL) sm.slist[tid] = kInvalid;
    if (tid == 0) sm.slist_n = 0;
    __syncthreads();
    uint32_t a_lo = kInv32, a_hi = 0u;
#pragma unroll
    for (int w = 0; w < SW; ++w) {
      a_lo = min(a_lo, sm.wave_a[w]);
      a_hi = max(a_hi, sm.wave_b[w]);
    }
    VATT_STAMP(dbg, 11);
    uint32_t r = c;          // rank wanted inside the current range
    bool low = false;        // false: descending on the high word; true: high word fixed to hv, on the low word
    uint32_t hv = 0u;
    for (int pass = 0; pass < 12; ++pass) {
      const uint32_t span = a_hi - a_lo;
      const int shift = span < 256u ? 0 : (32 - __clz(span)) - 8;
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const bool valid = (xh[e] & xl[e]) != kInv32;
        const uint32_t w = low ? xl[e] : xh[e];
        const bool act = valid && (!low || xh[e] == hv) && w >= a_lo && w <= a_hi;
        if (act) __hip_atomic_fetch_add(&sm.hist[(w - a_lo) >> shift], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      }
      VATT_STAMP(dbg, 20 + 4 * pass);
      __syncthreads();
      // inclusive prefix over the 256 buckets: one bucket per thread of the first four waves
      uint32_t v = 0, incl = 0;
      if (tid < 256) {
        v = sm.hist[tid];
        incl = wave_inclusive_scan_u32(v);
        if (lane == 63) sm.wave_a[wave] = incl;
      }
      __syncthreads();
      if (tid < 256) {
        sm.hist[tid] = 0;  // ready for the next pass
        uint32_t base = 0;
#pragma unroll
        for (int w = 0; w < 3; ++w) base += (w < wave) ? sm.wave_a[w] : 0u;
        incl += base;
        const uint32_t excl = incl - v;
        if (excl < r && r <= incl) {
          sm.sel_bucket = (uint32_t)tid;
          sm.sel_excl = excl;
          sm.sel_count = v;
        }
      }
      __syncthreads();
      VATT_STAMP(dbg, 21 + 4 * pass);
      const uint32_t bsel = sm.sel_bucket, m = sm.sel_count;
      r -= sm.sel_excl;
      a_lo += bsel << shift;
      a_hi = min(a_hi, a_lo + ((1u << shift) - 1u));
      // everything at or below this bucket: (c - r) elements under it plus its own m
      if ((c - r) + m <= cap) return low ? (((uint64_t)hv << 32) | a_hi) : (((uint64_t)a_hi << 32) | kInv32);
      if (m <= (uint32_t)SMALL) {
#pragma unroll
        for (int e = 0; e < E; ++e) {
          const bool valid = (xh[e] & xl[e]) != kInv32;
          const uint32_t w = low ? xl[e] : xh[e];
          if (valid && (!low || xh[e] == hv) && w >= a_lo && w <= a_hi) {
            const uint32_t pos = atomicAdd(&sm.slist_n, 1u);
            if (pos < (uint32_t)SMALL) sm.slist[pos] = ((uint64_t)xh[e] << 32) | xl[e];
          }
        }
        __syncthreads();
        VATT_STAMP(dbg, 90);
        if (tid < SMALL) {
          // rank inside the bucket = number of listed composites below mine (the list is padded with all-ones)
          const uint64_t mine = sm.slist[tid];
          uint32_t below = 0;
#pragma unroll
          for (int j = 0; j < SMALL; ++j) below += (sm.slist[j] < mine) ? 1u : 0u;
          if ((uint32_t)tid < m && below == r - 1u) sm.result = mine;
        }
        __syncthreads();
        VATT_STAMP(dbg, 91);
        return sm.result;
      }
      if (shift == 0 && !low) {
        // one high word left and still too many: continue on the low words of the composites that carry it
        low = true;
        hv = a_lo;
        a_lo = 0u;
        a_hi = 0xfffffffeu;
      }
    }
    return low ? (((uint64_t)hv << 32) | a_hi) : (((uint64_t)a_hi << 32) | kInv32);
  }
};

// ---------------------------------------------------------------------------
// Sampler bounds.  Keys are uniform on [0, 2^32): the c-th smallest of n_s keys sits near c / n_s * 2^32.
// upper_bound_key(c, n_s) is a key value below which at least c residual keys lie except with negligible
// probability (about six standard deviations); every use is verified by counting.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint64_t key_bound(double count, double ns) {
  if (count >= ns) return 4294967296ull;
  if (count <= 0.0) return 0ull;
  return (uint64_t)ceil(count / ns * 4294967296.0);
}
__device__ __forceinline__ uint64_t upper_bound_key(uint32_t c, int n_s) {
  const double ns = (double)n_s, cc = (double)c;
  const double sd = sqrt(cc * (1.0 - fmin(cc / ns, 1.0))) + 1.0;
  return key_bound(cc + 6.0 * sd + 8.0, ns);
}
__device__ __forceinline__ uint64_t lower_bound_key(uint32_t c, int n_s) {
  const double ns = (double)n_s, cc = (double)c;
  const double sd = sqrt(cc * (1.0 - fmin(cc / ns, 1.0))) + 1.0;
  const double lo = cc - 6.0 * sd - 8.0;
  return lo <= 0.0 ? 0ull : (uint64_t)floor(lo / ns * 4294967296.0);
}
// Size of the final sample that the stream-1 candidate list is built to serve.
__device__ __forceinline__ uint32_t stream1_design_count(const HeadSizes& hs) {
  return (uint32_t)min((int64_t)hs.n_s, 2 * (int64_t)hs.b0 + 64);
}

// One Philox block = keys of tokens 4j .. 4j+3.
__device__ __forceinline__ Philox4 token_block_keys(uint32_t j, uint32_t stream, uint32_t head, uint64_t seed) {
  return philox4x32_10(j, stream, head, 0u, (uint32_t)seed, (uint32_t)(seed >> 32));
}

// ---------------------------------------------------------------------------
// Stage 1: chunk top-k candidates (even workgroups) and sampler key candidates (odd workgroups).
// ---------------------------------------------------------------------------
struct Stage1Args {
  const float* scores;
  const int32_t* seq_lens;
  const uint64_t* seq_seeds;
  float* chunk_max;
  uint64_t* cand;
  int32_t* cand_cnt;
  uint64_t* key_list;  // [B*Hq][2][key_stride]
  uint32_t* key_cnt;   // [B*Hq][2], zeroed by the score kernel
  SelectParams sp;
  int n_pad, n_max, Hq, chunk_len, n_chunks, cand_cap, key_cap0, key_cap1, key_slice_len;
  unsigned long long* dbg;
};

constexpr int kKeyStage = 512;  // LDS staging slots per stream in a key workgroup

// Workgroups [0, n_chunks) of a head select chunk candidates; the rest generate sampler key candidates.
template <int NT, int E>
__global__ __launch_bounds__(NT) void stage1_kernel(Stage1Args A) {
  constexpr int ST = NT, SW = NT / kWave;
  __shared__ SelectSmem<NT> sel_sm;
  __shared__ float s_wmax[SW];
  __shared__ uint32_t s_n[2], s_base[2];
  __shared__ uint64_t s_stage[2][kKeyStage];

  const int role = (int)blockIdx.x >= A.n_chunks ? 1 : 0;
  const int chunk = role ? (int)blockIdx.x - A.n_chunks : (int)blockIdx.x;
  const int h = blockIdx.y, b = blockIdx.z;
  const int bh = b * A.Hq + h;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = min(max(A.seq_lens[b], 1), A.n_max);
  const HeadSizes hs = head_sizes(n, A.sp);
  const int span = role ? A.key_slice_len : A.chunk_len;
  const int lo = chunk * span;
  const int hi = min(lo + span, n);

  if (role == 1) {
    // ---- sampler key candidates of tokens [lo, hi) ----
    if (lo >= n || hs.n_s <= 0) return;
    const uint64_t seed = A.seq_seeds[b];
    uint64_t U[2];
    U[0] = A.key_cap0 > 0 ? upper_bound_key((uint32_t)hs.b0, hs.n_s) : 0ull;
    U[1] = A.key_cap1 > 0 ? upper_bound_key(stream1_design_count(hs), hs.n_s) : 0ull;
    if (tid < 2) s_n[tid] = 0;
    __syncthreads();
    const int t_lo = max(lo, hs.mid_lo), t_hi = min(hi, hs.mid_hi);
    for (int j = (t_lo >> 2) + tid; j < ((t_hi + 3) >> 2); j += ST) {
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        if (U[s] == 0ull) continue;
        const Philox4 ph = token_block_keys((uint32_t)j, (uint32_t)s, (uint32_t)h, seed);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = (j << 2) + e;
          if (i >= t_lo && i < t_hi && (uint64_t)ph.v[e] < U[s]) {
            const uint32_t pos = atomicAdd(&s_n[s], 1u);
            if (pos < (uint32_t)kKeyStage) s_stage[s][pos] = ((uint64_t)ph.v[e] << 32) | (uint32_t)i;
          }
        }
      }
    }
    __syncthreads();
    // an overfull stage is reported as an overfull list: the head kernel then draws that sample itself
    if (tid < 2 && s_n[tid] > 0)
      s_base[tid] = atomicAdd(&A.key_cnt[bh * 2 + tid], s_n[tid] > (uint32_t)kKeyStage ? 0x40000000u : s_n[tid]);
    __syncthreads();
    const int key_stride = max(A.key_cap0, A.key_cap1);
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const uint32_t cnt = min(s_n[s], (uint32_t)kKeyStage);
      const uint32_t base = cnt ? s_base[s] : 0u;
      const uint32_t cap = (uint32_t)(s == 0 ? A.key_cap0 : A.key_cap1);
      uint64_t* dst = A.key_list + ((int64_t)bh * 2 + s) * key_stride;
      for (uint32_t t = tid; t < cnt; t += ST)
        if (base + t < cap) dst[base + t] = s_stage[s][t];
    }
    return;
  }

  // ---- top-k candidates of the chunk [lo, hi) ----
  const int slot = bh * A.n_chunks + chunk;
  if (lo >= n) {
    if (tid == 0) {
      A.cand_cnt[slot] = 0;
      A.chunk_max[slot] = -INFINITY;
    }
    return;
  }
  VATT_STAMP(A.dbg, 0);
  const float* row = A.scores + (int64_t)bh * A.n_pad;
  float sc[E];
#pragma unroll
  for (int e = 0; e < E; ++e) sc[e] = row[min(lo + e * ST + tid, n - 1)];
  uint32_t xh[E], xl[E];
  float mx = -INFINITY;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int i = lo + e * ST + tid;
    const bool in_chunk = i < hi;
    const bool in_mid = in_chunk && i >= hs.mid_lo && i < hs.mid_hi;
    mx = in_chunk ? fmaxf(mx, sc[e]) : mx;
    xh[e] = in_mid ? ~float_order_key(sc[e]) : kInv32;
    xl[e] = in_mid ? (uint32_t)i : kInv32;
  }
  VATT_STAMP(A.dbg, 1);
  mx = wave_max(mx);
  if (lane == 0) s_wmax[wave] = mx;
  if (tid == 0) s_n[0] = 0;
  __syncthreads();
  if (tid == 0) {
    float t = s_wmax[0];
    for (int w = 1; w < SW; ++w) t = fmaxf(t, s_wmax[w]);
    A.chunk_max[slot] = t;
  }
  const int vlo = max(lo, hs.mid_lo), vhi = min(hi, hs.mid_hi);
  const int nvalid = max(vhi - vlo, 0);
  const int c = min(min(hs.k, nvalid), A.cand_cap);
  if (c == 0) {
    if (tid == 0) A.cand_cnt[slot] = 0;
    return;
  }
  VATT_STAMP(A.dbg, 2);
  const uint64_t T = (c == nvalid) ? (kInvalid - 1ull)
                                   : BlockSelect<NT, E>::run(xh, xl, (uint32_t)c, (uint32_t)min(nvalid, A.cand_cap),
                                                             sel_sm, A.dbg);
  VATT_STAMP(A.dbg, 3);
  uint64_t* out = A.cand + (int64_t)slot * A.cand_cap;
  uint32_t mine = 0;
#pragma unroll
  for (int e = 0; e < E; ++e) mine |= ((((uint64_t)xh[e] << 32) | xl[e]) <= T ? 1u : 0u) << e;
  if (mine) {
    uint32_t pos = atomicAdd(&s_n[0], (uint32_t)__popc(mine));
#pragma unroll
    for (int e = 0; e < E; ++e) {
      if ((mine >> e) & 1u) {
        if (pos < (uint32_t)A.cand_cap) out[pos] = ((uint64_t)xh[e] << 32) | xl[e];
        ++pos;
      }
    }
  }
  __syncthreads();
  // the select may return a superset of the chunk's top-k (everything down to a bucket boundary)
  if (tid == 0) A.cand_cnt[slot] = (int32_t)min(s_n[0], (uint32_t)A.cand_cap);
  VATT_STAMP(A.dbg, 4);
}

// ---------------------------------------------------------------------------
// Per-head kernel.
// ---------------------------------------------------------------------------
struct HeadArgs {
  const float* scores;
  const int32_t* seq_lens;
  const uint64_t* seq_seeds;
  const float* chunk_max;
  const uint64_t* cand;
  const int32_t* cand_cnt;
  const uint64_t* key_list;
  const uint32_t* key_cnt;
  HeadRec* head_rec;
  const double* vstat_part;  // [B*Hq][vstat_splits][2d+2] (targets N, SDPA)
  int32_t* out_idx;
  int32_t* out_counts;
  double* out_budget_raw;
  float* out_stats;
  SelectParams sp;
  double z_half, z_quarter, eps, cap_frac;
  int64_t seg_topk, seg_base, seg_dyn, seg_sink, seg_win;
  int64_t idx_cap;
  int n_pad, n_max, Hq, n_chunks, cand_cap, key_cap0, key_cap1, target, phase, force_slow, vstat_splits, head_dim;
  int k_max, b0_max, b_max;
  unsigned long long* dbg;
};

// Device functions of the per-head kernel for a workgroup of NT threads.
template <int NT>
struct HeadOps {
static constexpr int ST = NT, SW = NT / kWave;
static constexpr int EL = kListCap / NT;  // in-kernel sampler list composites per thread

struct HeadSmem {
  SelectSmem<NT> sel;
  BlockScanSmem<NT> scan;
  uint64_t list[kListCap];
  uint32_t hist[256];
  double red[3][SW];
  uint32_t list_n, sure_n;
  uint32_t u_a, u_b, u_c;
};

// Workgroup sums of up to three doubles at once; every thread gets all of them.
template <int N>
static __device__ __forceinline__ void block_sum(double (&v)[N], HeadSmem& sm) {
#pragma unroll
  for (int j = 0; j < N; ++j) v[j] = wave_sum(v[j]);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) {
#pragma unroll
    for (int j = 0; j < N; ++j) sm.red[j][threadIdx.x >> 6] = v[j];
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < N; ++j) {
    double t = 0.0;
#pragma unroll
    for (int w = 0; w < SW; ++w) t += sm.red[j][w];
    v[j] = t;
  }
}

// Token read back from an index list, forced into [0, n): a list entry can never address outside the row.
static __device__ __forceinline__ int list_tok(const int32_t* idx, int64_t pos, int n) { return min(max(idx[pos], 0), n - 1); }

// Write the set bits of bm[0, n) as ascending token indices to dst and add exp(s_i - m) (and its square) of
// those tokens into sum_w (sum_w2).  Returns the number of set bits.
static __device__ uint32_t compact_bitmap(const uint32_t* bm, int n, int32_t* dst, uint32_t dst_cap, const float* row, float m,
                                   double* sum_w, double* sum_w2, HeadSmem& sm) {
  const int words = (n + 31) >> 5;
  const int wpt = (words + ST - 1) / ST;
  const int w0 = threadIdx.x * wpt;
  uint32_t cnt = 0;
  for (int w = w0; w < min(w0 + wpt, words); ++w) cnt += __popc(bm[w]);
  uint32_t total;
  uint32_t pos = block_exclusive_scan<NT>(cnt, &total, sm.scan);
  double a = 0.0, a2 = 0.0;
  for (int w = w0; w < min(w0 + wpt, words); ++w) {
    uint32_t bits = bm[w];
    while (bits) {
      const int bpos = __ffs(bits) - 1;
      bits &= bits - 1u;
      const int i = (w << 5) + bpos;
      if (pos < dst_cap) dst[pos] = i;
      ++pos;
      if (sum_w) {
        const double wgt = (double)expf(row[i] - m);
        a += wgt;
        a2 += wgt * wgt;
      }
    }
  }
  if (sum_w) *sum_w += a;
  if (sum_w2) *sum_w2 += a2;
  return total;
}

// Residual tokens of the 4-token block j as a 4-bit mask.
static __device__ __forceinline__ uint32_t residual_nibble(const uint32_t* bm_f, const HeadSizes& hs, int j) {
  const int i0 = j << 2;
  uint32_t in_mid = 0;
#pragma unroll
  for (int e = 0; e < 4; ++e) in_mid |= ((i0 + e >= hs.mid_lo && i0 + e < hs.mid_hi) ? 1u : 0u) << e;
  const uint32_t taken = (bm_f[i0 >> 5] >> (i0 & 31)) & 15u;
  return in_mid & ~taken;
}

static __device__ __forceinline__ void mark_bit(uint32_t* bm, uint32_t i) { atomicOr(&bm[i >> 5], 1u << (i & 31)); }

// Select the `need` smallest composites of the LDS list sm.list[0, listed) and mark their tokens in bm_s.
static __device__ void mark_smallest_of_list(uint32_t* bm_s, uint32_t listed, uint32_t need, HeadSmem& sm) {
  uint32_t xh[EL], xl[EL];
#pragma unroll
  for (int e = 0; e < EL; ++e) {
    const uint32_t p = e * ST + threadIdx.x;
    const uint64_t t = p < listed ? sm.list[p] : kInvalid;
    xh[e] = (uint32_t)(t >> 32);
    xl[e] = (uint32_t)t;
  }
  const uint64_t T = (need >= listed) ? (kInvalid - 1ull) : BlockSelect<NT, EL>::run(xh, xl, need, need, sm.sel);
#pragma unroll
  for (int e = 0; e < EL; ++e)
    if ((((uint64_t)xh[e] << 32) | xl[e]) <= T) mark_bit(bm_s, xl[e]);
}

// Fast sample: from the candidate list that stage 1 built for this head and stream (every middle token
// whose key is under the design bound).  Usable when the list did not overflow and holds at least c
// residual tokens; then the c smallest residual composites in it are the sample.  bm_s must be zero.
template <int EK>
static __device__ bool sample_from_candidates(uint32_t* bm_s, const uint32_t* bm_f, const HeadSizes& hs, uint32_t c,
                                       const uint64_t* list, uint32_t count, uint32_t cap, HeadSmem& sm) {
  if (cap == 0 || count > cap) return false;
  uint32_t xh[EK], xl[EK];
  uint32_t valid = 0;
#pragma unroll
  for (int e = 0; e < EK; ++e) {
    const uint32_t p = e * ST + threadIdx.x;
    xh[e] = xl[e] = kInv32;
    if (p < count) {
      const uint64_t t = list[p];
      const uint32_t i = (uint32_t)t;
      const bool res = (int)i >= hs.mid_lo && (int)i < hs.mid_hi && !((bm_f[i >> 5] >> (i & 31)) & 1u);
      if (res) {
        xh[e] = (uint32_t)(t >> 32);
        xl[e] = i;
        ++valid;
      }
    }
  }
  valid = wave_sum_u32(valid);
  __syncthreads();
  if (threadIdx.x == 0) sm.u_a = 0;
  __syncthreads();
  if ((threadIdx.x & 63) == 0 && valid) atomicAdd(&sm.u_a, valid);
  __syncthreads();
  const uint32_t total = sm.u_a;
  if (total < c) return false;
  const uint64_t T = (total == c) ? (kInvalid - 1ull) : BlockSelect<NT, EK>::run(xh, xl, c, c, sm.sel);
#pragma unroll
  for (int e = 0; e < EK; ++e)
    if ((((uint64_t)xh[e] << 32) | xl[e]) <= T) mark_bit(bm_s, xl[e]);
  __syncthreads();
  return true;
}

// General sample: mark in bm_s the c residual tokens with the smallest (key, token) of the given stream,
// computing the keys here.  bm_s must be all zero on entry.  Returns 1 if the slow exact descent was needed.
static __device__ int sample_by_sweep(uint32_t* bm_s, const uint32_t* bm_f, const HeadSizes& hs, uint32_t c,
                               uint32_t stream, uint32_t head, uint64_t seed, int force_slow, HeadSmem& sm) {
  const int tid = threadIdx.x;
  const int j_lo = hs.mid_lo >> 2, j_hi = (hs.mid_hi + 3) >> 2;  // Philox blocks that touch the middle region
  const int words = (hs.n + 31) >> 5;
  if (c == 0) return 0;
  if (c >= (uint32_t)hs.n_s) {
    // the whole residual: no keys needed
    for (int w = tid; w < words; w += ST) {
      uint32_t m = 0;
      const int i0 = w << 5;
      if (i0 + 31 >= hs.mid_lo && i0 < hs.mid_hi) {
        const int a = max(hs.mid_lo - i0, 0), bnd = min(hs.mid_hi - i0, 32);
        m = (bnd >= 32 ? 0xffffffffu : ((1u << bnd) - 1u)) & ~((1u << a) - 1u);
      }
      bm_s[w] = m & ~bm_f[w];
    }
    __syncthreads();
    return 0;
  }

  bool done = false;
  if (!force_slow) {
    // One sweep with a verified guess: tokens with a key below L are certainly in, tokens in [L, U) are
    // listed and ranked exactly; the guess is checked by counting and otherwise discarded.
    const uint64_t Lq = lower_bound_key(c, hs.n_s), Uq = upper_bound_key(c, hs.n_s);
    if (tid == 0) {
      sm.list_n = 0;
      sm.sure_n = 0;
    }
    __syncthreads();
    uint32_t my_sure = 0;
    for (int j = j_lo + tid; j < j_hi; j += ST) {
      const uint32_t res = residual_nibble(bm_f, hs, j);
      if (res) {
        const Philox4 ph = token_block_keys((uint32_t)j, stream, head, seed);
        uint32_t mark = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if ((res >> e) & 1u) {
            const uint64_t key = ph.v[e];
            if (key < Lq) {
              mark |= 1u << e;
            } else if (key < Uq) {
              const uint32_t pos = atomicAdd(&sm.list_n, 1u);
              if (pos < (uint32_t)kListCap) sm.list[pos] = (key << 32) | (uint32_t)((j << 2) + e);
            }
          }
        }
        if (mark) {
          atomicOr(&bm_s[(j << 2) >> 5], mark << ((j << 2) & 31));
          my_sure += __popc(mark);
        }
      }
    }
    if (my_sure) atomicAdd(&sm.sure_n, my_sure);
    __syncthreads();
    const uint32_t sure = sm.sure_n, listed = sm.list_n;
    if (sure <= c && sure + listed >= c && listed <= (uint32_t)kListCap) {
      if (c > sure) mark_smallest_of_list(bm_s, listed, c - sure, sm);
      done = true;
    } else {
      for (int w = tid; w < words; w += ST) bm_s[w] = 0;  // discard the guess
    }
    __syncthreads();
  }
  if (done) return 0;

  // Slow exact path: radix descent over the composite with 8-bit digits, recomputing the keys in every
  // sweep; ends with one marking sweep.  Correct for any c and any key distribution.
  uint64_t prefix = 0, mask = 0, T = 0;
  uint32_t r = c;
  bool have_T = false;
  for (int shift = 56; shift >= 0 && !have_T; shift -= 8) {
    for (int d = tid; d < 256; d += ST) sm.hist[d] = 0;
    __syncthreads();
    for (int j = j_lo + tid; j < j_hi; j += ST) {
      const uint32_t res = residual_nibble(bm_f, hs, j);
      if (res) {
        const Philox4 ph = token_block_keys((uint32_t)j, stream, head, seed);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if ((res >> e) & 1u) {
            const uint64_t comp = ((uint64_t)ph.v[e] << 32) | (uint32_t)((j << 2) + e);
            if ((comp & mask) == prefix) atomicAdd(&sm.hist[(uint32_t)(comp >> shift) & 255u], 1u);
          }
        }
      }
    }
    __syncthreads();
    if (tid == 0) {
      uint32_t cum = 0, below = 0, active = 0, dsel = 255;
      bool found = false;
      for (int d = 0; d < 256; ++d) {
        const uint32_t t = sm.hist[d];
        if (!found && cum + t >= r) {
          found = true;
          dsel = d;
          below = cum;
          active = t;
        }
        cum += t;
      }
      sm.u_a = dsel;
      sm.u_b = below;
      sm.u_c = active;
    }
    __syncthreads();
    const uint32_t dsel = sm.u_a, below = sm.u_b, active = sm.u_c;
    r -= below;
    prefix |= (uint64_t)dsel << shift;
    mask |= 255ull << shift;
    if (active == r) {
      T = prefix | ((1ull << shift) - 1ull);
      have_T = true;
    } else if (active <= (uint32_t)kListCap) {
      if (tid == 0) sm.list_n = 0;
      __syncthreads();
      for (int j = j_lo + tid; j < j_hi; j += ST) {
        const uint32_t res = residual_nibble(bm_f, hs, j);
        if (res) {
          const Philox4 ph = token_block_keys((uint32_t)j, stream, head, seed);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            if ((res >> e) & 1u) {
              const uint64_t comp = ((uint64_t)ph.v[e] << 32) | (uint32_t)((j << 2) + e);
              if ((comp & mask) == prefix) {
                const uint32_t pos = atomicAdd(&sm.list_n, 1u);
                if (pos < (uint32_t)kListCap) sm.list[pos] = comp;
              }
            }
          }
        }
      }
      __syncthreads();
      const uint32_t listed = min(sm.list_n, (uint32_t)kListCap);
      uint32_t xh[EL], xl[EL];
#pragma unroll
      for (int e = 0; e < EL; ++e) {
        const uint32_t p = e * ST + tid;
        const uint64_t t = p < listed ? sm.list[p] : kInvalid;
        xh[e] = (uint32_t)(t >> 32);
        xl[e] = (uint32_t)t;
      }
      T = BlockSelect<NT, EL>::run(xh, xl, r, r, sm.sel);
      have_T = true;
    }
    __syncthreads();
  }
  if (!have_T) T = prefix;
  for (int j = j_lo + tid; j < j_hi; j += ST) {
    const uint32_t res = residual_nibble(bm_f, hs, j);
    if (res) {
      const Philox4 ph = token_block_keys((uint32_t)j, stream, head, seed);
      uint32_t mark = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if ((res >> e) & 1u) {
          const uint64_t comp = ((uint64_t)ph.v[e] << 32) | (uint32_t)((j << 2) + e);
          if (comp <= T) mark |= 1u << e;
        }
      }
      if (mark) atomicOr(&bm_s[(j << 2) >> 5], mark << ((j << 2) & 31));
    }
  }
  __syncthreads();
  return 1;
}

// Picks the candidate-list width for the list's capacity (a short list keeps the select cheap).
static __device__ __forceinline__ bool sample_from_list(uint32_t* bm_s, const uint32_t* bm_f, const HeadSizes& hs,
                                                        uint32_t c, const uint64_t* list, uint32_t count, uint32_t cap,
                                                        HeadSmem& sm) {
  if (cap <= 2048u) return sample_from_candidates<2048 / NT>(bm_s, bm_f, hs, c, list, count, cap, sm);
  return sample_from_candidates<kKeyListMax / NT>(bm_s, bm_f, hs, c, list, count, cap, sm);
}
};  // struct HeadOps

// NT = workgroup size; EM = top-k candidates a thread holds while merging (a head has <= EM * NT of them).
template <int NT, int EM>
__global__ __launch_bounds__(NT) void head_kernel(HeadArgs A) {
  using O = HeadOps<NT>;
  using HeadSmem = typename O::HeadSmem;
  constexpr int ST = NT, SW = NT / kWave;
  extern __shared__ __align__(16) unsigned char dyn_smem[];
  const int h = blockIdx.x, b = blockIdx.y;
  const int bh = b * A.Hq + h;
  const int tid = threadIdx.x;
  const int n = min(max(A.seq_lens[b], 1), A.n_max);
  const HeadSizes hs = head_sizes(n, A.sp);
  const int words_max = (A.n_max + 31) >> 5;
  const int words = (n + 31) >> 5;

  HeadSmem& sm = *reinterpret_cast<HeadSmem*>(dyn_smem);
  uint32_t* bm_f = reinterpret_cast<uint32_t*>(dyn_smem + ((sizeof(HeadSmem) + 15) & ~size_t(15)));
  uint32_t* bm_s = bm_f + words_max;

  const float* row = A.scores + (int64_t)bh * A.n_pad;
  int32_t* idx = A.out_idx + (int64_t)bh * A.idx_cap;
  const uint64_t seed = A.seq_seeds[b];
  const int key_stride = max(A.key_cap0, A.key_cap1);

  VATT_STAMP(A.dbg, 0);
  for (int w = tid; w < words; w += ST) {
    bm_f[w] = 0;
    bm_s[w] = 0;
  }
  // head maximum from the chunk maxima
  float m = -INFINITY;
  for (int c = tid; c < A.n_chunks; c += ST) m = fmaxf(m, A.chunk_max[bh * A.n_chunks + c]);
  m = wave_max(m);
  __syncthreads();
  if ((tid & 63) == 0) sm.red[0][tid >> 6] = (double)m;
  __syncthreads();
  m = (float)sm.red[0][0];
#pragma unroll
  for (int w = 1; w < SW; ++w) m = fmaxf(m, (float)sm.red[0][w]);
  __syncthreads();

  VATT_STAMP(A.dbg, 1);
  double acc_f = 0.0;  // this thread's share of D_f = sum over I_f of exp(s_i - m)
  // ---- I_t (Algorithm 1, line 3) ----
  if (A.phase != 2) {
    if (hs.k > 0) {
      uint32_t xh[EM], xl[EM];
      uint32_t total = 0;
      for (int c = 0; c < A.n_chunks; ++c) total += (uint32_t)A.cand_cnt[bh * A.n_chunks + c];
#pragma unroll
      for (int e = 0; e < EM; ++e) xh[e] = xl[e] = kInv32;
      {
        // flat candidate position p = e * ST + tid; chunk c holds positions [base, base + cnt)
        uint32_t base = 0;
        for (int c = 0; c < A.n_chunks; ++c) {
          const uint32_t cnt = (uint32_t)A.cand_cnt[bh * A.n_chunks + c];
          const uint64_t* src = A.cand + ((int64_t)bh * A.n_chunks + c) * A.cand_cap;
#pragma unroll
          for (int e = 0; e < EM; ++e) {
            const uint32_t p = (uint32_t)e * ST + tid;
            if (p >= base && p < base + cnt) {
              const uint64_t t = src[p - base];
              xh[e] = (uint32_t)(t >> 32);
              xl[e] = (uint32_t)t;
            }
          }
          base += cnt;
        }
      }
      VATT_STAMP(A.dbg, 2);
      const uint64_t T =
          ((uint32_t)hs.k >= total) ? (kInvalid - 1ull) : BlockSelect<NT, EM>::run(xh, xl, (uint32_t)hs.k, (uint32_t)hs.k, sm.sel, A.dbg ? A.dbg + 100 : nullptr);
      VATT_STAMP(A.dbg, 3);
#pragma unroll
      for (int e = 0; e < EM; ++e)
        if ((((uint64_t)xh[e] << 32) | xl[e]) <= T) O::mark_bit(bm_f, xl[e]);
      __syncthreads();
      O::compact_bitmap(bm_f, n, idx + A.seg_topk, (uint32_t)A.k_max, row, m, &acc_f, nullptr, sm);
      VATT_STAMP(A.dbg, 4);
    }
    for (int i = tid; i < hs.n_sink; i += ST) idx[A.seg_sink + i] = i;
    for (int i = tid; i < hs.n_win; i += ST) idx[A.seg_win + i] = hs.mid_hi + i;
  } else {
    // phase 2: rebuild the top-k bitmap from the list written in phase 1
    for (int t = tid; t < hs.k; t += ST) {
      const int i = O::list_tok(idx, A.seg_topk + t, n);
      O::mark_bit(bm_f, (uint32_t)i);
      acc_f += (double)expf(row[i] - m);
    }
  }
  for (int i = tid; i < hs.n_sink; i += ST) acc_f += (double)expf(row[i] - m);
  for (int i = tid; i < hs.n_win; i += ST) acc_f += (double)expf(row[hs.mid_hi + i] - m);
  __syncthreads();

  // ---- I_bs (Algorithm 2, line 1) and the sums over it ----
  int flags = 0;
  double acc_w = 0.0, acc_w2 = 0.0;
  if (hs.n_s > 0) {
    if (A.phase != 2) {
      bool ok = false;
      if (!A.force_slow)
        ok = O::sample_from_list(bm_s, bm_f, hs, (uint32_t)hs.b0, A.key_list + ((int64_t)bh * 2 + 0) * key_stride,
                                    A.key_cnt[bh * 2 + 0], (uint32_t)A.key_cap0, sm);
      if (!ok) {
        __syncthreads();
        for (int w = tid; w < words; w += ST) bm_s[w] = 0;
        __syncthreads();
        flags |= 2 | (O::sample_by_sweep(bm_s, bm_f, hs, (uint32_t)hs.b0, 0u, (uint32_t)h, seed, A.force_slow, sm) << 2);
      }
      VATT_STAMP(A.dbg, 5);
      O::compact_bitmap(bm_s, n, idx + A.seg_base, (uint32_t)A.b0_max, row, m, &acc_w, &acc_w2, sm);
      VATT_STAMP(A.dbg, 6);
      __syncthreads();
      for (int w = tid; w < words; w += ST) bm_s[w] = 0;
      __syncthreads();
    } else {
      for (int t = tid; t < hs.b0; t += ST) {
        const double wgt = (double)expf(row[O::list_tok(idx, A.seg_base + t, n)] - m);
        acc_w += wgt;
        acc_w2 += wgt * wgt;
      }
    }
  }
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
      A.head_rec[bh] = r;
      A.out_counts[(int64_t)bh * 8 + 7] = flags;
    }
    return;
  }

  // ---- statistics (Algorithm 2, get-stats): w_i = exp(s_i - m) ----
  double sums[3] = {acc_f, acc_w, acc_w2};
  O::block_sum(sums, sm);
  const double D_f = sums[0];
  double sigma2 = 0.0, b_star = 0.0, tr_sigma = 0.0, nhat_sq = 0.0;
  int bfin = 0;
  if (hs.n_s > 0) {
    const double b0d = (double)hs.b0;
    const double w_bar = sums[1] / b0d;
    // unbiased variance from the two sums; the scores are shifted so that the largest weight is 1
    sigma2 = hs.b0 > 1 ? fmax(sums[2] - sums[1] * w_bar, 0.0) / (b0d - 1.0) : 0.0;
    const double ns = (double)hs.n_s;
    const double D_hat = D_f + ns * w_bar;
    const double rho_D = ns * sqrt(sigma2) / D_hat;
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
      tr_sigma = hs.b0 > 1 ? fmax(t3[2] - t3[1] / b0d, 0.0) / (b0d - 1.0) : 0.0;
      const double num = ns * sqrt(tr_sigma), nn = sqrt(nhat_sq);
      rho_N = nn > 0.0 ? num / nn : (num > 0.0 ? INFINITY : 0.0);
    }
    if (A.target == VATT_TARGET_D) {
      const double t = A.z_half * rho_D / A.eps;
      b_star = t * t;
    } else if (A.target == VATT_TARGET_N) {
      const double t = A.z_half * rho_N / A.eps;
      b_star = t * t;
    } else {
      const double t = 2.0 * A.z_quarter * (rho_D + rho_N) / A.eps;
      b_star = t * t;
    }
    // b = min(n_s, max(b0, min(ceil(b*), ceil(cap * n_s))))
    const int cap = (int)ceil(A.cap_frac * ns);
    int want = hs.n_s;
    if (b_star == b_star && b_star < ns) want = (int)ceil(b_star);
    bfin = min(hs.n_s, max(hs.b0, min(want, cap)));
    bfin = min(bfin, A.b_max);
    if (tid == 0 && A.out_stats) {
      float* st = A.out_stats + (int64_t)bh * 4;
      st[0] = (float)D_hat;
      st[1] = (float)sigma2;
      st[2] = (float)tr_sigma;
      st[3] = (float)nhat_sq;
    }
  } else if (tid == 0 && A.out_stats) {
    float* st = A.out_stats + (int64_t)bh * 4;
    st[0] = (float)D_f;
    st[1] = st[2] = st[3] = 0.f;
  }

  VATT_STAMP(A.dbg, 7);
  // ---- I_dyn (Algorithm 1, line 7) ----
  if (bfin > 0) {
    bool ok = false;
    if (!A.force_slow && (uint32_t)bfin < (uint32_t)hs.n_s)
      ok = O::sample_from_list(bm_s, bm_f, hs, (uint32_t)bfin, A.key_list + ((int64_t)bh * 2 + 1) * key_stride,
                                  A.key_cnt[bh * 2 + 1], (uint32_t)A.key_cap1, sm);
    if (!ok) {
      __syncthreads();
      for (int w = tid; w < words; w += ST) bm_s[w] = 0;
      __syncthreads();
      const int slow = O::sample_by_sweep(bm_s, bm_f, hs, (uint32_t)bfin, 1u, (uint32_t)h, seed, A.force_slow, sm);
      flags |= ((uint32_t)bfin < (uint32_t)hs.n_s ? 8 : 0) | slow;
    }
    VATT_STAMP(A.dbg, 8);
    O::compact_bitmap(bm_s, n, idx + A.seg_dyn, (uint32_t)A.b_max, nullptr, 0.f, nullptr, nullptr, sm);
    VATT_STAMP(A.dbg, 9);
  }
  if (tid == 0) {
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
    A.head_rec[bh] = r;
  }
}

}  // namespace

hipError_t set_kernel_attributes(const Plan& pl) {
  const void* fns[3] = {reinterpret_cast<const void*>(head_kernel<256, 16>),
                        reinterpret_cast<const void*>(head_kernel<256, 32>),
                        reinterpret_cast<const void*>(head_kernel<1024, 32>)};
  for (const void* f : fns) {
    hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)pl.head_lds_bytes);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

size_t head_kernel_lds_bytes(int n_max, int head_threads) {
  const size_t words_max = (size_t)(n_max + 31) >> 5;
  const size_t fixed = head_threads == 256 ? sizeof(HeadOps<256>::HeadSmem) : sizeof(HeadOps<1024>::HeadSmem);
  return ((fixed + 15) & ~size_t(15)) + 2 * words_max * sizeof(uint32_t);
}

hipError_t launch_stage1(const Plan& pl, const int32_t* seq_lens, const uint64_t* seq_seeds, void* ws,
                         hipStream_t st) {
  const vatt_params& p = pl.p;
  char* w = static_cast<char*>(ws);
  Stage1Args A;
  A.scores = reinterpret_cast<const float*>(w + pl.off_scores);
  A.seq_lens = seq_lens;
  A.seq_seeds = seq_seeds;
  A.chunk_max = reinterpret_cast<float*>(w + pl.off_chunk_max);
  A.cand = reinterpret_cast<uint64_t*>(w + pl.off_cand);
  A.cand_cnt = reinterpret_cast<int32_t*>(w + pl.off_cand_cnt);
  A.key_list = reinterpret_cast<uint64_t*>(w + pl.off_key_list);
  A.key_cnt = reinterpret_cast<uint32_t*>(w + pl.off_key_cnt);
  A.sp = pl.sel;
  A.n_pad = pl.n_pad;
  A.n_max = p.n_max;
  A.Hq = p.n_q_heads;
  A.chunk_len = pl.chunk_len;
  A.n_chunks = pl.n_chunks;
  A.cand_cap = pl.cand_cap;
  A.key_cap0 = pl.key_cap[0];
  A.key_cap1 = pl.key_cap[1];
  A.dbg = reinterpret_cast<unsigned long long*>(w + pl.off_debug);
  A.key_slice_len = pl.key_slice_len;
  dim3 grid(pl.n_chunks + pl.n_key_slices, p.n_q_heads, p.batch);
  if (pl.stage_threads == 256)
    hipLaunchKernelGGL((stage1_kernel<256, kChunkElems>), grid, dim3(256), 0, st, A);
  else
    hipLaunchKernelGGL((stage1_kernel<1024, kChunkElems>), grid, dim3(1024), 0, st, A);
  return hipGetLastError();
}

hipError_t launch_head(const Plan& pl, int phase, const int32_t* seq_lens, const uint64_t* seq_seeds, void* ws,
                       int32_t* out_idx, int32_t* out_counts, double* out_budget_raw, float* out_stats,
                       hipStream_t st) {
  const vatt_params& p = pl.p;
  char* w = static_cast<char*>(ws);
  HeadArgs A;
  A.scores = reinterpret_cast<const float*>(w + pl.off_scores);
  A.seq_lens = seq_lens;
  A.seq_seeds = seq_seeds;
  A.chunk_max = reinterpret_cast<const float*>(w + pl.off_chunk_max);
  A.cand = reinterpret_cast<const uint64_t*>(w + pl.off_cand);
  A.cand_cnt = reinterpret_cast<const int32_t*>(w + pl.off_cand_cnt);
  A.key_list = reinterpret_cast<const uint64_t*>(w + pl.off_key_list);
  A.key_cnt = reinterpret_cast<const uint32_t*>(w + pl.off_key_cnt);
  A.head_rec = reinterpret_cast<HeadRec*>(w + pl.off_head_rec);
  A.vstat_part = reinterpret_cast<const double*>(w + pl.off_vstat_part);
  A.out_idx = out_idx;
  A.out_counts = out_counts;
  A.out_budget_raw = out_budget_raw;
  A.out_stats = out_stats;
  A.sp = pl.sel;
  A.z_half = pl.z_half;
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
  A.n_chunks = pl.n_chunks;
  A.cand_cap = pl.cand_cap;
  A.key_cap0 = pl.key_cap[0];
  A.key_cap1 = pl.key_cap[1];
  A.target = p.target;
  A.phase = phase;
  A.force_slow = pl.force_slow_sampler;
  A.vstat_splits = pl.vstat_splits;
  A.head_dim = p.head_dim;
  A.k_max = pl.k_max;
  A.b0_max = pl.b0_max;
  A.b_max = pl.b_max;
  A.dbg = reinterpret_cast<unsigned long long*>(w + pl.off_debug) + 64;
  const int64_t cands = (int64_t)pl.n_chunks * pl.cand_cap;
  const dim3 grid(p.n_q_heads, p.batch);
  if (pl.head_threads == 256 && cands <= 16 * 256)
    hipLaunchKernelGGL((head_kernel<256, 16>), grid, dim3(256), pl.head_lds_bytes, st, A);
  else if (pl.head_threads == 256)
    hipLaunchKernelGGL((head_kernel<256, 32>), grid, dim3(256), pl.head_lds_bytes, st, A);
  else
    hipLaunchKernelGGL((head_kernel<1024, 32>), grid, dim3(1024), pl.head_lds_bytes, st, A);
  return hipGetLastError();
}

}  // namespace vatt
