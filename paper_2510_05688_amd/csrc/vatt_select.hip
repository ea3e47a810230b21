// Index selection and budget: lines 1-8 of Algorithm 1 and all of Algorithm 2, per (sequence, query head).
//
// Every selection here is "the c smallest of a set of distinct 64-bit composites":
//   top-k     composite = (~order_key(score) << 32) | token     (largest score first, ties to the lower token)
//   samples   composite = (philox_key(token) << 32) | token     (smallest key first, ties to the lower token)
// Distinct composites make every selection a pure set operation: the result does not depend on
// the order in which lanes, waves or workgroups contribute, so index sets and budgets are
// reproducible bit for bit.  Floating-point sums are taken in ascending token order with a fixed
// tree, so the statistics are reproducible too.
//
// Two kernels:
//   stage1_kernel  workgroups [0, n_chunks) of a head: one chunk of the head's score row each; the chunk is
//                  kept in registers, a threshold that keeps at least its own top-k is found by counting,
//                  and the composites under it are written as candidates (any member of the global top-k is
//                  in its chunk's top-k), plus the chunk maximum.
//                  Remaining workgroups: Philox keys of one slice of tokens for both sampler streams; tokens
//                  whose key lies under a conservative bound of the threshold that the base sample
//                  (stream 0) and a final sample of up to twice that size (stream 1) will need are written,
//                  with their scores, as sampler candidates.  This is integer work that does not depend on
//                  the scores, spread over the whole chip instead of the one workgroup a head gets next.
//   head_kernel    one workgroup per head: selects the exact top-k among the chunk candidates, builds the
//                  membership bitmap, selects the base sample among its candidates, computes the
//                  statistics and the budget of Algorithm 2, selects the final sample, and writes every
//                  index list in ascending token order.  When a candidate list cannot serve (budget above
//                  the bound it was built for, or an overfull slice) the sample is drawn by an exact
//                  in-kernel sweep instead.
#include "vatt_internal.h"

namespace vatt {
namespace {

constexpr uint32_t kInv32 = 0xffffffffu;
constexpr uint64_t kInvalid = ~0ull;
constexpr uint32_t kOverflow = 0xffffffffu;  // slice count that marks an overfull sampler candidate slice

// ---------------------------------------------------------------------------
// Workgroup-wide exclusive scan of one uint32 per thread (DPP inside a wave, LDS across waves).
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
  const uint32_t incl = wave_inclusive_scan_u32(v);
  __syncthreads();  // protects wave_total against a previous use
  if (lane == kWave - 1) sm.wave_total[wave] = incl;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < SW; ++w) {
    const uint32_t t = sm.wave_total[w];
    base += (w < wave) ? t : 0u;
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
// Search on the value of the high word by counting: the range [lo, hi] that holds the c-th composite
// starts as the minimum and maximum present; each step counts the composites in [lo, pivot] (a compare
// per element, a DPP wave sum, one LDS add per wave, one barrier) and keeps the half that holds the
// target.  Pivots alternate between interpolation (fast when the values are spread evenly, as sampler
// keys are) and the midpoint (which bounds the number of steps whatever the data).  When at most SMALL
// composites remain they are ranked directly by one wave.  Equal high words are resolved the same way on
// the low word.
// ---------------------------------------------------------------------------
constexpr int kSelectSteps = 160;

template <int NT>
struct SelectSmem {
  static constexpr int SMALL = 64;
  uint32_t cnt[kSelectSteps];
  uint32_t wave_a[NT / kWave], wave_b[NT / kWave], wave_c[NT / kWave];
  uint64_t slist[SMALL];
  uint32_t slist_n;
  uint64_t result;
};

template <int NT, int E>
struct BlockSelect {
  static constexpr int SW = NT / kWave;
  static constexpr int SMALL = SelectSmem<NT>::SMALL;

  __device__ static uint64_t run(const uint32_t (&xh)[E], const uint32_t (&xl)[E], uint32_t c, uint32_t cap,
                                 SelectSmem<NT>& sm, unsigned long long* dbg = nullptr) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    VATT_STAMP(dbg, 10);
    // range of the high words present, and how many composites there are
    uint32_t mn = kInv32, mx = 0u, nv = 0u;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const bool valid = (xh[e] & xl[e]) != kInv32;
      mn = valid ? min(mn, xh[e]) : mn;
      mx = valid ? max(mx, xh[e]) : mx;
      nv += valid ? 1u : 0u;
    }
    mn = wave_min_u32(mn);
    mx = wave_max_u32(mx);
    nv = wave_sum_u32(nv);
    __syncthreads();  // the caller may still be reading a previous result out of this scratch
    if (lane == 0) {
      sm.wave_a[wave] = mn;
      sm.wave_b[wave] = mx;
      sm.wave_c[wave] = nv;
    }
    for (int i = tid; i < kSelectSteps; i += NT) sm.cnt[i] = 0;
    if (tid < SMALL) sm.slist[tid] = kInvalid;
    if (tid == 0) sm.slist_n = 0;
    __syncthreads();
    uint32_t lo = kInv32, hi = 0u, m = 0u;
#pragma unroll
    for (int w = 0; w < SW; ++w) {
      lo = min(lo, sm.wave_a[w]);
      hi = max(hi, sm.wave_b[w]);
      m += sm.wave_c[w];
    }
    VATT_STAMP(dbg, 11);
    uint32_t r = c;    // rank wanted inside [lo, hi]; c - r composites lie below the range, m inside it
    bool low = false;  // false: searching on the high word; true: high word fixed to hv, on the low word
    uint32_t hv = 0u;
    // the word being searched, all-ones for slots that are empty or out of play: one unsigned compare of
    // (w - lo) against (pivot - lo) then tells whether a slot lies in [lo, pivot]
    uint32_t w[E];
#pragma unroll
    for (int e = 0; e < E; ++e) w[e] = ((xh[e] & xl[e]) != kInv32) ? min(xh[e], 0xfffffffeu) : kInv32;
    // (a high word of all-ones is searched as 0xfffffffe; the two values are told apart again when the last
    // few composites are ranked, so only more than SMALL composites with those two high words could be
    // misordered, which for 32-bit hashes of distinct tokens does not happen)
    hi = min(hi, 0xfffffffeu);
    lo = min(lo, hi);
    for (int step = 0; step < kSelectSteps; ++step) {
      if ((c - r) + m <= cap) {  // everything up to hi may be taken
        VATT_NOTE(dbg, 15, step);
        break;
      }
      if (m <= (uint32_t)SMALL) {
        uint32_t in_range = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) in_range |= ((w[e] - lo <= hi - lo) ? 1u : 0u) << e;
        if (in_range) {
          uint32_t pos = atomicAdd(&sm.slist_n, (uint32_t)__popc(in_range));
#pragma unroll
          for (int e = 0; e < E; ++e) {
            if ((in_range >> e) & 1u) {
              if (pos < (uint32_t)SMALL) sm.slist[pos] = ((uint64_t)xh[e] << 32) | xl[e];
              ++pos;
            }
          }
        }
        __syncthreads();
        if (tid < SMALL) {
          // rank inside the range = number of listed composites below mine (the list is padded with all-ones)
          const uint64_t mine = sm.slist[tid];
          uint32_t below = 0;
#pragma unroll
          for (int j = 0; j < SMALL; ++j) below += (sm.slist[j] < mine) ? 1u : 0u;
          if ((uint32_t)tid < m && below == r - 1u) sm.result = mine;
        }
        __syncthreads();
        VATT_STAMP(dbg, 12);
        VATT_NOTE(dbg, 13, step);
        VATT_NOTE(dbg, 14, m);
        return sm.result;
      }
      if (lo == hi) {
        // more than SMALL composites share this high word: go on with their low words
        low = true;
        hv = lo;
#pragma unroll
        for (int e = 0; e < E; ++e) w[e] = (w[e] == hv) ? xl[e] : kInv32;
        lo = 0u;
        hi = 0xfffffffeu;
      }
      const uint32_t span = hi - lo;
      // Pivot: two interpolation steps that aim a little above and a little below the wanted rank (so that
      // the range closes in from both sides when the values are spread evenly), then a midpoint step (which
      // bounds the number of steps for any data).
      uint32_t off;
      const int kind = step % 3;
      if (kind == 2) {
        off = span >> 1;
      } else {
        const float mf = (float)(m + 1u);
        const float want = (float)r + 0.5f * (float)(cap - c);  // middle of the acceptable window
        const float dev = 2.0f * sqrtf(fmaxf(want * (1.0f - want * __builtin_amdgcn_rcpf(mf)), 0.0f)) + 1.0f;
        const float aim = kind == 0 ? want + dev : want - dev;
        const float f = fminf(fmaxf(aim * __builtin_amdgcn_rcpf(mf), 0.0f), 1.0f);
        off = (uint32_t)fminf((float)span * f, 4294967040.0f);
      }
      off = min(off, span - 1u);
      // wave-level count straight from the compare masks
      uint32_t wave_cnt = 0;
#pragma unroll
      for (int e = 0; e < E; ++e) wave_cnt += (uint32_t)__popcll(__ballot(w[e] - lo <= off));
      if (lane == 0 && wave_cnt) atomicAdd(&sm.cnt[step], wave_cnt);
      __syncthreads();
      const uint32_t tot = sm.cnt[step];
      if (tot >= r) {
        hi = lo + off;
        m = tot;
      } else {
        lo = lo + off + 1u;
        r -= tot;
        m -= tot;
      }
    }
    VATT_STAMP(dbg, 12);
    VATT_NOTE(dbg, 13, 1000);
    if (!low && hi == 0xfffffffeu) return kInvalid - 1ull;
    return low ? (((uint64_t)hv << 32) | hi) : (((uint64_t)hi << 32) | kInv32);
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
// Stage 1.
// ---------------------------------------------------------------------------
struct Stage1Args {
  const float* scores;
  const int32_t* seq_lens;
  const uint64_t* seq_seeds;
  float* chunk_max;
  uint64_t* cand;      // [B*Hq][n_chunks][cand_cap]
  int32_t* cand_cnt;   // [B*Hq][n_chunks]
  uint64_t* key_comp;  // [B*Hq][2][n_key_slices][key_slice_cap]
  float* key_score;    // same shape
  uint32_t* key_cnt;   // [B*Hq][2][n_key_slices]
  SelectParams sp;
  int n_pad, n_max, Hq, chunk_len, n_chunks, cand_cap, key_slice_len, n_key_slices, key_slice_cap, key_on0, key_on1;
  unsigned long long* dbg;
};

template <int NT, int E>
__global__ __launch_bounds__(NT) void stage1_kernel(Stage1Args A) {
  constexpr int SW = NT / kWave;
  __shared__ SelectSmem<NT> sel_sm;
  __shared__ BlockScanSmem<NT> scan_sm;
  __shared__ float s_wmax[SW];

  const int role = (int)blockIdx.x >= A.n_chunks ? 1 : 0;
  const int part = role ? (int)blockIdx.x - A.n_chunks : (int)blockIdx.x;
  const int h = blockIdx.y, b = blockIdx.z;
  const int bh = b * A.Hq + h;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = min(max(A.seq_lens[b], 1), A.n_max);
  const HeadSizes hs = head_sizes(n, A.sp);
  const int span = role ? A.key_slice_len : A.chunk_len;
  const int lo = part * span;
  const int hi = min(lo + span, n);
  const float* row = A.scores + (int64_t)bh * A.n_pad;

  if (role == 1) {
    // ---- sampler candidates among tokens [lo, hi): two Philox blocks per thread and stream ----
    uint32_t* cnt_out = A.key_cnt + ((int64_t)bh * 2) * A.n_key_slices + part;  // stream s at + s * n_key_slices
    const int t_lo = max(lo, hs.mid_lo), t_hi = min(hi, hs.mid_hi);
    if (lo >= n || hs.n_s <= 0 || t_lo >= t_hi || (!A.key_on0 && !A.key_on1)) {
      if (tid < 2) cnt_out[tid * A.n_key_slices] = 0u;
      return;
    }
    const uint64_t seed = A.seq_seeds[b];
    uint64_t U[2];
    U[0] = A.key_on0 ? upper_bound_key((uint32_t)hs.b0, hs.n_s) : 0ull;
    U[1] = A.key_on1 ? upper_bound_key(stream1_design_count(hs), hs.n_s) : 0ull;
    // key_slice_len = 8 * NT tokens: thread t owns Philox blocks j0 + t and j0 + NT + t
    const int j0 = lo >> 2;
    uint32_t keys[2][8];
    uint32_t hit[2] = {0u, 0u};
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int j = j0 + u * NT + tid;
        const Philox4 ph = token_block_keys((uint32_t)j, (uint32_t)s, (uint32_t)h, seed);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = (j << 2) + e;
          keys[s][u * 4 + e] = ph.v[e];
          hit[s] |= ((i >= t_lo && i < t_hi && (uint64_t)ph.v[e] < U[s]) ? 1u : 0u) << (u * 4 + e);
        }
      }
    }
    // positions inside the slice's two lists: both counts ride one scan (low and high half of a word)
    uint32_t total;
    const uint32_t excl = block_exclusive_scan<NT>((uint32_t)__popc(hit[0]) | ((uint32_t)__popc(hit[1]) << 16), &total,
                                                   scan_sm);
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const uint32_t tot_s = s ? (total >> 16) : (total & 0xffffu);
      uint32_t pos = s ? (excl >> 16) : (excl & 0xffffu);
      const int64_t base = (((int64_t)bh * 2 + s) * A.n_key_slices + part) * A.key_slice_cap;
      if (tot_s <= (uint32_t)A.key_slice_cap) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          if ((hit[s] >> q) & 1u) {
            const int i = ((j0 + (q >> 2) * NT + tid) << 2) + (q & 3);
            A.key_comp[base + pos] = ((uint64_t)keys[s][q] << 32) | (uint32_t)i;
            A.key_score[base + pos] = row[i];
            ++pos;
          }
        }
      }
      if (tid == 0) cnt_out[s * A.n_key_slices] = tot_s <= (uint32_t)A.key_slice_cap ? tot_s : kOverflow;
    }
    return;
  }

  // ---- top-k candidates of the chunk [lo, hi) ----
  const int slot = bh * A.n_chunks + part;
  if (lo >= n) {
    if (tid == 0) {
      A.cand_cnt[slot] = 0;
      A.chunk_max[slot] = -INFINITY;
    }
    return;
  }
  VATT_STAMP(A.dbg, 0);
  float sc[E];
#pragma unroll
  for (int e = 0; e < E; ++e) sc[e] = row[min(lo + e * NT + tid, n - 1)];
  uint32_t xh[E], xl[E];
  float mx = -INFINITY;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int i = lo + e * NT + tid;
    const bool in_chunk = i < hi;
    const bool in_mid = in_chunk && i >= hs.mid_lo && i < hs.mid_hi;
    mx = in_chunk ? fmaxf(mx, sc[e]) : mx;
    xh[e] = in_mid ? ~float_order_key(sc[e]) : kInv32;
    xl[e] = in_mid ? (uint32_t)i : kInv32;
  }
  VATT_STAMP(A.dbg, 1);
  mx = wave_max(mx);
  if (lane == 0) s_wmax[wave] = mx;
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
  // a superset of the chunk's top-k is as good as the exact set here: stop as soon as it fits the slot
  const uint64_t T = (c == nvalid) ? (kInvalid - 1ull)
                                   : BlockSelect<NT, E>::run(xh, xl, (uint32_t)c, (uint32_t)min(nvalid, A.cand_cap),
                                                             sel_sm, A.dbg);
  VATT_STAMP(A.dbg, 3);
  uint32_t take = 0;
#pragma unroll
  for (int e = 0; e < E; ++e) take |= ((((uint64_t)xh[e] << 32) | xl[e]) <= T ? 1u : 0u) << e;
  uint32_t total;
  uint32_t pos = block_exclusive_scan<NT>((uint32_t)__popc(take), &total, scan_sm);
  uint64_t* out = A.cand + (int64_t)slot * A.cand_cap;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    if ((take >> e) & 1u) {
      if (pos < (uint32_t)A.cand_cap) out[pos] = ((uint64_t)xh[e] << 32) | xl[e];
      ++pos;
    }
  }
  if (tid == 0) A.cand_cnt[slot] = (int32_t)min(total, (uint32_t)A.cand_cap);
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
  const uint64_t* key_comp;
  const float* key_score;
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
  int n_pad, n_max, Hq, n_chunks, cand_cap, cand_shift, n_key_slices, key_slice_cap, key_slice_shift, key_on0, key_on1;
  int target, phase, force_slow, vstat_splits, head_dim;
  int k_max, b0_max, b_max, wlist_len;
  unsigned long long* dbg;
};

// Device functions of the per-head kernel for a workgroup of NT threads.
template <int NT>
struct HeadOps {
  static constexpr int SW = NT / kWave;
  static constexpr int EL = kListCap / NT;  // in-kernel sampler list composites per thread

  struct HeadSmem {
    SelectSmem<NT> sel;
    BlockScanSmem<NT> scan;
    uint64_t list[kListCap];
    uint32_t hist[256];
    double red[3][SW];
    uint32_t slice_cnt[2][kMaxKeySlices];
    uint32_t chunk_cnt[kMaxChunks];
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
  static __device__ __forceinline__ int list_tok(const int32_t* idx, int64_t pos, int n) {
    return min(max(idx[pos], 0), n - 1);
  }

  static __device__ __forceinline__ void mark_bit(uint32_t* bm, uint32_t i) { atomicOr(&bm[i >> 5], 1u << (i & 31)); }

  // Exclusive prefix of the set-bit counts of bm[0, words) into wpre; returns the number of set bits.
  static __device__ uint32_t word_prefix(const uint32_t* bm, int words, uint32_t* wpre, HeadSmem& sm) {
    const int wpt = (words + NT - 1) / NT;
    const int w0 = threadIdx.x * wpt;
    uint32_t cnt = 0;
    for (int w = w0; w < min(w0 + wpt, words); ++w) cnt += __popc(bm[w]);
    uint32_t total;
    uint32_t pos = block_exclusive_scan<NT>(cnt, &total, sm.scan);
    for (int w = w0; w < min(w0 + wpt, words); ++w) {
      wpre[w] = pos;
      pos += __popc(bm[w]);
    }
    __syncthreads();
    return total;
  }
  // Position of token i in the ascending list of the set bits of bm.
  static __device__ __forceinline__ uint32_t list_pos(const uint32_t* bm, const uint32_t* wpre, uint32_t i) {
    return wpre[i >> 5] + __popc(bm[i >> 5] & ((1u << (i & 31)) - 1u));
  }

  // Slow list writer (used after the in-kernel sweeps, which do not keep the scores): writes the set bits of
  // bm as ascending tokens and, when wlist is given, exp(s_i - m) of each into wlist at the same position.
  static __device__ void write_list_from_bitmap(const uint32_t* bm, int n, const uint32_t* wpre, int32_t* dst,
                                                uint32_t dst_cap, const float* row, float m, float* wlist,
                                                uint32_t wlist_len) {
    const int words = (n + 31) >> 5;
    for (int w = threadIdx.x; w < words; w += NT) {
      uint32_t bits = bm[w];
      uint32_t pos = wpre[w];
      while (bits) {
        const int i = (w << 5) + (__ffs(bits) - 1);
        bits &= bits - 1u;
        if (pos < dst_cap) dst[pos] = i;
        if (wlist && pos < wlist_len) wlist[pos] = __expf(row[i] - m);
        ++pos;
      }
    }
    __syncthreads();
  }

  // Sums of wlist[0, count) and of its squares, taken in a fixed order.
  static __device__ __forceinline__ void sum_wlist(const float* wlist, uint32_t count, double* s1, double* s2) {
    double a = 0.0, a2 = 0.0;
    for (uint32_t t = threadIdx.x; t < count; t += NT) {
      const double w = (double)wlist[t];
      a += w;
      a2 += w * w;
    }
    *s1 += a;
    *s2 += a2;
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

  // Select the `need` smallest composites of the LDS list sm.list[0, listed) and mark their tokens in bm_s.
  static __device__ void mark_smallest_of_list(uint32_t* bm_s, uint32_t listed, uint32_t need, HeadSmem& sm) {
    uint32_t xh[EL], xl[EL];
#pragma unroll
    for (int e = 0; e < EL; ++e) {
      const uint32_t p = e * NT + threadIdx.x;
      const uint64_t t = p < listed ? sm.list[p] : kInvalid;
      xh[e] = (uint32_t)(t >> 32);
      xl[e] = (uint32_t)t;
    }
    const uint64_t T = (need >= listed) ? (kInvalid - 1ull) : BlockSelect<NT, EL>::run(xh, xl, need, need, sm.sel);
#pragma unroll
    for (int e = 0; e < EL; ++e)
      if ((((uint64_t)xh[e] << 32) | xl[e]) <= T) mark_bit(bm_s, xl[e]);
  }

  // Fast sample: among the candidates stage 1 wrote for this head and stream (every middle token whose key
  // is under the design bound, slice by slice, with its score).  Usable when no slice overflowed and the
  // residual tokens among the candidates number at least c; then the c smallest residual composites are
  // the sample.  Marks them in bm_s (all zero on entry), then writes the ascending token list to dst and,
  // when wlist is given, exp(score - m) of each to wlist at its list position.  tc / xs hold the candidate
  // slots of this thread (composite and score of slot e * NT + tid), read from global memory by the caller.
  template <int EK>
  static __device__ bool sample_from_candidates(uint32_t* bm_s, const uint32_t* bm_f, uint32_t* wpre,
                                                const HeadSizes& hs, uint32_t c, const uint64_t (&tc)[EK],
                                                const float (&xs)[EK], const uint32_t* slice_cnt, int n_slices,
                                                int slice_shift, int32_t* dst, uint32_t dst_cap, float m,
                                                float* wlist, uint32_t wlist_len, HeadSmem& sm,
                                                unsigned long long* dbg = nullptr) {
    const int tid = threadIdx.x;
    const int slots = n_slices << slice_shift;
    VATT_STAMP(dbg, 1);
    // slot p = e * NT + tid belongs to slice p >> slice_shift
    uint32_t xh[EK], xl[EK];
    uint32_t valid = 0, bad = 0;
#pragma unroll
    for (int e = 0; e < EK; ++e) {
      const int p = e * NT + tid;
      const int pc = min(p, slots - 1);
      const int sl = pc >> slice_shift, off = pc & ((1 << slice_shift) - 1);
      const uint32_t cnt = slice_cnt[sl];
      const uint64_t t = tc[e];
      const uint32_t i = (uint32_t)t;
      bad |= (p < slots && cnt == kOverflow) ? 1u : 0u;
      const bool present = p < slots && cnt != kOverflow && (uint32_t)off < cnt;
      const uint32_t ic = present ? min(i, (uint32_t)(hs.n - 1)) : 0u;
      const bool res = present && (int)i >= hs.mid_lo && (int)i < hs.mid_hi && !((bm_f[ic >> 5] >> (ic & 31)) & 1u);
      xh[e] = res ? (uint32_t)(t >> 32) : kInv32;
      xl[e] = res ? i : kInv32;
      valid += res ? 1u : 0u;
    }
    valid = wave_sum_u32(valid);
    bad = wave_sum_u32(bad);
    __syncthreads();
    if (tid == 0) {
      sm.u_a = 0;
      sm.u_b = 0;
    }
    __syncthreads();
    if ((tid & 63) == 0) {
      if (valid) atomicAdd(&sm.u_a, valid);
      if (bad) atomicAdd(&sm.u_b, 1u);
    }
    __syncthreads();
    const uint32_t total = sm.u_a;
    VATT_STAMP(dbg, 2);
    if (sm.u_b != 0 || total < c) return false;
    const uint64_t T = (total == c) ? (kInvalid - 1ull) : BlockSelect<NT, EK>::run(xh, xl, c, c, sm.sel, dbg);
#pragma unroll
    for (int e = 0; e < EK; ++e)
      if ((((uint64_t)xh[e] << 32) | xl[e]) <= T) mark_bit(bm_s, xl[e]);
    __syncthreads();
    VATT_STAMP(dbg, 3);
    word_prefix(bm_s, (hs.n + 31) >> 5, wpre, sm);
    VATT_STAMP(dbg, 4);
#pragma unroll
    for (int e = 0; e < EK; ++e) {
      if ((((uint64_t)xh[e] << 32) | xl[e]) <= T) {
        const uint32_t pos = list_pos(bm_s, wpre, xl[e]);
        if (pos < dst_cap) dst[pos] = (int32_t)xl[e];
        if (wlist && pos < wlist_len) wlist[pos] = __expf(xs[e] - m);
      }
    }
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
      for (int w = tid; w < words; w += NT) {
        uint32_t mm = 0;
        const int i0 = w << 5;
        if (i0 + 31 >= hs.mid_lo && i0 < hs.mid_hi) {
          const int a = max(hs.mid_lo - i0, 0), bnd = min(hs.mid_hi - i0, 32);
          mm = (bnd >= 32 ? 0xffffffffu : ((1u << bnd) - 1u)) & ~((1u << a) - 1u);
        }
        bm_s[w] = mm & ~bm_f[w];
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
      for (int j = j_lo + tid; j < j_hi; j += NT) {
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
        for (int w = tid; w < words; w += NT) bm_s[w] = 0;  // discard the guess
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
      for (int d = tid; d < 256; d += NT) sm.hist[d] = 0;
      __syncthreads();
      for (int j = j_lo + tid; j < j_hi; j += NT) {
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
        for (int j = j_lo + tid; j < j_hi; j += NT) {
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
          const uint32_t p = e * NT + tid;
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
    for (int j = j_lo + tid; j < j_hi; j += NT) {
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

  // Draw a sample of size c for `stream` and write its ascending token list; the return value reports the
  // path taken (flag bits of out_counts[7]).  tc / xs: this thread's slots of the stream's candidate list.
  template <int EK>
  static __device__ int draw_sample(uint32_t* bm_s, const uint32_t* bm_f, uint32_t* wpre, const HeadSizes& hs,
                                    uint32_t c, int stream, const HeadArgs& A, int h, uint64_t seed,
                                    const uint64_t (&tc)[EK], const float (&xs)[EK], const float* row, int32_t* dst,
                                    uint32_t dst_cap, float m, float* wlist, HeadSmem& sm) {
    const int words = (hs.n + 31) >> 5;
    const bool list_on = (stream == 0 ? A.key_on0 : A.key_on1) != 0;
    bool ok = false;
    if (!A.force_slow && list_on && c < (uint32_t)hs.n_s) {
      unsigned long long* dbg = A.dbg ? A.dbg + 200 + 100 * stream : nullptr;
      (void)dbg;
      ok = sample_from_candidates<EK>(bm_s, bm_f, wpre, hs, c, tc, xs, sm.slice_cnt[stream], A.n_key_slices,
                                      A.key_slice_shift, dst, dst_cap, m, wlist, (uint32_t)A.wlist_len, sm, dbg);
    }
    if (ok) return 0;
    __syncthreads();
    for (int w = threadIdx.x; w < words; w += NT) bm_s[w] = 0;
    __syncthreads();
    const int slow = sample_by_sweep(bm_s, bm_f, hs, c, (uint32_t)stream, (uint32_t)h, seed, A.force_slow, sm);
    word_prefix(bm_s, words, wpre, sm);
    write_list_from_bitmap(bm_s, hs.n, wpre, dst, dst_cap, row, m, wlist, (uint32_t)A.wlist_len);
    return (stream == 0 ? (2 | (slow << 2)) : ((c < (uint32_t)hs.n_s ? 8 : 0) | slow));
  }
};  // struct HeadOps

// NT = workgroup size; EM = top-k candidate slots a thread holds (n_chunks * cand_cap <= EM * NT); EK = sampler
// candidate slots a thread holds per stream (n_key_slices * key_slice_cap <= EK * NT when the lists are on).
template <int NT, int EM, int EK>
__global__ __launch_bounds__(NT) void head_kernel(HeadArgs A) {
  using O = HeadOps<NT>;
  using HeadSmem = typename O::HeadSmem;
  constexpr int SW = NT / kWave;
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
  uint32_t* wpre = bm_s + words_max;
  float* wlist = reinterpret_cast<float*>(wpre + words_max);

  const float* row = A.scores + (int64_t)bh * A.n_pad;
  int32_t* idx = A.out_idx + (int64_t)bh * A.idx_cap;
  const uint64_t seed = A.seq_seeds[b];

  VATT_STAMP(A.dbg, 0);
  // Everything this kernel needs from global memory is requested up front, so that the latencies overlap:
  // the head's top-k candidate slots and its sampler candidate slots (composite and score) of both streams.
  uint64_t tcand[EM];
  {
    const uint64_t* src = A.cand + (int64_t)bh * A.n_chunks * A.cand_cap;
    const int slots = A.n_chunks * A.cand_cap;
#pragma unroll
    for (int e = 0; e < EM; ++e) tcand[e] = (A.phase != 2) ? src[min(e * NT + tid, slots - 1)] : kInvalid;
  }
  uint64_t kc0[EK], kc1[EK];
  float ks0[EK], ks1[EK];
  {
    const int kslots = A.n_key_slices << A.key_slice_shift;
    const int64_t base = (int64_t)bh * 2 * kslots;
#pragma unroll
    for (int e = 0; e < EK; ++e) {
      const int pc = min(e * NT + tid, kslots - 1);
      const bool in = e * NT + tid < kslots;
      kc0[e] = (A.key_on0 && A.phase != 2 && in) ? A.key_comp[base + pc] : kInvalid;
      ks0[e] = (A.key_on0 && A.phase != 2 && in) ? A.key_score[base + pc] : 0.f;
      kc1[e] = (A.key_on1 && A.phase != 1 && in) ? A.key_comp[base + kslots + pc] : kInvalid;
      ks1[e] = (A.key_on1 && A.phase != 1 && in) ? A.key_score[base + kslots + pc] : 0.f;
    }
  }
  for (int w = tid; w < words; w += NT) {
    bm_f[w] = 0;
    bm_s[w] = 0;
  }
  for (int c = tid; c < A.n_chunks; c += NT) sm.chunk_cnt[c] = (uint32_t)A.cand_cnt[bh * A.n_chunks + c];
  for (int t = tid; t < 2 * A.n_key_slices; t += NT)
    sm.slice_cnt[t / A.n_key_slices][t % A.n_key_slices] = A.key_cnt[(int64_t)bh * 2 * A.n_key_slices + t];
  // head maximum from the chunk maxima
  float m = -INFINITY;
  for (int c = tid; c < A.n_chunks; c += NT) m = fmaxf(m, A.chunk_max[bh * A.n_chunks + c]);
  m = wave_max(m);
  __syncthreads();
  if ((tid & 63) == 0) sm.red[0][tid >> 6] = (double)m;
  __syncthreads();
  m = (float)sm.red[0][0];
#pragma unroll
  for (int w = 1; w < SW; ++w) m = fmaxf(m, (float)sm.red[0][w]);
  __syncthreads();

  VATT_STAMP(A.dbg, 1);
  double acc_f = 0.0, unused = 0.0;  // acc_f: this thread's share of D_f = sum over I_f of exp(s_i - m)
  // ---- I_t (Algorithm 1, line 3) ----
  if (A.phase != 2) {
    if (hs.k > 0) {
      // slot p = e * NT + tid of the candidate array belongs to chunk p >> cand_shift
      uint32_t xh[EM], xl[EM];
      const int slots = A.n_chunks * A.cand_cap;
      uint32_t total = 0;
      for (int c = 0; c < A.n_chunks; ++c) total += sm.chunk_cnt[c];
#pragma unroll
      for (int e = 0; e < EM; ++e) {
        const int p = e * NT + tid;
        const int pc = min(p, slots - 1);
        const int ch = pc >> A.cand_shift, off = pc & (A.cand_cap - 1);
        const bool ok = p < slots && (uint32_t)off < sm.chunk_cnt[ch];
        xh[e] = ok ? (uint32_t)(tcand[e] >> 32) : kInv32;
        xl[e] = ok ? (uint32_t)tcand[e] : kInv32;
      }
      VATT_STAMP(A.dbg, 2);
      const uint64_t T = ((uint32_t)hs.k >= total)
                             ? (kInvalid - 1ull)
                             : BlockSelect<NT, EM>::run(xh, xl, (uint32_t)hs.k, (uint32_t)hs.k, sm.sel,
                                                        A.dbg ? A.dbg + 100 : nullptr);
      VATT_STAMP(A.dbg, 3);
#pragma unroll
      for (int e = 0; e < EM; ++e)
        if ((((uint64_t)xh[e] << 32) | xl[e]) <= T) O::mark_bit(bm_f, xl[e]);
      __syncthreads();
      O::word_prefix(bm_f, words, wpre, sm);
      // every chosen candidate knows its place in the ascending list and carries its score in its high word
#pragma unroll
      for (int e = 0; e < EM; ++e) {
        if ((((uint64_t)xh[e] << 32) | xl[e]) <= T) {
          const uint32_t pos = O::list_pos(bm_f, wpre, xl[e]);
          if (pos < (uint32_t)A.k_max) idx[A.seg_topk + pos] = (int32_t)xl[e];
          if (pos < (uint32_t)A.wlist_len) wlist[pos] = __expf(float_from_order_key(~xh[e]) - m);
        }
      }
      __syncthreads();
      O::sum_wlist(wlist, (uint32_t)hs.k, &acc_f, &unused);
      __syncthreads();
      VATT_STAMP(A.dbg, 4);
    }
    for (int i = tid; i < hs.n_sink; i += NT) idx[A.seg_sink + i] = i;
    for (int i = tid; i < hs.n_win; i += NT) idx[A.seg_win + i] = hs.mid_hi + i;
  } else {
    // phase 2: rebuild the top-k bitmap from the list written in phase 1
    for (int t = tid; t < hs.k; t += NT) {
      const int i = O::list_tok(idx, A.seg_topk + t, n);
      O::mark_bit(bm_f, (uint32_t)i);
      acc_f += (double)__expf(row[i] - m);
    }
  }
  for (int i = tid; i < hs.n_sink; i += NT) acc_f += (double)__expf(row[i] - m);
  for (int i = tid; i < hs.n_win; i += NT) acc_f += (double)__expf(row[hs.mid_hi + i] - m);
  __syncthreads();

  // ---- I_bs (Algorithm 2, line 1) and the sums over it ----
  int flags = 0;
  double acc_w = 0.0, acc_w2 = 0.0;
  if (hs.n_s > 0) {
    if (A.phase != 2) {
      flags |= O::template draw_sample<EK>(bm_s, bm_f, wpre, hs, (uint32_t)hs.b0, 0, A, h, seed, kc0, ks0, row,
                                           idx + A.seg_base, (uint32_t)A.b0_max, m, wlist, sm);
      VATT_STAMP(A.dbg, 5);
      O::sum_wlist(wlist, (uint32_t)hs.b0, &acc_w, &acc_w2);
      __syncthreads();
      for (int w = tid; w < words; w += NT) bm_s[w] = 0;
      __syncthreads();
      VATT_STAMP(A.dbg, 6);
    } else {
      for (int t = tid; t < hs.b0; t += NT) {
        const double wgt = (double)__expf(row[O::list_tok(idx, A.seg_base + t, n)] - m);
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
    flags |= O::template draw_sample<EK>(bm_s, bm_f, wpre, hs, (uint32_t)bfin, 1, A, h, seed, kc1, ks1, row,
                                         idx + A.seg_dyn, (uint32_t)A.b_max, m, nullptr, sm);
    VATT_STAMP(A.dbg, 8);
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
  VATT_STAMP(A.dbg, 9);
}

typedef void (*HeadKernel)(HeadArgs);
// The instantiation for a plan: (workgroup size, top-k slots per thread, sampler slots per thread).
HeadKernel head_kernel_for(const Plan& pl) {
  const int64_t cands = (int64_t)pl.n_chunks * pl.cand_cap;
  if (pl.head_threads == 256) {
    if (cands <= 16 * 256) {
      if (pl.key_elems <= 8) return head_kernel<256, 16, 8>;
      return pl.key_elems <= 16 ? head_kernel<256, 16, 16> : head_kernel<256, 16, 32>;
    }
    if (pl.key_elems <= 8) return head_kernel<256, 32, 8>;
    return pl.key_elems <= 16 ? head_kernel<256, 32, 16> : head_kernel<256, 32, 32>;
  }
  return head_kernel<1024, 32, 4>;
}

}  // namespace

hipError_t set_kernel_attributes(const Plan& pl) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(head_kernel_for(pl)),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)pl.head_lds_bytes);
}

size_t head_kernel_lds_bytes(int n_max, int head_threads, int wlist_len) {
  const size_t words_max = (size_t)(n_max + 31) >> 5;
  const size_t fixed = head_threads == 256 ? sizeof(HeadOps<256>::HeadSmem) : sizeof(HeadOps<1024>::HeadSmem);
  return ((fixed + 15) & ~size_t(15)) + 3 * words_max * sizeof(uint32_t) + (size_t)wlist_len * sizeof(float);
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
  A.key_comp = reinterpret_cast<uint64_t*>(w + pl.off_key_comp);
  A.key_score = reinterpret_cast<float*>(w + pl.off_key_score);
  A.key_cnt = reinterpret_cast<uint32_t*>(w + pl.off_key_cnt);
  A.sp = pl.sel;
  A.n_pad = pl.n_pad;
  A.n_max = p.n_max;
  A.Hq = p.n_q_heads;
  A.chunk_len = pl.chunk_len;
  A.n_chunks = pl.n_chunks;
  A.cand_cap = pl.cand_cap;
  A.key_slice_len = pl.key_slice_len;
  A.n_key_slices = pl.n_key_slices;
  A.key_slice_cap = pl.key_slice_cap;
  A.key_on0 = pl.key_on[0];
  A.key_on1 = pl.key_on[1];
  A.dbg = reinterpret_cast<unsigned long long*>(w + pl.off_debug);
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
  A.key_comp = reinterpret_cast<const uint64_t*>(w + pl.off_key_comp);
  A.key_score = reinterpret_cast<const float*>(w + pl.off_key_score);
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
  A.cand_shift = pl.cand_shift;
  A.n_key_slices = pl.n_key_slices;
  A.key_slice_cap = pl.key_slice_cap;
  A.key_slice_shift = pl.key_slice_shift;
  A.key_on0 = pl.key_on[0];
  A.key_on1 = pl.key_on[1];
  A.target = p.target;
  A.phase = phase;
  A.force_slow = pl.force_slow_sampler;
  A.vstat_splits = pl.vstat_splits;
  A.head_dim = p.head_dim;
  A.k_max = pl.k_max;
  A.b0_max = pl.b0_max;
  A.b_max = pl.b_max;
  A.wlist_len = pl.wlist_len;
  A.dbg = reinterpret_cast<unsigned long long*>(w + pl.off_debug) + 64;
  hipLaunchKernelGGL(head_kernel_for(pl), dim3(p.n_q_heads, p.batch), dim3(pl.head_threads), pl.head_lds_bytes, st, A);
  return hipGetLastError();
}

}  // namespace vatt
