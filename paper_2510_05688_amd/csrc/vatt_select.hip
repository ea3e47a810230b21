// Index selection and budget: lines 1-8 of Algorithm 1 and all of Algorithm 2, per (sequence, query head).
//
// Top-k: every token of the middle region carries the 64-bit composite (~order_key(score) << 32) | token,
// distinct per token, so "the k largest scores, ties to the lower token" is "the k smallest composites": a pure
// set operation whose result does not depend on the order in which lanes, waves or workgroups contribute.
//
// Samples: sequential uniform draws from the middle region (Philox4x32-10 words, unbiased multiply-and-reject
// mapping), skipping top-k members and tokens drawn before; the first c accepted tokens are the sample (for
// c > n_s / 2 they are the tokens left out).  The kernel processes the draw sequence in batches: all draws of
// a batch are generated at once, repeated tokens are resolved to their earliest draw, and a prefix count in
// draw order finds where the sample is complete; the result equals the sequential procedure bit for bit.
//
// Floating-point sums are taken in a fixed order, so the statistics and the budget are reproducible too.
//
// Two kernels:
//   stage1_kernel  one workgroup per chunk of a head's score row: the chunk is kept in registers, a threshold
//                  that keeps at least its own top-k is found by counting, and the composites under it are
//                  written in ascending token order as candidates (any member of the global top-k is in its
//                  chunk's top-k), plus the chunk maximum.
//   head_kernel    one workgroup per head: selects the exact top-k among the chunk candidates, draws the base
//                  sample, computes the statistics and the budget of Algorithm 2, draws the final sample, and
//                  writes the index lists.
#include "vatt_internal.h"

namespace vatt {
namespace {

constexpr uint32_t kInv32 = 0xffffffffu;
constexpr uint64_t kInvalid = ~0ull;

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
// starts as the minimum and maximum present; each step splits it into up to eight equal bins, counts the
// composites of every bin (byte counters in registers, DPP wave sums, eight LDS adds per wave, one barrier)
// and keeps the bin that holds the target, so the span shrinks by four or more per step whatever the data.
// When at most SMALL composites remain they are ranked directly by one wave.  Equal high words are resolved
// the same way on the low word.
// ---------------------------------------------------------------------------
constexpr int kSelectSteps = 48;  // at most 16 steps per 32-bit word (a step divides the span by four or more)

template <int NT>
struct SelectSmem {
  static constexpr int SMALL = 64;
  uint32_t cnt[kSelectSteps * 8];
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
    for (int i = tid; i < kSelectSteps * 8; i += NT) sm.cnt[i] = 0;
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
        // list positions: a scan inside the wave, one LDS add per wave
        const uint32_t mine = (uint32_t)__popc(in_range);
        const uint32_t incl = wave_inclusive_scan_u32(mine);
        const uint32_t wave_tot = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
        uint32_t base = 0;
        if (lane == 0 && wave_tot) base = atomicAdd(&sm.slist_n, wave_tot);
        base = (uint32_t)__builtin_amdgcn_readfirstlane((int)base);
        if (in_range) {
          uint32_t pos = base + incl - mine;
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
      const uint32_t span = hi - lo;  // >= 1 here
      // Equal bins of width 2^s over [lo, hi], five to eight of them (span + 1 when the span is below 4): every
      // element adds one to a byte counter of its bin, the byte counters are widened and summed over the wave,
      // and lanes 0..7 add the wave's counts to the step's eight LDS counters.
      const int s = max(0, 29 - (int)__clz(span));
      uint64_t acc = 0;
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const uint32_t d = w[e] - lo;
        const uint32_t sh = ((d >> s) & 7u) << 3;
        acc += (d <= span) ? (1ull << sh) : 0ull;
      }
      const uint32_t a0 = (uint32_t)acc, a1 = (uint32_t)(acc >> 32);
      const uint32_t f0 = wave_sum_u32(a0 & 0x00ff00ffu), f1 = wave_sum_u32((a0 >> 8) & 0x00ff00ffu);
      const uint32_t f2 = wave_sum_u32(a1 & 0x00ff00ffu), f3 = wave_sum_u32((a1 >> 8) & 0x00ff00ffu);
      {
        const uint32_t fa = (lane & 4) ? ((lane & 1) ? f3 : f2) : ((lane & 1) ? f1 : f0);
        const uint32_t mine = (lane & 2) ? (fa >> 16) : (fa & 0xffffu);
        if (lane < 8 && mine) atomicAdd(&sm.cnt[step * 8 + lane], mine);
      }
      __syncthreads();
      uint32_t cum = 0, below = 0, inbin = 0, j = 0;
      bool found = false;
#pragma unroll
      for (int bq = 0; bq < 8; ++bq) {
        const uint32_t t = sm.cnt[step * 8 + bq];
        if (!found && cum + t >= r) {
          found = true;
          j = (uint32_t)bq;
          below = cum;
          inbin = t;
        }
        cum += t;
      }
      const uint32_t lo_new = lo + (j << s);
      hi = min(hi, lo_new + ((1u << s) - 1u));
      lo = lo_new;
      r -= below;
      m = inbin;
    }
    VATT_STAMP(dbg, 12);
    VATT_NOTE(dbg, 13, 1000);
    if (!low && hi == 0xfffffffeu) return kInvalid - 1ull;
    return low ? (((uint64_t)hv << 32) | hi) : (((uint64_t)hi << 32) | kInv32);
  }
};

// ---------------------------------------------------------------------------
// Positions of the taken elements of a workgroup in (element-major, thread-minor) order: element e of thread
// t comes before element e' of thread t' when e < e', or e == e' and t < t'.  With the interleaved slot
// layout p = e * NT + t this is ascending slot order.  pos[e] is valid where bit e of take is set.
// ---------------------------------------------------------------------------
template <int NT, int E>
struct OrderedSmem {
  uint32_t cnt[E * (NT / kWave)];
  uint32_t total;
};

template <int NT, int E>
__device__ __forceinline__ void ordered_positions(uint32_t take, uint32_t (&pos)[E], uint32_t* total,
                                                  OrderedSmem<NT, E>& sm) {
  static_assert(E <= kWave, "one lane per element publishes the wave count");
  constexpr int SW = NT / kWave;
  constexpr int CNT = E * SW;
  constexpr int PER = (CNT + kWave - 1) / kWave;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t mine = 0;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const uint64_t mask = __ballot((take >> e) & 1u);
    pos[e] = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
    const uint32_t c = (uint32_t)__popcll(mask);
    mine = (lane == e) ? c : mine;
  }
  __syncthreads();  // a previous use may still be read
  if (lane < E) sm.cnt[lane * SW + wave] = mine;
  __syncthreads();
  if (wave == 0) {
    uint32_t v[PER], s = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int q = lane * PER + i;
      v[i] = q < CNT ? sm.cnt[q] : 0u;
      s += v[i];
    }
    const uint32_t incl = wave_inclusive_scan_u32(s);
    uint32_t run = incl - s;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int q = lane * PER + i;
      if (q < CNT) sm.cnt[q] = run;
      run += v[i];
    }
    if (lane == kWave - 1) sm.total = incl;
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < E; ++e) pos[e] += sm.cnt[e * SW + wave];
  *total = sm.total;
}

// ---------------------------------------------------------------------------
// Stage 1: top-k candidates of one chunk of a head's score row.
// ---------------------------------------------------------------------------
struct Stage1Args {
  const float* scores;
  const int32_t* seq_lens;
  float* chunk_max;
  uint64_t* cand;      // [B*Hq][n_chunks][cand_cap]
  int32_t* cand_cnt;   // [B*Hq][n_chunks]
  SelectParams sp;
  int n_pad, n_max, Hq, chunk_len, n_chunks, cand_cap;
  unsigned long long* dbg;
};

template <int NT, int E>
__global__ __launch_bounds__(NT) void stage1_kernel(Stage1Args A) {
  constexpr int SW = NT / kWave;
  __shared__ SelectSmem<NT> sel_sm;
  __shared__ OrderedSmem<NT, E> ord_sm;
  __shared__ float s_wmax[SW];

  const int part = blockIdx.x;
  const int h = blockIdx.y, b = blockIdx.z;
  const int bh = b * A.Hq + h;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = min(max(A.seq_lens[b], 1), A.n_max);
  const HeadSizes hs = head_sizes(n, A.sp);
  const int lo = part * A.chunk_len;
  const int hi = min(lo + A.chunk_len, n);
  const float* row = A.scores + (int64_t)bh * A.n_pad;

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
  // element e of thread t is token lo + e * NT + t: element-major order is ascending token order
  uint32_t pos[E], total;
  ordered_positions<NT, E>(take, pos, &total, ord_sm);
  uint64_t* out = A.cand + (int64_t)slot * A.cand_cap;
#pragma unroll
  for (int e = 0; e < E; ++e)
    if (((take >> e) & 1u) && pos[e] < (uint32_t)A.cand_cap) out[pos[e]] = ((uint64_t)xh[e] << 32) | xl[e];
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
  int n_pad, n_max, Hq, n_chunks, cand_cap, cand_shift;
  int target, phase, small_batches, vstat_splits, head_dim;
  int k_max, b0_max, b_max;
  uint32_t draw_cap;  // 0: the default 64 L + 4096
  unsigned long long* dbg;
};

constexpr int kSmallBatchBlocks = 64;  // Philox blocks of a small batch (256 draws)

// flag bits of out_counts[7]
constexpr int kFlagBaseComplement = 1, kFlagDynComplement = 2, kFlagBaseBatches = 4, kFlagDynBatches = 8,
              kFlagDrawCap = 16;

// One batch of the draw sequence as a thread sees it: the four draws of one Philox block.
struct DrawBatch {
  uint32_t tok[4];  // proposed tokens
  float sc[4];      // their scores, when loaded ahead
  uint32_t ok;      // bit e: the draw counts (inside the batch and the draw cap, word not rejected, token not
                    // drawn in an earlier batch)
  uint32_t first;   // bit e: ok and no earlier draw of the batch proposes the same token
  int blocks;       // Philox blocks in the batch
  bool have_sc;
};

// Device functions of the per-head kernel for a workgroup of NT threads.
template <int NT>
struct HeadOps {
  static constexpr int SW = NT / kWave;

  struct HeadSmem {
    SelectSmem<NT> sel;
    BlockScanSmem<NT> scan;
    double red[3][SW];
    uint32_t chunk_cnt[kMaxChunks];
    uint32_t again;
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
  static __device__ __forceinline__ bool test_bit(const uint32_t* bm, uint32_t i) { return (bm[i >> 5] >> (i & 31)) & 1u; }

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

  // Bits of word w that lie in the middle region [mid_lo, mid_hi).
  static __device__ __forceinline__ uint32_t mid_mask(const HeadSizes& hs, int w) {
    const int i0 = w << 5;
    if (i0 + 31 < hs.mid_lo || i0 >= hs.mid_hi) return 0u;
    const int a = max(hs.mid_lo - i0, 0), bnd = min(hs.mid_hi - i0, 32);
    return (bnd >= 32 ? 0xffffffffu : ((1u << bnd) - 1u)) & ~((1u << a) - 1u);
  }

  // What one sample needs to know.
  struct Sampler {
    uint32_t* taken;      // tokens proposed so far (bitmap, LDS)
    uint32_t* scratch;    // all-zero bitmap between uses (LDS)
    uint32_t* mail;       // one slot per bitmap word, all-ones between uses (LDS)
    const uint32_t* bm_f; // top-k members (bitmap, LDS)
    uint32_t* wpre;       // word prefixes (LDS)
    const float* row;     // the head's scores
    uint64_t seed;
    uint32_t stream, head;
    uint32_t L, thr;      // middle-region length and 2^32 mod L
    uint32_t cap;         // draws allowed
    float m;
    unsigned long long* dbg;
  };

  // Generate the draws of Philox blocks [blk0, blk0 + blocks) of the stream and find, for every token that is
  // proposed more than once in the batch, its earliest draw.
  //
  // Every draw that counts sets its token's bit in `taken`; a draw that finds the bit already set knows that
  // the token is repeated and says so in `scratch`.  The draws of repeated tokens then post (draw number,
  // bit position) with an atomic minimum into the mail slot of their bitmap word; the smallest draw number
  // of a token wins its slot.  Two repeated tokens that share a word take turns (one more round per token).
  static __device__ __forceinline__ void make_batch(DrawBatch& B, const Sampler& S, const HeadSizes& hs, uint32_t blk0, int blocks,
                                    bool check_prev, bool load_scores, HeadSmem& sm) {
    const int tid = threadIdx.x;
    B.blocks = blocks;
    B.ok = 0;
    B.first = 0;
    B.have_sc = load_scores;
    VATT_STAMP(S.dbg, 0);
    if (tid < blocks) {
      const Philox4 ph = philox4x32_10(blk0 + (uint32_t)tid, S.stream, S.head, 0u, (uint32_t)S.seed,
                                       (uint32_t)(S.seed >> 32));
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t j = ((blk0 + (uint32_t)tid) << 2) + (uint32_t)e;
        const uint64_t x = (uint64_t)ph.v[e] * (uint64_t)S.L;
        const uint32_t t = (uint32_t)hs.mid_lo + (uint32_t)(x >> 32);
        bool v = j < S.cap && (uint32_t)x >= S.thr;
        if (check_prev) v = v && !test_bit(S.taken, t);
        B.tok[e] = t;
        B.ok |= (v ? 1u : 0u) << e;
      }
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) B.tok[e] = (uint32_t)hs.mid_lo;
    }
    if (load_scores) {
#pragma unroll
      for (int e = 0; e < 4; ++e) B.sc[e] = S.row[B.tok[e]];
    }
    VATT_STAMP(S.dbg, 1);
    if (check_prev) __syncthreads();  // every test of `taken` comes before the marks of this batch
    uint32_t lose = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if ((B.ok >> e) & 1u) {
        const uint32_t bit = 1u << (B.tok[e] & 31);
        const uint32_t old = atomicOr(&S.taken[B.tok[e] >> 5], bit);
        if (old & bit) {
          lose |= 1u << e;
          atomicOr(&S.scratch[B.tok[e] >> 5], bit);
        }
      }
    }
    __syncthreads();
    VATT_STAMP(S.dbg, 2);
    // draws whose token is proposed more than once in this batch
    uint32_t unresolved = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (((B.ok >> e) & 1u) && test_bit(S.scratch, B.tok[e])) unresolved |= 1u << e;
    uint32_t later = 0;
    for (;;) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if ((unresolved >> e) & 1u) atomicMin(&S.mail[B.tok[e] >> 5], ((uint32_t)(tid * 4 + e) << 5) | (B.tok[e] & 31));
      if (tid == 0) sm.again = 0;
      __syncthreads();
      uint32_t won = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if ((unresolved >> e) & 1u) {
          const uint32_t v = S.mail[B.tok[e] >> 5];
          if ((v & 31u) == (B.tok[e] & 31u)) {
            if ((v >> 5) == (uint32_t)(tid * 4 + e)) won |= 1u << e; else later |= 1u << e;
            unresolved &= ~(1u << e);
          }
        }
      }
      if (unresolved) sm.again = 1;
      __syncthreads();
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if ((won >> e) & 1u) S.mail[B.tok[e] >> 5] = kInv32;
      const bool again = sm.again != 0;
      __syncthreads();
      if (!again) break;
    }
    B.first = B.ok & ~later;
    VATT_STAMP(S.dbg, 3);
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if ((lose >> e) & 1u) atomicAnd(&S.scratch[B.tok[e] >> 5], ~(1u << (B.tok[e] & 31)));
    __syncthreads();
    VATT_STAMP(S.dbg, 4);
  }

  // Draw a sample of c residual tokens for the stream described by S.  `taken` must be all zero on entry
  // unless `spec` carries the first batch (have_spec; made from block 0 with make_batch), `scratch` all zero.
  // Writes the token list to dst (acceptance order, or ascending when the sample is a complement) and, when
  // sum_w is given, adds exp(s_i - m) and its square over the sample to this thread's partial sums.
  // Returns flag bits: 1 complement regime, 2 more than one batch, 4 draw cap reached.
  static __device__ __forceinline__ int draw_sample(const Sampler& S, const HeadSizes& hs, uint32_t c, const DrawBatch& spec, bool have_spec,
                                    int small_batches, int32_t* dst, uint32_t dst_cap, double* sum_w,
                                    double* sum_w2, HeadSmem& sm) {
    const int tid = threadIdx.x;
    const int words = (hs.n + 31) >> 5;
    const uint32_t ns = (uint32_t)hs.n_s;
    if (c == 0) return 0;
    int flags = 0;
    const bool all = c >= ns;
    const bool invert = all || 2u * c > ns;
    const uint32_t target = all ? 0u : (invert ? ns - c : c);
    if (all) {
      // the whole residual: no draws; forget a batch that was generated ahead
      __syncthreads();
      for (int w = tid; w < words; w += NT) S.taken[w] = 0;
      __syncthreads();
    }
    uint32_t have = 0, blk = 0;
    int batches = 0;
    bool use_spec = have_spec;
    double aw = 0.0, aw2 = 0.0;
    while (have < target) {
      if ((uint64_t)blk * 4ull >= (uint64_t)S.cap) break;
      DrawBatch B;
      if (use_spec) {
        B = spec;
        use_spec = false;
      } else {
        const uint32_t remaining = target - have;
        const int blocks = (small_batches || remaining <= 128u) ? kSmallBatchBlocks : min(NT, 256);
        make_batch(B, S, hs, blk, blocks, blk > 0, false, sm);
      }
      ++batches;
      VATT_STAMP(S.dbg, 10);
      // accept in draw order: first proposals of residual tokens, until the target is reached
      uint32_t acc = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (((B.first >> e) & 1u) && !test_bit(S.bm_f, B.tok[e])) acc |= 1u << e;
      uint32_t total;
      uint32_t pos = block_exclusive_scan<NT>((uint32_t)__popc(acc), &total, sm.scan);
      const uint32_t room = target - have;
      VATT_STAMP(S.dbg, 11);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if ((acc >> e) & 1u) {
          if (pos < room) {
            if (!invert) {
              if (have + pos < dst_cap) dst[have + pos] = (int32_t)B.tok[e];
              if (sum_w) {
                const double w = (double)__expf((B.have_sc ? B.sc[e] : S.row[B.tok[e]]) - S.m);
                aw += w;
                aw2 += w * w;
              }
            }
          } else if (invert) {
            atomicAnd(&S.taken[B.tok[e] >> 5], ~(1u << (B.tok[e] & 31)));  // drawn after the sample was complete
          }
          ++pos;
        }
      }
      have += min(total, room);
      blk += (uint32_t)B.blocks;
      VATT_STAMP(S.dbg, 12);
    }
    if (batches > 1) flags |= 2;
    __syncthreads();
    if (have < target) {
      // draw cap reached: complete with the lowest-index residual tokens not yet accepted
      flags |= 4;
      const uint32_t need = target - have;
      for (int w = tid; w < words; w += NT) S.scratch[w] = mid_mask(hs, w) & ~S.bm_f[w] & ~S.taken[w];
      __syncthreads();
      word_prefix(S.scratch, words, S.wpre, sm);
      for (int w = tid; w < words; w += NT) {
        uint32_t bits = S.scratch[w];
        uint32_t pos = S.wpre[w];
        while (bits && pos < need) {
          const uint32_t i = (uint32_t)(w << 5) + (uint32_t)(__ffs(bits) - 1);
          bits &= bits - 1u;
          if (invert) {
            atomicOr(&S.taken[i >> 5], 1u << (i & 31));
          } else {
            if (have + pos < dst_cap) dst[have + pos] = (int32_t)i;
            if (sum_w) {
              const double wt = (double)__expf(S.row[i] - S.m);
              aw += wt;
              aw2 += wt * wt;
            }
          }
          ++pos;
        }
      }
      __syncthreads();
      for (int w = tid; w < words; w += NT) S.scratch[w] = 0;
      __syncthreads();
    }
    if (invert) {
      // the sample is the residual minus the accepted tokens, in ascending order
      flags |= 1;
      for (int w = tid; w < words; w += NT) S.scratch[w] = mid_mask(hs, w) & ~S.bm_f[w] & ~S.taken[w];
      __syncthreads();
      word_prefix(S.scratch, words, S.wpre, sm);
      for (int w = tid; w < words; w += NT) {
        uint32_t bits = S.scratch[w];
        uint32_t pos = S.wpre[w];
        while (bits) {
          const int i = (w << 5) + (__ffs(bits) - 1);
          bits &= bits - 1u;
          if (pos < dst_cap) dst[pos] = i;
          if (sum_w) {
            const double wt = (double)__expf(S.row[i] - S.m);
            aw += wt;
            aw2 += wt * wt;
          }
          ++pos;
        }
      }
      __syncthreads();
      for (int w = tid; w < words; w += NT) S.scratch[w] = 0;
      __syncthreads();
    }
    if (sum_w) {
      *sum_w += aw;
      *sum_w2 += aw2;
    }
    return flags;
  }
};  // struct HeadOps

// Philox blocks of the batch that is generated ahead, before the top-k set is known.
template <int NT>
__device__ __forceinline__ int ahead_blocks(uint32_t L, int small_batches) {
  (void)L;
  return small_batches ? kSmallBatchBlocks : min(NT, 256);
}

// NT = workgroup size; EM = top-k candidate slots a thread holds (n_chunks * cand_cap <= EM * NT).
template <int NT, int EM>
__global__ __launch_bounds__(NT) void head_kernel(HeadArgs A) {
  using O = HeadOps<NT>;
  using HeadSmem = typename O::HeadSmem;
  using Sampler = typename O::Sampler;
  constexpr int SW = NT / kWave;
  extern __shared__ __align__(16) unsigned char dyn_smem[];
  __shared__ OrderedSmem<NT, EM> ord_sm;
  const int h = blockIdx.x, b = blockIdx.y;
  const int bh = b * A.Hq + h;
  const int tid = threadIdx.x;
  const int n = min(max(A.seq_lens[b], 1), A.n_max);
  const HeadSizes hs = head_sizes(n, A.sp);
  const int words_max = (A.n_max + 31) >> 5;
  const int words = (n + 31) >> 5;

  HeadSmem& sm = *reinterpret_cast<HeadSmem*>(dyn_smem);
  uint32_t* bm_f = reinterpret_cast<uint32_t*>(dyn_smem + ((sizeof(HeadSmem) + 15) & ~size_t(15)));
  uint32_t* taken0 = bm_f + words_max;
  uint32_t* taken1 = taken0 + words_max;
  uint32_t* scratch = taken1 + words_max;
  uint32_t* wpre = scratch + words_max;
  uint32_t* mail = wpre + words_max;

  const float* row = A.scores + (int64_t)bh * A.n_pad;
  int32_t* idx = A.out_idx + (int64_t)bh * A.idx_cap;
  const uint64_t seed = A.seq_seeds[b];

  VATT_STAMP(A.dbg, 0);
  // Everything the kernel needs from global memory up to the base sample is requested first, so that the
  // latencies overlap each other and the sampler work below: the head's top-k candidate slots, the chunk
  // counts and the chunk maxima.
  uint64_t tcand[EM];
  {
    const uint64_t* src = A.cand + (int64_t)bh * A.n_chunks * A.cand_cap;
    const int slots = A.n_chunks * A.cand_cap;
#pragma unroll
    for (int e = 0; e < EM; ++e) tcand[e] = (A.phase != 2) ? src[min(e * NT + tid, slots - 1)] : kInvalid;
  }
  static_assert(kMaxChunks <= 256, "one thread per chunk reads the chunk tables");
  const uint32_t my_cnt = tid < A.n_chunks ? (uint32_t)A.cand_cnt[bh * A.n_chunks + tid] : 0u;
  float m = tid < A.n_chunks ? A.chunk_max[bh * A.n_chunks + tid] : -INFINITY;
  for (int w = tid; w < words; w += NT) {
    bm_f[w] = 0;
    taken0[w] = 0;
    taken1[w] = 0;
    scratch[w] = 0;
    mail[w] = kInv32;
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
  S1.stream = 1u;
  S1.dbg = A.dbg ? A.dbg + 300 : nullptr;
  DrawBatch spec0 = {}, spec1 = {};
  const bool want0 = hs.n_s > 0 && A.phase != 2 && hs.b0 < hs.n_s;
  const bool want1 = hs.n_s > 0 && A.phase != 1;
  if (want0) O::make_batch(spec0, S0, hs, 0u, ahead_blocks<NT>(L, A.small_batches), false, true, sm);
  if (want1) O::make_batch(spec1, S1, hs, 0u, ahead_blocks<NT>(L, A.small_batches), false, false, sm);

  // chunk counts, and the head maximum from the chunk maxima
  if (tid < A.n_chunks) sm.chunk_cnt[tid] = my_cnt;
  m = wave_max(m);
  if ((tid & 63) == 0) sm.red[0][tid >> 6] = (double)m;
  __syncthreads();
  m = (float)sm.red[0][0];
#pragma unroll
  for (int w = 1; w < SW; ++w) m = fmaxf(m, (float)sm.red[0][w]);
  __syncthreads();
  S0.m = m;
  S1.m = m;

  VATT_STAMP(A.dbg, 1);
  double acc_f = 0.0;  // this thread's share of D_f = sum over I_f of exp(s_i - m)
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
      // candidates are stored chunk by chunk in ascending token order: ascending slot order is ascending
      // token order, and a chosen candidate carries its score in its high word
      uint32_t take = 0;
#pragma unroll
      for (int e = 0; e < EM; ++e) {
        const bool in = (((uint64_t)xh[e] << 32) | xl[e]) <= T;
        take |= (in ? 1u : 0u) << e;
        if (in) {
          O::mark_bit(bm_f, min(xl[e], (uint32_t)(n - 1)));
          acc_f += (double)__expf(float_from_order_key(~xh[e]) - m);
        }
      }
      uint32_t pos[EM], taken_n;
      ordered_positions<NT, EM>(take, pos, &taken_n, ord_sm);
#pragma unroll
      for (int e = 0; e < EM; ++e)
        if (((take >> e) & 1u) && pos[e] < (uint32_t)A.k_max) idx[A.seg_topk + pos[e]] = (int32_t)xl[e];
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
      const int f = O::draw_sample(S0, hs, (uint32_t)hs.b0, spec0, want0, A.small_batches,
                                   idx + A.seg_base, (uint32_t)A.b0_max, &acc_w, &acc_w2, sm);
      flags |= ((f & 1) ? kFlagBaseComplement : 0) | ((f & 2) ? kFlagBaseBatches : 0) | ((f & 4) ? kFlagDrawCap : 0);
      VATT_STAMP(A.dbg, 5);
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
  VATT_STAMP(A.dbg, 6);
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
    const int f = O::draw_sample(S1, hs, (uint32_t)bfin, spec1, want1, A.small_batches,
                                 idx + A.seg_dyn, (uint32_t)A.b_max, nullptr, nullptr, sm);
    flags |= ((f & 1) ? kFlagDynComplement : 0) | ((f & 2) ? kFlagDynBatches : 0) | ((f & 4) ? kFlagDrawCap : 0);
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
// The instantiation for a plan: (workgroup size, top-k slots per thread).
HeadKernel head_kernel_for(const Plan& pl) {
  const int64_t cands = (int64_t)pl.n_chunks * pl.cand_cap;
  if (pl.head_threads == 256) return cands <= 16 * 256 ? head_kernel<256, 16> : head_kernel<256, 32>;
  return head_kernel<1024, 32>;
}

}  // namespace

hipError_t set_kernel_attributes(const Plan& pl) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(head_kernel_for(pl)),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)pl.head_lds_bytes);
}

size_t head_kernel_lds_bytes(int n_max, int head_threads) {
  const size_t words_max = (size_t)(n_max + 31) >> 5;
  const size_t fixed = head_threads == 256 ? sizeof(HeadOps<256>::HeadSmem) : sizeof(HeadOps<1024>::HeadSmem);
  return ((fixed + 15) & ~size_t(15)) + 6 * words_max * sizeof(uint32_t);
}

hipError_t launch_stage1(const Plan& pl, const int32_t* seq_lens, void* ws, hipStream_t st) {
  const vatt_params& p = pl.p;
  char* w = static_cast<char*>(ws);
  Stage1Args A;
  A.scores = reinterpret_cast<const float*>(w + pl.off_scores);
  A.seq_lens = seq_lens;
  A.chunk_max = reinterpret_cast<float*>(w + pl.off_chunk_max);
  A.cand = reinterpret_cast<uint64_t*>(w + pl.off_cand);
  A.cand_cnt = reinterpret_cast<int32_t*>(w + pl.off_cand_cnt);
  A.sp = pl.sel;
  A.n_pad = pl.n_pad;
  A.n_max = p.n_max;
  A.Hq = p.n_q_heads;
  A.chunk_len = pl.chunk_len;
  A.n_chunks = pl.n_chunks;
  A.cand_cap = pl.cand_cap;
  A.dbg = reinterpret_cast<unsigned long long*>(w + pl.off_debug);
  dim3 grid(pl.n_chunks, p.n_q_heads, p.batch);
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
  A.target = p.target;
  A.phase = phase;
  A.small_batches = pl.sampler_small_batches;
  A.draw_cap = pl.sampler_draw_cap;
  A.vstat_splits = pl.vstat_splits;
  A.head_dim = p.head_dim;
  A.k_max = pl.k_max;
  A.b0_max = pl.b0_max;
  A.b_max = pl.b_max;
  A.dbg = reinterpret_cast<unsigned long long*>(w + pl.off_debug) + 64;
  hipLaunchKernelGGL(head_kernel_for(pl), dim3(p.n_q_heads, p.batch), dim3(pl.head_threads), pl.head_lds_bytes, st, A);
  return hipGetLastError();
}

}  // namespace vatt
