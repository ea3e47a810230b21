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
//   chunk_topk_kernel  one workgroup per (chunk of the score row, head): keeps the chunk in registers,
//                      radix-selects the chunk's own top-k and writes those composites as candidates
//                      (any member of the global top-k is in its chunk's top-k), plus the chunk maximum.
//   head_kernel        one workgroup per head: merges the candidates into the exact top-k, builds the
//                      membership bitmap, draws the base sample, computes the statistics and the budget
//                      of Algorithm 2, draws the final sample, and writes every index list in ascending
//                      token order.
#include "vatt_internal.h"

namespace vatt {
namespace {

constexpr uint64_t kInvalid = ~0ull;

// ---------------------------------------------------------------------------
// Workgroup-wide exclusive scan of one uint32 per thread.
// ---------------------------------------------------------------------------
template <int THREADS>
struct BlockScan {
  static constexpr int WAVES = THREADS / kWave;
  struct Smem {
    uint32_t wave_total[WAVES];
  };
  // Returns the exclusive prefix of v; *total gets the workgroup sum.  Ends with a barrier.
  __device__ static uint32_t exclusive(uint32_t v, uint32_t* total, Smem& sm) {
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
    for (int w = 0; w < WAVES; ++w) {
      const uint32_t t = sm.wave_total[w];
      if (w < wave) base += t;
      tot += t;
    }
    *total = tot;
    return base + incl - v;
  }
};

// ---------------------------------------------------------------------------
// Workgroup select: threshold T such that exactly c of the valid composites held in registers
// (E per thread, kInvalid = absent) are <= T.  Requires 1 <= c <= number of valid composites.
// Most-significant-digit-first radix descent with 4-bit digits, counted in registers; once the
// bucket holding the answer has at most SMALL members they are ranked directly in LDS.
// ---------------------------------------------------------------------------
template <int THREADS, int E>
struct BlockSelect {
  static constexpr int WAVES = THREADS / kWave;
  static constexpr int SMALL = 256;
  struct Smem {
    uint32_t wave_cnt[WAVES][16];
    uint32_t total[16];
    uint64_t list[SMALL];
    uint32_t list_n;
    uint64_t result;
  };

  __device__ static __forceinline__ uint64_t spread_bytes(uint32_t x) {
    return (uint64_t)(x & 0xffu) | ((uint64_t)(x & 0xff00u) << 8) | ((uint64_t)(x & 0xff0000u) << 16) |
           ((uint64_t)(x & 0xff000000u) << 24);
  }

  __device__ static uint64_t run(const uint64_t (&x)[E], int e_used, uint32_t c, Smem& sm) {
    static_assert(E <= 255, "per-thread digit counters are 8 bits wide");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint64_t prefix = 0, mask = 0;
    uint32_t r = c;
    for (int shift = 60; shift >= 0; shift -= 4) {
      uint64_t lo = 0, hi = 0;  // eight 8-bit counters each: digits 0-7 and 8-15
#pragma unroll
      for (int e = 0; e < E; ++e) {
        if (e < e_used) {
          const uint64_t v = x[e];
          if ((v & mask) == prefix) {
            const uint32_t d = (uint32_t)(v >> shift) & 15u;
            const uint64_t inc = 1ull << ((d & 7u) * 8u);
            if (d & 8u) hi += inc; else lo += inc;
          }
        }
      }
      // widen to 16-bit fields (a wave holds at most 64 * E <= 16320 per digit) and add across the wave
      uint64_t a0 = wave_sum(spread_bytes((uint32_t)lo));
      uint64_t a1 = wave_sum(spread_bytes((uint32_t)(lo >> 32)));
      uint64_t a2 = wave_sum(spread_bytes((uint32_t)hi));
      uint64_t a3 = wave_sum(spread_bytes((uint32_t)(hi >> 32)));
      if (lane == 0) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          sm.wave_cnt[wave][j] = (uint32_t)(a0 >> (16 * j)) & 0xffffu;
          sm.wave_cnt[wave][4 + j] = (uint32_t)(a1 >> (16 * j)) & 0xffffu;
          sm.wave_cnt[wave][8 + j] = (uint32_t)(a2 >> (16 * j)) & 0xffffu;
          sm.wave_cnt[wave][12 + j] = (uint32_t)(a3 >> (16 * j)) & 0xffffu;
        }
      }
      __syncthreads();
      if (tid < 16) {
        uint32_t t = 0;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) t += sm.wave_cnt[w][tid];
        sm.total[tid] = t;
      }
      __syncthreads();
      uint32_t cum = 0, below = 0, active = 0, dsel = 15;
      bool found = false;
#pragma unroll
      for (int d = 0; d < 16; ++d) {
        const uint32_t t = sm.total[d];
        if (!found && cum + t >= r) {
          found = true;
          dsel = d;
          below = cum;
          active = t;
        }
        cum += t;
      }
      r -= below;
      prefix |= (uint64_t)dsel << shift;
      mask |= 15ull << shift;
      if (active == r) {
        // the whole bucket is taken: every composite under this prefix is <= prefix | ones
        return prefix | ((1ull << shift) - 1ull);
      }
      if (active <= (uint32_t)SMALL) {
        if (tid == 0) sm.list_n = 0;
        __syncthreads();
#pragma unroll
        for (int e = 0; e < E; ++e) {
          if (e < e_used && (x[e] & mask) == prefix) {
            const uint32_t pos = atomicAdd(&sm.list_n, 1u);
            if (pos < (uint32_t)SMALL) sm.list[pos] = x[e];
          }
        }
        __syncthreads();
        if ((uint32_t)tid < active) {
          const uint64_t v = sm.list[tid];
          uint32_t rank = 0;
          for (uint32_t j = 0; j < active; ++j) rank += (sm.list[j] < v) ? 1u : 0u;
          if (rank == r - 1u) sm.result = v;
        }
        __syncthreads();
        const uint64_t res = sm.result;
        __syncthreads();
        return res;
      }
    }
    return prefix;
  }
};

// ---------------------------------------------------------------------------
// Chunk-level top-k candidates.
// ---------------------------------------------------------------------------
template <int THREADS>
__global__ __launch_bounds__(THREADS) void chunk_topk_kernel(const float* __restrict__ scores, int n_pad, int n_max,
                                                             const int32_t* __restrict__ seq_lens, SelectParams sp,
                                                             int Hq, int chunk_len, int n_chunks, int cand_cap,
                                                             float* __restrict__ chunk_max,
                                                             uint64_t* __restrict__ cand,
                                                             int32_t* __restrict__ cand_cnt) {
  constexpr int E = kSelElems;
  using Sel = BlockSelect<THREADS, E>;
  __shared__ typename Sel::Smem sel_sm;
  __shared__ float s_wmax[THREADS / kWave];
  __shared__ uint32_t s_out;

  const int chunk = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int bh = b * Hq + h;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = min(max(seq_lens[b], 1), n_max);
  const HeadSizes hs = head_sizes(n, sp);
  const int lo = chunk * chunk_len;
  const int hi = min(lo + chunk_len, n);
  const int slot = bh * n_chunks + chunk;
  if (lo >= n) {
    if (tid == 0) {
      cand_cnt[slot] = 0;
      chunk_max[slot] = -INFINITY;
    }
    return;
  }
  const float* row = scores + (int64_t)bh * n_pad;
  uint64_t x[E];
  float mx = -INFINITY;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int i = lo + e * THREADS + tid;
    x[e] = kInvalid;
    if (i < hi) {
      const float s = row[i];
      mx = fmaxf(mx, s);
      if (i >= hs.mid_lo && i < hs.mid_hi) x[e] = ((uint64_t)(~float_order_key(s)) << 32) | (uint32_t)i;
    }
  }
  mx = wave_max(mx);
  if (lane == 0) s_wmax[wave] = mx;
  if (tid == 0) s_out = 0;
  __syncthreads();
  if (tid == 0) {
    float t = s_wmax[0];
    for (int w = 1; w < THREADS / kWave; ++w) t = fmaxf(t, s_wmax[w]);
    chunk_max[slot] = t;
  }
  const int vlo = max(lo, hs.mid_lo), vhi = min(hi, hs.mid_hi);
  const int nvalid = max(vhi - vlo, 0);
  const int c = min(min(hs.k, nvalid), cand_cap);
  if (c == 0) {
    if (tid == 0) cand_cnt[slot] = 0;
    return;
  }
  const int e_used = min(E, (hi - lo + THREADS - 1) / THREADS);
  const uint64_t T = (c == nvalid) ? (kInvalid - 1ull) : Sel::run(x, e_used, (uint32_t)c, sel_sm);
  uint64_t* out = cand + (int64_t)slot * cand_cap;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    if (e < e_used && x[e] <= T) {
      const uint32_t pos = atomicAdd(&s_out, 1u);
      if (pos < (uint32_t)cand_cap) out[pos] = x[e];
    }
  }
  if (tid == 0) cand_cnt[slot] = c;
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
  int32_t* gather_cnt;
  const double* vstat_part;  // [B*Hq][vstat_splits][2d+2] (targets N, SDPA)
  int32_t* out_idx;
  int32_t* out_counts;
  double* out_budget_raw;
  float* out_stats;
  SelectParams sp;
  double z_half, z_quarter, eps, cap_frac;
  int64_t seg_topk, seg_base, seg_dyn, seg_sink, seg_win;
  int64_t idx_cap;
  int n_pad, n_max, Hq, n_chunks, cand_cap, target, phase, force_slow, vstat_splits, head_dim;
  int k_max, b0_max, b_max;
};

constexpr int HT = kHeadThreads;
constexpr int HW = HT / kWave;
constexpr int EL = kListCap / HT;  // list composites per thread

struct HeadSmem {
  BlockSelect<HT, kSelElems>::Smem sel_big;
  BlockSelect<HT, EL>::Smem sel_list;
  BlockScan<HT>::Smem scan;
  uint64_t list[kListCap];
  uint32_t hist[256];
  double red[HW];
  uint32_t list_n, sure_n;
  uint32_t u_a, u_b, u_c;
  uint64_t u64_a;
  double d_a;
  float f_a;
  int32_t b_final;
};

__device__ __forceinline__ double block_sum(double v, HeadSmem& sm) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm.red[threadIdx.x >> 6] = v;
  __syncthreads();
  double t = 0.0;
#pragma unroll
  for (int w = 0; w < HW; ++w) t += sm.red[w];
  return t;
}

__device__ __forceinline__ bool bit_test(const uint32_t* bm, int i) { return (bm[i >> 5] >> (i & 31)) & 1u; }

// Token read back from an index list, forced into [0, n): a list entry can never address outside the row.
__device__ __forceinline__ int list_tok(const int32_t* idx, int64_t pos, int n) { return min(max(idx[pos], 0), n - 1); }

// Write the set bits of bm[0, n) as ascending token indices to dst; returns their number.
__device__ uint32_t compact_bitmap(const uint32_t* bm, int n, int32_t* dst, uint32_t dst_cap, HeadSmem& sm) {
  const int words = (n + 31) >> 5;
  const int wpt = (words + HT - 1) / HT;
  const int w0 = threadIdx.x * wpt;
  uint32_t cnt = 0;
  for (int w = w0; w < min(w0 + wpt, words); ++w) cnt += __popc(bm[w]);
  uint32_t total;
  uint32_t pos = BlockScan<HT>::exclusive(cnt, &total, sm.scan);
  for (int w = w0; w < min(w0 + wpt, words); ++w) {
    uint32_t bits = bm[w];
    while (bits) {
      const int bpos = __ffs(bits) - 1;
      bits &= bits - 1u;
      if (pos < dst_cap) dst[pos] = (w << 5) + bpos;
      ++pos;
    }
  }
  return total;
}

// One Philox block = keys of tokens 4j .. 4j+3.
__device__ __forceinline__ Philox4 token_block_keys(uint32_t j, uint32_t stream, uint32_t head, uint64_t seed) {
  return philox4x32_10(j, stream, head, 0u, (uint32_t)seed, (uint32_t)(seed >> 32));
}

// Residual tokens of the 4-token block j as a 4-bit mask.
__device__ __forceinline__ uint32_t residual_nibble(const uint32_t* bm_f, const HeadSizes& hs, int j) {
  const int i0 = j << 2;
  uint32_t in_mid = 0;
#pragma unroll
  for (int e = 0; e < 4; ++e) in_mid |= ((i0 + e >= hs.mid_lo && i0 + e < hs.mid_hi) ? 1u : 0u) << e;
  const uint32_t taken = (bm_f[i0 >> 5] >> (i0 & 31)) & 15u;
  return in_mid & ~taken;
}

// Mark in bm_s the c residual tokens with the smallest (key, token) of the given stream.
// bm_s must be all zero on entry.  Returns 1 if the slow exact path was used.
__device__ int sample_residual(uint32_t* bm_s, const uint32_t* bm_f, const HeadSizes& hs, uint32_t c,
                               uint32_t stream, uint32_t head, uint64_t seed, int force_slow, HeadSmem& sm) {
  const int tid = threadIdx.x;
  const int j_lo = hs.mid_lo >> 2, j_hi = (hs.mid_hi + 3) >> 2;  // Philox blocks that touch the middle region
  const int words = (hs.n + 31) >> 5;
  if (c == 0) return 0;
  if (c >= (uint32_t)hs.n_s) {
    // the whole residual: no keys needed
    for (int w = tid; w < words; w += HT) {
      uint32_t m = 0;
      const int i0 = w << 5;
      if (i0 + 31 >= hs.mid_lo && i0 < hs.mid_hi) {
        const int a = max(hs.mid_lo - i0, 0), bnd = min(hs.mid_hi - i0, 32);
        m = (bnd >= 32 ? 0xffffffffu : ((1u << bnd) - 1u)) & ~((1u << a) - 1u);
        if (a >= 32) m = 0;
      }
      bm_s[w] = m & ~bm_f[w];
    }
    __syncthreads();
    return 0;
  }

  bool done = false;
  if (!force_slow) {
    // Fast path: keys are uniform, so the c-th smallest sits near c / n_s * 2^32.  Tokens with a key
    // below L are certainly in, tokens in [L, U) are listed and ranked exactly; the guess is verified
    // by counting and otherwise discarded.
    const double ns = (double)hs.n_s;
    const double sd = sqrt((double)c * (1.0 - (double)c / ns)) + 1.0;
    const double c_lo = fmax((double)c - 6.0 * sd - 8.0, 0.0);
    const double c_hi = fmin((double)c + 6.0 * sd + 8.0, ns);
    const uint64_t Lq = (uint64_t)floor(c_lo / ns * 4294967296.0);
    const uint64_t Uq = (c_hi >= ns) ? 4294967296ull : (uint64_t)ceil(c_hi / ns * 4294967296.0);
    if (tid == 0) {
      sm.list_n = 0;
      sm.sure_n = 0;
    }
    __syncthreads();
    uint32_t my_sure = 0;
    for (int j = j_lo + tid; j < j_hi; j += HT) {
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
    my_sure = wave_sum(my_sure);
    if ((tid & 63) == 0 && my_sure) atomicAdd(&sm.sure_n, my_sure);
    __syncthreads();
    const uint32_t sure = sm.sure_n, listed = sm.list_n;
    if (sure <= c && sure + listed >= c && listed <= (uint32_t)kListCap) {
      const uint32_t need = c - sure;
      if (need > 0) {
        uint64_t x[EL];
#pragma unroll
        for (int e = 0; e < EL; ++e) {
          const uint32_t p = e * HT + tid;
          x[e] = p < listed ? sm.list[p] : kInvalid;
        }
        const uint64_t T = (need == listed) ? (kInvalid - 1ull)
                                            : BlockSelect<HT, EL>::run(x, EL, need, sm.sel_list);
#pragma unroll
        for (int e = 0; e < EL; ++e) {
          if (x[e] <= T) {
            const uint32_t i = (uint32_t)x[e];
            atomicOr(&bm_s[i >> 5], 1u << (i & 31));
          }
        }
      }
      done = true;
    } else {
      for (int w = tid; w < words; w += HT) bm_s[w] = 0;  // discard the guess
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
    for (int d = tid; d < 256; d += HT) sm.hist[d] = 0;
    __syncthreads();
    for (int j = j_lo + tid; j < j_hi; j += HT) {
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
      for (int j = j_lo + tid; j < j_hi; j += HT) {
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
      uint64_t x[EL];
#pragma unroll
      for (int e = 0; e < EL; ++e) {
        const uint32_t p = e * HT + tid;
        x[e] = p < listed ? sm.list[p] : kInvalid;
      }
      T = BlockSelect<HT, EL>::run(x, EL, r, sm.sel_list);
      have_T = true;
    }
    __syncthreads();
  }
  if (!have_T) T = prefix;
  for (int j = j_lo + tid; j < j_hi; j += HT) {
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

__global__ __launch_bounds__(HT) void head_kernel(HeadArgs A) {
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

  for (int w = tid; w < words; w += HT) {
    bm_f[w] = 0;
    bm_s[w] = 0;
  }
  // head maximum from the chunk maxima
  float m = -INFINITY;
  for (int c = tid; c < A.n_chunks; c += HT) m = fmaxf(m, A.chunk_max[bh * A.n_chunks + c]);
  m = wave_max(m);
  __syncthreads();
  if ((tid & 63) == 0) sm.red[tid >> 6] = (double)m;
  __syncthreads();
  m = (float)sm.red[0];
#pragma unroll
  for (int w = 1; w < HW; ++w) m = fmaxf(m, (float)sm.red[w]);
  __syncthreads();

  // ---- I_t (Algorithm 1, line 3) ----
  if (A.phase != 2) {
    if (hs.k > 0) {
      uint64_t x[kSelElems];
      // gather the chunk candidates: chunk c contributes cand_cnt[c] composites
      uint32_t total = 0;
      for (int c = 0; c < A.n_chunks; ++c) total += (uint32_t)A.cand_cnt[bh * A.n_chunks + c];
      const int e_used = min(kSelElems, (int)((total + HT - 1) / HT));
#pragma unroll
      for (int e = 0; e < kSelElems; ++e) x[e] = kInvalid;
      {
        uint32_t base = 0;
        for (int c = 0; c < A.n_chunks; ++c) {
          const uint32_t cnt = (uint32_t)A.cand_cnt[bh * A.n_chunks + c];
          const uint64_t* src = A.cand + ((int64_t)bh * A.n_chunks + c) * A.cand_cap;
          // flat position p = base + t lives in register slot p / HT of thread p % HT
#pragma unroll
          for (int e = 0; e < kSelElems; ++e) {
            const uint32_t p = (uint32_t)e * HT + tid;
            if (p >= base && p < base + cnt) x[e] = src[p - base];
          }
          base += cnt;
        }
      }
      const uint64_t T = ((uint32_t)hs.k >= total) ? (kInvalid - 1ull)
                                                   : BlockSelect<HT, kSelElems>::run(x, e_used, (uint32_t)hs.k, sm.sel_big);
#pragma unroll
      for (int e = 0; e < kSelElems; ++e) {
        if (e < e_used && x[e] <= T) {
          const uint32_t i = (uint32_t)x[e];
          atomicOr(&bm_f[i >> 5], 1u << (i & 31));
        }
      }
      __syncthreads();
      compact_bitmap(bm_f, n, idx + A.seg_topk, (uint32_t)A.k_max, sm);
    }
    for (int i = tid; i < hs.n_sink; i += HT) idx[A.seg_sink + i] = i;
    for (int i = tid; i < hs.n_win; i += HT) idx[A.seg_win + i] = hs.mid_hi + i;
  } else {
    // phase 2: rebuild the top-k bitmap from the list written in phase 1
    for (int t = tid; t < hs.k; t += HT) {
      const uint32_t i = (uint32_t)list_tok(idx, A.seg_topk + t, n);
      atomicOr(&bm_f[i >> 5], 1u << (i & 31));
    }
  }
  __syncthreads();

  // ---- I_bs (Algorithm 2, line 1) ----
  int flags = 0;
  if (A.phase != 2 && hs.n_s > 0) {
    sample_residual(bm_s, bm_f, hs, (uint32_t)hs.b0, 0u, (uint32_t)h, seed, A.force_slow, sm);
    compact_bitmap(bm_s, n, idx + A.seg_base, (uint32_t)A.b0_max, sm);
    __syncthreads();
    for (int w = tid; w < words; w += HT) bm_s[w] = 0;
    __syncthreads();
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
    }
    return;
  }

  // ---- statistics (Algorithm 2, get-stats): w_i = exp(s_i - m) ----
  double D_f = 0.0;
  {
    double acc = 0.0;
    for (int i = tid; i < hs.n_sink; i += HT) acc += (double)expf(row[i] - m);
    for (int i = tid; i < hs.n_win; i += HT) acc += (double)expf(row[hs.mid_hi + i] - m);
    for (int t = tid; t < hs.k; t += HT) acc += (double)expf(row[list_tok(idx, A.seg_topk + t, n)] - m);
    D_f = block_sum(acc, sm);
  }
  double w_bar = 0.0, sigma2 = 0.0, b_star = 0.0, tr_sigma = 0.0, nhat_sq = 0.0;
  int bfin = 0;
  if (hs.n_s > 0) {
    double acc = 0.0;
    for (int t = tid; t < hs.b0; t += HT) acc += (double)expf(row[list_tok(idx, A.seg_base + t, n)] - m);
    w_bar = block_sum(acc, sm) / (double)hs.b0;
    acc = 0.0;
    for (int t = tid; t < hs.b0; t += HT) {
      const double dlt = (double)expf(row[list_tok(idx, A.seg_base + t, n)] - m) - w_bar;
      acc += dlt * dlt;
    }
    const double ss = block_sum(acc, sm);
    sigma2 = hs.b0 > 1 ? ss / (double)(hs.b0 - 1) : 0.0;
    const double ns = (double)hs.n_s;
    const double D_hat = D_f + ns * w_bar;
    const double rho_D = ns * sqrt(sigma2) / D_hat;
    double rho_N = 0.0;
    if (A.target != VATT_TARGET_D) {
      // numerator statistics from the V pass: per split {N_f[d], R1[d], R2, pad}
      const int d = A.head_dim;
      const int stride = 2 * d + 2;
      const double* vp = A.vstat_part + (int64_t)bh * A.vstat_splits * stride;
      double nh2 = 0.0, r1sq = 0.0, r2 = 0.0;
      if (tid < d) {
        double nf = 0.0, r1 = 0.0;
        for (int s = 0; s < A.vstat_splits; ++s) {
          nf += vp[s * stride + tid];
          r1 += vp[s * stride + d + tid];
        }
        const double nh = nf + ns * r1 / (double)hs.b0;
        nh2 = nh * nh;
        r1sq = r1 * r1;
      }
      if (tid == 0)
        for (int s = 0; s < A.vstat_splits; ++s) r2 += vp[s * stride + 2 * d];
      nhat_sq = block_sum(nh2, sm);
      const double r1n = block_sum(r1sq, sm);
      const double r2t = block_sum(r2, sm);
      tr_sigma = hs.b0 > 1 ? fmax(r2t - r1n / (double)hs.b0, 0.0) / (double)(hs.b0 - 1) : 0.0;
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
    if (tid == 0) {
      if (A.out_stats) {
        float* st = A.out_stats + (int64_t)bh * 4;
        st[0] = (float)D_hat;
        st[1] = (float)sigma2;
        st[2] = (float)tr_sigma;
        st[3] = (float)nhat_sq;
      }
    }
  } else if (tid == 0 && A.out_stats) {
    float* st = A.out_stats + (int64_t)bh * 4;
    st[0] = (float)D_f;
    st[1] = st[2] = st[3] = 0.f;
  }

  // ---- I_dyn (Algorithm 1, line 7) ----
  if (bfin > 0) {
    flags |= sample_residual(bm_s, bm_f, hs, (uint32_t)bfin, 1u, (uint32_t)h, seed, A.force_slow, sm);
    compact_bitmap(bm_s, n, idx + A.seg_dyn, (uint32_t)A.b_max, sm);
  }
  if (tid == 0) {
    int32_t* c = A.out_counts + (int64_t)bh * 8;
    c[0] = hs.n_sink;
    c[1] = hs.n_win;
    c[2] = hs.k;
    c[3] = hs.n_s > 0 ? hs.b0 : 0;
    c[4] = bfin;
    c[5] = hs.n_s;
    c[6] = n;
    c[7] = flags;
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
    A.gather_cnt[bh] = 0;
  }
}

}  // namespace

hipError_t set_kernel_attributes(const Plan& pl) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(head_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)pl.head_lds_bytes);
}

size_t head_kernel_lds_bytes(int n_max) {
  const size_t words_max = (size_t)(n_max + 31) >> 5;
  return ((sizeof(HeadSmem) + 15) & ~size_t(15)) + 2 * words_max * sizeof(uint32_t);
}

hipError_t launch_chunk_topk(const Plan& pl, const int32_t* seq_lens, void* ws, hipStream_t st) {
  const vatt_params& p = pl.p;
  char* w = static_cast<char*>(ws);
  dim3 grid(pl.n_chunks, p.n_q_heads, p.batch);
  const float* scores = reinterpret_cast<const float*>(w + pl.off_scores);
  float* cmax = reinterpret_cast<float*>(w + pl.off_chunk_max);
  uint64_t* cand = reinterpret_cast<uint64_t*>(w + pl.off_cand);
  int32_t* ccnt = reinterpret_cast<int32_t*>(w + pl.off_cand_cnt);
  if (pl.chunk_threads == kChunkThreadsSmall) {
    hipLaunchKernelGGL((chunk_topk_kernel<kChunkThreadsSmall>), grid, dim3(kChunkThreadsSmall), 0, st, scores,
                       pl.n_pad, p.n_max, seq_lens, pl.sel, p.n_q_heads, pl.chunk_len, pl.n_chunks, pl.cand_cap,
                       cmax, cand, ccnt);
  } else {
    hipLaunchKernelGGL((chunk_topk_kernel<kChunkThreadsLarge>), grid, dim3(kChunkThreadsLarge), 0, st, scores,
                       pl.n_pad, p.n_max, seq_lens, pl.sel, p.n_q_heads, pl.chunk_len, pl.n_chunks, pl.cand_cap,
                       cmax, cand, ccnt);
  }
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
  A.gather_cnt = reinterpret_cast<int32_t*>(w + pl.off_gather_cnt);
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
  A.target = p.target;
  A.phase = phase;
  A.force_slow = pl.force_slow_sampler;
  A.vstat_splits = pl.vstat_splits;
  A.head_dim = p.head_dim;
  A.k_max = pl.k_max;
  A.b0_max = pl.b0_max;
  A.b_max = pl.b_max;
  hipLaunchKernelGGL(head_kernel, dim3(p.n_q_heads, p.batch), dim3(HT), pl.head_lds_bytes, st, A);
  return hipGetLastError();
}

}  // namespace vatt
