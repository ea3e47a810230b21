// The sampler of Algorithm 1 and Algorithm 2 as device code shared by the selection kernels and by the score
// kernel (which can make the first batch of draws of every head while it streams K): sequential uniform draws
// from the middle region (Philox4x32-10 words, unbiased multiply-and-reject mapping), skipping top-k members and
// tokens drawn before; the first c accepted tokens are the sample.  The draw sequence is processed in batches:
// all draws of a batch are generated at once, repeated tokens are resolved to their earliest draw, and a
// prefix count in draw order finds where the sample is complete; the result equals the sequential procedure
// bit for bit.
#pragma once

#include "vatt_dev.h"

namespace vatt {

constexpr uint32_t kInv32 = 0xffffffffu;

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

// Where an accepted token goes: into the index list in global memory (dst, for the workgroup that writes the
// outputs) and, when a workgroup gathers its own share of the list (fused gather), every 2^shift-th entry into
// an LDS list.
struct Emit {
  int32_t* dst;
  uint32_t dst_cap;
  uint32_t* lds;      // nullptr: no LDS list
  uint32_t lds_cap;
  uint32_t shift, split;
  bool global;
  float* sc_dst;      // nullptr, or where the scores of the listed tokens go when the batch has them at hand
};
__device__ __forceinline__ void emit_tok(const Emit& E, uint32_t p, int32_t tok) {
  if (E.global && p < E.dst_cap) E.dst[p] = tok;
  if (E.lds && (p & ((1u << E.shift) - 1u)) == E.split && (p >> E.shift) < E.lds_cap) E.lds[p >> E.shift] = (uint32_t)tok;
}
__device__ __forceinline__ Emit emit_to(int32_t* dst, uint32_t dst_cap) {
  Emit E;
  E.dst = dst;
  E.dst_cap = dst_cap;
  E.lds = nullptr;
  E.lds_cap = 0;
  E.shift = 0;
  E.split = 0;
  E.global = true;
  E.sc_dst = nullptr;
  return E;
}

constexpr int kSmallBatchBlocks = 64;  // Philox blocks of a small batch (256 draws)

// flag bits of out_counts[7]
constexpr int kFlagBaseComplement = 1, kFlagDynComplement = 2, kFlagBaseBatches = 4, kFlagDynBatches = 8,
              kFlagDrawCap = 16, kFlagTopkGeneral = 32, kFlagBaseFromCache = 64;

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
    BlockScanSmem<NT> scan;
    double red[3][SW];
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
  // Bit e of the result: the bitmap bit of tok[e].  All four words are read before any is used (a test per token
  // behind a condition compiles to four LDS round trips one after the other); every token has to be a valid one.
  static __device__ __forceinline__ uint32_t test_bits4(const uint32_t* bm, const uint32_t (&tok)[4]) {
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) w[e] = bm[tok[e] >> 5];
    uint32_t r = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) r |= ((w[e] >> (tok[e] & 31)) & 1u) << e;
    return r;
  }

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
    uint32_t stream, head, query;
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
  //
  // lt: the Philox block (relative to blk0) this thread generates, normally its thread index.  Two streams can
  // share one call, each thread working for one of them (its own S, with bitmaps, scratch and mail of that
  // stream, and lt counted inside the stream's group of threads): the barriers are common, the rest is per
  // thread.
  static __device__ __forceinline__ void make_batch(DrawBatch& B, const Sampler& S, const HeadSizes& hs, uint32_t blk0, int blocks,
                                    bool check_prev, bool load_scores, HeadSmem& sm, int lt) {
    const int tid = lt;
    B.blocks = blocks;
    B.ok = 0;
    B.first = 0;
    B.have_sc = load_scores;
    VATT_STAMP(S.dbg, 0);
    if (tid >= 0 && tid < blocks) {
      const Philox4 ph = philox4x32_10(blk0 + (uint32_t)tid, S.stream, S.head, S.query, (uint32_t)S.seed,
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
    // (the four marks go out together: a void draw ORs in nothing)
    uint32_t lose = 0, old[4] = {0u, 0u, 0u, 0u};
    if (B.ok) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        old[e] = atomicOr(&S.taken[B.tok[e] >> 5], ((B.ok >> e) & 1u) << (B.tok[e] & 31));
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t bit = ((B.ok >> e) & 1u) << (B.tok[e] & 31);
      if (old[e] & bit) {
        lose |= 1u << e;
        atomicOr(&S.scratch[B.tok[e] >> 5], bit);
      }
    }
    __syncthreads();
    VATT_STAMP(S.dbg, 2);
    // draws whose token is proposed more than once in this batch
    uint32_t unresolved = B.ok & test_bits4(S.scratch, B.tok);
    uint32_t later = 0;
    for (;;) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if ((unresolved >> e) & 1u) atomicMin(&S.mail[B.tok[e] >> 5], ((uint32_t)(tid * 4 + e) << 5) | (B.tok[e] & 31));
      if (threadIdx.x == 0) sm.again = 0;
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
                                    int small_batches, const Emit& E, double* sum_w,
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
        const int blocks = (small_batches || remaining <= 128u) ? kSmallBatchBlocks
                                                                  : (remaining > 1024u ? min(NT, 1024) : min(NT, 256));
        make_batch(B, S, hs, blk, blocks, blk > 0, false, sm, (int)threadIdx.x);
      }
      ++batches;
      VATT_STAMP(S.dbg, 10);
      // accept in draw order: first proposals of residual tokens, until the target is reached
      const uint32_t acc = B.first & ~test_bits4(S.bm_f, B.tok);
      uint32_t total;
      uint32_t pos = block_exclusive_scan<NT>((uint32_t)__popc(acc), &total, sm.scan);
      const uint32_t room = target - have;
      VATT_STAMP(S.dbg, 11);
      // (written without nested per-draw branches: a divergent branch inside an unrolled loop serialises it)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool a = (acc >> e) & 1u;
        const bool take = a && pos < room;
        if (!invert) {
          if (take) emit_tok(E, have + pos, (int32_t)B.tok[e]);
          if (take && E.sc_dst && B.have_sc && have + pos < E.dst_cap) E.sc_dst[have + pos] = B.sc[e];
          if (sum_w) {
            const float sc = B.have_sc ? B.sc[e] : (take ? S.row[B.tok[e]] : 0.f);
            const double w = take ? (double)__expf(sc - S.m) : 0.0;
            aw += w;
            aw2 += w * w;
          }
        } else if (a && !take) {
          atomicAnd(&S.taken[B.tok[e] >> 5], ~(1u << (B.tok[e] & 31)));  // drawn after the sample was complete
        }
        pos += a ? 1u : 0u;
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
            emit_tok(E, have + pos, (int32_t)i);
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
          emit_tok(E, pos, i);
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

  // Rewrites a token list this workgroup wrote at dst (count distinct tokens below n) in ascending order:
  // the tokens are marked in the all-zero bitmap `scratch`, counted by bitmap word, and written back by
  // position; `scratch` is left all zero.  (An option of the plans: rows gathered in ascending order.)
  static __device__ void sort_ascending(int32_t* dst, uint32_t count, uint32_t* scratch, uint32_t* wpre, int n,
                                        HeadSmem& sm) {
    const int tid = threadIdx.x;
    const int words = (n + 31) >> 5;
    __syncthreads();  // the list is complete (global memory is coherent inside a workgroup)
    for (uint32_t t = tid; t < count; t += NT) mark_bit(scratch, (uint32_t)list_tok(dst, t, n));
    __syncthreads();
    word_prefix(scratch, words, wpre, sm);
    for (int w = tid; w < words; w += NT) {
      uint32_t bits = scratch[w];
      uint32_t pos = wpre[w];
      while (bits) {
        const int i = (w << 5) + (__ffs(bits) - 1);
        bits &= bits - 1u;
        if (pos < count) dst[pos] = i;
        ++pos;
      }
    }
    __syncthreads();
    for (int w = tid; w < words; w += NT) scratch[w] = 0;
    __syncthreads();
  }

  // Nested final sample (an option; Algorithm 1 draws the final sample afresh): the base sample, whose list
  // of b0 tokens this workgroup wrote at `base`, is kept as the head of the final sample, and the remaining
  // c - b0 tokens are drawn with the stream of S among the residual tokens outside the base sample.  The base
  // tokens are added to the bitmap of excluded tokens (bm, which S.bm_f points to) for that purpose.
  static __device__ __forceinline__ int draw_nested(const Sampler& S, HeadSizes hs, uint32_t b0, uint32_t c,
                                                    uint32_t* bm, const int32_t* base, int32_t* dst,
                                                    uint32_t dst_cap, int small_batches, HeadSmem& sm) {
    __syncthreads();  // the base list is complete (global memory is coherent inside a workgroup)
    for (uint32_t t = threadIdx.x; t < b0; t += NT) {
      const int tok = list_tok(base, t, hs.n);
      mark_bit(bm, (uint32_t)tok);
      if (t < dst_cap) dst[t] = tok;
    }
    __syncthreads();
    if (c <= b0 || dst_cap <= b0) return 0;
    hs.n_s -= (int)b0;
    const DrawBatch none = {};
    return draw_sample(S, hs, c - b0, none, false, small_batches, emit_to(dst + b0, dst_cap - b0), nullptr, nullptr, sm);
  }
};  // struct HeadOps

// Philox blocks of the batch that is generated ahead, before the top-k set is known.
template <int NT>
__device__ __forceinline__ int ahead_blocks(int small_batches) {
  // (a workgroup of 1024 threads serves long rows, whose samples hold thousands of tokens)
  return small_batches ? kSmallBatchBlocks : (NT >= 1024 ? 1024 : min(NT, 256));
}

// ---------------------------------------------------------------------------
// The first batch of draws of one sampler stream of one (sequence, head), with repeated tokens resolved, made
// ahead of the selection kernel: the draw sequences depend on the seed, the head and the sequence length only,
// not on the scores, so workgroups of the score launch make them while the others stream K.  The selection
// kernel (512 threads: the lower half owns stream 0, the upper half stream 1) then starts from these batches.
// ---------------------------------------------------------------------------
struct PreArgs {
  const int32_t* seq_lens;
  const uint64_t* seq_seeds;
  uint4* pre_tok;       // [B*Hq][512]: the four proposed tokens of every thread of the selection kernel
  uint32_t* pre_flags;  // [B*Hq][512]: ok | first << 4 | (made ? 256 : 0)
  SelectParams sp;
  int n_max, Hq, small_batches;
  uint32_t draw_cap;
  int job_rows;  // rows of the score grid that make batches instead of scores (0: none)
};

constexpr int kPreThreads = 256;  // workgroup size of a job: the score kernel's

// LDS layout of a job: HeadSmem, then three bitmaps of words_max words (drawn tokens, scratch, mail slots).
__host__ __device__ inline size_t prework_lds_bytes(int n_max) {
  const size_t words_max = ((size_t)(n_max + 63) >> 6) << 1;
  return ((sizeof(HeadOps<kPreThreads>::HeadSmem) + 15) & ~size_t(15)) + 3 * words_max * sizeof(uint32_t);
}

__device__ __forceinline__ void prework_job(const PreArgs& A, int b, int h, int stream, unsigned char* smem) {
  constexpr int NT = kPreThreads;
  using O = HeadOps<NT>;
  const int tid = threadIdx.x, bh = b * A.Hq + h;
  const int n = max(min(max(A.seq_lens[b], 1), A.n_max), 1);
  const HeadSizes hs = head_sizes(n, A.sp);
  const int words_max = ((A.n_max + 63) >> 6) << 1;
  const int words = (n + 31) >> 5;
  O::HeadSmem& sm = *reinterpret_cast<O::HeadSmem*>(smem);
  uint32_t* taken = reinterpret_cast<uint32_t*>(smem + ((sizeof(O::HeadSmem) + 15) & ~size_t(15)));
  uint32_t* scratch = taken + words_max;
  uint32_t* mail = scratch + words_max;
  for (int w = tid; w < words; w += NT) {
    taken[w] = 0;
    scratch[w] = 0;
    mail[w] = kInv32;
  }
  __syncthreads();
  const uint32_t L = (uint32_t)max(hs.mid_hi - hs.mid_lo, 1);
  O::Sampler S;
  S.taken = taken;
  S.scratch = scratch;
  S.mail = mail;
  S.bm_f = nullptr;
  S.wpre = nullptr;
  S.row = nullptr;
  S.seed = A.seq_seeds[b];
  S.stream = (uint32_t)stream;
  S.head = (uint32_t)h;
  S.query = 0u;
  S.L = L;
  S.thr = (uint32_t)((0x100000000ull - (uint64_t)L) % (uint64_t)L);
  {
    const uint64_t dflt = 64ull * (uint64_t)L + 4096ull;
    S.cap = (uint32_t)min(A.draw_cap ? (uint64_t)A.draw_cap : dflt, 0x80000000ull);
  }
  S.m = 0.f;
  S.dbg = nullptr;
  const int blocks = ahead_blocks<2 * NT>(A.small_batches);  // what the 512-thread selection kernel asks for
  const bool make = hs.n_s > 0 && hs.b0 < hs.n_s && blocks <= NT;
  DrawBatch mine = {};
  if (make) O::make_batch(mine, S, hs, 0u, blocks, false, false, sm, tid);
  const int64_t at = (int64_t)bh * (2 * NT) + stream * NT + tid;
  A.pre_tok[at] = make_uint4(mine.tok[0], mine.tok[1], mine.tok[2], mine.tok[3]);
  A.pre_flags[at] = (mine.ok & 15u) | ((mine.first & 15u) << 4) | (make ? 256u : 0u);
}

}  // namespace vatt
