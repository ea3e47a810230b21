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
#include "vatt_select.h"

namespace vatt {
namespace {

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
  // Selection-only kernel: where a list is written with the scores at hand (sink, window, top-k, and a final
  // sample that the first batch of draws holds) they are left at the list places, so that the gather kernel reads
  // them next to the list entries instead of from the score row by token.  A sample made another way is read by
  // token (HeadRec.tail_by_token).
  float* place_sc = A.place_sc + (int64_t)bh * A.idx_cap;
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
      // (selection-only kernel, which runs with every CU full: the scores of the final sample's proposals are
      // requested later, after the top-k step; a million scattered 4-byte reads at once, from all workgroups in
      // their first microseconds, held every workgroup up for five microseconds at config 3)
      O::make_batch(mine, half ? S1 : S0, hs, 0u, blocks, false, kFused || !half, sm, tid - half * (NT / 2));
    }
    spec0.blocks = spec1.blocks = blocks;
    spec0.have_sc = true;
    if (half) spec1 = mine; else spec0 = mine;
    spec1.have_sc = true;  // (the same answer in every thread; the lower half holds no draws of this stream)
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
            if (!kFused && pos < (uint32_t)A.k_max) place_sc[A.seg_topk + pos] = float_from_order_key(~(uint32_t)(c >> 32));
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
            else if (pos < (uint32_t)A.k_max) place_sc[A.seg_topk + pos] = row[i];
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
      else place_sc[A.seg_sink + i] = i == tid ? edge0 : row[i];
    }
    for (int i = tid; i < hs.n_win; i += NT) {
      if (writer) idx[A.seg_win + i] = hs.mid_hi + i;
      if (kFused) to_glist((uint32_t)(hs.n_sink + i), (uint32_t)(hs.mid_hi + i), i == tid ? edge1 : row[hs.mid_hi + i]);
      else place_sc[A.seg_win + i] = i == tid ? edge1 : row[hs.mid_hi + i];
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
  if (!kFused && pair_made && tid >= NT / 2) {  // (whole waves: the upper half holds the final sample's proposals)
#pragma unroll
    for (int e = 0; e < 4; ++e) spec1.sc[e] = row[spec1.tok[e]];
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
      r.tail_by_token = 1;  // (the statistics pass walks the base sample, whose scores are not at its places)
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
  // Long rows (1024 threads; their samples hold thousands of tokens and the first batch of draws usually holds
  // the whole final sample): the scores of that batch's proposals are requested now and arrive under the sums
  // and the budget; they go to the list places with the accepted tokens.  (In the 512-thread kernel, which is
  // short of registers, the same cost more than the gather gains: a sample that its shortcut above does not
  // cover is read by token.)
  constexpr bool kEmitScores = !kFused && NT >= 1024;
  if (kEmitScores && want1 && !spec1.have_sc) {
#pragma unroll
    for (int e = 0; e < 4; ++e) spec1.sc[e] = row[min(spec1.tok[e], (uint32_t)(n - 1))];
    spec1.have_sc = true;
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
          if (!kFused && pos < (uint32_t)A.b_max) place_sc[A.seg_dyn + pos] = spec1.sc[e];
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
  bool dyn_placed = fast_dyn;  // the final sample's scores are at its list places
  if (bfin > 0 && !fast_dyn) {
    Emit E1 = emit_to(idx + A.seg_dyn, (uint32_t)A.b_max);
    E1.global = writer;
    if (kEmitScores) E1.sc_dst = place_sc + A.seg_dyn;
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
    // (one batch made ahead with its scores held the whole sample, and the list stays in acceptance order)
    dyn_placed = kEmitScores && !A.nested && !A.ascending && want1 && spec1.have_sc && f == 0;
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
    r.tail_by_token = dyn_placed ? 0 : 1;
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

hipError_t set_kernel_attributes(const Plan& pl) {
  // The limit on dynamic LDS belongs to the kernel, not to the plan: it is raised to all a CU has (less the
  // kernels' static part), so that plans of different capacities can be used in any order.
  const int cap = 160 * 1024 - (int)head_kernel_static_lds_bytes();
  const void* kernels[6] = {reinterpret_cast<const void*>(head_kernel<kHeadThreads, 0, false>),
                            reinterpret_cast<const void*>(head_kernel<kHeadThreadsLong, 0, false>),
                            reinterpret_cast<const void*>(head_kernel<kHeadThreads, 128, false>),
                            reinterpret_cast<const void*>(head_kernel<kHeadThreads, 128, true>),
                            reinterpret_cast<const void*>(head_kernel<kHeadThreads, 64, false>),
                            reinterpret_cast<const void*>(head_kernel<kHeadThreads, 64, true>)};
  for (const void* f : kernels) {
    const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, cap);
    if (e != hipSuccess) return e;
  }
  return set_given_kernel_attributes(pl);
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

}  // namespace vatt
