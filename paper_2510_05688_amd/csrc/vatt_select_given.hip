// Selection with a caller-supplied top-k set: the kernel of both phases, with the scores of the listed tokens
// (first phase) or the gather (second phase) fused in at small batch, and its launchers.
#include <algorithm>

#include "vatt_select.h"

namespace vatt {
namespace {

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
      r.tail_by_token = 0;
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
    r.tail_by_token = 0;
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

}  // namespace

hipError_t set_given_kernel_attributes(const Plan& pl) {
  (void)pl;
  const int cap = 160 * 1024 - (int)head_kernel_static_lds_bytes();
  const void* kernels[5] = {reinterpret_cast<const void*>(given_topk_kernel<kHeadThreads, 0, false>),
                            reinterpret_cast<const void*>(given_topk_kernel<kHeadThreads, 128, false>),
                            reinterpret_cast<const void*>(given_topk_kernel<kHeadThreads, 128, true>),
                            reinterpret_cast<const void*>(given_topk_kernel<kHeadThreads, 64, false>),
                            reinterpret_cast<const void*>(given_topk_kernel<kHeadThreads, 64, true>)};
  for (const void* f : kernels) {
    const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, cap);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

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

}  // namespace vatt
