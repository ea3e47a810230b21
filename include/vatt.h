/*
 * vatt.h -- C ABI of libvatt: the decode step of verified sparse attention
 * (vAttention, arXiv 2510.05688) on one AMD MI355X (gfx950).
 *
 * One call of vatt_decode is one layer's attention for one decode step of a
 * batch: for every (sequence, query head) it runs Algorithm 1 of the paper
 * with Algorithm 2 inlined:
 *
 *   score     s_i = sm_scale * <K[i], q>                       (exponent of Eq. 1)
 *   I_f       sink tokens + local window + exact top-k of the tokens in
 *             between                                          (Alg. 1, index sets)
 *   I_bs      base sample of the residual tokens               (Alg. 2, sampling)
 *   stats     sigma^2, D (and Tr Sigma, ||N||) from I_f, I_bs  (Alg. 2, get-stats)
 *   b         CLT budget for the verified quantity X           (Corollaries for N and D,
 *                                                               Theorem 4.3)
 *   I_dyn     b residual tokens, uniform without replacement   (Alg. 1, sampling)
 *   O         N/D with N = N_f + (n_s/b) sum_{I_dyn} w_i V[i],
 *             D = D_f + (n_s/b) sum_{I_dyn} w_i                 (Section 4.1; Eq. 3)
 *
 * Conventions
 *   - Every function returns VATT_OK (0) or a negative VATT_E_* code.  Argument
 *     errors are found on the host before anything is launched.
 *   - "device" pointers are HIP device memory of the plan's device, owned by
 *     the caller; "host" pointers are ordinary process memory.  The library
 *     owns only the opaque plan (host memory).
 *   - vatt_decode, vatt_dense_decode, vatt_append_kv only enqueue kernels on
 *     the given HIP stream: no allocation, no synchronisation, no host read of
 *     device data.  A plan and its workspace may be used by one stream at a
 *     time.
 *   - bf16 tensors are raw 16-bit patterns (upper half of an IEEE binary32).
 *   - Query head h reads KV head h / (n_q_heads / n_kv_heads).
 *   - Everything after the score pass is per query head: each query head has
 *     its own top-k set, samples and budget (the paper's guarantee is per head).
 *
 * KV layouts
 *   contiguous: K, V are [batch, n_kv_heads, n_max, head_dim]
 *   paged:      K, V are [num_blocks, n_kv_heads, page_size, head_dim];
 *               block_table is int32 [batch, ceil(n_max / page_size)] and maps
 *               logical page p of sequence b to a physical block.  Entries
 *               outside [0, num_blocks) are clamped into range by the kernels
 *               (the result for that sequence is then meaningless, but no
 *               access leaves the allocation).
 *
 * Sampler (the paper asks for a uniform sample of the residual tokens in Alg. 1
 * and in Alg. 2, and leaves the procedure open)
 *   Stream 0 is the base sample, stream 1 the final sample.  Draw j of
 *   (sequence, query head h, stream) is the 32-bit word
 *       u_j = Philox4x32-10(counter = (j >> 2, stream, h, 0),
 *                           key = (seed & 0xffffffff, seed >> 32))[j & 3]
 *   with the sequence's seed for this call.  With L tokens between sink and
 *   window, x = u_j * L: the draw is void when x mod 2^32 < 2^32 mod L, else it
 *   proposes middle token x >> 32 (exactly uniform).  A proposal is accepted
 *   when the token is not in the top-k set and was not accepted before.  A
 *   sample of size c <= n_s / 2 is the first c accepted tokens; for larger c
 *   the first n_s - c accepted tokens are the ones left out; c = n_s is the
 *   whole residual.  This is simple random sampling without replacement,
 *   costs work proportional to min(c, n_s - c), does not depend on
 *   scheduling, and is reproducible from (seed, sequence, head).  After
 *   64 L + 4096 draws (never reached in practice) the missing tokens would be
 *   taken in index order.
 */
#ifndef VATT_H_
#define VATT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  VATT_OK = 0,
  VATT_E_INVALID_ARG = -1,       /* NULL pointer, non-positive size, epsilon/delta outside (0,1), ... */
  VATT_E_UNSUPPORTED_SHAPE = -2, /* head_dim not in {64,128}, group size not in {1,2,4,8}, ...        */
  VATT_E_WORKSPACE_TOO_SMALL = -3,
  VATT_E_HIP = -4,               /* a HIP runtime call failed (launch error, wrong device, ...)       */
  VATT_E_NO_DEVICE = -5          /* no HIP device / the HIP runtime is unusable                        */
};

enum { VATT_TARGET_D = 0, VATT_TARGET_N = 1, VATT_TARGET_SDPA = 2 };
enum { VATT_LAYOUT_CONTIGUOUS = 0, VATT_LAYOUT_PAGED = 1 };

/* Parameters of Algorithm 1 (its "Require" line) plus shapes.  Plain data, copied by vatt_plan_create. */
typedef struct vatt_params {
  int32_t batch;         /* B: sequences per call                                                    */
  int32_t n_q_heads;     /* Hq                                                                        */
  int32_t n_kv_heads;    /* Hkv; Hq % Hkv == 0 and Hq / Hkv in {1,2,4,8}                              */
  int32_t head_dim;      /* d in {64, 128}                                                            */
  int32_t n_max;         /* capacity in tokens per sequence; sizes workspace and index buffers.  The   */
                         /* selection kernel keeps six bitmaps of n_max bits in LDS (eight in its      */
                         /* 512-thread form): up to about 170 K tokens fit, beyond that                */
                         /* vatt_plan_create returns VATT_E_UNSUPPORTED_SHAPE                          */
  int32_t kv_layout;     /* VATT_LAYOUT_*                                                             */
  int32_t page_size;     /* tokens per block when paged (power of two, 8..256); ignored otherwise     */
  int32_t num_blocks;    /* physical blocks in the paged cache; ignored when contiguous               */
  int32_t sink;          /* |I_s|: absolute token count (the paper's experiments use 128)             */
  int32_t window;        /* |I_l|: absolute token count                                               */
  int32_t topk_abs;      /* k = topk_abs if > 0 else floor(topk_frac * n)            (f_t of Alg. 1)  */
  float   topk_frac;
  int32_t base_abs;      /* b0 = base_abs if > 0 else floor(base_frac * n_s), then clamped to [2,n_s] */
  float   base_frac;     /*                                                         (f_b of Alg. 2)  */
  float   epsilon;       /* in (0,1)                                                                  */
  float   delta;         /* in (0,1)                                                                  */
  int32_t target;        /* VATT_TARGET_*: which quantity is kept (epsilon, delta)-verified           */
  float   sm_scale;      /* softmax scale; 0 means 1/sqrt(head_dim)                                   */
  float   budget_cap_frac; /* b <= ceil(cap * n_s); 1 = uncapped (the paper); must be in (0,1]        */
} vatt_params;

typedef struct vatt_plan vatt_plan;

/* Regions of the workspace a caller may read (see vatt_plan_workspace_offset). */
enum {
  VATT_WS_SCORES = 0 /* float [B, Hq, n_max_padded]: s_i of the last vatt_decode or vatt_score call */
};

/*
 * Host only.  Validates the parameters, fixes launch geometry for the given device and computes the
 * workspace layout.  `device` is a HIP device ordinal; pass -1 to plan for a 256-CU gfx950 without
 * touching the HIP runtime (the plan can then be queried but not used to launch).
 * On success *out owns a plan to be released with vatt_plan_destroy.
 */
int vatt_plan_create(const vatt_params* params, int device, vatt_plan** out);
void vatt_plan_destroy(vatt_plan* plan);

/*
 * A plan for steps with q_len query tokens per sequence (the paper evaluates with the context processed
 * densely and the question tokens, like the generated ones, processed with sparse attention: the
 * split-prompt set-up of its appendix on evaluation set-ups).  The queries of a sequence are its q_len
 * newest tokens, whose K and V rows are already in the cache and counted in seq_lens; query token t
 * (0 .. q_len - 1, oldest first) sees the sequence up to and including itself, n - (q_len - 1 - t) tokens,
 * and runs Algorithm 1 on that prefix for every query head, with its own top-k set, samples and budget.
 * Its draws use the Philox counter (j >> 2, stream, h, t).  All query tokens and all query heads of a KV
 * head share one read of K in the score pass.
 * With such a plan every "[B, ...]" shape of q and of the outputs of vatt_decode, vatt_dense_decode and
 * vatt_score reads "[B, q_len, ...]" (seq_lens, seq_seeds, block_table and the caches stay per sequence,
 * and every seq_lens entry should be at least q_len: a query with no visible token is treated as seeing
 * one); the same holds for topk_idx and topk_cnt of vatt_decode_given_topk.  q_len = 1 is vatt_plan_create.
 * q_len may not exceed 256 and batch * q_len may not exceed 65535 (VATT_E_UNSUPPORTED_SHAPE).
 */
int vatt_plan_create_chunk(const vatt_params* params, int q_len, int device, vatt_plan** out);
int vatt_plan_query_len(const vatt_plan* plan);

/*
 * Options of the method (host only; vatt_plan_set_option).  All are off by default, which is the paper's
 * algorithm.  (include/vatt_testing.h declares further option numbers that only change how the same results
 * are computed; they exist for the test suite.)
 */
enum { VATT_OPT_BUDGET_BOUND = 4, VATT_OPT_NESTED_SAMPLES = 5, VATT_OPT_BUDGET_MULTIPLE = 7,
       VATT_OPT_ASCENDING_SAMPLES = 12, VATT_OPT_CACHE_SLOTS = 13 };
/*
 * VATT_OPT_CACHE_SLOTS = c (a multiple of 4 in 4 .. 8192): slots per (sequence, KV head) of the random cache of
 * base-sample rows (see vatt_random_cache_fill); the default is the largest base sample of the plan plus a
 * quarter plus 64, rounded up to a multiple of 64 and capped at 8192.  Set it before the cache buffer is sized.
 * VATT_OPT_ASCENDING_SAMPLES = 1: the base and final samples' segments of out_idx are written in ascending token
 * order (they are the same sets; by default they come in the order in which the sampler accepted the tokens).
 * The gather then walks every head's rows in address order.  Plans with this option keep selection and gather
 * in kernels of their own.
 */
/*
 * VATT_OPT_BUDGET_MULTIPLE = q (1 .. 65536; 1, the default, is Algorithm 2's rule): the budget b is rounded up
 * to the next multiple of q, e.g. 16, the V rows one wave of the gather reads per instruction at d = 128, or 64.
 * It never goes beyond min(n_s, max(b0, ceil(budget_cap_frac * n_s))), the largest value the plain rule can
 * give, so the index buffer needs no more room.  More samples than Algorithm 2 asks for keep its guarantee.
 * out_budget_raw still reports b* itself.
 */
/*
 * VATT_OPT_NESTED_SAMPLES = 1 departs from Algorithm 1, which draws the final sample afresh: the base sample
 * is kept as the head of the final sample and only b - b0 further tokens are drawn (stream 1) among the
 * residual tokens outside it.  For a fixed b the result is still a uniform b-subset of the residual; b itself
 * was computed from the base sample, so the estimate is no longer exactly unbiased.  It saves the second
 * sample where b = b0 (most heads) and, in vatt_decode_given_topk, the K rows of the base sample.  The final
 * sample's segment of out_idx then starts with the base sample in its own order.  0 (default) is the paper.
 */
/*
 * VATT_OPT_BUDGET_BOUND selects the tail bound behind the denominator budget of Algorithm 2:
 * VATT_BOUND_CLT (default) is the corollary for D, b* = (Phi^{-1}(1 - delta/2) n_s sigma / (eps D))^2;
 * VATT_BOUND_HOEFFDING is the more conservative alternative the paper's appendix on the tightness of the
 * bounds compares it with.  The paper prints no formula for it.  What is built is a reading fitted to the one
 * number the appendix reports (2.8 times the samples at delta = 0.2): the sub-Gaussian tail form
 * b* = 2 ln(2 / delta) (n_s sigma / (eps D))^2, i.e. the CLT budget with z^2 replaced by 2 ln(2 / delta).  It
 * uses the sample variance where Hoeffding's inequality proper uses the range of the weights, so it carries
 * no distribution-free finite-sample guarantee (the range-based form, (ln(2 / delta) / 2) (n_s R / (eps D))^2
 * with R <= 1 the weight range, would, and asks for far more samples than the appendix reports).
 * VATT_BOUND_HOEFFDING_RANGE is that range-based form: Hoeffding's inequality proper (it also holds for
 * sampling without replacement), b* = (ln(2 / delta) / 2) (n_s R / (eps D))^2 with R = exp(min_{I_t} s - m):
 * every residual token scores at most the weakest member of the exact top-k set, so the residual weights
 * lie in [0, R] (R = 1 when k = 0).  It needs no variance and holds for every distribution of the weights;
 * on all but very concentrated heads it asks for the whole residual.  vatt_decode only: a top-k set supplied
 * by the caller bounds nothing (vatt_decode_given_topk returns VATT_E_UNSUPPORTED_SHAPE under this bound).
 * Both Hoeffding forms: denominator target only (VATT_E_UNSUPPORTED_SHAPE otherwise).
 */
enum { VATT_BOUND_CLT = 0, VATT_BOUND_HOEFFDING = 1, VATT_BOUND_HOEFFDING_RANGE = 2 };
int vatt_plan_set_option(vatt_plan* plan, int option, int value);

/* Bytes of device workspace every launching call needs (256-byte aligned base). */
size_t vatt_plan_workspace_bytes(const vatt_plan* plan);
/* Byte offset of a VATT_WS_* region inside the workspace, or (size_t)-1 for an unknown region. */
size_t vatt_plan_workspace_offset(const vatt_plan* plan, int region);
/* Row stride, in floats, of the VATT_WS_SCORES region (n_max rounded up). */
size_t vatt_plan_score_stride(const vatt_plan* plan);

/*
 * Layout of out_idx: per (sequence, query head) `vatt_plan_index_capacity` int32 slots holding five
 * segments at fixed offsets, each filled from its start:
 *   segment 0 sink, 1 window, 2 top-k (these three in ascending token order), 3 base sample, 4 final sample
 *   (in the order in which the sampler accepted the tokens, or ascending when the sample is a complement).
 * vatt_plan_index_segment returns the offset (in ints) of a segment, or -1.
 */
size_t vatt_plan_index_capacity(const vatt_plan* plan);
int64_t vatt_plan_index_segment(const vatt_plan* plan, int segment);

/*
 * One vAttention decode step (Algorithm 1) for the whole batch.
 *   q            device, bf16 [B, Hq, d]
 *   k, v         device, bf16 cache in the plan's layout
 *   block_table  device, int32 [B, ceil(n_max / page_size)]; NULL when contiguous
 *   seq_lens     device, int32 [B]; tokens valid in each sequence, 1 <= n <= n_max
 *                (values outside are clamped by the kernels)
 *   seq_seeds    device, uint64 [B]; sampler seed of each sequence for this call
 *   workspace    device, 256-byte aligned; contents are scratch
 *   workspace_bytes  size of that buffer; less than vatt_plan_workspace_bytes is VATT_E_WORKSPACE_TOO_SMALL
 *   out_o        device, float [B, Hq, d]
 *   out_lse      device, float [B, Hq] or NULL: ln of the estimated denominator, ln(D), of Section 4.1
 *   out_idx      device, int32 [B, Hq, index_capacity]
 *   out_counts   device, int32 [B, Hq, 8] = { |I_s|, |I_l|, |I_t|, |I_bs|, b, n_s, n, flags }
 *                flags (informational): bit 0 base sample taken as a complement, bit 1 final sample taken as a
 *                complement, bit 2 base sample needed more than one batch of draws, bit 3 final sample did,
 *                bit 4 the draw limit was reached, bit 5 the top-k selection took its general path,
 *                bit 6 the base sample came from the random cache
 *   out_budget_raw device, double [B, Hq] or NULL: b* before rounding and clamping
 *   out_stats    device, float [B, Hq, 4] or NULL = { D_hat, sigma^2, Tr Sigma, ||N_hat||^2 }, all in the
 *                scale where the largest score of the head has weight 1 (w_i = exp(s_i - max s))
 *   stream       hipStream_t
 */
int vatt_decode(vatt_plan* plan, const void* q, const void* k, const void* v,
                const int32_t* block_table, const int32_t* seq_lens, const uint64_t* seq_seeds,
                void* workspace, size_t workspace_bytes, float* out_o, float* out_lse, int32_t* out_idx,
                int32_t* out_counts, double* out_budget_raw, float* out_stats, void* stream);

/*
 * vatt_decode without a workspace argument, for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The kernels are those of vatt_decode;
 * their scratch memory (scores, partial sums, per-head records) is an array inside the library,
 * vatt_static_scratch_bytes() = 16 MiB per GPU, which every GPU the library runs on holds until the process
 * ends.  The call allocates nothing, frees nothing and calls no allocating routine; the array's address on the
 * plan's device was looked up by vatt_plan_create.  A plan whose vatt_plan_workspace_bytes exceeds the array is
 * refused with VATT_E_WORKSPACE_TOO_SMALL (the 32K-token, batch-1 layer of 32 / 8 heads needs 12.3 MiB).
 * All calls on one GPU share that GPU's array, which keeps the last call's contents (nothing in it has to
 * start at zero: every region is written before it is read within a call): calls that overlap on one GPU,
 * from any streams or plans, race.  Other arguments, results and errors as in vatt_decode.
 */
size_t vatt_static_scratch_bytes(void);
int vatt_decode_static(vatt_plan* plan, const void* q, const void* k, const void* v,
                       const int32_t* block_table, const int32_t* seq_lens, const uint64_t* seq_seeds,
                       float* out_o, float* out_lse, int32_t* out_idx, int32_t* out_counts,
                       double* out_budget_raw, float* out_stats, void* stream);

/*
 * The same decode step with the top-k set supplied by the caller: Section 4.1 leaves the choice of I_t to any
 * (approximate) top-k method, and without the exact score pass only the attended tokens' K and V rows are read.
 *   topk_idx     device, int32 [B, Hq, k_max] with k_max = the length of the top-k segment of out_idx
 *                (vatt_plan_index_segment(plan, 3) - vatt_plan_index_segment(plan, 2)); tokens in any order
 *   topk_cnt     device, int32 [B, Hq]: entries used per head (clamped to [0, k_max])
 * I_t is the set of supplied tokens that lie between sink and window, without repeats; everything after it
 * follows Algorithm 1 as in vatt_decode: residual, base sample, statistics, budget, final sample, estimate.
 * Scores exist only for I_f, I_bs and I_dyn; out_stats and out_lse use the largest score among I_f and I_bs
 * as the shift (every quantity Algorithm 2 forms is a ratio and does not depend on it).
 * With the targets N and SDPA the score kernel of the listed tokens also reads their V rows for the numerator
 * statistics of Algorithm 2.  Other arguments as in vatt_decode.
 */
int vatt_decode_given_topk(vatt_plan* plan, const void* q, const void* k, const void* v,
                           const int32_t* block_table, const int32_t* seq_lens, const uint64_t* seq_seeds,
                           const int32_t* topk_idx, const int32_t* topk_cnt, void* workspace,
                           size_t workspace_bytes, float* out_o, float* out_lse, int32_t* out_idx,
                           int32_t* out_counts, double* out_budget_raw, float* out_stats, void* stream);

/*
 * Random cache of base-sample rows.  The implementation note after Theorem 4.3 observes that the base sample
 * can be served from a small random cache that is populated and updated during generation, without giving a
 * procedure; this library's reading: per (sequence, KV head) a cache of c slots holds a uniform random
 * c-subset of the tokens seen so far, in uniformly random slot order, each with a copy of its K and V row.
 * Token t (counted from 0) arrives with one draw r, uniform in [0, t]: while the cache is not full the entry
 * of slot r moves to slot t and the token takes slot r; afterwards the token replaces slot r when r < c
 * (reservoir sampling).  r comes from the four words of Philox4x32-10 under the counter (t, 2, KV head, 0)
 * and the key (low, high half of the sequence's cache seed), mapped to [0, t] by the multiply-and-reject
 * rule of the sampler (first accepted word, else the fourth).
 * A decode step that uses the cache takes as base sample of a query head the first b0 cached tokens, in slot
 * order, that are residual tokens of that head (outside sink, window and I_t): a uniform random subset in
 * random order, filtered by a condition that does not depend on the order, is a uniform b0-subset of the
 * residual.  The heads of a KV head then share most base-sample rows, and those rows are neighbours in
 * memory.  A head whose cache holds fewer than b0 residual tokens draws its base sample as without a cache
 * (flag bit 6 of out_counts is set where the cache was used).  The final sample is drawn afresh either way,
 * so the estimate stays unbiased, and the budget has the distribution it has with a drawn base sample.
 *
 *   rcache       device, 256-byte aligned, vatt_random_cache_bytes(plan) bytes, owned by the caller; the
 *                layout is the library's (one record per (sequence, KV head): slot count, token list,
 *                K rows, V rows)
 *   cache_seeds  device, uint64 [B]: one seed per sequence, the same for the whole life of the sequence
 *
 * vatt_random_cache_fill   builds the cache of sequences that exist already: the state after their tokens
 *                          0 .. seq_lens[b]-1 have arrived one by one (rows copied from k, v).
 * vatt_append_kv_cached    vatt_append_kv, and the appended token arrives in the cache (position
 *                          seq_lens[b] before the increment).  A sequence at n_max is left unchanged.
 * vatt_decode_given_topk_cached   vatt_decode_given_topk with the base sample taken from the cache.
 *                          Single-token steps only (VATT_E_UNSUPPORTED_SHAPE for q_len > 1 and with
 *                          VATT_OPT_ASCENDING_SAMPLES).  The cache has to hold tokens below seq_lens[b] only,
 *                          which it does when every token went in through the two calls above.
 * All three only enqueue kernels on `stream`; errors as in vatt_decode.
 */
size_t vatt_random_cache_bytes(const vatt_plan* plan);
int vatt_random_cache_slots(const vatt_plan* plan);
int vatt_random_cache_fill(vatt_plan* plan, const void* k, const void* v, const int32_t* block_table,
                           const int32_t* seq_lens, const uint64_t* cache_seeds, void* rcache, void* stream);
int vatt_append_kv_cached(vatt_plan* plan, const void* k_new, const void* v_new, void* k, void* v,
                          const int32_t* block_table, int32_t* seq_lens, const uint64_t* cache_seeds,
                          void* rcache, void* stream);
int vatt_decode_given_topk_cached(vatt_plan* plan, const void* q, const void* k, const void* v,
                                  const int32_t* block_table, const int32_t* seq_lens, const uint64_t* seq_seeds,
                                  const int32_t* topk_idx, const int32_t* topk_cnt, const void* rcache,
                                  void* workspace, size_t workspace_bytes, float* out_o, float* out_lse,
                                  int32_t* out_idx, int32_t* out_counts, double* out_budget_raw, float* out_stats,
                                  void* stream);

/*
 * Dense decode attention (Eq. 1) on the same cache: the sparsity speed-up denominator.
 * Arguments as in vatt_decode.  out_lse may be NULL.
 */
int vatt_dense_decode(vatt_plan* plan, const void* q, const void* k, const void* v,
                      const int32_t* block_table, const int32_t* seq_lens, void* workspace,
                      size_t workspace_bytes, float* out_o, float* out_lse, void* stream);

/*
 * Score pass alone (first step of Algorithm 1 with oracle top-k): fills the VATT_WS_SCORES region of the
 * workspace with s_i for every (sequence, query head, i < n).  Exposed for stage-wise parity checks and
 * for timing the K scan on its own.
 */
int vatt_score(vatt_plan* plan, const void* q, const void* k, const int32_t* block_table,
               const int32_t* seq_lens, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Append one token per sequence: writes k_new, v_new (device, bf16 [B, Hkv, d]) at position seq_lens[b]
 * of the cache and then increments seq_lens[b] (device, int32 [B]).  A sequence already at n_max is
 * left unchanged.
 */
int vatt_append_kv(vatt_plan* plan, const void* k_new, const void* v_new, void* k, void* v,
                   const int32_t* block_table, int32_t* seq_lens, void* stream);

/*
 * KV cache in host memory (the paper's efficiency experiment hosts the KV cache on the CPU and finds the time
 * per step proportional to the amount of KV cache read; its implementation notes keep only the small random
 * cache and the top-k method's own structures on the GPU).
 *
 * Wherever this header says "device" for k and v, the address of a cache that lives in pinned host memory
 * (hipHostMalloc, or any allocator built on it) may be passed instead: the kernels then read the rows they
 * need over the host link, and vatt_append_kv / vatt_append_kv_cached write the new rows there.  Every
 * other buffer (q, lists, lengths, seeds, the random cache, workspace, outputs) stays in device memory.  With
 * vatt_decode_given_topk_cached a step reads from the host only the K and V rows of I_f and of the final
 * sample: the base sample comes from the cache on the device.
 *
 * This call translates a pointer into such an allocation to the address the kernels must be given (on this
 * platform the same number) and is the check that the memory is of that kind: VATT_E_INVALID_ARG for ordinary
 * process memory, which a kernel must never be handed.  Host only; nothing is launched.
 *   host_ptr     host, anywhere inside a pinned allocation
 *   device_ptr   host, receives the address to pass as k or v (NULL on error)
 */
int vatt_host_kv_device_pointer(const void* host_ptr, void** device_ptr);

const char* vatt_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* VATT_H_ */
