// Host-side plan and the launchers each kernel file exports to the API file.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/vatt.h"
#include "../../include/vatt_testing.h"
#include "vatt_dev.h"

namespace vatt {

constexpr int kScoreTile = 64;        // keys per score-kernel workgroup (small tiles: many short workgroups fill and
                                      // drain the chip more evenly than few long ones; measured 64 > 128 > 256 > 32)
constexpr int kScoreTilePaged = 256;  // keys per score-kernel workgroup on a paged cache
constexpr int kSubTile = 8;            // keys per sub-tile maximum
constexpr int kHeadThreads = 512;      // workgroup size of the per-head kernel
constexpr int kHeadThreadsLong = 1024; // ... for rows whose 8-key maxima do not fit the registers of 512 threads
constexpr int kGatherThreads = 256;
// Launch orders of the score pass (see the score kernel); the values of VATT_OPT_SCORE_ORDER.
constexpr int kScoreOrderTile = 0, kScoreOrderKvHead = 1, kScoreOrderBlocks = 2;
constexpr int kDenseThreads = 256;
constexpr int kCacheSlotsMax = 8192;   // slots of the random cache of base-sample rows, per (sequence, KV head)

// What the per-head kernel leaves for the gather kernel.
struct HeadRec {
  float m;        // max score of the head
  float scale;    // n_s / b (0 when b == 0)
  int32_t n, n_sink, n_win, k, b, n_s;
  int32_t b_keep;  // leading entries of the final sample that repeat the base sample (nested samples), else 0
  int32_t base_cached;  // the base sample's entries are slots of the random cache (their rows are read from it)
  int32_t tail_by_token;  // the gather reads the sampled tokens' scores from the score row by token (else, like
                          // those of sink, window and top-k, from where the selection kernel left them: at the
                          // list places)
};

struct Plan {
  vatt_params p;
  int device;         // -1: geometry only
  int num_cus;
  int group;          // Hq / Hkv
  int q_len;          // query tokens per sequence and call (1: single-token decoding)
  int vbatch;         // batch * q_len: every (sequence, query token) pair is handled like a sequence of its own
  float sm_scale;
  double z_half;      // Phi^{-1}(1 - delta/2)
  double range_factor;  // > 0: the range-based Hoeffding budget, ln(2 / delta) / 2 (denominator target)
  double z_quarter;   // Phi^{-1}(1 - delta/4)
  double eps, cap_frac;
  SelectParams sel;
  // sizes
  int n_pad;          // score row stride (floats)
  int n_sub;          // sub-tiles of kSubTile keys per row (the score kernel leaves each one's largest score)
  int k_max, b0_max, b_max;
  int head_threads;   // workgroup size of the per-head kernel
  int split_cap;  // upper bound of the four split counts below that share the partial-sum regions
  int gather_splits, dense_splits, vstat_splits, given_splits;
  int given_fuse_splits;  // caller-supplied top-k: > 0, the second selection phase also gathers, with this many workgroups per head
  int sparse_splits;  // workgroups per head of the score kernel of the listed tokens when it only writes scores
  size_t idx_cap;
  int64_t seg_off[5];
  size_t head_lds_bytes;
  int topk_general_path;          // test hook: the top-k selection always takes its general path
  int sampler_small_batches;      // test hook: the sampler works in batches of 256 draws only
  uint32_t sampler_draw_cap;      // draws after which a sample is completed in index order (0: 64 L + 4096)
  int group_major;                // the later kernels launch the query heads of a KV head on one XCD (head_of_block)
  int score_order;                // launch order of the score pass (kScoreOrder*)
  int nested_samples;             // the final sample keeps the base sample and extends it (not the paper's fresh draw)
  int ascending_samples;          // the samples' index lists are written in ascending token order
  int budget_multiple;            // the budget is rounded up to a multiple of this (1: the paper's rule)
  int prework;                    // the sampler streams' first batches are made by workgroups of the score launch
  int fuse_splits;                // > 0: the selection kernel also gathers, with this many workgroups per head
  int cache_slots;                // slots per (sequence, KV head) of the random cache of base-sample rows
  // workspace offsets (bytes)
  size_t off_scores, off_sub_max, off_sparse, off_head_rec, off_gather_part,
      off_debug, off_vstat_part, off_dense_part, off_pre_tok, off_pre_flags, off_base_slot, ws_bytes;
  KVLayout kv_k, kv_v;  // templates; base pointers are passed per call
};

// Every launcher returns a hipError_t from hipGetLastError() after the launch.
// seq_seeds: needed (may be nullptr otherwise) when score_prework(pl)
hipError_t launch_score(const Plan& pl, const void* q, const void* k, const int32_t* block_table,
                        const int32_t* seq_lens, const uint64_t* seq_seeds, void* ws, hipStream_t st);
// The score pass of a multi-query step (q_len > 1): all query tokens and group heads share one read of K.
hipError_t launch_score_chunk(const Plan& pl, const void* q, const void* k, const int32_t* block_table,
                              const int32_t* seq_lens, void* ws, hipStream_t st);
// phase 0: everything (target D); phase 1: through the base sample; phase 2: budget and final sample.
hipError_t launch_head(const Plan& pl, int phase, const int32_t* seq_lens, const uint64_t* seq_seeds, void* ws,
                       int32_t* out_idx, int32_t* out_counts, double* out_budget_raw, float* out_stats,
                       hipStream_t st);
// The path with a caller-supplied top-k set: selection phase 0 (sets, base sample) and 1 (budget, final sample),
// scores of the listed tokens, gather with the final sample's scores computed on the way.
// Selection and gather in one kernel for small batches (denominator target, fresh final sample), then the merge
// of the per-workgroup partial sums.
hipError_t launch_head_fused(const Plan& pl, const void* v, const int32_t* block_table, const int32_t* seq_lens,
                             const uint64_t* seq_seeds, void* ws, int32_t* out_idx, int32_t* out_counts,
                             double* out_budget_raw, float* out_stats, bool pre_made, hipStream_t st);
// Whether workgroups of the score launch make the sampler streams' first batches for the fused selection kernel
// (single-token steps in the KV-head-major launch order only).
inline bool score_prework(const Plan& pl) {
  return pl.prework && pl.fuse_splits > 0 && !pl.nested_samples && !pl.ascending_samples && pl.q_len == 1 &&
         pl.p.target == VATT_TARGET_D && pl.score_order == kScoreOrderKvHead;
}
hipError_t launch_gather_merge(const Plan& pl, void* ws, int splits, float* out_o, float* out_lse, hipStream_t st);
int fused_splits_for(const Plan& pl);           // the plan's own choice (0: separate kernels)
bool fused_splits_fit(const Plan& pl, int splits);  // whether the fused kernel can run with that many
// rcache (may be nullptr): random cache the base sample is taken from when it holds enough residual tokens;
// the score kernel of the listed tokens then reads those tokens' rows from the cache.
hipError_t launch_given_select(const Plan& pl, int phase, const int32_t* seq_lens, const uint64_t* seq_seeds,
                               const int32_t* given_idx, const int32_t* given_cnt, const void* rcache, void* ws,
                               int32_t* out_idx, int32_t* out_counts, double* out_budget_raw, float* out_stats,
                               hipStream_t st);
// The second selection phase with the gather fused in (small batches, denominator target, fresh final sample),
// followed by the merge of the per-workgroup partials.
// (phase 0: first selection phase plus the scores of I_f and I_bs; phase 1: second phase plus the gather)
hipError_t launch_given_fused(const Plan& pl, int phase, const void* q, const void* k, const void* v,
                              const int32_t* block_table, const int32_t* seq_lens, const uint64_t* seq_seeds,
                              const int32_t* given_idx, const int32_t* given_cnt, const void* rcache, void* ws,
                              int32_t* out_idx, int32_t* out_counts, double* out_budget_raw, float* out_stats,
                              hipStream_t st);
hipError_t launch_given_merge(const Plan& pl, void* ws, int splits, float* out_o, float* out_lse, hipStream_t st);
int given_fused_splits_for(const Plan& pl);
bool given_fused_fits(const Plan& pl, int splits);
// (with targets N and SDPA it also reads the V rows of the listed tokens and leaves the numerator statistics)
hipError_t launch_sparse_score(const Plan& pl, const void* q, const void* k, const void* v,
                               const int32_t* block_table, const void* rcache, void* ws, const int32_t* out_idx,
                               hipStream_t st);
// Random cache of base-sample rows: layout for a plan, state after the tokens of existing sequences have
// arrived one by one, append of one token per sequence with its arrival in the cache, token lists for tests.
CacheLayout cache_layout(const Plan& pl);
hipError_t launch_cache_fill(const Plan& pl, const void* k, const void* v, const int32_t* block_table,
                             const int32_t* seq_lens, const uint64_t* cache_seeds, void* rcache, hipStream_t st);
hipError_t launch_append_cached(const Plan& pl, const void* k_new, const void* v_new, void* k, void* v,
                                const int32_t* block_table, int32_t* seq_lens, const uint64_t* cache_seeds,
                                void* rcache, hipStream_t st);
hipError_t launch_cache_read(const Plan& pl, const void* rcache, int32_t* out_tok, int32_t* out_count,
                             hipStream_t st);
hipError_t launch_given_gather(const Plan& pl, const void* q, const void* k, const void* v,
                               const int32_t* block_table, void* ws, const int32_t* out_idx, float* out_o,
                               float* out_lse, hipStream_t st);
hipError_t launch_vstats(const Plan& pl, const void* v, const int32_t* block_table, void* ws,
                         const int32_t* out_idx, hipStream_t st);
hipError_t launch_gather(const Plan& pl, const void* v, const int32_t* block_table, void* ws,
                         const int32_t* out_idx, float* out_o, float* out_lse, hipStream_t st);
hipError_t launch_dense(const Plan& pl, const void* q, const void* k, const void* v, const int32_t* block_table,
                        const int32_t* seq_lens, void* ws, float* out_o, float* out_lse, hipStream_t st);
hipError_t launch_append(const Plan& pl, const void* k_new, const void* v_new, void* k, void* v,
                         const int32_t* block_table, int32_t* seq_lens, hipStream_t st);
hipError_t set_kernel_attributes(const Plan& pl);        // every selection kernel: dynamic LDS limit
hipError_t set_given_kernel_attributes(const Plan& pl);  // (its part for the caller-supplied-top-k kernels)
// Dynamic and static LDS of the selection kernels, and the LDS list entries of the fused gathers.
size_t head_kernel_lds_bytes(int n_max, int head_threads);
size_t head_kernel_static_lds_bytes();
int fused_dlist_cap(const Plan& pl, int splits);
// Reads `bytes` (a multiple of 16) from src and discards them; sink is 4 KiB of device memory.
hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, hipStream_t st);
// Reads the 256-byte rows rows[0 .. count) (row numbers, clamped into [0, rows_total)) of src and discards them.
hipError_t launch_row_read(const void* src, size_t rows_total, const int32_t* rows, size_t count, void* sink,
                           hipStream_t st);

}  // namespace vatt

struct vatt_plan {
  vatt::Plan pl;
};
