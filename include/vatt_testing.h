/*
 * vatt_testing.h -- hooks of libvatt that are no part of its interface: option numbers that change how a
 * result is computed but never the result (the test suite uses them to force rarely taken paths), a debug
 * region of the workspace, and a read-only kernel that measurements use as a floor.  A caller of the library
 * needs none of this; include/vatt.h is the interface.
 */
#ifndef VATT_TESTING_H_
#define VATT_TESTING_H_

#include "vatt.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Further option numbers for vatt_plan_set_option.  Results are identical with every setting.
 *   VATT_OPT_SAMPLER_SMALL_BATCHES = 1: the sampler works through the draw sequence in batches of 256 draws
 *     only (it normally uses up to 1024, or 4096 with 1024 threads).
 *   VATT_OPT_SAMPLER_DRAW_CAP = c > 0: replaces the 64 L + 4096 draw limit by c draws (0 restores it), so that
 *     the completion rule can be exercised.  (This one does change which tokens a sample holds once the cap
 *     is reached; the oracle has the same parameter.)
 *   VATT_OPT_TOPK_GENERAL_PATH = 1: the top-k selection skips its usual shortcut (a lower bound of the
 *     threshold from the largest scores of every 8 keys) and takes the general path, a histogram over the
 *     whole score row, which otherwise only serves short or unusual rows.
 *   VATT_OPT_HEAD_THREADS = 512 or 1024: workgroup size of the selection kernel.  The plan picks 512 for
 *     n_max <= 32768, and 1024 for longer rows when that costs no parallelism.  To be set on the plan's device.
 *   VATT_OPT_SCORE_ORDER = 0 / 1 / 2: launch order of the score pass, i.e. which of the chip's XCDs reads which
 *     tile: 0 tile by tile across the XCDs, 1 all tiles of a KV head on one XCD, 2 like 0 in blocks of 256 KiB
 *     of K.  The plan picks 1 up to n_max = 65536 when the KV head count is a multiple of 8, else 2.
 *     Multi-query plans have order 0 only (VATT_E_UNSUPPORTED_SHAPE otherwise).
 *   VATT_OPT_FUSED_GATHER = 0, 1, 2, 4, 8 or 16: 0 keeps selection and gather in kernels of their own; S > 0
 *     runs them as one kernel with S workgroups per head (denominator target, 512-thread selection and fresh
 *     final samples only; VATT_E_UNSUPPORTED_SHAPE when the kernel's LDS does not hold that split).  The plan
 *     picks S > 0 for batches with fewer heads than half the chip's compute units.  The index sets, budgets
 *     and statistics are identical; the output sums run in another order.
 *   VATT_OPT_SCORE_PREWORK = 0 / 1: with the fused gather, whether the first batches of the sampler's draw
 *     sequences are made by the first workgroups of the score launch while the rest of it streams K (1, the
 *     default for such plans in the KV-head-major launch order) or by the selection kernel itself (0).
 *   VATT_OPT_GIVEN_SPLITS, VATT_OPT_SPARSE_SPLITS = 1 .. enough for 32 workgroups per CU (at most 32): workgroups per head of
 *     the gather kernel and of the score kernel of the listed tokens on the path with a caller-supplied top-k set
 *     (tuning aids; the plan picks both).
 *   VATT_OPT_GIVEN_FUSED = 0, 1, 2, 4, 8 or 16: on that path, 0 keeps the second selection phase and the gather
 *     in kernels of their own; S > 0 runs them as one kernel with S workgroups per head (denominator target and
 *     fresh final samples only; VATT_E_UNSUPPORTED_SHAPE when the kernel's LDS does not hold that split).  The
 *     plan picks S > 0 for batches with at most half as many heads as compute units.  Index sets, budgets and
 *     statistics are identical; the output sums run in another order.
 */
enum { VATT_OPT_SAMPLER_SMALL_BATCHES = 1, VATT_OPT_SAMPLER_DRAW_CAP = 2, VATT_OPT_TOPK_GENERAL_PATH = 3,
       VATT_OPT_HEAD_THREADS = 6, VATT_OPT_SCORE_ORDER = 8, VATT_OPT_FUSED_GATHER = 9, VATT_OPT_SCORE_PREWORK = 10,
       VATT_OPT_GIVEN_SPLITS = 14, VATT_OPT_SPARSE_SPLITS = 15, VATT_OPT_GIVEN_FUSED = 16 };

/* Workspace region (vatt_plan_workspace_offset): uint64 [512] of phase clock stamps, written only by builds
 * of the library made with -DVATT_TIMING. */
enum { VATT_WS_DEBUG = 1 };

/*
 * Measurement aid: one kernel that reads `bytes` bytes (a multiple of 16) from the 16-byte aligned device
 * buffer src and discards them.  Its duration is the practical floor for any single launch that must stream
 * that many bytes from HBM, which is what the K scan is compared with.
 *   sink    device, at least 4 KiB, may be written (practically never is)
 */
int vatt_stream_read(const void* src, size_t bytes, void* sink, void* stream);

/*
 * Measurement aid: one kernel that reads `count` rows of 256 bytes (a K or V row at head_dim 128) of the
 * 16-byte aligned device buffer src and discards them, in the access shape of the gather kernels (16 lanes per
 * row, 8 rows in flight per lane group, row numbers taken from a list).  Its duration is the practical floor
 * for gathering that many rows in one launch.
 *   rows_total  rows in src (at most 2^31 - 1); listed row numbers outside [0, rows_total) are clamped into it
 *   rows        device, int32 [count]
 *   sink        device, at least 4 KiB, may be written (practically never is)
 */
int vatt_row_read(const void* src, size_t rows_total, const int32_t* rows, size_t count, void* sink, void* stream);

/*
 * Token lists of a random cache of base-sample rows (vatt_random_cache_fill in vatt.h), for comparison with a
 * reference: out_tokens (device, int32 [B, Hkv, vatt_random_cache_slots(plan)]) gets the token of every slot in
 * slot order, -1 for slots not in use; out_counts (device, int32 [B, Hkv]) the number of slots in use.
 */
int vatt_random_cache_read(vatt_plan* plan, const void* rcache, int32_t* out_tokens, int32_t* out_counts,
                           void* stream);

#ifdef __cplusplus
}
#endif
#endif /* VATT_TESTING_H_ */
