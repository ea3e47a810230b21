// C ABI of libvatt: parameter validation, plan geometry, workspace layout and the launch sequences.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>

#include "vatt_internal.h"

namespace vatt {
namespace {

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// z with 1 - Phi(z) = t: safeguarded Newton on f(z) = erfc(z / sqrt 2) / 2 - t, f'(z) = -phi(z).
double upper_tail_quantile(double t) {
  double lo = -40.0, hi = 40.0, z = 0.0;
  for (int it = 0; it < 200; ++it) {
    const double f = 0.5 * std::erfc(z * M_SQRT1_2) - t;
    if (f > 0.0) lo = z; else hi = z;
    const double pdf = std::exp(-0.5 * z * z) * 0.3989422804014326779;
    double zn = (pdf > 1e-300) ? z + f / pdf : 0.5 * (lo + hi);
    if (!(zn > lo && zn < hi)) zn = 0.5 * (lo + hi);
    if (std::fabs(zn - z) <= 1e-16 * std::fmax(1.0, std::fabs(z))) {
      z = zn;
      break;
    }
    z = zn;
  }
  return z;
}

int ilog2_exact(int x) {
  int s = 0;
  while ((1 << s) < x) ++s;
  return ((1 << s) == x) ? s : -1;
}

int validate(const vatt_params& p) {
  if (p.batch <= 0 || p.n_q_heads <= 0 || p.n_kv_heads <= 0 || p.n_max <= 0) return VATT_E_INVALID_ARG;
  if (p.head_dim != 64 && p.head_dim != 128) return VATT_E_UNSUPPORTED_SHAPE;
  if (p.n_q_heads % p.n_kv_heads != 0) return VATT_E_INVALID_ARG;
  const int g = p.n_q_heads / p.n_kv_heads;
  if (g != 1 && g != 2 && g != 4 && g != 8) return VATT_E_UNSUPPORTED_SHAPE;
  if (p.kv_layout != VATT_LAYOUT_CONTIGUOUS && p.kv_layout != VATT_LAYOUT_PAGED) return VATT_E_INVALID_ARG;
  if (p.kv_layout == VATT_LAYOUT_PAGED) {
    if (p.page_size < 8 || p.page_size > 256 || ilog2_exact(p.page_size) < 0) return VATT_E_INVALID_ARG;
    if (p.num_blocks <= 0) return VATT_E_INVALID_ARG;
  }
  if (p.sink < 0 || p.window < 0 || p.topk_abs < 0 || p.base_abs < 0) return VATT_E_INVALID_ARG;
  if (!(p.topk_frac >= 0.f && p.topk_frac <= 1.f) || !(p.base_frac >= 0.f && p.base_frac <= 1.f))
    return VATT_E_INVALID_ARG;
  if (!(p.epsilon > 0.f && p.epsilon < 1.f) || !(p.delta > 0.f && p.delta < 1.f)) return VATT_E_INVALID_ARG;
  if (p.target != VATT_TARGET_D && p.target != VATT_TARGET_N && p.target != VATT_TARGET_SDPA)
    return VATT_E_INVALID_ARG;
  if (!(p.sm_scale >= 0.f) || !std::isfinite(p.sm_scale)) return VATT_E_INVALID_ARG;
  if (!(p.budget_cap_frac > 0.f && p.budget_cap_frac <= 1.f)) return VATT_E_INVALID_ARG;
  if ((int64_t)p.n_max > (int64_t)1 << 24) return VATT_E_UNSUPPORTED_SHAPE;
  return VATT_OK;
}

int build_plan(Plan& pl, const vatt_params& p, int q_len, int device) {
  pl.p = p;
  pl.q_len = q_len;
  pl.vbatch = p.batch * q_len;
  pl.device = device;
  pl.num_cus = 256;
  if (device >= 0) {
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || count <= 0) return VATT_E_NO_DEVICE;
    if (device >= count) return VATT_E_INVALID_ARG;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return VATT_E_HIP;
    pl.num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  }
  pl.group = p.n_q_heads / p.n_kv_heads;
  pl.sm_scale = p.sm_scale > 0.f ? p.sm_scale : (float)(1.0 / std::sqrt((double)p.head_dim));
  pl.eps = (double)p.epsilon;
  pl.cap_frac = (double)p.budget_cap_frac;
  pl.z_half = upper_tail_quantile((double)p.delta / 2.0);
  pl.range_factor = 0.0;
  pl.z_quarter = upper_tail_quantile((double)p.delta / 4.0);
  pl.sel.sink = p.sink;
  pl.sel.window = p.window;
  pl.sel.topk_abs = p.topk_abs;
  pl.sel.base_abs = p.base_abs;
  pl.sel.topk_frac = (double)p.topk_frac;
  pl.sel.base_frac = (double)p.base_frac;
  pl.sampler_small_batches = 0;
  pl.topk_general_path = 0;
  pl.sampler_draw_cap = 0;
  pl.nested_samples = 0;
  pl.budget_multiple = 1;
  pl.ascending_samples = 0;

  // Workgroups go to the eight XCDs round-robin in launch order.  With a multiple of 8 KV heads the selection,
  // gather and merge kernels launch the query heads of a KV head on one XCD (they read the same sink, window and
  // heavy V rows).  The score pass has three launch orders (see its kernel): by measurement the KV-head-major
  // one up to 64K tokens when the KV heads can be dealt out to the XCDs evenly, the blocks order otherwise (the
  // tile-major one is 1 - 2 % behind it and stays for tests).  The multi-query score kernel has one order of
  // its own.
  pl.group_major = (p.n_kv_heads % 8 == 0) ? 1 : 0;
  pl.score_order = (pl.group_major && p.n_max <= 65536) ? kScoreOrderKvHead : kScoreOrderBlocks;
  if (q_len != 1) pl.score_order = kScoreOrderTile;

  const int n_max = p.n_max;
  pl.n_pad = (int)align_up((size_t)n_max, 256);
  pl.n_sub = (int)align_up((size_t)n_max, kScoreTilePaged) / kSubTile;  // whole tiles of either tile size
  int k_max = p.topk_abs > 0 ? p.topk_abs : (int)std::floor((double)p.topk_frac * (double)n_max);
  pl.k_max = std::min(std::max(k_max, 0), n_max);
  int b0_max = p.base_abs > 0 ? p.base_abs : (int)std::floor((double)p.base_frac * (double)n_max);
  pl.b0_max = std::min(std::max(b0_max, 2), n_max);
  const int cap_max = (int)std::min((double)n_max, std::ceil((double)p.budget_cap_frac * (double)n_max));
  pl.b_max = std::max(pl.b0_max, cap_max);
  // random cache: room for the base sample plus the cached tokens that fall into sink, window or top-k
  pl.cache_slots = (int)std::min<size_t>(kCacheSlotsMax, align_up((size_t)pl.b0_max + pl.b0_max / 4 + 64, 64));

  // Rows of up to 32768 tokens keep their 8-key maxima in the registers of 512 threads, and two such workgroups
  // share a CU.  Longer rows get 1024 threads when that costs no parallelism: when only one workgroup fits a
  // CU's LDS anyway, or when there are no more heads than CUs.
  pl.head_threads = kHeadThreads;
  if (n_max > 8 * kHeadThreads * kSubTile &&
      (2 * (head_kernel_lds_bytes(n_max, kHeadThreads) + head_kernel_static_lds_bytes()) > 160 * 1024 ||
       pl.vbatch * p.n_q_heads <= pl.num_cus))
    pl.head_threads = kHeadThreadsLong;

  const int heads = pl.vbatch * p.n_q_heads;
  const int want_blocks = 2 * pl.num_cus;
  // most workgroups per head that any of the gathering kernels uses (sizes the regions of their partial sums)
  pl.split_cap = std::min(32, std::max(1, (32 * pl.num_cus + heads - 1) / heads));
  // measured (gather kernel alone, us, with 4 / 8 / 16 / 32 / 64 workgroups per head): 512 heads 42.4 / 41.2 / 41.3 /
  // 52.7 / 84.7; 128 heads with long lists 32.3 / 31.1 / 30.5 / 32.1 / 33.3; 1024 heads on a paged cache 57.8 /
  // 59.1 / 66.2 / 103.8 / 186.8: 16 workgroups per CU, at most 16 per head
  pl.gather_splits = std::min(16, std::max(1, (16 * pl.num_cus + heads - 1) / heads));
  pl.vstat_splits = pl.gather_splits;
  // (the kernels of the path with a caller-supplied top-k, by measurement: its gather, which also reads K rows
  // and carries running maxima, 16 workgroups per CU and at most 16 per head; its score kernel, which only
  // writes scores, 32 per CU and at most 16 per head.  At 512 heads: 128.5 us per step with 8 and 2 per head,
  // 122.4 us with 16 and 8; at 128 heads 8 to 16 of each are equal; at 32 heads 16 and 16 are best.)
  pl.given_splits = std::min(std::min(pl.split_cap, 16), std::max(1, (16 * pl.num_cus + heads - 1) / heads));
  pl.sparse_splits = std::min(std::min(pl.split_cap, 16), std::max(1, (32 * pl.num_cus + heads - 1) / heads));
  const int kv_heads = pl.vbatch * p.n_kv_heads;
  const int max_dense = std::max(1, (n_max + 255) / 256);
  pl.dense_splits = std::min(std::min(64, max_dense), std::max(1, (2 * want_blocks + kv_heads - 1) / kv_heads));

  pl.fuse_splits = fused_splits_for(pl);
  pl.prework = pl.fuse_splits > 0 ? 1 : 0;
  pl.given_fuse_splits = given_fused_splits_for(pl);

  pl.seg_off[0] = 0;
  pl.seg_off[1] = p.sink;
  pl.seg_off[2] = (int64_t)p.sink + p.window;
  pl.seg_off[3] = pl.seg_off[2] + pl.k_max;
  pl.seg_off[4] = pl.seg_off[3] + pl.b0_max;
  pl.idx_cap = align_up((size_t)(pl.seg_off[4] + pl.b_max), 4);
  pl.head_lds_bytes = head_kernel_lds_bytes(n_max, pl.head_threads);
  if (pl.head_lds_bytes + head_kernel_static_lds_bytes() > 160 * 1024) return VATT_E_UNSUPPORTED_SHAPE;

  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  };
  pl.off_scores = take((size_t)heads * pl.n_pad * sizeof(float));
  pl.off_sub_max = take((size_t)heads * pl.n_sub * sizeof(float));
  pl.off_sparse = take((size_t)heads * pl.idx_cap * sizeof(float));
  pl.off_head_rec = take((size_t)heads * sizeof(HeadRec));
  pl.off_gather_part = take((size_t)heads * std::max(pl.split_cap, 16) * (p.head_dim + 4) * sizeof(float));
  pl.off_debug = take(512 * sizeof(uint64_t));
  pl.off_vstat_part = take((size_t)heads * pl.split_cap * (2 * p.head_dim + 2) * sizeof(double));
  pl.off_dense_part = take((size_t)heads * pl.dense_splits * (p.head_dim + 4) * sizeof(float));
  pl.off_pre_tok = take((size_t)heads * kHeadThreads * sizeof(uint4));
  pl.off_pre_flags = take((size_t)heads * kHeadThreads * sizeof(uint32_t));
  pl.off_base_slot = take((size_t)heads * pl.b0_max * sizeof(int32_t));
  pl.ws_bytes = off;

  KVLayout L;
  std::memset(&L, 0, sizeof(L));
  L.head_dim = p.head_dim;
  if (p.kv_layout == VATT_LAYOUT_PAGED) {
    L.page_shift = ilog2_exact(p.page_size);
    L.pages_per_seq = (n_max + p.page_size - 1) / p.page_size;
    L.num_blocks = p.num_blocks;
    L.head_stride = (int64_t)p.page_size * p.head_dim;
    L.block_stride = (int64_t)p.n_kv_heads * p.page_size * p.head_dim;
  } else {
    L.head_stride = (int64_t)n_max * p.head_dim;
    L.seq_stride = (int64_t)p.n_kv_heads * n_max * p.head_dim;
    L.num_blocks = 1;
  }
  pl.kv_k = L;
  pl.kv_v = L;
  return VATT_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---------------------------------------------------------------------------
// Scratch memory of vatt_decode_static: a device array owned by the library, so that the call needs no
// workspace from the caller and nothing is ever allocated.  Every GPU the library runs on holds its own copy
// at its own address; `scratch` itself is only the host-side handle of the symbol, never a device address:
// resolve_scratch looks the address up once per device and everything else uses that pointer.
// ---------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __attribute__((used)) __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on device i, or null before resolve_scratch(i)
std::mutex g_scratch_mutex;

// To be called with `device` current.
hipError_t resolve_scratch(int device) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[device]) return hipSuccess;
  void* ptr = nullptr;
  const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
  if (e != hipSuccess) return e;
  if (!ptr || (reinterpret_cast<uintptr_t>(ptr) & 255u) != 0) return hipErrorInvalidSymbol;
  g_scratch_ptr[device] = ptr;
  return hipSuccess;
}

void* scratch_of(int device) {
  if (device < 0 || device >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  return g_scratch_ptr[device];
}

int check_common(const vatt_plan* plan, const void* ws, size_t ws_bytes, const int32_t* block_table) {
  if (!plan || !ws) return VATT_E_INVALID_ARG;
  if (plan->pl.device < 0) return VATT_E_NO_DEVICE;
  if (ws_bytes < plan->pl.ws_bytes) return VATT_E_WORKSPACE_TOO_SMALL;
  if ((reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return VATT_E_INVALID_ARG;
  if (plan->pl.p.kv_layout == VATT_LAYOUT_PAGED && !block_table) return VATT_E_INVALID_ARG;
  int cur = -1;
  if (hipGetDevice(&cur) != hipSuccess) return VATT_E_HIP;
  if (cur != plan->pl.device) return VATT_E_HIP;
  return VATT_OK;
}

#define VATT_LAUNCH(expr)                    \
  do {                                       \
    if ((expr) != hipSuccess) return VATT_E_HIP; \
  } while (0)

}  // namespace
}  // namespace vatt

using namespace vatt;

// The step with a caller-supplied top-k set; rcache (or nullptr) is the random cache the base sample may come from.
static int decode_given(const vatt::Plan& pl, const void* q, const void* k, const void* v, const int32_t* block_table,
                        const int32_t* seq_lens, const uint64_t* seq_seeds, const int32_t* topk_idx,
                        const int32_t* topk_cnt, const void* rcache, void* workspace, float* out_o, float* out_lse,
                        int32_t* out_idx, int32_t* out_counts, double* out_budget_raw, float* out_stats,
                        hipStream_t st) {
  using namespace vatt;
  // a supplied set need not hold the largest scores, so it gives no bound on the residual weights
  if (pl.range_factor > 0.0) return VATT_E_UNSUPPORTED_SHAPE;
  if (pl.given_fuse_splits > 0 && !pl.nested_samples && !pl.ascending_samples && pl.p.target == VATT_TARGET_D) {
    // small batches: three launches (selection + scores of I_f and I_bs, selection + gather, merge)
    VATT_LAUNCH(launch_given_fused(pl, 0, q, k, v, block_table, seq_lens, seq_seeds, topk_idx, topk_cnt, rcache,
                                   workspace, out_idx, out_counts, out_budget_raw, out_stats, st));
    VATT_LAUNCH(launch_given_fused(pl, 1, q, k, v, block_table, seq_lens, seq_seeds, topk_idx, topk_cnt, nullptr,
                                   workspace, out_idx, out_counts, out_budget_raw, out_stats, st));
    VATT_LAUNCH(launch_given_merge(pl, workspace, pl.given_fuse_splits, out_o, out_lse, st));
    return VATT_OK;
  }
  VATT_LAUNCH(launch_given_select(pl, 0, seq_lens, seq_seeds, topk_idx, topk_cnt, rcache, workspace, out_idx,
                                  out_counts, out_budget_raw, out_stats, st));
  VATT_LAUNCH(launch_sparse_score(pl, q, k, v, block_table, rcache, workspace, out_idx, st));
  VATT_LAUNCH(launch_given_select(pl, 1, seq_lens, seq_seeds, topk_idx, topk_cnt, nullptr, workspace, out_idx,
                                  out_counts, out_budget_raw, out_stats, st));
  VATT_LAUNCH(launch_given_gather(pl, q, k, v, block_table, workspace, out_idx, out_o, out_lse, st));
  return VATT_OK;
}

extern "C" {

int vatt_plan_create(const vatt_params* params, int device, vatt_plan** out) {
  return vatt_plan_create_chunk(params, 1, device, out);
}

int vatt_plan_create_chunk(const vatt_params* params, int q_len, int device, vatt_plan** out) {
  if (!params || !out) return VATT_E_INVALID_ARG;
  *out = nullptr;
  int rc = validate(*params);
  if (rc != VATT_OK) return rc;
  if (q_len < 1) return VATT_E_INVALID_ARG;
  if (q_len > 256) return VATT_E_UNSUPPORTED_SHAPE;
  if ((int64_t)params->batch * q_len > 65535) return VATT_E_UNSUPPORTED_SHAPE;
  vatt_plan* plan = new (std::nothrow) vatt_plan;
  if (!plan) return VATT_E_INVALID_ARG;
  std::memset(static_cast<void*>(plan), 0, sizeof(*plan));
  rc = build_plan(plan->pl, *params, q_len, device);
  if (rc == VATT_OK && device >= 0) {
    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess) rc = VATT_E_HIP;
    if (rc == VATT_OK && cur != device && hipSetDevice(device) != hipSuccess) rc = VATT_E_HIP;
    if (rc == VATT_OK && set_kernel_attributes(plan->pl) != hipSuccess) rc = VATT_E_HIP;
    if (rc == VATT_OK && resolve_scratch(device) != hipSuccess) rc = VATT_E_HIP;  // for vatt_decode_static
    if (cur >= 0 && cur != device) (void)hipSetDevice(cur);
  }
  if (rc != VATT_OK) {
    vatt_plan_destroy(plan);
    return rc;
  }
  *out = plan;
  return VATT_OK;
}

void vatt_plan_destroy(vatt_plan* plan) { delete plan; }

size_t vatt_plan_workspace_bytes(const vatt_plan* plan) { return plan ? plan->pl.ws_bytes : 0; }

size_t vatt_plan_workspace_offset(const vatt_plan* plan, int region) {
  if (!plan) return (size_t)-1;
  if (region == VATT_WS_SCORES) return plan->pl.off_scores;
  if (region == VATT_WS_DEBUG) return plan->pl.off_debug;
  return (size_t)-1;
}

size_t vatt_plan_score_stride(const vatt_plan* plan) { return plan ? (size_t)plan->pl.n_pad : 0; }

int vatt_plan_query_len(const vatt_plan* plan) { return plan ? plan->pl.q_len : 0; }

size_t vatt_plan_index_capacity(const vatt_plan* plan) { return plan ? plan->pl.idx_cap : 0; }

int64_t vatt_plan_index_segment(const vatt_plan* plan, int segment) {
  if (!plan || segment < 0 || segment > 4) return -1;
  return plan->pl.seg_off[segment];
}

int vatt_plan_set_option(vatt_plan* plan, int option, int value) {
  if (!plan) return VATT_E_INVALID_ARG;
  if (option == VATT_OPT_SAMPLER_SMALL_BATCHES) {
    plan->pl.sampler_small_batches = value ? 1 : 0;
    return VATT_OK;
  }
  if (option == VATT_OPT_TOPK_GENERAL_PATH) {
    plan->pl.topk_general_path = value ? 1 : 0;
    return VATT_OK;
  }
  if (option == VATT_OPT_HEAD_THREADS) {
    Plan& pl = plan->pl;
    if (value != kHeadThreads && value != kHeadThreadsLong) return VATT_E_INVALID_ARG;
    const size_t lds = head_kernel_lds_bytes(pl.p.n_max, value);
    if (lds + head_kernel_static_lds_bytes() > 160 * 1024) return VATT_E_UNSUPPORTED_SHAPE;
    pl.head_threads = value;
    pl.head_lds_bytes = lds;
    if (value != kHeadThreads) pl.fuse_splits = 0;
    if (pl.device >= 0 && set_kernel_attributes(pl) != hipSuccess) return VATT_E_HIP;
    return VATT_OK;
  }
  if (option == VATT_OPT_SCORE_PREWORK) {
    plan->pl.prework = value ? 1 : 0;
    return VATT_OK;
  }
  if (option == VATT_OPT_FUSED_GATHER) {
    if (value != 0 && !fused_splits_fit(plan->pl, value)) return VATT_E_UNSUPPORTED_SHAPE;
    plan->pl.fuse_splits = value;
    return VATT_OK;
  }
  if (option == VATT_OPT_GIVEN_FUSED) {
    if (value != 0 && !given_fused_fits(plan->pl, value)) return VATT_E_UNSUPPORTED_SHAPE;
    plan->pl.given_fuse_splits = value;
    return VATT_OK;
  }
  if (option == VATT_OPT_GIVEN_SPLITS || option == VATT_OPT_SPARSE_SPLITS) {
    if (value < 1 || value > plan->pl.split_cap) return VATT_E_INVALID_ARG;
    (option == VATT_OPT_GIVEN_SPLITS ? plan->pl.given_splits : plan->pl.sparse_splits) = value;
    return VATT_OK;
  }
  if (option == VATT_OPT_CACHE_SLOTS) {
    if (value < 1 || value > kCacheSlotsMax || (value & 3) != 0) return VATT_E_INVALID_ARG;
    plan->pl.cache_slots = value;
    return VATT_OK;
  }
  if (option == VATT_OPT_ASCENDING_SAMPLES) {
    plan->pl.ascending_samples = value ? 1 : 0;
    return VATT_OK;
  }
  if (option == VATT_OPT_NESTED_SAMPLES) {
    plan->pl.nested_samples = value ? 1 : 0;
    return VATT_OK;
  }
  if (option == VATT_OPT_BUDGET_BOUND) {
    Plan& pl = plan->pl;
    if (value == VATT_BOUND_CLT) {
      pl.z_half = upper_tail_quantile((double)pl.p.delta / 2.0);
      pl.range_factor = 0.0;
      return VATT_OK;
    }
    if (value != VATT_BOUND_HOEFFDING && value != VATT_BOUND_HOEFFDING_RANGE) return VATT_E_INVALID_ARG;
    if (pl.p.target != VATT_TARGET_D) return VATT_E_UNSUPPORTED_SHAPE;
    if (value == VATT_BOUND_HOEFFDING_RANGE) {
      // Hoeffding's inequality for weights in [0, R]: 2 exp(-2 b t^2 / R^2) <= delta
      pl.range_factor = 0.5 * std::log(2.0 / (double)pl.p.delta);
      return VATT_OK;
    }
    // sub-Gaussian tail 2 exp(-b t^2 / (2 sigma^2)) <= delta in place of the normal quantile
    pl.z_half = std::sqrt(2.0 * std::log(2.0 / (double)pl.p.delta));
    pl.range_factor = 0.0;
    return VATT_OK;
  }
  if (option == VATT_OPT_BUDGET_MULTIPLE) {
    if (value < 1 || value > 65536) return VATT_E_INVALID_ARG;
    plan->pl.budget_multiple = value;
    return VATT_OK;
  }
  if (option == VATT_OPT_SCORE_ORDER) {
    if (value != kScoreOrderTile && value != kScoreOrderKvHead && value != kScoreOrderBlocks) return VATT_E_INVALID_ARG;
    if (plan->pl.q_len != 1 && value != kScoreOrderTile) return VATT_E_UNSUPPORTED_SHAPE;
    plan->pl.score_order = value;
    return VATT_OK;
  }
  if (option == VATT_OPT_SAMPLER_DRAW_CAP) {
    if (value < 0) return VATT_E_INVALID_ARG;
    plan->pl.sampler_draw_cap = (uint32_t)value;
    return VATT_OK;
  }
  return VATT_E_INVALID_ARG;
}

int vatt_score(vatt_plan* plan, const void* q, const void* k, const int32_t* block_table, const int32_t* seq_lens,
               void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_common(plan, workspace, workspace_bytes, block_table);
  if (rc != VATT_OK) return rc;
  if (!q || !k || !seq_lens || !aligned16(q) || !aligned16(k)) return VATT_E_INVALID_ARG;
  if (plan->pl.q_len > 1)
    VATT_LAUNCH(launch_score_chunk(plan->pl, q, k, block_table, seq_lens, workspace, static_cast<hipStream_t>(stream)));
  else
    VATT_LAUNCH(launch_score(plan->pl, q, k, block_table, seq_lens, nullptr, workspace, static_cast<hipStream_t>(stream)));
  return VATT_OK;
}

size_t vatt_static_scratch_bytes(void) { return kStaticScratchBytes; }

int vatt_decode_static(vatt_plan* plan, const void* q, const void* k, const void* v, const int32_t* block_table,
                       const int32_t* seq_lens, const uint64_t* seq_seeds, float* out_o, float* out_lse,
                       int32_t* out_idx, int32_t* out_counts, double* out_budget_raw, float* out_stats,
                       void* stream) {
  if (!plan) return VATT_E_INVALID_ARG;
  if (plan->pl.device < 0) return VATT_E_NO_DEVICE;
  if (plan->pl.ws_bytes > kStaticScratchBytes) return VATT_E_WORKSPACE_TOO_SMALL;
  void* ws = scratch_of(plan->pl.device);  // found by vatt_plan_create for this device
  if (!ws) return VATT_E_HIP;
  return vatt_decode(plan, q, k, v, block_table, seq_lens, seq_seeds, ws, kStaticScratchBytes, out_o, out_lse,
                     out_idx, out_counts, out_budget_raw, out_stats, stream);
}

int vatt_decode(vatt_plan* plan, const void* q, const void* k, const void* v, const int32_t* block_table,
                const int32_t* seq_lens, const uint64_t* seq_seeds, void* workspace, size_t workspace_bytes,
                float* out_o, float* out_lse, int32_t* out_idx, int32_t* out_counts, double* out_budget_raw,
                float* out_stats, void* stream) {
  int rc = check_common(plan, workspace, workspace_bytes, block_table);
  if (rc != VATT_OK) return rc;
  if (!q || !k || !v || !seq_lens || !seq_seeds || !out_o || !out_idx || !out_counts) return VATT_E_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v)) return VATT_E_INVALID_ARG;
  const Plan& pl = plan->pl;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool fused = pl.p.target == VATT_TARGET_D && pl.fuse_splits > 0 && !pl.nested_samples && !pl.ascending_samples;
  if (pl.q_len > 1)
    VATT_LAUNCH(launch_score_chunk(pl, q, k, block_table, seq_lens, workspace, st));
  else
    VATT_LAUNCH(launch_score(pl, q, k, block_table, seq_lens, seq_seeds, workspace, st));
  if (fused) {
    // small batch: selection and gather in one kernel, several workgroups per head
    VATT_LAUNCH(launch_head_fused(pl, v, block_table, seq_lens, seq_seeds, workspace, out_idx, out_counts,
                                  out_budget_raw, out_stats, score_prework(pl), st));
    VATT_LAUNCH(launch_gather_merge(pl, workspace, pl.fuse_splits, out_o, out_lse, st));
    return VATT_OK;
  }
  if (pl.p.target == VATT_TARGET_D) {
    VATT_LAUNCH(launch_head(pl, 0, seq_lens, seq_seeds, workspace, out_idx, out_counts, out_budget_raw, out_stats, st));
  } else {
    VATT_LAUNCH(launch_head(pl, 1, seq_lens, seq_seeds, workspace, out_idx, out_counts, out_budget_raw, out_stats, st));
    VATT_LAUNCH(launch_vstats(pl, v, block_table, workspace, out_idx, st));
    VATT_LAUNCH(launch_head(pl, 2, seq_lens, seq_seeds, workspace, out_idx, out_counts, out_budget_raw, out_stats, st));
  }
  VATT_LAUNCH(launch_gather(pl, v, block_table, workspace, out_idx, out_o, out_lse, st));
  return VATT_OK;
}

int vatt_decode_given_topk(vatt_plan* plan, const void* q, const void* k, const void* v, const int32_t* block_table,
                           const int32_t* seq_lens, const uint64_t* seq_seeds, const int32_t* topk_idx,
                           const int32_t* topk_cnt, void* workspace, size_t workspace_bytes, float* out_o,
                           float* out_lse, int32_t* out_idx, int32_t* out_counts, double* out_budget_raw,
                           float* out_stats, void* stream) {
  int rc = check_common(plan, workspace, workspace_bytes, block_table);
  if (rc != VATT_OK) return rc;
  if (!q || !k || !v || !seq_lens || !seq_seeds || !topk_idx || !topk_cnt || !out_o || !out_idx || !out_counts)
    return VATT_E_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v)) return VATT_E_INVALID_ARG;
  return decode_given(plan->pl, q, k, v, block_table, seq_lens, seq_seeds, topk_idx, topk_cnt, nullptr, workspace, out_o,
                      out_lse, out_idx, out_counts, out_budget_raw, out_stats, static_cast<hipStream_t>(stream));
}

size_t vatt_random_cache_bytes(const vatt_plan* plan) {
  if (!plan) return 0;
  return (size_t)cache_layout(plan->pl).rec_bytes * (size_t)plan->pl.p.batch * (size_t)plan->pl.p.n_kv_heads;
}

int vatt_random_cache_slots(const vatt_plan* plan) { return plan ? plan->pl.cache_slots : 0; }

int vatt_random_cache_fill(vatt_plan* plan, const void* k, const void* v, const int32_t* block_table,
                           const int32_t* seq_lens, const uint64_t* cache_seeds, void* rcache, void* stream) {
  if (!plan) return VATT_E_INVALID_ARG;
  if (plan->pl.device < 0) return VATT_E_NO_DEVICE;
  if (plan->pl.p.kv_layout == VATT_LAYOUT_PAGED && !block_table) return VATT_E_INVALID_ARG;
  if (!k || !v || !seq_lens || !cache_seeds || !rcache) return VATT_E_INVALID_ARG;
  if (!aligned16(k) || !aligned16(v) || (reinterpret_cast<uintptr_t>(rcache) & 255u) != 0) return VATT_E_INVALID_ARG;
  VATT_LAUNCH(launch_cache_fill(plan->pl, k, v, block_table, seq_lens, cache_seeds, rcache,
                                static_cast<hipStream_t>(stream)));
  return VATT_OK;
}

int vatt_append_kv_cached(vatt_plan* plan, const void* k_new, const void* v_new, void* k, void* v,
                          const int32_t* block_table, int32_t* seq_lens, const uint64_t* cache_seeds, void* rcache,
                          void* stream) {
  if (!plan) return VATT_E_INVALID_ARG;
  if (plan->pl.device < 0) return VATT_E_NO_DEVICE;
  if (plan->pl.p.kv_layout == VATT_LAYOUT_PAGED && !block_table) return VATT_E_INVALID_ARG;
  if (!k_new || !v_new || !k || !v || !seq_lens || !cache_seeds || !rcache) return VATT_E_INVALID_ARG;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k) || !aligned16(v) ||
      (reinterpret_cast<uintptr_t>(rcache) & 255u) != 0)
    return VATT_E_INVALID_ARG;
  VATT_LAUNCH(launch_append_cached(plan->pl, k_new, v_new, k, v, block_table, seq_lens, cache_seeds, rcache,
                                   static_cast<hipStream_t>(stream)));
  return VATT_OK;
}

int vatt_decode_given_topk_cached(vatt_plan* plan, const void* q, const void* k, const void* v,
                                  const int32_t* block_table, const int32_t* seq_lens, const uint64_t* seq_seeds,
                                  const int32_t* topk_idx, const int32_t* topk_cnt, const void* rcache,
                                  void* workspace, size_t workspace_bytes, float* out_o, float* out_lse,
                                  int32_t* out_idx, int32_t* out_counts, double* out_budget_raw, float* out_stats,
                                  void* stream) {
  int rc = check_common(plan, workspace, workspace_bytes, block_table);
  if (rc != VATT_OK) return rc;
  if (!q || !k || !v || !seq_lens || !seq_seeds || !topk_idx || !topk_cnt || !rcache || !out_o || !out_idx || !out_counts)
    return VATT_E_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || (reinterpret_cast<uintptr_t>(rcache) & 255u) != 0)
    return VATT_E_INVALID_ARG;
  // the cache belongs to single-token steps of whole sequences, and its entries come in slot order
  if (plan->pl.q_len != 1 || plan->pl.ascending_samples) return VATT_E_UNSUPPORTED_SHAPE;
  return decode_given(plan->pl, q, k, v, block_table, seq_lens, seq_seeds, topk_idx, topk_cnt, rcache, workspace, out_o,
                      out_lse, out_idx, out_counts, out_budget_raw, out_stats, static_cast<hipStream_t>(stream));
}

int vatt_random_cache_read(vatt_plan* plan, const void* rcache, int32_t* out_tokens, int32_t* out_counts,
                           void* stream) {
  if (!plan || !rcache || !out_tokens || !out_counts) return VATT_E_INVALID_ARG;
  if (plan->pl.device < 0) return VATT_E_NO_DEVICE;
  VATT_LAUNCH(launch_cache_read(plan->pl, rcache, out_tokens, out_counts, static_cast<hipStream_t>(stream)));
  return VATT_OK;
}

int vatt_dense_decode(vatt_plan* plan, const void* q, const void* k, const void* v, const int32_t* block_table,
                      const int32_t* seq_lens, void* workspace, size_t workspace_bytes, float* out_o,
                      float* out_lse, void* stream) {
  int rc = check_common(plan, workspace, workspace_bytes, block_table);
  if (rc != VATT_OK) return rc;
  if (!q || !k || !v || !seq_lens || !out_o) return VATT_E_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v)) return VATT_E_INVALID_ARG;
  VATT_LAUNCH(launch_dense(plan->pl, q, k, v, block_table, seq_lens, workspace, out_o, out_lse,
                           static_cast<hipStream_t>(stream)));
  return VATT_OK;
}

int vatt_host_kv_device_pointer(const void* host_ptr, void** device_ptr) {
  if (!host_ptr || !device_ptr) return VATT_E_INVALID_ARG;
  *device_ptr = nullptr;
  hipPointerAttribute_t attr;
  if (hipPointerGetAttributes(&attr, host_ptr) != hipSuccess) {
    (void)hipGetLastError();  // ordinary process memory: not an error of the runtime's state, just not usable
    return VATT_E_INVALID_ARG;
  }
  if (attr.type != hipMemoryTypeHost) return VATT_E_INVALID_ARG;
  void* dev = nullptr;
  if (hipHostGetDevicePointer(&dev, const_cast<void*>(host_ptr), 0) != hipSuccess || !dev) {
    (void)hipGetLastError();
    return VATT_E_INVALID_ARG;
  }
  *device_ptr = dev;
  return VATT_OK;
}

int vatt_stream_read(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !sink || !aligned16(src) || (bytes & 15u) != 0) return VATT_E_INVALID_ARG;
  VATT_LAUNCH(launch_stream_read(src, bytes, sink, static_cast<hipStream_t>(stream)));
  return VATT_OK;
}

int vatt_row_read(const void* src, size_t rows_total, const int32_t* rows, size_t count, void* sink, void* stream) {
  if (!src || !rows || !sink || !aligned16(src) || rows_total == 0) return VATT_E_INVALID_ARG;
  VATT_LAUNCH(launch_row_read(src, rows_total, rows, count, sink, static_cast<hipStream_t>(stream)));
  return VATT_OK;
}

int vatt_append_kv(vatt_plan* plan, const void* k_new, const void* v_new, void* k, void* v,
                   const int32_t* block_table, int32_t* seq_lens, void* stream) {
  if (!plan) return VATT_E_INVALID_ARG;
  if (plan->pl.device < 0) return VATT_E_NO_DEVICE;
  if (plan->pl.p.kv_layout == VATT_LAYOUT_PAGED && !block_table) return VATT_E_INVALID_ARG;
  if (!k_new || !v_new || !k || !v || !seq_lens) return VATT_E_INVALID_ARG;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k) || !aligned16(v)) return VATT_E_INVALID_ARG;
  VATT_LAUNCH(launch_append(plan->pl, k_new, v_new, k, v, block_table, seq_lens, static_cast<hipStream_t>(stream)));
  return VATT_OK;
}

const char* vatt_status_string(int status) {
  switch (status) {
    case VATT_OK: return "ok";
    case VATT_E_INVALID_ARG: return "invalid argument";
    case VATT_E_UNSUPPORTED_SHAPE: return "unsupported shape";
    case VATT_E_WORKSPACE_TOO_SMALL: return "workspace too small";
    case VATT_E_HIP: return "HIP runtime error";
    case VATT_E_NO_DEVICE: return "no usable HIP device";
    default: return "unknown status";
  }
}

}  // extern "C"
