// Score pass: s_i = sm_scale * <K[i], q_h> for every key and every query head of the GQA group,
// reading each K row from HBM once per group (first step of Algorithm 1 with exact top-k; the
// exponent of Eq. 1).
//
// Work split: a workgroup of 4 waves owns TILE consecutive keys of one KV head (64 on a contiguous cache, 256 on
// a paged one, by measurement).  Workgroups go to the chip's eight XCDs round-robin in launch order, so the
// launch order decides which XCD reads which tile and writes which piece of a score row.  Three orders:
//   tile-major, grid = (key tiles, KV heads, sequences): neighbouring workgroups stream neighbouring memory and
//     the eight XCDs take turns along every row;
//   KV-head-major, grid = (KV heads, key tiles, sequences), for plans whose KV head count is a multiple of 8:
//     all tiles of KV head j run on XCD j mod 8, which streams that head's K rows front to back and writes
//     whole score rows;
//   blocks: tile-major, but the XCDs take turns in blocks of 256 KiB of K (16 tiles of 64 keys at d = 128)
//     instead of single tiles, so each writes runs of 4 KiB of every score row while all XCDs still work on
//     the same KV head; which XCD starts a row rotates with the KV head and the sequence (short sequences have
//     first blocks only: without the rotation a ragged paged batch ran 3.7 % slower than tile by tile).  (A read-only probe reads such blocks as fast as single tiles; blocks of 64 KiB, or of
//     4 MiB and more, read 6 - 8 % slower.)
// Measured (whole call): KV-head-major is the best order up to 64K tokens (2 - 4 % under tile-major at 8K - 32K,
// 7 % at 64K and batch 1), and 3 % behind it at 128K; blocks is 1 - 2 % under tile-major at every size tried,
// equal to KV-head-major at 32K and batch 16 and behind it at batch 1, and as good as tile-major on a ragged
// batch (an earlier form that gave every XCD one eighth of a row left the short sequences of a ragged batch to
// one XCD: 63 % slower).  The plan picks KV-head-major up to 64K tokens when it can deal the KV heads out to
// the XCDs evenly, and blocks otherwise.  (A read-only kernel loses 5 - 8 % in the KV-head-major pattern: the gain is on the write side.
// And nothing written here is still in an L2 when the next kernel reads it: the selection kernel's L2 hits and
// misses are the same in every order.)  A K row of d bf16 values is read by d/8 adjacent lanes with one 16-byte load
// each, so a wave instruction covers 4 (d = 128) or 8 (d = 64) whole rows as one contiguous 1 KiB
// segment.  Each lane multiplies its 8 columns with the matching 8 columns of the G queries
// (bf16 pair dot-products accumulating in fp32), the partial sums are added across the d/8 lanes on
// the DPP path, and the tile's G x TILE scores are staged in LDS so that they leave as whole
// 256-byte rows; the largest score of every 8 keys is written next to them.
#include <cstring>
#include <utility>

#include "vatt_internal.h"
#include "vatt_sampler.h"

namespace vatt {
namespace {

// Tiles per block of the blocks order: 256 KiB of K rows.
constexpr int score_block_tiles(int d, int tile) {
  const int t = (256 * 1024) / (tile * d * 2);
  return t > 0 ? t : 1;
}

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), acc,
                                         false);
}

template <int D, int G, bool PAGED, int TILE>
__global__ __launch_bounds__(256) void score_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                    KVLayout L, const int32_t* __restrict__ seq_lens,
                                                    float* __restrict__ scores, float* __restrict__ sub_max,
                                                    int n_sub, int n_pad, int n_max, int Hq, float sm_scale, int order,
                                                    PreArgs pre) {
  constexpr int LPR = D / 8;             // lanes per K row
  constexpr int RPW = kWave / LPR;       // rows per wave load
  constexpr int ROWS_PER_WAVE = TILE / 4;
  constexpr int LOADS = ROWS_PER_WAVE / RPW;
  constexpr int BATCH = LOADS < 8 ? LOADS : 8;

  // grid = (tiles, KV heads, sequences); (KV heads, tiles, sequences) in the KV-head-major order; in the blocks
  // order blockIdx.x = 8 k + x stands for tile k mod BL of block 8 (k / BL) + (x + KV head + sequence) mod 8
  // (gridDim.x: a multiple of 8 BL; the rotation spreads the first blocks, all that a short sequence has, over
  // the XCDs)
  constexpr int BL = score_block_tiles(D, TILE);
  // KV-head-major order with sampler pre-work: the first pre.job_rows rows of the grid (the workgroups that
  // start first) each make the first batch of draws of one (head, stream) and are done
  if (pre.job_rows > 0 && (int)blockIdx.y < pre.job_rows) {
    extern __shared__ __align__(16) unsigned char pre_smem[];
    const int job = (int)blockIdx.y * (int)gridDim.x + (int)blockIdx.x;
    if (job < 2 * Hq) prework_job(pre, (int)blockIdx.z, job >> 1, job & 1, pre_smem);
    return;
  }
  const int kvh = order == kScoreOrderKvHead ? blockIdx.x : blockIdx.y, b = blockIdx.z;
  const int tile = order == kScoreOrderKvHead ? (int)blockIdx.y - pre.job_rows
                   : order == kScoreOrderBlocks
                       ? (int)((((blockIdx.x / 8) / BL) * 8 + (blockIdx.x + blockIdx.y + blockIdx.z) % 8) * BL +
                               (blockIdx.x / 8) % BL)
                       : (int)blockIdx.x;
  const int tile_lo = tile * TILE;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = lane % LPR;   // which 8-column slice of the row
  const int rsub = lane / LPR;  // which row of the wave load
  // On a paged cache the block-table entries of the first rows are requested before the sequence length is
  // looked at (entries beyond it are never used): one link less in the chain length -> table -> K row.
  int64_t first_off[PAGED ? BATCH : 1];
  if constexpr (PAGED) {
#pragma unroll
    for (int u = 0; u < BATCH; ++u)
      first_off[u] = kv_row_offset<true>(L, b, kvh, min(tile_lo + wave * ROWS_PER_WAVE + u * RPW + rsub, n_max - 1));
  }
  const int n = min(max(seq_lens[b], 1), n_max);  // lengths outside [1, n_max] are clamped, as in every kernel
  if (tile_lo >= n) return;

  __shared__ float s_tile[G][TILE];

  uint32_t qw[G][4];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const uint4 t = *reinterpret_cast<const uint4*>(q + ((int64_t)b * Hq + (int64_t)kvh * G + g) * D + sub * 8);
    qw[g][0] = t.x;
    qw[g][1] = t.y;
    qw[g][2] = t.z;
    qw[g][3] = t.w;
  }

#pragma unroll
  for (int u0 = 0; u0 < LOADS; u0 += BATCH) {
    uint4 kv[BATCH];
    // (paged cache: the block-table entries of a batch are requested together, outside the test on the row
    // index; inside it, every row's entry would be awaited before the next row's is requested)
    int64_t off[BATCH];
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
      const int i = tile_lo + wave * ROWS_PER_WAVE + (u0 + u) * RPW + rsub;
      if constexpr (PAGED) off[u] = u0 == 0 ? first_off[u] : kv_row_offset<true>(L, b, kvh, min(i, n_max - 1));
      else off[u] = kv_row_offset<false>(L, b, kvh, i);
    }
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
      const int i = tile_lo + wave * ROWS_PER_WAVE + (u0 + u) * RPW + rsub;
      kv[u] = make_uint4(0u, 0u, 0u, 0u);
      if (i < n) kv[u] = load_stream_16(k + off[u] + sub * 8);
    }
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
      const int row = wave * ROWS_PER_WAVE + (u0 + u) * RPW + rsub;
      float mine = 0.f;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float a = 0.f;
        a = dot2_bf16(kv[u].x, qw[g][0], a);
        a = dot2_bf16(kv[u].y, qw[g][1], a);
        a = dot2_bf16(kv[u].z, qw[g][2], a);
        a = dot2_bf16(kv[u].w, qw[g][3], a);
        a = group_sum<LPR>(a);
        if (sub == g) mine = a;
      }
      // adding +0 folds a possible -0 into +0 so that the bit pattern orders like the value
      if (sub < G) s_tile[sub][row] = mine * sm_scale + 0.0f;
    }
  }
  __syncthreads();
  for (int t = tid; t < TILE; t += 256) {
    const int i = tile_lo + t;
    if (i < n) {
#pragma unroll
      for (int g = 0; g < G; ++g)
      {
        // tile-major order: a row's neighbouring tiles are written by other XCDs, non-temporal stores are best;
        // the other orders: this XCD writes long runs of the row, plain stores measured up to 3 % faster
        float* dst = &scores[((int64_t)b * Hq + (int64_t)kvh * G + g) * n_pad + i];
        if (order != kScoreOrderTile) *dst = s_tile[g][t]; else __builtin_nontemporal_store(s_tile[g][t], dst);
      }
    }
  }
  // Largest score of every 8 consecutive keys per query head: the selection kernel takes its head maximum
  // and a lower bound of the top-k threshold from these.
  static_assert(TILE % kWave == 0 && kSubTile == 8, "whole waves of keys, eight lanes per sub-tile");
  constexpr int CHUNKS = TILE / kWave;
  for (int c = wave; c < G * CHUNKS; c += 4) {
    const int g = c / CHUNKS, t = (c % CHUNKS) * kWave + lane;
    const float v = group_max8(tile_lo + t < n ? s_tile[g][t] : -INFINITY);
    if ((lane & 7) == 0) {
      const int64_t slot = ((int64_t)b * Hq + (int64_t)kvh * G + g) * n_sub + (tile_lo + t) / kSubTile;
      sub_max[slot] = v;
    }
  }
}

// The launch grid of an order, from the tile-major one (tiles, KV heads, sequences).
inline void shape_grid(dim3& grid, int order, int block_tiles) {
  if (order == kScoreOrderKvHead) std::swap(grid.x, grid.y);
  if (order == kScoreOrderBlocks) {  // whole groups of eight blocks; tiles beyond the last one exit at once
    const unsigned g = 8u * (unsigned)block_tiles;
    grid.x = (grid.x + g - 1) / g * g;
  }
}

template <int D, int G>
hipError_t launch_dg(const Plan& pl, const void* q, const void* k, const int32_t* block_table,
                     const int32_t* seq_lens, const uint64_t* seq_seeds, void* ws, hipStream_t st) {
  const vatt_params& p = pl.p;
  PreArgs pre;
  memset(&pre, 0, sizeof(pre));
  size_t lds = 0;
  int job_rows = 0;
  if (score_prework(pl) && seq_seeds) {
    char* w = static_cast<char*>(ws);
    pre.seq_lens = seq_lens;
    pre.seq_seeds = seq_seeds;
    pre.pre_tok = reinterpret_cast<uint4*>(w + pl.off_pre_tok);
    pre.pre_flags = reinterpret_cast<uint32_t*>(w + pl.off_pre_flags);
    pre.sp = pl.sel;
    pre.n_max = p.n_max;
    pre.Hq = p.n_q_heads;
    pre.small_batches = pl.sampler_small_batches;
    pre.draw_cap = pl.sampler_draw_cap;
    job_rows = (2 * p.n_q_heads + p.n_kv_heads - 1) / p.n_kv_heads;  // grid rows of n_kv_heads workgroups
    pre.job_rows = job_rows;
    lds = prework_lds_bytes(p.n_max);
  }

  KVLayout L = pl.kv_k;
  L.block_table = block_table;
  float* scores = reinterpret_cast<float*>(static_cast<char*>(ws) + pl.off_scores);
  float* smax = reinterpret_cast<float*>(static_cast<char*>(ws) + pl.off_sub_max);
  // (measured: 64-key tiles stream a contiguous cache best; a paged cache, whose workgroups first wait for their
  // block-table entries, does better with 256 keys in flight per workgroup)
  if (p.kv_layout == VATT_LAYOUT_PAGED) {
    dim3 grid((p.n_max + kScoreTilePaged - 1) / kScoreTilePaged, p.n_kv_heads, p.batch);
    shape_grid(grid, pl.score_order, score_block_tiles(D, kScoreTilePaged));
    grid.y += job_rows;  // (only set in the KV-head-major order, where y runs over the tiles)
    hipLaunchKernelGGL((score_kernel<D, G, true, kScoreTilePaged>), grid, dim3(256), lds, st,
                       static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k), L, seq_lens, scores, smax,
                       pl.n_sub, pl.n_pad, p.n_max, p.n_q_heads, pl.sm_scale, pl.score_order, pre);
  } else {
    dim3 grid((p.n_max + kScoreTile - 1) / kScoreTile, p.n_kv_heads, p.batch);
    shape_grid(grid, pl.score_order, score_block_tiles(D, kScoreTile));
    grid.y += job_rows;
    hipLaunchKernelGGL((score_kernel<D, G, false, kScoreTile>), grid, dim3(256), lds, st,
                       static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k), L, seq_lens, scores, smax,
                       pl.n_sub, pl.n_pad, p.n_max, p.n_q_heads, pl.sm_scale, pl.score_order, pre);
  }
  return hipGetLastError();
}

template <int D>
hipError_t launch_d(const Plan& pl, const void* q, const void* k, const int32_t* block_table,
                    const int32_t* seq_lens, const uint64_t* seq_seeds, void* ws, hipStream_t st) {
  switch (pl.group) {
    case 1: return launch_dg<D, 1>(pl, q, k, block_table, seq_lens, seq_seeds, ws, st);
    case 2: return launch_dg<D, 2>(pl, q, k, block_table, seq_lens, seq_seeds, ws, st);
    case 4: return launch_dg<D, 4>(pl, q, k, block_table, seq_lens, seq_seeds, ws, st);
    case 8: return launch_dg<D, 8>(pl, q, k, block_table, seq_lens, seq_seeds, ws, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

hipError_t launch_score(const Plan& pl, const void* q, const void* k, const int32_t* block_table,
                        const int32_t* seq_lens, const uint64_t* seq_seeds, void* ws, hipStream_t st) {
  if (pl.p.head_dim == 128) return launch_d<128>(pl, q, k, block_table, seq_lens, seq_seeds, ws, st);
  if (pl.p.head_dim == 64) return launch_d<64>(pl, q, k, block_table, seq_lens, seq_seeds, ws, st);
  return hipErrorInvalidValue;
}

}  // namespace vatt
