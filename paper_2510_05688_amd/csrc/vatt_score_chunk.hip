// Score pass of a multi-query step: the q_len newest tokens of every sequence are queries (the question
// tokens of the evaluation set-up in which only the context is processed densely), and every K row is read
// from HBM once for all of them and for all query heads of the GQA group.
//
// With Q query tokens and G heads per KV head, a K tile meets Q * G query vectors: a dense contraction
// [keys x d] . [d x (Q G)], which goes to the matrix cores.  One wave owns 16-key tiles; the MFMA
// v_mfma_f32_16x16x32_bf16 multiplies a 16 x 32 slice of K (A operand: lane l holds row l % 16, eight
// consecutive columns starting at 8 (l / 16)) with a 32 x 16 slice of the transposed queries (B operand: lane
// l holds query l % 16, the same eight columns) and accumulates 16 x 16 scores in fp32 (lane l: keys
// 4 (l / 16) .. + 3 of query l % 16); d / 32 instructions cover a row.  Products of bf16 values are exact
// in fp32, so only the order of the fp32 additions differs from the single-query kernel.
//
// Query token t of a sequence of n tokens sees n - (Q - 1 - t) of them; later keys are left out of its score
// row and of its 8-key maxima (they enter as -inf), which is all the causal mask needs: the selection kernel
// never looks beyond a row's own length.
//
// grid = (key tiles, KV heads, sequences).  Every wave owns 64 keys and works alone (no workgroup barrier):
// it requests its K rows, turns them into A operands through a small LDS tile of its own, and takes the query
// vectors 16 at a time (NQT groups) with the K fragments staying in registers.  The 16 x 64 scores of a group
// are staged in LDS so that they leave as whole 256-byte rows, with the largest of every 8 keys beside them,
// exactly as the single-query kernel leaves them.  The LDS executes the instructions of one wave in order, so
// a wave's own writes and reads of its tiles need no barrier.
#include <algorithm>

#include "vatt_internal.h"

namespace vatt {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kChunkWaveKeys = 64;  // keys per wave: four 16-key MFMA tiles
constexpr int kChunkWaves = 2;      // waves per workgroup; the waves do not interact (measured: 1, 2, 4 within 3 %)
constexpr int kChunkTile = kChunkWaveKeys * kChunkWaves;

template <int D, bool PAGED, int NQT>
__global__ __launch_bounds__(64 * kChunkWaves) void score_chunk_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, KVLayout L,
    const int32_t* __restrict__ seq_lens, float* __restrict__ scores, float* __restrict__ sub_max, int n_sub,
    int n_pad, int n_max, int Hq, int G, int Q, float sm_scale) {
  constexpr int S = D / 32;                 // MFMA steps per row
  constexpr int KT = kChunkWaveKeys / 16;   // 16-key tiles per wave
  constexpr int LD = kChunkWaveKeys + 4;    // LDS row stride in floats: 16-byte aligned, rows 4 banks apart
  static_assert(kSubTile == 8, "eight lanes per sub-tile");

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int kvh = blockIdx.y, b = blockIdx.z;
  const int n_b = min(max(seq_lens[b], 1), n_max);  // the newest query sees all of it
  const int tile_lo = (blockIdx.x * kChunkWaves + wave) * kChunkWaveKeys;
  if (tile_lo >= n_b) return;  // (no workgroup barrier below: every wave works alone)

  const int i16 = lane & 15, g4 = lane >> 4;
  const int QG = Q * G;

  // staging tile of this wave: 16 queries x 64 keys.  Only this wave touches it, and the LDS executes one
  // wave's instructions in order, so no barrier separates its writes from its reads.
  __shared__ __align__(16) float s_all[kChunkWaves][16][LD];
  float (*s_tile)[LD] = s_all[wave];

  // B operands: query vector c = t * G + g of this KV head, for c = c0 + 16 nt + i16.  16 NQT query vectors
  // are held at a time; a step with more of them takes them in rounds, with the K fragments staying put.
  uint4 bq[NQT][S];
  auto load_queries = [&](int c0) {
#pragma unroll
    for (int nt = 0; nt < NQT; ++nt) {
      const int c = c0 + nt * 16 + i16;
      const int t = c / G, g = c - t * G;
      const uint16_t* src = q + (((int64_t)b * Q + t) * Hq + (int64_t)kvh * G + g) * D + g4 * 8;
#pragma unroll
      for (int s = 0; s < S; ++s)
        bq[nt][s] = c < QG ? *reinterpret_cast<const uint4*>(src + s * 32) : make_uint4(0u, 0u, 0u, 0u);
    }
  };
  load_queries(0);

  // K rows are requested the way memory likes them: D/8 adjacent lanes read one whole row, so a wave
  // instruction covers 64 * 16 contiguous bytes (measured 12 % faster than loading the MFMA layout directly,
  // which touches 16 rows with 64 bytes each per instruction).
  constexpr int LPR = D / 8;        // lanes per row = 16-byte chunks per row
  constexpr int RPI = kWave / LPR;  // rows per wave instruction; 16 / RPI == S instructions per 16-key tile
  static_assert(16 / RPI == S, "a 16-key tile takes as many row loads as MFMA steps");
  const int lrow = lane / LPR, lchunk = lane % LPR;
  uint4 kc[KT][S];
  // (row offsets first, for all rows and outside the test on the row index: on a paged cache each takes a
  // block-table entry, and inside the test every row's entry would be awaited before the next row's is requested)
  int64_t koff[KT][S];
#pragma unroll
  for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
    for (int s = 0; s < S; ++s)
      koff[kt][s] = kv_row_offset<PAGED>(L, b, kvh, min(tile_lo + kt * 16 + s * RPI + lrow, n_b - 1));
  }
#pragma unroll
  for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
    for (int s = 0; s < S; ++s) {
      const int i = tile_lo + kt * 16 + s * RPI + lrow;
      kc[kt][s] = make_uint4(0u, 0u, 0u, 0u);
      if (i < n_b) kc[kt][s] = load_stream_16(k + koff[kt][s] + lchunk * 8);
    }
  }
  // ... and turned into A operands through a 16-row LDS tile of this wave (row stride LPR + 1 chunks keeps both
  // the row-wise writes and the column-wise reads off each other's banks): lane l then holds row l % 16,
  // chunks 4 s + l / 16.
  __shared__ uint4 t_all[kChunkWaves][16 * (LPR + 1)];
  uint4* t_tile = t_all[wave];
  uint4 ka[KT][S];
#pragma unroll
  for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
    for (int s = 0; s < S; ++s) t_tile[(s * RPI + lrow) * (LPR + 1) + lchunk] = kc[kt][s];
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int s = 0; s < S; ++s) ka[kt][s] = t_tile[i16 * (LPR + 1) + s * 4 + g4];
    __builtin_amdgcn_wave_barrier();
  }

  for (int c0 = 0; c0 < QG; c0 += 16 * NQT) {
  if (c0 > 0) load_queries(c0);
#pragma unroll
  for (int nt = 0; nt < NQT; ++nt) {
    if (c0 + nt * 16 >= QG) break;  // same for the whole grid
    f32x4_t acc[KT];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      acc[kt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < S; ++s)
        acc[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ka[kt][s]),
                                                          __builtin_bit_cast(bf16x8_t, bq[nt][s]), acc[kt], 0, 0, 0);
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      // adding +0 folds a possible -0 into +0 so that the bit pattern orders like the value
      const float4 out = make_float4(acc[kt][0] * sm_scale + 0.0f, acc[kt][1] * sm_scale + 0.0f,
                                     acc[kt][2] * sm_scale + 0.0f, acc[kt][3] * sm_scale + 0.0f);
      *reinterpret_cast<float4*>(&s_tile[i16][kt * 16 + 4 * g4]) = out;
    }
    __builtin_amdgcn_wave_barrier();
    const int i = tile_lo + lane;
    for (int c = 0; c < 16; ++c) {
      const int cg = c0 + nt * 16 + c;
      if (cg >= QG) break;
      const int t = cg / G, g = cg - t * G;
      const int n_t = max(n_b - (Q - 1 - t), 1);  // tokens this query sees (at least one, as in the other kernels)
      const int64_t row = ((int64_t)b * Q + t) * Hq + (int64_t)kvh * G + g;
      const float v = s_tile[c][lane];
      if (i < n_t) __builtin_nontemporal_store(v, &scores[row * n_pad + i]);
      const float mx = group_max8(i < n_t ? v : -INFINITY);
      if ((lane & 7) == 0) sub_max[row * n_sub + i / kSubTile] = mx;
    }
    __builtin_amdgcn_wave_barrier();
  }
  }
}

template <int D, bool PAGED, int NQT>
hipError_t launch_n(const Plan& pl, const void* q, const void* k, const int32_t* block_table,
                    const int32_t* seq_lens, void* ws, hipStream_t st) {
  const vatt_params& p = pl.p;
  KVLayout L = pl.kv_k;
  L.block_table = block_table;
  float* scores = reinterpret_cast<float*>(static_cast<char*>(ws) + pl.off_scores);
  float* smax = reinterpret_cast<float*>(static_cast<char*>(ws) + pl.off_sub_max);
  dim3 grid((p.n_max + kChunkTile - 1) / kChunkTile, p.n_kv_heads, p.batch);
  hipLaunchKernelGGL((score_chunk_kernel<D, PAGED, NQT>), grid, dim3(64 * kChunkWaves), 0, st,
                     static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k), L, seq_lens, scores, smax,
                     pl.n_sub, pl.n_pad, p.n_max, p.n_q_heads, pl.group, pl.q_len, pl.sm_scale);
  return hipGetLastError();
}

template <int D, bool PAGED>
hipError_t launch_p(const Plan& pl, const void* q, const void* k, const int32_t* block_table,
                    const int32_t* seq_lens, void* ws, hipStream_t st) {
  const int groups = std::min((pl.q_len * pl.group + 15) / 16, 4);  // more query vectors go in rounds of 64
  switch (groups) {
    case 1: return launch_n<D, PAGED, 1>(pl, q, k, block_table, seq_lens, ws, st);
    case 2: return launch_n<D, PAGED, 2>(pl, q, k, block_table, seq_lens, ws, st);
    case 3: return launch_n<D, PAGED, 3>(pl, q, k, block_table, seq_lens, ws, st);
    case 4: return launch_n<D, PAGED, 4>(pl, q, k, block_table, seq_lens, ws, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

hipError_t launch_score_chunk(const Plan& pl, const void* q, const void* k, const int32_t* block_table,
                              const int32_t* seq_lens, void* ws, hipStream_t st) {
  const bool paged = pl.p.kv_layout == VATT_LAYOUT_PAGED;
  if (pl.p.head_dim == 128)
    return paged ? launch_p<128, true>(pl, q, k, block_table, seq_lens, ws, st)
                 : launch_p<128, false>(pl, q, k, block_table, seq_lens, ws, st);
  if (pl.p.head_dim == 64)
    return paged ? launch_p<64, true>(pl, q, k, block_table, seq_lens, ws, st)
                 : launch_p<64, false>(pl, q, k, block_table, seq_lens, ws, st);
  return hipErrorInvalidValue;
}

}  // namespace vatt
