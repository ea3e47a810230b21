// Dense decode attention (Eq. 1) on the same cache, and the KV append.
//
// dense_kernel: grid = (KV heads, splits, sequences), KV head fastest: with 8 KV heads every XCD then streams
// the K and V rows of one KV head front to back (measured 3 % faster at batch 4 and 16 than with the splits
// fastest, the same at batch 1).  A workgroup owns a contiguous key range; each
// wave walks its quarter of it, 4 (d = 128) rows per load, computing the G scores of a row with
// the same lane layout as the score pass and keeping a running (max, sum, accumulator) per lane
// group -- no LDS traffic inside the loop.  Lane groups, waves and finally splits are merged by
// the usual log-sum-exp rule.  K and V are each read once: 2 * Hkv * n * d * 2 bytes per sequence.
#include "vatt_internal.h"

namespace vatt {
namespace {

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), acc,
                                         false);
}

constexpr float kNegBig = -1.0e30f;

struct DenseArgs {
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  KVLayout Lk, Lv;
  const int32_t* seq_lens;
  float* part;  // [B*Hq][splits][d + 4]: acc[d], max, sum
  float* out_o;
  float* out_lse;
  int n_max, Hq, splits;
  int q_len;  // query tokens per sequence: blockIdx.z = sequence * q_len + query token (each one scans the cache)
  float sm_scale;
};

// SHARE (multi-query steps): the query tokens of a sequence scan the same rows, so their workgroups for one
// (KV head, split) are launched next to each other, eight apart in launch order and therefore on one XCD at
// the same time, and read K and V with plain loads: the first to ask fetches a line from HBM, the others find
// it in that XCD's L2.  blockIdx.y = split * q_len + query token, blockIdx.z = sequence.
template <int D, int G, bool PAGED, bool SHARE>
__global__ __launch_bounds__(kDenseThreads) void dense_kernel(DenseArgs A) {
  constexpr int LPR = D / 8;
  constexpr int RPW = kWave / LPR;
  constexpr int WAVES = kDenseThreads / kWave;
  constexpr int U = 4;

  const int kvh = blockIdx.x;
  const int split = SHARE ? (int)blockIdx.y / A.q_len : (int)blockIdx.y;
  const int b = SHARE ? (int)blockIdx.z * A.q_len + (int)blockIdx.y % A.q_len : (int)blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = lane % LPR, rsub = lane / LPR;
  const int seq = b / A.q_len, qtok = b - seq * A.q_len;
  const int n = max(min(max(A.seq_lens[seq], 1), A.n_max) - (A.q_len - 1 - qtok), 1);  // clamp, then the causal cut
  // key range of this workgroup, then of this wave (multiples of RPW * U rows except at the end)
  const int step = RPW * U;
  const int per_blk = ((n + A.splits - 1) / A.splits + step * WAVES - 1) / (step * WAVES) * (step * WAVES);
  const int blk_lo = split * per_blk, blk_hi = min(blk_lo + per_blk, n);
  const int per_wave = per_blk / WAVES;
  const int lo = blk_lo + wave * per_wave, hi = min(lo + per_wave, blk_hi);

  uint32_t qw[G][4];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const uint4 t = *reinterpret_cast<const uint4*>(A.q + ((int64_t)b * A.Hq + (int64_t)kvh * G + g) * D + sub * 8);
    qw[g][0] = t.x;
    qw[g][1] = t.y;
    qw[g][2] = t.z;
    qw[g][3] = t.w;
  }
  float mrun[G], lrun[G], acc[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    mrun[g] = kNegBig;
    lrun[g] = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[g][c] = 0.f;
  }

  for (int i0 = lo; i0 < hi; i0 += step) {
    uint4 kk[U], vv[U];
    bool ok[U];
    int blk[U];
    // (paged cache: the block-table entries of all rows first, outside the test on the row index, so that no
    // row waits for the entry of the one before; K and V share the table)
#pragma unroll
    for (int u = 0; u < U; ++u) blk[u] = kv_block<PAGED>(A.Lk, seq, min(i0 + u * RPW + rsub, hi - 1));
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = i0 + u * RPW + rsub;
      ok[u] = i < hi;
      kk[u] = vv[u] = make_uint4(0u, 0u, 0u, 0u);
      if (ok[u]) {
        const uint16_t* pk = A.k + kv_row_offset_in<PAGED>(A.Lk, seq, kvh, i, blk[u]) + sub * 8;
        const uint16_t* pv = A.v + kv_row_offset_in<PAGED>(A.Lv, seq, kvh, i, blk[u]) + sub * 8;
        kk[u] = SHARE ? *reinterpret_cast<const uint4*>(pk) : load_stream_16(pk);
        vv[u] = SHARE ? *reinterpret_cast<const uint4*>(pv) : load_stream_16(pv);
      }
    }
    float s[G][U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float a = 0.f;
        a = dot2_bf16(kk[u].x, qw[g][0], a);
        a = dot2_bf16(kk[u].y, qw[g][1], a);
        a = dot2_bf16(kk[u].z, qw[g][2], a);
        a = dot2_bf16(kk[u].w, qw[g][3], a);
        a = group_sum<LPR>(a);
        s[g][u] = ok[u] ? a * A.sm_scale : kNegBig;
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float mnew = mrun[g];
#pragma unroll
      for (int u = 0; u < U; ++u) mnew = fmaxf(mnew, s[g][u]);
      const float alpha = __expf(mrun[g] - mnew);
      mrun[g] = mnew;
      lrun[g] *= alpha;
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[g][c] *= alpha;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float p = ok[u] ? __expf(s[g][u] - mnew) : 0.f;
        lrun[g] += p;
        const uint32_t ww[4] = {vv[u].x, vv[u].y, vv[u].z, vv[u].w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          acc[g][2 * c] += p * bf16_lo(ww[c]);
          acc[g][2 * c + 1] += p * bf16_hi(ww[c]);
        }
      }
    }
  }

  // merge the lane groups of the wave
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float mall = mrun[g];
#pragma unroll
    for (int o = LPR; o < kWave; o <<= 1) mall = fmaxf(mall, __shfl_xor(mall, o));
    const float sc = __expf(mrun[g] - mall);
    lrun[g] *= sc;
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[g][c] *= sc;
#pragma unroll
    for (int o = LPR; o < kWave; o <<= 1) {
      lrun[g] += __shfl_xor(lrun[g], o);
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[g][c] += __shfl_xor(acc[g][c], o);
    }
    mrun[g] = mall;
  }
  __shared__ float s_acc[WAVES][G][D];
  __shared__ float s_m[WAVES][G], s_l[WAVES][G];
  if (rsub == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int c = 0; c < 8; ++c) s_acc[wave][g][sub * 8 + c] = acc[g][c];
      if (sub == 0) {
        s_m[wave][g] = mrun[g];
        s_l[wave][g] = lrun[g];
      }
    }
  }
  __syncthreads();
  for (int t = tid; t < G * D; t += kDenseThreads) {
    const int g = t / D, c = t % D;
    float mall = s_m[0][g];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) mall = fmaxf(mall, s_m[w][g]);
    float a = 0.f, l = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      const float sc = __expf(s_m[w][g] - mall);
      a += s_acc[w][g][c] * sc;
      l += s_l[w][g] * sc;
    }
    float* part = A.part + (((int64_t)b * A.Hq + (int64_t)kvh * G + g) * A.splits + split) * (D + 4);
    part[c] = a;
    if (c == 0) {
      part[D] = mall;
      part[D + 1] = l;
    }
  }
}

// Log-sum-exp merge of the per-split partials of one head.  Two thread halves take alternate splits so
// that their loads are independent and can be in flight together.
template <int D>
__global__ __launch_bounds__(2 * D) void dense_merge_kernel(const float* __restrict__ part, int splits, int Hq,
                                                            int Hkv, float* __restrict__ out_o,
                                                            float* __restrict__ out_lse) {
  // blockIdx.x runs over the KV heads first, then over the heads of a group (as in the dense kernel's grid)
  const int h = head_of_block((int)blockIdx.x, Hq, Hkv, 1), b = blockIdx.y, bh = b * Hq + h;
  const int c = threadIdx.x % D, half = threadIdx.x / D;
  const float* p = part + (int64_t)bh * splits * (D + 4);
  __shared__ float s_m[128], s_l[128], s_a[D];
  for (int s = threadIdx.x; s < splits; s += 2 * D) {
    s_m[s] = p[s * (D + 4) + D];
    s_l[s] = p[s * (D + 4) + D + 1];
  }
  __syncthreads();
  float mall = kNegBig;
  for (int s = 0; s < splits; ++s) mall = fmaxf(mall, s_m[s]);
  float a = 0.f;
#pragma unroll 8
  for (int s = half; s < splits; s += 2) a += p[s * (D + 4) + c] * __expf(s_m[s] - mall);
  if (half == 1) s_a[c] = a;
  __syncthreads();
  if (half == 0) {
    float l = 0.f;
    for (int s = 0; s < splits; ++s) l += s_l[s] * __expf(s_m[s] - mall);
    out_o[(int64_t)bh * D + c] = (a + s_a[c]) / l;
    if (c == 0 && out_lse) out_lse[bh] = mall + logf(l);
  }
}

template <int D, int G>
hipError_t launch_dense_dg(const Plan& pl, DenseArgs& A, hipStream_t st) {
  const vatt_params& p = pl.p;
  const bool paged = p.kv_layout == VATT_LAYOUT_PAGED;
  if (pl.q_len > 1) {
    dim3 grid(p.n_kv_heads, pl.dense_splits * pl.q_len, p.batch);
    if (paged) hipLaunchKernelGGL((dense_kernel<D, G, true, true>), grid, dim3(kDenseThreads), 0, st, A);
    else hipLaunchKernelGGL((dense_kernel<D, G, false, true>), grid, dim3(kDenseThreads), 0, st, A);
  } else {
    dim3 grid(p.n_kv_heads, pl.dense_splits, pl.vbatch);
    if (paged) hipLaunchKernelGGL((dense_kernel<D, G, true, false>), grid, dim3(kDenseThreads), 0, st, A);
    else hipLaunchKernelGGL((dense_kernel<D, G, false, false>), grid, dim3(kDenseThreads), 0, st, A);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((dense_merge_kernel<D>), dim3(p.n_q_heads, pl.vbatch), dim3(2 * D), 0, st, A.part, pl.dense_splits,
                     p.n_q_heads, p.n_kv_heads, A.out_o, A.out_lse);
  return hipGetLastError();
}

template <int D>
hipError_t launch_dense_d(const Plan& pl, DenseArgs& A, hipStream_t st) {
  switch (pl.group) {
    case 1: return launch_dense_dg<D, 1>(pl, A, st);
    case 2: return launch_dense_dg<D, 2>(pl, A, st);
    case 4: return launch_dense_dg<D, 4>(pl, A, st);
    case 8: return launch_dense_dg<D, 8>(pl, A, st);
    default: return hipErrorInvalidValue;
  }
}

// One workgroup per sequence: all threads read the current length, then copy the new K and V rows of
// every KV head (16 bytes per thread), then one thread stores length + 1.
template <bool PAGED>
__global__ void append_kernel(const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new, uint16_t* k,
                              uint16_t* v, KVLayout L, int32_t* seq_lens, int n_max, int Hkv) {
  const int b = blockIdx.x;
  const int n = seq_lens[b];
  __syncthreads();
  if (n < 0 || n >= n_max) return;
  const int d = L.head_dim;
  const int per_head = d / 8;
  for (int t = threadIdx.x; t < Hkv * per_head; t += blockDim.x) {
    const int kvh = t / per_head, c = t % per_head;
    const int64_t src = ((int64_t)b * Hkv + kvh) * d + c * 8;
    const int64_t dst = kv_row_offset<PAGED>(L, b, kvh, n) + c * 8;
    *reinterpret_cast<uint4*>(k + dst) = *reinterpret_cast<const uint4*>(k_new + src);
    *reinterpret_cast<uint4*>(v + dst) = *reinterpret_cast<const uint4*>(v_new + src);
  }
  if (threadIdx.x == 0) seq_lens[b] = n + 1;
}

}  // namespace

hipError_t launch_dense(const Plan& pl, const void* q, const void* k, const void* v, const int32_t* block_table,
                        const int32_t* seq_lens, void* ws, float* out_o, float* out_lse, hipStream_t st) {
  DenseArgs A;
  A.q = static_cast<const uint16_t*>(q);
  A.k = static_cast<const uint16_t*>(k);
  A.v = static_cast<const uint16_t*>(v);
  A.Lk = pl.kv_k;
  A.Lk.block_table = block_table;
  A.Lv = pl.kv_v;
  A.Lv.block_table = block_table;
  A.seq_lens = seq_lens;
  A.part = reinterpret_cast<float*>(static_cast<char*>(ws) + pl.off_dense_part);
  A.out_o = out_o;
  A.out_lse = out_lse;
  A.n_max = pl.p.n_max;
  A.Hq = pl.p.n_q_heads;
  A.splits = pl.dense_splits;
  A.q_len = pl.q_len;
  A.sm_scale = pl.sm_scale;
  if (pl.p.head_dim == 128) return launch_dense_d<128>(pl, A, st);
  if (pl.p.head_dim == 64) return launch_dense_d<64>(pl, A, st);
  return hipErrorInvalidValue;
}

hipError_t launch_append(const Plan& pl, const void* k_new, const void* v_new, void* k, void* v,
                         const int32_t* block_table, int32_t* seq_lens, hipStream_t st) {
  KVLayout L = pl.kv_k;
  L.block_table = block_table;
  const int threads = 128;
  if (pl.p.kv_layout == VATT_LAYOUT_PAGED)
    hipLaunchKernelGGL((append_kernel<true>), dim3(pl.p.batch), dim3(threads), 0, st,
                       static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new),
                       static_cast<uint16_t*>(k), static_cast<uint16_t*>(v), L, seq_lens, pl.p.n_max,
                       pl.p.n_kv_heads);
  else
    hipLaunchKernelGGL((append_kernel<false>), dim3(pl.p.batch), dim3(threads), 0, st,
                       static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new),
                       static_cast<uint16_t*>(k), static_cast<uint16_t*>(v), L, seq_lens, pl.p.n_max,
                       pl.p.n_kv_heads);
  return hipGetLastError();
}

}  // namespace vatt
