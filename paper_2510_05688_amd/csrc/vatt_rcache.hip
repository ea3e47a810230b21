// Random cache of base-sample rows (the implementation note after Theorem 4.3): per (sequence, KV head) a
// fixed number of slots holds a uniform random subset of the tokens seen so far, in uniformly random order,
// with copies of their K and V rows.  Token t arrives with one draw r, uniform in [0, t]:
//   cache not full (t < slots):  the entry of slot r moves to slot t, the new token takes slot r
//                                (r == t: it takes slot t) - the entries stay in uniformly random order;
//   cache full:                  the new token replaces slot r when r < slots (reservoir sampling).
//
//   cache_fill_kernel     the state after tokens 0 .. n-1 have arrived one by one, for a cache that exists
//                         already (after a prefill).  The order-dependent first `slots` arrivals are replayed
//                         by one thread from draws made by all; afterwards slot s ends up with the last
//                         token whose draw was s, which is a maximum over independent draws.
//   append_cached_kernel  vatt_append_kv plus the arrival of the appended token in the cache.
//   cache_read_kernel     token lists and counts, for tests.
#include "vatt_internal.h"

namespace vatt {
namespace {

constexpr int kFillThreads = 256;

__device__ __forceinline__ void copy_row(uint16_t* dst, const uint16_t* src, int chunk) {
  *reinterpret_cast<uint4*>(dst + chunk * 8) = *reinterpret_cast<const uint4*>(src + chunk * 8);
}

template <bool PAGED>
__global__ __launch_bounds__(kFillThreads) void cache_fill_kernel(const uint16_t* __restrict__ k,
                                                                  const uint16_t* __restrict__ v, KVLayout L,
                                                                  const int32_t* __restrict__ seq_lens,
                                                                  const uint64_t* __restrict__ cache_seeds,
                                                                  void* rcache, CacheLayout C, int n_max, int Hkv) {
  extern __shared__ __align__(16) unsigned char dyn_smem[];
  int32_t* tok = reinterpret_cast<int32_t*>(dyn_smem);  // [slots]
  int32_t* jl = tok + C.slots;                           // [slots]: the draw of each of the first arrivals
  const int kvh = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int n = min(max(seq_lens[b], 0), n_max);
  const uint64_t seed = cache_seeds[b];
  const int fill = min(n, C.slots);
  for (int t = tid; t < fill; t += kFillThreads) jl[t] = (int32_t)cache_draw((uint32_t)t, (uint32_t)t + 1u, seed, (uint32_t)kvh);
  __syncthreads();
  if (tid == 0) {
    for (int t = 0; t < fill; ++t) {
      const int j = jl[t];
      if (j != t) tok[t] = tok[j];
      tok[j] = t;
    }
  }
  __syncthreads();
  // full cache: slot r keeps the latest token that drew r (every such token is later than the first arrivals)
  for (int t = C.slots + tid; t < n; t += kFillThreads) {
    const uint32_t r = cache_draw((uint32_t)t, (uint32_t)t + 1u, seed, (uint32_t)kvh);
    if (r < (uint32_t)C.slots) atomicMax(&tok[r], t);
  }
  __syncthreads();
  unsigned char* rec = cache_record(rcache, C, b, Hkv, kvh);
  int32_t* g_tok = reinterpret_cast<int32_t*>(rec + 16);
  uint16_t* ck = reinterpret_cast<uint16_t*>(rec + C.off_k);
  uint16_t* cv = reinterpret_cast<uint16_t*>(rec + C.off_v);
  if (tid == 0) *reinterpret_cast<int32_t*>(rec) = fill;
  for (int s = tid; s < fill; s += kFillThreads) g_tok[s] = tok[s];
  const int d = C.head_dim, per_row = d / 8;
  for (int e = tid; e < fill * per_row; e += kFillThreads) {
    const int s = e / per_row, c = e - s * per_row;
    const int64_t src = kv_row_offset<PAGED>(L, b, kvh, tok[s]);
    copy_row(ck + (int64_t)s * d, k + src, c);
    copy_row(cv + (int64_t)s * d, v + src, c);
  }
}

// One workgroup per sequence; thread e handles 16 bytes of one KV head's rows.  A sequence at n_max is left
// as it is, cache included.
template <bool PAGED>
__global__ void append_cached_kernel(const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new,
                                     uint16_t* k, uint16_t* v, KVLayout L, int32_t* seq_lens,
                                     const uint64_t* __restrict__ cache_seeds, void* rcache, CacheLayout C,
                                     int n_max, int Hkv) {
  const int b = blockIdx.x;
  const int n = seq_lens[b];
  __syncthreads();
  if (n < 0 || n >= n_max) return;
  const uint64_t seed = cache_seeds[b];
  const int d = L.head_dim;
  const int per_head = d / 8;
  for (int e = threadIdx.x; e < Hkv * per_head; e += blockDim.x) {
    const int kvh = e / per_head, c = e % per_head;
    const uint16_t* src_k = k_new + ((int64_t)b * Hkv + kvh) * d;
    const uint16_t* src_v = v_new + ((int64_t)b * Hkv + kvh) * d;
    const int64_t dst = kv_row_offset<PAGED>(L, b, kvh, n);
    copy_row(k + dst, src_k, c);
    copy_row(v + dst, src_v, c);
    // the token's arrival in the cache of (b, kvh): every thread of the head takes the same draw
    const int r = (int)cache_draw((uint32_t)n, (uint32_t)n + 1u, seed, (uint32_t)kvh);
    unsigned char* rec = cache_record(rcache, C, b, Hkv, kvh);
    int32_t* g_tok = reinterpret_cast<int32_t*>(rec + 16);
    uint16_t* ck = reinterpret_cast<uint16_t*>(rec + C.off_k);
    uint16_t* cv = reinterpret_cast<uint16_t*>(rec + C.off_v);
    if (n < C.slots) {
      if (r != n) {  // the entry of slot r moves to the new last slot
        copy_row(ck + (int64_t)n * d, ck + (int64_t)r * d, c);
        copy_row(cv + (int64_t)n * d, cv + (int64_t)r * d, c);
        if (c == 0) g_tok[n] = g_tok[r];
      }
      copy_row(ck + (int64_t)r * d, src_k, c);
      copy_row(cv + (int64_t)r * d, src_v, c);
      if (c == 0) {
        g_tok[r] = n;
        *reinterpret_cast<int32_t*>(rec) = n + 1;
      }
    } else if (r < C.slots) {
      copy_row(ck + (int64_t)r * d, src_k, c);
      copy_row(cv + (int64_t)r * d, src_v, c);
      if (c == 0) g_tok[r] = n;
    }
  }
  if (threadIdx.x == 0) seq_lens[b] = n + 1;
}

__global__ void cache_read_kernel(const void* rcache, CacheLayout C, int Hkv, int32_t* __restrict__ out_tok,
                                  int32_t* __restrict__ out_count) {
  const int kvh = blockIdx.x, b = blockIdx.y;
  const unsigned char* rec = cache_record(rcache, C, b, Hkv, kvh);
  const int32_t* g_tok = reinterpret_cast<const int32_t*>(rec + 16);
  const int count = min(max(*reinterpret_cast<const int32_t*>(rec), 0), C.slots);
  int32_t* dst = out_tok + ((int64_t)b * Hkv + kvh) * C.slots;
  for (int s = threadIdx.x; s < C.slots; s += blockDim.x) dst[s] = s < count ? g_tok[s] : -1;
  if (threadIdx.x == 0) out_count[b * Hkv + kvh] = count;
}

}  // namespace

CacheLayout cache_layout(const Plan& pl) {
  CacheLayout C;
  C.slots = pl.cache_slots;
  C.head_dim = pl.p.head_dim;
  C.off_k = 16 + (int64_t)4 * C.slots;
  C.off_v = C.off_k + (int64_t)2 * C.slots * C.head_dim;
  C.rec_bytes = (C.off_v + (int64_t)2 * C.slots * C.head_dim + 255) & ~(int64_t)255;
  return C;
}

hipError_t launch_cache_fill(const Plan& pl, const void* k, const void* v, const int32_t* block_table,
                             const int32_t* seq_lens, const uint64_t* cache_seeds, void* rcache, hipStream_t st) {
  KVLayout L = pl.kv_k;
  L.block_table = block_table;
  const CacheLayout C = cache_layout(pl);
  const dim3 grid(pl.p.n_kv_heads, pl.p.batch);
  const size_t lds = (size_t)2 * C.slots * sizeof(int32_t);
  if (pl.p.kv_layout == VATT_LAYOUT_PAGED)
    hipLaunchKernelGGL((cache_fill_kernel<true>), grid, dim3(kFillThreads), lds, st, static_cast<const uint16_t*>(k),
                       static_cast<const uint16_t*>(v), L, seq_lens, cache_seeds, rcache, C, pl.p.n_max,
                       pl.p.n_kv_heads);
  else
    hipLaunchKernelGGL((cache_fill_kernel<false>), grid, dim3(kFillThreads), lds, st, static_cast<const uint16_t*>(k),
                       static_cast<const uint16_t*>(v), L, seq_lens, cache_seeds, rcache, C, pl.p.n_max,
                       pl.p.n_kv_heads);
  return hipGetLastError();
}

hipError_t launch_append_cached(const Plan& pl, const void* k_new, const void* v_new, void* k, void* v,
                                const int32_t* block_table, int32_t* seq_lens, const uint64_t* cache_seeds,
                                void* rcache, hipStream_t st) {
  KVLayout L = pl.kv_k;
  L.block_table = block_table;
  const CacheLayout C = cache_layout(pl);
  const int threads = 128;
  if (pl.p.kv_layout == VATT_LAYOUT_PAGED)
    hipLaunchKernelGGL((append_cached_kernel<true>), dim3(pl.p.batch), dim3(threads), 0, st,
                       static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new),
                       static_cast<uint16_t*>(k), static_cast<uint16_t*>(v), L, seq_lens, cache_seeds, rcache, C,
                       pl.p.n_max, pl.p.n_kv_heads);
  else
    hipLaunchKernelGGL((append_cached_kernel<false>), dim3(pl.p.batch), dim3(threads), 0, st,
                       static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new),
                       static_cast<uint16_t*>(k), static_cast<uint16_t*>(v), L, seq_lens, cache_seeds, rcache, C,
                       pl.p.n_max, pl.p.n_kv_heads);
  return hipGetLastError();
}

hipError_t launch_cache_read(const Plan& pl, const void* rcache, int32_t* out_tok, int32_t* out_count,
                             hipStream_t st) {
  hipLaunchKernelGGL(cache_read_kernel, dim3(pl.p.n_kv_heads, pl.p.batch), dim3(256), 0, st, rcache,
                     cache_layout(pl), pl.p.n_kv_heads, out_tok, out_count);
  return hipGetLastError();
}

}  // namespace vatt
