// Device-side helpers shared by the vatt kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vatt {

constexpr int kWave = 64;

// Query head of a workgroup whose blockIdx.x runs over the heads.  Plain order: the head is blockIdx.x.
// Group-major order: blockIdx.x runs over the KV heads first and over the heads of a group second, so that
// (workgroups go to the XCDs round-robin in launch order, and with a KV head count that is a multiple of 8)
// the workgroups of all query heads of KV head j run on XCD j mod 8 and share its L2 while the kernel runs:
// they read the same sink and window rows of V and many of the same heavy tokens.
__device__ __forceinline__ int head_of_block(int x, int Hq, int Hkv, int group_major) {
  return group_major ? (x % Hkv) * (Hq / Hkv) + x / Hkv : x;
}

// Optional phase timing for kernel development: built with -DVATT_TIMING, thread 0 of workgroup 0 stores
// the shader clock at numbered points into the VATT_WS_DEBUG region of the workspace.  Compiled out
// otherwise.
#ifdef VATT_TIMING
#define VATT_STAMP(buf, id)                                                               \
  do {                                                                                    \
    if ((buf) && threadIdx.x == 0 && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0) \
      (buf)[id] = __builtin_readcyclecounter();                                           \
  } while (0)
#define VATT_NOTE(buf, id, val)                                                            \
  do {                                                                                    \
    if ((buf) && threadIdx.x == 0 && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0) \
      (buf)[id] = (unsigned long long)(val);                                              \
  } while (0)
#else
#define VATT_STAMP(buf, id) \
  do {                      \
  } while (0)
#define VATT_NOTE(buf, id, val) \
  do {                          \
  } while (0)
#endif

// ---------------------------------------------------------------------------
// KV cache addressing.  Contiguous: [B, Hkv, n_max, d].  Paged: [blocks, Hkv, page, d]
// with a block table [B, pages_per_seq].
// ---------------------------------------------------------------------------
struct KVLayout {
  const int32_t* block_table;  // nullptr when contiguous
  int64_t seq_stride;          // contiguous: Hkv * n_max * d        (elements)
  int64_t head_stride;         // contiguous: n_max * d; paged: page * d
  int64_t block_stride;        // paged: Hkv * page * d
  int32_t page_shift;          // log2(page)
  int32_t pages_per_seq;
  int32_t num_blocks;
  int32_t head_dim;
};

template <bool PAGED>
__device__ __forceinline__ int64_t kv_row_offset(const KVLayout& L, int b, int kvh, int i) {
  if constexpr (PAGED) {
    const int page = i >> L.page_shift;
    int blk = L.block_table[(int64_t)b * L.pages_per_seq + page];
    blk = min(max(blk, 0), L.num_blocks - 1);
    const int within = i & ((1 << L.page_shift) - 1);
    return (int64_t)blk * L.block_stride + (int64_t)kvh * L.head_stride + (int64_t)within * L.head_dim;
  } else {
    return (int64_t)b * L.seq_stride + (int64_t)kvh * L.head_stride + (int64_t)i * L.head_dim;
  }
}

// The same in two steps, for kernels that have several rows in flight: the block-table entries of all rows are
// requested first, then the rows (kv_row_offset in a loop leaves it to the compiler whether a row's table entry
// is awaited before the next row's is requested).
template <bool PAGED>
__device__ __forceinline__ int kv_block(const KVLayout& L, int b, int i) {
  if constexpr (PAGED) return L.block_table[(int64_t)b * L.pages_per_seq + (i >> L.page_shift)];
  else return 0;
}
template <bool PAGED>
__device__ __forceinline__ int64_t kv_row_offset_in(const KVLayout& L, int b, int kvh, int i, int blk) {
  if constexpr (PAGED) {
    blk = min(max(blk, 0), L.num_blocks - 1);
    const int within = i & ((1 << L.page_shift) - 1);
    return (int64_t)blk * L.block_stride + (int64_t)kvh * L.head_stride + (int64_t)within * L.head_dim;
  } else {
    return (int64_t)b * L.seq_stride + (int64_t)kvh * L.head_stride + (int64_t)i * L.head_dim;
  }
}

// ---------------------------------------------------------------------------
// A head's index lists are walked by position p of [sink | window | top-k | tail).  Offset into the lists of a
// position of the first three segments, by arithmetic alone: the kernels that gather rows compute the places
// of all rows they have in flight, then read all tokens, then request all rows, with no branch per row (a
// branch per row makes every index load wait for the row load before it).
// ---------------------------------------------------------------------------
__device__ __forceinline__ int64_t fixed_place(int p, int n_sink, int n_win, int64_t seg_sink, int64_t seg_win,
                                               int64_t seg_topk) {
  // (the three segment shifts are uniform values: two selects and an add, all in 32 bits; list offsets are small)
  const int o0 = (int)seg_sink, o1 = (int)seg_win - n_sink, o2 = (int)seg_topk - n_sink - n_win;
  const int off = p < n_sink ? o0 : (p < n_sink + n_win ? o1 : o2);
  return (int64_t)(p + off);
}

// ---------------------------------------------------------------------------
// 16-byte load of data that is read once (K and V rows): the non-temporal hint keeps the stream from
// displacing what the caches hold for reuse; measured +10 % on the K scan.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint4 load_stream_16(const uint16_t* p) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(t.x, t.y, t.z, t.w);
}

// ---------------------------------------------------------------------------
// bf16 pairs packed in a 32-bit word -> two fp32 values (exact).
// ---------------------------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// ---------------------------------------------------------------------------
// Cross-lane sums inside groups of 8 or 16 adjacent lanes, on the DPP path.
// After the call every lane of the group holds the group's sum.
// ---------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}

template <int LANES>
__device__ __forceinline__ float group_sum(float v) {
  static_assert(LANES == 8 || LANES == 16, "group of 8 or 16 lanes");
  v += dpp_f32<0xB1>(v);   // quad_perm [1,0,3,2]: partner lane ^ 1
  v += dpp_f32<0x4E>(v);   // quad_perm [2,3,0,1]: partner lane ^ 2
  v += dpp_f32<0x141>(v);  // row_half_mirror: the other quad of the 8-lane half
  if constexpr (LANES == 16) v += dpp_f32<0x140>(v);  // row_mirror: the other half of the 16-lane row
  return v;
}

// Maximum over each group of 8 adjacent lanes, left in every lane of the group.
__device__ __forceinline__ float group_max8(float v) {
  v = fmaxf(v, dpp_f32<0xB1>(v));   // partner lane ^ 1
  v = fmaxf(v, dpp_f32<0x4E>(v));   // partner lane ^ 2
  v = fmaxf(v, dpp_f32<0x141>(v));  // the other quad of the 8-lane half row
  return v;
}

// Wave-wide sum of a 32-bit integer, returned as a wave-uniform value: four DPP adds leave each row of
// 16 lanes with its row sum, four lane reads add the rows.  Every lane of the wave must be active.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, false);
}
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
  v += dpp_u32<0xB1>(v);
  v += dpp_u32<0x4E>(v);
  v += dpp_u32<0x141>(v);
  v += dpp_u32<0x140>(v);
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 0) + (uint32_t)__builtin_amdgcn_readlane((int)v, 16) +
         (uint32_t)__builtin_amdgcn_readlane((int)v, 32) + (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
}

__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
  v = min(v, dpp_u32<0xB1>(v));
  v = min(v, dpp_u32<0x4E>(v));
  v = min(v, dpp_u32<0x141>(v));
  v = min(v, dpp_u32<0x140>(v));
  return min(min((uint32_t)__builtin_amdgcn_readlane((int)v, 0), (uint32_t)__builtin_amdgcn_readlane((int)v, 16)),
             min((uint32_t)__builtin_amdgcn_readlane((int)v, 32), (uint32_t)__builtin_amdgcn_readlane((int)v, 48)));
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
  v = max(v, dpp_u32<0xB1>(v));
  v = max(v, dpp_u32<0x4E>(v));
  v = max(v, dpp_u32<0x141>(v));
  v = max(v, dpp_u32<0x140>(v));
  return max(max((uint32_t)__builtin_amdgcn_readlane((int)v, 0), (uint32_t)__builtin_amdgcn_readlane((int)v, 16)),
             max((uint32_t)__builtin_amdgcn_readlane((int)v, 32), (uint32_t)__builtin_amdgcn_readlane((int)v, 48)));
}

// Inclusive prefix sum over the 64 lanes of a wave on the DPP path: shifts by 1, 2, 4, 8 inside each row of
// 16 lanes (lanes shifted in from outside the row read 0), then the last lane of row 0/2 is added to row
// 1/3 and the last lane of the lower half to the upper half.  Every lane of the wave must be active.
__device__ __forceinline__ uint32_t wave_inclusive_scan_u32(uint32_t v) {
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, true);  // row_shr:1
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, true);  // row_shr:2
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, true);  // row_shr:4
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, true);  // row_shr:8
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false);  // row_bcast:15 -> rows 1, 3
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false);  // row_bcast:31 -> rows 2, 3
  return v;
}

// Wave-wide maximum / sums on the DPP path (four steps inside each row of 16 lanes, then the four rows through
// lane reads), returned as wave-uniform values.  The order of the additions is fixed, so the sums are
// reproducible.  Every lane of the wave must be active.
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_f32<0xB1>(v));
  v = fmaxf(v, dpp_f32<0x4E>(v));
  v = fmaxf(v, dpp_f32<0x141>(v));
  v = fmaxf(v, dpp_f32<0x140>(v));
  const int b = __float_as_int(v);
  return fmaxf(fmaxf(__int_as_float(__builtin_amdgcn_readlane(b, 0)), __int_as_float(__builtin_amdgcn_readlane(b, 16))),
               fmaxf(__int_as_float(__builtin_amdgcn_readlane(b, 32)), __int_as_float(__builtin_amdgcn_readlane(b, 48))));
}
// Wave-wide sum of a float in a fixed order, wave-uniform result.
__device__ __forceinline__ float wave_sum_f32(float v) {
  v += dpp_f32<0xB1>(v);
  v += dpp_f32<0x4E>(v);
  v += dpp_f32<0x141>(v);
  v += dpp_f32<0x140>(v);
  const int b = __float_as_int(v);
  return (__int_as_float(__builtin_amdgcn_readlane(b, 0)) + __int_as_float(__builtin_amdgcn_readlane(b, 16))) +
         (__int_as_float(__builtin_amdgcn_readlane(b, 32)) + __int_as_float(__builtin_amdgcn_readlane(b, 48)));
}
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
  const uint64_t b = (uint64_t)__double_as_longlong(v);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)b, CTRL, 0xf, 0xf, false);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(b >> 32), CTRL, 0xf, 0xf, false);
  return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}
__device__ __forceinline__ double readlane_f64(double v, int lane) {
  const uint64_t b = (uint64_t)__double_as_longlong(v);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)b, lane);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(b >> 32), lane);
  return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}
__device__ __forceinline__ double wave_sum(double v) {
  v += dpp_f64<0xB1>(v);
  v += dpp_f64<0x4E>(v);
  v += dpp_f64<0x141>(v);
  v += dpp_f64<0x140>(v);
  return (readlane_f64(v, 0) + readlane_f64(v, 16)) + (readlane_f64(v, 32) + readlane_f64(v, 48));
}
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
template <int CTRL>
__device__ __forceinline__ uint64_t dpp_u64(uint64_t b) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)b, CTRL, 0xf, 0xf, false);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(b >> 32), CTRL, 0xf, 0xf, false);
  return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ uint64_t readlane_u64(uint64_t b, int lane) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)b, lane);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(b >> 32), lane);
  return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ uint64_t wave_sum(uint64_t v) {
  v += dpp_u64<0xB1>(v);
  v += dpp_u64<0x4E>(v);
  v += dpp_u64<0x141>(v);
  v += dpp_u64<0x140>(v);
  return (readlane_u64(v, 0) + readlane_u64(v, 16)) + (readlane_u64(v, 32) + readlane_u64(v, 48));
}

// ---------------------------------------------------------------------------
// Order-preserving map fp32 -> uint32 (ascending).  -0 must have been folded into +0.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t float_order_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float float_from_order_key(uint32_t k) {
  const uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
  return __uint_as_float(u);
}

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11): ten rounds of
//   (c0,c1,c2,c3) <- (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0)),
// the key advancing by the Weyl constants between rounds.
// ---------------------------------------------------------------------------
struct Philox4 {
  uint32_t v[4];
};

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                  uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)c0 * 0xD2511F53ull;
    const uint64_t p1 = (uint64_t)c2 * 0xCD9E8D57ull;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  Philox4 o;
  o.v[0] = c0;
  o.v[1] = c1;
  o.v[2] = c2;
  o.v[3] = c3;
  return o;
}

// ---------------------------------------------------------------------------
// Random cache of base-sample rows (the implementation note after Theorem 4.3: the base sample can be served
// from a small random cache kept up to date during generation).  One record per (sequence, KV head):
//   int32 count (slots in use), 12 bytes of padding | int32 token[slots] | bf16 K rows [slots][d] |
//   bf16 V rows [slots][d]
// The slots hold a uniform random subset of the tokens seen so far, in uniformly random order (reservoir
// sampling), each with a copy of its K and V row.
// ---------------------------------------------------------------------------
struct CacheLayout {
  int32_t slots;
  int32_t head_dim;
  int64_t rec_bytes, off_k, off_v;  // bytes; the token list starts at byte 16 of a record
};

__device__ __forceinline__ unsigned char* cache_record(void* base, const CacheLayout& C, int b, int Hkv, int kvh) {
  return static_cast<unsigned char*>(base) + ((int64_t)b * Hkv + kvh) * C.rec_bytes;
}
__device__ __forceinline__ const unsigned char* cache_record(const void* base, const CacheLayout& C, int b, int Hkv,
                                                            int kvh) {
  return static_cast<const unsigned char*>(base) + ((int64_t)b * Hkv + kvh) * C.rec_bytes;
}

// Uniform integer in [0, R) for the arrival of token t: the four words of Philox4x32-10 under the counter
// (t, 2, KV head, 0) and the sequence's cache seed, each mapped by multiply-and-reject; the first accepted one
// counts, the fourth is taken regardless.  1 <= R <= 2^31.
constexpr uint32_t kCacheStream = 2u;
__device__ __forceinline__ uint32_t cache_draw(uint32_t t, uint32_t R, uint64_t seed, uint32_t kvh) {
  const Philox4 ph = philox4x32_10(t, kCacheStream, kvh, 0u, (uint32_t)seed, (uint32_t)(seed >> 32));
  const uint32_t thr = (uint32_t)((0x100000000ull - (uint64_t)R) % (uint64_t)R);
  uint32_t val = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const uint64_t x = (uint64_t)ph.v[w] * (uint64_t)R;
    val = (uint32_t)(x >> 32);
    if ((uint32_t)x >= thr) break;
  }
  return val;
}

// ---------------------------------------------------------------------------
// Per-head sizes of Algorithm 1's index sets, derived from the sequence length alone.
// ---------------------------------------------------------------------------
struct HeadSizes {
  int n, n_sink, n_win, mid_lo, mid_hi, k, n_s, b0;
};

struct SelectParams {
  int32_t sink, window, topk_abs, base_abs;
  double topk_frac, base_frac;  // the float parameters widened exactly
};

__host__ __device__ inline HeadSizes head_sizes(int n, const SelectParams& p) {
  HeadSizes h;
  h.n = n;
  h.n_sink = p.sink < n ? p.sink : n;
  h.n_win = p.window < n - h.n_sink ? p.window : n - h.n_sink;
  h.mid_lo = h.n_sink;
  h.mid_hi = n - h.n_win;
  const int m = h.mid_hi - h.mid_lo;
  int k = p.topk_abs > 0 ? p.topk_abs : (int)floor(p.topk_frac * (double)n);
  h.k = k < 0 ? 0 : (k > m ? m : k);
  h.n_s = m - h.k;
  int b0 = p.base_abs > 0 ? p.base_abs : (int)floor(p.base_frac * (double)h.n_s);
  h.b0 = b0 < 2 ? 2 : b0;
  h.b0 = h.b0 > h.n_s ? h.n_s : h.b0;
  return h;
}

}  // namespace vatt
