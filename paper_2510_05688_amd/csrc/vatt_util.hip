// Measurement aids.  stream_read_kernel only reads a buffer: what it achieves on a buffer of a given size is
// the practical ceiling for any kernel that has to stream that many bytes from HBM in one launch (at 64 MiB the
// launch itself is a visible part of the time), which is what the K scan is compared with.  row_read_kernel
// only reads listed rows of 256 bytes (one K or V row at d = 128) in the access shape of the gather kernels
// (16 lanes per row, 8 rows in flight per lane group, the row numbers from a list): the ceiling for those.
#include "vatt_internal.h"

namespace vatt {
namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
constexpr int kReadU = 4;  // 16-byte loads in flight per thread

__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4_t* __restrict__ src, size_t n_vec,
                                                          uint32_t* __restrict__ sink) {
  const size_t base = (size_t)blockIdx.x * 256 * kReadU + threadIdx.x;
  u32x4_t v[kReadU];
#pragma unroll
  for (int u = 0; u < kReadU; ++u) {
    const size_t i = base + (size_t)u * 256;
    v[u] = i < n_vec ? __builtin_nontemporal_load(src + i) : u32x4_t{0u, 0u, 0u, 0u};
  }
  uint32_t acc = 0;
#pragma unroll
  for (int u = 0; u < kReadU; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  // a data-dependent store that practically never happens keeps the loads from being removed
  if (acc == 0x9e3779b9u) sink[blockIdx.x & 1023] = acc;
}

constexpr int kRowsInFlight = 8, kRowLanes = 16, kRowsPerWg = 256;

__global__ __launch_bounds__(256) void row_read_kernel(const u32x4_t* __restrict__ src, uint32_t rows_total,
                                                       const int32_t* __restrict__ rows, size_t count,
                                                       uint32_t* __restrict__ sink) {
  const int sub = threadIdx.x % kRowLanes, grp = threadIdx.x / kRowLanes;
  const size_t first = (size_t)blockIdx.x * kRowsPerWg;
  uint32_t acc = 0;
  for (int j0 = 0; j0 < kRowsPerWg; j0 += kRowsInFlight * (256 / kRowLanes)) {
    uint32_t t[kRowsInFlight];
#pragma unroll
    for (int u = 0; u < kRowsInFlight; ++u) {
      const size_t j = min(first + (size_t)(j0 + u * (256 / kRowLanes) + grp), count - 1);  // (a repeat of the last row)
      t[u] = min((uint32_t)max(rows[j], 0), rows_total - 1u);                            // no access leaves the buffer
    }
    u32x4_t v[kRowsInFlight];
#pragma unroll
    for (int u = 0; u < kRowsInFlight; ++u) v[u] = __builtin_nontemporal_load(src + (size_t)t[u] * kRowLanes + sub);
#pragma unroll
    for (int u = 0; u < kRowsInFlight; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x9e3779b9u) sink[blockIdx.x & 1023] = acc;
}

}  // namespace

hipError_t launch_row_read(const void* src, size_t rows_total, const int32_t* rows, size_t count, void* sink,
                           hipStream_t st) {
  if (count == 0) return hipSuccess;
  const size_t blocks = (count + kRowsPerWg - 1) / kRowsPerWg;
  if (blocks > 0x7fffffffull || rows_total == 0 || rows_total > 0x7fffffffull) return hipErrorInvalidValue;
  hipLaunchKernelGGL(row_read_kernel, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<const u32x4_t*>(src),
                     (uint32_t)rows_total, rows, count, static_cast<uint32_t*>(sink));
  return hipGetLastError();
}

hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, hipStream_t st) {
  const size_t n_vec = bytes / 16;
  const size_t per = 256 * (size_t)kReadU;
  const size_t blocks = (n_vec + per - 1) / per;
  if (blocks == 0) return hipSuccess;
  if (blocks > 0x7fffffffull) return hipErrorInvalidValue;
  hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                     static_cast<const u32x4_t*>(src), n_vec, static_cast<uint32_t*>(sink));
  return hipGetLastError();
}

}  // namespace vatt
