/* A caller written in C: reads a workload from a file, puts it on GPU 0 with the HIP runtime's C API, runs
 * vatt_decode through include/vatt.h and writes what came back to another file.  No C++, no Python, no torch in
 * the process.  Built and run by tests/test_gpu_c_caller.py, which compares the outputs with the oracle.
 *
 *   decode_from_c <input> <output>
 *
 * input:  int32 header {B, Hq, Hkv, d, n_max, sink, window, topk_abs, base_abs}, float header {topk_frac,
 *         base_frac, epsilon, delta}, then q (uint16 [B, Hq, d]), k and v (uint16 [B, Hkv, n_max, d]),
 *         seq_lens (int32 [B]), seeds (uint64 [B]).
 * output: int64 header {idx_cap, seg0..seg4}, then out_o (float [B, Hq, d]), out_lse (float [B, Hq]),
 *         out_idx (int32 [B, Hq, idx_cap]), out_counts (int32 [B, Hq, 8]), out_budget_raw (double [B, Hq]),
 *         out_stats (float [B, Hq, 4]).
 */
#define __HIP_PLATFORM_AMD__ 1 /* the HIP runtime's C API header asks for the platform when hipcc is not the compiler */
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "vatt.h"

#define CHECK_HIP(call)                                                            \
  do {                                                                             \
    hipError_t e_ = (call);                                                        \
    if (e_ != hipSuccess) {                                                        \
      fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));                   \
      return 2;                                                                    \
    }                                                                              \
  } while (0)

static int read_all(FILE* f, void* dst, size_t bytes) { return fread(dst, 1, bytes, f) == bytes ? 0 : -1; }

/* Reads `bytes` from the file into a fresh device buffer. */
static int upload(FILE* f, size_t bytes, void** dev) {
  void* host = malloc(bytes);
  if (!host || read_all(f, host, bytes) != 0) {
    free(host);
    return -1;
  }
  if (hipMalloc(dev, bytes) != hipSuccess || hipMemcpy(*dev, host, bytes, hipMemcpyHostToDevice) != hipSuccess) {
    free(host);
    return -1;
  }
  free(host);
  return 0;
}

/* Copies a device buffer to the output file. */
static int download(FILE* f, const void* dev, size_t bytes) {
  void* host = malloc(bytes);
  int rc = -1;
  if (host && hipMemcpy(host, dev, bytes, hipMemcpyDeviceToHost) == hipSuccess && fwrite(host, 1, bytes, f) == bytes)
    rc = 0;
  free(host);
  return rc;
}

int main(int argc, char** argv) {
  int32_t hi[9];
  float hf[4];
  vatt_params p;
  vatt_plan* plan = NULL;
  void *q = NULL, *k = NULL, *v = NULL, *seq_lens = NULL, *seeds = NULL, *ws = NULL;
  void *out_o = NULL, *out_lse = NULL, *out_idx = NULL, *out_counts = NULL, *out_braw = NULL, *out_stats = NULL;
  size_t heads, kv_elems, idx_cap, ws_bytes;
  int64_t ho[6];
  FILE *fin, *fout;
  int rc, s;
  if (argc != 3) return 64;
  fin = fopen(argv[1], "rb");
  if (!fin || read_all(fin, hi, sizeof hi) != 0 || read_all(fin, hf, sizeof hf) != 0) return 65;
  memset(&p, 0, sizeof p);
  p.batch = hi[0];
  p.n_q_heads = hi[1];
  p.n_kv_heads = hi[2];
  p.head_dim = hi[3];
  p.n_max = hi[4];
  p.kv_layout = VATT_LAYOUT_CONTIGUOUS;
  p.sink = hi[5];
  p.window = hi[6];
  p.topk_abs = hi[7];
  p.base_abs = hi[8];
  p.topk_frac = hf[0];
  p.base_frac = hf[1];
  p.epsilon = hf[2];
  p.delta = hf[3];
  p.target = VATT_TARGET_D;
  p.sm_scale = 0.0f; /* 1 / sqrt(d) */
  p.budget_cap_frac = 1.0f;
  CHECK_HIP(hipSetDevice(0));
  rc = vatt_plan_create(&p, 0, &plan);
  if (rc != VATT_OK) {
    fprintf(stderr, "vatt_plan_create: %s\n", vatt_status_string(rc));
    return 3;
  }
  heads = (size_t)p.batch * (size_t)p.n_q_heads;
  kv_elems = (size_t)p.batch * (size_t)p.n_kv_heads * (size_t)p.n_max * (size_t)p.head_dim;
  if (upload(fin, heads * (size_t)p.head_dim * 2, &q) || upload(fin, kv_elems * 2, &k) || upload(fin, kv_elems * 2, &v) ||
      upload(fin, (size_t)p.batch * 4, &seq_lens) || upload(fin, (size_t)p.batch * 8, &seeds)) {
    fprintf(stderr, "could not read or upload the workload\n");
    return 4;
  }
  fclose(fin);
  idx_cap = vatt_plan_index_capacity(plan);
  ws_bytes = vatt_plan_workspace_bytes(plan);
  CHECK_HIP(hipMalloc(&ws, ws_bytes));
  CHECK_HIP(hipMalloc(&out_o, heads * (size_t)p.head_dim * 4));
  CHECK_HIP(hipMalloc(&out_lse, heads * 4));
  CHECK_HIP(hipMalloc(&out_idx, heads * idx_cap * 4));
  CHECK_HIP(hipMalloc(&out_counts, heads * 8 * 4));
  CHECK_HIP(hipMalloc(&out_braw, heads * 8));
  CHECK_HIP(hipMalloc(&out_stats, heads * 4 * 4));
  CHECK_HIP(hipMemset(out_idx, 0xff, heads * idx_cap * 4));
  CHECK_HIP(hipDeviceSynchronize());
  /* a workspace one byte short is refused before anything is launched */
  rc = vatt_decode(plan, q, k, v, NULL, (const int32_t*)seq_lens, (const uint64_t*)seeds, ws, ws_bytes - 1,
                   (float*)out_o, (float*)out_lse, (int32_t*)out_idx, (int32_t*)out_counts, (double*)out_braw,
                   (float*)out_stats, NULL);
  printf("short workspace: %s\n", vatt_status_string(rc));
  if (rc != VATT_E_WORKSPACE_TOO_SMALL) return 5;
  rc = vatt_decode(plan, q, k, v, NULL, (const int32_t*)seq_lens, (const uint64_t*)seeds, ws, ws_bytes,
                   (float*)out_o, (float*)out_lse, (int32_t*)out_idx, (int32_t*)out_counts, (double*)out_braw,
                   (float*)out_stats, NULL);
  printf("vatt_decode: %s\n", vatt_status_string(rc));
  if (rc != VATT_OK) return 6;
  CHECK_HIP(hipDeviceSynchronize());
  fout = fopen(argv[2], "wb");
  if (!fout) return 66;
  ho[0] = (int64_t)idx_cap;
  for (s = 0; s < 5; ++s) ho[1 + s] = vatt_plan_index_segment(plan, s);
  if (fwrite(ho, 1, sizeof ho, fout) != sizeof ho || download(fout, out_o, heads * (size_t)p.head_dim * 4) ||
      download(fout, out_lse, heads * 4) || download(fout, out_idx, heads * idx_cap * 4) ||
      download(fout, out_counts, heads * 8 * 4) || download(fout, out_braw, heads * 8) ||
      download(fout, out_stats, heads * 4 * 4)) {
    fprintf(stderr, "could not write the results\n");
    return 7;
  }
  fclose(fout);
  vatt_plan_destroy(plan);
  hipFree(q); hipFree(k); hipFree(v); hipFree(seq_lens); hipFree(seeds); hipFree(ws);
  hipFree(out_o); hipFree(out_lse); hipFree(out_idx); hipFree(out_counts); hipFree(out_braw); hipFree(out_stats);
  printf("done\n");
  return 0;
}
