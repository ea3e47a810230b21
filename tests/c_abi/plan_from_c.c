/* The public header must be plain C and the library usable without C++ or Python: this program includes
 * include/vatt.h as C99, makes a plan for a 256-CU gfx950 without touching a GPU (device -1), and prints its
 * geometry.  Built and run by tests/test_library_host.py. */
#include <stdio.h>
#include <string.h>

#include "vatt.h"

int main(void) {
  vatt_params p;
  vatt_plan* plan = NULL;
  vatt_plan* chunk = NULL;
  int rc;
  memset(&p, 0, sizeof p);
  p.batch = 1;
  p.n_q_heads = 32;
  p.n_kv_heads = 8;
  p.head_dim = 128;
  p.n_max = 32768;
  p.kv_layout = VATT_LAYOUT_CONTIGUOUS;
  p.sink = 128;
  p.window = 128;
  p.topk_frac = 0.025f;
  p.base_frac = 0.025f;
  p.epsilon = 0.05f;
  p.delta = 0.05f;
  p.target = VATT_TARGET_D;
  p.budget_cap_frac = 1.0f;
  rc = vatt_plan_create(&p, -1, &plan);
  if (rc != VATT_OK) {
    printf("vatt_plan_create: %s\n", vatt_status_string(rc));
    return 1;
  }
  printf("workspace_bytes %zu\n", vatt_plan_workspace_bytes(plan));
  printf("index_capacity %zu\n", vatt_plan_index_capacity(plan));
  printf("segments %lld %lld %lld %lld %lld\n", (long long)vatt_plan_index_segment(plan, 0),
         (long long)vatt_plan_index_segment(plan, 1), (long long)vatt_plan_index_segment(plan, 2),
         (long long)vatt_plan_index_segment(plan, 3), (long long)vatt_plan_index_segment(plan, 4));
  rc = vatt_plan_set_option(plan, VATT_OPT_BUDGET_BOUND, VATT_BOUND_HOEFFDING);
  printf("hoeffding option %s\n", vatt_status_string(rc));
  rc = vatt_plan_create_chunk(&p, 4, -1, &chunk);
  printf("chunk plan %s q_len %d\n", vatt_status_string(rc), vatt_plan_query_len(chunk));
  vatt_plan_destroy(chunk);
  vatt_plan_destroy(plan);
  plan = NULL;
  p.epsilon = 2.0f;
  rc = vatt_plan_create(&p, -1, &plan); /* fails and leaves *out NULL: nothing to destroy */
  printf("bad epsilon: %s (plan %s)\n", vatt_status_string(rc), plan ? "set" : "null");
  /* a plan made without a device cannot launch */
  p.epsilon = 0.05f;
  rc = vatt_plan_create(&p, -1, &plan);
  if (rc != VATT_OK) return 1;
  rc = vatt_score(plan, &p, &p, NULL, (const int32_t*)&p, &p, 1u << 30, NULL);
  printf("launch without a device: %s\n", vatt_status_string(rc));
  vatt_plan_destroy(plan);
  return 0;
}
