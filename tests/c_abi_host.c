/* A C99 caller of the library's host-side entry points: the header must compile as
 * strict C, and a handle must be usable without any device call (plan arithmetic,
 * workspace sizes, payload layout, argument checks).  Built and run by test_c_abi.py. */
#include <stdio.h>

#include "dgc.h"

int main(void) {
  dgc_config cfg;
  const int64_t offsets[4] = {0, 9408, 9472, 300000};
  dgc_handle* h = NULL;
  int64_t k = 0, sample = 0, rank = 0, draws = 0;
  size_t small = 0, big = 0;
  int64_t layout[4];
  if (dgc_config_default(&cfg) != DGC_OK) return 1;
  cfg.density = 0.001;
  if (dgc_create(&h, &cfg, 3, offsets) != DGC_OK) return 2;
  if (dgc_query_plan(h, 2, &k, &sample, &rank, &draws) != DGC_OK) return 3;
  if (dgc_workspace_bytes(h, &small) != DGC_OK || dgc_workspace_bytes_warmup(h, &big) != DGC_OK) return 4;
  if (dgc_recommended_payload_layout(h, 0.001, layout) != DGC_OK) return 5;
  /* null buffers are refused before anything is enqueued */
  if (dgc_compress(h, NULL, NULL, NULL, NULL, NULL, layout, NULL, NULL, 0, NULL, 0, NULL) != DGC_ERR_INVALID_ARG)
    return 6;
  if (dgc_set_density(h, 2.0) != DGC_ERR_INVALID_ARG) return 7;
  /* the host arithmetic at every density of the warm-up table, and the setters that change it */
  {
    const double table[3] = {0.5, 0.01, 0.002};
    int64_t it;
    if (dgc_set_warmup_schedule(h, table, 3) != DGC_OK || dgc_set_warmup_stage_length(h, 2) != DGC_OK) return 9;
    for (it = 0; it < 8; ++it) {
      int32_t j;
      if (dgc_set_iteration_density(h, it) != DGC_OK) return 10;
      for (j = 0; j < 3; ++j) {
        int64_t kk = 0, ss = 0, rr = 0, dd = 0;
        if (dgc_query_plan(h, j, &kk, &ss, &rr, &dd) != DGC_OK || kk < 1 || ss < 1 || rr < 1) return 11;
      }
      if (dgc_recommended_payload_layout(h, table[it / 2 < 2 ? it / 2 : 2], layout) != DGC_OK) return 12;
    }
    if (dgc_set_density(h, 0.001) != DGC_OK) return 13;
    if (dgc_recommended_payload_layout(h, 0.001, layout) != DGC_OK) return 14;
    if (dgc_set_scale_override(h, 0.5f) != DGC_OK || dgc_invalidate_workspace(h) != DGC_OK) return 15;
    if (dgc_query_plan(h, 3, &k, &sample, &rank, &draws) != DGC_ERR_INVALID_ARG) return 16;
    if (dgc_query_plan(h, 2, &k, &sample, &rank, &draws) != DGC_OK) return 17;
  }
  printf("k=%lld sample=%lld rank=%lld small=%lu big=%lu slots=%lld status=\"%s\" version=%d\n", (long long)k,
         (long long)sample, (long long)rank, (unsigned long)small, (unsigned long)big, (long long)layout[3],
         dgc_status_string(DGC_ERR_CAPACITY), (int)dgc_version());
  return dgc_destroy(h) == DGC_OK ? 0 : 8;
}
