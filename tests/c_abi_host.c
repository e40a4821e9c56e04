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
  printf("k=%lld sample=%lld rank=%lld small=%lu big=%lu slots=%lld status=\"%s\" version=%d\n", (long long)k,
         (long long)sample, (long long)rank, (unsigned long)small, (unsigned long)big, (long long)layout[3],
         dgc_status_string(DGC_ERR_CAPACITY), (int)dgc_version());
  return dgc_destroy(h) == DGC_OK ? 0 : 8;
}
