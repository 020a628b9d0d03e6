/* A plain C99 caller of the library: host-only entry points, printed one per line for the test that
 * builds and runs this file (tests/test_host_abi.py).  No GPU is touched. */
#include <stdio.h>
#include <string.h>

#include "qcache.h"

int main(void) {
  uint8_t mask[4] = {0, 1, 1, 0};
  qc_config cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.n_layers = 4;
  cfg.n_heads = 2;
  cfg.head_dim = 64;
  cfg.dtype = QC_BF16;
  cfg.max_batch = 3;
  cfg.max_seq = 192;
  cfg.max_vis = 64;
  cfg.max_text = 128;
  cfg.lazy_mask = mask;
  printf("kv_arena_bytes %zu\n", qc_kv_arena_bytes(&cfg));
  printf("q_arena_bytes %zu\n", qc_q_arena_bytes(&cfg));
  printf("page_table_bytes %zu\n", qc_page_table_bytes(&cfg));
  int32_t pages[3] = {-1, -1, -1};
  qc_status st = qc_pages_needed(&cfg, 130, 65, pages);
  printf("pages_needed %d %d %d %d\n", (int)st, (int)pages[0], (int)pages[1], (int)pages[2]);
  int32_t max_batch = -1;
  st = qc_plan_max_batch(&cfg, (size_t)1 << 20, QC_PLAN_KV | QC_PLAN_Q, &max_batch);
  printf("plan_max_batch %d %d\n", (int)st, (int)max_batch);
  st = qc_pages_needed(&cfg, 5, 6, pages);   /* more visual tokens than tokens: refused */
  printf("bad_call %d %s\n", (int)st, qc_status_str(st));
  printf("last_error %s\n", qc_last_error());
  return 0;
}
