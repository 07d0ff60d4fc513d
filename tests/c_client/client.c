/* A plain C caller of the library's C-ABI (no Python, no torch, no HIP call of its own): reads a scenario from a
 * text file, loads it, searches it exhaustively, bounded and through the entry point that allocates nothing, and
 * prints what it found.  tests/test_c_client.py builds it with gcc, runs it on the GPU machine and compares its output
 * with the CPU oracle on the same tables. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "chm.h"

static int read_ints(FILE *f, int n, int32_t *out) {
  for (int i = 0; i < n; ++i)
    if (fscanf(f, "%d", &out[i]) != 1) return 0;
  return 1;
}

static void print_best(const char *what, int rc, const chm_best *b) {
  printf("%s rc=%d index=%llu cost=%lld strategy=%d stages=%d cuts=", what, rc, (unsigned long long)b->index, (long long)b->cost,
         b->strategy, b->stages);
  for (int i = 0; i + 1 < b->stages; ++i) printf("%s%d", i ? "," : "", b->cuts[i]);
  printf(" t_step=%lld t_trans=%lld reroute=", (long long)b->t_step_us, (long long)b->t_trans_us);
  for (int a = 0; a < b->n_affected; ++a)
    for (int d = 0; d < 16; ++d) printf("%s%d", (a || d) ? "," : "", b->reroute[a][d]);
  printf("\n");
}

int main(int argc, char **argv) {
  if (argc < 2) return 2;
  FILE *f = fopen(argv[1], "r");
  if (!f) return 2;
  chm_scenario_desc d;
  memset(&d, 0, sizeof(d));
  int32_t head[12];
  /* L PP DP M n_failed comm cap reroute_cap horizon reconf0 reconf1 reconf2, then xfer and has_speed */
  if (!read_ints(f, 12, head)) return 2;
  int32_t tail[2];
  if (!read_ints(f, 2, tail)) return 2;
  d.L = head[0]; d.PP = head[1]; d.DP = head[2]; d.M = head[3]; d.n_failed = head[4];
  d.comm_us = head[5]; d.mem_cap_mib = head[6]; d.reroute_cap = head[7]; d.horizon_steps = head[8];
  d.reconf_us[0] = head[9]; d.reconf_us[1] = head[10]; d.reconf_us[2] = head[11];
  d.xfer_us_per_mib = tail[0];
  int32_t *fwd = malloc(sizeof(int32_t) * d.L), *bwd = malloc(sizeof(int32_t) * d.L), *mem = malloc(sizeof(int32_t) * d.L);
  int32_t *failed = malloc(sizeof(int32_t) * (d.n_failed + 1));
  int32_t *speed = malloc(sizeof(int32_t) * d.DP * d.PP);
  if (!read_ints(f, d.L, fwd) || !read_ints(f, d.L, bwd) || !read_ints(f, d.L, mem) || !read_ints(f, d.n_failed, failed)) return 2;
  if (tail[1] && !read_ints(f, d.DP * d.PP, speed)) return 2;
  fclose(f);
  d.fwd_us = fwd; d.bwd_us = bwd; d.mem_mib = mem; d.failed_nodes = failed;
  d.speed_q16 = tail[1] ? (const uint32_t *)speed : NULL;

  chm_scenario *s = NULL;
  int rc = chm_load_scenario(&d, &s);
  if (rc != CHM_OK) { printf("load rc=%d (%s)\n", rc, chm_strerror(rc)); return 1; }
  chm_space sp;
  chm_plan_space(s, &sp);
  printf("space families=%d plans=%llu\n", sp.n_families, (unsigned long long)sp.n_plans);
  chm_best b;
  rc = chm_search_best(s, 7u, &b, NULL);            /* NULL = the default stream */
  print_best("exhaustive", rc, &b);
  for (int k = 0; k < 3; ++k) {
    rc = chm_search_best(s, 1u << k, &b, NULL);
    char name[32];
    snprintf(name, sizeof(name), "strategy%d", k);
    print_best(name, rc, &b);
  }
  rc = chm_search_best_static(s, 7u, &b, NULL);
  print_best("static", rc, &b);
  chm_set_bounded_search(s, 2);
  rc = chm_search_best(s, 7u, &b, NULL);
  print_best("bounded", rc, &b);
  chm_scenario *two[1] = {s};
  chm_best bb[1];
  int32_t codes[1];
  chm_set_bounded_search(s, 0);
  rc = chm_search_best_batch(two, 1, 7u, bb, codes, NULL);
  print_best("batch", rc ? rc : codes[0], &bb[0]);
  chm_free_scenario(s);
  free(fwd); free(bwd); free(mem); free(failed); free(speed);
  return 0;
}
