/* The C ABI used from plain C: the paper's W_init = 32, G_init = 8 example (Sec. 4.3, boundary
 * walk-through appendix) on a host-only context.  Prints key = value lines that the test compares
 * with tests/golden/walkthrough_w32_g8.txt.  Built with gcc -std=c99 -pedantic by test_c_abi.py. */
#include <stdio.h>
#include <string.h>

#include "recover.h"

static uint32_t next_id = 0; /* ids only have to ascend within a replica */

/* Every live replica accumulates until its quota is met (Alg. 1, local accumulation). */
static int fill_quota(recover_ctx *ctx, int W, const int32_t *role) {
  int r, k;
  for (r = 0; r < W; ++r) {
    if (role[r] == RECOVER_ROLE_DEAD) continue;
    for (k = 0; k < 64; ++k) {
      int rc = recover_accumulate(ctx, r, next_id++, NULL, RECOVER_F32, 0, 1, NULL);
      if (rc == RECOVER_SKIPPED) break;
      if (rc != RECOVER_OK) return rc;
    }
  }
  return 0;
}

int main(void) {
  enum { W = 32, G = 8 };
  int64_t off[2] = {0, 1024};
  int32_t role[W], target[W], contributed[W], bm[W], failed[1];
  recover_config cfg;
  recover_decision d;
  recover_ctx *ctx = NULL;
  int r, n9 = 0, n8 = 0, rc;

  memset(&cfg, 0, sizeof cfg);
  cfg.W_init = W;
  cfg.G_init = G;
  cfg.n_elems = 1024;
  cfg.n_tensors = 1;
  cfg.tensor_offsets = off;
  cfg.flags = RECOVER_FLAG_HOST_ONLY;
  if (recover_init(&cfg, &ctx) != RECOVER_OK) { printf("init failed: %s\n", recover_last_error(NULL)); return 1; }
  memset(&d, 0, sizeof d);
  d.role = role; d.target = target; d.contributed = contributed; d.is_boundary_minor = bm;
  recover_query(ctx, &d);
  printf("B = %d\n", d.n_maj * d.G_cur);
  if ((rc = fill_quota(ctx, W, role)) != 0) { printf("accumulate: %d %s\n", rc, recover_last_error(ctx)); return 1; }

  failed[0] = 31;                                   /* r32 fails during iteration t* */
  if (recover_policy_adjust(ctx, failed, 1, &d) != RECOVER_OK) return 1;
  printf("W_cur_after_first = %d\nC_cur = %d\nat_boundary = %d\nG_ext = %d\nn_bdry = %d\nloop_bound_after = %d\n",
         d.W_cur, d.C_cur, d.at_boundary, d.G_ext, d.n_bdry, d.loop_bound);
  for (r = 0; r < W; ++r) { if (role[r] != RECOVER_ROLE_DEAD) { n9 += target[r] == 9; n8 += target[r] == 8; } }
  printf("majors_extended = %d\nboundary_minors_at_8 = %d\n", n9, n8);
  printf("restore_mode_first = %s\n", d.restore_mode == RECOVER_RESTORE_NONBLOCKING ? "nonblocking" : "other");
  if (recover_restore(ctx, -1, 1, NULL) != RECOVER_OK) return 1;
  if (fill_quota(ctx, W, role) != 0) return 1;               /* the extended pass */
  if (recover_reduce(ctx, 0, 1, 0, NULL) != RECOVER_OK) return 1;
  if (recover_adamw_step(ctx, 1e-3f, 0.9f, 0.95f, 1e-8f, 0.1f, NULL) != RECOVER_OK) {
    printf("adamw: %s\n", recover_last_error(ctx));
    return 1;
  }
  if (recover_policy_adjust(ctx, NULL, 0, &d) != RECOVER_OK) return 1; /* advancement */
  printf("G_cur = %d\nn_maj = %d\nR_cur = %d\nn_min = %d\nn_ms = %d\nn_mi = %d\n", d.G_cur, d.n_maj, d.R_cur, d.n_min,
         d.n_ms, d.n_mi);
  for (r = 0; r < W; ++r) {
    if (role[r] == RECOVER_ROLE_MINOR) printf("minor_is = %d\n", r + 1);
    if (role[r] == RECOVER_ROLE_MINOR_SPARE) printf("minor_spare_is = %d\n", r + 1);
  }
  if (fill_quota(ctx, W, role) != 0) return 1;
  failed[0] = 28;                                   /* the minor r29 fails: the minor-spare r31 takes over */
  if (recover_policy_adjust(ctx, failed, 1, &d) != RECOVER_OK) return 1;
  printf("at_boundary_second = %d\nloop_bound_second = %d\n", d.at_boundary, d.loop_bound);
  printf("restore_mode_second = %s\n", d.restore_mode == RECOVER_RESTORE_BLOCKING ? "blocking" : "other");
  for (r = 0; r < W; ++r)
    if (r == 30 && role[r] == RECOVER_ROLE_MINOR) printf("promoted_second = %d\n", r + 1);
  recover_destroy(ctx);
  return 0;
}
