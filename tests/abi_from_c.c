/* The boundary used from plain C: the header must compile as C99 and the library must link and answer without a
 * GPU (a context made with device = -1 validates arguments and never launches). */
#include <stdio.h>
#include <string.h>

#include "ag.h"
#include "ag_bench.h"

int main(void) {
  ag_ctx *ctx = NULL;
  if (ag_create(&ctx, -1, 1 << 20) != AG_OK || !ctx) { puts("create failed"); return 1; }
  /* null tensors: rejected before anything else */
  if (ag_gate(ctx, NULL, NULL, AG_BF16, 1, 64, 64, NULL, NULL, 4, 0.5f, 0, NULL, NULL) != AG_EINVAL) { puts("null not rejected"); return 2; }
  if (strlen(ag_last_error(ctx)) == 0) { puts("no message"); return 3; }
  /* valid arguments but no device: AG_EHIP, nothing launched */
  static unsigned short x[64 * 64], w[64 * 4];
  static float bias[4];
  static unsigned char flags[4 * 64];
  ag_status st = ag_gate(ctx, NULL, x, AG_BF16, 1, 64, 64, w, bias, 4, AG_TAU_PRETRAIN, 0, NULL, flags);
  if (st != AG_EHIP) { printf("expected AG_EHIP, got %d\n", (int)st); return 4; }
  if (ag_workspace_bytes(1, 4096, 32, 32, 128, AG_BF16, 4096, 0) == 0) { puts("workspace size 0"); return 5; }
  if (ag_timing_kernels() < 7) { puts("timing ids"); return 6; }
  ag_destroy(ctx);
  puts("ok");
  return 0;
}
