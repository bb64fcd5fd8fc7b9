/* Plain C99 user of the library's C ABI: only calls that need no GPU (option defaults,
 * workspace sizing, argument checks, error strings).  Built and run by tests/test_abi.py. */
#include <stdio.h>
#include <string.h>

#include "cce.h"

int main(void) {
  cce_opts o;
  cce_default_opts(CCE_BF16, &o);
  if (o.dtype != CCE_BF16 || o.flags != (CCE_FILTER_DE | CCE_FILTER_DC) || o.workspace != NULL) return 1;
  size_t fwd = cce_workspace_bytes(CCE_OP_FORWARD, 8192, 2304, 256000, &o);
  size_t bwd = cce_workspace_bytes(CCE_OP_BACKWARD, 8192, 2304, 256000, &o);
  size_t mn = cce_workspace_bytes(CCE_OP_BACKWARD_MIN, 8192, 2304, 256000, &o);
  size_t wide = cce_workspace_bytes(CCE_OP_BACKWARD_WIDE, 8192, 2304, 256000, &o);
  if (!(fwd > 0 && mn > 0 && mn < bwd && bwd < wide)) return 2;
  /* null pointers are rejected before anything is launched */
  float x;
  int st = cce_forward_ex(NULL, NULL, NULL, 8, 64, 16, 0.0f, -100, &x, &x, &o);
  if (st != CCE_EINVAL) return 3;
  if (strlen(cce_strerror(st)) == 0 || strcmp(cce_strerror(CCE_OK), cce_strerror(st)) == 0) return 4;
  int br = 0, bc = 0;
  cce_filter_block(8192, 2304, 256000, &o, &br, &bc);
  printf("forward %zu backward %zu min %zu wide %zu block %dx%d\n", fwd, bwd, mn, wide, br, bc);
  return 0;
}
