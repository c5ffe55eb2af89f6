/* A plain C99 client of include/asl.h: checks that the header compiles as C, prints the layout of the
 * ABI structs, and makes one host-only call.  Built and run by tests/test_abi.py. */
#include <stddef.h>
#include <stdio.h>

#include "asl.h"

int main(void) {
  printf("params %zu %zu %zu %zu %zu\n", sizeof(asl_params), offsetof(asl_params, k_stride_head),
         offsetof(asl_params, v_stride_tok), offsetof(asl_params, scale), offsetof(asl_params, flags));
  printf("state %zu %zu %zu\n", sizeof(asl_state), offsetof(asl_state, init_set), offsetof(asl_state, last_layer));
  printf("stat %zu %zu %zu %zu %zu\n", sizeof(asl_stat), offsetof(asl_stat, rel_var), offsetof(asl_stat, numerator),
         offsetof(asl_stat, union_size), offsetof(asl_stat, selected));
  printf("workspace %zu\n", asl_workspace_bytes(131072, 9, 1024));
  printf("status %d %d %d %d %d\n", (int)ASL_OK, (int)ASL_EINVAL, (int)ASL_ENOMEM, (int)ASL_EHIP, (int)ASL_EUNSUPPORTED);
  return 0;
}
