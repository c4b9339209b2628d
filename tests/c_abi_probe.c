/* A plain C99 translation unit that includes the library's header and calls the entry
 * points that need no GPU: proves that the boundary is usable from C (no C++ types, no
 * torch types), and prints values that the test compares with the oracle's. */
#include <stdio.h>
#include <stddef.h>
#include "trjacobi.h"

int main(void) {
  /* SplitMix64, seed 1234567, draws 1..3 */
  for (int k = 1; k <= 3; ++k) printf("%llu\n", (unsigned long long)trj_splitmix64(1234567u, (uint64_t)k));

  /* prompt lookup on a worked case: suffix (5,1) occurred before, most recently followed by 7,5 */
  int32_t ctx[8] = {5, 1, 9, 5, 1, 7, 5, 1};
  int32_t found[4] = {-1, -1, -1, -1};
  int32_t n_found = -1;
  int32_t rc = trj_prompt_lookup(ctx, 8, 2, 2, found, &n_found);
  printf("%d %d %d %d\n", (int)rc, (int)n_found, (int)found[0], (int)found[1]);

  /* argument errors come back as codes, nothing aborts */
  size_t bytes = 0;
  printf("%d\n", (int)trj_workspace_bytes(NULL, 64, 1, 1088, &bytes));
  trj_model_desc d = {2, 256, 4, 64, 1024, 2048, 1e-5f, 1e4f, TRJ_F32, 0};
  rc = trj_workspace_bytes(&d, 15, 1, 143, &bytes);
  printf("%d %d\n", (int)rc, bytes > 0);
  printf("%s\n", trj_version());
  return 0;
}
