/* Plain C99 client of include/deft.h: proves the header is valid C and that the host entry
 * points can be called without Python.  Built and run by tests/test_host_library.py. */
#include <stdio.h>
#include <string.h>

#include "deft.h"

int main(void) {
  const int64_t tensor_sizes[3] = {11, 3, 6}; /* N = 20, n = 2: the first tensor splits 6 + 5 */
  int64_t offsets[7];
  int32_t layer_tensor[6];
  int32_t L = 0;
  if (deft_partition(tensor_sizes, 3, 2, offsets, layer_tensor, 6, &L) != DEFT_OK) return 1;
  if (L != 4 || offsets[1] != 6 || offsets[2] != 11 || offsets[3] != 14 || offsets[4] != 20) return 2;
  if (deft_check_layout(offsets, L, 20) != DEFT_OK) return 3;
  {
    const double sumsq[4] = {64.0, 16.0, 4.0, 4.0};
    double norms[4];
    int64_t sizes[4], k[4];
    int32_t owner[4], mine[4], count = 0, l;
    double out5[5];
    for (l = 0; l < 4; ++l) sizes[l] = offsets[l + 1] - offsets[l];
    if (deft_norms_from_sumsq(sumsq, 4, norms) != DEFT_OK || norms[0] != 8.0) return 4;
    /* K = floor(20 * 0.4 + 0.5) = 8 over norms 8,4,2,2: 4, 2, 1, 1 */
    if (deft_alloc_k(norms, sizes, 4, 20, 0.4, k) != DEFT_OK) return 5;
    if (k[0] != 4 || k[1] != 2 || k[2] != 1 || k[3] != 1) return 6;
    if (deft_assign_layers(sizes, k, 4, 2, 0, 0, owner, mine, &count) != DEFT_OK) return 7;
    if (owner[0] != 0 || owner[1] != 1 || count < 1 || mine[0] != 0) return 8;
    if (deft_cost_model(sizes, k, owner, 4, 2, 20, 8, NULL, out5) != DEFT_OK) return 9;
  }
  if (deft_partition(tensor_sizes, 3, 0, offsets, layer_tensor, 6, &L) != DEFT_EINVAL) return 10;
  if (strcmp(deft_strerror(DEFT_ECAP), "output capacity too small") != 0) return 11;
  if (deft_workspace_bytes(DEFT_OP_NORMS, 1 << 20, 4) == 0) return 12;
  /* device entry points reject bad arguments before touching a GPU */
  if (deft_layer_norms(NULL, 16, NULL, 1, NULL, NULL, 0, NULL) != DEFT_EINVAL) return 13;
  if (topk_global(NULL, 16, 4, NULL, NULL, NULL, 0, DEFT_SHAPE_AUTO, NULL) != DEFT_EINVAL) return 14;
  if (deft_gather_zero(NULL, 16, NULL, 0, NULL, NULL) != DEFT_OK) return 15;
  {
    int64_t K = 0, count = -1;
    int32_t leader = -1;
    /* Alg. 3, first statement: 300938 * 0.01 = 3009.38 -> 3009; 150 * 0.01 = 1.5 -> 2 */
    if (deft_total_k(300938, 0.01, &K) != DEFT_OK || K != 3009) return 16;
    if (deft_total_k(150, 0.01, &K) != DEFT_OK || K != 2) return 17;
    if (deft_total_k(150, 0.0, &K) != DEFT_EINVAL) return 18;
    /* cyclic local Top-k: iteration 7 of 4 workers is worker 3's turn; the others select
     * nothing and touch no device */
    if (deft_cltk_leader(7, 4, &leader) != DEFT_OK || leader != 3) return 19;
    if (deft_cltk_select(NULL, 1000, 0.01, 4, 1, 7, NULL, NULL, 0, NULL, 0, DEFT_SHAPE_AUTO, NULL,
                         &count) != DEFT_OK || count != 0) return 20;
    if (deft_cltk_select(NULL, 1000, 0.01, 4, 3, 7, NULL, NULL, 0, NULL, 0, DEFT_SHAPE_AUTO, NULL,
                         &count) != DEFT_ECAP) return 21;
  }
  printf("c abi ok\n");
  return 0;
}
