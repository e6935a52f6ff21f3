/* Driver for the sanitizer build of the host planner (csrc/deft_host.cpp compiled with
 * -fsanitize=address,undefined by tests/test_host_library.py).  It walks the host entry points
 * over seeded shapes, with every output array allocated at exactly the documented size, so an
 * out-of-bounds access, an overflow or a use of uninitialised capacity is reported by the
 * sanitizer run-time (which then aborts).  Results are checked only for their invariants. */
#include <stdio.h>
#include <stdlib.h>

#include "deft.h"

static uint64_t state = 88172645463325252ull;
static uint64_t next_u64(void) { /* xorshift64 */
  state ^= state << 13; state ^= state >> 7; state ^= state << 17;
  return state;
}

int main(void) {
  int round;
  for (round = 0; round < 400; ++round) {
    const int32_t T = 1 + (int32_t)(next_u64() % 40);
    const int32_t n = 1 + (int32_t)(next_u64() % 9);
    int64_t* sizes_t = (int64_t*)malloc(sizeof(int64_t) * T);
    int64_t N = 0, need = 0, K = 0, sum_k = 0;
    int32_t t, L = 0, l, count = 0, leader = 0;
    for (t = 0; t < T; ++t) {
      sizes_t[t] = (int64_t)(next_u64() % (round % 3 == 0 ? 12 : 5000));
      N += sizes_t[t];
    }
    if (N == 0) { sizes_t[0] = 3; N = 3; }
    for (t = 0; t < T; ++t) {
      const int64_t s = sizes_t[t];
      need += s == 0 ? 0 : (s * n > N ? (s < n ? s : n) : 1);
    }
    {
      /* capacity exactly what is needed: one layer fewer must be refused, untouched */
      int64_t* off = (int64_t*)malloc(sizeof(int64_t) * (need + 1));
      int32_t* lt = (int32_t*)malloc(sizeof(int32_t) * (need > 0 ? need : 1));
      if (need > 0 && deft_partition(sizes_t, T, n, off, lt, (int32_t)need - 1, &L) != DEFT_ECAP) return 2;
      if (deft_partition(sizes_t, T, n, off, lt, (int32_t)need, &L) != DEFT_OK || L != need) return 3;
      if (deft_check_layout(off, L, N) != DEFT_OK) return 4;
      {
        int64_t* sz = (int64_t*)malloc(sizeof(int64_t) * L);
        int64_t* k = (int64_t*)malloc(sizeof(int64_t) * L);
        double* ss = (double*)malloc(sizeof(double) * L);
        double* nr = (double*)malloc(sizeof(double) * L);
        int32_t* owner = (int32_t*)malloc(sizeof(int32_t) * L);
        int32_t* mine = (int32_t*)malloc(sizeof(int32_t) * L);
        double* Ci = (double*)malloc(sizeof(double) * n);
        double out5[5];
        const double d = 1.0 / (double)(1 + next_u64() % 200);
        for (l = 0; l < L; ++l) {
          sz[l] = off[l + 1] - off[l];
          if (sz[l] < 1 || sz[l] > (N + n - 1) / n) return 5; /* Sec. 4.1: at most ceil(n_g/n) */
          ss[l] = (next_u64() % 7 == 0) ? 0.0 : (double)(next_u64() % 100000) / 64.0;
        }
        if (deft_norms_from_sumsq(ss, L, nr) != DEFT_OK) return 6;
        if (deft_total_k(N, d, &K) != DEFT_OK || K < 0 || K > N) return 7;
        if (deft_alloc_k(nr, sz, L, N, d, k) != DEFT_OK) return 8;
        for (l = 0; l < L; ++l) {
          if (k[l] < 1 || k[l] > sz[l]) return 9;
          sum_k += k[l];
        }
        if (deft_assign_layers(sz, k, L, n, (int64_t)(next_u64() % 100), (int32_t)(next_u64() % n),
                               owner, mine, &count) != DEFT_OK) return 10;
        if (count < 0 || count > L) return 11;
        for (l = 0; l < L; ++l) if (owner[l] < 0 || owner[l] >= n) return 12;
        if (K >= 1 && deft_cost_model(sz, k, owner, L, n, N, K, Ci, out5) != DEFT_OK) return 13;
        if (deft_cltk_leader((int64_t)round, n, &leader) != DEFT_OK || leader != round % n) return 14;
        free(sz); free(k); free(ss); free(nr); free(owner); free(mine); free(Ci);
      }
      free(off); free(lt);
    }
    free(sizes_t);
  }
  printf("host sanitize ok\n");
  return 0;
}
