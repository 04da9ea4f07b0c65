/* The header is plain C and the host-only entry points work from a C program: layout of an
 * encoded matrix, its shared-exponent form, greedy and sampling acceptance, the objective of the
 * format search (Sec. 4.2, Sec. 2.2, Eq. 1, Eq. 2).  Exit code 0 = all checks passed. */
#include <stdio.h>
#include <string.h>

#include "cassandra.h"

#define CHECK(cond)                                              \
  do {                                                           \
    if (!(cond)) {                                               \
      fprintf(stderr, "line %d: %s\n", __LINE__, #cond);         \
      return 1;                                                  \
    }                                                            \
  } while (0)

int main(void) {
  cas_fmt fmt;
  cas_wdesc d;
  cas_mxdesc mx;
  int32_t draft[3] = {1, 2, 3}, target[4] = {1, 2, 9, 4}, out[4], n = -1;
  double p[2] = {0.2, 0.1}, q[2] = {0.4, 0.4}, r[2] = {0.4, 0.3}, j = 0.0;

  memset(&fmt, 0, sizeof fmt);
  fmt.keep_permille = 600;
  fmt.trunc_bits = 4;
  CHECK(cas_weight_desc(4096, 4096, &fmt, &d) == CAS_OK);
  CHECK(d.K == 2458 && d.bw == 128 && d.sw == 922 && d.lw == 308 && d.pw == 819);
  fmt.trunc_bits = 9;
  CHECK(cas_weight_desc(8, 8, &fmt, &d) == CAS_EINVAL);
  fmt.trunc_bits = 4;
  fmt.exp_mode = 1;
  CHECK(cas_weight_desc(8, 8, &fmt, &d) == CAS_ENOTSUP);
  fmt.exp_mode = 0;
  CHECK(cas_weight_desc(4096, 4096, &fmt, &d) == CAS_OK);
  CHECK(cas_mx_plan(&d, &mx) == CAS_OK);
  CHECK(mx.fw == (2458 * 5 + 31) / 32 && mx.ew == 128 && mx.spec_bytes % 256 == 0);

  CHECK(cas_accept(draft, target, 3, &n, out) == CAS_OK);
  CHECK(n == 2 && out[0] == 1 && out[1] == 2 && out[2] == 9);
  /* Eq. 1: r_1 = 0.4 <= p/q = 0.5 accepts the first token, r_2 = 0.3 > 0.25 rejects the second */
  CHECK(cas_accept_sampling(p, q, r, 2, &n) == CAS_OK && n == 1);
  /* Eq. 2 with no cache term: J = alpha / (S_w * kept fraction * (16 - t)) */
  CHECK(cas_objective(1.0, 4096.0, 600, 4, 0.0, 600, 4, 16, &j) == CAS_OK);
  CHECK(j > 0.0 && 1.0 / j > 29491.1 && 1.0 / j < 29491.3);
  CHECK(strcmp(cas_strerror(CAS_OK), "ok") == 0);
  puts("abi host calls ok");
  return 0;
}
