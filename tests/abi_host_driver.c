/* Host-side exercise of the C ABI of libctm.so, in plain C, without a GPU: every entry point is called with arguments
 * that must be refused (or answered) on the host.  Built and run by tests/test_abi.py against the ordinary library,
 * and by tests/sanitize_host.py against a library whose host code is compiled with AddressSanitizer and
 * UndefinedBehaviorSanitizer (this program is then compiled with them too, so their runtime loads first).
 * Exit status 0 and the line "abi host driver: ok" mean every check held. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "ctm.h"
#include "ctm_bench.h"

static int failures = 0;
#define EXPECT(cond) do { if (!(cond)) { printf("FAILED line %d: %s  [last error: %s]\n", __LINE__, #cond, ctm_last_error()); ++failures; } } while (0)

int main(void) {
  ctm_mlp *out = (ctm_mlp *)0x1;
  int dims[3] = {5, 16, 1};
  const void *fake[2] = {(const void *)0x1000, (const void *)0x2000};
  /* handle creation: every host-side refusal */
  EXPECT(ctm_create_mlp(2, dims, fake, NULL, CTM_F32, CTM_ACT_TANH, NULL, NULL) == CTM_ERR_NULL);
  EXPECT(ctm_create_mlp(2, NULL, fake, NULL, CTM_F32, CTM_ACT_TANH, NULL, &out) == CTM_ERR_NULL && out == NULL);
  EXPECT(ctm_create_mlp(2, dims, fake, NULL, (ctm_dtype)7, CTM_ACT_TANH, NULL, &out) == CTM_ERR_DTYPE);
  EXPECT(ctm_create_mlp(2, dims, fake, NULL, CTM_F32, (ctm_act)9, NULL, &out) == CTM_ERR_DTYPE);
  EXPECT(ctm_create_mlp(1, dims, fake, NULL, CTM_F32, CTM_ACT_TANH, NULL, &out) == CTM_ERR_SHAPE);
  EXPECT(ctm_create_mlp(65, dims, fake, NULL, CTM_F32, CTM_ACT_TANH, NULL, &out) == CTM_ERR_SHAPE);
  { int bad[3] = {5, 0, 1}; EXPECT(ctm_create_mlp(2, bad, fake, NULL, CTM_F32, CTM_ACT_TANH, NULL, &out) == CTM_ERR_SHAPE); }
  { int wide[3] = {5, 16, 1025}; EXPECT(ctm_create_mlp(2, wide, fake, NULL, CTM_F32, CTM_ACT_TANH, NULL, &out) == CTM_ERR_UNSUPPORTED); }
  { const void *holes[2] = {(const void *)0x1000, NULL}; EXPECT(ctm_create_mlp(2, dims, holes, NULL, CTM_F32, CTM_ACT_TANH, NULL, &out) == CTM_ERR_NULL); }
  { const void *odd[2] = {(const void *)0x1002, (const void *)0x2000}; EXPECT(ctm_create_mlp(2, dims, odd, NULL, CTM_F64, CTM_ACT_SIN, NULL, &out) == CTM_ERR_ALIGN); }
  EXPECT(out == NULL);
  EXPECT(strlen(ctm_last_error()) > 0);
  /* a well-formed request on a machine without a GPU (or with one: then the device pointers are bogus and the request is
     never made): creation either fails cleanly after the handle was allocated on the host, or is skipped */
  if (getenv("CTM_DRIVER_NO_GPU")) {
    int rc = ctm_create_mlp(2, dims, fake, NULL, CTM_F32, CTM_ACT_TANH, NULL, &out);
    EXPECT(rc == CTM_ERR_HIP || rc == CTM_ERR_ALLOC);
    EXPECT(out == NULL);
  }
  /* pure host queries */
  EXPECT(ctm_rows_per_point(2, 50) == 52 && ctm_rows_per_point(4, 32) == 98);
  EXPECT(ctm_rows_per_point(3, 4) == -1 && ctm_rows_per_point(2, 0) == -1);
  {
    int P, MB, Rp, np;
    EXPECT(ctm_tile_plan(CTM_F32, 2, 50, &P, &MB, &Rp, &np) == CTM_OK && P == 4 && MB == 13 && Rp == 50 && np == 1);
    EXPECT(ctm_tile_plan(CTM_F64, 4, 300, &P, &MB, &Rp, &np) == CTM_OK && np == 4 && Rp * np >= 300 && P * (2 + 3 * Rp) <= 16 * MB);
    EXPECT(ctm_tile_plan(CTM_F32, 2, 1000000, NULL, NULL, NULL, &np) == CTM_OK && np > 1);
    EXPECT(ctm_tile_plan(CTM_F32, 3, 5, &P, &MB, &Rp, &np) == CTM_ERR_UNSUPPORTED);
    EXPECT(ctm_tile_plan((ctm_dtype)5, 2, 5, &P, &MB, &Rp, &np) == CTM_ERR_DTYPE);
    EXPECT(ctm_tile_plan(CTM_F32, 2, 0, &P, &MB, &Rp, &np) == CTM_ERR_SHAPE);
  }
  {
    long long n = 0, d = 0;
    int i22[2] = {2, 2}, j31[2] = {3, 1}, j40[2] = {4, 0}, j22[2] = {2, 2}, j32[2] = {3, 2};
    EXPECT(ctm_interpolation_gamma(2, i22, j31, &n, &d) == CTM_OK && n == -1 && d == 3);
    EXPECT(ctm_interpolation_gamma(2, i22, j40, &n, &d) == CTM_OK && n == 13 && d == 192);
    EXPECT(ctm_interpolation_gamma(2, i22, j22, &n, &d) == CTM_OK && n == 5 && d == 8);
    EXPECT(ctm_interpolation_gamma(2, i22, j32, &n, &d) == CTM_ERR_SHAPE);
    EXPECT(ctm_interpolation_gamma(5, i22, j22, &n, &d) == CTM_ERR_SHAPE);
    EXPECT(ctm_interpolation_gamma(2, NULL, j22, &n, &d) == CTM_ERR_NULL);
    /* the largest orders the call accepts: every j of |j| = 8 over four directions */
    int i4[4] = {2, 2, 2, 2}, j4[4];
    long count = 0;
    for (j4[0] = 0; j4[0] <= 8; ++j4[0])
      for (j4[1] = 0; j4[0] + j4[1] <= 8; ++j4[1])
        for (j4[2] = 0; j4[0] + j4[1] + j4[2] <= 8; ++j4[2]) {
          j4[3] = 8 - j4[0] - j4[1] - j4[2];
          EXPECT(ctm_interpolation_gamma(4, i4, j4, &n, &d) == CTM_OK && d > 0);
          ++count;
        }
    EXPECT(count == 165);
  }
  /* operator calls, size queries, recording / reverse calls without a handle */
  EXPECT(ctm_laplacian(NULL, NULL, 4, NULL, 5, 0, 1.0, NULL, NULL, NULL, 0, NULL) == CTM_ERR_NULL);
  EXPECT(ctm_laplacian_static(NULL, NULL, 4, NULL, 5, 0, 1.0, NULL, NULL, NULL) == CTM_ERR_NULL);
  EXPECT(ctm_weighted_laplacian(NULL, NULL, 4, NULL, 5, NULL, NULL, NULL, 0, NULL) == CTM_ERR_NULL);
  EXPECT(ctm_weighted_laplacian_rand(NULL, NULL, 4, NULL, 5, 0, NULL, 0, 0, NULL, NULL, NULL, 0, NULL) == CTM_ERR_NULL);
  EXPECT(ctm_biharmonic_rand(NULL, NULL, 4, NULL, 5, 0, NULL, NULL, NULL, 0, NULL) == CTM_ERR_NULL);
  EXPECT(ctm_biharmonic_exact(NULL, NULL, 4, NULL, NULL, NULL, 0, NULL) == CTM_ERR_NULL);
  EXPECT(ctm_taylor_standard(NULL, 2, NULL, 4, NULL, 5, 0, 1.0, NULL, NULL, NULL, 0, NULL) == CTM_ERR_NULL);
  EXPECT(ctm_taylor_standard(NULL, 3, NULL, 4, NULL, 5, 0, 1.0, NULL, NULL, NULL, 0, NULL) == CTM_ERR_UNSUPPORTED);
  EXPECT(ctm_laplacian_fwd(NULL, NULL, 4, NULL, 5, 0, 1.0, NULL, NULL, NULL, 0, NULL) == CTM_ERR_NULL);
  EXPECT(ctm_laplacian_bwd(NULL, 4, 5, 1.0, NULL, 0, NULL, NULL, NULL, NULL, NULL, 0, NULL) == CTM_ERR_NULL);
  EXPECT(ctm_biharmonic_rand_fwd(NULL, NULL, 4, NULL, 5, 0, NULL, NULL, NULL, 0, NULL) == CTM_ERR_NULL);
  EXPECT(ctm_biharmonic_rand_bwd(NULL, 4, 5, NULL, 0, NULL, NULL, NULL, NULL, NULL, 0, NULL) == CTM_ERR_NULL);
  EXPECT(ctm_biharmonic_exact_fwd(NULL, NULL, 4, NULL, NULL, NULL, 0, NULL) == CTM_ERR_NULL);
  EXPECT(ctm_biharmonic_exact_bwd(NULL, 4, NULL, 0, NULL, NULL, NULL, NULL, NULL, 0, NULL) == CTM_ERR_NULL);
  EXPECT(ctm_update_mlp(NULL, NULL, NULL, NULL) == CTM_ERR_NULL);
  EXPECT(ctm_destroy_mlp(NULL) == CTM_OK);
  EXPECT(ctm_workspace_bytes(NULL, 2, 4, 5) == 0 && ctm_workspace_bytes_standard(NULL, 2, 4, 5) == 0);
  EXPECT(ctm_tape_bytes(NULL, 4, 5) == 0 && ctm_backward_workspace_bytes(NULL, 4, 5) == 0);
  EXPECT(ctm_biharmonic_tape_bytes(NULL, 4, 5) == 0 && ctm_biharmonic_backward_workspace_bytes(NULL, 4, 5) == 0);
  EXPECT(ctm_biharmonic_exact_tape_bytes(NULL, 4) == 0 && ctm_biharmonic_exact_backward_workspace_bytes(NULL, 4) == 0);
  EXPECT(ctm_biharmonic_exact_workspace_bytes(NULL, 4) == 0);
  EXPECT(ctm_weighted_laplacian_rand_workspace_bytes(NULL, 4, 5, 3, 0, 0) == 0);
  /* the benchmark diagnostics with nothing recorded */
  {
    double ms[3] = {1, 1, 1};
    long n[3] = {1, 1, 1};
    EXPECT(ctm_profile_begin() == CTM_OK);
    EXPECT(ctm_profile_end(ms, n) == CTM_OK && ms[1] == 0.0 && n[1] == 0);
    EXPECT(ctm_profile_end(NULL, NULL) == CTM_OK);
  }
  if (failures) { printf("abi host driver: %d check(s) failed\n", failures); return 1; }
  printf("abi host driver: ok\n");
  return 0;
}
