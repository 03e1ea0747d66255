// Host-only driver for the sanitizer build of ea_host.cpp (argument validation, tiling plans,
// workspace layout): sweeps shapes and sizes through them and checks the invariants the kernels
// and the entry points rely on.  Built with -fsanitize=address,undefined by
// tests/test_host_sanitizers.py; exits 0 when every check holds.
#include <initializer_list>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../paper_2510_00636_amd/csrc/ea_common.h"

static int failures = 0;
#define CHECK(cond)                                                              \
  do {                                                                           \
    if (!(cond)) {                                                               \
      fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond);   \
      ++failures;                                                                \
    }                                                                            \
  } while (0)

static ea_params params(int B, int Hq, int Hkv, int d, int dtype) {
  ea_params p;
  memset(&p, 0, sizeof p);
  p.batch = B; p.n_q_heads = Hq; p.n_kv_heads = Hkv; p.head_dim = d; p.dtype = dtype;
  p.q_is_rotated = 1; p.horizon_T = 512; p.epsilon = 0.02f;
  return p;
}

int main() {
  const int dims[] = {64, 128, 256};
  const int groups[] = {1, 2, 3, 4, 5, 7, 8, 16, 64};
  const int64_t sizes[] = {1, 31, 32, 33, 2047, 2048, 4608, 32768, 131072, (int64_t)1 << 22, (int64_t)1 << 26};
  const int cus[] = {1, 64, 256, 304};
  for (int d : dims)
    for (int G : groups)
      for (int Hkv : {1, 8})
        for (int B : {1, 4})
          for (int dtype : {(int)EA_F32, (int)EA_BF16}) {
            ea_params p = params(B, G * Hkv, Hkv, d, dtype);
            ea::Dims dd;
            CHECK(ea::check_params(&p, &dd) == EA_OK);
            CHECK(dd.units() == B * Hkv && dd.qheads() == B * G * Hkv && dd.G == G);
            for (int64_t n : sizes) {
              for (int cu : cus) {
                ea::ScorePlan sp = ea::make_score_plan(dd, n, cu);
                CHECK(sp.passes >= 1 && sp.GH >= 1 && sp.passes * sp.GH >= G);
                CHECK(sp.nfrag >= 1 && sp.npart >= 1 && sp.nchunk >= 1);
                CHECK((int64_t)sp.npart * sp.pg >= n);             // the partial blocks cover every key
                if (!sp.hw) CHECK(sp.lds_bytes <= 160 * 1024);
              }
              for (int64_t w : {(int64_t)1, (int64_t)128, (int64_t)4096}) {
                ea::WsLayout L = ea::make_ws_layout(dd, n, w);
                const size_t at[] = {L.tab, L.qproj, L.mu, L.sigma, L.frags, L.post, L.logits, L.vnorm, L.part,
                                     L.lse, L.scores, L.idx, L.base, L.hist, L.blk, L.flags, L.total};
                for (size_t i = 0; i + 1 < sizeof at / sizeof at[0]; ++i) {
                  CHECK(at[i] % 256 == 0);
                  CHECK(at[i] < at[i + 1]);                       // ordered, none empty
                }
                CHECK(ea_workspace_bytes(&p, n, w) == L.total);
                // the plan the launch uses (real CU count) never needs more than the layout reserved
                for (int cu : cus) {
                  ea::ScorePlan sp = ea::make_score_plan(dd, n, cu);
                  CHECK((size_t)dd.units() * sp.passes * sp.nfrag * 1024 <= L.post - L.frags);
                  if (dtype == EA_BF16) CHECK((size_t)dd.qheads() * sp.npart * 8 <= L.lse - L.part);
                }
              }
            }
          }
  // rejected parameters
  ea::Dims dd;
  ea_params p = params(1, 30, 8, 128, EA_BF16);
  CHECK(ea::check_params(&p, &dd) == EA_ERR_INVALID_ARG);
  p = params(1, 8, 8, 96, EA_BF16);
  CHECK(ea::check_params(&p, &dd) == EA_ERR_UNSUPPORTED);
  p = params(0, 8, 8, 128, EA_BF16);
  CHECK(ea::check_params(&p, &dd) == EA_ERR_INVALID_ARG);
  p = params(1, 8, 8, 128, 9);
  CHECK(ea::check_params(&p, &dd) == EA_ERR_UNSUPPORTED);
  p = params(1, 130, 1, 128, EA_BF16);
  CHECK(ea::check_params(&p, &dd) == EA_ERR_UNSUPPORTED);
  CHECK(ea::check_params(nullptr, &dd) == EA_ERR_INVALID_ARG);
  p = params(1, 8, 8, 128, EA_BF16);
  CHECK(ea_workspace_bytes(&p, 0, 128) == 0 && ea_workspace_bytes(&p, ((int64_t)1 << 26) + 1, 128) == 0);
  CHECK(ea_workspace_bytes(&p, 1024, 4097) == 0 && ea_workspace_bytes(nullptr, 1024, 128) == 0);
  // ea_n_keep: Listing 1's truncation, and its domain
  CHECK(ea_n_keep(1024, 0.5) == 512 && ea_n_keep(7, 0.5) == 3 && ea_n_keep(10, 0.0) == 10 && ea_n_keep(10, 1.0) == 0);
  CHECK(ea_n_keep(-1, 0.5) == -1 && ea_n_keep(10, 1.5) == -1 && ea_n_keep(10, -0.1) == -1);
  CHECK(ea_n_keep(((int64_t)1 << 40), 0.25) == ((int64_t)3 << 38));
  for (int s = -2; s < 8; ++s) CHECK(strlen(ea_status_string((ea_status)s)) > 0);
  if (failures) {
    fprintf(stderr, "%d check(s) failed\n", failures);
    return 1;
  }
  printf("host checks passed\n");
  return 0;
}
