// Instances of the matrix-core score kernel for head dimension 64.
#include "ea_score_mfma.h"

namespace ea {

hipError_t launch_score_mfma_d64(const ScoreArgs& a, const ScorePlan& sp, hipStream_t st) {
#define EA_CASE(GG, WW)                 \
  if (sp.GH == GG && sp.NW == WW)     \
  return (a.n < 32 || a.pm.table) ? launch_one<64, GG, WW, true>(a, sp, st) : launch_one<64, GG, WW, false>(a, sp, st)
  EA_CASE(1, 8);
  EA_CASE(2, 8);
  EA_CASE(4, 8);
  EA_CASE(8, 8);
#undef EA_CASE
  return hipErrorInvalidValue;
}

}  // namespace ea
