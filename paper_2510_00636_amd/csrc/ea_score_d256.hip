// Instances of the matrix-core score kernel for head dimension 256.
#include "ea_score_mfma.h"

namespace ea {

hipError_t launch_score_mfma_d256(const ScoreArgs& a, const ScorePlan& sp, hipStream_t st) {
#define EA_CASE(GG, WW)                 \
  if (sp.GH == GG && sp.NW == WW)     \
  return (a.n < 32 || a.pm.table) ? launch_one<256, GG, WW, true>(a, sp, st) : launch_one<256, GG, WW, false>(a, sp, st)
  EA_CASE(1, 4);
  EA_CASE(2, 4);
#undef EA_CASE
  return hipErrorInvalidValue;
}

}  // namespace ea
