// Instances of the matrix-core score kernel for head dimension 128 (four and five query heads per pass).
#include "ea_score_mfma.h"

namespace ea {

hipError_t launch_score_mfma_d128b(const ScoreArgs& a, const ScorePlan& sp, hipStream_t st) {
#define EA_CASE(GG, WW)                 \
  if (sp.GH == GG && sp.NW == WW)     \
  return (a.n < 32 || a.pm.table) ? launch_one<128, GG, WW, true>(a, sp, st) : launch_one<128, GG, WW, false>(a, sp, st)
  EA_CASE(4, kNW128);
  EA_CASE(5, kNW128);
#undef EA_CASE
  return hipErrorInvalidValue;
}

}  // namespace ea
