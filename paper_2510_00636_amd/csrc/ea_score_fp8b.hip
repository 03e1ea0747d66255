// More instances of the matrix-core score kernel for caches stored as OCP e4m3 bytes: head
// dimension 128 with four or five query heads per pass, head dimension 256.
#include "ea_score_mfma.h"

namespace ea {

hipError_t launch_score_mfma_fp8b(int D, const ScoreArgs& a, const ScorePlan& sp, hipStream_t st) {
#define EA_CASE(DD, GG, WW)                          \
  if (D == DD && sp.GH == GG && sp.NW == WW)         \
  return a.n < 32 ? launch_one<DD, GG, WW, true, true>(a, sp, st) : launch_one<DD, GG, WW, false, true>(a, sp, st)
  EA_CASE(128, 4, kNW128);
  EA_CASE(128, 5, kNW128);
  EA_CASE(256, 1, 4);
  EA_CASE(256, 2, 4);
#undef EA_CASE
  return hipErrorInvalidValue;
}

}  // namespace ea
