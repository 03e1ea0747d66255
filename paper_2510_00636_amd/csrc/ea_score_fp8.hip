// Instances of the matrix-core score kernel for caches stored as OCP e4m3 bytes (head dimension
// 128: groups of one to five query heads per pass; 256: one or two).  The row-clamping instance
// serves heads shorter than one tile.
#include "ea_score_mfma.h"

namespace ea {

hipError_t launch_score_mfma_fp8(int D, const ScoreArgs& a, const ScorePlan& sp, hipStream_t st) {
#define EA_CASE(DD, GG, WW)                          \
  if (D == DD && sp.GH == GG && sp.NW == WW)         \
  return a.n < 32 ? launch_one<DD, GG, WW, true, true>(a, sp, st) : launch_one<DD, GG, WW, false, true>(a, sp, st)
  EA_CASE(128, 1, kNW128);
  EA_CASE(128, 2, kNW128);
  EA_CASE(128, 3, kNW128);
#undef EA_CASE
  return launch_score_mfma_fp8b(D, a, sp, st);
}

}  // namespace ea
