/*
 * libea -- measurement and debugging aids.  NOT part of the serving path: unlike the entry
 * points of ea.h, the calls declared here create HIP events, synchronise the host with the
 * stream and copy to host memory.  bench.py and the tests use them; a serving loop does not.
 */
#ifndef EA_PROFILE_H
#define EA_PROFILE_H

#include "ea.h"

#ifdef __cplusplus
extern "C" {
#endif

/* The same work as ea_compress_layer (Listing 1 end to end, without the optional outputs), with a
 * HIP event recorded on `stream` between stages.  It creates and destroys the events, WAITS for
 * the layer to finish, and writes the milliseconds of each stage to stage_ms (HOST pointer,
 * EA_N_STAGES floats):
 *   0 clear + rotary table + statistics   1 matrix-core operand preparation
 *   2 score pass A (K/V streaming kernel)  3 score pass B (normalise, weight by ||v||)
 *   4 selection                            5 compaction */
#define EA_N_STAGES 6
ea_status ea_compress_layer_timed(const ea_params* p, const void* q_win, int64_t window,
                                  int64_t q_pos0, const double* inv_freq, int64_t t_next, void* k,
                                  void* v, int64_t n, int64_t n_cap, int64_t n_keep, void* ws,
                                  size_t ws_bytes, void* stream, float* stage_ms);

/* What the kernels noted in the workspace about inputs outside their documented domain.  WAITS
 * for `stream`, then copies the status bits out of `ws` (laid out for the same p, n, window as
 * the calls that used it) into *status (HOST pointer):
 *   EA_STATUS_BAD_SCORE     selection met a negative or NaN score (Sec. 2.2 scores are products
 *                           of non-negative factors; bit patterns then do not order like values)
 *   EA_STATUS_COMPACT_WAIT  an in-place compaction chunk gave up waiting for the chunks whose
 *                           source rows it would overwrite (idx not strictly ascending); its
 *                           stores were skipped, so those destination rows are stale
 *   EA_STATUS_BAD_INDEX     ea_compact met an idx list that is not strictly ascending with
 *                           j <= idx[j] < n (the rows were still moved, clamped into the tensor;
 *                           in place the result is then unspecified)
 * ea_compress_layer, ea_select and ea_compact clear the bits when they start: the word tells
 * about the last of them that used the workspace. */
#define EA_STATUS_BAD_SCORE 1u
#define EA_STATUS_COMPACT_WAIT 2u
#define EA_STATUS_BAD_INDEX 4u
ea_status ea_debug_status(const ea_params* p, int64_t n, int64_t window, const void* ws,
                          size_t ws_bytes, void* stream, uint32_t* status);

#ifdef __cplusplus
}
#endif
#endif /* EA_PROFILE_H */
