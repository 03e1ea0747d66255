/*
 * libea -- Expected-Attention KV-cache compression for AMD MI355X (gfx950), C ABI.
 *
 * The library implements the compress step of "Expected Attention" (Sec. 2.2, Eq. 5-9 and
 * Listing 1 of the paper): per-head statistics of recent queries with the rotary matrix
 * averaged over the next T positions, the closed-form expected attention of every cached
 * key, the value-norm-weighted score of every KV pair, top-k selection per KV head and the
 * gather that compacts K and V.  Every step runs in hand-written HIP kernels.
 *
 * Conventions common to all entry points
 *   - All tensor pointers are DEVICE pointers (16-byte aligned) unless marked host.
 *     `p` (ea_params) is a HOST pointer and is read before the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work on that stream and return; they never synchronise the host, create
 *     streams, allocate, free or keep device memory.  Scratch comes through `ws`
 *     (at least ea_workspace_bytes() bytes, 256-byte aligned, owned by the caller, contents
 *     undefined between calls).  Calls sharing one `ws` must be ordered on one stream; calls
 *     on different streams need a workspace each and may then run concurrently (layers of a
 *     cache are independent).
 *   - Errors are return codes; nothing aborts or throws across the ABI.  Argument errors are
 *     detected on the host before any launch, so outputs are untouched on EA_ERR_INVALID_ARG,
 *     EA_ERR_UNSUPPORTED and EA_ERR_WORKSPACE.  A failed launch returns EA_ERR_DEVICE.
 *   - Layouts (row-major, innermost last):
 *       q_win  [B, Hq,  w,     d]   the w most recent queries, row s at position q_pos0+s
 *       k, v   [B, Hkv, n_cap, d]   only rows < n are read; head stride is n_cap*d
 *       mu     [B, Hq,  d]   fp32     sigma [B, Hq, d, d] fp32
 *       scores [B, Hkv, n]   fp32     idx   [B, Hkv, n_keep] int32, ascending positions
 *     Query head g belongs to KV head g / (Hq/Hkv).
 *   - Channel pairing of the rotary embedding: rope_layout 0 pairs (c, c+d/2), 1 pairs
 *     (2c, 2c+1); pair c turns by position * inv_freq[c].
 *   - Domain: finite inputs; bf16 keys are narrowed to fp16 for the matrix cores, so
 *     |k| <= 65504 (the squared keys of the diagonal correction saturate for |k| > 4096);
 *     1 <= n <= 2^26 rows per head.  Measurement and debugging calls (they block) are in
 *     ea_profile.h, not here.
 */
#ifndef EA_H
#define EA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  EA_OK = 0,
  EA_ERR_INVALID_ARG = 1,  /* null / misaligned pointer, size out of range                    */
  EA_ERR_UNSUPPORTED = 2,  /* head_dim, dtype, group size or window the kernels do not cover */
  EA_ERR_WORKSPACE = 3,    /* ws_bytes smaller than ea_workspace_bytes()                      */
  EA_ERR_DEVICE = 4        /* a kernel launch failed (hipGetLastError)                        */
} ea_status;

typedef enum {
  EA_F32 = 0,
  EA_BF16 = 1,
  EA_FP8_E4M3 = 2 /* rows of d bytes: accepted by ea_compact and ea_compact_unordered only (see ea_score_fp8) */
} ea_dtype;

typedef struct {
  int32_t batch;        /* B  >= 1                                                          */
  int32_t n_q_heads;    /* Hq, a multiple of n_kv_heads                                     */
  int32_t n_kv_heads;   /* Hkv >= 1                                                         */
  int32_t head_dim;     /* d in {64, 128, 256}                                              */
  int32_t dtype;        /* ea_dtype of q_win, k, v                                          */
  int32_t rope_layout;  /* 0 half-split pairs (c, c+d/2); 1 interleaved pairs (2c, 2c+1)    */
  int32_t q_is_rotated; /* 1: q_win holds post-rotary queries (un-rotated inside); 0: pre   */
  int32_t cov_ddof;     /* covariance divisor is w - cov_ddof; 0 or 1                       */
  int32_t horizon_T;    /* T of Eq. 6 (paper: 512), >= 1                                    */
  float epsilon;        /* eps of Eq. 9 (paper: 0.02, or 0), >= 0                           */
} ea_params;

/* Bytes of scratch any entry point needs for caches of up to n rows per head and a query
 * window of up to `window` rows.  Returns 0 if the parameters are invalid. */
size_t ea_workspace_bytes(const ea_params* p, int64_t n, int64_t window);

/* Eq. 5-6: statistics of the position-averaged query distribution.
 *   u_s = R(q_pos0+s)^T q_s (skipped when q_is_rotated = 0); m, S = mean / covariance of
 *   the u_s; R-bar = average of R(t_next .. t_next+T-1); mu = R-bar m; sigma = R-bar S R-bar^T.
 * inv_freq: DEVICE pointer, fp64 [d/2].  Needs 1 + cov_ddof <= window <= 4096.
 * bf16 windows: the covariance sums run on the fp16 matrix cores over samples scaled by a power
 * of two taken from the head's first 64 (32 at d = 256) samples; a later sample more than 2000
 * times larger than all of those in some channel overflows to non-finite statistics. */
ea_status ea_query_stats(const ea_params* p, const void* q_win, int64_t window, int64_t q_pos0,
                         const double* inv_freq, int64_t t_next, float* mu, float* sigma,
                         void* ws, size_t ws_bytes, void* stream);

/* Eq. 5-6 as printed, from the buffer of recent hidden states that the decoding set-up of
 * Sec. 3.1 keeps for the statistics: mu = R-bar W_Q mu_h, sigma = R-bar W_Q Sigma_h W_Q^T R-bar^T with
 * mu_h, Sigma_h the mean and covariance of the buffered hidden states.
 *   hidden [B, w, d_model], w_q [Hq, d, d_model] (row c of head g = the weights of query channel c),
 *   both in p->dtype.  rope_layout, cov_ddof, horizon_T as for ea_query_stats; q_is_rotated is not
 *   used (the projection of a hidden state carries no rotation yet). */
ea_status ea_query_stats_hidden(const ea_params* p, const void* hidden, const void* w_q, int64_t d_model,
                                int64_t window, const double* inv_freq, int64_t t_next, float* mu,
                                float* sigma, void* ws, size_t ws_bytes, void* stream);

/* Eq. 7-9 with ||v|| for ||W_o v|| (Sec. 3.1, implementation details) and the GQA group mean:
 *   l[g,i] = mu_g.k_i/sqrt(d) + k_i^T sigma_g k_i/(2d);  a[g,.] = softmax_i l[g,.];
 *   scores[h,i] = (mean_{g in group h} a[g,i] + epsilon) * ||v_i||_2.
 * sigma must be a covariance matrix (positive semi-definite up to rounding; it need not be
 * exactly symmetric): its diagonal is taken as the bound of its entries when it is scaled
 * into fp16 range for the matrix cores.  Reads k, v rows < n once.  n >= 1.
 * Accuracy of the bf16 path: sigma reaches the matrix cores in fp16 (its diagonal compensated),
 * the keys exactly, sums in fp32; the logit then carries an absolute error of the order of
 * 2^-12 times sum_{i != j} |sigma_ij k_i k_j| / 2d, i.e. scores agree with an fp64 evaluation to
 * about 6e-4 relative on Llama- / Gemma- / Qwen-shaped inputs and to 2e-3 as long as the quadratic
 * term stays in the tens; near-rank-one covariances from windows of a few samples can exceed it. */
ea_status ea_score(const ea_params* p, const void* k, const void* v, int64_t n, int64_t n_cap,
                   const float* mu, const float* sigma, float* scores,
                   void* ws, size_t ws_bytes, void* stream);

/* Eq. 9 as printed, with the output projection: ||W_o v|| in place of ||v||.  Query head g sends the
 * value head of its group through its own d columns of W_o, so
 *   scores[h,i] = (1/G) sum_{g in group h} (a[g,i] + epsilon) * ||W_o^(g) v_i||_2 .
 * The norm is sqrt(v^T M_g v) with M_g = W_o^(g)^T W_o^(g), a quadratic form like Eq. 7's:
 *   ea_wo_gram         gram [Hq, d, d] fp32 (out) from w_o [Hq, d_model, d] in p->dtype (row m of head
 *                      g = the weights that take head g's d channels to output channel m).  Depends on
 *                      the weights only: once per layer.  p->batch is not used.
 *   ea_value_norms_wo  wnorm [B, Hq, n] fp32 (out) = ||W_o^(g) v_i|| for the value rows < n of the
 *                      head's group; reads v once per pass of the score kernel.  Values do not
 *                      change while they are cached, so a caller may keep wnorm across compress
 *                      passes and compact it with the cache.
 *   ea_score_wo        ea_score with wnorm [B, Hq, n] in place of ||v||.
 * Errors as for ea_score; 1 <= d_model <= 2^20. */
ea_status ea_wo_gram(const ea_params* p, const void* w_o, int64_t d_model, float* gram, void* stream);
ea_status ea_value_norms_wo(const ea_params* p, const void* v, int64_t n, int64_t n_cap, const float* gram,
                            float* wnorm, void* ws, size_t ws_bytes, void* stream);
ea_status ea_score_wo(const ea_params* p, const void* k, const void* v, int64_t n, int64_t n_cap,
                      const float* mu, const float* sigma, const float* wnorm, float* scores,
                      void* ws, size_t ws_bytes, void* stream);

/* Sec. 2.2 "Compression", Listing 1 top-k: per KV head the n_keep pairs of highest score,
 * equal scores going to the lower position; idx is written in ascending position order.
 * Scores must be non-negative and not NaN (compared by bit pattern).  0 <= n_keep <= n. */
ea_status ea_select(const ea_params* p, const float* scores, int64_t n, int64_t n_keep,
                    int32_t* idx, void* ws, size_t ws_bytes, void* stream);

/* For callers that cannot allocate or pass a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): ea_select with its scratch (radix
 * histograms, per-block counts; about 1.6 MiB) in a static device array inside the library
 * instead of `ws`.  Same inputs, outputs and result as ea_select.  It allocates nothing and
 * calls no allocating routine.  Limits: batch * n_kv_heads <= EA_SELECT_STATIC_MAX_UNITS and
 * n <= EA_SELECT_STATIC_MAX_N, else EA_ERR_UNSUPPORTED (nothing launched).  Every call on a GPU
 * shares that GPU's array: calls that overlap in time on one GPU (different streams) race;
 * calls ordered on one stream, or otherwise serialised, are fine. */
#define EA_SELECT_STATIC_MAX_UNITS 64
#define EA_SELECT_STATIC_MAX_N (1 << 20)
ea_status ea_select_static(const ea_params* p, const float* scores, int64_t n, int64_t n_keep,
                           int32_t* idx, void* stream);

/* Listing 1 gather: row idx[j] of every head of k and v moves to row j of k_out / v_out
 * (same [B, Hkv, n_cap, d] layout).  k_out == k and v_out == v compacts in place; otherwise
 * the outputs must not overlap the inputs.  idx must be strictly ascending with values < n.
 * Rows >= n_keep of the outputs are left as they were. */
ea_status ea_compact(const ea_params* p, const void* k, const void* v, int64_t n, int64_t n_cap,
                     const int32_t* idx, int64_t n_keep, void* k_out, void* v_out,
                     void* ws, size_t ws_bytes, void* stream);

/* Listing 1 end to end on one layer: statistics -> scores -> selection -> in-place compaction
 * of k and v, all enqueued on `stream` with no host synchronisation in between.
 * scores_out ([B,Hkv,n]) and idx_out ([B,Hkv,n_keep]) may be NULL. */
ea_status ea_compress_layer(const ea_params* p, const void* q_win, int64_t window, int64_t q_pos0,
                            const double* inv_freq, int64_t t_next, void* k, void* v, int64_t n,
                            int64_t n_cap, int64_t n_keep, float* scores_out, int32_t* idx_out,
                            void* ws, size_t ws_bytes, void* stream);

/* Sec. 2.2, "Head-Adaptive Compression": one budget of Hkv * n_keep pairs per (sequence, layer),
 * shared by the layer's KV heads, "allowing more important heads to retain more KV pairs".  The
 * paper only cites the idea; the rule here: every head first keeps its own `floor` best pairs
 * (0 <= floor <= n_keep), the rest of the budget goes to the best remaining pairs of the whole
 * layer; equal scores go to the lower head, then to the lower position.
 *   idx      [B, Hkv, n] int32 (a head's list starts at multiples of n): the first lengths[b,h]
 *            entries of each list are that head's kept positions, ascending; the rest is untouched
 *   lengths  [B, Hkv] int32 DEVICE; their sum over a sequence's heads is Hkv * n_keep
 * Scores as for ea_select.  Needs Hkv * n <= 2^26. */
ea_status ea_select_adaptive(const ea_params* p, const float* scores, int64_t n, int64_t n_keep,
                             int64_t floor, int32_t* idx, int32_t* lengths, void* ws, size_t ws_bytes,
                             void* stream);

/* ea_compress_layer with the head-adaptive budget (the set-up of the paper's reported results,
 * Sec. 2.2 "Head-Adaptive Compression" and Sec. 3.1): statistics -> scores -> ea_select_adaptive ->
 * ragged in-place compaction, on `stream`, no host synchronisation.  idx_out [B, Hkv, n] and
 * lengths_out [B, Hkv] (both required, DEVICE) are those of ea_select_adaptive; afterwards head
 * (b, h) holds lengths_out[b, h] rows.  scores_out ([B, Hkv, n]) may be NULL. */
ea_status ea_compress_layer_adaptive(const ea_params* p, const void* q_win, int64_t window, int64_t q_pos0,
                                     const double* inv_freq, int64_t t_next, void* k, void* v, int64_t n,
                                     int64_t n_cap, int64_t n_keep, int64_t floor, float* scores_out,
                                     int32_t* idx_out, int32_t* lengths_out, void* ws, size_t ws_bytes,
                                     void* stream);

/* Listing 1's gather with a kept count per head, in place: row idx[b,h,j] of head (b,h) moves to
 * row j for j < lengths[b,h] (idx, lengths as written by ea_select_adaptive).  Rows from
 * lengths[b,h] on are left as they were. */
ea_status ea_compact_ragged(const ea_params* p, void* k, void* v, int64_t n, int64_t n_cap,
                            const int32_t* idx, const int32_t* lengths, void* ws, size_t ws_bytes,
                            void* stream);

/* The cheap scorers of the paper's decoding comparison (Sec. 3.1, "Baselines"), each from the one
 * sentence the paper gives it, producing scores[B, Hkv, n] for the same ea_select / ea_compact
 * back half (larger score = kept first):
 *   EA_SCORER_KNORM      "preserving keys with the lowest L2 norm":  1 / ||k_i||_2
 *   EA_SCORER_STREAMING  "maintains initial sink tokens": +inf for the first n_sink pairs, i + 1
 *                        for the others (the rest of the budget goes to the most recent pairs);
 *                        n <= 2^24 (positions must be exact in fp32), else EA_ERR_UNSUPPORTED
 *   EA_SCORER_KEYDIFF    "distance metrics between key embeddings":  1 - cos(k_i, a), a = mean of
 *                        the head's unit-normalised keys (a key of zero norm counts as zero)
 * Reads k rows < n (twice for KEYDIFF), never v.  n_sink is only used by STREAMING (0 <= n_sink). */
typedef enum { EA_SCORER_KNORM = 0, EA_SCORER_STREAMING = 1, EA_SCORER_KEYDIFF = 2 } ea_scorer;
ea_status ea_score_baseline(const ea_params* p, int32_t scorer, const void* k, int64_t n, int64_t n_cap,
                            int64_t n_sink, float* scores, void* ws, size_t ws_bytes, void* stream);

/* Order-free compaction, in place.  Attention over the cache is a sum over cached pairs (Eq. 2-3)
 * and every key carries its rotary position (Eq. 1), so the kept pairs need not keep their order:
 * kept rows below n_keep stay where they are, the kept rows at or beyond n_keep fill, in ascending
 * order, the evicted positions below n_keep, in ascending order.  Rows >= n_keep are left as they
 * were.  idx as for ea_compact.  perm_out (nullable, [B, Hkv, n_keep] int32) receives, for every
 * position of the compacted cache, the row it held before.  Needs no scratch. */
ea_status ea_compact_unordered(const ea_params* p, void* k, void* v, int64_t n, int64_t n_cap,
                               const int32_t* idx, int64_t n_keep, int32_t* perm_out, void* stream);

/* ea_compress_layer with the order-free compaction as its last step (the decode-time use: few
 * pairs are evicted per pass, so few rows move).  idx_out is still the ascending kept list. */
ea_status ea_compress_layer_unordered(const ea_params* p, const void* q_win, int64_t window,
                                      int64_t q_pos0, const double* inv_freq, int64_t t_next, void* k,
                                      void* v, int64_t n, int64_t n_cap, int64_t n_keep,
                                      float* scores_out, int32_t* idx_out, int32_t* perm_out, void* ws,
                                      size_t ws_bytes, void* stream);

/* Paged caches (the block-table layout of paged-attention servers), for the cache of Listing 1
 * when it does not live in one tensor per head: K and V are pools
 *   k_pool, v_pool  [num_blocks, Hkv, block_size, d]   bf16
 * and logical block j of sequence b (its rows j*block_size .. (j+1)*block_size - 1, for all of the
 * sequence's KV heads) is pool block block_table[b, j].  The three calls below are ea_score,
 * ea_compact (in place) and ea_compress_layer over such a cache: same arithmetic, same results for
 * the same logical rows.  After a compaction the logical rows [0, n_keep) of every head are valid;
 * the blocks from ceil(n_keep / block_size) on hold nothing the cache needs and may be returned to
 * the pool by the caller (the library never writes the table).  Table entries outside
 * [0, num_blocks) are clamped into the pool (wrong results, no access outside it).
 * order_free != 0 selects the order-free compaction (see ea_compact_unordered); perm_out is only
 * written then (nullable).  EA_ERR_UNSUPPORTED for fp32 caches and for block sizes that are not a
 * power of two in [16, 65536]. */
typedef struct {
  const int32_t* block_table; /* DEVICE [B, max_blocks] int32                                */
  int32_t block_size;         /* rows per block                                              */
  int32_t max_blocks;         /* entries per sequence in block_table; max_blocks * block_size >= n */
  int64_t num_blocks;         /* blocks in each pool                                         */
} ea_paged;
ea_status ea_score_paged(const ea_params* p, const void* k_pool, const void* v_pool, const ea_paged* pg,
                         int64_t n, const float* mu, const float* sigma, float* scores, void* ws,
                         size_t ws_bytes, void* stream);
ea_status ea_compact_paged(const ea_params* p, void* k_pool, void* v_pool, const ea_paged* pg, int64_t n,
                           const int32_t* idx, int64_t n_keep, int32_t order_free, int32_t* perm_out,
                           void* ws, size_t ws_bytes, void* stream);
ea_status ea_compress_layer_paged(const ea_params* p, const void* q_win, int64_t window, int64_t q_pos0,
                                  const double* inv_freq, int64_t t_next, void* k_pool, void* v_pool,
                                  const ea_paged* pg, int64_t n, int64_t n_keep, int32_t order_free,
                                  float* scores_out, int32_t* idx_out, int32_t* perm_out, void* ws,
                                  size_t ws_bytes, void* stream);

/* Caches stored in 8 bits (Related Works, "Quantization": orthogonal to eviction, the two combine).
 * k8, v8 [B, Hkv, n_cap, d] hold OCP e4m3 ("float8_e4m3fn") bytes and the real key / value is
 * k_scale[b,h] * k8[b,h] / v_scale[b,h] * v8[b,h]  (k_scale, v_scale: fp32 DEVICE [B, Hkv], NULL = 1).
 * ea_score_fp8 and ea_compress_layer_fp8 are ea_score and ea_compress_layer over such a cache
 * (order_free / perm_out as for ea_compress_layer_paged): the bytes widen exactly to the fp16
 * operands of the matrix cores, so the arithmetic is that of the bf16 path on the dequantised
 * values.  p->dtype is the type of q_win and must be EA_BF16; head_dim 128 or 256 (else
 * EA_ERR_UNSUPPORTED).  The compaction calls move rows without looking into them: for ea_compact
 * and ea_compact_unordered on such a cache set p->dtype = EA_FP8_E4M3 (rows of d bytes); the scales
 * belong to the head and do not move. */
ea_status ea_score_fp8(const ea_params* p, const void* k8, const void* v8, const float* k_scale,
                       const float* v_scale, int64_t n, int64_t n_cap, const float* mu, const float* sigma,
                       float* scores, void* ws, size_t ws_bytes, void* stream);
ea_status ea_compress_layer_fp8(const ea_params* p, const void* q_win, int64_t window, int64_t q_pos0,
                                const double* inv_freq, int64_t t_next, void* k8, void* v8,
                                const float* k_scale, const float* v_scale, int64_t n, int64_t n_cap,
                                int64_t n_keep, int32_t order_free, float* scores_out, int32_t* idx_out,
                                int32_t* perm_out, void* ws, size_t ws_bytes, void* stream);

/* Listing 1: int(n * (1 - ratio)) in IEEE double, truncated toward zero; -1 if ratio is
 * outside [0, 1] or n < 0.  Host only. */
int64_t ea_n_keep(int64_t n, double ratio);

/* Static string for a status code.  Host only. */
const char* ea_status_string(ea_status s);

#ifdef __cplusplus
}
#endif
#endif /* EA_H */
