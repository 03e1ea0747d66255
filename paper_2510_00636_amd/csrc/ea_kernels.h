// Launch wrappers of the HIP kernels (one translation unit per stage).
#pragma once
#include <hip/hip_runtime.h>

#include "ea_common.h"

namespace ea {

// pool row of logical row `row` of unit (b, h); a table entry outside the pool is clamped into it,
// so a malformed table can never send an access outside the allocation
__device__ __forceinline__ size_t paged_row(const PageMap& m, int unit, int row) {
  const int b = unit / m.hkv, h = unit - b * m.hkv;
  long long blk = m.table[(size_t)b * m.max_blocks + (row >> m.sh)];
  blk = blk < 0 ? 0 : (blk >= m.num_blocks ? m.num_blocks - 1 : blk);
  return ((size_t)(blk * m.hkv + h) << m.sh) + (size_t)(row & ((1 << m.sh) - 1));
}

// ea_stats.hip
hipError_t launch_rope_table(const Dims& d, const double* inv_freq, int64_t q_pos0, int64_t t_next,
                             int w, float2* tab, uint32_t* clear, size_t clear_words, hipStream_t st);
hipError_t launch_stats(const Dims& d, const void* q_win, int w, const float2* tab, float* mu,
                        float* sigma, hipStream_t st);
hipError_t launch_prep_frags(const Dims& d, const ScorePlan& sp, const float* mu,
                             const float* sigma, uint4* frags, float* post, hipStream_t st);

// ea_score.hip
// tickets + unit * ticket_stride: 8 tile counters per pass of the unit (at most 64 passes), zero at launch
hipError_t launch_score_mfma(const Dims& d, const ScorePlan& sp, const void* k, const void* v,
                             int64_t n, int64_t n_cap, const uint4* frags, const float* post,
                             float* logits, float* vnorm, float2* part, uint32_t* tickets,
                             int ticket_stride, hipStream_t st, const PageMap* pm = nullptr,
                             const float* kscale = nullptr, const float* vscale = nullptr, bool skip_v = false);
// skip_v: V is neither read nor turned into norms (the caller weighs the pairs with norms of its own)
// kscale, vscale [units] (nullable): per-head scales of caches stored as e4m3 bytes (d.kv_fp8)
hipError_t launch_score_f32(const Dims& d, const void* k, const void* v, int64_t n, int64_t n_cap,
                            const float* mu, const float* sigma, double* logits, float* vnorm,
                            double2* part, int* nchunk_out, hipStream_t st);
// scores = (mean_g exp(l_g - lse_g) + eps) * vnorm; hist0 (nullable): first radix digit
// part: npart (max, sum exp) pairs per query head, each over a fixed block of keys; lse: scratch of
// one LT per query head (used when a head has too many partials to reduce inside pass B)
hipError_t launch_finalize(const Dims& d, int64_t n, const void* logits, int logits_f64,
                           const float* vnorm, const void* part, int npart, void* lse, float* scores,
                           uint32_t* hist0, hipStream_t st, const float* wnorm = nullptr, int lse_pass = 0);
// lse_pass: the partials do not exist yet; take them from the (fp32) logits, one per kLseBlock keys
// wnorm[i] = sqrt(max(2 d logits[i], 0)) for i < count
hipError_t launch_wnorm(const void* logits, int logits_f64, size_t count, int D, float* wnorm, hipStream_t st);

// ea_select.hip
// heads this short are selected by one workgroup per unit out of LDS, in one launch (no global
// histograms: hist0 from the finalize pass is not needed then)
constexpr int64_t kSelSmallMax = 16384;   // (32768-row heads: 12.4 us per layer in one launch, 9.8 in four)
inline bool select_in_one_launch(int64_t n) { return n <= kSelSmallMax; }
hipError_t launch_select(const Dims& d, const float* scores, int64_t n, int64_t n_keep, int32_t* idx,
                         uint32_t* hist, uint32_t* blk, bool hist0_done, hipStream_t st);
hipError_t launch_zero(uint32_t* p, size_t count, hipStream_t st, uint32_t* extra = nullptr);

// ea_compact.hip
hipError_t launch_compact(const Dims& d, const void* k, const void* v, int64_t n, int64_t n_cap,
                          const int32_t* idx, int64_t n_keep, void* k_out, void* v_out,
                          uint32_t* flags, uint32_t* status, hipStream_t st,
                          const int32_t* lengths = nullptr, int64_t idx_stride = 0, const PageMap* pm = nullptr);
// pm != nullptr: k and v are block pools (in place only; n_cap unused)
// lengths != nullptr: unit u keeps lengths[u] <= n_keep rows, listed from idx + u * idx_stride

// ea_select.hip, head-adaptive budgets: +inf into scores[unit][idx[unit][j]], j < n_mark; then the
// split of a pooled, ascending list flat[b][0 .. H*n_keep) over [H][n] into per-head lists
hipError_t launch_mark_inf(float* scores, const int32_t* idx, int units, int64_t n, int64_t n_mark, hipStream_t st);
hipError_t launch_split_pooled(const int32_t* flat, int B, int H, int64_t n, int64_t n_keep, int32_t* idx,
                               int32_t* lengths, hipStream_t st);

// order-free variant, in place: only the kept rows at or beyond n_keep move, into the evicted
// positions below it; perm (nullable) [units][n_keep] receives the source row of every position
hipError_t launch_compact_fill(const Dims& d, void* k, void* v, int64_t n, int64_t n_cap,
                               const int32_t* idx, int64_t n_keep, int32_t* perm, hipStream_t st,
                               const PageMap* pm = nullptr);

// ea_frontend.hip: q [B, Hq, w, d] fp32 = W_Q [Hq, d, dm] applied to hidden [B, w, dm] (dtype of d)
hipError_t launch_project(const Dims& d, const void* hidden, const void* wq, int w, int dm, float* q,
                          hipStream_t st);
// gram[g] = W_o^(g)^T W_o^(g) for w_o [Hq, dm, D] in the cache dtype
hipError_t launch_gram(const Dims& d, const void* w_o, int dm, float* gram, hipStream_t st);

// ea_baselines.hip: scorer = ea_scorer; scratch: units * kBaselineChunks * D floats
hipError_t launch_baseline(const Dims& d, int kind, const void* k, int64_t n, int64_t n_cap,
                           int64_t n_sink, float* scores, float* scratch, hipStream_t st);

int device_num_cu();

// hipFuncSetAttribute(MaxDynamicSharedMemorySize) once per (kernel, device) instead of on every
// launch: a static instance of this sits next to each launch of a kernel that needs more than
// 64 KiB of LDS.  Racing first calls at worst set the attribute twice.
struct LdsOptIn {
  size_t have[64] = {0};
  hipError_t ensure(const void* kern, size_t bytes) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = -1;
    if (dev >= 0 && have[dev] >= bytes) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess && dev >= 0) have[dev] = bytes;
    return e;
  }
};

}  // namespace ea
