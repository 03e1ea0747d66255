// extern "C" entry points of libea: host-side validation, then the launch sequence on the
// caller's stream.  No allocation, no synchronisation, no state besides a cached CU count and
// the per-device address of the static scratch array of ea_select_static.
#include <hip/hip_runtime.h>

#include <mutex>

#include "../../include/ea_profile.h"
#include "ea_kernels.h"

namespace ea {

int device_num_cu() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
      n = 256;
    cached[dev] = n;
  }
  return cached[dev];
}

static inline bool aligned16(const void* p) { return p && ((uintptr_t)p & 15u) == 0; }
static inline bool aligned256(const void* p) { return p && ((uintptr_t)p & 255u) == 0; }
#define EA_TRY(expr)                                   \
  do {                                                 \
    if ((expr) != hipSuccess) return EA_ERR_DEVICE;    \
  } while (0)

static ea_status check_ws(const Dims& d, int64_t n, int64_t window, void* ws, size_t ws_bytes,
                          WsLayout* L) {
  if (!aligned256(ws)) return EA_ERR_INVALID_ARG;
  *L = make_ws_layout(d, n, window);
  if (ws_bytes < L->total) return EA_ERR_WORKSPACE;
  return EA_OK;
}

// clear / clear_words: scratch words zeroed by the table kernel on its way (may be none)
static ea_status run_stats(const Dims& d, const void* q_win, int64_t window, int64_t q_pos0,
                           const double* inv_freq, int64_t t_next, float* mu, float* sigma,
                           char* ws, const WsLayout& L, hipStream_t st, uint32_t* clear = nullptr,
                           size_t clear_words = 0) {
  float2* tab = (float2*)(ws + L.tab);
  EA_TRY(launch_rope_table(d, inv_freq, q_pos0, t_next, (int)window, tab, clear, clear_words, st));
  EA_TRY(launch_stats(d, q_win, (int)window, tab, mu, sigma, st));
  return EA_OK;
}

// hist0 != nullptr: the finalize pass also fills the first radix-select histogram.
// ev (nullable): ev[0] is recorded after the operand preparation, ev[1] after pass A.
// The score kernel's tile counters live in words of the third histogram that the 1024-bin
// last radix digit never touches; `hist_zeroed` says whether the caller's clearing launch has
// covered them already.
static ea_status run_score(const Dims& d, const void* k, const void* v, int64_t n, int64_t n_cap,
                           const float* mu, const float* sigma, float* scores, uint32_t* hist0,
                           bool hist_zeroed, char* ws, const WsLayout& L, hipStream_t st,
                           hipEvent_t* ev = nullptr, const float* wnorm = nullptr, float* wnorm_out = nullptr,
                           const PageMap* pm = nullptr, const float* kscale = nullptr, const float* vscale = nullptr) {
  // wnorm: Eq. 9 with per-query-head norms ||W_o v||.  wnorm_out: stop after pass A and turn its
  // quadratic forms into such norms (the caller passed the values as keys, mu = 0, Sigma = M_g).
  float* vnorm = (float*)(ws + L.vnorm);
  uint32_t* hist = (uint32_t*)(ws + L.hist);
  if (d.dtype == EA_BF16 && !hist_zeroed) EA_TRY(launch_zero(hist, (size_t)d.units() * 3 * kSelBins, st));
  if (d.dtype == EA_BF16) {
    ScorePlan sp = make_score_plan(d, n, device_num_cu(), pm != nullptr);
    uint4* frags = (uint4*)(ws + L.frags);
    float* post = (float*)(ws + L.post);
    EA_TRY(launch_prep_frags(d, sp, mu, sigma, frags, post, st));
    if (ev) EA_TRY(hipEventRecord(ev[0], st));
    EA_TRY(launch_score_mfma(d, sp, k, v, n, n_cap, frags, post, (float*)(ws + L.logits), vnorm,
                             (float2*)(ws + L.part), hist + 2 * kSelBins + kTicketSlot, 3 * kSelBins,
                             st, pm, kscale, vscale, wnorm != nullptr || wnorm_out != nullptr));
    if (ev) EA_TRY(hipEventRecord(ev[1], st));
    if (wnorm_out) return launch_wnorm(ws + L.logits, 0, (size_t)d.qheads() * n, d.D, wnorm_out, st) == hipSuccess
                              ? EA_OK : EA_ERR_DEVICE;
    EA_TRY(launch_finalize(d, n, ws + L.logits, 0, vnorm, ws + L.part, sp.npart, ws + L.lse, scores,
                           hist0, st, wnorm, sp.lse_pass));
  } else {
    int nchunk = 0;
    if (ev) EA_TRY(hipEventRecord(ev[0], st));
    EA_TRY(launch_score_f32(d, k, v, n, n_cap, mu, sigma, (double*)(ws + L.logits), vnorm,
                            (double2*)(ws + L.part), &nchunk, st));
    if (ev) EA_TRY(hipEventRecord(ev[1], st));
    if (wnorm_out) return launch_wnorm(ws + L.logits, 1, (size_t)d.qheads() * n, d.D, wnorm_out, st) == hipSuccess
                              ? EA_OK : EA_ERR_DEVICE;
    EA_TRY(launch_finalize(d, n, ws + L.logits, 1, vnorm, ws + L.part, nchunk, ws + L.lse, scores,
                           hist0, st, wnorm));
  }
  return EA_OK;
}

static size_t hist_words(const Dims& d) { return (size_t)d.units() * 3 * kSelBins; }
static size_t flag_words(const Dims& d, int64_t n_keep) {
  return 2 * (size_t)d.units() * ((n_keep + kCompactRows - 1) / kCompactRows + kCompactTicketStride);
}
// [a, a + bytes) and [b, b + bytes) share bytes without being the same range
static bool partly_overlap(const void* a, const void* b, size_t bytes) {
  const uintptr_t x = (uintptr_t)a, y = (uintptr_t)b;
  return x != y && x < y + bytes && y < x + bytes;
}

// ---- scratch of ea_select_static: the radix histograms and per-block counts of the selection,
// for callers that cannot hand over (or allocate) a workspace.  Every GPU the library runs on
// holds its own copy of the array, at its own address, until the process ends.  In host code
// the array's name is only a handle for hipGetSymbolAddress: the address that kernels, and the
// clearing launch, get is the one that call returns for the current device.
constexpr int kStaticMaxUnits = EA_SELECT_STATIC_MAX_UNITS;
constexpr int64_t kStaticMaxN = EA_SELECT_STATIC_MAX_N;
constexpr size_t kStaticHistWords = (size_t)kStaticMaxUnits * 3 * kSelBins;
constexpr size_t kStaticBlkWords = (size_t)kStaticMaxUnits * (kStaticMaxN / kSelBlock) * 2;
static __device__ __align__(256) uint32_t scratch[kStaticHistWords + kStaticBlkWords];

static uint32_t* static_scratch_for_current_device() {
  static std::mutex mu;
  static uint32_t* ptr[64] = {nullptr};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    ptr[dev] = (uint32_t*)p;
  }
  return ptr[dev];
}

}  // namespace ea

using namespace ea;

extern "C" {

ea_status ea_query_stats(const ea_params* p, const void* q_win, int64_t window, int64_t q_pos0,
                         const double* inv_freq, int64_t t_next, float* mu, float* sigma, void* ws,
                         size_t ws_bytes, void* stream) {
  Dims d;
  ea_status s = check_params(p, &d);
  if (s != EA_OK) return s;
  if (!aligned16(q_win) || !aligned16(mu) || !aligned16(sigma) || !inv_freq ||
      ((uintptr_t)inv_freq & 7u))
    return EA_ERR_INVALID_ARG;
  if (window < 1 + d.ddof || q_pos0 < 0 || t_next < 0) return EA_ERR_INVALID_ARG;
  if (window > kMaxWindow) return EA_ERR_UNSUPPORTED;
  WsLayout L;
  if ((s = check_ws(d, 1, window, ws, ws_bytes, &L)) != EA_OK) return s;
  return run_stats(d, q_win, window, q_pos0, inv_freq, t_next, mu, sigma, (char*)ws, L,
                   (hipStream_t)stream);
}

ea_status ea_query_stats_hidden(const ea_params* p, const void* hidden, const void* w_q, int64_t d_model,
                                int64_t window, const double* inv_freq, int64_t t_next, float* mu,
                                float* sigma, void* ws, size_t ws_bytes, void* stream) {
  Dims d;
  ea_status s = check_params(p, &d);
  if (s != EA_OK) return s;
  if (!aligned16(hidden) || !aligned16(w_q) || !aligned16(mu) || !aligned16(sigma) || !inv_freq ||
      ((uintptr_t)inv_freq & 7u))
    return EA_ERR_INVALID_ARG;
  if (window < 1 + d.ddof || t_next < 0 || d_model < 1 || d_model > (1 << 20)) return EA_ERR_INVALID_ARG;
  if (window > kMaxWindow) return EA_ERR_UNSUPPORTED;
  WsLayout L;
  if ((s = check_ws(d, 1, window, ws, ws_bytes, &L)) != EA_OK) return s;
  hipStream_t st = (hipStream_t)stream;
  float* q = (float*)((char*)ws + L.qproj);
  EA_TRY(launch_project(d, hidden, w_q, (int)window, (int)d_model, q, st));
  Dims dq = d;                       // the projected queries: fp32, not yet rotated
  dq.dtype = EA_F32;
  dq.q_is_rotated = 0;
  return run_stats(dq, q, window, 0, inv_freq, t_next, mu, sigma, (char*)ws, L, st);
}

ea_status ea_score(const ea_params* p, const void* k, const void* v, int64_t n, int64_t n_cap,
                   const float* mu, const float* sigma, float* scores, void* ws, size_t ws_bytes,
                   void* stream) {
  Dims d;
  ea_status s = check_params(p, &d);
  if (s != EA_OK) return s;
  if (!aligned16(k) || !aligned16(v) || !aligned16(mu) || !aligned16(sigma) || !aligned16(scores))
    return EA_ERR_INVALID_ARG;
  if (n < 1 || n > n_cap || n > kMaxN) return EA_ERR_INVALID_ARG;
  WsLayout L;
  if ((s = check_ws(d, n, 1, ws, ws_bytes, &L)) != EA_OK) return s;
  return run_score(d, k, v, n, n_cap, mu, sigma, scores, nullptr, false, (char*)ws, L,
                   (hipStream_t)stream);
}

ea_status ea_wo_gram(const ea_params* p, const void* w_o, int64_t d_model, float* gram, void* stream) {
  Dims d;
  ea_status s = check_params(p, &d);
  if (s != EA_OK) return s;
  if (!aligned16(w_o) || !aligned16(gram) || d_model < 1 || d_model > (1 << 20)) return EA_ERR_INVALID_ARG;
  EA_TRY(launch_gram(d, w_o, (int)d_model, gram, (hipStream_t)stream));
  return EA_OK;
}

ea_status ea_value_norms_wo(const ea_params* p, const void* v, int64_t n, int64_t n_cap, const float* gram,
                            float* wnorm, void* ws, size_t ws_bytes, void* stream) {
  Dims d;
  ea_status s = check_params(p, &d);
  if (s != EA_OK) return s;
  if (!aligned16(v) || !aligned16(gram) || !aligned16(wnorm)) return EA_ERR_INVALID_ARG;
  if (n < 1 || n > n_cap || n > kMaxN) return EA_ERR_INVALID_ARG;
  WsLayout L;
  if ((s = check_ws(d, n, 1, ws, ws_bytes, &L)) != EA_OK) return s;
  hipStream_t st = (hipStream_t)stream;
  // pass A over the value rows with mu = 0 and Sigma = M_g (the same M for every sequence)
  float* mu0 = (float*)((char*)ws + L.mu);
  float* sg = (float*)((char*)ws + L.sigma);
  EA_TRY(launch_zero((uint32_t*)mu0, (size_t)d.qheads() * d.D, st));
  const size_t per_b = (size_t)d.Hq * d.D * d.D * sizeof(float);
  for (int b = 0; b < d.B; ++b)
    EA_TRY(hipMemcpyAsync((char*)sg + b * per_b, gram, per_b, hipMemcpyDeviceToDevice, st));
  return run_score(d, v, v, n, n_cap, mu0, sg, nullptr, nullptr, false, (char*)ws, L, st, nullptr, nullptr,
                   wnorm);
}

ea_status ea_score_wo(const ea_params* p, const void* k, const void* v, int64_t n, int64_t n_cap,
                      const float* mu, const float* sigma, const float* wnorm, float* scores, void* ws,
                      size_t ws_bytes, void* stream) {
  Dims d;
  ea_status s = check_params(p, &d);
  if (s != EA_OK) return s;
  if (!aligned16(k) || !aligned16(v) || !aligned16(mu) || !aligned16(sigma) || !aligned16(scores) ||
      !aligned16(wnorm))
    return EA_ERR_INVALID_ARG;
  if (n < 1 || n > n_cap || n > kMaxN) return EA_ERR_INVALID_ARG;
  WsLayout L;
  if ((s = check_ws(d, n, 1, ws, ws_bytes, &L)) != EA_OK) return s;
  return run_score(d, k, v, n, n_cap, mu, sigma, scores, nullptr, false, (char*)ws, L,
                   (hipStream_t)stream, nullptr, wnorm);
}

ea_status ea_select(const ea_params* p, const float* scores, int64_t n, int64_t n_keep, int32_t* idx,
                    void* ws, size_t ws_bytes, void* stream) {
  Dims d;
  ea_status s = check_params(p, &d);
  if (s != EA_OK) return s;
  if (n < 1 || n > kMaxN || n_keep < 0 || n_keep > n) return EA_ERR_INVALID_ARG;
  if (!aligned16(scores) || (n_keep > 0 && !aligned16(idx))) return EA_ERR_INVALID_ARG;
  WsLayout L;
  if ((s = check_ws(d, n, 1, ws, ws_bytes, &L)) != EA_OK) return s;
  if (n_keep == 0) return EA_OK;
  hipStream_t st = (hipStream_t)stream;
  uint32_t* hist = (uint32_t*)((char*)ws + L.hist);
  EA_TRY(launch_zero(hist, hist_words(d), st));
  EA_TRY(launch_select(d, scores, n, n_keep, idx, hist, (uint32_t*)((char*)ws + L.blk), false, st));
  return EA_OK;
}

ea_status ea_select_static(const ea_params* p, const float* scores, int64_t n, int64_t n_keep,
                           int32_t* idx, void* stream) {
  Dims d;
  ea_status s = check_params(p, &d);
  if (s != EA_OK) return s;
  if (n < 1 || n_keep < 0 || n_keep > n) return EA_ERR_INVALID_ARG;
  if (!aligned16(scores) || (n_keep > 0 && !aligned16(idx))) return EA_ERR_INVALID_ARG;
  if (n > kStaticMaxN || d.units() > kStaticMaxUnits) return EA_ERR_UNSUPPORTED;
  if (n_keep == 0) return EA_OK;
  uint32_t* hist = static_scratch_for_current_device();
  if (!hist) return EA_ERR_DEVICE;
  hipStream_t st = (hipStream_t)stream;
  // the array keeps the previous call's contents: the histograms must start at zero (a fill
  // kernel, so that the call can be captured in a graph); the block counts are overwritten
  EA_TRY(launch_zero(hist, hist_words(d), st));
  EA_TRY(launch_select(d, scores, n, n_keep, idx, hist, hist + kStaticHistWords, false, st));
  return EA_OK;
}

ea_status ea_compact(const ea_params* p, const void* k, const void* v, int64_t n, int64_t n_cap,
                     const int32_t* idx, int64_t n_keep, void* k_out, void* v_out, void* ws,
                     size_t ws_bytes, void* stream) {
  Dims d;
  ea_status s = check_params(p, &d, true);
  if (s != EA_OK) return s;
  if (!aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out))
    return EA_ERR_INVALID_ARG;
  if (n < 1 || n > n_cap || n > kMaxN || n_keep < 0 || n_keep > n)
    return EA_ERR_INVALID_ARG;
  if ((k_out == k) != (v_out == v)) return EA_ERR_INVALID_ARG;   // both in place or neither
  if (k_out == v || v_out == k || (k_out == v_out)) return EA_ERR_INVALID_ARG;
  {
    // the four tensors are either the same range (in place) or disjoint ranges
    const size_t bytes = (size_t)d.units() * (size_t)n_cap * d.D * d.esize();
    const void* t[4] = {k, v, k_out, v_out};
    for (int i = 0; i < 4; ++i)
      for (int j = i + 1; j < 4; ++j)
        if (partly_overlap(t[i], t[j], bytes)) return EA_ERR_INVALID_ARG;
  }
  if (n_keep > 0 && !aligned16(idx)) return EA_ERR_INVALID_ARG;
  WsLayout L;
  if ((s = check_ws(d, n, 1, ws, ws_bytes, &L)) != EA_OK) return s;
  if (n_keep == 0) return EA_OK;
  hipStream_t st = (hipStream_t)stream;
  uint32_t* flags = (uint32_t*)((char*)ws + L.flags);
  uint32_t* status = (uint32_t*)((char*)ws + L.hist) + 2 * kSelBins + kStatusSlot;
  EA_TRY(launch_zero(flags, k_out == k ? flag_words(d, n_keep) : 0, st, status));
  EA_TRY(launch_compact(d, k, v, n, n_cap, idx, n_keep, k_out, v_out, flags, status, st));
  return EA_OK;
}

// ea_paged -> PageMap, validated on the host (the table's entries are device memory: the kernels
// clamp them into the pool)
static ea_status check_paged(const Dims& d, const ea_paged* pg, int64_t n, PageMap* pm) {
  if (!pg || !pg->block_table || ((uintptr_t)pg->block_table & 3u)) return EA_ERR_INVALID_ARG;
  const int64_t bs = pg->block_size;
  if (bs < 16 || bs > 65536 || (bs & (bs - 1)) != 0) return EA_ERR_UNSUPPORTED;
  if (pg->max_blocks < 1 || pg->num_blocks < 1 || pg->num_blocks > ((int64_t)1 << 31)) return EA_ERR_INVALID_ARG;
  if ((int64_t)pg->max_blocks * bs < n) return EA_ERR_INVALID_ARG;
  if (d.dtype != EA_BF16) return EA_ERR_UNSUPPORTED;
  pm->table = pg->block_table;
  pm->sh = 0;
  while (((int64_t)1 << pm->sh) < bs) ++pm->sh;
  pm->max_blocks = pg->max_blocks;
  pm->hkv = d.Hkv;
  pm->num_blocks = pg->num_blocks;
  return EA_OK;
}

// unordered: the order-free compaction (perm_out then receives the source row of every position)
// pm: the caches are block pools (n_cap is then not used)
static ea_status compress_impl(const ea_params* p, const void* q_win, int64_t window,
                               int64_t q_pos0, const double* inv_freq, int64_t t_next, void* k,
                               void* v, int64_t n, int64_t n_cap, int64_t n_keep, float* scores_out,
                               int32_t* idx_out, void* ws, size_t ws_bytes, void* stream,
                               hipEvent_t* ev, bool unordered = false, int32_t* perm_out = nullptr,
                               const PageMap* pm = nullptr, bool fp8 = false, const float* kscale = nullptr,
                               const float* vscale = nullptr) {
  Dims d;
  ea_status s = check_params(p, &d);
  if (s != EA_OK) return s;
  if (fp8) {
    if (d.dtype != EA_BF16 || d.D == 64) return EA_ERR_UNSUPPORTED;
    if ((kscale && ((uintptr_t)kscale & 3u)) || (vscale && ((uintptr_t)vscale & 3u))) return EA_ERR_INVALID_ARG;
    d.kv_fp8 = 1;
  }
  if (!aligned16(q_win) || !aligned16(k) || !aligned16(v) || k == v || !inv_freq ||
      ((uintptr_t)inv_freq & 7u))
    return EA_ERR_INVALID_ARG;
  if ((scores_out && !aligned16(scores_out)) || (idx_out && !aligned16(idx_out)) ||
      (perm_out && !aligned16(perm_out)))
    return EA_ERR_INVALID_ARG;
  if (window < 1 + d.ddof || q_pos0 < 0 || t_next < 0) return EA_ERR_INVALID_ARG;
  if (window > kMaxWindow) return EA_ERR_UNSUPPORTED;
  if (n < 1 || n > n_cap || n > kMaxN || n_keep < 0 || n_keep > n)
    return EA_ERR_INVALID_ARG;
  WsLayout L;
  if ((s = check_ws(d, n, window, ws, ws_bytes, &L)) != EA_OK) return s;
  hipStream_t st = (hipStream_t)stream;
  char* w = (char*)ws;
  float* mu = (float*)(w + L.mu);
  float* sigma = (float*)(w + L.sigma);
  float* scores = scores_out ? scores_out : (float*)(w + L.scores);
  int32_t* idx = idx_out ? idx_out : (int32_t*)(w + L.idx);
  uint32_t* hist = (uint32_t*)(w + L.hist);
  uint32_t* flags = (uint32_t*)(w + L.flags);
  if (ev) EA_TRY(hipEventRecord(ev[0], st));
  // hist .. flags are adjacent regions of ws: one clearing launch covers histograms (with the
  // status word and the tile counters in their free words), block counts and the compaction flags
  const size_t clear_words = (L.flags - L.hist) / 4 + flag_words(d, n_keep);
  if ((s = run_stats(d, q_win, window, q_pos0, inv_freq, t_next, mu, sigma, w, L, st, hist,
                     clear_words)) != EA_OK)
    return s;
  if (ev) EA_TRY(hipEventRecord(ev[1], st));
  if ((s = run_score(d, k, v, n, n_cap, mu, sigma, scores,
                     n_keep > 0 && !select_in_one_launch(n) ? hist : nullptr, true, w, L, st,
                     ev ? ev + 2 : nullptr, nullptr, nullptr, pm, kscale, vscale)) != EA_OK)
    return s;
  if (ev) EA_TRY(hipEventRecord(ev[4], st));
  if (n_keep > 0)
    EA_TRY(launch_select(d, scores, n, n_keep, idx, hist, (uint32_t*)(w + L.blk), true, st));
  if (ev) EA_TRY(hipEventRecord(ev[5], st));
  if (n_keep > 0 && unordered)
    EA_TRY(launch_compact_fill(d, k, v, n, n_cap, idx, n_keep, perm_out, st, pm));
  else if (n_keep > 0)
    EA_TRY(launch_compact(d, k, v, n, n_cap, idx, n_keep, k, v, flags, hist + 2 * kSelBins + kStatusSlot, st,
                          nullptr, 0, pm));
  if (ev) EA_TRY(hipEventRecord(ev[6], st));
  return EA_OK;
}

ea_status ea_compress_layer(const ea_params* p, const void* q_win, int64_t window, int64_t q_pos0,
                            const double* inv_freq, int64_t t_next, void* k, void* v, int64_t n,
                            int64_t n_cap, int64_t n_keep, float* scores_out, int32_t* idx_out,
                            void* ws, size_t ws_bytes, void* stream) {
  return compress_impl(p, q_win, window, q_pos0, inv_freq, t_next, k, v, n, n_cap, n_keep,
                       scores_out, idx_out, ws, ws_bytes, stream, nullptr);
}

// Pooled selection of ea_select_adaptive on the caller's stream.  `lifted`: a buffer of units * n
// floats that is not `scores` (only used with a floor); `top`: units * floor ints of scratch.
static ea_status run_select_adaptive(const Dims& d, const float* scores, int64_t n, int64_t n_keep, int64_t floor,
                                     int32_t* idx, int32_t* lengths, float* lifted, int32_t* top, char* w,
                                     const WsLayout& L, hipStream_t st) {
  uint32_t* hist = (uint32_t*)(w + L.hist);
  uint32_t* blk = (uint32_t*)(w + L.blk);
  int32_t* flat = (int32_t*)(w + L.idx);                // [B][Hkv * n_keep], ascending in [0, Hkv * n)
  const float* pooled = scores;
  if (floor > 0 && n_keep > 0) {
    // every head's own best `floor` pairs, then a copy of the scores with those lifted to +inf
    EA_TRY(launch_zero(hist, hist_words(d), st));
    EA_TRY(launch_select(d, scores, n, floor, top, hist, blk, false, st));
    EA_TRY(hipMemcpyAsync(lifted, scores, (size_t)d.units() * n * sizeof(float), hipMemcpyDeviceToDevice, st));
    EA_TRY(launch_mark_inf(lifted, top, d.units(), n, floor, st));
    pooled = lifted;
  }
  Dims layer = d;                                       // one pooled list per sequence
  layer.Hq = d.G;
  layer.Hkv = 1;
  if (n_keep > 0) {
    EA_TRY(launch_zero(hist, hist_words(d), st));
    EA_TRY(launch_select(layer, pooled, (int64_t)d.Hkv * n, (int64_t)d.Hkv * n_keep, flat, hist, blk, false, st));
  }
  EA_TRY(launch_split_pooled(flat, d.B, d.Hkv, n, n_keep, idx, lengths, st));
  return EA_OK;
}

ea_status ea_select_adaptive(const ea_params* p, const float* scores, int64_t n, int64_t n_keep,
                             int64_t floor, int32_t* idx, int32_t* lengths, void* ws, size_t ws_bytes,
                             void* stream) {
  Dims d;
  ea_status s = check_params(p, &d);
  if (s != EA_OK) return s;
  if (n < 1 || n > kMaxN || n_keep < 0 || n_keep > n || floor < 0 || floor > n_keep) return EA_ERR_INVALID_ARG;
  if (!aligned16(scores) || !aligned16(idx) || !lengths || ((uintptr_t)lengths & 3u)) return EA_ERR_INVALID_ARG;
  if ((int64_t)d.Hkv * n > kMaxN) return EA_ERR_UNSUPPORTED;      // the pooled list of a layer
  WsLayout L;
  if ((s = check_ws(d, n, 1, ws, ws_bytes, &L)) != EA_OK) return s;
  char* w = (char*)ws;
  return run_select_adaptive(d, scores, n, n_keep, floor, idx, lengths, (float*)(w + L.scores),
                             (int32_t*)(w + L.logits), w, L, (hipStream_t)stream);
}

ea_status ea_compress_layer_adaptive(const ea_params* p, const void* q_win, int64_t window, int64_t q_pos0,
                                     const double* inv_freq, int64_t t_next, void* k, void* v, int64_t n,
                                     int64_t n_cap, int64_t n_keep, int64_t floor, float* scores_out,
                                     int32_t* idx_out, int32_t* lengths_out, void* ws, size_t ws_bytes,
                                     void* stream) {
  Dims d;
  ea_status s = check_params(p, &d);
  if (s != EA_OK) return s;
  if (!aligned16(q_win) || !aligned16(k) || !aligned16(v) || k == v || !inv_freq || ((uintptr_t)inv_freq & 7u))
    return EA_ERR_INVALID_ARG;
  if ((scores_out && !aligned16(scores_out)) || !aligned16(idx_out) || !lengths_out || ((uintptr_t)lengths_out & 3u))
    return EA_ERR_INVALID_ARG;
  if (window < 1 + d.ddof || q_pos0 < 0 || t_next < 0) return EA_ERR_INVALID_ARG;
  if (window > kMaxWindow) return EA_ERR_UNSUPPORTED;
  if (n < 1 || n > n_cap || n > kMaxN || n_keep < 0 || n_keep > n || floor < 0 || floor > n_keep)
    return EA_ERR_INVALID_ARG;
  if ((int64_t)d.Hkv * n > kMaxN) return EA_ERR_UNSUPPORTED;
  if (partly_overlap(k, v, (size_t)d.units() * (size_t)n_cap * d.D * d.esize())) return EA_ERR_INVALID_ARG;
  WsLayout L;
  if ((s = check_ws(d, n, window, ws, ws_bytes, &L)) != EA_OK) return s;
  hipStream_t st = (hipStream_t)stream;
  char* w = (char*)ws;
  float* mu = (float*)(w + L.mu);
  float* sigma = (float*)(w + L.sigma);
  float* scores = scores_out ? scores_out : (float*)(w + L.scores);
  if ((s = run_stats(d, q_win, window, q_pos0, inv_freq, t_next, mu, sigma, w, L, st)) != EA_OK) return s;
  if ((s = run_score(d, k, v, n, n_cap, mu, sigma, scores, nullptr, false, w, L, st)) != EA_OK) return s;
  // after pass B the logit and value-norm scratch is free: the floor's lists and the lifted copy
  // of the scores go there
  if ((s = run_select_adaptive(d, scores, n, n_keep, floor, idx_out, lengths_out, (float*)(w + L.vnorm),
                               (int32_t*)(w + L.logits), w, L, st)) != EA_OK)
    return s;
  uint32_t* flags = (uint32_t*)(w + L.flags);
  uint32_t* status = (uint32_t*)(w + L.hist) + 2 * kSelBins + kStatusSlot;
  EA_TRY(launch_zero(flags, flag_words(d, n), st));
  EA_TRY(launch_compact(d, k, v, n, n_cap, idx_out, n, k, v, flags, status, st, lengths_out, n));
  return EA_OK;
}

ea_status ea_compact_ragged(const ea_params* p, void* k, void* v, int64_t n, int64_t n_cap,
                            const int32_t* idx, const int32_t* lengths, void* ws, size_t ws_bytes,
                            void* stream) {
  Dims d;
  ea_status s = check_params(p, &d);
  if (s != EA_OK) return s;
  if (!aligned16(k) || !aligned16(v) || k == v || !aligned16(idx) || !lengths || ((uintptr_t)lengths & 3u))
    return EA_ERR_INVALID_ARG;
  if (n < 1 || n > n_cap || n > kMaxN) return EA_ERR_INVALID_ARG;
  if (partly_overlap(k, v, (size_t)d.units() * (size_t)n_cap * d.D * d.esize())) return EA_ERR_INVALID_ARG;
  WsLayout L;
  if ((s = check_ws(d, n, 1, ws, ws_bytes, &L)) != EA_OK) return s;
  hipStream_t st = (hipStream_t)stream;
  uint32_t* flags = (uint32_t*)((char*)ws + L.flags);
  uint32_t* status = (uint32_t*)((char*)ws + L.hist) + 2 * kSelBins + kStatusSlot;
  EA_TRY(launch_zero(flags, flag_words(d, n), st, status));
  EA_TRY(launch_compact(d, k, v, n, n_cap, idx, n, k, v, flags, status, st, lengths, n));
  return EA_OK;
}

ea_status ea_score_baseline(const ea_params* p, int32_t scorer, const void* k, int64_t n, int64_t n_cap,
                            int64_t n_sink, float* scores, void* ws, size_t ws_bytes, void* stream) {
  Dims d;
  ea_status s = check_params(p, &d);
  if (s != EA_OK) return s;
  if (scorer != EA_SCORER_KNORM && scorer != EA_SCORER_STREAMING && scorer != EA_SCORER_KEYDIFF)
    return EA_ERR_INVALID_ARG;
  if (!aligned16(k) || !aligned16(scores)) return EA_ERR_INVALID_ARG;
  if (n < 1 || n > n_cap || n > kMaxN || n_sink < 0) return EA_ERR_INVALID_ARG;
  if (scorer == EA_SCORER_STREAMING && n > ((int64_t)1 << 24)) return EA_ERR_UNSUPPORTED;
  WsLayout L;
  if ((s = check_ws(d, n, 1, ws, ws_bytes, &L)) != EA_OK) return s;
  EA_TRY(launch_baseline(d, scorer, k, n, n_cap, n_sink, scores, (float*)((char*)ws + L.base),
                         (hipStream_t)stream));
  return EA_OK;
}

ea_status ea_compact_unordered(const ea_params* p, void* k, void* v, int64_t n, int64_t n_cap,
                               const int32_t* idx, int64_t n_keep, int32_t* perm_out, void* stream) {
  Dims d;
  ea_status s = check_params(p, &d, true);
  if (s != EA_OK) return s;
  if (!aligned16(k) || !aligned16(v) || k == v) return EA_ERR_INVALID_ARG;
  if (n < 1 || n > n_cap || n > kMaxN || n_keep < 0 || n_keep > n) return EA_ERR_INVALID_ARG;
  if (partly_overlap(k, v, (size_t)d.units() * (size_t)n_cap * d.D * d.esize())) return EA_ERR_INVALID_ARG;
  if (n_keep > 0 && (!aligned16(idx) || (perm_out && !aligned16(perm_out)))) return EA_ERR_INVALID_ARG;
  if (n_keep == 0) return EA_OK;
  EA_TRY(launch_compact_fill(d, k, v, n, n_cap, idx, n_keep, perm_out, (hipStream_t)stream));
  return EA_OK;
}

ea_status ea_compress_layer_unordered(const ea_params* p, const void* q_win, int64_t window,
                                      int64_t q_pos0, const double* inv_freq, int64_t t_next, void* k,
                                      void* v, int64_t n, int64_t n_cap, int64_t n_keep,
                                      float* scores_out, int32_t* idx_out, int32_t* perm_out, void* ws,
                                      size_t ws_bytes, void* stream) {
  return compress_impl(p, q_win, window, q_pos0, inv_freq, t_next, k, v, n, n_cap, n_keep,
                       scores_out, idx_out, ws, ws_bytes, stream, nullptr, true, perm_out);
}

ea_status ea_score_paged(const ea_params* p, const void* k_pool, const void* v_pool, const ea_paged* pg,
                         int64_t n, const float* mu, const float* sigma, float* scores, void* ws,
                         size_t ws_bytes, void* stream) {
  Dims d;
  ea_status s = check_params(p, &d);
  if (s != EA_OK) return s;
  if (!aligned16(k_pool) || !aligned16(v_pool) || !aligned16(mu) || !aligned16(sigma) || !aligned16(scores))
    return EA_ERR_INVALID_ARG;
  if (n < 1 || n > kMaxN) return EA_ERR_INVALID_ARG;
  PageMap pm;
  if ((s = check_paged(d, pg, n, &pm)) != EA_OK) return s;
  WsLayout L;
  if ((s = check_ws(d, n, 1, ws, ws_bytes, &L)) != EA_OK) return s;
  return run_score(d, k_pool, v_pool, n, 0, mu, sigma, scores, nullptr, false, (char*)ws, L,
                   (hipStream_t)stream, nullptr, nullptr, nullptr, &pm);
}

ea_status ea_compact_paged(const ea_params* p, void* k_pool, void* v_pool, const ea_paged* pg, int64_t n,
                           const int32_t* idx, int64_t n_keep, int32_t order_free, int32_t* perm_out,
                           void* ws, size_t ws_bytes, void* stream) {
  Dims d;
  ea_status s = check_params(p, &d);
  if (s != EA_OK) return s;
  if (!aligned16(k_pool) || !aligned16(v_pool) || k_pool == v_pool) return EA_ERR_INVALID_ARG;
  if (n < 1 || n > kMaxN || n_keep < 0 || n_keep > n) return EA_ERR_INVALID_ARG;
  if (n_keep > 0 && (!aligned16(idx) || (perm_out && !aligned16(perm_out)))) return EA_ERR_INVALID_ARG;
  PageMap pm;
  if ((s = check_paged(d, pg, n, &pm)) != EA_OK) return s;
  {
    const size_t bytes = (size_t)pg->num_blocks * d.Hkv * pg->block_size * d.D * d.esize();
    if (partly_overlap(k_pool, v_pool, bytes)) return EA_ERR_INVALID_ARG;
  }
  WsLayout L;
  if ((s = check_ws(d, n, 1, ws, ws_bytes, &L)) != EA_OK) return s;
  if (n_keep == 0) return EA_OK;
  hipStream_t st = (hipStream_t)stream;
  if (order_free) {
    EA_TRY(launch_compact_fill(d, k_pool, v_pool, n, 0, idx, n_keep, perm_out, st, &pm));
    return EA_OK;
  }
  uint32_t* flags = (uint32_t*)((char*)ws + L.flags);
  uint32_t* status = (uint32_t*)((char*)ws + L.hist) + 2 * kSelBins + kStatusSlot;
  EA_TRY(launch_zero(flags, flag_words(d, n_keep), st, status));
  EA_TRY(launch_compact(d, k_pool, v_pool, n, 0, idx, n_keep, k_pool, v_pool, flags, status, st, nullptr, 0, &pm));
  return EA_OK;
}

ea_status ea_compress_layer_paged(const ea_params* p, const void* q_win, int64_t window, int64_t q_pos0,
                                  const double* inv_freq, int64_t t_next, void* k_pool, void* v_pool,
                                  const ea_paged* pg, int64_t n, int64_t n_keep, int32_t order_free,
                                  float* scores_out, int32_t* idx_out, int32_t* perm_out, void* ws,
                                  size_t ws_bytes, void* stream) {
  Dims d;
  ea_status s = check_params(p, &d);
  if (s != EA_OK) return s;
  if (n < 1 || n > kMaxN) return EA_ERR_INVALID_ARG;
  PageMap pm;
  if ((s = check_paged(d, pg, n, &pm)) != EA_OK) return s;
  if (aligned16(k_pool) && aligned16(v_pool) &&
      partly_overlap(k_pool, v_pool, (size_t)pg->num_blocks * d.Hkv * pg->block_size * d.D * d.esize()))
    return EA_ERR_INVALID_ARG;
  // n_cap = n for the shared checks; the kernels do not use it with a page map
  return compress_impl(p, q_win, window, q_pos0, inv_freq, t_next, k_pool, v_pool, n, n, n_keep, scores_out,
                       idx_out, ws, ws_bytes, stream, nullptr, order_free != 0, order_free ? perm_out : nullptr,
                       &pm);
}

ea_status ea_score_fp8(const ea_params* p, const void* k8, const void* v8, const float* k_scale,
                       const float* v_scale, int64_t n, int64_t n_cap, const float* mu, const float* sigma,
                       float* scores, void* ws, size_t ws_bytes, void* stream) {
  Dims d;
  ea_status s = check_params(p, &d);
  if (s != EA_OK) return s;
  if (d.dtype != EA_BF16 || d.D == 64) return EA_ERR_UNSUPPORTED;
  if (!aligned16(k8) || !aligned16(v8) || !aligned16(mu) || !aligned16(sigma) || !aligned16(scores))
    return EA_ERR_INVALID_ARG;
  if ((k_scale && ((uintptr_t)k_scale & 3u)) || (v_scale && ((uintptr_t)v_scale & 3u))) return EA_ERR_INVALID_ARG;
  if (n < 1 || n > n_cap || n > kMaxN) return EA_ERR_INVALID_ARG;
  d.kv_fp8 = 1;
  WsLayout L;
  if ((s = check_ws(d, n, 1, ws, ws_bytes, &L)) != EA_OK) return s;
  return run_score(d, k8, v8, n, n_cap, mu, sigma, scores, nullptr, false, (char*)ws, L, (hipStream_t)stream,
                   nullptr, nullptr, nullptr, nullptr, k_scale, v_scale);
}

ea_status ea_compress_layer_fp8(const ea_params* p, const void* q_win, int64_t window, int64_t q_pos0,
                                const double* inv_freq, int64_t t_next, void* k8, void* v8,
                                const float* k_scale, const float* v_scale, int64_t n, int64_t n_cap,
                                int64_t n_keep, int32_t order_free, float* scores_out, int32_t* idx_out,
                                int32_t* perm_out, void* ws, size_t ws_bytes, void* stream) {
  return compress_impl(p, q_win, window, q_pos0, inv_freq, t_next, k8, v8, n, n_cap, n_keep, scores_out, idx_out,
                       ws, ws_bytes, stream, nullptr, order_free != 0, order_free ? perm_out : nullptr, nullptr,
                       true, k_scale, v_scale);
}

ea_status ea_compress_layer_timed(const ea_params* p, const void* q_win, int64_t window,
                                  int64_t q_pos0, const double* inv_freq, int64_t t_next, void* k,
                                  void* v, int64_t n, int64_t n_cap, int64_t n_keep, void* ws,
                                  size_t ws_bytes, void* stream, float* stage_ms) {
  if (!stage_ms) return EA_ERR_INVALID_ARG;
  hipEvent_t ev[EA_N_STAGES + 1];
  int made = 0;
  ea_status s = EA_OK;
  for (; made <= EA_N_STAGES; ++made)
    if (hipEventCreate(&ev[made]) != hipSuccess) { s = EA_ERR_DEVICE; break; }
  if (s == EA_OK)
    s = compress_impl(p, q_win, window, q_pos0, inv_freq, t_next, k, v, n, n_cap, n_keep, nullptr,
                      nullptr, ws, ws_bytes, stream, ev);
  if (s == EA_OK && hipEventSynchronize(ev[EA_N_STAGES]) != hipSuccess) s = EA_ERR_DEVICE;
  if (s == EA_OK)
    for (int i = 0; i < EA_N_STAGES; ++i)
      if (hipEventElapsedTime(&stage_ms[i], ev[i], ev[i + 1]) != hipSuccess) s = EA_ERR_DEVICE;
  for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
  return s;
}

ea_status ea_debug_status(const ea_params* p, int64_t n, int64_t window, const void* ws,
                          size_t ws_bytes, void* stream, uint32_t* status) {
  Dims d;
  ea_status s = check_params(p, &d);
  if (s != EA_OK) return s;
  if (!status || n < 1 || n > kMaxN || window < 1 || window > kMaxWindow) return EA_ERR_INVALID_ARG;
  WsLayout L;
  if ((s = check_ws(d, n, window, const_cast<void*>(ws), ws_bytes, &L)) != EA_OK) return s;
  hipStream_t st = (hipStream_t)stream;
  uint32_t w = 0u;
  EA_TRY(hipStreamSynchronize(st));
  EA_TRY(hipMemcpy(&w, (const char*)ws + L.hist + (2 * (size_t)kSelBins + kStatusSlot) * 4, 4, hipMemcpyDeviceToHost));
  *status = w & (EA_STATUS_BAD_SCORE | EA_STATUS_COMPACT_WAIT | EA_STATUS_BAD_INDEX);
  return EA_OK;
}

}  // extern "C"
