// Host-only part of libea: argument validation, tiling plans, workspace layout, and the two
// host helpers of the ABI.  Nothing here touches the GPU, so it is testable without one.
#include <math.h>

#include "ea_common.h"

namespace ea {

ea_status check_params(const ea_params* p, Dims* d, bool rows_only) {
  if (!p) return EA_ERR_INVALID_ARG;
  if (p->batch < 1 || p->n_kv_heads < 1 || p->n_q_heads < 1) return EA_ERR_INVALID_ARG;
  if (p->n_q_heads % p->n_kv_heads != 0) return EA_ERR_INVALID_ARG;
  if (p->cov_ddof != 0 && p->cov_ddof != 1) return EA_ERR_INVALID_ARG;
  if (p->rope_layout != 0 && p->rope_layout != 1) return EA_ERR_INVALID_ARG;
  if (p->q_is_rotated != 0 && p->q_is_rotated != 1) return EA_ERR_INVALID_ARG;
  if (p->horizon_T < 1) return EA_ERR_INVALID_ARG;
  if (!(p->epsilon >= 0.0f) || !isfinite(p->epsilon)) return EA_ERR_INVALID_ARG;
  const bool fp8 = p->dtype == EA_FP8_E4M3;
  if (p->dtype != EA_F32 && p->dtype != EA_BF16 && !(fp8 && rows_only)) return EA_ERR_UNSUPPORTED;
  if (p->head_dim != 64 && p->head_dim != 128 && p->head_dim != 256) return EA_ERR_UNSUPPORTED;
  if (fp8 && p->head_dim == 64) return EA_ERR_UNSUPPORTED;
  int G = p->n_q_heads / p->n_kv_heads;
  if (G > 64) return EA_ERR_UNSUPPORTED;
  if ((int64_t)p->batch * p->n_q_heads > (1 << 20)) return EA_ERR_UNSUPPORTED;
  d->B = p->batch;
  d->Hq = p->n_q_heads;
  d->Hkv = p->n_kv_heads;
  d->G = G;
  d->D = p->head_dim;
  d->half = p->head_dim / 2;
  d->dtype = fp8 ? (int)EA_BF16 : p->dtype;
  d->kv_fp8 = fp8 ? 1 : 0;
  d->rope_layout = p->rope_layout;
  d->q_is_rotated = p->q_is_rotated;
  d->ddof = p->cov_ddof;
  d->T = p->horizon_T;
  d->eps = p->epsilon;
  return EA_OK;
}

// Largest number of query heads whose fragments fit the 160 KiB LDS next to the per-wave
// staging buffers, and the template instance (GH) that covers ceil(G / passes) heads.
ScorePlan make_score_plan(const Dims& d, int64_t n, int num_cu, int paged) {
  ScorePlan s;
  s.hw = 0;
  s.tpt = 1;
  s.lse_pass = 0;
  if (!paged && !d.kv_fp8 && d.D == 128 && d.dtype == EA_BF16 && d.G % 4 == 0 && n >= 2048 && (int64_t)d.units() * (d.G / 4) <= 8) {
    // groups of four query heads at d = 128, calls of up to 8 (KV head, group) units: fragments in
    // registers, one wavefront per head, two workgroups of four wavefronts per CU.  Measured per
    // layer of 8 KV heads x 131072 keys: 128 us against 129 us for the LDS-fragment kernel and a
    // cheaper finalize pass (coarser partials) when a call holds one layer; with two or more
    // layers per call the LDS-fragment kernel is the faster one (115 against 121 us).
    s.hw = 1;
    s.GH = 4;
    s.passes = d.G / 4;
    s.NW = 4;
    s.nfrag = 4 * frags_per_head(128) + 2 * ksteps(128);
    s.lds_bytes = 0;
    const int64_t ntiles = (n + 31) / 32;
    int64_t wgs = 2 * (int64_t)num_cu / ((int64_t)d.units() * s.passes);
    if (wgs < 1) wgs = 1;
    if (wgs > 1024) wgs = 1024;
    // a ticket is four tiles where that still leaves every workgroup several tickets
    s.tpt = (ntiles + 3) / 4 >= 4 * wgs ? 4 : 1;
    const int64_t nblocks = (ntiles + s.tpt - 1) / s.tpt;
    if (wgs > nblocks) wgs = nblocks;
    s.nchunk = (int)wgs;
    s.span = (int)((n + wgs - 1) / wgs);
    s.pg = 32 * s.tpt;
    s.npart = (int)nblocks;
    return s;
  }
  const int NF = frags_per_head(d.D), NKS = ksteps(d.D);
  const size_t lds_max = 160 * 1024, slack = 1024;
  const int inst64[] = {1, 2, 4, 8}, inst128[] = {1, 2, 3, 4, 5}, inst256[] = {1};
  const int* inst = d.D == 64 ? inst64 : d.D == 128 ? inst128 : inst256;
  const int ninst = d.D == 64 ? 4 : d.D == 128 ? 5 : 1;
  s.NW = d.D == 256 ? 4 : d.D == 128 ? kNW128 : 8;
  const size_t stage = (size_t)s.NW * 16 * d.D * 2;
  int ghmax = 1;
  for (int i = 0; i < ninst; ++i)
    if ((size_t)(inst[i] * NF + 2 * NKS) * 1024 + stage + slack <= lds_max) ghmax = inst[i];
  s.passes = (d.G + ghmax - 1) / ghmax;
  int need = (d.G + s.passes - 1) / s.passes;
  s.GH = ghmax;
  for (int i = ninst - 1; i >= 0; --i)
    if (inst[i] >= need) s.GH = inst[i];
  s.nfrag = s.GH * NF + 2 * NKS;
  s.lds_bytes = (size_t)s.nfrag * 1024 + stage + slack;
  if (d.D == 256 && d.G >= 2) {
    // two query heads per pass: their triangular fragments in LDS (144 KiB), the extra tile's in
    // registers, K staged through 4 KiB per wave: exactly the 160 KiB a workgroup may have
    s.GH = 2;
    s.passes = (d.G + 1) / 2;
    s.nfrag = 2 * NF + 2 * NKS;
    s.lds_bytes = (size_t)2 * NF * 1024 + (size_t)s.NW * 4096;
  }
  const int tile = s.NW * 32;
  int64_t wgs = num_cu / d.units();
  if (wgs < 1) wgs = 1;
  if (wgs > 1024) wgs = 1024;
  int64_t span = (n + wgs - 1) / wgs;
  span = (span + tile - 1) / tile * tile;
  if (span < tile) span = tile;
  s.span = (int)span;
  s.nchunk = (int)((n + span - 1) / span);
  s.lse_pass = 1;
  s.pg = kLseBlock;
  s.npart = (int)((n + s.pg - 1) / s.pg);
  return s;
}

WsLayout make_ws_layout(const Dims& d, int64_t n, int64_t window) {
  WsLayout w;
  size_t o = 0;
  auto take = [&](size_t bytes) {
    size_t at = o;
    o = align_up(o + bytes, 256);
    return at;
  };
  const size_t qh = (size_t)d.qheads(), un = (size_t)d.units();
  ScorePlan sp = make_score_plan(d, n, 256);
  w.tab = take((size_t)window * d.half * 2 * sizeof(float));
  w.qproj = take(qh * (size_t)window * d.D * sizeof(float));   // projected queries of ea_query_stats_hidden
  w.mu = take(qh * d.D * sizeof(float));
  w.sigma = take(qh * d.D * d.D * sizeof(float));
  w.frags = take(un * sp.passes * sp.nfrag * 1024);
  w.post = take(qh * 2 * sizeof(float));
  w.logits = take(qh * (size_t)n * 8);          // fp32 logits (bf16 path) or fp64 (fp32 path)
  w.vnorm = take(un * (size_t)n * sizeof(float));
  // (max, sum exp) partials: float2 per fixed block of keys (bf16 path), double2 per chunk (fp32 path)
  size_t part_bytes = qh * (((size_t)n + 31) / 32) * 8;     // the finest block any plan uses
  if (part_bytes < qh * 1024 * 16) part_bytes = qh * 1024 * 16;
  w.part = take(part_bytes);
  w.lse = take(qh * sizeof(double));
  w.scores = take(un * (size_t)n * sizeof(float));
  w.idx = take(un * (size_t)n * sizeof(int32_t));
  w.base = take(un * kBaselineChunks * d.D * sizeof(float));    // KeyDiff partial sums
  w.hist = take(un * 3 * kSelBins * sizeof(uint32_t) + 256);
  size_t nblk = ((size_t)n + kSelBlock - 1) / kSelBlock;
  w.blk = take(un * nblk * 2 * sizeof(uint32_t));
  size_t nch = ((size_t)n + kCompactRows - 1) / kCompactRows;
  w.flags = take(2 * un * (nch + kCompactTicketStride) * sizeof(uint32_t));   // ticket counters, then flags
  w.total = o;
  return w;
}

}  // namespace ea

extern "C" {

size_t ea_workspace_bytes(const ea_params* p, int64_t n, int64_t window) {
  ea::Dims d;
  if (ea::check_params(p, &d, true) != EA_OK) return 0;
  if (n < 1 || n > ea::kMaxN || window < 1 || window > ea::kMaxWindow) return 0;
  return ea::make_ws_layout(d, n, window).total;
}

int64_t ea_n_keep(int64_t n, double ratio) {
  if (n < 0 || !(ratio >= 0.0) || !(ratio <= 1.0)) return -1;
  return (int64_t)((double)n * (1.0 - ratio));
}

const char* ea_status_string(ea_status s) {
  switch (s) {
    case EA_OK: return "ok";
    case EA_ERR_INVALID_ARG: return "invalid argument";
    case EA_ERR_UNSUPPORTED: return "unsupported configuration";
    case EA_ERR_WORKSPACE: return "workspace too small";
    case EA_ERR_DEVICE: return "device launch failed";
  }
  return "unknown status";
}

}  // extern "C"
