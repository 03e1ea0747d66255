// Internal definitions shared by the host shim and the HIP kernels of libea.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include "../../include/ea.h"

namespace ea {

#ifndef EA_NW128
#define EA_NW128 8              // wavefronts per workgroup of the d = 128 score kernel
#endif

constexpr int kMaxWindow = 4096;
constexpr int kSelBins = 2048;        // radix-select digit width: 11 + 11 + 10 bits
constexpr int kSelBlock = 4096;       // scores per workgroup in the select passes
constexpr int kCompactRows = 96;     // destination rows per workgroup chunk in ea_compact (not a power of two on purpose)

struct Dims {
  int B, Hq, Hkv, G, D, half;
  int dtype, rope_layout, q_is_rotated, ddof, T;
  float eps;
  int units() const { return B * Hkv; }
  int qheads() const { return B * Hq; }
  int esize() const { return dtype == EA_BF16 ? 2 : 4; }
};

// How the matrix-core score kernel is tiled for one (d, G): heads per pass, passes, waves.
struct ScorePlan {
  int GH;       // query heads whose Sigma fragments are LDS-resident in one pass
  int passes;   // ceil(G / GH); K is streamed once per pass
  int NW;       // wavefronts per workgroup
  int nfrag;    // 1 KiB fragments per (unit, pass)
  int span;     // keys per workgroup were the head split evenly (the kernel deals tiles by ticket)
  int nchunk;   // workgroups per unit = ceil(n / span)
  size_t lds_bytes;
};

struct WsLayout {
  size_t tab, mu, sigma, frags, post, logits, vnorm, part, scores, idx, hist, blk, flags, total;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

ea_status check_params(const ea_params* p, Dims* d);
ScorePlan make_score_plan(const Dims& d, int64_t n, int num_cu);
WsLayout make_ws_layout(const Dims& d, int64_t n, int64_t window);

// fragments per head of the triangular Sigma tiling, and per pass
inline int frags_per_head(int D) { int njt = D / 32; return njt * (njt + 1); }
inline int ksteps(int D) { return D / 16; }

}  // namespace ea
