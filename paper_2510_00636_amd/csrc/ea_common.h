// Internal definitions shared by the host shim and the HIP kernels of libea.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include "../../include/ea.h"

namespace ea {

constexpr int kNW128 = 8;            // wavefronts per workgroup of the d = 128 score kernel
constexpr int kMaxWindow = 4096;
constexpr int64_t kMaxN = (int64_t)1 << 26;   // cached rows per head the launch grids cover
constexpr int kSelBins = 2048;        // radix-select digit width: 11 + 11 + 10 bits
constexpr int kSelBlock = 4096;       // scores per workgroup in the select passes
constexpr int kLseBlock = 2048;       // keys per softmax partial when the partials are taken from the stored logits
constexpr int kCompactRows = 96;     // destination rows per workgroup chunk in ea_compact (not a power of two on purpose)
// rows of 128 bytes (8-bit caches at d = 128, 16-bit at d = 64) come twice as many to a chunk: the
// same 24 KiB per workgroup for its ticket, its flags and its index loads
constexpr int compact_rows(int row_bytes) { return row_bytes <= 128 ? 2 * kCompactRows : kCompactRows; }

struct Dims {
  int B, Hq, Hkv, G, D, half;
  int dtype, rope_layout, q_is_rotated, ddof, T;
  float eps;
  int kv_fp8;     // 1: K and V rows are e4m3 bytes (dtype then describes q_win only)
  int units() const { return B * Hkv; }
  int qheads() const { return B * Hq; }
  int esize() const { return kv_fp8 ? 1 : dtype == EA_BF16 ? 2 : 4; }    // of a cached element
};

// How the matrix-core score kernel is tiled for one (d, G): heads per pass, passes, waves.
struct ScorePlan {
  int GH;       // query heads whose Sigma fragments are LDS-resident in one pass
  int passes;   // ceil(G / GH); K is streamed once per pass
  int NW;       // wavefronts per workgroup
  int nfrag;    // 1 KiB fragments per (unit, pass)
  int span;     // keys per workgroup were the head split evenly (the kernel deals tiles by ticket)
  int nchunk;   // workgroups per unit = ceil(n / span)
  int hw;       // 1: the register-fragment kernel (one wavefront per query head, d = 128, groups of four)
  int tpt;      // that kernel: tiles of 32 keys per ticket (1 or 4)
  int pg;       // keys per softmax partial (max, sum exp): partial j covers keys [j*pg, (j+1)*pg)
  int npart;    // partials per query head = ceil(n / pg)
  int lse_pass; // 1: pass A leaves only logits; the partials are taken from them by a pass of their own
  size_t lds_bytes;
};

// Paged caches: K and V are pools [num_blocks][Hkv][bs][d]; logical block j of sequence b is pool
// block table[b * max_blocks + j]; bs = 1 << sh.  table == nullptr: contiguous tensors.
struct PageMap {
  const int32_t* table;
  int sh, max_blocks, hkv;
  long long num_blocks;
};

struct WsLayout {
  size_t tab, qproj, mu, sigma, frags, post, logits, vnorm, part, lse, scores, idx, base, hist, blk, flags, total;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// rows_only: the call only moves cache rows, so p->dtype may also be EA_FP8_E4M3
ea_status check_params(const ea_params* p, Dims* d, bool rows_only = false);
// paged: the caches are block pools (the register-fragment kernel does not read those)
ScorePlan make_score_plan(const Dims& d, int64_t n, int num_cu, int paged = 0);
WsLayout make_ws_layout(const Dims& d, int64_t n, int64_t window);

// Free words of unit 0's third radix histogram (its last digit has 1024 bins): (T, q) of the
// selection at 1024/1025, a status word at kStatusSlot, the score kernel's tile counters from
// kTicketSlot on.  The launch that clears the histograms clears them all.
constexpr int kStatusSlot = 1030;
constexpr int kTicketSlot = 1040;
// Status bits (see ea_debug_status)
constexpr uint32_t kStatusBadScore = 1u;      // ea_select met a negative or NaN score
constexpr uint32_t kStatusCompactWait = 2u;   // in-place ea_compact gave up waiting: stores skipped
constexpr uint32_t kStatusBadIndex = 4u;      // ea_compact met an idx list that is not strictly ascending in [j, n)
constexpr int kBaselineChunks = 256;          // most row chunks per head in the KeyDiff mean
constexpr int kCompactTicketStride = 64;      // words per (unit, tensor) at the head of the flag region

// fragments per head of the triangular Sigma tiling, and per pass
inline int frags_per_head(int D) { int njt = D / 32; return njt * (njt + 1); }
inline int ksteps(int D) { return D / 16; }

}  // namespace ea
