// Gather / compaction of K and V (Listing 1: keys[indices], values[indices]).
//
// Row idx[j] of each (unit, tensor) moves to row j.  idx is strictly ascending, so idx[j] >= j:
// a row only ever moves toward the front.  Work is cut into chunks of kCompactRows destination rows.
// A chunk first loads all of its source rows into registers, then stores them.
//
// In place, chunk c's destination rows [j0, j1) may be source rows of an earlier chunk c' < c
// of the same tensor (never of a later one, whose sources lie at or beyond its own, higher,
// destinations).  So chunk c may store only after every such c' has finished *loading*.
// Each chunk publishes a "loaded" flag right after its loads complete -- a step that waits on
// nothing -- and chunk c polls the flags of the contiguous range of earlier chunks whose
// source interval [idx[first], idx[last]] meets [j0, j1); the range is found with a 64-ary
// search over idx.  Chunk numbers are handed out by atomic tickets, so every chunk a
// workgroup waits on is already running: the wait always ends.
#include <hip/hip_runtime.h>

#include "ea_kernels.h"

namespace ea {

constexpr int kCompactSpinLimit = 1 << 20;
constexpr int kTicketStride = kCompactTicketStride;   // words between the ticket counters of two tensors

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // native vector: stays in VGPRs

struct CompactArgs {
  const u32x4* src[2];
  u32x4* dst[2];
  const int32_t* idx;
  long long n_cap;
  int n, n_keep, units, nch;
  uint32_t* flags;    // [2*units][kTicketStride] ticket counters, then [2*units][nch] loaded flags
  int inplace;
  uint32_t* status;   // status word (bits kStatusCompactWait, kStatusBadIndex)
  const int32_t* lengths;   // nullable: kept rows of every unit (head-adaptive budgets); then n_keep is
  long long idx_stride;     // only the grid's upper bound, and a unit's list starts at unit * idx_stride
  PageMap pm;               // PAGED instances: src / dst are block pools (in place)
};

// First x in [0, c) for which the monotone predicate pred(x) (false ... false true ... true)
// holds, or c if it never does.  All 64 lanes of one wavefront call it; 64 probes per round.
template <typename Pred>
__device__ int first_true(int c, int lane, Pred pred) {
  int lo = 0, hi = c;                      // invariant: pred false below lo, answer in [lo, hi]
  while (lo < hi) {
    const int stride = (hi - lo + 63) / 64;
    const int probe = lo + lane * stride;
    const bool ok = probe >= hi ? true : pred(probe);
    const unsigned long long b = __ballot(ok);
    if (b == 0ull) {                       // all 64 probes false (and none reached hi)
      lo = lo + 63 * stride + 1;
      continue;
    }
    const int first = __ffsll((long long)b) - 1;
    const int nhi = min(lo + first * stride, hi);
    if (first > 0) lo = lo + (first - 1) * stride + 1;
    hi = nhi;
  }
  return hi;
}

// RB = row bytes.  Four mover wavefronts carry kCompactRows rows (kCompactRows * RB / 4096
// 16-byte pieces per thread); a fifth, control, wavefront takes the ticket, finds the chunks to wait for while
// the movers' loads are in flight, publishes this chunk's flag and polls the others.
//
// Tickets are per (unit, tensor): a workgroup serves tensor blockIdx % (2*units) and draws its
// chunk number from that tensor's own counter.  Hazards only exist inside one tensor, so the
// "everything I wait for is already running" argument holds per counter, and the counters
// (one per tensor, in separate cache lines) are not a serial bottleneck the way one global
// counter is.
template <int RB, bool PAGED>
__global__ __launch_bounds__(320) void k_compact(CompactArgs a) {
  constexpr int CPR = RB / 16;                 // 16-byte pieces per row
  constexpr int ROWS = compact_rows(RB);       // destination rows per chunk
  constexpr int NLD = ROWS * CPR / 256;
  constexpr int NCHK = (ROWS + 63) / 64;
  __shared__ int s_c, s_lo, s_hi, s_ident, s_abort;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool control = wave == 4;
  const int ntu = 2 * a.units;
  const int tu = blockIdx.x % ntu;
  uint32_t* flag = a.flags + (size_t)ntu * kTicketStride + (size_t)tu * a.nch;
  if (control && lane == 0) {
    uint32_t* ticket = a.flags + (size_t)tu * kTicketStride;
    s_c = a.inplace ? (int)atomicAdd(ticket, 1u) : (int)(blockIdx.x / ntu);
    s_lo = 0;
    s_hi = -1;
    s_abort = 0;
  }
  __syncthreads();
  const int c = s_c;
  const int unit = tu >> 1, tensor = tu & 1;
  const int n_keep = a.lengths ? a.lengths[unit] : a.n_keep;
  const int j0 = c * ROWS, j1 = min(j0 + ROWS, n_keep);
  if (j0 >= n_keep) return;           // ragged lists: this unit has fewer chunks than the grid allows for
  const int32_t* idx = a.idx + (size_t)unit * a.idx_stride;
  const u32x4* src = a.src[tensor] + (PAGED ? (size_t)0 : (size_t)unit * a.n_cap * CPR);
  u32x4* dst = a.dst[tensor] + (PAGED ? (size_t)0 : (size_t)unit * a.n_cap * CPR);
  // row of the tensor (or, paged, of the pool) that holds logical row `row` of this unit
  auto where = [&](int row) -> size_t { return PAGED ? paged_row(a.pm, unit, row) : (size_t)row; };
  // Rows are strictly ascending with idx[j] >= j, so idx[j1-1] == j1-1 means nothing moves.  Only
  // the control wavefront looks this up; the movers request their rows at once (waiting for the
  // answer would put one more memory round trip in front of every chunk) and learn it, through
  // s_ident, at the barrier before the stores.
  bool identity = false;
  if (control && a.inplace) identity = idx[j1 - 1] == j1 - 1;
  // The control wavefront also looks at the chunk's indices themselves (two per lane, requested
  // here, judged after the searches below): strictly ascending, idx[j] >= j, inside the tensor.
  // A list that is not makes the in-place hazard analysis void; the status word records it.
  int chk_cur[NCHK], chk_prev[NCHK];
#pragma unroll
  for (int t = 0; t < NCHK; ++t) { chk_cur[t] = 0; chk_prev[t] = -1; }
  if (control && tensor == 0) {
#pragma unroll
    for (int t = 0; t < NCHK; ++t) {
      const int j = min(j0 + lane + 64 * t, j1 - 1);
      chk_cur[t] = idx[j];
      chk_prev[t] = j > 0 ? idx[j - 1] : -1;
    }
  }

  u32x4 buf[NLD];
  size_t drow[PAGED ? NLD : 1];      // PAGED: pool rows of the destinations, looked up with the loads
  if (!control) {
    // First every index, then every row, none of them under a per-thread condition: a load
    // inside "if (row < j1)" is followed by a wait for everything in flight, which made the
    // eight index -> row pairs of a thread sixteen round trips in a row.  Pieces past the end of
    // a ragged last chunk load its last row again and are not stored.
    int srow[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) srow[i] = idx[min(j0 + (tid + 256 * i) / CPR, j1 - 1)];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int col = (tid + 256 * i) % CPR;
      // a malformed index can never leave the tensor: clamp to [0, n)
      // rows are read once and written once: non-temporal hints on both (4 % on this kernel)
      buf[i] = __builtin_nontemporal_load(&src[where(min(max(srow[i], 0), a.n - 1)) * CPR + col]);
    }
    if constexpr (PAGED) {
#pragma unroll
      for (int i = 0; i < NLD; ++i) drow[i] = where(min(j0 + (tid + 256 * i) / CPR, j1 - 1));
    }
    if (a.inplace) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // rows are in registers
  } else if (a.inplace && !identity) {
    // earlier chunks c' whose sources [idx[first], idx[last]] meet my rows [j0, j1)
    const int lo = first_true(c, lane, [&](int x) { return idx[x * ROWS + ROWS - 1] >= j0; });
    const int hi = first_true(c, lane, [&](int x) { return idx[x * ROWS] >= j1; }) - 1;
    if (lane == 0) { s_lo = lo; s_hi = hi; }
  }
  if (control && tensor == 0) {
    bool bad = false;
#pragma unroll
    for (int t = 0; t < NCHK; ++t) {
      const int j = min(j0 + lane + 64 * t, j1 - 1);
      bad |= chk_cur[t] <= chk_prev[t] || chk_cur[t] < j || chk_cur[t] >= a.n;
    }
    if (__ballot(bad) != 0ull && lane == 0) atomicOr(a.status, kStatusBadIndex);
  }
  if (a.inplace) {
    if (control && lane == 0) s_ident = identity;
    __syncthreads();                 // every mover's loads have landed
    if (control) {
      // Relaxed, device-scope flag: what it guards are this chunk's *loads*, which have
      // already returned, so nothing has to be flushed before it (a release would write back
      // this XCD's L2 on every chunk).
      if (lane == 0) __hip_atomic_store(&flag[c], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      // The awaited chunks hold lower tickets of the same counter, so they are running and
      // will publish; the spin bound only keeps a malformed idx from turning into a hang.  A wait
      // that runs out never stores past an unseen flag: the chunk's stores are skipped and the
      // workspace's status word says so (ea_debug_status).
      bool seen = true;
      for (int cc = s_lo + lane; cc <= s_hi; cc += 64) {
        int spin = 0;
        while (__hip_atomic_load(&flag[cc], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) {
          if (++spin >= kCompactSpinLimit) { seen = false; break; }
          __builtin_amdgcn_s_sleep(4);
        }
      }
      if (!seen) {
        s_abort = 1;
        atomicOr(a.status, kStatusCompactWait);
      }
    }
    __syncthreads();                 // stores are issued only after every awaited flag was seen
    identity = s_ident != 0 || s_abort != 0;
  }
  if (!control && !identity) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int e = tid + 256 * i, row = e / CPR, col = e % CPR;
      const size_t to = PAGED ? drow[i] : (size_t)(j0 + row);
      if (j0 + row < j1) __builtin_nontemporal_store(buf[i], &dst[to * CPR + col]);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Order-free compaction.  Attention over the cache is a sum over cached pairs (Eq. 2-3 of the
// paper) and the keys carry their rotary position inside them (Eq. 1), so the order of the kept
// pairs is free.  Then only the kept rows at or beyond the new length have to move: row idx[j0 + i]
// (j0 = number of kept rows below n_keep) goes to the i-th evicted position below n_keep.  The
// i-th such hole sits right after j kept rows, j being the smallest index with idx[j] - j > i
// (idx[j] - j = holes before kept row j), i.e. at position i + j.  Sources lie at or beyond
// n_keep and destinations below it, on rows nobody reads: no ordering between workgroups.
constexpr int kFillRows = 64;       // moved rows per workgroup

struct FillArgs {
  u32x4* t[2];
  const int32_t* idx;
  int32_t* perm;      // nullable: [units][n_keep], source row now at each position
  long long n_cap;
  int n, n_keep, units, nch;
  PageMap pm;         // PAGED instances: t[] are block pools
};

template <int RB, bool PAGED>
__global__ __launch_bounds__(256) void k_compact_fill(FillArgs a) {
  constexpr int CPR = RB / 16;
  constexpr int NLD = kFillRows * CPR / 256;
  __shared__ int s_j0;
  __shared__ int s_src[kFillRows], s_dst[kFillRows];
  const int tid = threadIdx.x, lane = tid & 63;
  const int ntu = 2 * a.units;
  const int tu = blockIdx.x % ntu, c = blockIdx.x / ntu;
  const int unit = tu >> 1, tensor = tu & 1;
  const int32_t* idx = a.idx + (size_t)unit * a.n_keep;
  if (tid < 64) {
    const int j0 = first_true(a.n_keep, lane, [&](int x) { return idx[x] >= a.n_keep; });
    if (lane == 0) s_j0 = j0;
  }
  __syncthreads();
  const int j0 = s_j0, m = a.n_keep - j0;
  int32_t* perm = a.perm ? a.perm + (size_t)unit * a.n_keep : nullptr;
  if (perm && tensor == 0)          // rows that stay: every workgroup of the unit takes a stride of them
    for (int j = c * 256 + tid; j < j0; j += a.nch * 256) perm[idx[j]] = idx[j];
  const int i0 = c * kFillRows;
  if (i0 >= m) return;
  if (tid < kFillRows) {
    const int i = min(i0 + tid, m - 1);
    int lo = 0, hi = j0;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (idx[mid] - mid > i) hi = mid; else lo = mid + 1;
    }
    const int src = min(max(idx[j0 + i], 0), a.n - 1), dst = i + lo;   // never outside the tensor
    s_src[tid] = src;
    s_dst[tid] = dst;
    if (perm && tensor == 0 && i0 + tid < m) perm[dst] = src;
  }
  __syncthreads();
  u32x4* base = a.t[tensor] + (PAGED ? (size_t)0 : (size_t)unit * a.n_cap * CPR);
  auto where = [&](int row) -> size_t { return PAGED ? paged_row(a.pm, unit, row) : (size_t)row; };
  u32x4 buf[NLD];
#pragma unroll
  for (int q = 0; q < NLD; ++q) {
    const int e = tid + 256 * q;
    buf[q] = __builtin_nontemporal_load(&base[where(s_src[e / CPR]) * CPR + e % CPR]);
  }
#pragma unroll
  for (int q = 0; q < NLD; ++q) {
    const int e = tid + 256 * q, row = e / CPR;
    if (i0 + row < m) __builtin_nontemporal_store(buf[q], &base[where(s_dst[row]) * CPR + e % CPR]);
  }
}

hipError_t launch_compact_fill(const Dims& d, void* k, void* v, int64_t n, int64_t n_cap,
                               const int32_t* idx, int64_t n_keep, int32_t* perm, hipStream_t st,
                               const PageMap* pm) {
  FillArgs a;
  a.pm = pm ? *pm : PageMap{nullptr, 0, 0, 1, 0};
  a.t[0] = (u32x4*)k;
  a.t[1] = (u32x4*)v;
  a.idx = idx;
  a.perm = perm;
  a.n_cap = n_cap;
  a.n = (int)n;
  a.n_keep = (int)n_keep;
  a.units = d.units();
  const int64_t most = n_keep < n - n_keep ? n_keep : n - n_keep;      // rows that can have to move
  a.nch = (int)((most + kFillRows - 1) / kFillRows);
  if (a.nch < 1) a.nch = 1;
  const unsigned grid = 2u * a.units * a.nch;
#define EA_FILL(RB)                                                   \
  case RB:                                                             \
    if (pm) k_compact_fill<RB, true><<<grid, 256, 0, st>>>(a);         \
    else k_compact_fill<RB, false><<<grid, 256, 0, st>>>(a);           \
    break
  switch (d.D * d.esize()) {
    EA_FILL(128);
    EA_FILL(256);
    EA_FILL(512);
    EA_FILL(1024);
    default: return hipErrorInvalidValue;
  }
#undef EA_FILL
  return hipGetLastError();
}

hipError_t launch_compact(const Dims& d, const void* k, const void* v, int64_t n, int64_t n_cap,
                          const int32_t* idx, int64_t n_keep, void* k_out, void* v_out,
                          uint32_t* flags, uint32_t* status, hipStream_t st, const int32_t* lengths,
                          int64_t idx_stride, const PageMap* pm) {
  CompactArgs a;
  a.pm = pm ? *pm : PageMap{nullptr, 0, 0, 1, 0};
  a.lengths = lengths;
  a.idx_stride = lengths ? idx_stride : n_keep;
  a.n = (int)n;
  a.src[0] = (const u32x4*)k;
  a.src[1] = (const u32x4*)v;
  a.dst[0] = (u32x4*)k_out;
  a.dst[1] = (u32x4*)v_out;
  a.idx = idx;
  a.n_cap = n_cap;
  a.n_keep = (int)n_keep;
  a.units = d.units();
  const int rb = d.D * d.esize();
  const int rows = rb == 128 ? compact_rows(128) : rb == 256 ? compact_rows(256) : rb == 512 ? compact_rows(512) : compact_rows(1024);
  a.nch = (int)((n_keep + rows - 1) / rows);       // (never more chunks than the flag region was sized for)
  a.flags = flags;
  a.status = status;
  a.inplace = (k_out == k && v_out == v) ? 1 : 0;
  const unsigned grid = 2u * a.units * a.nch;
#define EA_COMPACT(RB)                                                \
  case RB:                                                             \
    if (pm) k_compact<RB, true><<<grid, 320, 0, st>>>(a);              \
    else k_compact<RB, false><<<grid, 320, 0, st>>>(a);                \
    break
  switch (rb) {
    EA_COMPACT(128);
    EA_COMPACT(256);
    EA_COMPACT(512);
    EA_COMPACT(1024);
    default: return hipErrorInvalidValue;
  }
#undef EA_COMPACT
  return hipGetLastError();
}

}  // namespace ea
