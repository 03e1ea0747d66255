// Gather / compaction of K and V (Listing 1: keys[indices], values[indices]).
//
// Row idx[j] of each (unit, tensor) moves to row j.  idx is strictly ascending, so idx[j] >= j:
// a row only ever moves toward the front.  Work is cut into chunks of 64 destination rows.
// A chunk first loads all of its source rows into registers, then stores them.
//
// In place, chunk c's destination rows [j0, j1) may be source rows of an earlier chunk c' < c
// of the same tensor (never of a later one, whose sources lie at or beyond its own, higher,
// destinations).  So chunk c may store only after every such c' has finished *loading*.
// Each chunk publishes a "loaded" flag right after its loads complete -- a step that waits on
// nothing -- and chunk c polls the flags of the contiguous range of earlier chunks whose
// source interval [idx[first], idx[last]] meets [j0, j1); the range is found with a 64-ary
// search over idx.  Chunk numbers are handed out by an atomic ticket, so every chunk a
// workgroup waits on is already running: the wait always ends.
#include <hip/hip_runtime.h>

#include "ea_kernels.h"

namespace ea {

constexpr int kCompactSpinLimit = 1 << 20;

struct CompactArgs {
  const uint4* src[2];
  uint4* dst[2];
  const int32_t* idx;
  long long n_cap;
  int n, n_keep, units, nch;
  uint32_t* flags;    // [2*units*nch] loaded flags, then [1] ticket
  int inplace;
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

// RB = row bytes.  256 threads move 64 rows: RB/64 16-byte pieces per thread.
template <int RB>
__global__ __launch_bounds__(256) void k_compact(CompactArgs a) {
  constexpr int CPR = RB / 16;                 // 16-byte pieces per row
  constexpr int NLD = kCompactRows * CPR / 256;
  __shared__ int s_id;
  const int tid = threadIdx.x;
  const int ntu = 2 * a.units;
  if (tid == 0) s_id = a.inplace ? (int)atomicAdd(&a.flags[(size_t)ntu * a.nch], 1u) : (int)blockIdx.x;
  __syncthreads();
  const int id = s_id;
  const int tu = id % ntu, c = id / ntu;
  const int unit = tu >> 1, tensor = tu & 1;
  const int j0 = c * kCompactRows, j1 = min(j0 + kCompactRows, a.n_keep);
  const int32_t* idx = a.idx + (size_t)unit * a.n_keep;
  const uint4* src = a.src[tensor] + (size_t)unit * a.n_cap * CPR;
  uint4* dst = a.dst[tensor] + (size_t)unit * a.n_cap * CPR;
  // rows are strictly ascending with idx[j] >= j, so idx[j1-1] == j1-1 means nothing moves
  const bool identity = a.inplace && idx[j1 - 1] == j1 - 1;

  uint4 buf[NLD];
  if (!identity) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int e = tid + 256 * i, row = e / CPR, col = e % CPR;
      // a malformed index can never leave the tensor: clamp to [0, n)
      if (j0 + row < j1) buf[i] = src[(size_t)min(max(idx[j0 + row], 0), a.n - 1) * CPR + col];
    }
  }
  if (a.inplace) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                                    // every row of this chunk is in registers
    uint32_t* flag = a.flags + (size_t)tu * a.nch;
    if (tid == 0) __hip_atomic_store(&flag[c], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    if (!identity && tid < 64) {
      // earlier chunks c' whose sources [idx[64c'], idx[64c'+63]] meet my rows [j0, j1)
      const int lo = first_true(c, tid, [&](int x) { return idx[x * kCompactRows + kCompactRows - 1] >= j0; });
      const int hi = first_true(c, tid, [&](int x) { return idx[x * kCompactRows] >= j1; }) - 1;
      // The awaited chunks hold lower tickets, so they are running and will publish; the
      // spin bound only makes sure that a malformed idx cannot turn into a hang.
      for (int cc = lo + tid; cc <= hi; cc += 64)
        for (int spin = 0; spin < kCompactSpinLimit &&
             __hip_atomic_load(&flag[cc], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) == 0u; ++spin)
          __builtin_amdgcn_s_sleep(4);
    }
    __syncthreads();
  }
  if (!identity) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int e = tid + 256 * i, row = e / CPR, col = e % CPR;
      if (j0 + row < j1) dst[(size_t)(j0 + row) * CPR + col] = buf[i];
    }
  }
}

hipError_t launch_compact(const Dims& d, const void* k, const void* v, int64_t n, int64_t n_cap,
                          const int32_t* idx, int64_t n_keep, void* k_out, void* v_out,
                          uint32_t* flags, hipStream_t st) {
  CompactArgs a;
  a.n = (int)n;
  a.src[0] = (const uint4*)k;
  a.src[1] = (const uint4*)v;
  a.dst[0] = (uint4*)k_out;
  a.dst[1] = (uint4*)v_out;
  a.idx = idx;
  a.n_cap = n_cap;
  a.n_keep = (int)n_keep;
  a.units = d.units();
  a.nch = (int)((n_keep + kCompactRows - 1) / kCompactRows);
  a.flags = flags;
  a.inplace = (k_out == k && v_out == v) ? 1 : 0;
  const int rb = d.D * d.esize();
  const unsigned grid = 2u * a.units * a.nch;
  switch (rb) {
    case 128: k_compact<128><<<grid, 256, 0, st>>>(a); break;
    case 256: k_compact<256><<<grid, 256, 0, st>>>(a); break;
    case 512: k_compact<512><<<grid, 256, 0, st>>>(a); break;
    case 1024: k_compact<1024><<<grid, 256, 0, st>>>(a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace ea
