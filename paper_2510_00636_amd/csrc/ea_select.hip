// Top-k selection per KV head (Sec. 2.2 "Compression", Listing 1 top-k) as an exact radix
// select on the fp32 bit patterns (non-negative floats order like unsigned integers).
//
// Three histogram passes (11 + 11 + 10 bits) narrow down the bit pattern T of the n_keep-th
// largest score and the number q of scores equal to T that must still be kept; every
// workgroup re-derives the digits found so far from the shared histograms (a 2048-entry
// suffix scan, cheaper than another launch).  Then a count pass and an emit pass write the
// kept positions in ascending order: score > T, or == T among the first q such positions.
#include <hip/hip_runtime.h>

#include "ea_kernels.h"

namespace ea {

constexpr int kSelThreads = 256;
constexpr int kSelPer = kSelBlock / kSelThreads;   // 16 consecutive scores per thread

// zeroes p[0, count) and, if given, the single word *extra
__global__ void k_zero(uint32_t* p, size_t count, uint32_t* extra) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) p[i] = 0;
  if (extra && i == 0) *extra = 0;
}

hipError_t launch_zero(uint32_t* p, size_t count, hipStream_t st, uint32_t* extra) {
  if (count == 0 && !extra) return hipSuccess;
  k_zero<<<(unsigned)((count + 255) / 256 + (count == 0)), 256, 0, st>>>(p, count, extra);
  return hipGetLastError();
}

// Bin b (counting down from the top) with  count(bins > b) < target <= count(bins >= b);
// *rem = target - count(bins > b).  Called by all 64 lanes of ONE wavefront; the result is
// uniform.  nbins is 2048 or 1024; lane l owns the nbins/64 bins just below nbins - l*nbins/64.
__device__ int find_bin_wave(const uint32_t* __restrict__ hist, int nbins, uint32_t target,
                             uint32_t* rem, int lane) {
  const int per = nbins / 64;                        // 32 or 16
  const int lo = nbins - per * (lane + 1);
  uint32_t loc[32];
  uint32_t sum = 0;
  const uint4* hp = reinterpret_cast<const uint4*>(hist + lo);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    if (4 * j < per) {
      const uint4 v = hp[j];
      loc[4 * j] = v.x; loc[4 * j + 1] = v.y; loc[4 * j + 2] = v.z; loc[4 * j + 3] = v.w;
      sum += v.x + v.y + v.z + v.w;
    } else {
      loc[4 * j] = loc[4 * j + 1] = loc[4 * j + 2] = loc[4 * j + 3] = 0;
    }
  }
  uint32_t incl = sum;                               // inclusive scan over lanes (lane 0 = top bins)
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  const uint32_t excl = incl - sum;
  const bool mine = excl < target && target <= incl;
  int b = 0;
  uint32_t r = 0;
  if (mine) {
    uint32_t cum = excl;
    b = lo;
    r = target - cum;
#pragma unroll
    for (int j = 31; j >= 0; --j) {                  // walk this lane's bins from the top down
      if (j < per) {
        if (target > cum && target <= cum + loc[j]) { b = lo + j; r = target - cum; }
        cum += loc[j];
      }
    }
  }
  const unsigned long long m = __ballot(mine);
  const int src = m ? __ffsll((long long)m) - 1 : 0;
  *rem = __shfl(r, src);
  return __shfl(b, src);
}

struct SelArgs {
  const float* scores;
  long long n;
  uint32_t n_keep;
  uint32_t* hist;    // [units][3][2048]; slot [unit][2][1024 + {0,1}] receives (T, q)
  uint32_t* blk;     // [units][nblk][2] = (count > T, count == T)
  int32_t* idx;      // [units][n_keep]
  int nblk;
};

// Digits fixed by the histogram passes before pass P: wavefront 0 re-derives them (a few
// hundred cycles, cheaper than another launch) and the workgroup reads them from s_res.
template <int P>
__device__ void resolve(const SelArgs& a, int unit, uint32_t* s_res, uint32_t* prefix, uint32_t* rem) {
  if (P >= 1 && threadIdx.x < 64) {
    const int lane = threadIdx.x;
    const uint32_t* h = a.hist + (size_t)unit * 3 * kSelBins;
    uint32_t r = a.n_keep, pre = 0;
    const int b0 = find_bin_wave(h, 2048, r, &r, lane);
    pre = (uint32_t)b0;
    if (P >= 2) { const int b1 = find_bin_wave(h + kSelBins, 2048, r, &r, lane); pre = (pre << 11) | (uint32_t)b1; }
    if (P >= 3) { const int b2 = find_bin_wave(h + 2 * kSelBins, 1024, r, &r, lane); pre = (pre << 10) | (uint32_t)b2; }
    if (lane == 0) { s_res[0] = pre; s_res[1] = r; }
  }
  __syncthreads();
  *prefix = P >= 1 ? s_res[0] : 0u;
  *rem = P >= 1 ? s_res[1] : a.n_keep;
  __syncthreads();
}

template <int P>
__global__ __launch_bounds__(kSelThreads) void k_sel_hist(SelArgs a) {
  __shared__ uint32_t s_hist[kSelBins];
  __shared__ uint32_t s_tmp[258];
  const int tid = threadIdx.x, unit = blockIdx.x;
  uint32_t prefix = 0, rem;
  resolve<P>(a, unit, s_tmp, &prefix, &rem);
  for (int i = tid; i < kSelBins; i += kSelThreads) s_hist[i] = 0;
  __syncthreads();
  const uint32_t* sc = reinterpret_cast<const uint32_t*>(a.scores) + (size_t)unit * a.n;
  const long long base = (long long)blockIdx.y * kSelBlock;
  // All loads first and none under a condition (indices past the end are clamped): a load inside
  // "if (i < n)" is followed by a wait for it, one memory round trip per score.
  uint32_t uu[kSelPer];
#pragma unroll
  for (int j = 0; j < kSelPer; ++j) uu[j] = sc[min(base + j * kSelThreads + tid, a.n - 1)];
#pragma unroll
  for (int j = 0; j < kSelPer; ++j) {
    const long long i = base + j * kSelThreads + tid;
    if (i < a.n) {
      const uint32_t u = uu[j];
      if (P == 0) {
        atomicAdd(&s_hist[u >> 21], 1u);
        // outside the domain (negative or NaN): the order of bit patterns is not the order of
        // values there; the selection still completes, the status word records it
        if (u > 0x7f800000u) atomicOr(a.hist + 2 * kSelBins + kStatusSlot, kStatusBadScore);
      }
      if (P == 1 && (u >> 21) == prefix) atomicAdd(&s_hist[(u >> 10) & 2047u], 1u);
      if (P == 2 && (u >> 10) == prefix) atomicAdd(&s_hist[u & 1023u], 1u);
    }
  }
  __syncthreads();
  uint32_t* out = a.hist + ((size_t)unit * 3 + P) * kSelBins;
  for (int i = tid; i < kSelBins; i += kSelThreads) {
    const uint32_t c = s_hist[i];
    if (c) atomicAdd(&out[i], c);
  }
}

// (count > T, count == T) of every 4096-score block; block 0 also publishes (T, q).
__global__ __launch_bounds__(kSelThreads) void k_sel_count(SelArgs a) {
  __shared__ uint32_t s_tmp[258];
  __shared__ uint32_t s_cnt[2];
  const int tid = threadIdx.x, unit = blockIdx.x;
  uint32_t T, q;
  resolve<3>(a, unit, s_tmp, &T, &q);
  if (tid < 2) s_cnt[tid] = 0;
  __syncthreads();
  const uint32_t* sc = reinterpret_cast<const uint32_t*>(a.scores) + (size_t)unit * a.n;
  const long long base = (long long)blockIdx.y * kSelBlock;
  uint32_t gt = 0, eq = 0;
  uint32_t uu[kSelPer];
#pragma unroll
  for (int j = 0; j < kSelPer; ++j) uu[j] = sc[min(base + j * kSelThreads + tid, a.n - 1)];
#pragma unroll
  for (int j = 0; j < kSelPer; ++j) {
    const long long i = base + j * kSelThreads + tid;
    const uint32_t u = uu[j];
    gt += i < a.n && u > T;
    eq += i < a.n && u == T;
  }
  for (int o = 32; o >= 1; o >>= 1) { gt += __shfl_xor(gt, o); eq += __shfl_xor(eq, o); }
  if ((tid & 63) == 0) { atomicAdd(&s_cnt[0], gt); atomicAdd(&s_cnt[1], eq); }
  __syncthreads();
  if (tid == 0) {
    a.blk[((size_t)unit * a.nblk + blockIdx.y) * 2 + 0] = s_cnt[0];
    a.blk[((size_t)unit * a.nblk + blockIdx.y) * 2 + 1] = s_cnt[1];
    if (blockIdx.y == 0) {
      uint32_t* slot = a.hist + ((size_t)unit * 3 + 2) * kSelBins + 1024;
      slot[0] = T;
      slot[1] = q;
    }
  }
}

// exclusive scan of one value per thread over the 256 threads of the workgroup: a shuffle scan
// inside each wavefront, then the four wave totals through LDS
__device__ uint32_t block_excl_scan(uint32_t v, uint32_t* s_tmp, uint32_t* total) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint32_t incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  __syncthreads();                       // s_tmp may still be read from an earlier call
  if (lane == 63) s_tmp[wave] = incl;
  __syncthreads();
  uint32_t before = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kSelThreads / 64; ++w) {
    const uint32_t t = s_tmp[w];
    before += w < wave ? t : 0u;
    tot += t;
  }
  *total = tot;
  return before + incl - v;
}

__global__ __launch_bounds__(kSelThreads) void k_sel_emit(SelArgs a) {
  __shared__ uint32_t s_tmp[258];
  __shared__ int32_t s_idx[kSelBlock];
  __shared__ uint32_t s_base[2];
  const int tid = threadIdx.x, unit = blockIdx.x, blk = blockIdx.y;
  const uint32_t* slot = a.hist + ((size_t)unit * 3 + 2) * kSelBins + 1024;
  const uint32_t T = slot[0], q = slot[1];
  if (tid < 64) {
    // kept pairs and ==T pairs in the blocks before this one: the lanes of wavefront 0 take the
    // earlier blocks in order (64 at a time) and scan them
    const uint32_t* b = a.blk + (size_t)unit * a.nblk * 2;
    uint32_t kept = 0, eqs = 0;                     // totals of all earlier blocks seen so far
    for (int j0 = 0; j0 < blk; j0 += 64) {
      const int j = j0 + tid;
      const uint32_t g = j < blk ? b[2 * j] : 0u, e = j < blk ? b[2 * j + 1] : 0u;
      uint32_t ei = e;                              // inclusive scan of e over the lanes
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = __shfl_up(ei, o);
        if (tid >= o) ei += up;
      }
      const uint32_t eq_before = eqs + ei - e;      // ==T pairs before block j
      const uint32_t room = q > eq_before ? q - eq_before : 0u;
      uint32_t k = g + (e < room ? e : room);       // kept pairs of block j
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) k += __shfl_xor(k, o);
      kept += k;
      eqs += __shfl(ei, 63);
    }
    if (tid == 0) { s_base[0] = kept; s_base[1] = eqs; }
  }
  __syncthreads();
  const uint32_t base_kept = s_base[0], base_eq = s_base[1];
  const uint32_t* sc = reinterpret_cast<const uint32_t*>(a.scores) + (size_t)unit * a.n;
  const long long i0 = (long long)blk * kSelBlock + (long long)tid * kSelPer;
  uint32_t u[kSelPer];
  uint32_t eq = 0;
#pragma unroll
  for (int j = 0; j < kSelPer; ++j) u[j] = sc[min(i0 + j, a.n - 1)];
#pragma unroll
  for (int j = 0; j < kSelPer; ++j) eq += (i0 + j < a.n) && u[j] == T;
  uint32_t tot;
  uint32_t eq_before = base_eq + block_excl_scan(eq, s_tmp, &tot);
  uint32_t keepmask = 0, nk = 0;
#pragma unroll
  for (int j = 0; j < kSelPer; ++j) {
    bool in = i0 + j < a.n;
    bool k = in && (u[j] > T || (u[j] == T && eq_before < q));
    if (in && u[j] == T) ++eq_before;
    keepmask |= (uint32_t)k << j;
    nk += k;
  }
  // kept positions of the block are gathered in LDS and written out as one contiguous run
  uint32_t lp = block_excl_scan(nk, s_tmp, &tot);
#pragma unroll
  for (int j = 0; j < kSelPer; ++j)
    if ((keepmask >> j) & 1u) s_idx[lp++] = (int32_t)(i0 + j);
  __syncthreads();
  int32_t* out = a.idx + (size_t)unit * a.n_keep;
  for (uint32_t t = tid; t < tot; t += kSelThreads)
    if (base_kept + t < a.n_keep) out[base_kept + t] = s_idx[t];
}

// ---------------------------------------------------------------------------------------
// Short heads (n <= kSelSmallMax): the whole head fits in LDS, so one workgroup per unit does
// all of the above in one launch -- scores are read from memory once, the three histograms and
// the emit pass work on the LDS copy.  Same result as the multi-launch path, bit for bit.
constexpr int kSelSmallThreads = 1024;

// exclusive scan of one value per thread over the 1024 threads of the workgroup
__device__ uint32_t block_excl_scan_1024(uint32_t v, uint32_t* s_w, uint32_t* total) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint32_t incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  __syncthreads();                       // s_w may still be read from an earlier call
  if (lane == 63) s_w[wave] = incl;
  __syncthreads();
  uint32_t before = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kSelSmallThreads / 64; ++w) {
    const uint32_t t = s_w[w];
    before += w < wave ? t : 0u;
    tot += t;
  }
  *total = tot;
  return before + incl - v;
}

__global__ __launch_bounds__(kSelSmallThreads) void k_sel_small(SelArgs a) {
  extern __shared__ __align__(16) uint32_t s_dyn[];
  __shared__ uint32_t s_w[kSelSmallThreads / 64];
  __shared__ uint32_t s_res[2];
  const int tid = threadIdx.x, lane = tid & 63, unit = blockIdx.x, n = (int)a.n;
  uint32_t* s_hist = s_dyn;                       // [2048]
  uint32_t* s_sc = s_dyn + kSelBins;              // [n] score bit patterns
  const uint32_t* sc = reinterpret_cast<const uint32_t*>(a.scores) + (size_t)unit * a.n;

  uint32_t prefix = 0, rem = a.n_keep;
#pragma unroll
  for (int P = 0; P < 3; ++P) {
    for (int i = tid; i < kSelBins; i += kSelSmallThreads) s_hist[i] = 0;
    __syncthreads();
    // eight scores per thread at a time, all their loads issued before the first is used
    for (int i0 = tid; i0 < n; i0 += 8 * kSelSmallThreads) {
      uint32_t uu[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int i = min(i0 + e * kSelSmallThreads, n - 1);
        uu[e] = P == 0 ? sc[i] : s_sc[i];
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int i = i0 + e * kSelSmallThreads;
        if (i < n) {
          const uint32_t u = uu[e];
          if (P == 0) {
            s_sc[i] = u;
            atomicAdd(&s_hist[u >> 21], 1u);
            if (u > 0x7f800000u) atomicOr(a.hist + 2 * kSelBins + kStatusSlot, kStatusBadScore);
          }
          if (P == 1 && (u >> 21) == prefix) atomicAdd(&s_hist[(u >> 10) & 2047u], 1u);
          if (P == 2 && (u >> 10) == prefix) atomicAdd(&s_hist[u & 1023u], 1u);
        }
      }
    }
    __syncthreads();
    if (tid < 64) {
      uint32_t r;
      const int b = find_bin_wave(s_hist, P == 2 ? 1024 : 2048, rem, &r, lane);
      if (lane == 0) { s_res[0] = (prefix << (P == 2 ? 10 : 11)) | (uint32_t)b; s_res[1] = r; }
    }
    __syncthreads();
    prefix = s_res[0];
    rem = s_res[1];
    __syncthreads();
  }
  const uint32_t T = prefix, q = rem;             // threshold pattern, ties at T to keep

  // every thread owns a contiguous run of positions, so "first q ties by index" is a scan
  const int per = (n + kSelSmallThreads - 1) / kSelSmallThreads;
  const int i0 = min(tid * per, n), i1 = min(i0 + per, n);
  uint32_t gt = 0, eq = 0;
  for (int i = i0; i < i1; ++i) {
    const uint32_t u = s_sc[i];
    gt += u > T;
    eq += u == T;
  }
  uint32_t tot;
  uint32_t eq_before = block_excl_scan_1024(eq, s_w, &tot);
  const uint32_t room = q > eq_before ? q - eq_before : 0u;
  uint32_t pos = block_excl_scan_1024(gt + (eq < room ? eq : room), s_w, &tot);
  int32_t* out = a.idx + (size_t)unit * a.n_keep;
  for (int i = i0; i < i1; ++i) {
    const uint32_t u = s_sc[i];
    const bool k = u > T || (u == T && eq_before < q);
    if (u == T) ++eq_before;
    if (k) {
      if (pos < a.n_keep) out[pos] = (int32_t)i;
      ++pos;
    }
  }
}

hipError_t launch_select(const Dims& d, const float* scores, int64_t n, int64_t n_keep, int32_t* idx,
                         uint32_t* hist, uint32_t* blk, bool hist0_done, hipStream_t st) {
  SelArgs a;
  a.scores = scores;
  a.n = n;
  a.n_keep = (uint32_t)n_keep;
  a.hist = hist;
  a.blk = blk;
  a.idx = idx;
  a.nblk = (int)((n + kSelBlock - 1) / kSelBlock);
  if (select_in_one_launch(n)) {
    const size_t lds = ((size_t)kSelBins + (size_t)n + 4) * sizeof(uint32_t);
    static LdsOptIn opt;
    hipError_t e = opt.ensure(reinterpret_cast<const void*>(k_sel_small),
                              ((size_t)kSelBins + (size_t)kSelSmallMax + 4) * sizeof(uint32_t));
    if (e != hipSuccess) return e;
    k_sel_small<<<d.units(), kSelSmallThreads, lds, st>>>(a);
    return hipGetLastError();
  }
  dim3 grid(d.units(), a.nblk);
  if (!hist0_done) k_sel_hist<0><<<grid, kSelThreads, 0, st>>>(a);
  k_sel_hist<1><<<grid, kSelThreads, 0, st>>>(a);
  k_sel_hist<2><<<grid, kSelThreads, 0, st>>>(a);
  k_sel_count<<<grid, kSelThreads, 0, st>>>(a);
  k_sel_emit<<<grid, kSelThreads, 0, st>>>(a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Head-adaptive budgets (Sec. 2.2, "Head-Adaptive Compression"): the selection runs once over the
// pooled scores of a layer's KV heads, [H][n] read as one list of H*n, after every head's own
// `floor` best pairs have been lifted to +inf so that the pooled selection takes them first.
__global__ void k_mark_inf(float* __restrict__ scores, const int32_t* __restrict__ idx, long long n,
                           long long n_mark) {
  const long long j = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const int unit = blockIdx.y;
  if (j < n_mark) scores[(size_t)unit * n + idx[(size_t)unit * n_mark + j]] = INFINITY;
}

hipError_t launch_mark_inf(float* scores, const int32_t* idx, int units, int64_t n, int64_t n_mark, hipStream_t st) {
  if (n_mark == 0) return hipSuccess;
  dim3 grid((unsigned)((n_mark + 255) / 256), units);
  k_mark_inf<<<grid, 256, 0, st>>>(scores, idx, n, n_mark);
  return hipGetLastError();
}

// kSplitChunks workgroups per (sequence, head): the head's stretch of the pooled ascending list is
// found by two binary searches (every workgroup repeats them: forty loads), then copied with the
// head's offset taken off, each workgroup one slice of it.
constexpr int kSplitChunks = 32;
__global__ __launch_bounds__(256) void k_split_pooled(const int32_t* __restrict__ flat, int H, long long n,
                                                      long long n_keep, int32_t* __restrict__ idx,
                                                      int32_t* __restrict__ lengths) {
  const int b = blockIdx.x / H, h = blockIdx.x % H, chunk = blockIdx.y;
  const long long total = (long long)H * n_keep;
  const int32_t* f = flat + (size_t)b * total;
  auto lower = [&](long long key) {
    long long lo = 0, hi = total;
    while (lo < hi) {
      const long long mid = (lo + hi) >> 1;
      if (f[mid] < key) lo = mid + 1; else hi = mid;
    }
    return lo;
  };
  const long long lo = lower((long long)h * n), hi = lower((long long)(h + 1) * n);
  if (threadIdx.x == 0 && chunk == 0) lengths[blockIdx.x] = (int32_t)(hi - lo);
  int32_t* out = idx + (size_t)blockIdx.x * n;
  const long long per = (hi - lo + kSplitChunks - 1) / kSplitChunks;
  const long long j0 = lo + chunk * per, j1 = min(hi, j0 + per);
  for (long long j = j0 + threadIdx.x; j < j1; j += 256) out[j - lo] = f[j] - (int32_t)(h * n);
}

hipError_t launch_split_pooled(const int32_t* flat, int B, int H, int64_t n, int64_t n_keep, int32_t* idx,
                               int32_t* lengths, hipStream_t st) {
  k_split_pooled<<<dim3(B * H, kSplitChunks), 256, 0, st>>>(flat, H, n, n_keep, idx, lengths);
  return hipGetLastError();
}

}  // namespace ea
