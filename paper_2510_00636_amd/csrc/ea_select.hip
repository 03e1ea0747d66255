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

__global__ void k_zero(uint32_t* p, size_t count) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) p[i] = 0;
}

hipError_t launch_zero(uint32_t* p, size_t count, hipStream_t st) {
  if (count == 0) return hipSuccess;
  k_zero<<<(unsigned)((count + 255) / 256), 256, 0, st>>>(p, count);
  return hipGetLastError();
}

// Bin b (counting down from the top) with  count(bins > b) < target <= count(bins >= b);
// *rem = target - count(bins > b).  All 256 threads call it; result is uniform.
// hist has nbins (multiple of 256, <= 2048) entries; s_tmp holds 257 words.
__device__ int find_bin(const uint32_t* __restrict__ hist, int nbins, uint32_t target,
                        uint32_t* rem, uint32_t* s_tmp) {
  const int tid = threadIdx.x;
  const int per = nbins / kSelThreads;
  // thread t owns bins [nbins - per*(t+1), nbins - per*t): descending order across threads
  const int hi = nbins - per * tid;
  uint32_t loc[8];
  uint32_t sum = 0;
  for (int j = 0; j < per; ++j) { loc[j] = hist[hi - 1 - j]; sum += loc[j]; }
  __syncthreads();
  s_tmp[tid] = sum;
  __syncthreads();
  // inclusive scan over threads (Hillis-Steele)
  for (int o = 1; o < kSelThreads; o <<= 1) {
    uint32_t add = tid >= o ? s_tmp[tid - o] : 0;
    __syncthreads();
    s_tmp[tid] += add;
    __syncthreads();
  }
  const uint32_t incl = s_tmp[tid], excl = incl - sum;
  if (excl < target && target <= incl) {
    uint32_t cum = excl;
    int b = hi - 1;
    for (int j = 0; j < per; ++j) {
      if (target <= cum + loc[j]) { b = hi - 1 - j; break; }
      cum += loc[j];
    }
    s_tmp[256] = (uint32_t)b;
    s_tmp[257] = target - cum;
  }
  __syncthreads();
  const int b = (int)s_tmp[256];
  *rem = s_tmp[257];
  __syncthreads();
  return b;
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

// Digits already fixed before pass P; returns true prefix for matching and the remaining rank.
template <int P>
__device__ void resolve(const SelArgs& a, int unit, uint32_t* s_tmp, uint32_t* prefix, uint32_t* rem) {
  const uint32_t* h = a.hist + (size_t)unit * 3 * kSelBins;
  uint32_t r = a.n_keep, pre = 0;
  if (P >= 1) { int b0 = find_bin(h, 2048, r, &r, s_tmp); pre = (uint32_t)b0; }
  if (P >= 2) { int b1 = find_bin(h + kSelBins, 2048, r, &r, s_tmp); pre = (pre << 11) | (uint32_t)b1; }
  if (P >= 3) { int b2 = find_bin(h + 2 * kSelBins, 1024, r, &r, s_tmp); pre = (pre << 10) | (uint32_t)b2; }
  *prefix = pre;
  *rem = r;
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
  for (int j = 0; j < kSelPer; ++j) {
    const long long i = base + j * kSelThreads + tid;
    if (i < a.n) {
      const uint32_t u = sc[i];
      if (P == 0) atomicAdd(&s_hist[u >> 21], 1u);
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
  for (int j = 0; j < kSelPer; ++j) {
    const long long i = base + j * kSelThreads + tid;
    if (i < a.n) {
      const uint32_t u = sc[i];
      gt += u > T;
      eq += u == T;
    }
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

// exclusive scan of one value per thread over the 256 threads of the workgroup
__device__ uint32_t block_excl_scan(uint32_t v, uint32_t* s_tmp, uint32_t* total) {
  const int tid = threadIdx.x;
  __syncthreads();
  s_tmp[tid] = v;
  __syncthreads();
  for (int o = 1; o < kSelThreads; o <<= 1) {
    uint32_t add = tid >= o ? s_tmp[tid - o] : 0;
    __syncthreads();
    s_tmp[tid] += add;
    __syncthreads();
  }
  const uint32_t incl = s_tmp[tid];
  *total = s_tmp[kSelThreads - 1];
  __syncthreads();
  return incl - v;
}

__global__ __launch_bounds__(kSelThreads) void k_sel_emit(SelArgs a) {
  __shared__ uint32_t s_tmp[258];
  __shared__ uint32_t s_base[2];
  const int tid = threadIdx.x, unit = blockIdx.x, blk = blockIdx.y;
  const uint32_t* slot = a.hist + ((size_t)unit * 3 + 2) * kSelBins + 1024;
  const uint32_t T = slot[0], q = slot[1];
  if (tid == 0) {
    // kept pairs and ==T pairs in the blocks before this one
    uint32_t kept = 0, eqs = 0;
    const uint32_t* b = a.blk + (size_t)unit * a.nblk * 2;
    for (int j = 0; j < blk; ++j) {
      const uint32_t g = b[2 * j], e = b[2 * j + 1];
      const uint32_t room = q > eqs ? q - eqs : 0;
      kept += g + (e < room ? e : room);
      eqs += e;
    }
    s_base[0] = kept;
    s_base[1] = eqs;
  }
  __syncthreads();
  const uint32_t base_kept = s_base[0], base_eq = s_base[1];
  const uint32_t* sc = reinterpret_cast<const uint32_t*>(a.scores) + (size_t)unit * a.n;
  const long long i0 = (long long)blk * kSelBlock + (long long)tid * kSelPer;
  uint32_t u[kSelPer];
  uint32_t eq = 0;
#pragma unroll
  for (int j = 0; j < kSelPer; ++j) {
    u[j] = (i0 + j < a.n) ? sc[i0 + j] : 0u;
    eq += (i0 + j < a.n) && u[j] == T;
  }
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
  uint32_t pos = base_kept + block_excl_scan(nk, s_tmp, &tot);
  int32_t* out = a.idx + (size_t)unit * a.n_keep;
#pragma unroll
  for (int j = 0; j < kSelPer; ++j)
    if ((keepmask >> j) & 1u) {
      if (pos < a.n_keep) out[pos] = (int32_t)(i0 + j);
      ++pos;
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
  dim3 grid(d.units(), a.nblk);
  if (!hist0_done) k_sel_hist<0><<<grid, kSelThreads, 0, st>>>(a);
  k_sel_hist<1><<<grid, kSelThreads, 0, st>>>(a);
  k_sel_hist<2><<<grid, kSelThreads, 0, st>>>(a);
  k_sel_count<<<grid, kSelThreads, 0, st>>>(a);
  k_sel_emit<<<grid, kSelThreads, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace ea
