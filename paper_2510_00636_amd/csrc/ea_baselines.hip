// The cheap scorers the paper compares against in its decoding experiments (Sec. 3.1,
// "Baselines"), written from the one sentence it gives each, so that they can be measured on the
// same select + compact back half as Expected Attention:
//   KNorm         keeps the keys of lowest L2 norm              score = 1 / ||k_i||
//   StreamingLLM  keeps the initial sink tokens (and, with the rest of the budget, the most
//                 recent pairs)                                 score = +inf (i < n_sink), i + 1
//   KeyDiff       a distance between key embeddings             score = 1 - cos(k_i, a),
//                 a = mean of the head's unit-normalised keys
// All three read K at most twice and never touch V; sixteen lanes share a key row.
#include <hip/hip_runtime.h>

#include "ea_kernels.h"

namespace ea {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// the lane's share of key row `row`: channels 8*l + 128*j (bf16) or 4*l + 64*j (fp32), l = lane % 16
template <int D, bool BF16>
struct RowPiece {
  static constexpr int NP = BF16 ? (D + 127) / 128 : D / 64;
  static constexpr int W = BF16 ? 8 : 4;
  float x[NP * W];
  __device__ __forceinline__ void load(const void* base, long long row, int l) {
#pragma unroll
    for (int j = 0; j < NP; ++j) {
      const int c0 = W * l + 16 * W * j;
      const bool ok = c0 < D;
      if (BF16) {
        const u32x4 r = ok ? *reinterpret_cast<const u32x4*>((const uint16_t*)base + row * D + c0)
                           : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          x[8 * j + 2 * e] = __uint_as_float(r[e] << 16);
          x[8 * j + 2 * e + 1] = __uint_as_float(r[e] & 0xffff0000u);
        }
      } else {
        const float4 r = *reinterpret_cast<const float4*>((const float*)base + row * D + c0);
        x[4 * j] = r.x; x[4 * j + 1] = r.y; x[4 * j + 2] = r.z; x[4 * j + 3] = r.w;
      }
    }
  }
  __device__ __forceinline__ float sumsq() const {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NP * W; ++i) s = fmaf(x[i], x[i], s);
    return s;
  }
};

// sum over the 16 lanes that share a row (every lane gets the total)
__device__ __forceinline__ float row_sum16(float x) {
  x += __shfl_xor(x, 1);
  x += __shfl_xor(x, 2);
  x += __shfl_xor(x, 4);
  x += __shfl_xor(x, 8);
  return x;
}

constexpr int kBaseRowsPerWg = 128;     // 16 rows at a time, 8 rounds
constexpr int kKeydiffRowsPerWg = 1024; // KeyDiff's second pass: the anchor is rebuilt once per workgroup

template <int D, bool BF16>
__global__ __launch_bounds__(256) void k_knorm(const void* __restrict__ k, long long n, long long n_cap,
                                               int units, float* __restrict__ scores) {
  const int tid = threadIdx.x, l = tid & 15, rw = tid >> 4;
  const int unit = blockIdx.x % units;
  const long long r0 = (long long)(blockIdx.x / units) * kBaseRowsPerWg;
  const char* base = (const char*)k + (size_t)unit * n_cap * D * (BF16 ? 2 : 4);
#pragma unroll
  for (int it = 0; it < kBaseRowsPerWg / 16; ++it) {
    const long long row = r0 + it * 16 + rw;
    RowPiece<D, BF16> p;
    p.load(base, min(row, n - 1), l);
    const float ss = row_sum16(p.sumsq());
    if (l == 0 && row < n) scores[(size_t)unit * n + row] = 1.0f / sqrtf(ss);
  }
}

__global__ void k_streaming(long long n, long long n_sink, int units, float* __restrict__ scores) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const float s = i < n_sink ? INFINITY : (float)(i + 1);
  for (int u = 0; u < units; ++u) scores[(size_t)u * n + i] = s;
}

// KeyDiff pass 1: per (unit, chunk of rows) the sum of the unit-normalised keys, rows taken in a
// fixed order so that the mean, and with it every score, has the same bits on every run.
template <int D, bool BF16>
__global__ __launch_bounds__(256) void k_keydiff_partial(const void* __restrict__ k, long long n,
                                                         long long n_cap, int units, int rows_per_wg,
                                                         float* __restrict__ partial) {
  typedef RowPiece<D, BF16> RP;
  __shared__ float s_acc[16][D];
  const int tid = threadIdx.x, l = tid & 15, rw = tid >> 4;
  const int unit = blockIdx.x % units, chunk = blockIdx.x / units;
  const long long r0 = (long long)chunk * rows_per_wg, r1 = min(r0 + (long long)rows_per_wg, n);
  const char* base = (const char*)k + (size_t)unit * n_cap * D * (BF16 ? 2 : 4);
  float acc[RP::NP * RP::W];
#pragma unroll
  for (int i = 0; i < RP::NP * RP::W; ++i) acc[i] = 0.f;
  // eight rows per lane group in flight; they are added in the order a one-row loop would take them
  constexpr int U = 8;
  for (long long row = r0 + rw; row < r1; row += 16 * U) {
    RP p[U];
#pragma unroll
    for (int u = 0; u < U; ++u) p[u].load(base, min(row + 16 * u, n - 1), l);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (row + 16 * u < r1) {
        const float ss = row_sum16(p[u].sumsq());
        const float inv = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
#pragma unroll
        for (int i = 0; i < RP::NP * RP::W; ++i) acc[i] = fmaf(p[u].x[i], inv, acc[i]);
      }
    }
  }
#pragma unroll
  for (int j = 0; j < RP::NP; ++j)
#pragma unroll
    for (int e = 0; e < RP::W; ++e) {
      const int c = RP::W * l + 16 * RP::W * j + e;
      if (c < D) s_acc[rw][c] = acc[RP::W * j + e];
    }
  __syncthreads();
  for (int c = tid; c < D; c += 256) {
    float s = 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q) s += s_acc[q][c];
    partial[((size_t)unit * gridDim.x / units + chunk) * D + c] = s;
  }
}

// KeyDiff pass 2: the anchor a (partials added in chunk order), then 1 - cos(k_i, a) per row
template <int D, bool BF16>
__global__ __launch_bounds__(256) void k_keydiff_score(const void* __restrict__ k, long long n,
                                                       long long n_cap, int units, int nchunk,
                                                       const float* __restrict__ partial,
                                                       float* __restrict__ scores) {
  typedef RowPiece<D, BF16> RP;
  __shared__ float s_a[D];
  __shared__ float s_inv;
  const int tid = threadIdx.x, l = tid & 15, rw = tid >> 4;
  const int unit = blockIdx.x % units;
  const long long r0 = (long long)(blockIdx.x / units) * kKeydiffRowsPerWg;
  for (int c = tid; c < D; c += 256) {
    float s = 0.f;
    for (int q = 0; q < nchunk; ++q) s += partial[((size_t)unit * nchunk + q) * D + c];
    s_a[c] = s / (float)n;
  }
  __syncthreads();
  if (tid < 64) {
    float ss = 0.f;
    for (int c = tid; c < D; c += 64) ss = fmaf(s_a[c], s_a[c], ss);
    for (int o = 32; o >= 1; o >>= 1) ss += __shfl_xor(ss, o);
    if (tid == 0) s_inv = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
  }
  __syncthreads();
  const float inv_a = s_inv;
  const char* base = (const char*)k + (size_t)unit * n_cap * D * (BF16 ? 2 : 4);
  // the lane's channels of the anchor, once
  float an[RP::NP * RP::W];
#pragma unroll
  for (int j = 0; j < RP::NP; ++j)
#pragma unroll
    for (int e = 0; e < RP::W; ++e) {
      const int c = RP::W * l + 16 * RP::W * j + e;
      an[RP::W * j + e] = c < D ? s_a[c] : 0.f;
    }
  for (int it0 = 0; it0 < kKeydiffRowsPerWg / 16 && r0 + it0 * 16 < n; it0 += 8) {
  RP pp[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) pp[u].load(base, min(r0 + (it0 + u) * 16 + rw, n - 1), l);
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const long long row = r0 + (it0 + u) * 16 + rw;
    const RP& p = pp[u];
    float dot = 0.f;
#pragma unroll
    for (int j = 0; j < RP::NP; ++j)
#pragma unroll
      for (int e = 0; e < RP::W; ++e) {
        const int c = RP::W * l + 16 * RP::W * j + e;
        if (c < D) dot = fmaf(p.x[RP::W * j + e], an[RP::W * j + e], dot);
      }
    const float ss = row_sum16(p.sumsq());
    dot = row_sum16(dot);
    const float cosv = ss > 0.f ? dot * inv_a / sqrtf(ss) : 0.f;
    if (l == 0 && row < n) scores[(size_t)unit * n + row] = 1.0f - cosv;
  }
  }
}

template <int D, bool BF16>
static hipError_t launch_baseline_t(const Dims& d, int kind, const void* k, int64_t n, int64_t n_cap,
                                    float* scores, float* scratch, hipStream_t st) {
  const unsigned nblk = (unsigned)((n + kBaseRowsPerWg - 1) / kBaseRowsPerWg);
  if (kind == EA_SCORER_KNORM) {
    k_knorm<D, BF16><<<nblk * d.units(), 256, 0, st>>>(k, n, n_cap, d.units(), scores);
  } else {
    int nchunk = (int)((n + 4095) / 4096);
    if (nchunk > 256) nchunk = 256;
    const int rows = (int)((n + nchunk - 1) / nchunk);
    nchunk = (int)((n + rows - 1) / rows);
    k_keydiff_partial<D, BF16><<<nchunk * d.units(), 256, 0, st>>>(k, n, n_cap, d.units(), rows, scratch);
    const unsigned nblk2 = (unsigned)((n + kKeydiffRowsPerWg - 1) / kKeydiffRowsPerWg);
    k_keydiff_score<D, BF16><<<nblk2 * d.units(), 256, 0, st>>>(k, n, n_cap, d.units(), nchunk, scratch, scores);
  }
  return hipGetLastError();
}

hipError_t launch_baseline(const Dims& d, int kind, const void* k, int64_t n, int64_t n_cap,
                           int64_t n_sink, float* scores, float* scratch, hipStream_t st) {
  if (kind == EA_SCORER_STREAMING) {
    k_streaming<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(n, n_sink, d.units(), scores);
    return hipGetLastError();
  }
  const bool bf = d.dtype == EA_BF16;
#define EA_BASE(DD)                                                                          \
  if (d.D == DD)                                                                             \
    return bf ? launch_baseline_t<DD, true>(d, kind, k, n, n_cap, scores, scratch, st)       \
              : launch_baseline_t<DD, false>(d, kind, k, n, n_cap, scores, scratch, st);
  EA_BASE(64)
  EA_BASE(128)
  EA_BASE(256)
#undef EA_BASE
  return hipErrorInvalidValue;
}

}  // namespace ea
