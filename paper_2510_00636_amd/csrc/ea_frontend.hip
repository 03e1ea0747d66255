// Eq. 5 of the paper as printed starts from the hidden states: the queries are W_Q h (before the
// rotary embedding), so mean and covariance of the buffered hidden states, pushed through W_Q,
// are mean and covariance of the projected queries.  This file projects the buffer,
//     q[b][g][s][:] = W_Q[g] h[b][s][:]      (fp32 accumulation, fp32 result),
// and the statistics kernel then runs on q as un-rotated fp32 queries.  Forming the d_model x
// d_model covariance of the hidden states first, as the equation is written, would cost
// d_model / d times the arithmetic for the same result.
#include <hip/hip_runtime.h>

#include "ea_kernels.h"

namespace ea {

template <bool BF16>
__device__ __forceinline__ float load_elem(const void* p, size_t i) {
  if (BF16) return __uint_as_float((uint32_t)((const uint16_t*)p)[i] << 16);
  return ((const float*)p)[i];
}

// One workgroup = a 32 (samples) x 32 (channels) tile of one (sequence, query head); the d_model
// axis goes through LDS 32 at a time.  Thread (ty, tx) = (tid / 32, tid % 32) owns outputs
// (s0 + ty + 8 i, c0 + tx), i < 4.
template <bool BF16>
__global__ __launch_bounds__(256) void k_project(const void* __restrict__ hidden, const void* __restrict__ wq,
                                                 int w, int dm, int D, int Hq, float* __restrict__ q) {
  __shared__ float s_h[32][33], s_w[32][33];
  const int tid = threadIdx.x, tx = tid & 31, ty = tid >> 5;
  const int s0 = blockIdx.x * 32, c0 = blockIdx.y * 32;
  const int b = blockIdx.z / Hq, g = blockIdx.z % Hq;
  const size_t hbase = (size_t)b * w * dm, wbase = (size_t)g * D * dm;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int m0 = 0; m0 < dm; m0 += 32) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = ty + 8 * i, m = m0 + tx;
      const int s = min(s0 + row, w - 1);
      s_h[row][tx] = m < dm ? load_elem<BF16>(hidden, hbase + (size_t)s * dm + m) : 0.f;
      s_w[row][tx] = m < dm ? load_elem<BF16>(wq, wbase + (size_t)(c0 + row) * dm + m) : 0.f;
    }
    __syncthreads();
#pragma unroll 8
    for (int m = 0; m < 32; ++m) {
      const float wv = s_w[tx][m];
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = fmaf(s_h[ty + 8 * i][m], wv, acc[i]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int s = s0 + ty + 8 * i;
    if (s < w) q[(((size_t)b * Hq + g) * w + s) * D + c0 + tx] = acc[i];
  }
}

// Eq. 9 as printed weighs a pair by ||W_o v||.  With M_g = W_o^(g)^T W_o^(g) (d x d, from the d
// columns of W_o that query head g feeds) that norm is sqrt(v^T M_g v): a quadratic form of the
// same shape as Eq. 7's, so the score kernels evaluate it.  M_g depends on the weights only and is
// formed once per layer: one workgroup = a 32 x 32 tile of one head's M, the d_model axis through
// LDS 32 rows at a time, fp32 accumulation in row order.
template <bool BF16>
__global__ __launch_bounds__(256) void k_gram(const void* __restrict__ wo, int dm, int D, float* __restrict__ gram) {
  __shared__ float s_a[32][33], s_b[32][33];
  const int tid = threadIdx.x, tx = tid & 31, ty = tid >> 5;
  const int a0 = blockIdx.x * 32, b0 = blockIdx.y * 32, g = blockIdx.z;
  const size_t base = (size_t)g * dm * D;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int m0 = 0; m0 < dm; m0 += 32) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = m0 + ty + 8 * i;
      s_a[ty + 8 * i][tx] = m < dm ? load_elem<BF16>(wo, base + (size_t)m * D + a0 + tx) : 0.f;
      s_b[ty + 8 * i][tx] = m < dm ? load_elem<BF16>(wo, base + (size_t)m * D + b0 + tx) : 0.f;
    }
    __syncthreads();
#pragma unroll 8
    for (int m = 0; m < 32; ++m) {
      const float bv = s_b[m][tx];
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = fmaf(s_a[m][ty + 8 * i], bv, acc[i]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) gram[((size_t)g * D + a0 + ty + 8 * i) * D + b0 + tx] = acc[i];
}

hipError_t launch_gram(const Dims& d, const void* w_o, int dm, float* gram, hipStream_t st) {
  dim3 grid(d.D / 32, d.D / 32, d.Hq);
  if (d.dtype == EA_BF16)
    k_gram<true><<<grid, 256, 0, st>>>(w_o, dm, d.D, gram);
  else
    k_gram<false><<<grid, 256, 0, st>>>(w_o, dm, d.D, gram);
  return hipGetLastError();
}

hipError_t launch_project(const Dims& d, const void* hidden, const void* wq, int w, int dm, float* q,
                          hipStream_t st) {
  dim3 grid((w + 31) / 32, d.D / 32, d.qheads());
  if (d.dtype == EA_BF16)
    k_project<true><<<grid, 256, 0, st>>>(hidden, wq, w, dm, d.D, d.Hq, q);
  else
    k_project<false><<<grid, 256, 0, st>>>(hidden, wq, w, dm, d.D, d.Hq, q);
  return hipGetLastError();
}

}  // namespace ea
