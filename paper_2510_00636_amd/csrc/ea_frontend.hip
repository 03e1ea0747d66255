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

// The same projection on the matrix cores, for bf16 inputs whose rows are 16-byte aligned
// (d_model a multiple of 8): one workgroup = a 32 (samples) x 32 (channels) tile, its operands
// read straight from global memory in the layout v_mfma_f32_32x32x16_bf16 takes them -- lane
// (r, hh) = (lane % 32, lane / 32) holds 8 consecutive d_model entries of row r, of the hidden
// states as A operand and of W_Q as B operand; the instruction does not care which 16 of the
// d_model entries it is given as long as both operands agree, so per block of 64 entries half hh
// takes the 32 contiguous ones at 32 hh (64 contiguous bytes per lane, 128 per row) and the block
// is four instructions.  The four wavefronts split the d_model axis into four contiguous quarters
// (a short dependent chain each, 2048 wavefronts in flight at the Llama-8B shape); the four partial
// tiles meet in LDS and are added in wavefront order, so the result does not depend on timing.
// bf16 products are exact in fp32.
typedef __bf16 pj_bf16x8 __attribute__((ext_vector_type(8)));
typedef float pj_floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t pj_u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void k_project_mfma(const uint16_t* __restrict__ hidden,
                                                      const uint16_t* __restrict__ wq, int w, int dm, int D, int Hq,
                                                      float* __restrict__ q) {
  __shared__ float s_acc[4][16][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 31, hh = lane >> 5;
  const int t0 = blockIdx.x * 32, b = blockIdx.z;
  const int g = (blockIdx.y * 32) / D, c0 = (blockIdx.y * 32) % D;
  const int kq = ((dm + 255) / 256) * 64;               // entries per wavefront, a multiple of the block
  const int kbeg = wave * kq, kend = min(dm, kbeg + kq);
  const uint16_t* arow = hidden + ((size_t)b * w + min(t0 + r, w - 1)) * dm + hh * 32;
  const uint16_t* brow = wq + ((size_t)g * D + c0 + r) * dm + hh * 32;
  pj_floatx16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  const pj_u32x4 zero4 = {0u, 0u, 0u, 0u};
  auto fetch = [&](int k0, pj_u32x4 (&a)[4], pj_u32x4 (&bq)[4]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int kk = k0 + hh * 32 + j * 8;              // d_model % 8 == 0: a chunk lies inside the row or outside
      const bool ok = kk < kend;                        // (kend - kbeg is a multiple of 8 as well)
      a[j] = ok ? *reinterpret_cast<const pj_u32x4*>(arow + k0 + j * 8) : zero4;
      bq[j] = ok ? *reinterpret_cast<const pj_u32x4*>(brow + k0 + j * 8) : zero4;
    }
  };
  pj_u32x4 a0[4], b0[4], a1[4], b1[4];
  fetch(kbeg, a0, b0);
  for (int k0 = kbeg; k0 < kend; k0 += 128) {
    fetch(k0 + 64, a1, b1);                             // (past the end: all chunks are zeros, nothing is read)
#pragma unroll
    for (int j = 0; j < 4; ++j)
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(pj_bf16x8, a0[j]),
                                                    __builtin_bit_cast(pj_bf16x8, b0[j]), acc, 0, 0, 0);
    fetch(k0 + 128, a0, b0);
#pragma unroll
    for (int j = 0; j < 4; ++j)
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(pj_bf16x8, a1[j]),
                                                    __builtin_bit_cast(pj_bf16x8, b1[j]), acc, 0, 0, 0);
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) s_acc[wave][v][lane] = acc[v];
  __syncthreads();
  // accumulator register v of lane (r, hh) is the tile's entry (row 8 (v / 4) + 4 hh + v % 4, column r);
  // wavefront i adds and stores registers 4 i .. 4 i + 3
  float* out = q + (((size_t)b * Hq + g) * w) * D + c0 + r;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int v = 4 * wave + i;
    const float sum = ((s_acc[0][v][lane] + s_acc[1][v][lane]) + s_acc[2][v][lane]) + s_acc[3][v][lane];
    const int t = t0 + 8 * wave + 4 * hh + i;
    if (t < w) out[(size_t)t * D] = sum;
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
  if (d.dtype == EA_BF16 && dm % 8 == 0 && ((uintptr_t)hidden % 16) == 0 && ((uintptr_t)wq % 16) == 0) {
    dim3 gm((w + 31) / 32, d.Hq * d.D / 32, d.B);
    k_project_mfma<<<gm, 256, 0, st>>>((const uint16_t*)hidden, (const uint16_t*)wq, w, dm, d.D, d.Hq, q);
    return hipGetLastError();
  }
  dim3 grid((w + 31) / 32, d.D / 32, d.qheads());
  if (d.dtype == EA_BF16)
    k_project<true><<<grid, 256, 0, st>>>(hidden, wq, w, dm, d.D, d.Hq, q);
  else
    k_project<false><<<grid, 256, 0, st>>>(hidden, wq, w, dm, d.D, d.Hq, q);
  return hipGetLastError();
}

}  // namespace ea
