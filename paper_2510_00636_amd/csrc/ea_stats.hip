// Query statistics (Eq. 5-6) and the conversion of (mu, Sigma) into matrix-core operands.
//
// The window queries are mapped by one linear map per (sample, channel pair),
//     u~_s = R-bar R(p_s)^T q_s ,
// and mu = mean_s u~_s, Sigma = cov_s u~_s.  This equals R-bar m and R-bar S R-bar^T of
// Eq. 6 because mean and covariance commute with a fixed linear map; it lets one kernel
// produce Sigma directly.  Angles and the averaged rotation are evaluated in fp64: at
// position 1e5 an fp32 angle is already off by ~1e-2 rad.
#include <hip/hip_runtime.h>

#include "ea_kernels.h"

namespace ea {

// ---------------------------------------------------------------------------------------
// tab[s][c] = (A, Bc): the 2x2 block  [[A, -Bc], [Bc, A]] = R-bar_c * Rot(-p_s theta_c).
// R-bar_c = mean_{j<T} Rot((t_next + j) theta_c) has the closed form of a Dirichlet kernel:
//   mean_j exp(i (t_next + j) theta) = exp(i theta (t_next + (T-1)/2)) sin(T theta/2) / (T sin(theta/2)).
__global__ void k_rope_table(const double* __restrict__ inv_freq, long long q_pos0,
                             long long t_next, int T, int w, int half, int q_is_rotated,
                             float2* __restrict__ tab) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= w * half) return;
  int s = i / half, c = i - s * half;
  double th = inv_freq[c];
  double sh = sin(0.5 * th);
  double cb, sb;
  if (T == 1 || fabs(sh) < 1e-300) {
    sincos(th * (double)t_next, &sb, &cb);
  } else {
    double amp = sin(0.5 * th * (double)T) / ((double)T * sh);
    double ph = th * ((double)t_next + 0.5 * (double)(T - 1));
    sincos(ph, &sb, &cb);
    cb *= amp;
    sb *= amp;
  }
  double ca = 1.0, sa = 0.0;
  if (q_is_rotated) sincos(th * (double)(q_pos0 + s), &sa, &ca);
  tab[i] = make_float2((float)(cb * ca + sb * sa), (float)(sb * ca - cb * sa));
}

__device__ __forceinline__ float load_q(const void* q, size_t i, int dtype) {
  if (dtype == EA_BF16) return __uint_as_float((uint32_t)((const uint16_t*)q)[i] << 16);
  return ((const float*)q)[i];
}

// ---------------------------------------------------------------------------------------
// One workgroup = 16 rows of one head's Sigma.  Pass 1 forms the mean of the transformed
// samples; pass 2 walks the window in chunks of SC samples staged (centred) in LDS and
// accumulates the outer products in fp32.
constexpr int kStatsRB = 16;   // Sigma rows per workgroup
constexpr int kStatsSC = 32;   // samples per LDS chunk

template <int D>
__global__ __launch_bounds__(256) void k_stats(const void* __restrict__ q_win, int dtype,
                                               int w, int layout, int ddof,
                                               const float2* __restrict__ tab,
                                               float* __restrict__ mu,
                                               float* __restrict__ sigma) {
  constexpr int HALF = D / 2;
  constexpr int NGRP = 256 / HALF;            // thread groups over channel pairs
  constexpr int RG = 256 / D;                 // row groups in the accumulation phase
  constexpr int NO = kStatsRB / RG;           // Sigma rows per thread
  __shared__ float s_mean[D];
  __shared__ float s_part[NGRP][D];
  __shared__ __align__(16) float s_u[kStatsSC][D];

  const int head = blockIdx.x, rb = blockIdx.y, tid = threadIdx.x;
  const size_t qbase = (size_t)head * w * D;
  const int c = tid % HALF, grp = tid / HALF;
  const int ia = layout ? 2 * c : c, ib = layout ? 2 * c + 1 : c + HALF;

  // pass 1: column sums of the transformed samples
  float sa = 0.f, sb = 0.f;
  for (int s = grp; s < w; s += NGRP) {
    float2 t = tab[s * HALF + c];
    float qa = load_q(q_win, qbase + (size_t)s * D + ia, dtype);
    float qb = load_q(q_win, qbase + (size_t)s * D + ib, dtype);
    sa += t.x * qa - t.y * qb;
    sb += t.y * qa + t.x * qb;
  }
  s_part[grp][ia] = sa;
  s_part[grp][ib] = sb;
  __syncthreads();
  if (tid < D) {
    float m = 0.f;
    for (int g = 0; g < NGRP; ++g) m += s_part[g][tid];
    m /= (float)w;
    s_mean[tid] = m;
    if (rb == 0) mu[(size_t)head * D + tid] = m;
  }
  __syncthreads();

  // pass 2: centred outer products
  const int j = tid % D, rg = tid / D;
  const int i0 = rb * kStatsRB + rg * NO;
  float acc[NO];
#pragma unroll
  for (int o = 0; o < NO; ++o) acc[o] = 0.f;
  for (int s0 = 0; s0 < w; s0 += kStatsSC) {
    const int ns = min(kStatsSC, w - s0);
    for (int e = tid; e < ns * HALF; e += 256) {
      int sl = e / HALF, cc = e - sl * HALF;
      int ja = layout ? 2 * cc : cc, jb = layout ? 2 * cc + 1 : cc + HALF;
      int s = s0 + sl;
      float2 t = tab[s * HALF + cc];
      float qa = load_q(q_win, qbase + (size_t)s * D + ja, dtype);
      float qb = load_q(q_win, qbase + (size_t)s * D + jb, dtype);
      s_u[sl][ja] = t.x * qa - t.y * qb - s_mean[ja];
      s_u[sl][jb] = t.y * qa + t.x * qb - s_mean[jb];
    }
    __syncthreads();
    for (int sl = 0; sl < ns; ++sl) {
      float xj = s_u[sl][j];
#pragma unroll
      for (int o = 0; o < NO; ++o) acc[o] = fmaf(s_u[sl][i0 + o], xj, acc[o]);
    }
    __syncthreads();
  }
  const float inv = 1.0f / (float)(w - ddof);
#pragma unroll
  for (int o = 0; o < NO; ++o)
    sigma[((size_t)head * D + i0 + o) * D + j] = acc[o] * inv;
}

// ---------------------------------------------------------------------------------------
// Matrix-core operands for the score kernel, one workgroup per (unit, pass).
//
// The quadratic form k^T Sigma k is evaluated as sum_j (sum_c k_c M[c][j]) k_j where M folds
// the symmetric pair (c, j) and (j, c) onto one side at the granularity of 16-channel
// "folded blocks" fb(c) = (c mod d/2) / 16:  M[c][j] = Sigma[c][j] + Sigma[j][c] when
// fb(c) < fb(j), Sigma[c][j] when fb(c) == fb(j), and 0 otherwise -- the zero blocks are
// simply not stored, which removes 3/8 of the matrix-core work.  M is scaled by a power of
// two into fp16 range and rounded to fp16; the rounding error of its diagonal (the dominant
// error term, since k_c^2 never cancels) is kept as a residual row that multiplies k_c^2 in
// an extra accumulator tile.  mu is split into an fp16 head and tail in the same tile.
//
// Fragment (1 KiB = 64 lanes x 8 halves) for (head g, output tile jt, k-step kt):
//   lane l (rho = l % 32, hl = l / 32), element i:
//     input channel   c_in  = hl * d/2 + kt * 8 + i
//     output channel  c_out = ((rho / 4) % 2) * d/2 + jt * 16 + 4 * (rho / 8) + rho % 4
// so that in the 32x32 accumulator layout a lane (hh = l / 32) holds exactly the output
// channels hh * d/2 + x that it also feeds as inputs: the epilogue dot with k needs no
// data movement.
__device__ __forceinline__ float scale_for(float maxabs) {
  if (!(maxabs > 0.f) || !isfinite(maxabs)) return 1.0f;
  int e;
  frexpf(maxabs, &e);                 // maxabs = f * 2^e, f in [0.5, 1)
  int sh = 13 - e;                    // scaled max in [2^12, 2^13)
  sh = max(-100, min(100, sh));
  return ldexpf(1.0f, sh);
}

constexpr int kPrepSplit = 16;   // workgroups per (unit, pass)

template <int D>
__global__ __launch_bounds__(256) void k_prep_frags(const float* __restrict__ mu,
                                                    const float* __restrict__ sigma, int G,
                                                    int GH, int passes, int nfrag,
                                                    uint4* __restrict__ frags,
                                                    float* __restrict__ post) {
  constexpr int HALF = D / 2, NKS = D / 16, NJT = D / 32, NF = NJT * (NJT + 1);
  __shared__ float s_scale[16];       // [2g] = sM, [2g+1] = smu   (GH <= 8)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int unit = blockIdx.x / passes, pass = blockIdx.x % passes;
  const int g0 = pass * GH;
  // Per-head scales, one wavefront per head.  Sigma is a covariance matrix, so
  // |Sigma[a][b]| <= max_c Sigma[c][c]: the diagonal alone bounds every entry of M (<= 2x).
  for (int g = wave; g < GH; g += 4) {
    const int gq = g0 + g;
    float mxS = 0.f, mxM = 0.f;
    if (gq < G) {
      const float* S = sigma + ((size_t)unit * G + gq) * D * D;
      const float* m = mu + ((size_t)unit * G + gq) * D;
      for (int e = lane; e < D; e += 64) {
        mxS = fmaxf(mxS, fabsf(S[(size_t)e * D + e]));
        mxM = fmaxf(mxM, fabsf(m[e]));
      }
    }
    for (int o = 32; o >= 1; o >>= 1) {
      mxS = fmaxf(mxS, __shfl_xor(mxS, o));
      mxM = fmaxf(mxM, __shfl_xor(mxM, o));
    }
    if (lane == 0) {
      const float sM = scale_for(2.0f * mxS), sm = scale_for(mxM);
      s_scale[2 * g] = sM;
      s_scale[2 * g + 1] = sm;
      if (gq < G && blockIdx.y == 0) {
        post[((size_t)unit * G + gq) * 2 + 0] = 1.0f / (2.0f * (float)D * sM);
        post[((size_t)unit * G + gq) * 2 + 1] = 1.0f / (sqrtf((float)D) * sm);
      }
    }
  }
  __syncthreads();

  uint4* out = frags + ((size_t)unit * passes + pass) * nfrag * 64;
  for (int item = blockIdx.y * 256 + tid; item < nfrag * 64; item += kPrepSplit * 256) {
    const int f = item >> 6, l = item & 63;
    const int rho = l & 31, hl = l >> 5;
    _Float16 h[8];
    if (f < GH * NF) {
      const int g = f / NF;
      int rem = f - g * NF, jt = 0;
      while (rem >= 2 * jt + 2) { rem -= 2 * jt + 2; ++jt; }
      const int kt = rem;
      const int gq = g0 + g;
      const int c_out = ((rho >> 2) & 1) * HALF + jt * 16 + 4 * (rho >> 3) + (rho & 3);
      const int c_in0 = hl * HALF + kt * 8;
      const float sM = s_scale[2 * g];
      const float* S = sigma + ((size_t)unit * G + gq) * D * D;
      float val[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) val[i] = 0.f;
      if (gq < G) {
        // the pair (c_in, c_out) and its mirror contribute the same product k_in * k_out, so the
        // contiguous row S[c_out][c_in0 .. c_in0+7] serves for the block on and above the
        // diagonal; blocks strictly above also take the mirrored entries S[c_in][c_out]
        const float4 lo = *reinterpret_cast<const float4*>(S + (size_t)c_out * D + c_in0);
        const float4 hi = *reinterpret_cast<const float4*>(S + (size_t)c_out * D + c_in0 + 4);
        val[0] = lo.x; val[1] = lo.y; val[2] = lo.z; val[3] = lo.w;
        val[4] = hi.x; val[5] = hi.y; val[6] = hi.z; val[7] = hi.w;
        if ((kt >> 1) < jt) {
#pragma unroll
          for (int i = 0; i < 8; ++i) val[i] += S[(size_t)(c_in0 + i) * D + c_out];
        }
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) h[i] = (_Float16)(val[i] * sM);
    } else {
      const int fe = f - GH * NF;
      const bool is_res = fe >= NKS;
      const int kt = is_res ? fe - NKS : fe;
      // rows: [0, GH) mu head, [GH, 2GH) mu tail, [2GH, 3GH) diagonal residual of M
      int g = -1, kind = -1;
      if (!is_res && rho < 2 * GH) { g = rho % GH; kind = rho / GH; }
      if (is_res && rho >= 2 * GH && rho < 3 * GH) { g = rho - 2 * GH; kind = 2; }
      const int gq = g0 + g;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int c_in = hl * HALF + kt * 8 + i;
        float val = 0.f;
        if (g >= 0 && gq < G) {
          if (kind == 2) {
            float m = sigma[(((size_t)unit * G + gq) * D + c_in) * D + c_in] * s_scale[2 * g];
            val = m - (float)(_Float16)m;
          } else {
            float m = mu[((size_t)unit * G + gq) * D + c_in] * s_scale[2 * g + 1];
            float hi = (float)(_Float16)m;
            val = kind == 0 ? hi : m - hi;
          }
        }
        h[i] = (_Float16)val;
      }
    }
    uint4 pk;
    pk.x = (uint32_t)__builtin_bit_cast(uint16_t, h[0]) | ((uint32_t)__builtin_bit_cast(uint16_t, h[1]) << 16);
    pk.y = (uint32_t)__builtin_bit_cast(uint16_t, h[2]) | ((uint32_t)__builtin_bit_cast(uint16_t, h[3]) << 16);
    pk.z = (uint32_t)__builtin_bit_cast(uint16_t, h[4]) | ((uint32_t)__builtin_bit_cast(uint16_t, h[5]) << 16);
    pk.w = (uint32_t)__builtin_bit_cast(uint16_t, h[6]) | ((uint32_t)__builtin_bit_cast(uint16_t, h[7]) << 16);
    out[item] = pk;
  }
}

// ---------------------------------------------------------------------------------------
hipError_t launch_rope_table(const Dims& d, const double* inv_freq, int64_t q_pos0, int64_t t_next,
                             int w, float2* tab, hipStream_t st) {
  int total = w * d.half;
  k_rope_table<<<(total + 255) / 256, 256, 0, st>>>(inv_freq, q_pos0, t_next, d.T, w, d.half,
                                                    d.q_is_rotated, tab);
  return hipGetLastError();
}

hipError_t launch_stats(const Dims& d, const void* q_win, int w, const float2* tab, float* mu,
                        float* sigma, hipStream_t st) {
  dim3 grid(d.qheads(), d.D / kStatsRB);
  if (d.D == 64)
    k_stats<64><<<grid, 256, 0, st>>>(q_win, d.dtype, w, d.rope_layout, d.ddof, tab, mu, sigma);
  else if (d.D == 128)
    k_stats<128><<<grid, 256, 0, st>>>(q_win, d.dtype, w, d.rope_layout, d.ddof, tab, mu, sigma);
  else
    k_stats<256><<<grid, 256, 0, st>>>(q_win, d.dtype, w, d.rope_layout, d.ddof, tab, mu, sigma);
  return hipGetLastError();
}

hipError_t launch_prep_frags(const Dims& d, const ScorePlan& sp, const float* mu,
                             const float* sigma, uint4* frags, float* post, hipStream_t st) {
  dim3 grid(d.units() * sp.passes, kPrepSplit);
  if (d.D == 64)
    k_prep_frags<64><<<grid, 256, 0, st>>>(mu, sigma, d.G, sp.GH, sp.passes, sp.nfrag, frags, post);
  else if (d.D == 128)
    k_prep_frags<128><<<grid, 256, 0, st>>>(mu, sigma, d.G, sp.GH, sp.passes, sp.nfrag, frags, post);
  else
    k_prep_frags<256><<<grid, 256, 0, st>>>(mu, sigma, d.G, sp.GH, sp.passes, sp.nfrag, frags, post);
  return hipGetLastError();
}

}  // namespace ea
