// Scoring kernels: Eq. 7 (expected unnormalised attention, as a logit), Eq. 8 (softmax over
// all cached keys) and Eq. 9 with ||v|| and the GQA group mean.
//
//   pass A  k_score_mfma / k_score_hw / k_score_f32 : stream K and V once; per key the G logits
//           l_g = mu_g.k/sqrt(d) + k^T Sigma_g k/(2d) and ||v||.
//           (max, sum exp) per query head and fixed block of keys: k_score_hw and k_score_f32 keep
//           them on the way, for k_score_mfma k_lse_part takes them from the stored logits.
//   pass B  k_finalize : combine the pairs into log-sum-exp per head, then
//           score = (mean_g exp(l_g - lse_g) + eps) * ||v||.
#include "ea_score_mfma.h"

namespace ea {

hipError_t launch_score_mfma(const Dims& d, const ScorePlan& sp, const void* k, const void* v,
                             int64_t n, int64_t n_cap, const uint4* frags, const float* post,
                             float* logits, float* vnorm, float2* part, uint32_t* tickets,
                             int ticket_stride, hipStream_t st, const PageMap* pm, const float* kscale,
                             const float* vscale, bool skip_v) {
  ScoreArgs a;
  a.skip_v = skip_v ? 1 : 0;
  a.pm = pm ? *pm : PageMap{nullptr, 0, 0, 1, 0};
  a.kscale = kscale;
  a.vscale = vscale;
  a.k = (const u32x4*)k;
  a.v = (const u32x4*)v;
  a.n = n;
  a.n_cap = n_cap;
  a.frags = (const u32x4*)frags;
  a.post = post;
  a.logits = logits;
  a.vnorm = vnorm;
  a.part = part;
  a.G = d.G;
  a.passes = sp.passes;
  a.nchunk = sp.nchunk;
  a.npart = sp.npart;
  a.tpt = sp.tpt;
  a.units = d.units();
  a.nfrag = sp.nfrag;
  a.tickets = tickets;
  a.ticket_stride = ticket_stride;
  if (d.kv_fp8) return launch_score_mfma_fp8(d.D, a, sp, st);
  if (sp.hw) return launch_score_hw(a, sp, st);
  switch (d.D) {
    case 64: return launch_score_mfma_d64(a, sp, st);
    case 128: return sp.GH <= 3 ? launch_score_mfma_d128(a, sp, st) : launch_score_mfma_d128b(a, sp, st);
    case 256: return launch_score_mfma_d256(a, sp, st);
  }
  return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------------
// fp32 caches: everything in fp64 on the vector units (the 1e-5 score tolerance of this
// path leaves no room for fp32 accumulation of a d^2-term quadratic form).  One workgroup
// = (unit, query head, span of keys); 64 keys at a time, K tile in LDS, thread (key, quarter
// of the output channels).
template <int D>
__global__ __launch_bounds__(256) void k_score_f32(const float* __restrict__ k,
                                                   const float* __restrict__ v, long long n,
                                                   long long n_cap, const float* __restrict__ mu,
                                                   const float* __restrict__ sigma, int G, int units,
                                                   int span, int nchunk, double* __restrict__ logits,
                                                   float* __restrict__ vnorm,
                                                   double2* __restrict__ part) {
  constexpr int QW = D / 4;
  extern __shared__ float s_k[];            // [64][D + 1]
  __shared__ double s_red[4][64];
  __shared__ double s_ms[2];
  const int tid = threadIdx.x, r = tid & 63, qd = tid >> 6;
  const int unit = blockIdx.x % units;
  const int t2 = blockIdx.x / units;
  const int gq = t2 % G, chunk = t2 / G;
  const float* S = sigma + ((size_t)unit * G + gq) * D * D;
  const float* M = mu + ((size_t)unit * G + gq) * D;
  const float* kb = k + (size_t)unit * n_cap * D;
  const float* vb = v + (size_t)unit * n_cap * D;
  const long long key_lo = (long long)chunk * span, key_hi = min(key_lo + (long long)span, n);
  double m_run = -INFINITY, s_run = 0.0;   // thread r < 64 of quarter 0 tracks key slot r
  for (long long key0 = key_lo; key0 < key_hi; key0 += 64) {
    __syncthreads();
    for (int e = tid; e < 64 * D; e += 256) {
      int rr = e / D, c = e - rr * D;
      long long row = min(key0 + rr, n - 1);
      s_k[rr * (D + 1) + c] = kb[row * D + c];
    }
    __syncthreads();
    double y[QW];
#pragma unroll
    for (int j = 0; j < QW; ++j) y[j] = 0.0;
    for (int c = 0; c < D; ++c) {
      const double kc = (double)s_k[r * (D + 1) + c];
      const float* Sr = S + (size_t)c * D + qd * QW;
#pragma unroll
      for (int j = 0; j < QW; ++j) y[j] = fma(kc, (double)Sr[j], y[j]);
    }
    double quad = 0.0, lin = 0.0;
#pragma unroll
    for (int j = 0; j < QW; ++j) {
      const double kj = (double)s_k[r * (D + 1) + qd * QW + j];
      quad = fma(y[j], kj, quad);
      lin = fma((double)M[qd * QW + j], kj, lin);
    }
    s_red[qd][r] = lin / sqrt((double)D) + quad / (2.0 * D);
    __syncthreads();
    if (qd == 0 && key0 + r < n) {
      double lg = s_red[0][r] + s_red[1][r] + s_red[2][r] + s_red[3][r];
      logits[((size_t)unit * G + gq) * n + key0 + r] = lg;
      double mn = fmax(m_run, lg);
      s_run = s_run * exp(m_run - mn) + exp(lg - mn);
      m_run = mn;
    }
    if (gq == 0) {   // value norms, once per unit
      __syncthreads();
      long long row = min(key0 + r, n - 1);
      double ss = 0.0;
      for (int j = 0; j < QW; ++j) {
        double x = (double)vb[row * D + qd * QW + j];
        ss = fma(x, x, ss);
      }
      s_red[qd][r] = ss;
      __syncthreads();
      if (qd == 0 && key0 + r < n)
        vnorm[(size_t)unit * n + key0 + r] =
            (float)sqrt(s_red[0][r] + s_red[1][r] + s_red[2][r] + s_red[3][r]);
    }
  }
  // reduce the 64 key slots
  __syncthreads();
  if (qd == 0) {
    double m = m_run, s = s_run;
    for (int o = 32; o >= 1; o >>= 1) {
      double m2 = __shfl_xor(m, o), s2 = __shfl_xor(s, o);
      double mn = fmax(m, m2);
      if (mn == -INFINITY) { s = 0.0; m = mn; }
      else { s = s * exp(m - mn) + s2 * exp(m2 - mn); m = mn; }
    }
    if (r == 0) part[((size_t)unit * G + gq) * nchunk + chunk] = make_double2(m, s);
  }
  (void)s_ms;
}

hipError_t launch_score_f32(const Dims& d, const void* k, const void* v, int64_t n, int64_t n_cap,
                            const float* mu, const float* sigma, double* logits, float* vnorm,
                            double2* part, int* nchunk_out, hipStream_t st) {
  int64_t span = (n + 1023) / 1024;
  span = (span + 63) / 64 * 64;
  if (span < 64) span = 64;
  int nchunk = (int)((n + span - 1) / span);
  *nchunk_out = nchunk;
  int grid = d.units() * d.G * nchunk;
  size_t lds = (size_t)64 * (d.D + 1) * sizeof(float);
#define EA_F32(DD)                                                                              \
  if (d.D == DD) {                                                                              \
    auto kern = k_score_f32<DD>;                                                                \
    static LdsOptIn opt;                                                                        \
    hipError_t e = opt.ensure(reinterpret_cast<const void*>(kern), lds);                        \
    if (e != hipSuccess) return e;                                                              \
    kern<<<grid, 256, lds, st>>>((const float*)k, (const float*)v, n, n_cap, mu, sigma, d.G,    \
                                 d.units(), (int)span, nchunk, logits, vnorm, part);            \
    return hipGetLastError();                                                                   \
  }
  EA_F32(64)
  EA_F32(128)
  EA_F32(256)
#undef EA_F32
  return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------------
// Pass B.  One workgroup = `rounds` x 1024 keys of one unit.  LT is the logit type (float: bf16
// caches, double: fp32 caches).  With hist0 != nullptr the first radix-select digit (top 11
// bits of the score's bit pattern) is histogrammed on the way out.
//
// The (max, sum exp) partials of pass A belong to fixed blocks of keys (partial j of a head
// covers the same keys in every run) and are combined here in index order, so the log-sum-exp,
// and with it every score, comes out bit-identical from run to run however pass A's tiles were
// dealt to workgroups.
template <typename LT>
struct LT2;
template <>
struct LT2<float> { typedef float2 type; };
template <>
struct LT2<double> { typedef double2 type; };

__device__ __forceinline__ float ea_exp(float x) { return expf(x); }
__device__ __forceinline__ double ea_exp(double x) { return exp(x); }
__device__ __forceinline__ float ea_log(float x) { return logf(x); }
__device__ __forceinline__ double ea_log(double x) { return log(x); }

template <typename LT>
__device__ __forceinline__ void merge_lt(LT& m, LT& s, LT m2, LT s2) {
  LT mn = m > m2 ? m : m2;
  if (mn == -INFINITY) { s = 0; m = mn; }
  else { s = s * ea_exp(m - mn) + s2 * ea_exp(m2 - mn); m = mn; }
}

// log-sum-exp of one head from its npart partials, by one wavefront: lane l takes partials
// l, l + 64, ... in increasing order, then a fixed butterfly over the lanes.
template <typename LT>
__device__ __forceinline__ LT wave_lse(const typename LT2<LT>::type* __restrict__ p, int npart, int lane) {
  LT m = -INFINITY, s = 0;
  for (int c = lane; c < npart; c += 64) merge_lt<LT>(m, s, p[c].x, p[c].y);
  for (int o = 32; o >= 1; o >>= 1) {
    LT m2 = __shfl_xor(m, o), s2 = __shfl_xor(s, o);
    merge_lt<LT>(m, s, m2, s2);
  }
  return m + ea_log(s);
}

// (max, sum exp) of one block of kLseBlock keys of one query head, from the logits pass A stored:
// the LDS-fragment kernels leave the softmax to this pass, so the partial of a block is the same
// number on every run whichever waves scored its keys (fixed reduction tree), and the score
// kernel's inner loop carries no exponentials or cross-lane reductions.  The logits were written
// a moment ago and are read from the caches.
__global__ __launch_bounds__(256) void k_lse_part(const float* __restrict__ logits, long long n, int npart,
                                                  float2* __restrict__ part) {
  constexpr int PER = kLseBlock / 256;
  __shared__ float s_red[2][4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int head = blockIdx.x / npart, j = blockIdx.x - head * npart;
  const float* lp = logits + (size_t)head * n;
  const long long base = (long long)j * kLseBlock;
  float x[PER];
#pragma unroll
  for (int it = 0; it < PER; ++it) {          // no load under a condition: indices past the end are clamped
    const long long i = base + it * 256 + tid;
    const float v = lp[min(i, n - 1)];
    x[it] = i < n ? v : -INFINITY;
  }
  float m = x[0];
#pragma unroll
  for (int it = 1; it < PER; ++it) m = fmaxf(m, x[it]);
  for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
  if (lane == 0) s_red[0][wave] = m;
  __syncthreads();
  m = fmaxf(fmaxf(s_red[0][0], s_red[0][1]), fmaxf(s_red[0][2], s_red[0][3]));   // a block holds a key: finite
  float s = 0.f;
#pragma unroll
  for (int it = 0; it < PER; ++it) s += expf(x[it] - m);
  for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o);
  if (lane == 0) s_red[1][wave] = s;
  __syncthreads();
  if (tid == 0) part[(size_t)head * npart + j] = make_float2(m, (s_red[1][0] + s_red[1][1]) + (s_red[1][2] + s_red[1][3]));
}

// Heads with very many partials: one workgroup per query head reduces them once, ahead of
// pass B (otherwise every workgroup of pass B would walk the whole list).
template <typename LT>
__global__ __launch_bounds__(256) void k_lse(const typename LT2<LT>::type* __restrict__ part, int npart,
                                             LT* __restrict__ lse) {
  __shared__ LT s_m[4], s_s[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const typename LT2<LT>::type* p = part + (size_t)blockIdx.x * npart;
  LT m = -INFINITY, s = 0;
  for (int c = tid; c < npart; c += 256) merge_lt<LT>(m, s, p[c].x, p[c].y);
  for (int o = 32; o >= 1; o >>= 1) {
    LT m2 = __shfl_xor(m, o), s2 = __shfl_xor(s, o);
    merge_lt<LT>(m, s, m2, s2);
  }
  if (lane == 0) { s_m[wave] = m; s_s[wave] = s; }
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < 4; ++w) merge_lt<LT>(m, s, s_m[w], s_s[w]);
    lse[blockIdx.x] = m + ea_log(s);
  }
}

template <typename LT>
__global__ __launch_bounds__(256) void k_finalize(const LT* __restrict__ logits,
                                                  const float* __restrict__ vnorm,
                                                  const typename LT2<LT>::type* __restrict__ part,
                                                  const LT* __restrict__ lse_in, int G, int npart,
                                                  long long n, float eps, int units, int rounds,
                                                  float* __restrict__ scores,
                                                  uint32_t* __restrict__ hist0,
                                                  const float* __restrict__ wnorm) {
  __shared__ LT s_lse[64];
  __shared__ uint32_t s_hist[kSelBins];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int unit = blockIdx.x % units;
  const long long blk = blockIdx.x / units;
  if (hist0)
    for (int i = tid; i < kSelBins; i += 256) s_hist[i] = 0;
  for (int g = wave; g < G; g += 4) {
    const LT v = lse_in ? lse_in[(size_t)unit * G + g]
                        : wave_lse<LT>(part + ((size_t)unit * G + g) * npart, npart, lane);
    if (lane == 0) s_lse[g] = v;
  }
  __syncthreads();
  const LT invG = (LT)1 / (LT)G;
  for (int rd = 0; rd < rounds; ++rd) {
    const long long base = (blk * rounds + rd) * 1024;
    if (base >= n) break;
    // The four keys of a thread go through the heads together and no load sits under a condition
    // (indices past the end are clamped): loads inside "if (i < n)" come back one at a time.
    long long ic[4];
    float vn[4];
    LT acc[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      ic[it] = min(base + it * 256 + tid, n - 1);
      vn[it] = vnorm[(size_t)unit * n + ic[it]];
      acc[it] = 0;
    }
    for (int g = 0; g < G; ++g) {
      const LT* lp = logits + ((size_t)unit * G + g) * n;
      const LT lse = s_lse[g];
      LT lv[4];
#pragma unroll
      for (int it = 0; it < 4; ++it) lv[it] = lp[ic[it]];
      if (wnorm) {        // Eq. 9 with the output projection: every query head weighs by its own norm
        const float* wp = wnorm + ((size_t)unit * G + g) * n;
#pragma unroll
        for (int it = 0; it < 4; ++it) acc[it] += (ea_exp(lv[it] - lse) + (LT)eps) * (LT)wp[ic[it]];
      } else {
#pragma unroll
        for (int it = 0; it < 4; ++it) acc[it] += ea_exp(lv[it] - lse);
      }
    }
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const long long i = base + it * 256 + tid;
      if (i < n) {
        float sc = wnorm ? (float)(acc[it] * invG) : (float)((acc[it] * invG + (LT)eps) * (LT)vn[it]);
        scores[(size_t)unit * n + i] = sc;
        if (hist0) {
          atomicAdd(&s_hist[__float_as_uint(sc) >> 21], 1u);
          if (__float_as_uint(sc) > 0x7f800000u)      // NaN (non-finite inputs): see ea_debug_status
            atomicOr(hist0 + 2 * kSelBins + kStatusSlot, kStatusBadScore);
        }
      }
    }
  }
  if (hist0) {
    __syncthreads();
    for (int i = tid; i < kSelBins; i += 256) {
      uint32_t c = s_hist[i];
      if (c) atomicAdd(&hist0[(size_t)unit * 3 * kSelBins + i], c);
    }
  }
}

// ||W_o^(g) v_i|| from the quadratic form pass A leaves in `logits` when it is run over the value
// rows with mu = 0 and Sigma = M_g = W_o^(g)^T W_o^(g):  logits = v^T M_g v / (2 d).
template <typename LT>
__global__ void k_wnorm(const LT* __restrict__ logits, size_t count, float two_d, float* __restrict__ wnorm) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) {
    const LT q = logits[i] * (LT)two_d;
    wnorm[i] = q > (LT)0 ? (float)sqrt(q) : 0.f;
  }
}

hipError_t launch_wnorm(const void* logits, int logits_f64, size_t count, int D, float* wnorm, hipStream_t st) {
  const unsigned grid = (unsigned)((count + 255) / 256);
  if (logits_f64)
    k_wnorm<double><<<grid, 256, 0, st>>>((const double*)logits, count, 2.0f * (float)D, wnorm);
  else
    k_wnorm<float><<<grid, 256, 0, st>>>((const float*)logits, count, 2.0f * (float)D, wnorm);
  return hipGetLastError();
}

constexpr int kLseInlineMax = 256;    // more partials per head than this: reduce them in k_lse first
                                      // (one short launch; every finalize workgroup then reads G numbers
                                      // instead of re-reducing the list: at 1024 partials per head, one
                                      // 131072-key layer per call, pass B takes 14.8 instead of 18.1 us)

hipError_t launch_finalize(const Dims& d, int64_t n, const void* logits, int logits_f64,
                           const float* vnorm, const void* part, int npart, void* lse, float* scores,
                           uint32_t* hist0, hipStream_t st, const float* wnorm, int lse_pass) {
  // 1024 keys per workgroup; four rounds of them (fewer histogram flushes) once that still leaves
  // a few thousand workgroups: the pass is bound by memory latency and wants the chip full
  const int rounds = (n + 1023) / 1024 * d.units() >= 4096 ? 4 : 1;
  const int64_t nblk = (n + 1024 * rounds - 1) / (1024 * rounds);
  const unsigned grid = (unsigned)(nblk * d.units());
  const bool pre = npart > kLseInlineMax;
  if (logits_f64) {
    if (pre) k_lse<double><<<d.qheads(), 256, 0, st>>>((const double2*)part, npart, (double*)lse);
    k_finalize<double><<<grid, 256, 0, st>>>((const double*)logits, vnorm, (const double2*)part,
                                             pre ? (const double*)lse : nullptr, d.G, npart, n, d.eps,
                                             d.units(), rounds, scores, hist0, wnorm);
  } else {
    if (lse_pass)
      k_lse_part<<<(unsigned)((size_t)d.qheads() * npart), 256, 0, st>>>((const float*)logits, n, npart, (float2*)part);
    if (pre) k_lse<float><<<d.qheads(), 256, 0, st>>>((const float2*)part, npart, (float*)lse);
    k_finalize<float><<<grid, 256, 0, st>>>((const float*)logits, vnorm, (const float2*)part,
                                            pre ? (const float*)lse : nullptr, d.G, npart, n, d.eps,
                                            d.units(), rounds, scores, hist0, wnorm);
  }
  return hipGetLastError();
}

}  // namespace ea
