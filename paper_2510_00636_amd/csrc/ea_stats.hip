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
                             float2* __restrict__ tab, uint32_t* __restrict__ clear,
                             size_t clear_words) {
  const size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  // riding along: zero the counters / histograms / flags of the later stages (one launch less)
  for (size_t i = gid; i < clear_words; i += (size_t)gridDim.x * blockDim.x) clear[i] = 0u;
  int i = (int)gid;
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

// ---------------------------------------------------------------------------------------
// Sigma is symmetric, so only its 32 x 32 tiles on and above the diagonal are computed (3 of 4 at
// d = 64, 10 of 16 at d = 128, 36 of 64 at d = 256) and every tile above the diagonal is stored
// twice, once transposed.  A head's tiles are dealt to kStatsParts<D> workgroups (1 / 2 / 4), each
// of which reads the window ONCE, in chunks of up to 64 samples: every thread issues all its
// 16-byte query loads and table loads of a chunk together (one memory latency per chunk instead
// of one per sample; the next chunk's loads go out before the current chunk's arithmetic), maps
// them to u~, subtracts the head's first sample u~_0 and writes the result to LDS; the four
// wavefronts then add the chunk's outer products to their accumulator tiles with fp32
// matrix-core instructions, two samples per instruction.
// With x = u~ - u~_0,
//     mean  = u~_0 + (1/w) sum_s x_s
//     Sigma = (1/(w - ddof)) (sum_s x_s x_s^T - w xbar xbar^T)
// exactly; the shift keeps |x| at the scale of the spread, so the subtraction of the second
// term costs no accuracy even for channels whose mean is many standard deviations from zero.
// Column sums are formed on the way in (each thread keeps the sums of the 16 channels of its
// items, all of one channel group) and combined in a fixed order, so results are reproducible.
// The fp32 matrix-core work is what bounds the kernel for long windows (64 cycles per pair of
// samples and tile): the triangle and the even deal over workgroups are what keep it short.
constexpr int kStatsWC = 64;    // samples per LDS chunk
template <int D, int PARTS_ = 0> struct StatsTiling {
  static constexpr int NCT = D / 32;                       // 32-column tiles across Sigma
  static constexpr int NT = NCT * (NCT + 1) / 2;           // tiles on and above the diagonal
  static constexpr int PARTS = PARTS_ > 0 ? PARTS_ : D <= 64 ? 1 : (D <= 128 ? 2 : 4);
  static constexpr int TP = (NT + PARTS - 1) / PARTS;      // tiles per workgroup
  // A workgroup's first 4 WHOLE tiles go one (or WHOLE) to each wavefront; the SHARED tiles left
  // over are each split four ways by samples and the four partial tiles added at the end, so
  // every wavefront carries the same matrix-core load.
  static constexpr int WHOLE = TP >= 4 ? TP / 4 : 1;
  static constexpr int SHARED = TP >= 4 ? TP % 4 : 0;
  static constexpr int SLOTS = WHOLE + SHARED;             // accumulator tiles per wavefront
};

// Channels of pair e of channel group g: ja for the first, jb for the second element of the pair.
template <int D>
__device__ __forceinline__ int stats_ja(int layout, int g, int e) { return layout ? 2 * (8 * g + e) : 8 * g + e; }
template <int D>
__device__ __forceinline__ int stats_jb(int layout, int g, int e) { return layout ? 2 * (8 * g + e) + 1 : 8 * g + e + D / 2; }

// One item = one sample's channel group g: 8 pairs (qa[e], qb[e]) of the query row and their 2x2
// blocks tb[e] of the table row.  An item is fetched as raw words (bf16 rows stay packed, half
// the registers, while the loads are in flight) and unpacked where it is used.
template <bool BF16>
struct StatsRaw {
  uint4 w[BF16 ? 2 : 4];
  float4 t[4];
};
template <int D, bool BF16>
__device__ __forceinline__ void stats_fetch_item(const void* __restrict__ q_win, size_t row, int g, int layout,
                                                 const float2* __restrict__ tabrow, StatsRaw<BF16>& raw) {
  constexpr int HALF = D / 2;
  // half-split: channels 8g.. and HALF+8g..; interleaved: 16 consecutive channels = 8 pairs
  const size_t oa = row + (layout ? 16 * g : 8 * g), ob = row + (layout ? 16 * g + 8 : HALF + 8 * g);
  if (BF16) {
    raw.w[0] = *reinterpret_cast<const uint4*>((const uint16_t*)q_win + oa);
    raw.w[1] = *reinterpret_cast<const uint4*>((const uint16_t*)q_win + ob);
  } else {
    raw.w[0] = *reinterpret_cast<const uint4*>((const float*)q_win + oa);
    raw.w[1] = *reinterpret_cast<const uint4*>((const float*)q_win + oa + 4);
    raw.w[BF16 ? 0 : 2] = *reinterpret_cast<const uint4*>((const float*)q_win + ob);
    raw.w[BF16 ? 1 : 3] = *reinterpret_cast<const uint4*>((const float*)q_win + ob + 4);
  }
  const float4* tp = reinterpret_cast<const float4*>(tabrow + 8 * g);
#pragma unroll
  for (int e = 0; e < 4; ++e) raw.t[e] = tp[e];
}
template <bool BF16>
__device__ __forceinline__ void stats_unpack_item(const StatsRaw<BF16>& raw, int layout, float (&qa)[8],
                                                  float (&qb)[8], float2 (&tb)[8]) {
  float xa[8], xb[8];
  if (BF16) {
    const uint32_t wa[4] = {raw.w[0].x, raw.w[0].y, raw.w[0].z, raw.w[0].w};
    const uint32_t wb[4] = {raw.w[1].x, raw.w[1].y, raw.w[1].z, raw.w[1].w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      xa[2 * e] = __uint_as_float(wa[e] << 16);
      xa[2 * e + 1] = __uint_as_float(wa[e] & 0xffff0000u);
      xb[2 * e] = __uint_as_float(wb[e] << 16);
      xb[2 * e + 1] = __uint_as_float(wb[e] & 0xffff0000u);
    }
  } else {
    const uint4 a0 = raw.w[0], a1 = raw.w[1], b0 = raw.w[BF16 ? 0 : 2], b1 = raw.w[BF16 ? 1 : 3];
    const uint32_t wa[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
    const uint32_t wb[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) { xa[e] = __uint_as_float(wa[e]); xb[e] = __uint_as_float(wb[e]); }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    // pair e of the group: (xa[e], xb[e]) half-split; (x[2e], x[2e+1]) of the 16 interleaved
    qa[e] = layout ? (e < 4 ? xa[2 * e] : xb[2 * e - 8]) : xa[e];
    qb[e] = layout ? (e < 4 ? xa[2 * e + 1] : xb[2 * e - 7]) : xb[e];
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    tb[2 * e] = make_float2(raw.t[e].x, raw.t[e].y);
    tb[2 * e + 1] = make_float2(raw.t[e].z, raw.t[e].w);
  }
}
typedef float floatx16_t __attribute__((ext_vector_type(16)));

// Register budget: three workgroups per CU at d <= 128 (168 registers), two at d = 256 (256),
// without spills for bf16 input (prefetched items stay packed, u~_0 lives in LDS, the tile numbers
// are scalar).  With more registers per wavefront the 640 workgroups of a decode-shape call do not
// fit on the chip at once.  A budget met only by spilling is no use here: a kernel that needs
// scratch memory costs some 10 us more per launch when several streams are in use.
template <int D, bool BF16>
__global__ __launch_bounds__(256, (D <= 128 ? 3 : 2)) void k_stats(const void* __restrict__ q_win, int w, int layout,
                                               int ddof, const float2* __restrict__ tab,
                                               float* __restrict__ mu, float* __restrict__ sigma) {
  constexpr int HALF = D / 2, G8 = HALF / 8;          // groups of 8 channel pairs per sample
  constexpr int ITEMS = kStatsWC * G8 / 256;          // (sample, group) items per thread and chunk
  typedef StatsTiling<D> TL;
  constexpr int NCT = TL::NCT, TPW = TL::SLOTS;
  static_assert(256 % G8 == 0 && ITEMS >= 1, "one channel group per thread");
  extern __shared__ __align__(16) float s_dyn[];
  float* s_u = s_dyn;                                 // [kStatsWC][D]   x = u~ - u~_0 of the chunk
  float* s_part = s_dyn + kStatsWC * D;               // [4][D]          column sums per wavefront
  float* s_shift = s_part + 4 * D;                    // [D]             u~_0
  float* s_xbar = s_shift + D;                        // [D]             (1/w) sum_s x_s
  const int head = blockIdx.x, part = blockIdx.y, tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);        // wave-uniform: tile numbers stay scalar
  const size_t qbase = (size_t)head * w * D;
  const int nchunks = (w + kStatsWC - 1) / kStatsWC;
  const int g = tid % G8;                             // the channel group of all this thread's items

  // the first chunk's loads go out before anything waits on memory
  StatsRaw<BF16> raw[ITEMS];
  auto load_chunk = [&](int ch) __attribute__((always_inline)) {
    const int s0 = ch * kStatsWC, ns = min(kStatsWC, w - s0);
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int sl = (tid + it * 256) / G8;
      if (sl < ns)
        stats_fetch_item<D, BF16>(q_win, qbase + (size_t)(s0 + sl) * D, g, layout,
                                  tab + (size_t)(s0 + sl) * HALF, raw[it]);
    }
  };
  load_chunk(0);
  // u~_0 of the head, kept in LDS (every thread reads its own group's 16 values per item)
  if (tid < G8) {
    float qa[8], qb[8];
    float2 tb[8];
    StatsRaw<BF16> raw0;
    stats_fetch_item<D, BF16>(q_win, qbase, g, layout, tab, raw0);
    stats_unpack_item<BF16>(raw0, layout, qa, qb, tb);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      s_shift[stats_ja<D>(layout, g, e)] = tb[e].x * qa[e] - tb[e].y * qb[e];
      s_shift[stats_jb<D>(layout, g, e)] = tb[e].y * qa[e] + tb[e].x * qb[e];
    }
  }
  __syncthreads();
  float suma[8], sumb[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { suma[e] = 0.f; sumb[e] = 0.f; }

  // Outer products on the matrix cores in fp32: v_mfma_f32_32x32x2_f32 adds, for two samples at a
  // time, the 32 x 32 block  x[rows] x[cols]^T.  Lane l feeds row (or column) l % 32 of sample
  // l / 32 of the pair; wavefront `wave` owns the column tiles wave, wave + 4, ...
  const int r32 = lane & 31, hh = lane >> 5;
  // this wavefront's tiles: number wave + 4 t of the workgroup's share for the whole ones, then the
  // shared ones; rows of the triangle in order
  int t_rb[TPW], t_ct[TPW];
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    const int local = t < TL::WHOLE ? wave + 4 * t : 4 * TL::WHOLE + (t - TL::WHOLE);
    int idx = part * TL::TP + local, rb = 0;
    const bool ok = local < TL::TP && idx < TL::NT;
    if (!ok) idx = 0;
#pragma unroll
    for (int r = 0; r < NCT; ++r)
      if (idx >= NCT - rb && rb == r) { idx -= NCT - rb; ++rb; }
    t_rb[t] = ok ? rb : -1;
    t_ct[t] = rb + idx;
  }
  floatx16_t acc[TPW];
#pragma unroll
  for (int t = 0; t < TPW; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;

  for (int ch = 0; ch < nchunks; ++ch) {
    const int s0 = ch * kStatsWC, ns = min(kStatsWC, w - s0);
    if (ch > 0) __syncthreads();                      // the previous chunk has been consumed
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int sl = (tid + it * 256) / G8;
      if (sl < ns) {
        float qa[8], qb[8], xa[8], xb[8];
        float2 tb[8];
        stats_unpack_item<BF16>(raw[it], layout, qa, qb, tb);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          xa[e] = tb[e].x * qa[e] - tb[e].y * qb[e] - s_shift[stats_ja<D>(layout, g, e)];
          xb[e] = tb[e].y * qa[e] + tb[e].x * qb[e] - s_shift[stats_jb<D>(layout, g, e)];
          suma[e] += xa[e];
          sumb[e] += xb[e];
        }
        if (layout == 0) {                            // half-split: two runs of 8 consecutive channels
          float4* pa = reinterpret_cast<float4*>(s_u + sl * D + 8 * g);
          float4* pb = reinterpret_cast<float4*>(s_u + sl * D + HALF + 8 * g);
          pa[0] = make_float4(xa[0], xa[1], xa[2], xa[3]);
          pa[1] = make_float4(xa[4], xa[5], xa[6], xa[7]);
          pb[0] = make_float4(xb[0], xb[1], xb[2], xb[3]);
          pb[1] = make_float4(xb[4], xb[5], xb[6], xb[7]);
        } else {                                      // interleaved: 16 consecutive channels
          float4* pi = reinterpret_cast<float4*>(s_u + sl * D + 16 * g);
#pragma unroll
          for (int e = 0; e < 4; ++e) pi[e] = make_float4(xa[2 * e], xb[2 * e], xa[2 * e + 1], xb[2 * e + 1]);
        }
      }
    }
    __syncthreads();
    if (ch + 1 < nchunks) load_chunk(ch + 1);         // in flight during the matrix-core loop
    // a few sample pairs per step: all their LDS reads first, then the MFMAs (samples past the
    // chunk's end count as zero)
    constexpr int PS = TPW == 1 ? 4 : 2;
    const int npair = (ns + 1) / 2;
    for (int sp = 0; sp < npair; sp += PS) {
      float av[PS][TPW], bv[PS][TPW];
      const bool mine = ((sp / PS) & 3) == wave;       // this step's samples of the shared tiles
#pragma unroll
      for (int u = 0; u < PS; ++u) {
        const int sl = 2 * (sp + u) + hh;
        const bool ok = sl < ns;
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
          const bool okt = ok && t_rb[t] >= 0 && (t < TL::WHOLE || mine);
          av[u][t] = okt ? s_u[sl * D + t_rb[t] * 32 + r32] : 0.f;
          bv[u][t] = okt ? s_u[sl * D + t_ct[t] * 32 + r32] : 0.f;
        }
      }
#pragma unroll
      for (int u = 0; u < PS; ++u)
#pragma unroll
        for (int t = 0; t < TPW; ++t)
          if (t_rb[t] >= 0 && (t < TL::WHOLE || mine))
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u][t], bv[u][t], acc[t], 0, 0, 0);
    }
  }
  if (TL::SHARED > 0) {
    // the four partial tiles of every shared tile, added in wavefront order by wavefront 0
    static_assert(TL::SHARED * 4 * 16 * 64 <= kStatsWC * D, "partial tiles fit in the chunk buffer");
    __syncthreads();
#pragma unroll
    for (int r = 0; r < TL::SHARED; ++r)
#pragma unroll
      for (int v = 0; v < 16; ++v) s_u[((r * 4 + wave) * 16 + v) * 64 + lane] = acc[TL::WHOLE + r][v];
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int r = 0; r < TL::SHARED; ++r)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float* pp = s_u + (r * 4 * 16 + v) * 64 + lane;
          acc[TL::WHOLE + r][v] = (pp[0] + pp[16 * 64]) + (pp[2 * 16 * 64] + pp[3 * 16 * 64]);
        }
    }
  }

  // column sums: lanes that share a channel group (stride G8) first, then the four wavefronts
#pragma unroll
  for (int e = 0; e < 8; ++e) {
#pragma unroll
    for (int o = G8; o < 64; o <<= 1) {
      suma[e] += __shfl_xor(suma[e], o);
      sumb[e] += __shfl_xor(sumb[e], o);
    }
  }
  if (lane < G8) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      s_part[wave * D + stats_ja<D>(layout, g, e)] = suma[e];
      s_part[wave * D + stats_jb<D>(layout, g, e)] = sumb[e];
    }
  }
  __syncthreads();
  const float invw = 1.0f / (float)w;
  for (int c = tid; c < D; c += 256) {
    const float xb = ((s_part[c] + s_part[D + c]) + (s_part[2 * D + c] + s_part[3 * D + c])) * invw;
    s_xbar[c] = xb;
    if (part == 0) mu[(size_t)head * D + c] = s_shift[c] + xb;
  }
  __syncthreads();
  // accumulator register v of lane (r32, hh) is row 8 (v / 4) + 4 hh + v % 4, column r32 of the tile
  const float fw = (float)w, inv = 1.0f / (float)(w - ddof);
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    if (t_rb[t] >= 0 && (t < TL::WHOLE || wave == 0)) {
      const int i0 = t_rb[t] * 32, j = t_ct[t] * 32 + r32;
      const bool mirror = t_rb[t] != t_ct[t];
      const float xj = s_xbar[j];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int i = i0 + 8 * (v / 4) + 4 * hh + v % 4;
        const float val = (acc[t][v] - fw * s_xbar[i] * xj) * inv;
        sigma[((size_t)head * D + i) * D + j] = val;
        if (mirror) sigma[((size_t)head * D + j) * D + i] = val;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// The same statistics for bf16 windows with the outer products on the fp16 matrix cores.
//
// fp32 matrix-core instructions run at the rate of the vector units (and do not overlap with
// vector work), which made the kernel above the largest stage of a decode-time pass (512-sample
// windows).  Here every shifted sample x = u~ - u~_0 is scaled by a power of two s and split into
// two fp16 numbers, x s = hi + lo (hi = x s rounded toward zero to fp16, lo = the remainder
// rounded to fp16: 21 significant bits together), and
//     sum_s x x^T  =  (1/s^2) sum_s (hi hi^T + hi lo^T + lo hi^T)  + O(2^-21)
// runs as three v_mfma_f32_32x32x16_f16 per tile and 16 samples (96 cycles instead of 512), with
// fp32 accumulation.  The samples are the contraction index, so the chunk is staged transposed:
// two planes [channel][chunk of 64 or 32 samples] of fp16 with a row pitch of 8 more (conflict-free
// 16-byte reads).
// s is taken from the largest |x| of the head's first chunk (that chunk lands in [16, 32)), which
// leaves a factor 2048 of headroom for later samples before fp16 overflows (an overflow shows as
// non-finite statistics, and then as the NaN-score bit of the status word).  Mean, column sums,
// the shift and the final algebra are those of k_stats, in fp32.
typedef _Float16 stats_half8 __attribute__((ext_vector_type(8)));
typedef _Float16 stats_half2 __attribute__((ext_vector_type(2)));
// samples per staged chunk: 64, and 32 at d = 256 (registers: a thread keeps its share of the next
// chunk's queries and table rows in flight during the matrix-core loop)
constexpr int stats_split_chunk(int D) { return D >= 256 ? 32 : 64; }

template <int D, int LAYOUT, int PARTS = 0>
__global__ __launch_bounds__(256, (D <= 128 && !(D == 128 && PARTS == 1) ? 3 : 2)) void k_stats_split(const void* __restrict__ q_win, int w,
                                                                         int ddof,
                                                                         const float2* __restrict__ tab,
                                                                         float* __restrict__ mu,
                                                                         float* __restrict__ sigma) {
  constexpr int HALF = D / 2, G8 = HALF / 8, layout = LAYOUT;   // the channel pairing is a compile-time constant:
                                                                // every LDS address below is a base plus an immediate
  constexpr int WC = stats_split_chunk(D);            // samples per chunk
  constexpr int ITEMS = WC * G8 / 256;                // consecutive samples per thread and chunk
  constexpr int P = WC + 8;                           // halves per channel row of a plane
  // Rows eight channels apart start 0 or 32 banks apart whatever the (16-byte aligned) pitch, and
  // those are the rows the lanes of one staging write go to (one channel of every group): the
  // 16-byte column blocks of a row are therefore XOR-swizzled by the row's channel group, which
  // spreads the groups over the blocks (writes conflict-free at d = 128, two-way at d = 256) and
  // leaves the 16 lanes of a matrix-operand read (two groups of equal swizzle) in one block.
  constexpr int NB = WC / 8;                          // column blocks per row
  constexpr int BW = G8 >= 16 ? 1 : 16 / G8;          // blocks one wave-wide staging write spans
  auto swz_of_group = [](int gg) { return ITEMS >= 2 ? ((gg >> 1) * BW) % NB : 0; };
  auto group_of_channel = [](int c) { return LAYOUT ? c / 16 : (c % HALF) / 8; };
  typedef StatsTiling<D, PARTS> TL;
  constexpr int NCT = TL::NCT, TPW = TL::SLOTS;
  static_assert(ITEMS >= 1 && 256 % G8 == 0, "one channel group per thread");
  static_assert(TL::SHARED * 4 * 16 * 64 * 4 <= 2 * D * P * 2, "partial tiles fit in the planes");
  extern __shared__ __align__(16) float s_dyn[];
  _Float16* s_hi = reinterpret_cast<_Float16*>(s_dyn);            // [D][P]
  _Float16* s_lo = s_hi + D * P;                                   // [D][P]
  float* s_part = reinterpret_cast<float*>(s_lo + D * P);          // [4][D] column sums per wavefront
  float* s_shift = s_part + 4 * D;                                 // [D] u~_0
  float* s_xbar = s_shift + D;                                     // [D]
  float* s_max = s_xbar + D;                                       // [4]
  const int head = blockIdx.x, part = blockIdx.y, tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const size_t qbase = (size_t)head * w * D;
  const int nchunks = (w + WC - 1) / WC;
  const int g = tid % G8, sl_t = ITEMS * (tid / G8);   // this thread's channel group and first sample of a chunk

  StatsRaw<true> raw[ITEMS];
  auto load_chunk = [&](int ch) __attribute__((always_inline)) {
    const int s0 = ch * WC, ns = min(WC, w - s0);
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int sl = min(sl_t + it, ns - 1);            // no load under a condition: past the end, the last sample again
      stats_fetch_item<D, true>(q_win, qbase + (size_t)(s0 + sl) * D, g, layout, tab + (size_t)(s0 + sl) * HALF, raw[it]);
    }
  };
  load_chunk(0);
  if (tid < G8) {
    float qa[8], qb[8];
    float2 tb[8];
    StatsRaw<true> raw0;
    stats_fetch_item<D, true>(q_win, qbase, g, layout, tab, raw0);
    stats_unpack_item<true>(raw0, layout, qa, qb, tb);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      s_shift[stats_ja<D>(layout, g, e)] = tb[e].x * qa[e] - tb[e].y * qb[e];
      s_shift[stats_jb<D>(layout, g, e)] = tb[e].y * qa[e] + tb[e].x * qb[e];
    }
  }
  __syncthreads();
  float suma[8], sumb[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { suma[e] = 0.f; sumb[e] = 0.f; }

  const int r32 = lane & 31, kg = lane >> 5;
  int t_rb[TPW], t_ct[TPW];
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    const int local = t < TL::WHOLE ? wave + 4 * t : 4 * TL::WHOLE + (t - TL::WHOLE);
    int idx = part * TL::TP + local, rb = 0;
    const bool ok = local < TL::TP && idx < TL::NT;
    if (!ok) idx = 0;
#pragma unroll
    for (int r = 0; r < NCT; ++r)
      if (idx >= NCT - rb && rb == r) { idx -= NCT - rb; ++rb; }
    t_rb[t] = ok ? rb : -1;
    t_ct[t] = rb + idx;
  }
  floatx16_t acc[TPW];
#pragma unroll
  for (int t = 0; t < TPW; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;

  // x = u~ - u~_0 of item `it` of the chunk in flight (zeros past the chunk's end): [0, 8) the first,
  // [8, 16) the second channels of the group's pairs
  auto item_x = [&](int it, int ns, float (&x)[16]) __attribute__((always_inline)) {
    float qa[8], qb[8];
    float2 tb[8];
    stats_unpack_item<true>(raw[it], layout, qa, qb, tb);
    const bool ok = sl_t + it < ns;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      x[e] = ok ? tb[e].x * qa[e] - tb[e].y * qb[e] - s_shift[stats_ja<D>(layout, g, e)] : 0.f;
      x[8 + e] = ok ? tb[e].y * qa[e] + tb[e].x * qb[e] - s_shift[stats_jb<D>(layout, g, e)] : 0.f;
    }
  };

  float scale = 1.0f;
  for (int ch = 0; ch < nchunks; ++ch) {
    const int ns = min(WC, w - ch * WC);
    // ---- this thread's samples of the chunk, then at once the requests for the next chunk: they
    //      travel during the conversion, the barriers and the matrix-core loop below
    float xs[ITEMS][16];
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) item_x(it, ns, xs[it]);
    if (ch + 1 < nchunks) load_chunk(ch + 1);
    if (ch == 0) {
      // the head's scale: a power of two that puts the first chunk's largest |x| into [16, 32)
      float amax = 0.f;
#pragma unroll
      for (int it = 0; it < ITEMS; ++it)
#pragma unroll
        for (int c16 = 0; c16 < 16; ++c16) amax = fmaxf(amax, fabsf(xs[it][c16]));
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o));
      if (lane == 0) s_max[wave] = amax;
      __syncthreads();
      const float m = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
      if (m > 0.f && m < INFINITY) {
        int ex;
        frexpf(m, &ex);                               // m = f 2^ex, f in [0.5, 1)
        scale = ldexpf(1.0f, max(-100, min(100, 5 - ex)));
      }
    } else {
      __syncthreads();                                // the previous chunk has been consumed
    }
    // ---- fp16 (hi, lo) of x * scale into the transposed planes, column sums on the way
#pragma unroll
    for (int it = 0; it < ITEMS; it += 2) {
#pragma unroll
      for (int c16 = 0; c16 < 16; ++c16) {
        const int e = c16 & 7;
        const int c = c16 < 8 ? stats_ja<D>(layout, g, e) : stats_jb<D>(layout, g, e);
        const float x0 = xs[it][c16];
        const float y0 = x0 * scale;
        if constexpr (ITEMS >= 2) {
          const float x1 = xs[it + 1][c16];
          if (c16 < 8) suma[e] += x0 + x1; else sumb[e] += x0 + x1;
          const float y1 = x1 * scale;
          const stats_half2 h = __builtin_bit_cast(stats_half2, __builtin_amdgcn_cvt_pkrtz(y0, y1));
          const stats_half2 l = {(_Float16)(y0 - (float)h[0]), (_Float16)(y1 - (float)h[1])};
          const int col = ((((sl_t + it) >> 3) ^ swz_of_group(g)) << 3) + ((sl_t + it) & 7);
          *reinterpret_cast<stats_half2*>(s_hi + c * P + col) = h;
          *reinterpret_cast<stats_half2*>(s_lo + c * P + col) = l;
        } else {
          if (c16 < 8) suma[e] += x0; else sumb[e] += x0;
          const stats_half2 h = __builtin_bit_cast(stats_half2, __builtin_amdgcn_cvt_pkrtz(y0, 0.f));
          s_hi[c * P + sl_t] = h[0];
          s_lo[c * P + sl_t] = (_Float16)(y0 - (float)h[0]);
        }
      }
    }
    __syncthreads();
    // ---- three matrix-core instructions per tile and 16 samples
    const int nks = (ns + 15) / 16;
#pragma unroll 1
    for (int ks = 0; ks < nks; ++ks) {
#pragma unroll
      for (int t = 0; t < TPW; ++t) {
        if (t_rb[t] >= 0 && (t < TL::WHOLE || ((ch * (WC / 16) + ks) & 3) == wave)) {
          const int ca = t_rb[t] * 32 + r32, cb = t_ct[t] * 32 + r32;
          const int ra = ca * P + (((ks * 2 + kg) ^ swz_of_group(group_of_channel(ca))) << 3);
          const int rbw = cb * P + (((ks * 2 + kg) ^ swz_of_group(group_of_channel(cb))) << 3);
          const stats_half8 ah = *reinterpret_cast<const stats_half8*>(s_hi + ra);
          const stats_half8 al = *reinterpret_cast<const stats_half8*>(s_lo + ra);
          const stats_half8 bh = *reinterpret_cast<const stats_half8*>(s_hi + rbw);
          const stats_half8 bl = *reinterpret_cast<const stats_half8*>(s_lo + rbw);
          acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh, acc[t], 0, 0, 0);
          acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bl, acc[t], 0, 0, 0);
          acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, bh, acc[t], 0, 0, 0);
        }
      }
    }
  }
  if (TL::SHARED > 0) {
    // the four partial tiles of every shared tile, added in wavefront order by wavefront 0
    float* s_u = s_dyn;
    __syncthreads();
#pragma unroll
    for (int r = 0; r < TL::SHARED; ++r)
#pragma unroll
      for (int v = 0; v < 16; ++v) s_u[((r * 4 + wave) * 16 + v) * 64 + lane] = acc[TL::WHOLE + r][v];
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int r = 0; r < TL::SHARED; ++r)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float* pp = s_u + (r * 4 * 16 + v) * 64 + lane;
          acc[TL::WHOLE + r][v] = (pp[0] + pp[16 * 64]) + (pp[2 * 16 * 64] + pp[3 * 16 * 64]);
        }
    }
  }

  // column sums: lanes that share a channel group (stride G8) first, then the four wavefronts
#pragma unroll
  for (int e = 0; e < 8; ++e) {
#pragma unroll
    for (int o = G8; o < 64; o <<= 1) {
      suma[e] += __shfl_xor(suma[e], o);
      sumb[e] += __shfl_xor(sumb[e], o);
    }
  }
  if (lane < G8) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      s_part[wave * D + stats_ja<D>(layout, g, e)] = suma[e];
      s_part[wave * D + stats_jb<D>(layout, g, e)] = sumb[e];
    }
  }
  __syncthreads();
  const float invw = 1.0f / (float)w;
  for (int c = tid; c < D; c += 256) {
    const float xb = ((s_part[c] + s_part[D + c]) + (s_part[2 * D + c] + s_part[3 * D + c])) * invw;
    s_xbar[c] = xb;
    if (part == 0) mu[(size_t)head * D + c] = s_shift[c] + xb;
  }
  __syncthreads();
  // In the matrix-core product a lane's B operand is column r32 and its A rows come back as
  // accumulator register v = row 8 (v / 4) + 4 kg + v % 4: the tile's entry (row, column r32).
  const float fw = (float)w, inv = 1.0f / (float)(w - ddof), unscale = 1.0f / (scale * scale);
  // A tile above the diagonal is also stored transposed.  Straight from the accumulators that is
  // 64 separate 4-byte writes per instruction (a lane holds one column).  At d = 256 (28 of 36 tiles
  // are mirrored, 64 MB of Sigma per launch of the four-sequence shape) the tile takes a trip
  // through the wavefront's own patch of LDS (the planes are free by now) and leaves as rows; at
  // d <= 128 that costs the registers that keep three workgroups on a CU without scratch memory,
  // and the direct stores are the faster ones (5.6 against 10.4 us per layer at the decode shape).
  constexpr bool kViaLds = D >= 256;
  if constexpr (!kViaLds) {
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
      if (t_rb[t] >= 0 && (t < TL::WHOLE || wave == 0)) {
        const int i0 = t_rb[t] * 32, j = t_ct[t] * 32 + r32;
        const bool mirror = t_rb[t] != t_ct[t];
        const float xj = s_xbar[j];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int i = i0 + 8 * (v / 4) + 4 * kg + v % 4;
          const float val = (acc[t][v] * unscale - fw * s_xbar[i] * xj) * inv;
          sigma[((size_t)head * D + i) * D + j] = val;
          if (mirror) sigma[((size_t)head * D + j) * D + i] = val;
        }
      }
    }
  } else {
    float* s_tr = s_dyn + wave * (32 * 33);
    static_assert(4 * 32 * 33 * 4 <= 2 * D * P * 2, "transposition patches fit in the planes");
    __syncthreads();                 // every wavefront is done with the planes (and the partial tiles)
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
      if (t_rb[t] >= 0 && (t < TL::WHOLE || wave == 0)) {
        const int i0 = t_rb[t] * 32, j0 = t_ct[t] * 32, j = j0 + r32;
        const bool mirror = t_rb[t] != t_ct[t];
        const float xj = s_xbar[j];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int il = 8 * (v / 4) + 4 * kg + v % 4;
          const float val = (acc[t][v] * unscale - fw * s_xbar[i0 + il] * xj) * inv;
          sigma[((size_t)head * D + i0 + il) * D + j] = val;
          if (mirror) s_tr[r32 * 33 + il] = val;         // [column][row]
        }
        if (mirror) {
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
          __builtin_amdgcn_wave_barrier();
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int jl = 2 * v + kg;                    // column of the tile = row of the transposed one
            sigma[((size_t)head * D + j0 + jl) * D + i0 + r32] = s_tr[jl * 33 + r32];
          }
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
          __builtin_amdgcn_wave_barrier();
        }
      }
    }
  }
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
                             int w, float2* tab, uint32_t* clear, size_t clear_words, hipStream_t st) {
  int total = w * d.half;
  k_rope_table<<<(total + 255) / 256, 256, 0, st>>>(inv_freq, q_pos0, t_next, d.T, w, d.half,
                                                    d.q_is_rotated, tab, clear, clear_words);
  return hipGetLastError();
}

template <int D, bool BF16>
static hipError_t launch_stats_one(const Dims& d, const void* q_win, int w, const float2* tab,
                                   float* mu, float* sigma, hipStream_t st) {
  auto kern = k_stats<D, BF16>;
  const size_t lds = (size_t)(kStatsWC * D + 6 * D) * sizeof(float);
  static LdsOptIn opt;                    // one per kernel instance
  hipError_t e = opt.ensure(reinterpret_cast<const void*>(kern), lds);
  if (e != hipSuccess) return e;
  dim3 grid(d.qheads(), StatsTiling<D>::PARTS);
  kern<<<grid, 256, lds, st>>>(q_win, w, d.rope_layout, d.ddof, tab, mu, sigma);
  return hipGetLastError();
}

template <int D, int LAYOUT, int PARTS>
static hipError_t launch_stats_split_parts(const Dims& d, const void* q_win, int w, const float2* tab, float* mu,
                                           float* sigma, hipStream_t st) {
  auto kern = k_stats_split<D, LAYOUT, PARTS>;
  const size_t lds = (size_t)2 * D * (stats_split_chunk(D) + 8) * sizeof(_Float16) + (size_t)(6 * D + 4) * sizeof(float);
  static LdsOptIn opt;
  hipError_t e = opt.ensure(reinterpret_cast<const void*>(kern), lds);
  if (e != hipSuccess) return e;
  dim3 grid(d.qheads(), StatsTiling<D, PARTS>::PARTS);
  kern<<<grid, 256, lds, st>>>(q_win, w, d.ddof, tab, mu, sigma);
  return hipGetLastError();
}
// Every workgroup of a head stages all of the head's samples, so a head split over two workgroups
// pays the staging twice: with enough heads to fill the chip (the decode-time shape: 960 per call)
// one workgroup takes all ten tiles of a d = 128 head.
constexpr int kStatsWholeHeadMin = 384;
template <int D, int LAYOUT>
static hipError_t launch_stats_split_one(const Dims& d, const void* q_win, int w, const float2* tab, float* mu,
                                         float* sigma, hipStream_t st) {
  if constexpr (D == 128) {
    if (d.qheads() >= kStatsWholeHeadMin) return launch_stats_split_parts<D, LAYOUT, 1>(d, q_win, w, tab, mu, sigma, st);
  }
  return launch_stats_split_parts<D, LAYOUT, 0>(d, q_win, w, tab, mu, sigma, st);
}
template <int D>
static hipError_t launch_stats_split(const Dims& d, const void* q_win, int w, const float2* tab, float* mu,
                                     float* sigma, hipStream_t st) {
  return d.rope_layout ? launch_stats_split_one<D, 1>(d, q_win, w, tab, mu, sigma, st)
                       : launch_stats_split_one<D, 0>(d, q_win, w, tab, mu, sigma, st);
}

hipError_t launch_stats(const Dims& d, const void* q_win, int w, const float2* tab, float* mu,
                        float* sigma, hipStream_t st) {
  const bool bf = d.dtype == EA_BF16;
  // bf16 windows: outer products on the fp16 matrix cores (split operands); fp32 windows: fp32 ones
  if (bf && d.D == 64) return launch_stats_split<64>(d, q_win, w, tab, mu, sigma, st);
  if (bf && d.D == 128) return launch_stats_split<128>(d, q_win, w, tab, mu, sigma, st);
  if (bf) return launch_stats_split<256>(d, q_win, w, tab, mu, sigma, st);
  if (d.D == 64) return launch_stats_one<64, false>(d, q_win, w, tab, mu, sigma, st);
  if (d.D == 128) return launch_stats_one<128, false>(d, q_win, w, tab, mu, sigma, st);
  return launch_stats_one<256, false>(d, q_win, w, tab, mu, sigma, st);
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
