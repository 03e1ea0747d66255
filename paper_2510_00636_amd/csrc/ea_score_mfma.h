// The matrix-core score kernel (pass A of the scoring stage) as a template, with the device
// helpers it uses.  Each ea_score_d*.hip instantiates it for one head dimension, so that the
// instances compile in parallel.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

#include "ea_kernels.h"

namespace ea {

constexpr int kFragPrefetch = 4;  // LDS fragments in flight ahead of the MFMA that consumes them

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
// native 16-byte vector: plain loads/stores the optimiser can keep in registers (HIP's uint4 is
// a struct whose copies go through memcpy)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kTicketWays = 8;

struct ScoreArgs {
  const u32x4* k;
  const u32x4* v;
  long long n, n_cap;
  const u32x4* frags;
  const float* post;
  float* logits;
  float* vnorm;
  float2* part;           // register-fragment kernel only: its (max, sum exp) partials
  int G, passes, nchunk, units, nfrag;     // nchunk: workgroups per (unit, pass)
  int npart;              // that kernel: partials per query head, partial j covers keys [pg*j, pg*j + pg)
  int tpt;                // register-fragment kernel: tiles per ticket (pg = 32 * tpt); else unused
  uint32_t* tickets;      // tickets + unit * ticket_stride + pass * kTicketWays + way: tile counters, zero at launch
  int ticket_stride;
  PageMap pm;             // pm.table != nullptr: k and v are block pools (CLAMP instances only)
  const float* kscale;    // FP8 instances: real key = kscale[unit] * stored value (nullptr: 1)
  const float* vscale;    // likewise for the values
  int skip_v;             // 1: the caller has its own per-pair weights; V is not read, vnorm not written
};

__device__ __forceinline__ half8 bf16x8_to_half8(u32x4 r) {
  // bf16 -> fp32 is a 16-bit shift; fp32 -> fp16 is exact for |x| in [2^-14, 65504]
  // (a bf16 significand has 8 bits, fp16 keeps 11), so round-toward-zero loses nothing there.
  auto cv = [](uint32_t w) {
    return __builtin_amdgcn_cvt_pkrtz(__uint_as_float(w << 16), __uint_as_float(w & 0xffff0000u));
  };
  auto a = cv(r[0]), b = cv(r[1]), c = cv(r[2]), d = cv(r[3]);
  half8 o;
  o[0] = a[0]; o[1] = a[1]; o[2] = b[0]; o[3] = b[1];
  o[4] = c[0]; o[5] = c[1]; o[6] = d[0]; o[7] = d[1];
  return o;
}

// 16 fp8 (OCP e4m3) values -> two half8: exact (a 4-bit significand and an exponent range of
// 2^-9 .. 448 both fit fp16)
__device__ __forceinline__ void fp8x16_to_half8x2(u32x4 r, half8& lo, half8& hi) {
  auto lo2 = [](uint32_t w) {          // bytes 0, 1 of the word
    const auto f = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false);
    return __builtin_amdgcn_cvt_pkrtz(f[0], f[1]);
  };
  auto hi2 = [](uint32_t w) {          // bytes 2, 3
    const auto f = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
    return __builtin_amdgcn_cvt_pkrtz(f[0], f[1]);
  };
  const uint32_t w0 = r[0], w1 = r[1], w2 = r[2], w3 = r[3];
  const auto a = lo2(w0), b = hi2(w0), c = lo2(w1), d = hi2(w1);
  const auto e = lo2(w2), f = hi2(w2), g = lo2(w3), h = hi2(w3);
  lo[0] = a[0]; lo[1] = a[1]; lo[2] = b[0]; lo[3] = b[1]; lo[4] = c[0]; lo[5] = c[1]; lo[6] = d[0]; lo[7] = d[1];
  hi[0] = e[0]; hi[1] = e[1]; hi[2] = f[0]; hi[3] = f[1]; hi[4] = g[0]; hi[5] = g[1]; hi[6] = h[0]; hi[7] = h[1];
}

__device__ __forceinline__ float sumsq_fp8x16(u32x4 r) {
  float s = 0.f;
  const uint32_t w[4] = {r[0], r[1], r[2], r[3]};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const auto a = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], false);
    const auto b = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], true);
    s = fmaf(a[0], a[0], s);
    s = fmaf(a[1], a[1], s);
    s = fmaf(b[0], b[0], s);
    s = fmaf(b[1], b[1], s);
  }
  return s;
}

__device__ __forceinline__ float sumsq_bf16x8(u32x4 r) {
  // plain scalar copies first: __builtin_bit_cast applied directly to a vector-element
  // expression (r.y ...) reads element 0 of the vector
  const uint32_t w0 = r[0], w1 = r[1], w2 = r[2], w3 = r[3];
  const bf16x2 a = __builtin_bit_cast(bf16x2, w0), b = __builtin_bit_cast(bf16x2, w1);
  const bf16x2 c = __builtin_bit_cast(bf16x2, w2), d = __builtin_bit_cast(bf16x2, w3);
  float s = 0.f;
  s = __builtin_amdgcn_fdot2_f32_bf16(a, a, s, false);
  s = __builtin_amdgcn_fdot2_f32_bf16(b, b, s, false);
  s = __builtin_amdgcn_fdot2_f32_bf16(c, c, s, false);
  s = __builtin_amdgcn_fdot2_f32_bf16(d, d, s, false);
  return s;
}

// x of lane l plus x of lane l ^ 32, in every lane: one v_permlane32_swap (it hands both
// halves of the wavefront the other half's registers) instead of a trip through LDS.
__device__ __forceinline__ float sum_halves(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// x + (x of another lane of the same 16-lane row), selected by a DPP control word
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true);
  return x + __int_as_float(y);
}

// Sum over aligned groups of N consecutive lanes (N = 8, 16 or 32); every lane gets the total.
template <int N>
__device__ __forceinline__ float group_sum(float x) {
  x = dpp_add<0xB1>(x);                       // quad_perm [1,0,3,2]
  x = dpp_add<0x4E>(x);                       // quad_perm [2,3,0,1]
  x = dpp_add<0x141>(x);                      // row_half_mirror: lanes 0-7 <-> 7-0 of each half row
  if (N >= 16) x = dpp_add<0x140>(x);         // row_mirror
  if (N >= 32) x += __shfl_xor(x, 16);
  return x;
}

// Max / sum over the first 32 lanes of the wavefront as a wave-uniform value: butterfly inside
// each row of 16 lanes, then the two row totals are read out with v_readlane (no trip through
// LDS, no wait).  The callers hold the same data in lanes l and l + 32.
template <int CTRL>
__device__ __forceinline__ float dpp_max(float x) {
  int y = __builtin_amdgcn_update_dpp(__float_as_int(x), __float_as_int(x), CTRL, 0xf, 0xf, false);
  return fmaxf(x, __int_as_float(y));
}
__device__ __forceinline__ float max_lanes32(float x) {
  x = dpp_max<0xB1>(x);
  x = dpp_max<0x4E>(x);
  x = dpp_max<0x141>(x);
  x = dpp_max<0x140>(x);
  return fmaxf(__int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 0)),
               __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 16)));
}
__device__ __forceinline__ float sum_lanes32(float x) {
  x = dpp_add<0xB1>(x);
  x = dpp_add<0x4E>(x);
  x = dpp_add<0x141>(x);
  x = dpp_add<0x140>(x);
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 0)) +
         __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 16));
}

// compile-time loop: f(std::integral_constant<int, 0>) ... f(<N-1>), so that every register
// array index below is a constant
template <int N, int I = 0, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<N, I + 1>(f);
  }
}

// output tile index jt of the rem-th fragment of a head (tile jt owns fragments
// jt*(jt+1) .. jt*(jt+1) + 2jt + 1 of the triangular tiling)
constexpr int tri_jt(int rem) {
  int jt = 0;
  while (rem >= (jt + 1) * (jt + 2)) ++jt;
  return jt;
}
// LDS fragment index used by matrix-core step f (the extra tile's fragments are stored last)
template <int GH, int NF, int NX>
constexpr int step_frag(int f) { return f < NX ? GH * NF + f : f - NX; }

// The 2*NL global loads of the next tile are spread evenly over the steps [NX, NS).
template <int NX, int NS, int NL>
constexpr int load_slot(int i) { return NX + (i * (NS - NX)) / (2 * NL); }
// accumulator row rho of a 32x32 tile lives in register ROW_V(rho) of the lanes with
// lane / 32 == ROW_HH(rho)  (column = lane % 32)
#define ROW_V(rho) (4 * ((rho) / 8) + (rho) % 4)
#define ROW_HH(rho) (((rho) / 4) % 2)

// ---------------------------------------------------------------------------------------
// One wavefront scores 32 keys per iteration.  Lane l = (r = l % 32, hh = l / 32) owns the
// channels hh*d/2 .. hh*d/2 + d/2 - 1 of key r as fp16 (B operand of the 32x32x16 MFMA), the
// fragments of M (A operand) come from LDS, and the accumulator layout hands the lane the
// same channels back, so  sum_j acc_j k_j  is 16 mixed-precision FMAs per output tile.
// K rows reach that layout through a per-wave LDS staging buffer (coalesced 16-byte global
// loads in, conflict-free 16-byte LDS reads out); V rows are squared and summed straight
// from the coalesced layout.  The next tile's K and V loads are issued before the matrix
// work of the current one.
//
// Ragged tail: the last tile of a head is moved back to start at n - 32, so it overlaps its
// predecessor instead of running past the tensor; the keys it shares with the predecessor are
// recomputed and masked out of the stores.  The CLAMP instance clamps every row index to n - 1
// instead (per-lane piece addresses, a few more vector instructions per tile): it serves heads
// shorter than one tile (n < 32) and paged caches (tiles then start at multiples of 32, so a tile
// lies inside one block, or in two for blocks of 16 rows).
//
// FP8 instances read caches stored as OCP e4m3 bytes with one fp32 scale per (sequence, KV head):
// a 16-byte chunk then holds 16 channels (two k-steps of a lane), rows are half as long, the
// staging takes half the phases, and the scales go into the per-head post factors (k_scale on
// the linear term, its square on the quadratic one) and onto the value norm.
template <int D, int GH, int NW, bool CLAMP, bool FP8 = false>
__global__ __launch_bounds__(NW * 64) void k_score_mfma(ScoreArgs a) {
  constexpr int NKS = D / 16, NJT = D / 32, NF = NJT * (NJT + 1);
  constexpr int NFRAG = GH * NF + 2 * NKS;
  constexpr int EPC = FP8 ? 16 : 8;     // channels per 16-byte chunk
  constexpr int CPR = D / EPC;          // 16-byte chunks per row
  constexpr int RPL = 64 / CPR;         // rows per wave-wide load
  constexpr int NL = 32 / RPL;          // wave-wide loads per 32-key tile
  // Two query heads at d = 256: their triangular fragments fill 144 of the 160 KiB of LDS, so the
  // extra tile's fragments live in registers (one wave per SIMD has 512 of them) and K is staged
  // in four phases through a 4 KiB slab per wave.  Both heads then share one pass over K: every
  // key is loaded, converted and staged once, and the extra tile is computed once for both.
  constexpr bool XR = D == 256 && GH == 2;
  constexpr int NPH = (XR ? 4 : 2) / (FP8 ? 2 : 1);   // staging phases per tile
  constexpr int NLF = XR ? GH * NF : NFRAG;   // fragments held in LDS
  constexpr int CH = CPR / 2;           // chunks per half row (the half a lane holds as B operands)
  constexpr int CPP = CH / NPH;         // of those, staged per phase
  constexpr int RP = CPR / NPH;         // staged chunks per row and phase
  constexpr int RPS = 16 / RP;          // staged rows per 256 bytes (one sweep of the LDS banks)
  extern __shared__ u32x4 smem[];
  const half8* fr = reinterpret_cast<const half8*>(smem);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform: lives in an SGPR
  u32x4* stg = smem + NLF * 64 + wave * (32 * RP);

  // Workgroups are dealt to the chip's 8 dies round-robin by index; the transposition below
  // gives every unit workgroups on all of them.  Together with the tile tickets further down it
  // lets the faster dies (clocks under matrix-core load differ by 15 % and more) take a larger
  // share of a head instead of idling while the slowest one finishes.
  int bid = blockIdx.x;
  if ((gridDim.x & 7u) == 0) bid = (bid & 7) * (int)(gridDim.x >> 3) + (bid >> 3);
  const int unit = bid % a.units;
  const int t2 = bid / a.units;
  const int chunk = t2 % a.nchunk, pass = t2 / a.nchunk;
  const int g0 = pass * GH;
  const bool do_v = pass == 0 && !a.skip_v;

  // Prologue order: tile tickets, then the loads of this (unit, pass)'s fragments, then the
  // first tile's K and V loads (they need the first ticket, which has had the fragment loads'
  // issue time to come back), and only then the fragments' way into LDS and the barrier: the
  // first tile travels while the workgroup assembles its fragments.
  const int ntiles = (int)((a.n + 31) / 32);
  // Up to kTicketWays counters per (unit, pass), each dealing the tiles of one residue class, so
  // that a head scored by hundreds of workgroups (few KV heads per call) does not queue up on one
  // address: an atomic on one address takes about 13 ns.  A workgroup uses the counter of its
  // index modulo the number of counters in use.
  const int ways = max(1, min(kTicketWays, a.nchunk / 8));    // at least 8 workgroups per counter
  const int way = chunk % ways;
  uint32_t* tk = a.tickets + (size_t)unit * a.ticket_stride + pass * kTicketWays + way;
  // The counter's value is only turned into a tile number where it is used, an iteration later:
  // any arithmetic on it here would make the wave wait for the atomic's round trip on the spot
  // (the library is also built with the compiler's wave-aggregation of atomics switched off,
  // which inserts exactly such an immediate use).
  auto grab = [&]() -> int {               // valid in lane 0; v_readfirstlane where it is used
    int t = 0;
    if (lane == 0) t = (int)atomicAdd(tk, 1u);
    return t;
  };
  const int t_cur_raw = grab();
  int t_nxt_raw = grab();
  constexpr int NFIT = XR ? 1 : (NFRAG + NW - 1) / NW;
  u32x4 ftmp[NFIT];
  half8 xf[XR ? 2 * NKS : 1];            // XR: the extra tile's fragments
  const u32x4* fsrc = a.frags + ((size_t)unit * a.passes + pass) * NFRAG * 64;
  if constexpr (!XR) {
#pragma unroll
    for (int it = 0; it < NFIT; ++it) {
      const int i = tid + it * NW * 64;
      ftmp[it] = i < NFRAG * 64 ? fsrc[i] : u32x4{0u, 0u, 0u, 0u};
    }
  } else {
#pragma unroll
    for (int i = 0; i < 2 * NKS; ++i) xf[i] = __builtin_bit_cast(half8, fsrc[(GH * NF + i) * 64 + lane]);
  }
  float pq[GH], pm[GH];
  const float ks = (FP8 && a.kscale) ? a.kscale[unit] : 1.0f;
  const float vs2 = (FP8 && a.vscale) ? a.vscale[unit] * a.vscale[unit] : 1.0f;
#pragma unroll
  for (int g = 0; g < GH; ++g) {
    const bool ok = g0 + g < a.G;
    pq[g] = ok ? a.post[((size_t)unit * a.G + g0 + g) * 2 + 0] * (ks * ks) : 0.f;
    pm[g] = ok ? a.post[((size_t)unit * a.G + g0 + g) * 2 + 1] * ks : 0.f;
  }

  const int r = lane & 31, hh = lane >> 5;
  const int lrow = lane / CPR, lch = lane % CPR;
  // Tiles of 32 keys are handed out by a ticket counter per (unit, pass), last tile of the head
  // first: at any moment the waves of a unit stream one contiguous region (which spreads the
  // traffic over all HBM channels), and what the pass reads last, the early rows, is what the
  // compaction that follows reads first, while it may still be in the memory-side cache.
  // A wave holds two tickets ahead (the tile it prefetches and the one after), so the counter's
  // round trip never shows.
  auto tile_key = [&](int ticket) -> long long { return (long long)(ntiles - 1 - ticket) * 32; };
  const u32x4* kbase = a.k + (size_t)unit * a.n_cap * CPR;
  const u32x4* vbase = a.v + (size_t)unit * a.n_cap * CPR;
  // CLAMP: where the tile at key0 lies -- the tensor's (or, for paged caches, the pool's) row that
  // holds tile row 0 and the one that holds tile row 16 (blocks of 16 rows: a tile spans two of
  // them; the lookups are wave-uniform) -- and the 16-byte piece this lane fetches with wave-wide
  // load j, rows past the end of the head clamped to its last row.
  auto tile_rows = [&](long long k0, size_t& r0, size_t& r1) {
    if (a.pm.table) {
      r0 = paged_row(a.pm, unit, (int)k0);
      r1 = (a.pm.sh < 5 && k0 + 16 < a.n) ? paged_row(a.pm, unit, (int)k0 + 16) : r0 + 16;
    } else {
      r0 = (size_t)unit * a.n_cap + k0;
      r1 = r0 + 16;
    }
  };
  auto lane_piece = [&](long long k0, int j, size_t r0, size_t r1) -> size_t {
    const int lim = (int)min((long long)31, a.n - 1 - k0);
    const int re = min(j * RPL + lrow, lim);
    return (re < 16 ? r0 + re : r1 + (re - 16)) * CPR + lch;
  };

  // One 32-key tile = NL wave-wide 16-byte loads per tensor, addressed as (uniform tile base)
  // + lane*16 + j*1024 so that the address arithmetic stays on the scalar unit.  K and V are
  // read once: the loads carry the non-temporal hint, which keeps them from pushing the logits
  // (read back by the finalize pass) and the fragments out of the caches -- 5 % on this kernel,
  // 14 % on the finalize pass.  At d = 256 a KV head's query heads take one pass over K each
  // (their fragments do not fit in LDS together); the passes run side by side, and there K is
  // loaded with the default policy so that the second reader finds it in a cache (5 %).
  constexpr bool kNtK = D <= 128 || XR;
  u32x4 kraw[NL], vraw[NL];
  auto tile_base = [&](long long k0) -> long long {          // first row actually loaded
    return (!CLAMP && k0 + 32 > a.n) ? a.n - 32 : k0;
  };
#pragma unroll
  for (int j = 0; j < NL; ++j) { kraw[j] = u32x4{0u, 0u, 0u, 0u}; vraw[j] = u32x4{0u, 0u, 0u, 0u}; }
  int t_cur = __builtin_amdgcn_readfirstlane(t_cur_raw) * ways + way;
  long long key0 = t_cur < ntiles ? tile_key(t_cur) : 0;
  if (t_cur < ntiles) {                                      // first tile: plain loads
    if constexpr (!CLAMP) {
      const u32x4* kp = kbase + tile_base(key0) * CPR;
      const u32x4* vp = vbase + tile_base(key0) * CPR;
#pragma unroll
      for (int j = 0; j < NL; ++j) kraw[j] = kNtK ? __builtin_nontemporal_load(&kp[j * 64 + lane]) : kp[j * 64 + lane];
      if (do_v) {
#pragma unroll
        for (int j = 0; j < NL; ++j) vraw[j] = __builtin_nontemporal_load(&vp[j * 64 + lane]);
      }
    } else {
      size_t r0, r1;
      tile_rows(key0, r0, r1);
#pragma unroll
      for (int j = 0; j < NL; ++j) {
        kraw[j] = a.k[lane_piece(key0, j, r0, r1)];
        if (do_v) vraw[j] = a.v[lane_piece(key0, j, r0, r1)];
      }
    }
  }

  if constexpr (!XR) {
#pragma unroll
    for (int it = 0; it < NFIT; ++it) {
      const int i = tid + it * NW * 64;
      if (i < NFRAG * 64) smem[i] = ftmp[it];
    }
  } else {
    // 144 fragments through a few registers at a time (the prologue runs once per workgroup)
    static_assert(!XR || NLF % (4 * NW) == 0, "fragment count");
    for (int b = 0; b < NLF / NW; b += 4) {
      u32x4 t[4];
#pragma unroll
      for (int it = 0; it < 4; ++it) t[it] = fsrc[tid + (b + it) * NW * 64];
#pragma unroll
      for (int it = 0; it < 4; ++it) smem[tid + (b + it) * NW * 64] = t[it];
    }
  }
  __syncthreads();

  // Results of a tile are stored one iteration later, right after the staging of the next
  // tile: global stores share the in-order counter of the loads, and stores issued while
  // loads are pending make every later wait for a load also wait for the store.
  float lg_prev[GH], vsq_prev = 0.f;
#pragma unroll
  for (int g = 0; g < GH; ++g) lg_prev[g] = 0.f;
  long long key_prev = 0;
  bool have_prev = false;
  auto store_prev = [&]() {
    const long long b0 = tile_base(key_prev);
    const long long key = b0 + r;
    if (hh == 0 && key >= key_prev && key < a.n) {
#pragma unroll
      for (int g = 0; g < GH; ++g)
        if (g0 + g < a.G) a.logits[((size_t)unit * a.G + g0 + g) * a.n + key] = lg_prev[g];
    }
    if (do_v) {
      const long long row = b0 + lch * RPL + lrow;
      if (lch < NL && row >= key_prev && row < a.n)
        a.vnorm[(size_t)unit * a.n + row] = __builtin_amdgcn_sqrtf(FP8 ? vsq_prev * vs2 : vsq_prev);
    }
  };

  for (; t_cur < ntiles; key0 = tile_key(t_cur)) {
    // ---- K: coalesced registers -> LDS -> MFMA B layout.  Two phases, each staging one half
    //      of every lane's k-steps for all 32 rows (half-size buffer, all lanes busy).
    half8 Kh[NKS];
#pragma unroll
    for (int hf = 0; hf < NPH; ++hf) {
      if (((lch % CH) / CPP) == hf) {
        const int sc = (lch / CH) * CPP + (lch % CPP);
#pragma unroll
        for (int j = 0; j < NL; ++j) {
          const int rho = j * RPL + lrow;
          stg[rho * RP + (sc ^ ((rho / RPS) & (RP - 1)))] = kraw[j];
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int q = 0; q < CPP; ++q) {
        const int sc = hh * CPP + q;
        const u32x4 piece = stg[r * RP + (sc ^ ((r / RPS) & (RP - 1)))];
        if constexpr (FP8) fp8x16_to_half8x2(piece, Kh[2 * (hf * CPP + q)], Kh[2 * (hf * CPP + q) + 1]);
        else Kh[hf * CPP + q] = bf16x8_to_half8(piece);
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
    if (have_prev) store_prev();

    // ---- where the next tile comes from.  Without a next tile the loads below still run (the
    //      matrix-core phase is one straight-line block) but all lanes read the head's first
    //      16 bytes: no traffic to speak of.
    const int t_nxt = __builtin_amdgcn_readfirstlane(t_nxt_raw) * ways + way;
    const bool has_next = t_nxt < ntiles;
    const long long nkey0 = has_next ? tile_key(t_nxt) : 0;
    const u32x4* kp_n = has_next ? kbase + tile_base(nkey0) * CPR : kbase;
    const u32x4* vp_n = (has_next && do_v) ? vbase + tile_base(nkey0) * CPR : vbase;
    const int kl = has_next ? lane : 0, vl = (has_next && do_v) ? lane : 0;
    const int kj = has_next ? 64 : 0, vj = (has_next && do_v) ? 64 : 0;
    size_t noff[CLAMP ? NL : 1];        // CLAMP: this lane's pieces of the next tile's loads
    if constexpr (CLAMP) {
      size_t r0 = 0, r1 = 0;
      if (has_next) tile_rows(nkey0, r0, r1);
      kp_n = a.k;                       // (without a next tile: piece 0 of the tensor, as above)
      vp_n = a.v;
#pragma unroll
      for (int j = 0; j < NL; ++j) noff[j] = has_next ? lane_piece(nkey0, j, r0, r1) : (size_t)0;
    }

    // ---- matrix-core phase: NS = 2*NKS + GH*NF steps, one LDS fragment and one MFMA each.
    //   steps [0, NKS)       extra tile, rows g / GH+g = fp16 head / tail of mu, times k
    //   steps [NKS, 2NKS)    extra tile, rows 2GH+g = rounding residual of diag(M), times k^2/256
    //   then per output tile t = (head g, 32 output channels jt): 2jt+2 steps over the k-steps on
    //   or below the diagonal; its accumulator is then dotted with k (16 FMAs).
    // Everything else of the iteration rides in the shadow of the MFMAs:
    //   * fragments are fetched PD steps ahead into a register ring;
    //   * the 16 FMAs of tile t are issued four per step during steps end(t)+2 .. end(t)+5
    //     (three accumulators rotate, so a tile is not rewritten before it has been read);
    //   * the squared norm of V chunk j is formed at step j;
    //   * the 2*NL global loads of the next tile are spread over the steps after the extra
    //     tile, one at a time, so they never queue up in front of the memory pipeline.
    // The matrix-core phase runs at a raised wave priority: when the other wave of the SIMD is in
    // its staging or store phase, this wave's instructions are issued first and the matrix pipeline
    // stays fed (4 % on the kernel; the level, 1 to 3, makes no difference).
    __builtin_amdgcn_s_setprio(1);
    float lin[GH], partial[GH], vsq = 0.f;
    static_for<GH>([&](auto g_) { partial[decltype(g_)::value] = 0.f; lin[decltype(g_)::value] = 0.f; });
    {
      // (the five-head instance prefetches one fragment less: with four it spills, and a kernel that
      // needs scratch memory pays for it at every launch)
      constexpr int NX = 2 * NKS, NS = NX + GH * NF, NT = GH * NJT, PD = GH >= 5 ? 3 : kFragPrefetch;
      half8 fb[PD + 1];
      floatx16 ex, accb[3];
      // step f reads LDS fragment lfrag(f) into ring slot f % (PD + 1); with the extra tile in
      // registers the LDS stream starts at step NX
      constexpr int F0 = XR ? NX : 0;
      auto lfrag = [](int f) constexpr { return XR ? f - NX : step_frag<GH, NF, NX>(f); };
      static_for<PD>([&](auto i_) {
        constexpr int i = decltype(i_)::value;
        fb[(F0 + i) % (PD + 1)] = fr[lfrag(F0 + i) * 64 + lane];
      });
      __builtin_amdgcn_sched_barrier(0);
      // FMAs 4q .. 4q+3 of the dot product of tile tt
      auto dot4 = [&](auto tt_, auto q_) {
        constexpr int tt = decltype(tt_)::value, q = decltype(q_)::value;
        constexpr int g = tt / NJT, jt = tt % NJT;
        static_for<4>([&](auto v_) {
          constexpr int v = 4 * q + decltype(v_)::value;
          constexpr int x = jt * 16 + v;
          partial[g] = fmaf(accb[tt % 3][v], (float)Kh[x / 8][x % 8], partial[g]);
        });
        // pin: otherwise the optimiser sinks the dot products to the end of the phase and keeps
        // every accumulator tile alive
        if constexpr (q == 3) asm volatile("" : "+v"(partial[g]));
      };
      static_for<NS + 6>([&](auto f_) {
        constexpr int f = decltype(f_)::value;
        if constexpr (f < NS) {
          if constexpr (f + PD < NS && f >= F0)
            fb[(f + PD) % (PD + 1)] = fr[lfrag(f + PD) * 64 + lane];
          half8 A;
          if constexpr (XR && f < NX) A = xf[f];
          else A = fb[f % (PD + 1)];
          constexpr floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
          if constexpr (f < NKS) {
            ex = __builtin_amdgcn_mfma_f32_32x32x16_f16(A, Kh[f], f == 0 ? zero : ex, 0, 0, 0);
          } else if constexpr (f < NX) {
            half8 t = Kh[f - NKS] * (_Float16)0.0625f;
            // |k| > 4096 would square to infinity (and infinity times a zero residual is NaN): the
            // correction saturates there instead, an error far below the rounding it corrects
            t = __builtin_elementwise_min(t * t, (half8)(_Float16)65504.0f);
            ex = __builtin_amdgcn_mfma_f32_32x32x16_f16(A, t, ex, 0, 0, 0);
          } else {
            constexpr int m = f - NX, g = m / NF, rem = m % NF;
            constexpr int jt = tri_jt(rem), kt = rem - jt * (jt + 1), t = g * NJT + jt;
            accb[t % 3] = __builtin_amdgcn_mfma_f32_32x32x16_f16(A, Kh[kt], kt == 0 ? zero : accb[t % 3], 0, 0, 0);
          }
        }
        // ---- vector work placed in this step
        // The ticket after next is drawn right after the last V chunk has been consumed: the waits
        // for the V chunks cover everything issued before them, so a ticket drawn earlier would be
        // waited for there; drawn here it is older than every load of the next tile and has
        // returned long before it is read.
        if constexpr (f == NL) t_nxt_raw = grab();
        if constexpr (f < NL) {                   // V chunk f: lane lch == f keeps its row's sum
          const float ss = group_sum<CPR>(FP8 ? sumsq_fp8x16(vraw[f]) : sumsq_bf16x8(vraw[f]));
          vsq = lch == f ? ss : vsq;
        }
        if constexpr (f == NX + 1) {              // rows of the extra tile, two steps after its end
          static_for<GH>([&](auto g_) {
            constexpr int g = decltype(g_)::value;
            float e = 0.f;
            if (hh == ROW_HH(g)) e += ex[ROW_V(g)] * pm[g];
            if (hh == ROW_HH(GH + g)) e += ex[ROW_V(GH + g)] * pm[g];
            if (hh == ROW_HH(2 * GH + g)) e += ex[ROW_V(2 * GH + g)] * (256.0f * pq[g]);
            lin[g] = e;
          });
        }
        static_for<NT>([&](auto tt_) {
          constexpr int tt = decltype(tt_)::value;
          constexpr int e = NX + (tt / NJT) * NF + (tt % NJT + 1) * (tt % NJT + 2) - 1;   // last step of tile tt
          if constexpr (f >= e + 2 && f < e + 6) dot4(tt_, std::integral_constant<int, f - e - 2>{});
        });
        // ---- loads of the next tile that belong to this step (K first, then V)
        static_for<2 * NL>([&](auto i_) {
          constexpr int i = decltype(i_)::value;
          if constexpr (f < NS && load_slot<NX, NS, NL>(i) == f) {
            if constexpr (CLAMP) {
              if constexpr (i < NL) kraw[i] = kNtK ? __builtin_nontemporal_load(&kp_n[noff[i]]) : kp_n[noff[i]];
              else vraw[i - NL] = __builtin_nontemporal_load(&vp_n[do_v ? noff[i - NL] : (size_t)0]);
            } else {
              if constexpr (i < NL) kraw[i] = kNtK ? __builtin_nontemporal_load(&kp_n[i * kj + kl]) : kp_n[i * kj + kl];
              else vraw[i - NL] = __builtin_nontemporal_load(&vp_n[(i - NL) * vj + vl]);
            }
          }
        });
        // Nothing may move across a step: the program order written above -- fragment read PD
        // steps ahead, one MFMA, the vector / memory work that rides in its shadow -- is the
        // software pipeline.  (Left alone, the scheduler sinks every LDS read next to its MFMA.)
        __builtin_amdgcn_sched_barrier(0);
      });
    }
    __builtin_amdgcn_s_setprio(0);
    // The softmax over keys (Eq. 8) is not this kernel's business: the (max, sum exp) partials are
    // taken from the stored logits per fixed block of keys by a pass of their own (k_lse_part), so
    // they do not depend on which wave scored which tile.
#pragma unroll
    for (int g = 0; g < GH; ++g) lg_prev[g] = sum_halves(partial[g] * pq[g] + lin[g]);
    vsq_prev = vsq;
    key_prev = key0;
    have_prev = true;
    t_cur = t_nxt;
  }
  if (have_prev) store_prev();

}

template <int D, int GH, int NW, bool CLAMP, bool FP8 = false>
inline hipError_t launch_one(const ScoreArgs& a, const ScorePlan& sp, hipStream_t st) {
  static_assert(!FP8 || D >= 128, "fp8 rows of 64 channels are not covered");
  auto kern = k_score_mfma<D, GH, NW, CLAMP, FP8>;
  static LdsOptIn opt;                    // one per kernel instance
  hipError_t e = opt.ensure(reinterpret_cast<const void*>(kern), sp.lds_bytes);
  if (e != hipSuccess) return e;
  int grid = a.units * a.nchunk * a.passes;
  kern<<<grid, NW * 64, sp.lds_bytes, st>>>(a);
  return hipGetLastError();
}


// per-head-dimension dispatchers (ea_score_d64.hip, ea_score_d128.hip, ea_score_d128b.hip,
// ea_score_d256.hip); each returns hipErrorInvalidValue for a (GH, NW) it does not hold
hipError_t launch_score_mfma_d64(const ScoreArgs& a, const ScorePlan& sp, hipStream_t st);
hipError_t launch_score_mfma_d128(const ScoreArgs& a, const ScorePlan& sp, hipStream_t st);
hipError_t launch_score_mfma_d128b(const ScoreArgs& a, const ScorePlan& sp, hipStream_t st);
hipError_t launch_score_mfma_d256(const ScoreArgs& a, const ScorePlan& sp, hipStream_t st);
// ea_score_fp8.hip: the instances for caches stored as e4m3 bytes (d = 128 and 256)
hipError_t launch_score_mfma_fp8(int D, const ScoreArgs& a, const ScorePlan& sp, hipStream_t st);
hipError_t launch_score_mfma_fp8b(int D, const ScoreArgs& a, const ScorePlan& sp, hipStream_t st);
// ea_score_hw.hip: fragments in registers, one wavefront per query head (d = 128, groups of four)
hipError_t launch_score_hw(const ScoreArgs& a, const ScorePlan& sp, hipStream_t st);

}  // namespace ea
