// Score pass A for a group of four query heads at d = 128 with the Sigma fragments held in
// REGISTERS (Eq. 7 of the paper: l_g = mu_g.k/sqrt(d) + k^T Sigma_g k/(2d) for every cached key).
//
// The LDS-fragment kernel (ea_score_mfma.h) reads one 1 KiB fragment from LDS per matrix-core
// instruction; with four SIMDs that is the whole LDS bandwidth of a CU at the matrix cores'
// peak.  Here a workgroup is four wavefronts, one per query head of the GQA group: each keeps 16
// of its own head's 20 triangular fragments in registers for the whole kernel (the other four,
// and its share of the extra tile, are re-read from LDS per tile), and the four of them share
// ONE tile of 32 keys per iteration, converted to fp16 once and laid out in LDS as matrix-core
// B operands.  Per tile a wavefront reads 18 KiB from LDS for 24 matrix-core instructions
// instead of 24 KiB, two such workgroups fit a CU, and the softmax partials belong to fixed
// blocks of 128 keys (a quarter of the partials the per-tile scheme leaves to the finalize pass).
//
//   * K tile: each wavefront loads a quarter of the next tiles' rows (coalesced 16-byte loads,
//     held in registers two to three iterations ahead), converts them bf16 -> fp16 and writes
//     them to the LDS tile  [16-byte chunk j of the row][key r]  with a chunk stride of 33 slots
//     (conflict-free both ways, and every address a lane needs is one base plus a constant);
//     lane (r, hh) reads chunk hh*8 + kt of key r as its B operand of k-step kt.
//   * V rows: same quarter split; squared norms straight from the coalesced registers.
//   * extra tile (rows: fp16 head / tail of mu_g, rounding residual of diag(Sigma_g) times k^2):
//     its 16 k-steps are split over the four wavefronts, four each; the partial row sums go
//     through LDS and every wavefront picks up its own head's three rows one iteration later.
//   * softmax partials: a ticket is a block of `tpt` consecutive tiles; a wavefront keeps the
//     running (max, sum exp) of its head over the block and stores it to the block's slot, so
//     the finalize pass combines the same numbers in the same order on every run.
//
// Fragment layout, scales and the meaning of `post` are those of k_prep_frags (ea_stats.hip).
#include "ea_score_mfma.h"

namespace ea {

constexpr int kHwLookahead = 3;      // the load cursor runs this many tiles ahead of the tile being scored

template <int D>
__global__ __launch_bounds__(256, 2) void k_score_hw(ScoreArgs a) {
  static_assert(D == 128, "instance for head dimension 128");
  constexpr int NKS = 8, NF = 20, GH = 4, CPR = 16, NFRAG = GH * NF + 2 * NKS;
  constexpr int LA = kHwLookahead;
  __shared__ u32x4 s_k[2][16 * 33];          // fp16 K tile [16-byte chunk j of the row][key r], chunk stride 33: double buffered
  __shared__ float s_p[2][4][GH][64];        // extra-tile partial rows: [buffer][source wave][head][lane]
  __shared__ int s_tk[8];                    // ring of drawn blocks, by draw ordinal
  __shared__ u32x4 s_x[2 * NKS * 64];        // the extra tile's 16 fragments (read back four per wave and tile)
  __shared__ u32x4 s_f0[GH * 4 * 64];        // each head's first four fragments (tile 0, half of tile 1): registers are short by about that much
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 31, hh = lane >> 5;
  const int lrow = lane >> 4, lch = lane & 15;

  int bid = blockIdx.x;
  if ((gridDim.x & 7u) == 0) bid = (bid & 7) * (int)(gridDim.x >> 3) + (bid >> 3);   // every unit on all dies
  const int unit = bid % a.units;
  const int t2 = bid / a.units;
  const int chunk = t2 % a.nchunk, pass = t2 / a.nchunk;
  const int g0 = pass * GH;
  const bool do_v = pass == 0 && !a.skip_v;
  const int tpt = a.tpt, tsh = tpt == 4 ? 2 : 0;
  const int ntiles = (int)((a.n + 31) / 32);
  const int nblocks = (ntiles + tpt - 1) >> tsh;
  const int ways = max(1, min(kTicketWays, a.nchunk / 8));
  const int way = chunk % ways;
  uint32_t* tk = a.tickets + (size_t)unit * a.ticket_stride + pass * kTicketWays + way;

  // ---- prologue: first draws, fragments, first three tiles
  constexpr int NPRE = LA + 2;               // at most this many ordinals are needed before the loop's own draws arrive
  const int npre = ((LA + 1) >> tsh) + 1;
  if (tid == 0) {
    uint32_t raw[NPRE];
#pragma unroll
    for (int i = 0; i < NPRE; ++i) raw[i] = i < npre ? atomicAdd(tk, 1u) : 0u;
#pragma unroll
    for (int i = 0; i < NPRE; ++i)
      if (i < npre) s_tk[i] = nblocks - 1 - ((int)raw[i] * ways + way);
  }
  half8 F[NF];
  {
    const u32x4* src = a.frags + ((size_t)unit * a.passes + pass) * NFRAG * 64;
#pragma unroll
    for (int i = 4; i < NF; ++i) F[i] = __builtin_bit_cast(half8, src[(w * NF + i) * 64 + lane]);
#pragma unroll
    for (int i = 0; i < 4; ++i) s_f0[(w * 4 + i) * 64 + lane] = src[(w * NF + i) * 64 + lane];
#pragma unroll
    for (int i = 0; i < 4; ++i) s_x[tid + 256 * i] = src[GH * NF * 64 + tid + 256 * i];
  }
  // post[2g] = 1 / (2 d sM_g), post[2g+1] = 1 / (sqrt(d) smu_g)
  float pm[GH], cq[GH];
  float pq_mine = 0.f;
#pragma unroll
  for (int g = 0; g < GH; ++g) {
    const float pq = a.post[((size_t)unit * a.G + g0 + g) * 2 + 0];
    pm[g] = a.post[((size_t)unit * a.G + g0 + g) * 2 + 1];
    cq[g] = 256.0f * pq;
    pq_mine = w == g ? pq : pq_mine;
  }
  __syncthreads();

  // All row arithmetic is 32-bit (n <= 2^26); a tile's global address is a per-tile scalar base
  // plus a per-lane offset that never changes.  The loop body is ONE basic block (the instruction
  // scheduler interleaves matrix-core and vector work only inside a block), so nothing in it is
  // conditional: stores that must not happen go to a dump area instead (the upper half of the
  // logit scratch, which only the fp32 path uses), loads without a tile read the head's first rows.
  const int n = (int)a.n;
  const char* kbase = (const char*)(a.k + (size_t)unit * a.n_cap * CPR);
  const char* vbase = (const char*)(a.v + (size_t)unit * a.n_cap * CPR);
  const uint32_t ld_off = (uint32_t)((2 * w) * 1024 + lane * 16);
  const uint32_t ld_off_v = do_v ? ld_off : 0u;           // later passes: every lane on the same 16 bytes
  float* lg_out = a.logits + ((size_t)unit * a.G + g0 + w) * a.n;
  float* vn_out = a.vnorm + (size_t)unit * a.n;
  float2* part_out = a.part + ((size_t)unit * a.G + g0 + w) * a.npart;
  float* dump = a.logits + (size_t)a.units * a.G * a.n;   // at least n floats; indexed like a head's rows; contents never read
  float* vn_eff = do_v ? vn_out : dump;       // later passes hold no V rows: their "norms" go to the dump

  // A tile is one int: its index (rows [32 t, 32 t + 32)), -1 = no more work; an index >= ntiles is
  // padding of the head's last, ragged, block (scored on dummy data, nothing stored).
  int lc_ord = 0, lc_left = tpt;
  int lc_tile;
  {
    const int blk = s_tk[0];
    lc_tile = blk < 0 ? -1 : blk << tsh;
  }
  // cand: the ring entry of the next ordinal, read at the top of every iteration whether it is
  // needed or not (it is only looked at when the current block is used up, and by then published)
  auto next_tile = [&](int cand) -> int {
    const bool fresh = lc_left == 0;
    int blk = cand >= nblocks ? -1 : cand;   // never leave the head, whatever the ring holds
    const int first = blk < 0 ? -1 : blk << tsh;
    lc_ord += fresh ? 1 : 0;
    lc_tile = fresh ? first : lc_tile;
    lc_left = fresh ? tpt : lc_left;
    const int t = lc_tile;
    lc_tile += lc_tile >= 0 ? 1 : 0;
    --lc_left;
    return t;
  };
  auto ring_next = [&]() -> int { return __builtin_amdgcn_readfirstlane(s_tk[(lc_ord + 1) & 7]); };
  auto is_real = [&](int t) -> bool { return (unsigned)t < (unsigned)ntiles; };
  // first row actually loaded: the head's last tile is moved back to end at row n
  auto base_row = [&](int t) -> int { return is_real(t) ? min(t * 32, n - 32) : 0; };

  u32x4 rawK[2][2], rawV[2][2];              // [tile parity][load]: this wave's quarter of a tile
  auto issue_loads = [&](auto slot_, int t) {
    constexpr int SL = decltype(slot_)::value;
    const size_t off = (size_t)base_row(t) * (CPR * 16);
    const char* kp = kbase + off;
    const char* vp = vbase + (do_v ? off : (size_t)0);
#pragma unroll
    for (int j = 0; j < 2; ++j)
      rawK[SL][j] = __builtin_nontemporal_load((const u32x4*)(kp + (ld_off + j * 1024)));
#pragma unroll
    for (int j = 0; j < 2; ++j)
      rawV[SL][j] = __builtin_nontemporal_load((const u32x4*)(vp + (ld_off_v + (do_v ? j * 1024 : 0))));
  };
  // raw quarter -> fp16 rows of the LDS tile `buf`; value norms of the quarter's rows
  const int st_idx0 = lch * 33 + 8 * w + lrow, st_idx1 = st_idx0 + 4;
  const int vn_row = 8 * w + 4 * (lch & 1) + lrow;   // even / odd lanes of a row group store the norm of load 0 / 1
  auto stage_tile = [&](auto slot_, int buf, int t) {
    constexpr int SL = decltype(slot_)::value;
    s_k[buf][st_idx0] = __builtin_bit_cast(u32x4, bf16x8_to_half8(rawK[SL][0]));
    s_k[buf][st_idx1] = __builtin_bit_cast(u32x4, bf16x8_to_half8(rawK[SL][1]));
    const float s0 = group_sum<16>(sumsq_bf16x8(rawV[SL][0]));
    const float s1 = group_sum<16>(sumsq_bf16x8(rawV[SL][1]));
    // Stored without a condition: the eight lanes that share a row write the same value, rows that
    // a moved-back last tile shares with its predecessor get the same bits again (same data, same
    // arithmetic), and so do rows 0..31 when there is no tile (the loads then read those rows).
    vn_eff[base_row(t) + vn_row] = __builtin_amdgcn_sqrtf((lch & 1) ? s1 : s0);
  };

  int t_cur = next_tile(ring_next()), t_n1 = next_tile(ring_next()), t_n2 = next_tile(ring_next());
  issue_loads(std::integral_constant<int, 0>{}, t_cur);
  issue_loads(std::integral_constant<int, 1>{}, t_n1);
  stage_tile(std::integral_constant<int, 0>{}, 0, t_cur);
  issue_loads(std::integral_constant<int, 0>{}, t_n2);
  __syncthreads();

  float m_run = -INFINITY, s_run = 0.f;      // this head's softmax state over the current block
  float quad_prev = 0.f;
  int t_prev = -1;
  uint32_t pend = 0;                         // wave 0, lane 0: the draw waiting to be published
  int s = 0;

  const int kh_idx = (hh * 8) * 33 + r;        // lane's B operand of k-step kt: s_k[.][kh_idx + kt * 33]
  auto body = [&](auto pb_) {
    constexpr int PB = decltype(pb_)::value;
    constexpr floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // ---- LDS reads of the iteration: ring entry, B operands, and the previous tile's extra-tile
    //      rows from all four wavefronts
    const int cand = ring_next();
    half8 Kh[NKS], Kx[2], XL[2], XS[2], sq[2];
#pragma unroll
    for (int kt = 0; kt < NKS; ++kt)
      Kh[kt] = __builtin_bit_cast(half8, s_k[PB][kh_idx + kt * 33]);
    const float lin = (s_p[PB ^ 1][0][w][lane] + s_p[PB ^ 1][1][w][lane]) +
                      (s_p[PB ^ 1][2][w][lane] + s_p[PB ^ 1][3][w][lane]);
    __builtin_amdgcn_sched_barrier(0);

    // ---- 24 steps, one matrix-core instruction each, in this order:
    //   0..7   output tile 3 of the head's quadratic form (k-steps 0..7: on or below the diagonal)
    //   8..13  tile 2     14..17  tile 1     18..19  tile 0
    //   20..23 this wave's four steps of the extra tile (two on k, two on k^2 / 256)
    // and the vector / memory work placed in the shadow of each (nothing moves across a step):
    //   0..1   the previous tile's logit, its store and the running softmax
    //   2..6   staging of tile s+1 (bf16 -> fp16 into the other LDS buffer, value norms)
    //   7      request of tile s+3 into the registers just staged
    //   the dot product of a finished tile with k two and three steps after its last instruction
    //   16     fetch of the extra tile's operands; 18, 21 their squares
    floatx16 acc3, acc2, acc1, acc0, ex;
    float partial = 0.f, vs0 = 0.f, vs1 = 0.f, lg = 0.f;
    int t_n3 = -1;
    auto dot8 = [&](auto jt_, auto h_, const floatx16& acc) {
      constexpr int jt = decltype(jt_)::value, h = decltype(h_)::value;
      static_for<8>([&](auto v_) {
        constexpr int v = 8 * h + decltype(v_)::value;
        constexpr int x = jt * 16 + v;
        partial = fmaf(acc[v], (float)Kh[x / 8][x % 8], partial);
      });
      asm volatile("" : "+v"(partial));      // pin: left alone, the dot products sink to the end of the block
    };
    using C0 = std::integral_constant<int, 0>;
    using C1 = std::integral_constant<int, 1>;
    using C2 = std::integral_constant<int, 2>;
    using C3 = std::integral_constant<int, 3>;
    static_for<24>([&](auto f_) {
      constexpr int f = decltype(f_)::value;
      // -- the step's matrix-core instruction
      if constexpr (f < 8) acc3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(F[12 + f], Kh[f], f == 0 ? zero : acc3, 0, 0, 0);
      else if constexpr (f < 14) acc2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(F[6 + f - 8], Kh[f - 8], f == 8 ? zero : acc2, 0, 0, 0);
      else if constexpr (f < 18) acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(F[2 + f - 14], Kh[f - 14], f == 14 ? zero : acc1, 0, 0, 0);
      else if constexpr (f < 20) acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(F[f - 18], Kh[f - 18], f == 18 ? zero : acc0, 0, 0, 0);
      else if constexpr (f < 22) ex = __builtin_amdgcn_mfma_f32_32x32x16_f16(XL[f - 20], Kx[f - 20], f == 20 ? zero : ex, 0, 0, 0);
      else ex = __builtin_amdgcn_mfma_f32_32x32x16_f16(XS[f - 22], sq[f - 22], ex, 0, 0, 0);
      // -- vector and memory work of the step
      if constexpr (f == 0) {
        // the previous tile's logit: its quadratic part was formed last iteration, the extra-tile
        // rows of all four wavefronts are in LDS since the barrier
        lg = sum_halves(fmaf(quad_prev, pq_mine, lin));
        // stored without a per-lane condition (see the value norms); only the very first iteration,
        // which has no previous tile, must not reach the logits
        float* dst = t_prev >= 0 ? lg_out : dump;
        dst[base_row(t_prev) + r] = lg;
      }
      if constexpr (f == 1) {
        const int key = base_row(t_prev) + r;
        const bool valid = is_real(t_prev) && key >= t_prev * 32;      // key < n by construction
        const float mn = valid ? fmaxf(m_run, lg) : m_run;
        const float e1 = __expf(m_run - mn), e2 = valid ? __expf(lg - mn) : 0.f;
        s_run = fmaf(s_run, mn == -INFINITY ? 0.f : e1, e2);
        m_run = mn;
      }
      if constexpr (f == 2) s_k[PB ^ 1][st_idx0] = __builtin_bit_cast(u32x4, bf16x8_to_half8(rawK[PB ^ 1][0]));
      if constexpr (f == 3) s_k[PB ^ 1][st_idx1] = __builtin_bit_cast(u32x4, bf16x8_to_half8(rawK[PB ^ 1][1]));
      if constexpr (f == 4) vs0 = group_sum<16>(sumsq_bf16x8(rawV[PB ^ 1][0]));
      if constexpr (f == 5) vs1 = group_sum<16>(sumsq_bf16x8(rawV[PB ^ 1][1]));
      if constexpr (f == 6) {
        // Stored without a condition: the eight lanes that share a row write the same value, rows
        // that a moved-back last tile shares with its predecessor get the same bits again (same
        // data, same arithmetic), and so do rows 0..31 when there is no tile (the loads then read
        // those rows).
        vn_eff[base_row(t_n1) + vn_row] = __builtin_amdgcn_sqrtf((lch & 1) ? vs1 : vs0);
      }
      if constexpr (f == 7) {
        t_n3 = next_tile(cand);
        issue_loads(std::integral_constant<int, PB ^ 1>{}, t_n3);
      }
      if constexpr (f == 11) {
#pragma unroll
        for (int jx = 2; jx < 4; ++jx) F[jx] = __builtin_bit_cast(half8, s_f0[(w * 4 + jx) * 64 + lane]);
      }
      if constexpr (f == 9) dot8(C3{}, C0{}, acc3);
      if constexpr (f == 10) dot8(C3{}, C1{}, acc3);
      if constexpr (f == 15) dot8(C2{}, C0{}, acc2);
      if constexpr (f == 16) {
        dot8(C2{}, C1{}, acc2);
#pragma unroll
        for (int jx = 0; jx < 2; ++jx) {
          Kx[jx] = __builtin_bit_cast(half8, s_k[PB][kh_idx + (2 * w + jx) * 33]);
          XL[jx] = __builtin_bit_cast(half8, s_x[(2 * w + jx) * 64 + lane]);
          XS[jx] = __builtin_bit_cast(half8, s_x[(NKS + 2 * w + jx) * 64 + lane]);
          F[jx] = __builtin_bit_cast(half8, s_f0[(w * 4 + jx) * 64 + lane]);
        }
      }
      if constexpr (f == 18 || f == 21) {
        constexpr int jx = f == 18 ? 0 : 1;
        const half8 t = Kx[jx] * (_Float16)0.0625f;
        // saturate instead of overflowing for |k| > 4096: infinity times a zero residual is NaN
        sq[jx] = __builtin_elementwise_min(t * t, (half8)(_Float16)65504.0f);
      }
      if constexpr (f == 19) dot8(C1{}, C0{}, acc1);
      if constexpr (f == 20) dot8(C1{}, C1{}, acc1);
      if constexpr (f == 22) dot8(C0{}, C0{}, acc0);
      if constexpr (f == 23) dot8(C0{}, C1{}, acc0);
    });
    // the order asked of the scheduler: one matrix-core instruction, then the vector and memory
    // work that fits in its shadow
    static_for<24>([&](auto) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // MFMA
      __builtin_amdgcn_sched_group_barrier(0x002, 7, 0);     // VALU
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);     // LDS read
      __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);     // LDS write
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);     // global load
      __builtin_amdgcn_sched_group_barrier(0x040, 1, 0);     // global store
    });
    __builtin_amdgcn_sched_barrier(0);
    // lower half-wave: rows g (head of mu_g) and 8 + g (diagonal residual); upper half-wave:
    // rows 4 + g (tail of mu_g) and 12 + g (empty fragment rows: exact zeros); the halves are
    // added when the logit is formed
#pragma unroll
    for (int g = 0; g < GH; ++g) s_p[PB][w][g][lane] = fmaf(ex[4 + g], cq[g], ex[g] * pm[g]);

    // ---- tail: the parts that need a branch
    const int t_done = t_prev;               // the tile whose logit was just formed
    if (t_done >= 0 && (t_done & (tpt - 1)) == tpt - 1) {     // it was the last of its block (uniform)
      const float m = max_lanes32(m_run);
      const float sm = sum_lanes32(m_run == -INFINITY ? 0.f : s_run * __expf(m_run - m));
      if (lane == 0) part_out[t_done >> tsh] = make_float2(m, sm);
      m_run = -INFINITY;
      s_run = 0.f;
    }
    // tickets (wavefront 0): publish the draw of the previous iteration, then draw again
    if (s >= 1 && ((s + LA + 1) & (tpt - 1)) == 0 && tid == 0)
      s_tk[((s + LA + 1) >> tsh) & 7] = nblocks - 1 - ((int)pend * ways + way);
    if (((s + LA + 2) & (tpt - 1)) == 0 && tid == 0) pend = atomicAdd(tk, 1u);

    quad_prev = partial;
    t_prev = t_cur;
    t_cur = t_n1;
    t_n1 = t_n2;
    t_n2 = t_n3;
    ++s;
    __syncthreads();
  };

  for (;;) {
    if (t_cur < 0) break;
    body(std::integral_constant<int, 0>{});
    if (t_cur < 0) break;
    body(std::integral_constant<int, 1>{});
  }
  // the last tile's logit: one more half-iteration without matrix work
  {
    const int pb = (s - 1) & 1;
    const float lin = (s_p[pb][0][w][lane] + s_p[pb][1][w][lane]) + (s_p[pb][2][w][lane] + s_p[pb][3][w][lane]);
    const float lg = sum_halves(fmaf(quad_prev, pq_mine, lin));
    const int key = base_row(t_prev) + r;
    const bool valid = is_real(t_prev) && key >= t_prev * 32;
    if (valid && hh == 0) lg_out[key] = lg;
    if (valid) {
      const float mn = fmaxf(m_run, lg);
      s_run = s_run * __expf(m_run - mn) + __expf(lg - mn);
      m_run = mn;
    }
    if (t_prev >= 0 && (t_prev & (tpt - 1)) == tpt - 1) {
      const float m = max_lanes32(m_run);
      const float sm = sum_lanes32(m_run == -INFINITY ? 0.f : s_run * __expf(m_run - m));
      if (lane == 0) part_out[t_prev >> tsh] = make_float2(m, sm);
    }
  }
}

hipError_t launch_score_hw(const ScoreArgs& a, const ScorePlan& sp, hipStream_t st) {
  const int grid = a.units * a.nchunk * a.passes;
  k_score_hw<128><<<grid, 256, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace ea
