// bf16 MFMA GEMM kernel with the LoRA term folded in as extra contraction steps (gfx950),
// on v_mfma_f32_16x16x32_bf16.
//
//   C[M,N] = A[M,Kd] * op(Bm) + rows_k( L[rows_k, :r_k] * R_k )
//     NN = true  (forward,  Eq. "forward"):      Bm = W [Kd,N] (contraction index = rows of W),  R_k = B_k [r_k, N]
//     NN = false (backward, Eq. "grad_output"):  Bm = W [N,Kd] (contraction index = columns),     R_k = A_k [N, r_k]
//
// Why this MFMA shape: under this operator's data the board runs at its power cap, so what a
// kernel sustains is set by energy per flop.  A 16x16x32 MFMA sums 32 products into each
// accumulator element, a 32x32x16 MFMA 16: half the accumulator traffic per flop.  A loop of
// MFMAs plus the LDS fragment reads of this tile shape sustains about 10 % more with the
// 16x16x32 shape on the same data.
//
// Tile 256 x 256 x 64, WAVES_M x WAVES_N waves (2 x 4: wave tile WM x WN = 128 x 64), fp32
// accumulators in AccVGPRs, LDS tiles filled by direct global->LDS loads (16 B per lane) into
// three stages for A and two for Bm.  A wave-wide direct load fills 1 KiB of contiguous LDS, so the bank-conflict
// swizzle is applied by choosing which global 16-byte chunk each lane fetches:
//   * K-contiguous tiles (A, and Bm when !NN): 256 rows x 128 B; chunk c of row r sits at chunk
//     position c ^ ((r >> 1) & 7); a fragment (16 rows x 32 contraction indices) is one
//     ds_read_b128 per lane: lane l reads chunk 4 q + l / 16 of row l % 16 (q = which half of the tile).
//   * Bm when NN: 64 contraction rows x 512 B; chunk c of row k sits at
//     c ^ (((k & 3) << 2) | (((k >> 3) & 1) << 1)); read with two ds_read_b64_tr_b16 per lane,
//     which hand it eight consecutive contraction indices of one output column -- no transposed
//     copy of W is ever made.
// The weight fragment is the MFMA's first operand, so a lane ends up with four consecutive
// output columns of one row; the output tile goes through LDS once more so that it leaves the CU
// as full row segments.
//
// Schedule.  A contraction tile is four sub-steps: (first 32 contraction indices, upper half of
// the wave's rows), (same, lower half), (last 32, upper), (last 32, lower); a sub-step runs
// 4 x WN/16 MFMAs on 4 row fragments and WN/16 weight fragments.  Row fragments are read one
// sub-step ahead of their use (two register sets); a weight fragment serves both sub-steps of
// its half tile and is re-read in place right behind its last MFMA, a sub-step before its next
// use.  At most one memory instruction rides behind each MFMA:
//   sub-steps 0..2 of tile kt: MFMAs | LDS reads of the next sub-step's fragments
//   s_waitcnt vmcnt(4), lgkmcnt(0); barrier  (tile kt+1 visible -- the 4 loads still in flight are
//                                             A's of tile kt+2; every wave holds its last fragments
//                                             of tile kt in registers: kt's stages are free)
//   sub-step 3: MFMAs | LDS reads of tile kt+1's first fragments | the direct loads of Bm's tile
//               kt+2, then of A's tile kt+3
// A is loaded two tiles ahead because its rows come from HBM, once per launch: with one tile of
// lead the blocks that share a row strip stalled together on every cold line (the time lost grew
// linearly with the rate at which A is read from HBM, at every shape measured).  Bm, the weight,
// is read from the Infinity Cache and keeps one tile of lead; 3 + 2 stages of 32 KiB are all of
// the CU's 160 KiB of LDS, which is why the block's piece table lives in a register.
//
// Rows: the grid tiles a virtual row axis on which every row range of the call (the rows before
// the first task, each task's rows, the rows after the last task) is padded to a multiple of 32.
// A 32-row fragment pair therefore never holds rows of two tasks, and a task's LoRA tile runs its
// MFMAs only on that task's rows: no row ever meets another task's adapter (not even multiplied
// by zero, which would turn an Inf or NaN of a diverged adapter into NaN in its neighbours'
// rows).  Padding rows re-read the range's last row and are not stored.
#pragma once

#include <type_traits>

#include "mfma_staging.h"
#include "mlora_common.h"

namespace mlora {
namespace gemmk {

using namespace stage;

constexpr int BM = 256, BN = 256;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// Kernel arguments (passed by value, read with scalar loads).  The contraction may run over
// NSEG operand pairs in turn, all accumulating into the same output tile:
//   C = sum_g ( A_g[M,Kd_g] * op(Bm_g) + rows_k( L_g[rows_k, :r_gk] * R_gk ) )
// NSEG = 1 is the plain operator; NSEG > 1 is the input gradient of several projections that
// share their input (dX = sum_p dY_p W_p^T + ...), kept in fp32 until the single store.
template <int NSEG>
struct GemmArgs {
  bf16* C;
  int M, N, tiles_m, tiles_n;            // tiles_m counts tiles of the virtual row axis
  int K;                                 // tasks
  int off[kMaxK + 1];                    // split positions (rows of C)
  const bf16* A[NSEG];                   // [M, Kd_g]
  const bf16* Bm[NSEG];                  // NN: [Kd_g, N]; NT: [N, Kd_g]
  const bf16* L[NSEG];                   // [M, ldz_g] low-rank intermediate (Z or G)
  int Kd[NSEG];
  int ldz[NSEG];
  unsigned char rank[NSEG][kMaxK];       // r_gk <= 128
  PtrTable R[NSEG];                      // NN: B_k [r, N]; NT: A_k [N, r]
};

// 16 zero bytes in device memory: where the lanes of a LoRA tile point whose row, column or rank
// index lies outside the task (a direct-to-LDS load cannot be masked)
__device__ uint4 g_zero_chunk;


// c += a x b on a 16 x 16 x 32 bf16 MFMA, accumulating in place in AccVGPRs.  Written as inline
// assembly with the accumulator as a tied operand: with the builtin the register allocator is
// free to give the result another register than the input, and in a loop of 128 MFMAs on 32
// accumulators it then rotates the accumulators through the register file with one copy per
// MFMA.  Every accumulator is used again at the earliest 16 MFMAs later and read by other
// instructions only after the main loop's final barrier, so no wait states are owed here.
__device__ __forceinline__ void mfma_16x16x32(f32x4& c, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}

template <int WAVES_M, int WAVES_N, bool NN, int NSEG>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void k_gemm_mfma(const GemmArgs<NSEG> ga) {
  constexpr int BK = 64;
  bf16* __restrict__ C = ga.C;
  const int M = ga.M, N = ga.N, tiles_m = ga.tiles_m, tiles_n = ga.tiles_n;
  constexpr int NW = WAVES_M * WAVES_N;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int FM = WM / 16, FN = WN / 16;    // 16-row fragments, 16-column weight fragments of the wave tile
  constexpr int HM = FM / 2;                   // row fragments per sub-step
  constexpr int NMF = HM * FN;                 // MFMAs per sub-step
  constexpr int ROWB = BK * 2, CPR = BK / 8, RW = 256 / ROWB, RPI = 1024 / ROWB;
  constexpr int TILE_BYTES = BM * ROWB;        // the NN weight tile (BK x 512 B) has the same size
  constexpr int LPW = TILE_BYTES / 1024 / NW;  // wave-wide loads per wave per operand tile
  constexpr int PER_TILE = 2 * LPW;
  static_assert(WM == 128, "the sub-steps halve a 128-row wave tile");

  // Three stages for the A side, two for the Bm side: all 160 KiB of the CU's LDS.  The rows of
  // A come from HBM (every element once per launch, cold), the weight from the Infinity Cache; a
  // cold line takes longer than the one contraction tile a two-stage ring gives it, and every
  // block that shares the strip waits for it together.  With the third stage the A loads run two
  // tiles ahead of their use, the Bm loads one.
  __shared__ __attribute__((aligned(1024))) char sA0[TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) char sA1[TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) char sA2[TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) char sB0[TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) char sB1[TILE_BYTES];
  char* const sA[3] = {sA0, sA1, sA2};
  char* const sB[2] = {sB0, sB1};

  // block -> tile.  Tiles are taken in a grouped order (8 row tiles x all column tiles per group,
  // column by column), cut into chunks of 32: a chunk is an 8 x 4 patch of output tiles sharing
  // 8 row strips of A and 4 strips of Bm.  Consecutive block ids go round-robin over the 8 XCDs
  // and an XCD runs 32 blocks at a time, so block b = 8 l + x (XCD x) takes tile l % 32 of chunk
  // 8 (l / 32) + x: the blocks resident on one XCD share their strips in that XCD's L2 (hit rate
  // 79 %, the share an 8 x 4 patch allows), and the eight XCDs work on eight neighbouring chunks,
  // i.e. on one or two row groups of A at a time.  (Giving each XCD a contiguous eighth of the
  // order instead, eight row groups at a time: level on benchmark-like data, 2-10 % slower when
  // the weight is 141 MB, because every XCD then walks all of it on its own.)  Other patch shapes: 4 x 8
  // misses more where the column tiles are no multiple of 8, 16 x 2 is 9 % slower.
  // The tiles beyond the last full round of 256 are taken in block order.
  const int total = tiles_m * tiles_n;
  const int bid = blockIdx.x;
  int t = bid;
  if (bid < (total / 256) * 256) {
    const int xcd = bid % 8, local = bid / 8;
    t = 256 * (local / 32) + 32 * xcd + (local % 32);
  }
  constexpr int GM = 8;
  const int gsize = GM * tiles_n;
  const int group = t / gsize;
  const int first_m = group * GM;
  const int gm = (tiles_m - first_m) < GM ? (tiles_m - first_m) : GM;
  const int in_g = t - group * gsize;
  const int tm = first_m + in_g % gm, tn = in_g / gm;
  const int col0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  // ---- the block's 8 pieces of 32 virtual rows: first real row, number of real rows (0 = beyond
  // the last row: such a piece re-reads row M-1 and stores nothing) and task (-1 = rows of no
  // task).  Range s of the call is [b_s, b_{s+1}) with b_0 = 0, b_{1+k} = off[k], b_{K+2} = M;
  // task k owns range 1 + k.
  // The table lives in one vector register (the stages leave no LDS for it): every wave works it
  // out for itself, lane 8 c + f holding column c (0: first row, 1: rows, 2: task) of piece f.
  // Every use looks up a wave-uniform piece, so an entry is read with v_readlane.
  constexpr int NFR = BM / 32;
  int v_tab;
  {
    const int v0 = tm * BM + 32 * (lane & (NFR - 1));
    int vstart = 0, prev = 0, frow = M - 1, fn = 0, ftask = -1;
    for (int r = 0; r < ga.K + 2; ++r) {
      const int b1 = r <= ga.K ? ga.off[r] : M;
      const int len = b1 - prev, vlen = (len + 31) & ~31;
      if (v0 >= vstart && v0 < vstart + vlen) {
        const int o = v0 - vstart;
        frow = prev + o;
        fn = (len - o) < 32 ? (len - o) : 32;
        ftask = (r >= 1 && r <= ga.K) ? r - 1 : -1;
      }
      vstart += vlen;
      prev = b1;
    }
    const int col = lane / NFR;
    v_tab = col == 0 ? frow : (col == 1 ? fn : ftask);
  }
  auto tab = [&](int c, int f) { return __builtin_amdgcn_readlane(v_tab, __builtin_amdgcn_readfirstlane(NFR * c + f)); };
  auto frag_row = [&](int f) { return tab(0, f); };
  auto frag_n = [&](int f) { return tab(1, f); };
  auto frag_task = [&](int f) { return tab(2, f); };
  const int row0 = frag_row(0);  // the block's lowest real row
  // real row behind row rl (0..255) of the block's tile; the 8 rows of one wave-wide load lie in
  // one piece, so f is wave-uniform there
  auto real_row = [&](int rl) {
    const int f = rl >> 5, o = rl & 31;
    const int n = frag_n(f);
    return frag_row(f) + (o < n ? o : (n > 0 ? n - 1 : 0));
  };

  // ---- direct-to-LDS loads: wave-uniform base of the tile's rows (advanced per contraction
  // tile with scalar arithmetic) plus a constant 32-bit per-lane byte offset; both are set per
  // operand pair by set_operands()
  const char* abase = nullptr;
  const char* bbase = nullptr;
  unsigned aoff[LPW], boff[LPW];
  size_t bstep = 0;  // bytes per contraction tile of Bm
  auto nn_swz = [](int kr) { return ((kr & 3) << 2) | (((kr >> 3) & 1) << 1); };
  auto set_operands = [&](const bf16* A, const bf16* Bm, int Kd) {
    abase = reinterpret_cast<const char*>(A + (size_t)row0 * Kd);
    bbase = NN ? reinterpret_cast<const char*>(Bm + col0) : reinterpret_cast<const char*>(Bm + (size_t)col0 * Kd);
#pragma unroll
    for (int it = 0; it < LPW; ++it) {
      const int w = wave + NW * it;
      {
        const int rl = RPI * w + lane / CPR;
        const int c = (lane % CPR) ^ ((rl / RW) % CPR);
        const int gr = real_row(rl);
        aoff[it] = (unsigned)(((size_t)(gr - row0) * Kd + c * 8) * 2);
      }
      if (NN) {
        const int kr = 2 * w + (lane >> 5);
        const int c = (lane & 31) ^ nn_swz(kr);
        int n = col0 + c * 8;
        n = n < N ? n : N - 8;
        boff[it] = (unsigned)(((size_t)kr * N + (n - col0)) * 2);
      } else {
        const int rl = RPI * w + lane / CPR;
        const int c = (lane % CPR) ^ ((rl / RW) % CPR);
        int gn = col0 + rl;
        gn = gn < N ? gn : N - 1;
        boff[it] = (unsigned)(((size_t)(gn - col0) * Kd + c * 8) * 2);
      }
    }
    bstep = (NN ? (size_t)BK * N : (size_t)BK) * 2;
  };

  // fragment addressing: lane l = 16 kg + r16 holds contraction indices 8 kg .. 8 kg + 7 (of the
  // 32 of a half tile) of row / column r16 of the fragment
  const int r16 = lane & 15, kg = lane >> 4;
  const int fsw = (r16 >> 1) & 7;
  const int a_row_off = (wm * WM + r16) * ROWB;
  const int b_row_off = (wn * WN + r16) * ROWB;
  const int kq = r16 >> 2;
  const int nn_k = 8 * kg + kq;                   // first of the lane's two 4-row pieces of the W tile
  const int nn_n = wn * WN + 4 * (r16 & 3);

  f32x4 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;

  bf16x8 af[2][HM], bfr[FN];

  // weight fragment j of half q of the tile in sb
  auto read_b = [&](const char* sb, int q, int j) {
    if (NN) {
      const int k = 32 * q + nn_k;
      const int n = nn_n + 16 * j;
      const int phys = (n >> 3) ^ ((kq << 2) | ((kg & 1) << 1));
      const char* p0 = sb + k * 512 + phys * 16 + (n & 7) * 2;
      bfr[j] = lds_read_tr_pair(p0, p0 + 4 * 512);
    } else {
      bfr[j] = *(const bf16x8*)(sb + b_row_off + j * 16 * ROWB + (((4 * q + kg) ^ fsw) << 4));
    }
  };
  // row fragment i (0..HM-1) of half h of the wave's rows, half q of the tile in sa
  auto read_a = [&](const char* sa, int q, int h, int i, bf16x8 (&af)[HM]) {
    af[i] = *(const bf16x8*)(sa + a_row_off + (h * HM + i) * 16 * ROWB + (((4 * q + kg) ^ fsw) << 4));
  };

  // ---- LoRA contraction tiles.  After the last operand pair's base tiles the same pipeline
  // runs one more tile per (task k that owns rows of this block, 64 ranks of it): its A side is
  // the task's slice of L (Z or G; zeros for the other pieces), its B side the same ranks of R_k
  // (B_k or A_k), fetched into the same LDS layouts by the same direct loads two tiles ahead --
  // so the LoRA term costs ceil(r_k / 64) more tiles on the same accumulators and no exposed
  // load latency.  The pieces of one task are consecutive, so the block's tasks are the runs of
  // the task column of the piece table.
  struct LoraTile {
    int sg, k, q0;
  };
  int n_lora = 0;
  for (int sg = 0; sg < NSEG; ++sg)
    for (int f = 0; f < NFR; ++f) {
      const int k = frag_task(f);
      if (k >= 0 && (f == 0 || frag_task(f - 1) != k)) n_lora += (ga.rank[sg][k] + BK - 1) / BK;
    }
  auto find_lora = [&](int e) {
    LoraTile t{0, -1, 0};
    for (int sg = 0; sg < NSEG; ++sg)
      for (int f = 0; f < NFR; ++f) {
        const int k = frag_task(f);
        if (k < 0 || (f > 0 && frag_task(f - 1) == k)) continue;
        const int nch = (ga.rank[sg][k] + BK - 1) / BK;
        if (e >= 0 && e < nch) t = LoraTile{sg, k, e * BK};
        e -= nch;
      }
    return t;
  };
  // what the load slots of a tile fetch: base tile kt of the current operand pair, or a LoRA tile
  struct LoadCtx {
    bool lora;
    const char* atile;
    const char* btile;
    LoraTile lt;
  };
  auto base_ctx = [&](int kt) {
    return LoadCtx{false, abase + (size_t)kt * (BK * 2), bbase + (size_t)kt * bstep, LoraTile{0, -1, 0}};
  };
  const char* const zeros = reinterpret_cast<const char*>(&g_zero_chunk);
  // wave-wide load number idx (0..LPW-1: A side, LPW..PER_TILE-1: Bm side) of the tile `lc` describes
  auto issue_one = [&](const LoadCtx& lc, int idx, char* sa, char* sb) {
    if (!lc.lora) {
      if (idx < LPW)
        load_lds_16B_sbase(lc.atile, aoff[idx], sa + (wave + NW * idx) * 1024);
      else
        load_lds_16B_sbase(lc.btile, boff[idx - LPW], sb + (wave + NW * (idx - LPW)) * 1024);
      return;
    }
    const LoraTile& t = lc.lt;
    if (idx < LPW) {
      const bf16* L = ga.L[t.sg];
      const int ldz = ga.ldz[t.sg];
      const int w = wave + NW * idx;
      const int rl = RPI * w + lane / CPR;
      const int c = (lane % CPR) ^ ((rl / RW) % CPR);
      const int q = t.q0 + c * 8;
      const bool mine = frag_task(rl >> 5) == t.k;  // wave-uniform: the 8 rows of this load share a piece
      const char* p = (mine && q < ldz) ? reinterpret_cast<const char*>(L + (size_t)real_row(rl) * ldz + q) : zeros;
      load_lds_16B(p, sa + w * 1024);
    } else {
      const int r = ga.rank[t.sg][t.k];
      const bf16* Rk = static_cast<const bf16*>(ga.R[t.sg].p[t.k]);
      const int w = wave + NW * (idx - LPW);
      const char* p = zeros;
      if (NN) {
        const int kr = 2 * w + (lane >> 5);
        const int c = (lane & 31) ^ nn_swz(kr);
        const int q = t.q0 + kr, n = col0 + c * 8;
        if (q < r && n < N) p = reinterpret_cast<const char*>(Rk + (size_t)q * N + n);
      } else {
        const int rl = RPI * w + lane / CPR;
        const int c = (lane % CPR) ^ ((rl / RW) % CPR);
        const int n = col0 + rl, q = t.q0 + c * 8;
        if (n < N && q < r) p = reinterpret_cast<const char*>(Rk + (size_t)n * r + q);
      }
      load_lds_16B(p, sb + w * 1024);
    }
  };

  // Which of the wave's WM / 32 pieces take part in a tile: all of them in a base tile, the
  // pieces of task k in a LoRA tile of task k (the others' MFMAs are skipped).
  // `q1`: whether the second half of the tile's 64 contraction indices holds anything -- a LoRA
  // tile whose remaining ranks are at most 32 (rank 8, 16, 32: most adapters) runs the MFMAs of
  // its first half only (the other half of the staged operands is zeros).
  struct FragOn {
    bool on[WM / 32];
    bool q1;
  };
  auto frags_of = [&](const LoraTile& t, bool base) {
    FragOn f;
#pragma unroll
    for (int i = 0; i < WM / 32; ++i) f.on[i] = base || frag_task(wm * (WM / 32) + i) == t.k;
    f.q1 = base || (int)ga.rank[t.sg][t.k < 0 ? 0 : t.k] - t.q0 > 32;
    return f;
  };

  // Sub-step S (0..3) of a tile: the MFMAs of (half q = S / 2 of the contraction tile, half
  // h = S % 2 of the wave's rows), weight fragment by weight fragment (MFMA number m uses weight
  // fragment m / HM and row fragment m % HM of set h).  Row fragments are double-buffered: the HM
  // fragments of the next sub-step are read behind the first HM MFMAs.  Weight fragments are
  // not: they serve both sub-steps of a half tile, and in the second of them (h = 1) fragment j
  // is re-read for the next half tile right behind its last MFMA (slot HM j + HM - 1), a whole
  // sub-step before its next use -- 16 registers instead of 32.  The reads come from (rsa, rsb)
  // (if rd); in sub-step 3, after the barrier, the remaining slots carry the PER_TILE loads of
  // the tile `lc` into (lsa, lsb) (if ld).  rd and ld are std::true_type / std::false_type in
  // the steady-state loop, so that it compiles to straight-line code, and plain bools in the few
  // tiles around it; `fo` is std::true_type there (base tiles: every piece) and a FragOn in
  // the tiles that may be LoRA tiles.
  auto substep = [&](auto S_, auto rd, const char* rsa, const char* rsb, auto ldb, const LoadCtx& lcb, char* lsb, auto lda,
                     const LoadCtx& lca, char* lsa, const auto& fo) {
    constexpr int S = decltype(S_)::value;
    constexpr int q = S / 2, h = S % 2;
    constexpr int NS_ = (S + 1) % 4;                 // the sub-step whose row fragments are read now
    constexpr int nq = NS_ / 2, nh = NS_ % 2;
    static_assert((FN - 1) * (HM - 1) >= PER_TILE, "load slots");
#pragma unroll
    for (int m = 0; m < NMF; ++m) {
      const int j = m / HM, i = m % HM;
      bool on = true;
      if constexpr (!std::is_same_v<std::decay_t<decltype(fo)>, std::true_type>) on = fo.on[(h * HM + i) / 2] && (q == 0 || fo.q1);
      if (on) mfma_16x16x32(acc[h * HM + i][j], bfr[j], af[h][i]);
      if (rd && m < HM) read_a(rsa, nq, nh, m, af[nh]);
      if (rd && h == 1 && i == HM - 1) read_b(rsb, nq, j);
      if (S == 3 && m >= HM && i != HM - 1) {
        // the Bm side first: the next barrier waits for it and lets the A loads behind it fly on
        const int idx = (j - 1) * (HM - 1) + i;
        if (ldb && idx < LPW) issue_one(lcb, LPW + idx, nullptr, lsb);
        if (lda && idx >= LPW && idx < PER_TILE) issue_one(lca, idx - LPW, lsa, nullptr);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  constexpr std::true_type yes{};
  constexpr std::false_type no{};
  constexpr std::integral_constant<int, 0> S0{};
  constexpr std::integral_constant<int, 1> S1{};
  constexpr std::integral_constant<int, 2> S2{};
  constexpr std::integral_constant<int, 3> S3{};
  const LoadCtx none{false, nullptr, nullptr, LoraTile{0, -1, 0}};

  // A tile whose operands sit in (ca, cb): sub-steps 0..2, barrier, sub-step 3 with the reads of
  // the next tile's first fragments from (na, nb) (if rd), the Bm loads of the tile after that,
  // `lcb`, into cb (if ldb) and the A loads of the tile after that one, `lca`, into ca (if lda).
  // `abehind`: whether A loads were issued behind the Bm loads the barrier waits for (the
  // previous tile's lda) -- vector loads return in order, so the wait leaves exactly those LPW
  // loads in flight.
  auto tile = [&](char* ca, char* cb, const char* na, const char* nb, auto rd, auto ldb, const LoadCtx& lcb, auto lda,
                  const LoadCtx& lca, auto abehind, const auto& fo) {
    substep(S0, yes, ca, cb, no, none, nullptr, no, none, nullptr, fo);
    substep(S1, yes, ca, cb, no, none, nullptr, no, none, nullptr, fo);
    substep(S2, yes, ca, cb, no, none, nullptr, no, none, nullptr, fo);
    // the next tile has landed (this wave's part), every fragment of this tile is in registers
    // (the weight fragments of this half tile stay in use until sub-step 3 re-reads them)
    if (abehind)
      wait_vmcnt<LPW>();
    else
      wait_vmcnt<0>();
    wait_lds();
    __builtin_amdgcn_s_barrier();
    substep(S3, rd, na, nb, ldb, lcb, cb, lda, lca, ca, fo);
  };

  // ---- main contraction loop.  Tile v of a pass uses A stage v % 3 and Bm stage v % 2; the steady
  // state is unrolled by six so that stage addresses are constants.  Operand pairs run one after
  // the other.  When a pair's last tile has passed its barrier every wave holds that tile's last
  // fragments in registers, so all stages are free for the next pair's first tiles.
  for (int sg = 0; sg < NSEG; ++sg) {
    set_operands(ga.A[sg], ga.Bm[sg], ga.Kd[sg]);
    const int KT = ga.Kd[sg] / BK;
    const int VT = KT + (sg == NSEG - 1 ? n_lora : 0);  // tiles of this pass: base tiles, then LoRA tiles
    auto ctx_of = [&](int v) {
      if (v < KT) return base_ctx(v);
      return LoadCtx{true, nullptr, nullptr, find_lora(v - KT)};
    };
    auto issue_a = [&](const LoadCtx& lc, char* sa) {
#pragma unroll
      for (int idx = 0; idx < LPW; ++idx) issue_one(lc, idx, sa, nullptr);
    };
    auto issue_b = [&](const LoadCtx& lc, char* sb) {
#pragma unroll
      for (int idx = 0; idx < LPW; ++idx) issue_one(lc, LPW + idx, nullptr, sb);
    };
    // tiles 0 and 1 whole and the A side of tile 2; the first reads need tile 0
    issue_a(base_ctx(0), sA[0]);
    issue_b(base_ctx(0), sB[0]);
    if (VT > 2) {
      issue_a(ctx_of(1), sA[1]);
      issue_b(ctx_of(1), sB[1]);
      issue_a(ctx_of(2), sA[2]);
      wait_vmcnt<3 * LPW>();
    } else if (VT > 1) {
      issue_a(ctx_of(1), sA[1]);
      issue_b(ctx_of(1), sB[1]);
      wait_vmcnt<2 * LPW>();
    } else {
      wait_vmcnt<0>();
    }
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int j = 0; j < FN; ++j) read_b(sB[0], 0, j);
#pragma unroll
    for (int i = 0; i < HM; ++i) read_a(sA[0], 0, 0, i, af[0]);
    __builtin_amdgcn_sched_barrier(0);
    // steady state, six base tiles per trip: each has a successor to read, a base tile two ahead
    // for its Bm loads and one three ahead for its A loads
    int v = 0;
    for (; v + 8 < KT; v += 6) {
      tile(sA[0], sB[0], sA[1], sB[1], yes, yes, base_ctx(v + 2), yes, base_ctx(v + 3), yes, yes);
      tile(sA[1], sB[1], sA[2], sB[0], yes, yes, base_ctx(v + 3), yes, base_ctx(v + 4), yes, yes);
      tile(sA[2], sB[0], sA[0], sB[1], yes, yes, base_ctx(v + 4), yes, base_ctx(v + 5), yes, yes);
      tile(sA[0], sB[1], sA[1], sB[0], yes, yes, base_ctx(v + 5), yes, base_ctx(v + 6), yes, yes);
      tile(sA[1], sB[0], sA[2], sB[1], yes, yes, base_ctx(v + 6), yes, base_ctx(v + 7), yes, yes);
      tile(sA[2], sB[1], sA[0], sB[0], yes, yes, base_ctx(v + 7), yes, base_ctx(v + 8), yes, yes);
    }
    // (v is a multiple of 6 here.)  The up to seven base tiles left that still have all of the
    // above: the same straight-line code, with the stage addresses in registers
    auto stage_a = [&](int u) { return u % 3 == 0 ? sA0 : (u % 3 == 1 ? sA1 : sA2); };
    auto stage_b = [&](int u) { return u % 2 == 0 ? sB0 : sB1; };
    for (; v + 3 < KT; ++v)
      tile(stage_a(v), stage_b(v), stage_a(v + 1), stage_b(v + 1), yes, yes, base_ctx(v + 2), yes, base_ctx(v + 3), yes, yes);
    // the last base tiles and the LoRA tiles
    auto frags_at = [&](int u) { return u < KT ? frags_of(LoraTile{0, -1, 0}, true) : frags_of(find_lora(u - KT), false); };
    for (; v < VT; ++v) {
      tile(stage_a(v), stage_b(v), stage_a(v + 1), stage_b(v + 1), v + 1 < VT, v + 2 < VT, v + 2 < VT ? ctx_of(v + 2) : none,
           v + 3 < VT, v + 3 < VT ? ctx_of(v + 3) : none, v + 2 < VT, frags_at(v));
    }
  }  // operand pairs

  // ---- output: through LDS, so that the tile leaves as 16 B per lane in full row segments of
  // the wave's sub-tile.  Each wave owns WM x WN x 2 bytes of the stage arrays (row stride WN x 2
  // bytes, chunk c of row m at c ^ swizzle(m)); nothing is shared between waves after the barrier.
  constexpr int OCH = WN / 8;                 // 16-byte chunks per output row of the wave's sub-tile
  constexpr int OROWB = WN * 2;               // bytes per such row
  constexpr int ORPI = 64 / OCH;              // rows per wave-wide store
  constexpr int WBYTES = WM * OROWB;          // bytes per wave
  static_assert(NW * WBYTES == 4 * TILE_BYTES && (TILE_BYTES % WBYTES) == 0, "sub-tiles must tile the stage arrays");
  constexpr int WPA = TILE_BYTES / WBYTES;    // waves per stage array
  typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
  auto oswz = [](int m) { return OCH == 8 ? ((m >> 1) & 7) : (m & (OCH - 1)); };
  __syncthreads();
  char* ep = sA0;
  if (wave / WPA == 1) ep = sA1;
  if (wave / WPA == 2) ep = sB0;
  if (wave / WPA == 3) ep = sB1;
  ep += (wave % WPA) * WBYTES;
  // lane 16 kg + r16 holds row 16 i + r16, columns 16 j + 4 kg + 0..3 of the wave's sub-tile
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      bf16x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = static_cast<bf16>(acc[i][j][e]);
      const int m = 16 * i + r16, c = 2 * j + (kg >> 1);
      *(bf16x4*)(ep + m * OROWB + ((c ^ oswz(m)) << 4) + 8 * (kg & 1)) = o;
    }
#pragma unroll
  for (int it = 0; it < WM / ORPI; ++it) {
    const int r = ORPI * it + lane / OCH, cp = lane % OCH;
    const int c = cp ^ oswz(r);
    const uint4 v = *(const uint4*)(ep + r * OROWB + cp * 16);
    // the row's piece of the block (WM is a multiple of 32; the rows of one store share a piece)
    const int f = (wm * WM + ORPI * it) >> 5, o = r & 31;
    const int grow = frag_row(f) + o, gcol = col0 + wn * WN + c * 8;
    // non-temporal: the output is not read again by this launch, so it should not displace the
    // operand strips in the L2 / Infinity Cache (measured +0.7 % on the whole forward + backward)
    if (o < frag_n(f) && gcol < N)
      __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v), (u32x4*)(C + (size_t)grow * N + gcol));
  }
}

}  // namespace gemmk
}  // namespace mlora
