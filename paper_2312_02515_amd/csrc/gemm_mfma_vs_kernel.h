// bf16 MFMA GEMM kernel with the LoRA term folded in as extra contraction steps (gfx950):
// the register-staged form.
//
//   C[M,N] = A[M,Kd] * op(Bm) + rows_k( L[rows_k, :r_k] * R_k )
//     NN = true  (forward,  Eq. "forward"):      Bm = W [Kd,N] (contraction index = rows of W),  R_k = B_k [r_k, N]
//     NN = false (backward, Eq. "grad_output"):  Bm = W [N,Kd] (contraction index = columns),     R_k = A_k [N, r_k]
//
// Tile 256 x 256 x 64, 4 waves (2 x 2, wave tile 128 x 128, one wave per SIMD), fp32 accumulation
// in v_mfma_f32_32x32x16_bf16 with the 256 accumulators of a lane in AccVGPRs.  LDS holds two
// stages of (A tile, Bm tile), 32 KiB each, in the layouts of gemm_mfma_kernel.h:
//   * K-contiguous tiles (A, and Bm when !NN): 256 rows x 128 B; chunk c of row r sits at chunk
//     position c ^ ((r >> 1) & 7); read with ds_read_b128.
//   * Bm when NN: 64 contraction rows x 512 B; chunk c of row k sits at c ^ ((k & 3) << 2); read
//     with ds_read_b64_tr_b16 (four consecutive contraction indices of one output column per
//     lane) -- no transposed copy of W is ever made.
//
// How a tile gets into LDS is what differs.  The texture path delivers 64 B per clock to a CU; a
// 64 KiB contraction tile keeps it busy for half of the tile's MFMA time.  A load that writes
// LDS directly can only be issued once its stage is free, i.e. in the last quarter of a tile, so
// all waves issue their loads in one burst, the path's queue fills and the waves stall at the
// load instructions with the matrix pipe idle behind them.  Here a load lands in registers, so
// it can be issued at any time: every wave issues one global load per four MFMAs, all the way
// through the tile, and copies the registers to LDS (ds_write_b128, a fast path) a tile later,
// when the stage has been released.  Per MFMA step of 16 MFMAs a wave issues 8 fragment reads
// (for the next step), 4 LDS writes (a quarter of the tile after next) and 4 global loads
// (refilling the registers just written, with the tile after that): one memory instruction
// behind every MFMA.
//
// Rows: as in gemm_mfma_kernel.h the grid tiles a virtual row axis on which every row range of
// the call is padded to whole 32-row MFMA fragments, so that a fragment never holds rows of two
// tasks and a task's LoRA tile runs its MFMAs only on that task's fragments.
#pragma once

#include <type_traits>

#include "gemm_mfma_kernel.h"

namespace mlora {
namespace gemmvs {

using namespace stage;
using gemmk::BM;
using gemmk::BN;
using gemmk::GemmArgs;

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

template <int WAVES_M, int WAVES_N, bool NN, int NSEG>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void k_gemm_mfma_vs(const GemmArgs<NSEG> ga) {
  constexpr int BK = 64;
  bf16* __restrict__ C = ga.C;
  const int M = ga.M, N = ga.N, tiles_m = ga.tiles_m, tiles_n = ga.tiles_n;
  constexpr int NW = WAVES_M * WAVES_N;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int FM = WM / 32, FN = WN / 32;
  constexpr int NMF = FM * FN;                 // MFMAs per step
  constexpr int NOPS = FM + FN;                // fragment reads per step
  constexpr int ROWB = BK * 2, CPR = BK / 8, RW = 256 / ROWB, RPI = 1024 / ROWB;
  constexpr int TILE_BYTES = BM * ROWB;        // the NN weight tile (BK x 512 B) has the same size
  constexpr int LPW = TILE_BYTES / 1024 / NW;  // wave-wide loads per wave per operand tile
  constexpr int NLD = 2 * LPW;                 // ... per contraction tile

  __shared__ __attribute__((aligned(1024))) char sA0[TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) char sA1[TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) char sB0[TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) char sB1[TILE_BYTES];
  char* const sA[2] = {sA0, sA1};
  char* const sB[2] = {sB0, sB1};

  // block -> tile: consecutive block ids go round-robin over the 8 XCDs; each XCD gets a
  // contiguous range of a grouped order (8 row tiles x all column tiles per group), so that the
  // blocks resident on one XCD share operand strips in its L2
  const int total = tiles_m * tiles_n;
  const int bid = blockIdx.x;
  const int per = total / 8, rem = total % 8;
  const int xcd = bid % 8, local = bid / 8;
  const int t = xcd * per + (xcd < rem ? xcd : rem) + local;
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

  // ---- the block's 8 fragments of 32 virtual rows: first real row, number of real rows
  // (0 = beyond the last row: such a fragment re-reads row M-1 and stores nothing) and task
  // (-1 = rows of no task).  Range s of the call is [b_s, b_{s+1}) with b_0 = 0, b_{1+k} = off[k],
  // b_{K+2} = M; task k owns range 1 + k.
  constexpr int NFR = BM / 32;
  __shared__ int s_frow[NFR], s_fn[NFR], s_ftask[NFR];
  if (tid < NFR) {
    const int v0 = tm * BM + 32 * tid;
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
    s_frow[tid] = frow;
    s_fn[tid] = fn;
    s_ftask[tid] = ftask;
  }
  __syncthreads();
  auto frag_row = [&](int f) { return __builtin_amdgcn_readfirstlane(s_frow[f]); };
  auto frag_n = [&](int f) { return __builtin_amdgcn_readfirstlane(s_fn[f]); };
  auto frag_task = [&](int f) { return __builtin_amdgcn_readfirstlane(s_ftask[f]); };
  const int row0 = frag_row(0);  // the block's lowest real row
  // real row behind row rl (0..255) of the block's tile; the 8 rows of one wave-wide load lie in
  // one fragment, so f is wave-uniform there
  auto real_row = [&](int rl) {
    const int f = rl >> 5, o = rl & 31;
    const int n = frag_n(f);
    return frag_row(f) + (o < n ? o : (n > 0 ? n - 1 : 0));
  };

  // Accumulators in AccVGPRs: naming one "a" register operand makes the compiler select the
  // AGPR form of the MFMAs; the 256 architectural VGPRs stay free for fragments and staging.
  {
    float agpr_hint = 0.f;
    asm volatile("" : "+a"(agpr_hint));
  }

  // ---- global loads: wave-uniform base of the tile's rows (advanced per contraction tile with
  // scalar arithmetic) plus a constant 32-bit per-lane byte offset; set per operand pair.
  // Wave-wide load number idx (0..LPW-1: A side, LPW..NLD-1: Bm side) fills the 1 KiB piece
  // (wave + NW * idx') of its operand's LDS tile, lane l the 16 bytes at 16 l of the piece; the
  // bank-conflict swizzles are applied by choosing which global chunk each lane fetches.
  const char* abase = nullptr;
  const char* bbase = nullptr;
  unsigned aoff[LPW], boff[LPW];
  size_t bstep = 0;  // bytes per contraction tile of Bm
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
        const int c = (lane & 31) ^ ((kr & 3) << 2);
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

  const int l32 = lane & 31, lhi = lane >> 5;
  const int fsw = (l32 / RW) % CPR;
  const int a_row_off = (wm * WM + l32) * ROWB;
  const int b_row_off = (wn * WN + l32) * ROWB;
  const int L16 = lane & 15, blk = lane >> 4, kq = L16 >> 2;
  const int nn_k = 8 * (blk >> 1) + kq;
  const int nn_n = wn * WN + 16 * (blk & 1) + 4 * (L16 & 3);

  // fragment read number op (0..NOPS-1) of step ks of the tile in (sa, sb): weight fragments first
  auto read_op = [&](const char* sa, const char* sb, int ks, int op, bf16x8 (&af)[FM], bf16x8 (&bfr)[FN]) {
    const int coff = ((2 * ks + lhi) ^ fsw) << 4;
    if (op < FN) {
      const int j = op;
      if (NN) {
        const int k = 16 * ks + nn_k;
        const int n = nn_n + 32 * j;
        const int phys = (n >> 3) ^ (kq << 2);
        const char* p0 = sb + k * 512 + phys * 16 + (n & 7) * 2;
        bfr[j] = lds_read_tr_pair(p0, p0 + 4 * 512);
      } else {
        bfr[j] = *(const bf16x8*)(sb + b_row_off + j * 32 * ROWB + coff);
      }
    } else {
      const int i = op - FN;
      af[i] = *(const bf16x8*)(sa + a_row_off + i * 32 * ROWB + coff);
    }
  };

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  bf16x8 af[2][FM], bfr[2][FN];
  u32x4 buf[2][NLD];  // the staging registers: this wave's share of two contraction tiles in flight

  // ---- LoRA contraction tiles.  After the last operand pair's base tiles the same pipeline
  // runs one more tile per (task k that owns fragments of this block, 64 ranks of it): its A side
  // is the task's slice of L (Z or G; zeros for the other fragments), its B side the same ranks of
  // R_k (B_k or A_k), in the same LDS layouts.  The fragments of one task are consecutive, so the
  // block's tasks are the runs of s_ftask.
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
  // what a tile's global loads fetch: base tile kt of the current operand pair, or a LoRA tile
  struct LoadCtx {
    bool lora;
    const char* atile;
    const char* btile;
    LoraTile lt;
  };
  auto base_ctx = [&](int kt) {
    return LoadCtx{false, abase + (size_t)kt * (BK * 2), bbase + (size_t)kt * bstep, LoraTile{0, -1, 0}};
  };
  const u32x4 zero4 = {0u, 0u, 0u, 0u};
  // raw buffer descriptor over everything from `base` on (no range limit: every lane offset is in
  // bounds by construction)
  auto rsrc_of = [](const char* base) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(base), 0, 0xffffffff, 0x00020000);
  };
  // global load number idx of the tile `lc` describes, into its staging register
  auto gload = [&](const LoadCtx& lc, int set, int idx) {
    if (!lc.lora) {
      // buffer load: the tile's base travels in a scalar resource descriptor, the lane's offset
      // is the same register for every tile -- no address arithmetic per load
      if (idx < LPW)
        buf[set][idx] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_of(lc.atile), aoff[idx], 0, 0);
      else
        buf[set][idx] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_of(lc.btile), boff[idx - LPW], 0, 0);
      return;
    }
    const LoraTile& t = lc.lt;
    u32x4 v = zero4;
    if (idx < LPW) {
      const bf16* L = ga.L[t.sg];
      const int ldz = ga.ldz[t.sg];
      const int w = wave + NW * idx;
      const int rl = RPI * w + lane / CPR;
      const int c = (lane % CPR) ^ ((rl / RW) % CPR);
      const int q = t.q0 + c * 8;
      const bool mine = frag_task(rl >> 5) == t.k;  // wave-uniform: the 8 rows of this load share a fragment
      if (mine && q < ldz) v = *reinterpret_cast<const u32x4*>(L + (size_t)real_row(rl) * ldz + q);
    } else {
      const int r = ga.rank[t.sg][t.k];
      const bf16* Rk = static_cast<const bf16*>(ga.R[t.sg].p[t.k]);
      const int w = wave + NW * (idx - LPW);
      if (NN) {
        const int kr = 2 * w + (lane >> 5);
        const int c = (lane & 31) ^ ((kr & 3) << 2);
        const int q = t.q0 + kr, n = col0 + c * 8;
        if (q < r && n < N) v = *reinterpret_cast<const u32x4*>(Rk + (size_t)q * N + n);
      } else {
        const int rl = RPI * w + lane / CPR;
        const int c = (lane % CPR) ^ ((rl / RW) % CPR);
        const int n = col0 + rl, q = t.q0 + c * 8;
        if (n < N && q < r) v = *reinterpret_cast<const u32x4*>(Rk + (size_t)n * r + q);
      }
    }
    buf[set][idx] = v;
  };
  // staging register idx -> its 1 KiB piece of the stage (sa, sb)
  const int lane16 = lane * 16;
  auto lwrite = [&](int set, int idx, char* sa, char* sb) {
    char* dst = idx < LPW ? sa + (wave + NW * idx) * 1024 : sb + (wave + NW * (idx - LPW)) * 1024;
    *reinterpret_cast<u32x4*>(dst + lane16) = buf[set][idx];
  };

  // Which of the wave's FM fragments take part in a tile: all of them in a base tile, the
  // fragments of task k in a LoRA tile of task k (the others' MFMAs are skipped).
  struct FragOn {
    bool on[FM];
  };
  auto frags_of = [&](int k) {  // k < 0: base tile
    FragOn f;
#pragma unroll
    for (int i = 0; i < FM; ++i) f.on[i] = k < 0 || frag_task(wm * FM + i) == k;
    return f;
  };

  // One MFMA step (number `stp` of the tile) on fragment set `cur`.  Memory instructions ride
  // behind the MFMAs; with g = NMF * stp + m the tile-wide slot number:
  //   m < NOPS           : fragment read m of the next step into set `cur ^ 1`            (if rd)
  //   g = 3 x, x < NLD   : LDS write of staging register x of set `ws` into (wsa, wsb)   (if wr)
  //   g = 4 x + 3        : global load refilling that register from the tile `lc`        (if ld)
  // so a register is written to LDS before it is refilled, the writes are over before the
  // barrier (slot 3 NMF) and the loads are spread over the whole tile.  rd, wr, ld are
  // std::true_type in the steady-state loop (straight-line code) and plain bools in the tiles
  // around it; `fo` is std::true_type there (base tiles: every fragment) or a FragOn.
  static_assert(3 * (NLD - 1) < 3 * NMF && 4 * (NLD - 1) + 3 < 4 * NMF, "slots");
  auto step = [&](auto stp_, int cur, auto rd, const char* rsa, const char* rsb, int rks, auto ws_, auto wr, char* wsa,
                  char* wsb, auto ld, const LoadCtx& lc, const auto& fo) {
    constexpr int stp = decltype(stp_)::value;
    constexpr int ws = decltype(ws_)::value;
#pragma unroll
    for (int m = 0; m < NMF; ++m) {
      const int i = m / FN, j = m % FN;
      constexpr int dummy = 0;
      (void)dummy;
      const int g = NMF * stp + m;
      bool on = true;
      if constexpr (!std::is_same_v<std::decay_t<decltype(fo)>, std::true_type>) on = fo.on[i];
      if (on) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cur][j], af[cur][i], acc[i][j], 0, 0, 0);
      if (rd && m < NOPS) read_op(rsa, rsb, rks, m, af[cur ^ 1], bfr[cur ^ 1]);
      if (wr && g % 3 == 0 && g / 3 < NLD) lwrite(ws, g / 3, wsa, wsb);
      if (ld && g % 4 == 3 && g / 4 < NLD) gload(lc, ws, g / 4);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  constexpr std::true_type yes{};
  const LoadCtx none{false, nullptr, nullptr, LoraTile{0, -1, 0}};
  constexpr std::integral_constant<int, 0> c0{};
  constexpr std::integral_constant<int, 1> c1{};
  constexpr std::integral_constant<int, 2> c2_{};
  constexpr std::integral_constant<int, 3> c3_{};

  // Tile v, held by LDS stage s = v % 2.  Register set s ^ 1 holds tile v+1 (loaded two tiles
  // ago): it is written into stage s ^ 1 during steps 0..2 and refilled with tile v+3; set s
  // (tile v+2, loaded one tile ago) rests.  After step 2 every wave has its last fragments of
  // tile v in registers and tile v+1 is complete in LDS: barrier, then step 3 reads the first
  // fragments of tile v+1.
  //   h1, h3: tiles v+1, v+3 exist;  c3: what tile v+3 loads
  auto tile = [&](auto stage, auto h1, auto h3, const LoadCtx& c3, const auto& fo) {
    constexpr int s = decltype(stage)::value;
    constexpr std::integral_constant<int, s ^ 1> ws{};
    step(c0, 0, yes, sA[s], sB[s], 1, ws, h1, sA[s ^ 1], sB[s ^ 1], h3, c3, fo);
    step(c1, 1, yes, sA[s], sB[s], 2, ws, h1, sA[s ^ 1], sB[s ^ 1], h3, c3, fo);
    step(c2_, 0, yes, sA[s], sB[s], 3, ws, h1, sA[s ^ 1], sB[s ^ 1], h3, c3, fo);
    wait_lds();
    __builtin_amdgcn_s_barrier();
    step(c3_, 1, h1, sA[s ^ 1], sB[s ^ 1], 0, ws, h1, sA[s ^ 1], sB[s ^ 1], h3, c3, fo);
  };
  constexpr std::integral_constant<int, 0> stage0{};
  constexpr std::integral_constant<int, 1> stage1{};

  // ---- contraction: operand pairs run one after the other (the pipeline drains in between)
  for (int sg = 0; sg < NSEG; ++sg) {
    set_operands(ga.A[sg], ga.Bm[sg], ga.Kd[sg]);
    const int KT = ga.Kd[sg] / BK;
    const int VT = KT + (sg == NSEG - 1 ? n_lora : 0);  // tiles of this pass: base tiles, then LoRA tiles
    auto ctx_of = [&](int v) {
      if (v < KT) return base_ctx(v);
      if (v < VT) return LoadCtx{true, nullptr, nullptr, find_lora(v - KT)};
      return none;
    };
    if (sg > 0) __syncthreads();  // every wave is done reading the previous pair's last tile
    // prologue: tile 0 through register set 0 into stage 0, tile 1 into set 1, tile 2 into set 0
    {
      const LoadCtx t0 = base_ctx(0);
#pragma unroll
      for (int idx = 0; idx < NLD; ++idx) gload(t0, 0, idx);
      if (VT > 1) {
        const LoadCtx t1 = ctx_of(1);
#pragma unroll
        for (int idx = 0; idx < NLD; ++idx) gload(t1, 1, idx);
      }
#pragma unroll
      for (int idx = 0; idx < NLD; ++idx) lwrite(0, idx, sA[0], sB[0]);
      if (VT > 2) {
        const LoadCtx t2 = ctx_of(2);
#pragma unroll
        for (int idx = 0; idx < NLD; ++idx) gload(t2, 0, idx);
      }
    }
    wait_lds();
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int op = 0; op < NOPS; ++op) read_op(sA[0], sB[0], 0, op, af[0], bfr[0]);
    __builtin_amdgcn_sched_barrier(0);
    // steady state, two base tiles per trip: tiles up to v + 4 are base tiles
    int v = 0;
    for (; v + 4 < KT; v += 2) {
      tile(stage0, yes, yes, base_ctx(v + 3), yes);
      tile(stage1, yes, yes, base_ctx(v + 4), yes);
    }
    // the last base tiles and the LoRA tiles
    auto frags_at = [&](int u) { return frags_of(u < KT ? -1 : find_lora(u - KT).k); };
    for (; v < VT; v += 2) {
      tile(stage0, v + 1 < VT, v + 3 < VT, ctx_of(v + 3), frags_at(v));
      if (v + 1 < VT) tile(stage1, v + 2 < VT, v + 4 < VT, ctx_of(v + 4), frags_at(v + 1));
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
  auto oswz = [](int m) { return OCH == 8 ? ((m >> 1) & 7) : (m & (OCH - 1)); };
  __syncthreads();
  char* ep = sA0;
  if (wave / WPA == 1) ep = sA1;
  if (wave / WPA == 2) ep = sB0;
  if (wave / WPA == 3) ep = sB1;
  ep += (wave % WPA) * WBYTES;
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = static_cast<bf16>(acc[i][j][4 * g + e]);
        const int m = 32 * i + l32, c = 4 * j + g;
        *(bf16x4*)(ep + m * OROWB + ((c ^ oswz(m)) << 4) + 8 * lhi) = o;
      }
#pragma unroll
  for (int it = 0; it < WM / ORPI; ++it) {
    const int r = ORPI * it + lane / OCH, cp = lane % OCH;
    const int c = cp ^ oswz(r);
    const uint4 v = *(const uint4*)(ep + r * OROWB + cp * 16);
    const int f = (wm * WM + r) >> 5, o = r & 31;  // the row's fragment of the block (WM is a multiple of 32)
    const int grow = s_frow[f] + o, gcol = col0 + wn * WN + c * 8;
    // non-temporal: the output is not read again by this launch, so it should not displace the
    // operand strips in the L2 / Infinity Cache
    if (o < s_fn[f] && gcol < N)
      __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v), (u32x4*)(C + (size_t)grow * N + gcol));
  }
}

}  // namespace gemmvs
}  // namespace mlora
