// bf16 MFMA GEMM kernel with the LoRA term folded in as extra contraction steps (gfx950):
// four-stage ring of 32-wide contraction tiles, filled by direct global->LDS loads that are
// issued evenly over the whole main loop.
//
//   C[M,N] = A[M,Kd] * op(Bm) + rows_k( L[rows_k, :r_k] * R_k )
//     NN = true  (forward,  Eq. "forward"):      Bm = W [Kd,N] (contraction index = rows of W),  R_k = B_k [r_k, N]
//     NN = false (backward, Eq. "grad_output"):  Bm = W [N,Kd] (contraction index = columns),     R_k = A_k [N, r_k]
//
// Tile 256 x 256 x 32, WAVES_M x WAVES_N waves, fp32 accumulation in v_mfma_f32_32x32x16_bf16
// with the accumulators in AccVGPRs.  Why a ring: the path that carries a CU's loads delivers
// 64 B per clock, and a 256 x 256 tile needs 1 KiB of operands per 128 KFLOP -- at full matrix
// rate that path is busy half of the time.  With two 64-wide stages a stage can only be refilled
// in the last quarter of the tile that frees it, so all waves issue their loads in one burst,
// the path's queue fills, and the waves stall at the load instructions with the matrix pipe idle
// behind them.  With four stages of 32 the tile freed at a barrier is refilled during the whole
// next tile: every wave issues one load per four MFMAs, all the way through the loop, and each
// load has two tiles' time to land.
//   tile v (stage v % 4):
//     step 0: MFMAs (v, 0) | LDS reads of (v, 1)        | second half of the loads of tile v + 3
//     wait until this wave's loads of tile v + 1 have landed; barrier
//       (tile v + 1 is visible; every wave holds its last fragments of tile v in registers,
//        so stage v % 4 is free)
//     step 1: MFMAs (v, 1) | LDS reads of (v + 1, 0)    | first half of the loads of tile v + 4
// LDS layouts (a wave-wide direct load fills 1 KiB of contiguous LDS, so the bank-conflict
// swizzle is applied by choosing which global 16-byte chunk each lane fetches):
//   * K-contiguous tiles (A, and Bm when !NN): 256 rows x 64 B; chunk c of row r sits at chunk
//     position c ^ ((r >> 2) & 3); read with ds_read_b128.
//   * Bm when NN: 32 contraction rows x 512 B; chunk c of row k sits at c ^ ((k & 3) << 2); read
//     with ds_read_b64_tr_b16 -- no transposed copy of W is ever made.
// Rows: as in gemm_mfma_kernel.h the grid tiles a virtual row axis on which every row range of
// the call is padded to whole 32-row MFMA fragments, so that a fragment never holds rows of two
// tasks and a task's LoRA tile runs its MFMAs only on that task's fragments.
#pragma once

#include <type_traits>

#include "gemm_mfma_kernel.h"

namespace mlora {
namespace gemmr {

using namespace stage;
using gemmk::BM;
using gemmk::BN;
using gemmk::g_zero_chunk;
using gemmk::GemmArgs;

template <int WAVES_M, int WAVES_N, bool NN, int NSEG>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void k_gemm_mfma_ring(const GemmArgs<NSEG> ga) {
  constexpr int BK = 32, NS = 4, KS = BK / 16;
  bf16* __restrict__ C = ga.C;
  const int M = ga.M, N = ga.N, tiles_m = ga.tiles_m, tiles_n = ga.tiles_n;
  constexpr int NW = WAVES_M * WAVES_N;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int FM = WM / 32, FN = WN / 32;
  constexpr int NMF = FM * FN;                 // MFMAs per step
  constexpr int NOPS = FM + FN;                // fragment reads per step
  constexpr int ROWB = BK * 2, CPR = BK / 8, RW = 256 / ROWB, RPI = 1024 / ROWB;
  constexpr int TILE_BYTES = BM * ROWB;        // 16 KiB; the NN weight tile (BK x 512 B) has the same size
  constexpr int LPW = TILE_BYTES / 1024 / NW;  // wave-wide loads per wave per operand tile
  constexpr int PT = 2 * LPW;                  // ... per contraction tile
  constexpr int QL = PT / KS;                  // loads per MFMA step
  constexpr int LDE = NMF / QL;                // a load behind every LDE-th MFMA
  static_assert(KS == 2 && PT % KS == 0 && NMF % QL == 0 && NOPS + QL <= NMF, "one memory instruction per MFMA slot");
  static_assert(2 * PT + QL < 64, "vmcnt range");

  __shared__ __attribute__((aligned(1024))) char sAll[2 * NS * TILE_BYTES];
  auto sA = [&](int s) { return sAll + s * TILE_BYTES; };
  auto sB = [&](int s) { return sAll + (NS + s) * TILE_BYTES; };

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
  // real row behind row rl (0..255) of the block's tile; the 16 rows of one wave-wide load lie
  // in one fragment, so f is wave-uniform there
  auto real_row = [&](int rl) {
    const int f = rl >> 5, o = rl & 31;
    const int n = frag_n(f);
    return frag_row(f) + (o < n ? o : (n > 0 ? n - 1 : 0));
  };

  // Accumulators in AccVGPRs: naming one "a" register operand makes the compiler select the
  // AGPR form of the MFMAs, which keeps the accumulator traffic off the VGPR ports that the
  // LDS fragment reads write through.
  {
    float agpr_hint = 0.f;
    asm volatile("" : "+a"(agpr_hint));
  }

  // ---- direct-to-LDS loads: wave-uniform base of the tile's rows (advanced per contraction
  // tile with scalar arithmetic) plus a constant 32-bit per-lane byte offset; set per operand pair
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

  // ---- LoRA contraction tiles.  After the last operand pair's base tiles the same pipeline
  // runs one more tile per (task k that owns fragments of this block, 32 ranks of it): its A side
  // is the task's slice of L (Z or G; zeros for the other fragments), its B side the same ranks of
  // R_k (B_k or A_k), fetched into the same LDS layouts by the same direct loads.  The fragments
  // of one task are consecutive, so the block's tasks are the runs of s_ftask.
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
  // what a tile's loads fetch: base tile kt of the current operand pair, or a LoRA tile
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
  // wave-wide load number idx (0..LPW-1: A side, LPW..PT-1: Bm side) of the tile `lc` describes
  // into stage (sa, sb); lanes outside a LoRA tile's task, rank or columns fetch 16 zero bytes
  // (a direct-to-LDS load cannot be masked)
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
      const bool mine = frag_task(rl >> 5) == t.k;  // wave-uniform: the 16 rows of this load share a fragment
      const char* p = (mine && q < ldz) ? reinterpret_cast<const char*>(L + (size_t)real_row(rl) * ldz + q) : zeros;
      load_lds_16B(p, sa + w * 1024);
    } else {
      const int r = ga.rank[t.sg][t.k];
      const bf16* Rk = static_cast<const bf16*>(ga.R[t.sg].p[t.k]);
      const int w = wave + NW * (idx - LPW);
      const char* p = zeros;
      if (NN) {
        const int kr = 2 * w + (lane >> 5);
        const int c = (lane & 31) ^ ((kr & 3) << 2);
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

  // One MFMA step on fragment set `cur`, at most one memory instruction behind every MFMA: a
  // load of half number `half` (0, 1) of the tile `lc` into (lsa, lsb) behind every LDE-th MFMA
  // (if ld), the fragment reads of the next step into set `cur ^ 1` behind the others (if rd).
  // rd, ld are std::true_type in the steady-state loop (straight-line code) and plain bools in the
  // tiles around it; `fo` is std::true_type there (base tiles: every fragment) or a FragOn.
  auto step = [&](int cur, auto rd, const char* rsa, const char* rsb, int rks, auto ld, const LoadCtx& lc, int half,
                  char* lsa, char* lsb, const auto& fo) {
#pragma unroll
    for (int m = 0; m < NMF; ++m) {
      const int i = m / FN, j = m % FN;
      bool on = true;
      if constexpr (!std::is_same_v<std::decay_t<decltype(fo)>, std::true_type>) on = fo.on[i];
      if (on) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cur][j], af[cur][i], acc[i][j], 0, 0, 0);
      if (m % LDE == LDE - 1) {
        if (ld) issue_one(lc, QL * half + m / LDE, lsa, lsb);
      } else {
        const int op = m - m / LDE;  // the read slots in order
        if (rd && op < NOPS) read_op(rsa, rsb, rks, op, af[cur ^ 1], bfr[cur ^ 1]);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  constexpr std::true_type yes{};
  const LoadCtx none{false, nullptr, nullptr, LoraTile{0, -1, 0}};

  // waits until at most `n` of this wave's loads are in flight (n is a multiple of PT / 2 here)
  auto wait_loads = [&](int n) {
    if (n >= 2 * PT)
      wait_vmcnt<2 * PT>();
    else if (n >= PT + QL)
      wait_vmcnt<PT + QL>();
    else if (n >= PT)
      wait_vmcnt<PT>();
    else if (n >= QL)
      wait_vmcnt<QL>();
    else
      wait_vmcnt<0>();
  };

  // Tile v in stage s.  h1, h3, h4: tiles v+1, v+3, v+4 exist; c3, c4: what tiles v+3, v+4 load;
  // inflight = this wave's loads younger than tile v+1's at the barrier (tiles v+2, v+3).
  auto tile = [&](auto stage, auto h1, auto h3, auto h4, const LoadCtx& c3, const LoadCtx& c4, auto inflight,
                  const auto& fo) {
    const int s = stage;
    const int s1 = (s + 1) % NS, s3 = (s + 3) % NS;
    step(0, yes, sA(s), sB(s), 1, h3, c3, 1, sA(s3), sB(s3), fo);
    if constexpr (std::is_same_v<decltype(inflight), std::true_type>)
      wait_vmcnt<2 * PT>();
    else
      wait_loads(inflight);
    wait_lds();
    __builtin_amdgcn_s_barrier();
    step(1, h1, sA(s1), sB(s1), 0, h4, c4, 0, sA(s), sB(s), fo);
  };
  constexpr std::integral_constant<int, 0> st0{};
  constexpr std::integral_constant<int, 1> st1{};
  constexpr std::integral_constant<int, 2> st2{};
  constexpr std::integral_constant<int, 3> st3{};

  // ---- contraction: operand pairs run one after the other (the ring drains in between)
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
    // prologue: tiles 0, 1, 2 and the first half of tile 3 -- the state a tile's step 1 leaves behind
    int issued = 0;
    for (int u = 0; u < 3 && u < VT; ++u) {
      const LoadCtx cu = ctx_of(u);
#pragma unroll
      for (int idx = 0; idx < PT; ++idx) issue_one(cu, idx, sA(u), sB(u));
      issued += PT;
    }
    if (VT > 3) {
      const LoadCtx cu = ctx_of(3);
#pragma unroll
      for (int idx = 0; idx < QL; ++idx) issue_one(cu, idx, sA(3), sB(3));
      issued += QL;
    }
    wait_loads(issued - PT);  // tile 0 has landed
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int op = 0; op < NOPS; ++op) read_op(sA(0), sB(0), 0, op, af[0], bfr[0]);
    __builtin_amdgcn_sched_barrier(0);
    // steady state, four base tiles per trip (stage addresses are constants): tiles up to v + 7
    // are base tiles
    int v = 0;
    for (; v + 7 < KT; v += 4) {
      tile(st0, yes, yes, yes, base_ctx(v + 3), base_ctx(v + 4), yes, yes);
      tile(st1, yes, yes, yes, base_ctx(v + 4), base_ctx(v + 5), yes, yes);
      tile(st2, yes, yes, yes, base_ctx(v + 5), base_ctx(v + 6), yes, yes);
      tile(st3, yes, yes, yes, base_ctx(v + 6), base_ctx(v + 7), yes, yes);
    }
    // the last base tiles and the LoRA tiles
    for (; v < VT; ++v) {
      const int inflight = (v + 2 < VT ? PT : 0) + (v + 3 < VT ? PT : 0);
      tile(v % NS, v + 1 < VT, v + 3 < VT, v + 4 < VT, ctx_of(v + 3), ctx_of(v + 4), inflight,
           frags_of(v < KT ? -1 : find_lora(v - KT).k));
    }
  }  // operand pairs

  // ---- output: through LDS, so that the tile leaves as 16 B per lane in full row segments of
  // the wave's sub-tile.  Each wave owns WM x WN x 2 bytes of the ring (row stride WN x 2 bytes,
  // chunk c of row m at c ^ swizzle(m)); nothing is shared between waves after the barrier.
  constexpr int OCH = WN / 8;                 // 16-byte chunks per output row of the wave's sub-tile
  constexpr int OROWB = WN * 2;               // bytes per such row
  constexpr int ORPI = 64 / OCH;              // rows per wave-wide store
  constexpr int WBYTES = WM * OROWB;          // bytes per wave
  static_assert(NW * WBYTES == 2 * NS * TILE_BYTES, "sub-tiles must tile the ring");
  typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
  auto oswz = [](int m) { return OCH == 8 ? ((m >> 1) & 7) : (m & (OCH - 1)); };
  __syncthreads();
  char* ep = sAll + wave * WBYTES;
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

}  // namespace gemmr
}  // namespace mlora
