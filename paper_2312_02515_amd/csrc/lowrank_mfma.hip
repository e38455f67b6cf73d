// bf16 MFMA kernels for the low-rank products of the BatchLoRA operator (gfx950).
// Each one streams a full activation tensor once, so HBM bandwidth bounds them;
// MFMA keeps the arithmetic (up to 128 flop per byte at rank 64) off the critical path.
//
//   lowrank_rows   Z = s_k x_k A_k          (forward workflow, section 3.3.1; A_k is [h, r_k])
//                  G = s_k dy_k B_k^T       (first factor of Eq. "grad_lora" / "grad_output"; B_k is [r_k, d])
//   grad           dA_k = x_k^T G           (Eq. "grad_lora", left)
//                  dB_k = Z^T dy_k          (Eq. "grad_lora", right)
//
// One launch covers all tasks: a block finds its task from the split positions.
// Tiles are staged with direct global->LDS loads (16 B per lane) into a 3-stage
// ring, two tiles in flight per block and two blocks per CU (an HBM-bound stream needs tens of KiB in
// flight per CU); operands whose contraction index is not contiguous in memory (A_k, and
// everything in the two gradient products, where the contraction runs over
// tokens) are read from LDS with the transposing ds_read_b64_tr_b16.
#include "mfma_staging.h"
#include "mlora_common.h"

namespace mlora {
namespace {

using namespace stage;

// Bank-conflict swizzle of a small tile stored with the contraction index as its rows
// ([64 k][w] bf16) and read with transposing LDS reads, which touch 4 consecutive rows x 64 B per
// 16 lanes: with rows of 128 or 256 B those rows would share banks, so the 64-byte segments of
// row k are permuted by XOR with seg_swizzle(k, w).  A direct-to-LDS load fills LDS contiguously,
// so the permutation is applied by choosing which global chunk each lane fetches, and undone in
// the read address (column n -> n ^ (seg_swizzle << 5)).
__device__ __forceinline__ int seg_swizzle(int k, int w) {
  return w == 128 ? (k & 3) : (w == 64 ? ((k >> 1) & 1) : 0);
}
// element offset inside the tile that LDS chunk position `chunk` (16 B units) must be filled with
__device__ __forceinline__ int swizzled_source(int chunk, int w) {
  const int cpr = w / 8;
  const int row = chunk / cpr, pc = chunk % cpr;
  const int seg = (pc >> 2) ^ seg_swizzle(row, w);
  return row * w + (((seg << 2) | (pc & 3)) << 3);
}


// ------------------------------------------------------------------------------------------
// Arguments of the two kernels, passed by value.  NP > 1 serves projections that share their
// input: the big operand (X) is streamed once and multiplied with every projection's small
// operand; each projection has its own ranks, scalings, pointers and output.
// ------------------------------------------------------------------------------------------
template <int NP>
struct RowsArgs {
  const bf16* In;                       // [T, inner]
  int inner;
  int K;
  int off[kMaxK + 1];
  bf16* Out[NP];                        // [T, ldz_p]
  int ldz[NP];
  unsigned char rank[NP][kMaxK];
  float s[NP][kMaxK];
  PtrTable M[NP];
};

template <int NP>
struct GradArgs {
  const bf16* Big;                      // [T, wide]
  int wide, T;
  int K;
  int off[kMaxK + 1];
  const bf16* Small[NP];                // [T, ldz_p]
  int ldz[NP];
  unsigned char rank[NP][kMaxK];
  OutTable out[NP];
  int accumulate, chunks;
  // splits > 1 (NP == 1 only): a task's tokens are cut into `splits` ranges, one block each;
  // block (task k, range s) overwrites its partial sums at part + (s * rtotal + rbase_k) * wide
  // (same element order as the output), and k_grad_reduce adds the ranges in order
  int splits, rtotal;
  float* part;
};

// ------------------------------------------------------------------------------------------
// Out_p[i, 0:ldz_p] = s_pk * In[i, :] * M_pk   for the rows i of task k; columns >= r_pk are zero.
//   SMALL_KMAJOR = true : M_k = A_k  [inner, r_k]  (rows of A_k are contraction indices)
//   SMALL_KMAJOR = false: M_k = B_k^T, B_k [r_k, inner]
// Block: TM rows of one task (TM = 32, 64 or 128), one wave per 32 rows, contraction tiles of 64.
// NQ = 32-column groups of the widest Out_p.
// ------------------------------------------------------------------------------------------
template <bool SMALL_KMAJOR, int NQ, int NS, int TM, int NP>
__global__ __launch_bounds__(TM * 2) void k_lowrank_mfma(const RowsArgs<NP> ra) {
  constexpr int NWV = TM / 32;                     // waves per block
  constexpr int SPW = (4 * NQ + NWV - 1) / NWV;    // 1 KiB pieces of one small operand per wave
  constexpr int SBYTES = NQ * 32 * 128;
  // a small-operand tile is followed by 64 zero bytes: where lanes beyond the tile's columns point
  constexpr int SREG = SBYTES + 1024;              // per projection; keeps every 1 KiB load slot aligned
  __shared__ __attribute__((aligned(1024))) char sX0[TM * 128];
  __shared__ __attribute__((aligned(1024))) char sX1[TM * 128];
  __shared__ __attribute__((aligned(1024))) char sX2[TM * 128];
  __shared__ __attribute__((aligned(1024))) char sX3[NS > 3 ? TM * 128 : 16];
  __shared__ __attribute__((aligned(1024))) char sS0[NP * SREG];
  __shared__ __attribute__((aligned(1024))) char sS1[NP * SREG];
  __shared__ __attribute__((aligned(1024))) char sS2[NP * SREG];
  __shared__ __attribute__((aligned(1024))) char sS3[NS > 3 ? NP * SREG : 64];
  static_assert(NS == 3 || NS == 4, "ring depth");
  static_assert(SMALL_KMAJOR || NP == 1, "shared-input form exists for the k-major operand only");
  char* const sX[4] = {sX0, sX1, sX2, sX3};
  char* const sS[4] = {sS0, sS1, sS2, sS3};

  const bf16* __restrict__ In = ra.In;
  const int inner = ra.inner;
  int b = blockIdx.x, k = 0;
  for (; k < ra.K; ++k) {
    const int nb = (ra.off[k + 1] - ra.off[k] + TM - 1) / TM;
    if (b < nb) break;
    b -= nb;
  }
  if (k >= ra.K) return;
  const int lo = ra.off[k] + b * TM;
  const int hi = (ra.off[k + 1] < lo + TM) ? ra.off[k + 1] : lo + TM;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  if (tid < 16) {
#pragma unroll
    for (int s_ = 0; s_ < NS; ++s_)
#pragma unroll
      for (int p = 0; p < NP; ++p) reinterpret_cast<int*>(sS[s_] + p * SREG + SBYTES)[tid] = 0;
  }

  const bf16* xptr[4];
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int rl = 8 * (wave + NWV * it) + (lane >> 3);
    const int c = (lane & 7) ^ ((rl >> 1) & 7);
    int row = lo + rl;
    row = row < hi ? row : hi - 1;
    xptr[it] = In + (size_t)row * inner + c * 8;
  }
  int r[NP];
  size_t sstep[NP];
  const bf16* sptr[NP][SPW];
#pragma unroll
  for (int p = 0; p < NP; ++p) {
    r[p] = ra.rank[p][k];
    const bf16* Mk = static_cast<const bf16*>(ra.M[p].p[k]);
    const int pieces = r[p] / 8;  // 1 KiB pieces of the small operand's tile
#pragma unroll
    for (int it = 0; it < SPW; ++it) {
      // pieces beyond the operand's rank re-fetch piece 0 into their own (never read) slot, so
      // that every wave issues the same number of loads per tile
      const int piece = (wave + NWV * it) < pieces ? (wave + NWV * it) : 0;
      if (SMALL_KMAJOR) {
        sptr[p][it] = Mk + swizzled_source(piece * 64 + lane, r[p]);
      } else {
        int q = 8 * piece + (lane >> 3);
        const int c = (lane & 7) ^ ((q >> 1) & 7);
        q = q < r[p] ? q : r[p] - 1;
        sptr[p][it] = Mk + (size_t)q * inner + c * 8;
      }
    }
    sstep[p] = SMALL_KMAJOR ? (size_t)64 * r[p] : (size_t)64;
  }

  auto issue = [&](int kt, char* sx, char* ss) {
#pragma unroll
    for (int it = 0; it < 4; ++it) load_lds_16B(xptr[it] + (size_t)kt * 64, sx + (wave + NWV * it) * 1024);
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
      for (int it = 0; it < SPW; ++it)
        load_lds_16B(sptr[p][it] + (size_t)kt * sstep[p], ss + p * SREG + (wave + NWV * it) * 1024);
  };
  // loads per wave per tile; the same for every wave because NWV divides 4 NQ
  static_assert((4 * NQ) % NWV == 0, "small-operand pieces must split evenly over the waves");
  constexpr int PER_TILE = 4 + NP * SPW;
  static_assert((NS - 2) * PER_TILE < 64, "vmcnt range");

  const int l32 = lane & 31, lhi = lane >> 5;
  const int fsw = (l32 >> 1) & 7;
  const int L16 = lane & 15, blk = lane >> 4, kq = L16 >> 2;
  const int tr_k = 8 * (blk >> 1) + kq;
  const int tr_n = 16 * (blk & 1) + 4 * (L16 & 3);

  f32x16 acc[NP][NQ];
#pragma unroll
  for (int p = 0; p < NP; ++p)
#pragma unroll
    for (int j = 0; j < NQ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[p][j][e] = 0.f;

  auto compute = [&](const char* sx, const char* ssall) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int coff = ((2 * ks + lhi) ^ fsw) << 4;
      const bf16x8 xf = *(const bf16x8*)(sx + (32 * wave + l32) * 128 + coff);
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        const char* ss = ssall + p * SREG;
#pragma unroll
        for (int j = 0; j < NQ; ++j) {
          if (32 * j < r[p]) {
            bf16x8 sf;
            if (SMALL_KMAJOR) {
              const int n = 32 * j + tr_n;
              const int kk = 16 * ks + tr_k;
              const int ns = n ^ (seg_swizzle(kk, r[p]) << 5);
              const char* p0 = ss + ((n < r[p]) ? (kk * r[p] + ns) * 2 : SBYTES);
              const char* p1 = ss + ((n < r[p]) ? ((kk + 4) * r[p] + ns) * 2 : SBYTES);
              sf = join(lds_read_tr(p0), lds_read_tr(p1));
            } else {
              sf = *(const bf16x8*)(ss + (32 * j + l32) * 128 + coff);
            }
            acc[p][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sf, xf, acc[p][j], 0, 0, 0);
          }
        }
      }
    }
  };

  // NS-stage ring, one barrier per tile: before tile kt is read, this wave's loads of tile kt
  // have landed (the loads of the NS-2 younger tiles may stay in flight); the barrier then makes
  // every wave's part of tile kt visible and tells that all waves are done with tile kt-1,
  // whose stage is refilled next.
  const int KT = inner / 64;
  __syncthreads();  // the zero pads
#pragma unroll
  for (int s_ = 0; s_ < NS - 1; ++s_)
    if (s_ < KT) issue(s_, sX[s_], sS[s_]);
  for (int kt0 = 0; kt0 < KT; kt0 += NS) {
#pragma unroll
    for (int s_ = 0; s_ < NS; ++s_) {
      const int kt = kt0 + s_;
      if (kt < KT) {
        if (kt + NS - 2 < KT)
          wait_vmcnt<(NS - 2) * PER_TILE>();
        else
          wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        if (kt + NS - 1 < KT) issue(kt + NS - 1, sX[(s_ + NS - 1) % NS], sS[(s_ + NS - 1) % NS]);
        compute(sX[s_], sS[s_]);
      }
    }
  }

  // lane holds row m = 32*wave + l32 and columns q = 32j + 8g + 4*lhi + 0..3
  const int row = lo + 32 * wave + l32;
  if (row < hi) {
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      const float s = ra.s[p][k];
      const int ldz = ra.ldz[p];
      bf16* __restrict__ Out = ra.Out[p];
#pragma unroll
      for (int j = 0; j < NQ; ++j) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int q = 32 * j + 8 * g + 4 * lhi;
          if (q < ldz) {
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = static_cast<bf16>((q + e < r[p]) ? acc[p][j][4 * g + e] * s : 0.f);
            *(bf16x4*)(Out + (size_t)row * ldz + q) = o;
          }
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// The same product for calls with few rows (the 32-row tiling still leaves the chip short of
// waves): a block owns 32 rows and its 4 waves split the contraction -- wave w takes the tiles
// kt = w, w + 4, ... through a ring of its own (no barrier in the loop: a wave reads only what
// its own loads wrote), then waves 1..3 hand their partial sums to wave 0 through LDS, which adds
// them in that order (deterministic) and writes the rows.  Ranks up to 64.
// ------------------------------------------------------------------------------------------
template <bool SMALL_KMAJOR, int NQ, int NS>
__global__ __launch_bounds__(256) void k_lowrank_mfma_splitk(const RowsArgs<1> ra) {
  constexpr int TM = 32, NSPLIT = 4;
  constexpr int SBYTES = NQ * 32 * 128;
  constexpr int SREG = SBYTES + 1024;
  constexpr int XB = TM * 128;
  static_assert(NQ <= 2, "LDS holds four rings only up to rank 64");
  __shared__ __attribute__((aligned(1024))) char sXall[NSPLIT * NS * XB];
  __shared__ __attribute__((aligned(1024))) char sSall[NSPLIT * NS * SREG];
  static_assert(3 * NQ * 16 * 256 <= NSPLIT * NS * SREG, "partial sums fit the small-operand rings");

  const bf16* __restrict__ In = ra.In;
  const int inner = ra.inner;
  int b = blockIdx.x, k = 0;
  for (; k < ra.K; ++k) {
    const int nb = (ra.off[k + 1] - ra.off[k] + TM - 1) / TM;
    if (b < nb) break;
    b -= nb;
  }
  if (k >= ra.K) return;
  const int lo = ra.off[k] + b * TM;
  const int hi = (ra.off[k + 1] < lo + TM) ? ra.off[k + 1] : lo + TM;
  const int r = ra.rank[0][k];
  const bf16* Mk = static_cast<const bf16*>(ra.M[0].p[k]);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  char* const sXw = sXall + wave * NS * XB;
  char* const sSw = sSall + wave * NS * SREG;
  if (lane < 16) {
#pragma unroll
    for (int s_ = 0; s_ < NS; ++s_) reinterpret_cast<int*>(sSw + s_ * SREG + SBYTES)[lane] = 0;
  }

  const bf16* xptr[4];
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int rl = 8 * it + (lane >> 3);
    const int c = (lane & 7) ^ ((rl >> 1) & 7);
    int row = lo + rl;
    row = row < hi ? row : hi - 1;
    xptr[it] = In + (size_t)row * inner + c * 8;
  }
  const int pieces = r / 8;
  const bf16* sptr[4 * NQ];
#pragma unroll
  for (int it = 0; it < 4 * NQ; ++it) {
    const int piece = it < pieces ? it : 0;
    if (SMALL_KMAJOR) {
      sptr[it] = Mk + swizzled_source(piece * 64 + lane, r);
    } else {
      int q = 8 * piece + (lane >> 3);
      const int c = (lane & 7) ^ ((q >> 1) & 7);
      q = q < r ? q : r - 1;
      sptr[it] = Mk + (size_t)q * inner + c * 8;
    }
  }
  const size_t sstep = SMALL_KMAJOR ? (size_t)64 * r : (size_t)64;
  constexpr int PER_TILE = 4 + 4 * NQ;

  auto issue = [&](int kt, int stage) {
    char* sx = sXw + stage * XB;
    char* ss = sSw + stage * SREG;
#pragma unroll
    for (int it = 0; it < 4; ++it) load_lds_16B(xptr[it] + (size_t)kt * 64, sx + it * 1024);
#pragma unroll
    for (int it = 0; it < 4 * NQ; ++it) load_lds_16B(sptr[it] + (size_t)kt * sstep, ss + it * 1024);
  };

  const int l32 = lane & 31, lhi = lane >> 5;
  const int fsw = (l32 >> 1) & 7;
  const int L16 = lane & 15, blk = lane >> 4, kq = L16 >> 2;
  const int tr_k = 8 * (blk >> 1) + kq;
  const int tr_n = 16 * (blk & 1) + 4 * (L16 & 3);

  f32x16 acc[NQ];
#pragma unroll
  for (int j = 0; j < NQ; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;

  auto compute = [&](int stage) {
    const char* sx = sXw + stage * XB;
    const char* ss = sSw + stage * SREG;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int coff = ((2 * ks + lhi) ^ fsw) << 4;
      const bf16x8 xf = *(const bf16x8*)(sx + l32 * 128 + coff);
#pragma unroll
      for (int j = 0; j < NQ; ++j) {
        if (32 * j < r) {
          bf16x8 sf;
          if (SMALL_KMAJOR) {
            const int n = 32 * j + tr_n;
            const int kk = 16 * ks + tr_k;
            const int ns = n ^ (seg_swizzle(kk, r) << 5);
            const char* p0 = ss + ((n < r) ? (kk * r + ns) * 2 : SBYTES);
            const char* p1 = ss + ((n < r) ? ((kk + 4) * r + ns) * 2 : SBYTES);
            sf = join(lds_read_tr(p0), lds_read_tr(p1));
          } else {
            sf = *(const bf16x8*)(ss + (32 * j + l32) * 128 + coff);
          }
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sf, xf, acc[j], 0, 0, 0);
        }
      }
    }
  };

  // this wave's tiles: kt = wave + 4 i, i < n
  const int KT = inner / 64;
  const int n = (KT - wave + NSPLIT - 1) / NSPLIT;
#pragma unroll
  for (int s_ = 0; s_ < NS - 1; ++s_)
    if (s_ < n) issue(wave + NSPLIT * s_, s_);
  for (int i0 = 0; i0 < n; i0 += NS) {
#pragma unroll
    for (int s_ = 0; s_ < NS; ++s_) {
      const int i = i0 + s_;
      if (i < n) {
        if (i + NS - 2 < n)
          wait_vmcnt<(NS - 2) * PER_TILE>();
        else
          wait_vmcnt<0>();
        // the stage of tile i-1 is refilled: its fragment reads have returned
        wait_lds();
        if (i + NS - 1 < n) issue(wave + NSPLIT * (i + NS - 1), (s_ + NS - 1) % NS);
        compute(s_);
      }
    }
  }

  // partial sums of waves 1..3 -> LDS (the rings are idle after the barrier), wave 0 adds them
  __syncthreads();
  float* red = reinterpret_cast<float*>(sSall);
  if (wave > 0) {
#pragma unroll
    for (int j = 0; j < NQ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) red[(((wave - 1) * NQ + j) * 16 + e) * 64 + lane] = acc[j][e];
  }
  __syncthreads();
  if (wave > 0) return;
#pragma unroll
  for (int w = 0; w < NSPLIT - 1; ++w)
#pragma unroll
    for (int j = 0; j < NQ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[j][e] += red[((w * NQ + j) * 16 + e) * 64 + lane];

  const float s = ra.s[0][k];
  const int ldz = ra.ldz[0];
  bf16* __restrict__ Out = ra.Out[0];
  const int row = lo + l32;
  if (row < hi) {
#pragma unroll
    for (int j = 0; j < NQ; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int q = 32 * j + 8 * g + 4 * lhi;
        if (q < ldz) {
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = static_cast<bf16>((q + e < r) ? acc[j][4 * g + e] * s : 0.f);
          *(bf16x4*)(Out + (size_t)row * ldz + q) = o;
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Gradient products whose contraction runs over the tokens of one task:
//   WIDE_FIRST = true : out_pk[c, q] (+)= sum_t Big[t, c] * Small_p[t, q]   (dA_k = x_k^T G,  out row stride r_k)
//   WIDE_FIRST = false: out_k[q, j]  (+)= sum_t Small[t, q] * Big[t, j]     (dB_k = Z^T dy_k, out row stride wide)
// Big is [T, wide] (X or dY), Small_p is [T, ldz_p] (G or Z, zero in columns >= r_pk).
// Block: one task, 128 columns of Big, all its tokens in tiles of 64; 4 waves x 32 columns.
// The whole reduction of an output element happens inside one block: deterministic, no atomics.
// ------------------------------------------------------------------------------------------
template <bool WIDE_FIRST, int NQ, int NS, int NP>
__global__ __launch_bounds__(256) void k_grad_mfma(const GradArgs<NP> ga) {
  constexpr int WC = 128;
  constexpr int SBYTES = NQ * 32 * 128;  // 64 tokens x ldz x 2 B, ldz <= 32 NQ
  // a small-operand tile is followed by 64 zero bytes: where lanes beyond the tile's columns point
  constexpr int SREG = SBYTES + 1024;    // per projection; keeps every 1 KiB load slot aligned
  __shared__ __attribute__((aligned(1024))) char sB0[64 * WC * 2];
  __shared__ __attribute__((aligned(1024))) char sB1[64 * WC * 2];
  __shared__ __attribute__((aligned(1024))) char sB2[64 * WC * 2];
  __shared__ __attribute__((aligned(1024))) char sB3[NS > 3 ? 64 * WC * 2 : 16];
  __shared__ __attribute__((aligned(1024))) char sS0[NP * SREG];
  __shared__ __attribute__((aligned(1024))) char sS1[NP * SREG];
  __shared__ __attribute__((aligned(1024))) char sS2[NP * SREG];
  __shared__ __attribute__((aligned(1024))) char sS3[NS > 3 ? NP * SREG : 64];
  static_assert(NS == 3 || NS == 4, "ring depth");
  static_assert(WIDE_FIRST || NP == 1, "shared-input form exists for dA only");
  char* const sB[4] = {sB0, sB1, sB2, sB3};
  char* const sS[4] = {sS0, sS1, sS2, sS3};

  const bf16* __restrict__ Big = ga.Big;
  const int wide = ga.wide;
  const int ch = blockIdx.x % ga.chunks;
  const int sp = (blockIdx.x / ga.chunks) % ga.splits;
  const int k = blockIdx.x / (ga.chunks * ga.splits);
  const int col0 = ch * WC;
  int lo = ga.off[k], hi = ga.off[k + 1];
  if (ga.splits > 1) {
    // token range of this block: whole 64-token tiles, possibly empty (then zeros are written)
    const int len = ((hi - lo + ga.splits - 1) / ga.splits + 63) / 64 * 64;
    lo = lo + sp * len < hi ? lo + sp * len : hi;
    hi = lo + len < hi ? lo + len : hi;
  }
  const int tk = hi - lo;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  if (tid < 16) {
#pragma unroll
    for (int s_ = 0; s_ < NS; ++s_)
#pragma unroll
      for (int p = 0; p < NP; ++p) reinterpret_cast<int*>(sS[s_] + p * SREG + SBYTES)[tid] = 0;
  }

  // Big tile: 64 token rows x 256 B; wave instruction w covers rows 4w..4w+3
  int brow[4], bcol[4];
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int rl = 4 * (wave + 4 * it) + (lane >> 4);
    const int c = (lane & 15) ^ ((rl & 3) << 2);
    int col = col0 + c * 8;
    col = col < wide ? col : wide - 8;
    brow[it] = rl;
    bcol[it] = col;
  }
  // Small tiles: 64 tokens x ldz_p, contiguous in memory; piece = 1 KiB = 64 chunks of 16 B
  int ldz[NP];
  int srow[NP][NQ], scol[NP][NQ];
#pragma unroll
  for (int p = 0; p < NP; ++p) {
    ldz[p] = ga.ldz[p];
    const int cpr = ldz[p] / 8;  // chunks per token row = 1 KiB pieces per tile
#pragma unroll
    for (int it = 0; it < NQ; ++it) {
      // pieces beyond the tile re-fetch piece 0 into their own (never read) slot, so that every
      // wave issues the same number of loads per tile
      const int piece = (wave + 4 * it) < cpr ? (wave + 4 * it) : 0;
      const int src = swizzled_source(piece * 64 + lane, ldz[p]);
      srow[p][it] = src / ldz[p];
      scol[p][it] = src % ldz[p];
    }
  }
  constexpr int PER_TILE = 4 + NP * NQ;
  static_assert((NS - 2) * PER_TILE < 64, "vmcnt range");

  auto issue = [&](int kt, char* sb, char* ss) {
    const int t0 = lo + kt * 64;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      // rows past the block's token range re-read its last row (they meet zeros of the masked
      // small operand): a block touches no row of another task, whatever that row holds
      int tok = t0 + brow[it];
      tok = tok < hi ? tok : hi - 1;
      load_lds_16B(Big + (size_t)tok * wide + bcol[it], sb + (wave + 4 * it) * 1024);
    }
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
      for (int it = 0; it < NQ; ++it) {
        int tok = t0 + srow[p][it];
        tok = tok < hi ? tok : hi - 1;
        load_lds_16B(ga.Small[p] + (size_t)tok * ldz[p] + scol[p][it], ss + p * SREG + (wave + 4 * it) * 1024);
      }
  };

  const int l32 = lane & 31, lhi = lane >> 5;
  const int L16 = lane & 15, blk = lane >> 4, kq = L16 >> 2;
  const int tr_k = 8 * (blk >> 1) + kq;
  const int tr_n = 16 * (blk & 1) + 4 * (L16 & 3);
  const int wide_n = 32 * wave + tr_n;
  const int wide_off = (((wide_n >> 3) ^ (kq << 2)) << 4) + (wide_n & 7) * 2;

  f32x16 acc[NP][NQ];
#pragma unroll
  for (int p = 0; p < NP; ++p)
#pragma unroll
    for (int j = 0; j < NQ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[p][j][e] = 0.f;

  // `valid` = number of tokens of this tile that belong to the task (64 except in the last tile)
  auto compute = [&](const char* sb, const char* ssall, int valid) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int kk = 16 * ks + tr_k;
      const bf16x8 wf = join(lds_read_tr(sb + kk * 256 + wide_off), lds_read_tr(sb + (kk + 4) * 256 + wide_off));
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        const char* ss = ssall + p * SREG;
#pragma unroll
        for (int j = 0; j < NQ; ++j) {
          if (32 * j < ldz[p]) {
            const int n = 32 * j + tr_n;
            const int ns = n ^ (seg_swizzle(kk, ldz[p]) << 5);
            const char* p0 = ss + ((n < ldz[p]) ? (kk * ldz[p] + ns) * 2 : SBYTES);
            const char* p1 = ss + ((n < ldz[p]) ? ((kk + 4) * ldz[p] + ns) * 2 : SBYTES);
            short4v s0 = lds_read_tr(p0), s1 = lds_read_tr(p1);
            if (valid < 64) {
              // the lane's 8 contraction indices are tokens 16ks + 8*lhi + 0..7 of the tile
              const int tbase = 16 * ks + 8 * lhi;
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                if (tbase + e >= valid) s0[e] = 0;
                if (tbase + 4 + e >= valid) s1[e] = 0;
              }
            }
            const bf16x8 sf = join(s0, s1);
            if (WIDE_FIRST)
              acc[p][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, sf, acc[p][j], 0, 0, 0);
            else
              acc[p][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sf, wf, acc[p][j], 0, 0, 0);
          }
        }
      }
    }
  };

  const int KT = (tk + 63) / 64;
  __syncthreads();  // the zero pads
#pragma unroll
  for (int s_ = 0; s_ < NS - 1; ++s_)
    if (s_ < KT) issue(s_, sB[s_], sS[s_]);
  for (int kt0 = 0; kt0 < KT; kt0 += NS) {
#pragma unroll
    for (int s_ = 0; s_ < NS; ++s_) {
      const int kt = kt0 + s_;
      if (kt < KT) {
        if (kt + NS - 2 < KT)
          wait_vmcnt<(NS - 2) * PER_TILE>();
        else
          wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        if (kt + NS - 1 < KT) issue(kt + NS - 1, sB[(s_ + NS - 1) % NS], sS[(s_ + NS - 1) % NS]);
        const int left = tk - kt * 64;
        compute(sB[s_], sS[s_], left < 64 ? left : 64);
      }
    }
  }

  int accumulate = ga.accumulate;
#pragma unroll
  for (int p = 0; p < NP; ++p) {
    float* o = ga.out[p].p[k];
    const int r = ga.rank[p][k];
    if (NP == 1 && ga.splits > 1) {
      int rbase = 0;
      for (int kk = 0; kk < k; ++kk) rbase += ga.rank[0][kk];
      o = ga.part + ((size_t)sp * ga.rtotal + rbase) * wide;
      accumulate = 0;
    }
    if (WIDE_FIRST) {
      // D[i = column c of Big][j = q]: lane holds q = 32j + l32 and c = col0 + 32*wave + 8g + 4*lhi + e
#pragma unroll
      for (int j = 0; j < NQ; ++j) {
        const int q = 32 * j + l32;
        if (q < r) {
#pragma unroll
          for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int c = col0 + 32 * wave + 8 * g + 4 * lhi + e;
              if (c < wide) {
                float* dst = o + (size_t)c * r + q;
                *dst = accumulate ? *dst + acc[p][j][4 * g + e] : acc[p][j][4 * g + e];
              }
            }
        }
      }
    } else {
      // D[i = q][j = column of Big]: lane holds column col0 + 32*wave + l32 and q = 32j + 8g + 4*lhi + e
      const int col = col0 + 32 * wave + l32;
      if (col < wide) {
#pragma unroll
        for (int j = 0; j < NQ; ++j)
#pragma unroll
          for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int q = 32 * j + 8 * g + 4 * lhi + e;
              if (q < r) {
                float* dst = o + (size_t)q * wide + col;
                *dst = accumulate ? *dst + acc[p][j][4 * g + e] : acc[p][j][4 * g + e];
              }
            }
      }
    }
  }
}

// Adds the token ranges' partial sums of k_grad_mfma in range order (deterministic) into the
// tasks' outputs.  One thread per output element; `total` = rtotal * wide elements.
struct ReduceArgs {
  const float* part;
  int splits, rtotal, wide, K, accumulate;
  unsigned char rank[kMaxK];
  OutTable out;
};
__global__ __launch_bounds__(256) void k_grad_reduce(const ReduceArgs a) {
  const size_t total = (size_t)a.rtotal * a.wide;
  const size_t g = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (g >= total) return;
  float sum = 0.f;
  for (int s_ = 0; s_ < a.splits; ++s_) sum += a.part[(size_t)s_ * total + g];
  // which task: element g lies in [rbase_k * wide, (rbase_k + r_k) * wide)
  size_t base = 0;
  int k = 0;
  for (; k < a.K; ++k) {
    const size_t n = (size_t)a.rank[k] * a.wide;
    if (g < base + n) break;
    base += n;
  }
  float* dst = a.out.p[k] + (g - base);
  *dst = a.accumulate ? *dst + sum : sum;
}

// Ring depth: three stages (two tiles in flight) keep a block at 75 KiB of LDS for ranks up to 64,
// so two blocks share a CU; measured 8 % faster than four stages with one block per CU.
constexpr int kRing = 3;

int nq_of(int ldz) { return ldz <= 32 ? 1 : (ldz <= 64 ? 2 : 4); }

int row_blocks(const SegTable& st, int tm) {
  int blocks = 0;
  for (int k = 0; k < st.K; ++k) blocks += (st.off[k + 1] - st.off[k] + tm - 1) / tm;
  return blocks;
}

// the largest row tile that still gives every CU (256) a block: at equal block counts the
// larger tile is faster (fewer fetches of the small operand per row)
int pick_row_tile(const SegTable& st) {
  int tm = 128;
  if (row_blocks(st, tm) < 256) tm = 64;
  if (tm == 64 && row_blocks(st, tm) < 256) tm = 32;
  return tm;
}

// Algorithmic bytes of one launch: the tasks' rows of the big operand read once, the outputs
// written once, the small operands read once.
template <int NP>
double rows_bytes(const RowsArgs<NP>& a) {
  const double rows = a.K > 0 ? a.off[a.K] - a.off[0] : 0;
  double b = rows * a.inner * 2.0;
  for (int p = 0; p < NP; ++p) {
    b += rows * a.ldz[p] * 2.0;
    for (int k = 0; k < a.K; ++k) b += (double)a.rank[p][k] * a.inner * 2.0;
  }
  return b;
}

template <int NP>
double grad_bytes(const GradArgs<NP>& a) {
  const double rows = a.K > 0 ? a.off[a.K] - a.off[0] : 0;
  double b = rows * a.wide * 2.0;
  for (int p = 0; p < NP; ++p) {
    b += rows * a.ldz[p] * 2.0;
    for (int k = 0; k < a.K; ++k) b += (double)a.rank[p][k] * a.wide * 4.0;
  }
  return b;
}

template <bool KMAJOR, int NQ, int TM, int NP>
hipError_t launch_rows_one(const RowsArgs<NP>& a, int blocks, hipStream_t s) {
  if constexpr (NP * NQ <= 8) {
    const int slot = profile_begin(kProfileRows, rows_bytes(a), s);
    hipLaunchKernelGGL((k_lowrank_mfma<KMAJOR, NQ, kRing, TM, NP>), dim3(blocks), dim3(TM * 2), 0, s, a);
    const hipError_t e = hipGetLastError();
    profile_end(slot, s);
    return e;
  } else {
    return hipErrorInvalidValue;
  }
}

template <bool KMAJOR, int NQ, int NP>
hipError_t launch_rows_tm(const RowsArgs<NP>& a, int tm, int blocks, hipStream_t s) {
  if (tm == 128) return launch_rows_one<KMAJOR, NQ, 128, NP>(a, blocks, s);
  if (tm == 64) return launch_rows_one<KMAJOR, NQ, 64, NP>(a, blocks, s);
  return launch_rows_one<KMAJOR, NQ, 32, NP>(a, blocks, s);
}

template <bool KMAJOR, int NQ>
hipError_t launch_rows_splitk(const RowsArgs<1>& a, int blocks, hipStream_t s) {
  const int slot = profile_begin(kProfileRows, rows_bytes(a), s);
  hipLaunchKernelGGL((k_lowrank_mfma_splitk<KMAJOR, NQ, kRing>), dim3(blocks), dim3(256), 0, s, a);
  const hipError_t e = hipGetLastError();
  profile_end(slot, s);
  return e;
}

template <bool KMAJOR, int NP>
hipError_t launch_rows(const RowsArgs<NP>& a, int nq, int tm, int blocks, hipStream_t s) {
  if constexpr (NP == 1) {
    // few rows: four waves per 32-row block, each on a quarter of the contraction
    if (tm == 32 && nq <= 2 && a.inner >= 1024 && blocks <= 1024) {
      return nq == 1 ? launch_rows_splitk<KMAJOR, 1>(a, blocks, s) : launch_rows_splitk<KMAJOR, 2>(a, blocks, s);
    }
  }
  if (nq == 1) return launch_rows_tm<KMAJOR, 1, NP>(a, tm, blocks, s);
  if (nq == 2) return launch_rows_tm<KMAJOR, 2, NP>(a, tm, blocks, s);
  return launch_rows_tm<KMAJOR, 4, NP>(a, tm, blocks, s);
}

template <bool WIDE_FIRST, int NQ, int NP>
hipError_t launch_grad_one(const GradArgs<NP>& a, int blocks, hipStream_t s) {
  if constexpr (NP * NQ <= 8) {
    const int slot = profile_begin(kProfileGrad, grad_bytes(a), s);
    hipLaunchKernelGGL((k_grad_mfma<WIDE_FIRST, NQ, kRing, NP>), dim3(blocks), dim3(256), 0, s, a);
    const hipError_t e = hipGetLastError();
    profile_end(slot, s);
    return e;
  } else {
    return hipErrorInvalidValue;
  }
}

template <bool WIDE_FIRST, int NP>
hipError_t launch_grad(const GradArgs<NP>& a, int nq, int blocks, hipStream_t s) {
  if (nq == 1) return launch_grad_one<WIDE_FIRST, 1, NP>(a, blocks, s);
  if (nq == 2) return launch_grad_one<WIDE_FIRST, 2, NP>(a, blocks, s);
  return launch_grad_one<WIDE_FIRST, 4, NP>(a, blocks, s);
}

template <int NP>
hipError_t rows_group(const LowrankGroupItem* it, const SegTable& st, const bf16* In, int inner, int nq, hipStream_t s) {
  RowsArgs<NP> a;
  a.In = In;
  a.inner = inner;
  a.K = st.K;
  for (int k = 0; k <= kMaxK; ++k) a.off[k] = st.off[k];
  for (int p = 0; p < NP; ++p) {
    a.Out[p] = it[p].rows_out;
    a.ldz[p] = it[p].ldz;
    for (int k = 0; k < kMaxK; ++k) {
      a.rank[p][k] = (unsigned char)(k < st.K ? it[p].rank[k] : 0);
      a.s[p][k] = k < st.K ? it[p].s[k] : 0.f;
    }
    a.M[p] = *it[p].M;
  }
  const int tm = pick_row_tile(st);
  const int blocks = row_blocks(st, tm);
  if (blocks == 0) return hipSuccess;
  return launch_rows<true, NP>(a, nq, tm, blocks, s);
}

template <int NP>
hipError_t grad_group(const LowrankGroupItem* it, const SegTable& st, const bf16* Big, int wide, int T, int nq,
                      int accumulate, hipStream_t s) {
  GradArgs<NP> a;
  a.Big = Big;
  a.wide = wide;
  a.T = T;
  a.K = st.K;
  for (int k = 0; k <= kMaxK; ++k) a.off[k] = st.off[k];
  for (int p = 0; p < NP; ++p) {
    a.Small[p] = it[p].grad_small;
    a.ldz[p] = it[p].ldz;
    for (int k = 0; k < kMaxK; ++k) a.rank[p][k] = (unsigned char)(k < st.K ? it[p].rank[k] : 0);
    a.out[p] = *it[p].grad_out;
  }
  a.accumulate = accumulate;
  a.chunks = (wide + 127) / 128;
  a.splits = 1;
  a.rtotal = 0;
  a.part = nullptr;
  return launch_grad<true, NP>(a, nq, st.K * a.chunks, s);
}

}  // namespace

// Z = s x A (a_major = true, M = A_k) or G = s dy B^T (a_major = false, M = B_k).
hipError_t lowrank_rows_mfma(const CallCtx& c, const bf16* In, int inner, bf16* Out, const PtrTable& M,
                             bool a_major) {
  const int tm = pick_row_tile(c.st);
  const int blocks = row_blocks(c.st, tm);
  if (blocks == 0) return hipSuccess;
  RowsArgs<1> a;
  a.In = In;
  a.inner = inner;
  a.K = c.st.K;
  for (int k = 0; k <= kMaxK; ++k) a.off[k] = c.st.off[k];
  a.Out[0] = Out;
  a.ldz[0] = c.ldz;
  for (int k = 0; k < kMaxK; ++k) {
    a.rank[0][k] = (unsigned char)c.st.rank[k];
    a.s[0][k] = c.st.s[k];
  }
  a.M[0] = M;
  const int nq = nq_of(c.ldz);
  return a_major ? launch_rows<true, 1>(a, nq, tm, blocks, c.stream) : launch_rows<false, 1>(a, nq, tm, blocks, c.stream);
}

// dA_k = x_k^T G (wide_first = true; Big = X [T,h], Small = G) or dB_k = Z^T dy_k (Big = dY [T,d], Small = Z).
// Token ranges per task for the gradient kernels: 1 when tasks x column blocks fill the chip,
// otherwise enough ranges for about two blocks per CU (at most 16, at least 256 tokens each).
int grad_splits(const SegTable& st, int wide) {
  const int blocks = st.K * ((wide + 127) / 128);
  if (st.K == 0 || blocks >= 384) return 1;
  int longest = 0;
  for (int k = 0; k < st.K; ++k) longest = st.off[k + 1] - st.off[k] > longest ? st.off[k + 1] - st.off[k] : longest;
  int s = (512 + blocks - 1) / blocks;
  s = s < 16 ? s : 16;
  s = s < longest / 256 ? s : longest / 256;
  return s > 1 ? s : 1;
}

// Bytes of partial sums grad_mfma needs for an output of `wide` columns (0 when it does not split).
size_t grad_partial_bytes(const SegTable& st, int wide) {
  const int s = grad_splits(st, wide);
  if (s <= 1) return 0;
  size_t rtotal = 0;
  for (int k = 0; k < st.K; ++k) rtotal += st.rank[k];
  return align_up((size_t)s * rtotal * wide * sizeof(float), 256);
}

hipError_t grad_mfma(const CallCtx& c, const bf16* Big, int wide, const bf16* Small, const OutTable& out,
                     int accumulate, bool wide_first, float* partial) {
  if (c.K == 0) return hipSuccess;
  GradArgs<1> a;
  a.Big = Big;
  a.wide = wide;
  a.T = c.T;
  a.K = c.st.K;
  for (int k = 0; k <= kMaxK; ++k) a.off[k] = c.st.off[k];
  a.Small[0] = Small;
  a.ldz[0] = c.ldz;
  for (int k = 0; k < kMaxK; ++k) a.rank[0][k] = (unsigned char)c.st.rank[k];
  a.out[0] = out;
  a.accumulate = accumulate;
  a.chunks = (wide + 127) / 128;
  a.splits = partial != nullptr ? grad_splits(c.st, wide) : 1;
  a.rtotal = 0;
  for (int k = 0; k < c.K; ++k) a.rtotal += c.st.rank[k];
  a.part = partial;
  const int nq = nq_of(c.ldz);
  const int blocks = c.K * a.chunks * a.splits;
  hipError_t e =
      wide_first ? launch_grad<true, 1>(a, nq, blocks, c.stream) : launch_grad<false, 1>(a, nq, blocks, c.stream);
  if (e != hipSuccess || a.splits == 1) return e;
  ReduceArgs r;
  r.part = partial;
  r.splits = a.splits;
  r.rtotal = a.rtotal;
  r.wide = wide;
  r.K = c.K;
  r.accumulate = accumulate;
  for (int k = 0; k < kMaxK; ++k) r.rank[k] = (unsigned char)c.st.rank[k];
  r.out = out;
  const size_t total = (size_t)a.rtotal * wide;
  // timed with the gradient kernels (its time counts, the launch adds no algorithmic bytes)
  const int slot = profile_begin(kProfileGrad, 0.0, c.stream);
  hipLaunchKernelGGL(k_grad_reduce, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, c.stream, r);
  e = hipGetLastError();
  profile_end(slot, c.stream);
  return e;
}

// Whether np projections whose widest low-rank row stride is max_ldz fit the shared-input kernels
// (accumulators: np x ceil(max_ldz / 32) MFMA column groups, at most 8).
bool lowrank_group_ok(int np, int max_ldz) { return np >= 2 && np <= 4 && np * nq_of(max_ldz) <= 8; }

// Z_p = s_pk x_k A_pk for np projections in one pass over X.
hipError_t lowrank_rows_mfma_group(int np, const LowrankGroupItem* items, const SegTable& st, const bf16* X, int h,
                                   hipStream_t stream) {
  int mx = 0;
  for (int p = 0; p < np; ++p) mx = items[p].ldz > mx ? items[p].ldz : mx;
  if (!lowrank_group_ok(np, mx)) return hipErrorInvalidValue;
  const int nq = nq_of(mx);
  if (np == 2) return rows_group<2>(items, st, X, h, nq, stream);
  if (np == 3) return rows_group<3>(items, st, X, h, nq, stream);
  return rows_group<4>(items, st, X, h, nq, stream);
}

// dA_pk = x_k^T G_p for np projections in one pass over X.
hipError_t grad_mfma_group(int np, const LowrankGroupItem* items, const SegTable& st, const bf16* X, int h, int T,
                           int accumulate, hipStream_t stream) {
  if (st.K == 0) return hipSuccess;
  int mx = 0;
  for (int p = 0; p < np; ++p) mx = items[p].ldz > mx ? items[p].ldz : mx;
  if (!lowrank_group_ok(np, mx)) return hipErrorInvalidValue;
  const int nq = nq_of(mx);
  if (np == 2) return grad_group<2>(items, st, X, h, T, nq, accumulate, stream);
  if (np == 3) return grad_group<3>(items, st, X, h, T, nq, accumulate, stream);
  return grad_group<4>(items, st, X, h, T, nq, accumulate, stream);
}

}  // namespace mlora
