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


// ------------------------------------------------------------------------------------------
// Out[i, 0:ldz] = s_k * In[i, :] * M_k   for the rows i of task k; columns >= r_k are zero.
//   SMALL_KMAJOR = true : M_k = A_k  [inner, r_k]  (rows of A_k are contraction indices)
//   SMALL_KMAJOR = false: M_k = B_k^T, B_k [r_k, inner]
// Block: TM rows of one task (TM = 32, 64 or 128), one wave per 32 rows, contraction tiles of 64.
// ------------------------------------------------------------------------------------------
template <bool SMALL_KMAJOR, int NQ, int NS, int TM>
__global__ __launch_bounds__(TM * 2) void k_lowrank_mfma(const bf16* __restrict__ In, int inner,
                                                         bf16* __restrict__ Out, int ldz, SegTable st, PtrTable Mp) {
  constexpr int NWV = TM / 32;                     // waves per block
  constexpr int SPW = (4 * NQ + NWV - 1) / NWV;    // 1 KiB pieces of the small operand per wave
  constexpr int SBYTES = NQ * 32 * 128;
  __shared__ __attribute__((aligned(1024))) char sX0[TM * 128];
  __shared__ __attribute__((aligned(1024))) char sX1[TM * 128];
  __shared__ __attribute__((aligned(1024))) char sX2[TM * 128];
  __shared__ __attribute__((aligned(1024))) char sX3[NS > 3 ? TM * 128 : 16];
  // 64 zero bytes behind each small-operand tile: where lanes beyond the tile's columns point
  __shared__ __attribute__((aligned(1024))) char sS0[SBYTES + 64];
  __shared__ __attribute__((aligned(1024))) char sS1[SBYTES + 64];
  __shared__ __attribute__((aligned(1024))) char sS2[SBYTES + 64];
  __shared__ __attribute__((aligned(1024))) char sS3[NS > 3 ? SBYTES + 64 : 64];
  static_assert(NS == 3 || NS == 4, "ring depth");
  char* const sX[4] = {sX0, sX1, sX2, sX3};
  char* const sS[4] = {sS0, sS1, sS2, sS3};

  int b = blockIdx.x, k = 0;
  for (; k < st.K; ++k) {
    const int nb = (st.off[k + 1] - st.off[k] + TM - 1) / TM;
    if (b < nb) break;
    b -= nb;
  }
  if (k >= st.K) return;
  const int lo = st.off[k] + b * TM;
  const int hi = (st.off[k + 1] < lo + TM) ? st.off[k + 1] : lo + TM;
  const int r = st.rank[k];
  const float s = st.s[k];
  const bf16* Mk = static_cast<const bf16*>(Mp.p[k]);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  if (tid < 16) {
#pragma unroll
    for (int s_ = 0; s_ < NS; ++s_) reinterpret_cast<int*>(sS[s_] + SBYTES)[tid] = 0;
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
  const int pieces = r / 8;  // 1 KiB pieces of the small operand's tile
  const bf16* sptr[SPW];
#pragma unroll
  for (int it = 0; it < SPW; ++it) {
    // pieces beyond the operand's rank re-fetch piece 0 into their own (never read) slot, so
    // that every wave issues the same number of loads per tile
    const int piece = (wave + NWV * it) < pieces ? (wave + NWV * it) : 0;
    if (SMALL_KMAJOR) {
      sptr[it] = Mk + piece * 512 + lane * 8;
    } else {
      int q = 8 * piece + (lane >> 3);
      const int c = (lane & 7) ^ ((q >> 1) & 7);
      q = q < r ? q : r - 1;
      sptr[it] = Mk + (size_t)q * inner + c * 8;
    }
  }
  const size_t sstep = SMALL_KMAJOR ? (size_t)64 * r : (size_t)64;

  auto issue = [&](int kt, char* sx, char* ss) {
#pragma unroll
    for (int it = 0; it < 4; ++it) load_lds_16B(xptr[it] + (size_t)kt * 64, sx + (wave + NWV * it) * 1024);
#pragma unroll
    for (int it = 0; it < SPW; ++it)
      if (wave + NWV * it < 4 * NQ) load_lds_16B(sptr[it] + (size_t)kt * sstep, ss + (wave + NWV * it) * 1024);
  };
  // loads per wave per tile; the same for every wave when NWV divides 4 NQ (it always does here)
  static_assert((4 * NQ) % NWV == 0, "small-operand pieces must split evenly over the waves");
  constexpr int PER_TILE = 4 + SPW;

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

  auto compute = [&](const char* sx, const char* ss) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int coff = ((2 * ks + lhi) ^ fsw) << 4;
      const bf16x8 xf = *(const bf16x8*)(sx + (32 * wave + l32) * 128 + coff);
#pragma unroll
      for (int j = 0; j < NQ; ++j) {
        if (32 * j < r) {
          bf16x8 sf;
          if (SMALL_KMAJOR) {
            const int n = 32 * j + tr_n;
            const int kk = 16 * ks + tr_k;
            const char* p0 = ss + ((n < r) ? (kk * r + n) * 2 : SBYTES);
            const char* p1 = ss + ((n < r) ? ((kk + 4) * r + n) * 2 : SBYTES);
            sf = join(lds_read_tr(p0), lds_read_tr(p1));
          } else {
            sf = *(const bf16x8*)(ss + (32 * j + l32) * 128 + coff);
          }
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sf, xf, acc[j], 0, 0, 0);
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
//   WIDE_FIRST = true : out_k[p, q] (+)= sum_t Big[t, p] * Small[t, q]   (dA_k = x_k^T G,  out row stride r_k)
//   WIDE_FIRST = false: out_k[q, j] (+)= sum_t Small[t, q] * Big[t, j]   (dB_k = Z^T dy_k, out row stride wide)
// Big is [T, wide] (X or dY), Small is [T, ldz] (G or Z, zero in columns >= r_k).
// Block: one task, 128 columns of Big, all its tokens in tiles of 64; 4 waves x 32 columns.
// The whole reduction of an output element happens inside one block: deterministic, no atomics.
// ------------------------------------------------------------------------------------------
template <bool WIDE_FIRST, int NQ, int NS>
__global__ __launch_bounds__(256) void k_grad_mfma(const bf16* __restrict__ Big, int wide, int T,
                                                   const bf16* __restrict__ Small, int ldz, SegTable st,
                                                   OutTable out, int accumulate, int chunks) {
  constexpr int WC = 128;
  constexpr int SBYTES = NQ * 32 * 128;  // 64 tokens x ldz x 2 B, ldz <= 32 NQ
  __shared__ __attribute__((aligned(1024))) char sB0[64 * WC * 2];
  __shared__ __attribute__((aligned(1024))) char sB1[64 * WC * 2];
  __shared__ __attribute__((aligned(1024))) char sB2[64 * WC * 2];
  __shared__ __attribute__((aligned(1024))) char sB3[NS > 3 ? 64 * WC * 2 : 16];
  // 64 zero bytes behind each small-operand tile: where lanes beyond the tile's columns point
  __shared__ __attribute__((aligned(1024))) char sS0[SBYTES + 64];
  __shared__ __attribute__((aligned(1024))) char sS1[SBYTES + 64];
  __shared__ __attribute__((aligned(1024))) char sS2[SBYTES + 64];
  __shared__ __attribute__((aligned(1024))) char sS3[NS > 3 ? SBYTES + 64 : 64];
  static_assert(NS == 3 || NS == 4, "ring depth");
  char* const sB[4] = {sB0, sB1, sB2, sB3};
  char* const sS[4] = {sS0, sS1, sS2, sS3};

  const int k = blockIdx.x / chunks, ch = blockIdx.x % chunks;
  const int col0 = ch * WC;
  const int lo = st.off[k], hi = st.off[k + 1];
  const int tk = hi - lo;
  const int r = st.rank[k];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  if (tid < 16) {
#pragma unroll
    for (int s_ = 0; s_ < NS; ++s_) reinterpret_cast<int*>(sS[s_] + SBYTES)[tid] = 0;
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
  // Small tile: 64 tokens x ldz, contiguous in memory; piece = 1 KiB = 64 chunks of 16 B
  const int cpr = ldz / 8;  // chunks per token row
  const int pieces = ldz / 8;
  int srow[NQ], scol[NQ];
#pragma unroll
  for (int it = 0; it < NQ; ++it) {
    // pieces beyond the tile re-fetch piece 0 into their own (never read) slot, so that every
    // wave issues the same number of loads per tile
    const int piece = (wave + 4 * it) < pieces ? (wave + 4 * it) : 0;
    const int chunk = piece * 64 + lane;
    srow[it] = chunk / cpr;
    scol[it] = (chunk % cpr) * 8;
  }
  constexpr int PER_TILE = 4 + NQ;

  auto issue = [&](int kt, char* sb, char* ss) {
    const int t0 = lo + kt * 64;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      int tok = t0 + brow[it];
      tok = tok < T ? tok : T - 1;
      load_lds_16B(Big + (size_t)tok * wide + bcol[it], sb + (wave + 4 * it) * 1024);
    }
#pragma unroll
    for (int it = 0; it < NQ; ++it) {
      int tok = t0 + srow[it];
      tok = tok < T ? tok : T - 1;
      load_lds_16B(Small + (size_t)tok * ldz + scol[it], ss + (wave + 4 * it) * 1024);
    }
  };

  const int l32 = lane & 31, lhi = lane >> 5;
  const int L16 = lane & 15, blk = lane >> 4, kq = L16 >> 2;
  const int tr_k = 8 * (blk >> 1) + kq;
  const int tr_n = 16 * (blk & 1) + 4 * (L16 & 3);
  const int wide_n = 32 * wave + tr_n;
  const int wide_off = (((wide_n >> 3) ^ (kq << 2)) << 4) + (wide_n & 7) * 2;

  f32x16 acc[NQ];
#pragma unroll
  for (int j = 0; j < NQ; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;

  // `valid` = number of tokens of this tile that belong to the task (64 except in the last tile)
  auto compute = [&](const char* sb, const char* ss, int valid) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int kk = 16 * ks + tr_k;
      const bf16x8 wf = join(lds_read_tr(sb + kk * 256 + wide_off), lds_read_tr(sb + (kk + 4) * 256 + wide_off));
#pragma unroll
      for (int j = 0; j < NQ; ++j) {
        if (32 * j < ldz) {
          const int n = 32 * j + tr_n;
          const char* p0 = ss + ((n < ldz) ? (kk * ldz + n) * 2 : SBYTES);
          const char* p1 = ss + ((n < ldz) ? ((kk + 4) * ldz + n) * 2 : SBYTES);
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
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, sf, acc[j], 0, 0, 0);
          else
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sf, wf, acc[j], 0, 0, 0);
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

  float* o = out.p[k];
  if (WIDE_FIRST) {
    // D[i = column p of Big][j = q]: lane holds q = 32j + l32 and p = col0 + 32*wave + 8g + 4*lhi + e
#pragma unroll
    for (int j = 0; j < NQ; ++j) {
      const int q = 32 * j + l32;
      if (q < r) {
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int p = col0 + 32 * wave + 8 * g + 4 * lhi + e;
            if (p < wide) {
              float* dst = o + (size_t)p * r + q;
              *dst = accumulate ? *dst + acc[j][4 * g + e] : acc[j][4 * g + e];
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
              *dst = accumulate ? *dst + acc[j][4 * g + e] : acc[j][4 * g + e];
            }
          }
    }
  }
}

// Ring depth: three stages (two tiles in flight) keep a block at 72 KiB of LDS for ranks up to 64,
// so two blocks share a CU; measured 8 % faster than four stages with one block per CU.
constexpr int kRing = 3;

template <bool KMAJOR, int TM, int NS>
void launch_rows_tm(int nq, dim3 grid, hipStream_t s, const bf16* In, int inner, bf16* Out, int ldz, const SegTable& st,
                    const PtrTable& M) {
  if (nq == 1)
    hipLaunchKernelGGL((k_lowrank_mfma<KMAJOR, 1, NS, TM>), grid, dim3(TM * 2), 0, s, In, inner, Out, ldz, st, M);
  else if (nq == 2)
    hipLaunchKernelGGL((k_lowrank_mfma<KMAJOR, 2, NS, TM>), grid, dim3(TM * 2), 0, s, In, inner, Out, ldz, st, M);
  else
    hipLaunchKernelGGL((k_lowrank_mfma<KMAJOR, 4, NS, TM>), grid, dim3(TM * 2), 0, s, In, inner, Out, ldz, st, M);
}

int row_blocks(const SegTable& st, int tm) {
  int blocks = 0;
  for (int k = 0; k < st.K; ++k) blocks += (st.off[k + 1] - st.off[k] + tm - 1) / tm;
  return blocks;
}

template <bool WIDE_FIRST>
void launch_grad(int nq, dim3 grid, hipStream_t s, const bf16* Big, int wide, int T, const bf16* Small, int ldz,
                 const SegTable& st, const OutTable& out, int accumulate, int chunks) {
  if (nq == 1)
    hipLaunchKernelGGL((k_grad_mfma<WIDE_FIRST, 1, kRing>), grid, dim3(256), 0, s, Big, wide, T, Small, ldz, st, out,
                       accumulate, chunks);
  else if (nq == 2)
    hipLaunchKernelGGL((k_grad_mfma<WIDE_FIRST, 2, kRing>), grid, dim3(256), 0, s, Big, wide, T, Small, ldz, st, out,
                       accumulate, chunks);
  else
    hipLaunchKernelGGL((k_grad_mfma<WIDE_FIRST, 4, kRing>), grid, dim3(256), 0, s, Big, wide, T, Small, ldz, st, out,
                       accumulate, chunks);
}

int nq_of(int ldz) { return ldz <= 32 ? 1 : (ldz <= 64 ? 2 : 4); }

}  // namespace

// Z = s x A (a_major = true, M = A_k) or G = s dy B^T (a_major = false, M = B_k).
hipError_t lowrank_rows_mfma(const CallCtx& c, const bf16* In, int inner, bf16* Out, const PtrTable& M,
                             bool a_major) {
  // the largest row tile that still gives every CU (256) a block: at equal block counts the
  // larger tile is faster (fewer fetches of the small operand per row)
  int tm = 128;
  if (row_blocks(c.st, tm) < 256) tm = 64;
  if (tm == 64 && row_blocks(c.st, tm) < 256) tm = 32;
  const int blocks = row_blocks(c.st, tm);
  if (blocks == 0) return hipSuccess;
  const int nq = nq_of(c.ldz);
  const dim3 grid(blocks);
#define MLORA_ROWS(KM)                                                                           \
  do {                                                                                           \
    if (tm == 128) launch_rows_tm<KM, 128, kRing>(nq, grid, c.stream, In, inner, Out, c.ldz, c.st, M);     \
    else if (tm == 64) launch_rows_tm<KM, 64, kRing>(nq, grid, c.stream, In, inner, Out, c.ldz, c.st, M);  \
    else launch_rows_tm<KM, 32, kRing>(nq, grid, c.stream, In, inner, Out, c.ldz, c.st, M);                \
  } while (0)
  if (a_major)
    MLORA_ROWS(true);
  else
    MLORA_ROWS(false);
#undef MLORA_ROWS
  return hipGetLastError();
}

// dA_k = x_k^T G (wide_first = true; Big = X [T,h], Small = G) or dB_k = Z^T dy_k (Big = dY [T,d], Small = Z).
hipError_t grad_mfma(const CallCtx& c, const bf16* Big, int wide, const bf16* Small, const OutTable& out,
                     int accumulate, bool wide_first) {
  if (c.K == 0) return hipSuccess;
  const int chunks = (wide + 127) / 128;
  const dim3 grid(c.K * chunks);
  if (wide_first)
    launch_grad<true>(nq_of(c.ldz), grid, c.stream, Big, wide, c.T, Small, c.ldz, c.st, out, accumulate, chunks);
  else
    launch_grad<false>(nq_of(c.ldz), grid, c.stream, Big, wide, c.T, Small, c.ldz, c.st, out, accumulate, chunks);
  return hipGetLastError();
}

}  // namespace mlora
