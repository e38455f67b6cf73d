// bf16 MFMA GEMM with the LoRA term folded in as extra contraction steps (gfx950).
//
//   forward  (Eq. "forward"):      Y  = X W   + Z B_k      (NN: W is [h,d], contraction index = rows of W)
//   backward (Eq. "grad_output"):  dX = dY W^T + G A_k^T   (NT: W is [h,d], contraction index = columns of W)
//
// where Z = s_k x_k A_k and G = s_k dy_k B_k^T are the [T, ldz] low-rank
// intermediates.  The base product is launched once over all tasks' rows; after
// its contraction loop each 256-row tile runs, for every task whose rows it
// holds, a few more MFMA steps whose left operand is the task's slice of Z (or
// G), zero outside the task's rows, and whose right operand is B_k (or A_k^T).
// The output tile is written once with the LoRA term already in it.
//
// Tile 256 x 256 x 64, fp32 accumulation in v_mfma_f32_32x32x16_bf16.  Both
// operand tiles are fetched with direct global->LDS loads (16 B per lane,
// global_load_lds_dwordx4) into a double buffer.  Each wave instruction of such
// a load fills 1 KiB of contiguous LDS, so the bank-conflict swizzle is applied
// by choosing which global 16-byte chunk each lane fetches.
//   * K-contiguous tiles (X, dY, W in NT mode): 256 rows x 128 B; the chunk c of
//     row r is stored at chunk position c ^ ((r >> 1) & 7); operands are read
//     with ds_read_b128.
//   * W in NN mode: 64 contraction rows x 512 B; chunk c of row k is stored at
//     c ^ ((k & 3) << 2); operands are read with ds_read_b64_tr_b16, which hands
//     each lane four consecutive contraction indices of one output column.
// The MFMA is issued with the weight fragment as its first operand so that each
// lane ends up with four consecutive output columns of one row (8-byte stores).
#include <mutex>
#include <vector>

#include "mlora_common.h"

namespace mlora {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(8))) short short8v;

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int TILE_BYTES = 32768;

#define AS1 __attribute__((address_space(1)))
#define AS3 __attribute__((address_space(3)))

__device__ __forceinline__ void load_lds_16B(const void* g, char* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const AS1 void*)g, (AS3 void*)lds_wave_base, 16, 0, 0);
}

__device__ __forceinline__ bf16x8 lds_read_tr_pair(const char* p0, const char* p1) {
  short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((AS3 short4v*)p0);
  short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((AS3 short4v*)p1);
  short8v v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

template <int WAVES_M, int WAVES_N, bool NN>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void k_gemm_mfma(
    const bf16* __restrict__ A, const bf16* __restrict__ Bm, bf16* __restrict__ C, int M, int N, int Kd,
    const bf16* __restrict__ L, int ldz, SegTable st, PtrTable R, int tiles_m, int tiles_n) {
  constexpr int NW = WAVES_M * WAVES_N, NT = NW * 64;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int FM = WM / 32, FN = WN / 32;
  constexpr int LPW = 32 / NW;  // 1 KiB load instructions per wave per operand tile

  __shared__ __attribute__((aligned(1024))) char sA0[TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) char sA1[TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) char sB0[TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) char sB1[TILE_BYTES];

  // ---- block -> tile: consecutive block ids go round-robin over the 8 XCDs, so give each
  // XCD one contiguous range of a grouped tile order (8 row tiles x all column tiles per group)
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
  const int row0 = tm * BM, col0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  // ---- per-lane global source of every direct-to-LDS load of one k-tile
  const bf16* aptr[LPW];
  const bf16* bptr[LPW];
#pragma unroll
  for (int it = 0; it < LPW; ++it) {
    const int w = wave + NW * it;
    {
      const int rl = 8 * w + (lane >> 3);
      const int c = (lane & 7) ^ ((rl >> 1) & 7);
      int gr = row0 + rl;
      gr = gr < M ? gr : M - 1;
      aptr[it] = A + (size_t)gr * Kd + c * 8;
    }
    if (NN) {
      const int kr = 2 * w + (lane >> 5);
      const int c = (lane & 31) ^ ((kr & 3) << 2);
      int n = col0 + c * 8;
      n = n < N ? n : N - 8;
      bptr[it] = Bm + (size_t)kr * N + n;
    } else {
      const int rl = 8 * w + (lane >> 3);
      const int c = (lane & 7) ^ ((rl >> 1) & 7);
      int gn = col0 + rl;
      gn = gn < N ? gn : N - 1;
      bptr[it] = Bm + (size_t)gn * Kd + c * 8;
    }
  }
  const size_t bstep = NN ? (size_t)BK * N : (size_t)BK;

  auto issue = [&](int kt, char* sa, char* sb) {
#pragma unroll
    for (int it = 0; it < LPW; ++it) load_lds_16B(aptr[it] + (size_t)kt * BK, sa + (wave + NW * it) * 1024);
#pragma unroll
    for (int it = 0; it < LPW; ++it) load_lds_16B(bptr[it] + (size_t)kt * bstep, sb + (wave + NW * it) * 1024);
  };

  // ---- fragment addressing
  const int l32 = lane & 31, lhi = lane >> 5;
  const int fsw = (l32 >> 1) & 7;
  const int a_row_off = (wm * WM + l32) * 128;
  const int b_row_off = (wn * WN + l32) * 128;                       // NT
  const int L16 = lane & 15, blk = lane >> 4, kq = L16 >> 2;          // NN (transposing reads)
  const int nn_k = 8 * (blk >> 1) + kq;
  const int nn_n = wn * WN + 16 * (blk & 1) + 4 * (L16 & 3);

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  auto compute = [&](const char* sa, const char* sb, int ksteps) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      if (ks < ksteps) {
        bf16x8 af[FM], bfr[FN];
        const int coff = ((2 * ks + lhi) ^ fsw) << 4;
#pragma unroll
        for (int i = 0; i < FM; ++i) af[i] = *(const bf16x8*)(sa + a_row_off + i * 32 * 128 + coff);
#pragma unroll
        for (int j = 0; j < FN; ++j) {
          if (NN) {
            const int k = 16 * ks + nn_k;
            const int n = nn_n + 32 * j;
            const int phys = (n >> 3) ^ (kq << 2);
            const char* p0 = sb + k * 512 + phys * 16 + (n & 7) * 2;
            bfr[j] = lds_read_tr_pair(p0, p0 + 4 * 512);
          } else {
            bfr[j] = *(const bf16x8*)(sb + b_row_off + j * 32 * 128 + coff);
          }
        }
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
          for (int j = 0; j < FN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
      }
    }
  };

  // ---- main contraction loop, double-buffered
  const int KT = Kd / BK;
  issue(0, sA0, sB0);
  for (int kt = 0; kt < KT; kt += 2) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (kt + 1 < KT) issue(kt + 1, sA1, sB1);
    compute(sA0, sB0, 4);
    if (kt + 1 >= KT) break;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (kt + 2 < KT) issue(kt + 2, sA0, sB0);
    compute(sA1, sB1, 4);
  }

  // ---- LoRA extension: tasks whose rows intersect this tile
  const int rend = (row0 + BM) < M ? (row0 + BM) : M;
  for (int k = 0; k < st.K; ++k) {
    const int lo = st.off[k] > row0 ? st.off[k] : row0;
    const int hi = st.off[k + 1] < rend ? st.off[k + 1] : rend;
    if (lo >= hi) continue;
    const int r = st.rank[k];
    const bf16* Rk = static_cast<const bf16*>(R.p[k]);
    for (int q0 = 0; q0 < r; q0 += BK) {
      __syncthreads();
      for (int e = tid; e < 2048; e += NT) {
        const int rl = e >> 3, c = e & 7;
        const int row = row0 + rl, q = q0 + c * 8;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (row >= lo && row < hi && q < ldz) v = *(const uint4*)(L + (size_t)row * ldz + q);
        *(uint4*)(sA0 + rl * 128 + ((c ^ ((rl >> 1) & 7)) << 4)) = v;
      }
      for (int e = tid; e < 2048; e += NT) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (NN) {
          const int kr = e >> 5, c = e & 31;
          const int q = q0 + kr, n = col0 + c * 8;
          if (q < r && n < N) v = *(const uint4*)(Rk + (size_t)q * N + n);
          *(uint4*)(sB0 + kr * 512 + ((c ^ ((kr & 3) << 2)) << 4)) = v;
        } else {
          const int rl = e >> 3, c = e & 7;
          const int n = col0 + rl, q = q0 + c * 8;
          if (n < N && q < r) v = *(const uint4*)(Rk + (size_t)n * r + q);
          *(uint4*)(sB0 + rl * 128 + ((c ^ ((rl >> 1) & 7)) << 4)) = v;
        }
      }
      __syncthreads();
      const int left = (r - q0 + 15) / 16;
      compute(sA0, sB0, left < 4 ? left : 4);
    }
  }

  // ---- store: lane holds, per 32x32 block, column m = l32 and rows n = 8g + 4*lhi + 0..3
#pragma unroll
  for (int i = 0; i < FM; ++i) {
    const int m = row0 + wm * WM + 32 * i + l32;
    if (m < M) {
#pragma unroll
      for (int j = 0; j < FN; ++j) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int n = col0 + wn * WN + 32 * j + 8 * g + 4 * lhi;
          if (n < N) {
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = static_cast<bf16>(acc[i][j][4 * g + e]);
            *(bf16x4*)(C + (size_t)m * N + n) = o;
          }
        }
      }
    }
  }
}

// ---- optional per-launch timing of this kernel with HIP events on the launch stream ----
struct GemmProfile {
  bool on = false;
  std::vector<hipEvent_t> start, stop;
  std::vector<double> flops;
  size_t used = 0;
};
GemmProfile g_prof;
std::mutex g_prof_mu;
constexpr size_t kMaxProfiled = 4096;

}  // namespace

int gemm_profile_enable(int enable) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  const int old = g_prof.on ? 1 : 0;
  g_prof.on = enable != 0;
  return old;
}

// Waits for every recorded launch, sums durations and flops, then forgets them.
hipError_t gemm_profile_read(double* ms_total, double* flops_total, int* launches) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  double ms = 0, fl = 0;
  for (size_t i = 0; i < g_prof.used; ++i) {
    hipError_t e = hipEventSynchronize(g_prof.stop[i]);
    if (e != hipSuccess) return e;
    float t = 0.f;
    e = hipEventElapsedTime(&t, g_prof.start[i], g_prof.stop[i]);
    if (e != hipSuccess) return e;
    ms += t;
    fl += g_prof.flops[i];
  }
  if (ms_total) *ms_total = ms;
  if (flops_total) *flops_total = fl;
  if (launches) *launches = (int)g_prof.used;
  g_prof.used = 0;
  return hipSuccess;
}

bool gemm_mfma_ok(int M, int N, int Kd) { return M >= 1 && (N % 64) == 0 && (Kd % 64) == 0 && N >= 64 && Kd >= 64; }

// C[M,N] = A[M,Kd] * (nn ? Bm[Kd,N] : Bm[N,Kd]^T) + rows_k( L[rows_k, :r_k] * (nn ? R_k[r_k,N] : R_k[N,r_k]^T) )
hipError_t gemm_mfma(const bf16* A, const bf16* Bm, bf16* C, int M, int N, int Kd, bool nn, const bf16* L, int ldz,
                     const SegTable& st, const PtrTable& R, hipStream_t stream) {
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  const dim3 grid(tiles_m * tiles_n);
  int slot = -1;
  {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if (g_prof.on && g_prof.used < kMaxProfiled) {
      if (g_prof.used == g_prof.start.size()) {
        hipEvent_t a, b;
        if (hipEventCreate(&a) == hipSuccess && hipEventCreate(&b) == hipSuccess) {
          g_prof.start.push_back(a);
          g_prof.stop.push_back(b);
          g_prof.flops.push_back(0.0);
        }
      }
      if (g_prof.used < g_prof.start.size()) {
        slot = (int)g_prof.used++;
        double f = 2.0 * M * (double)N * Kd;
        for (int k = 0; k < st.K; ++k) f += 2.0 * (st.off[k + 1] - st.off[k]) * (double)st.rank[k] * N;
        g_prof.flops[slot] = f;
        (void)hipEventRecord(g_prof.start[slot], stream);
      }
    }
  }
  if (nn)
    hipLaunchKernelGGL((k_gemm_mfma<2, 4, true>), grid, dim3(512), 0, stream, A, Bm, C, M, N, Kd, L, ldz, st, R,
                       tiles_m, tiles_n);
  else
    hipLaunchKernelGGL((k_gemm_mfma<2, 4, false>), grid, dim3(512), 0, stream, A, Bm, C, M, N, Kd, L, ldz, st, R,
                       tiles_m, tiles_n);
  const hipError_t err = hipGetLastError();
  if (slot >= 0) (void)hipEventRecord(g_prof.stop[slot], stream);
  return err;
}

}  // namespace mlora
