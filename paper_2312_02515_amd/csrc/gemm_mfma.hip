// Host side of the bf16 MFMA base product with LoRA contraction steps: launch geometry and the
// optional per-launch HIP-event timing.  The kernel itself is in gemm_mfma_kernel.h.
//
//   forward  (Eq. "forward"):      Y  = X W   + Z B_k      (W is [h,d], contraction index = rows of W)
//   backward (Eq. "grad_output"):  dX = dY W^T + G A_k^T   (W is [h,d], contraction index = columns of W)
//
// where Z = s_k x_k A_k and G = s_k dy_k B_k^T are the [T, ldz] low-rank intermediates.  The
// base product is launched once over all tasks' rows; the output tile is written once with the
// LoRA term already in it (no full-size intermediate for the LoRA part of dX exists).
#include <mutex>
#include <vector>

#include "gemm_mfma_kernel.h"
#include "mlora_common.h"

namespace mlora {
namespace {

constexpr int BM = gemmk::BM, BN = gemmk::BN;

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
    hipLaunchKernelGGL((gemmk::k_gemm_mfma<2, 4, true, 64>), grid, dim3(512), 0, stream, A, Bm, C, M, N, Kd, L, ldz, st, R,
                       tiles_m, tiles_n);
  else
    hipLaunchKernelGGL((gemmk::k_gemm_mfma<2, 4, false, 64>), grid, dim3(512), 0, stream, A, Bm, C, M, N, Kd, L, ldz, st, R,
                       tiles_m, tiles_n);
  const hipError_t err = hipGetLastError();
  if (slot >= 0) (void)hipEventRecord(g_prof.stop[slot], stream);
  return err;
}

}  // namespace mlora
