// Host side of the bf16 MFMA base product with LoRA contraction steps: launch geometry.
// The kernel itself is in gemm_mfma_kernel.h.
//
//   forward  (Eq. "forward"):      Y  = X W   + Z B_k      (W is [h,d], contraction index = rows of W)
//   backward (Eq. "grad_output"):  dX = dY W^T + G A_k^T   (W is [h,d], contraction index = columns of W)
//
// where Z = s_k x_k A_k and G = s_k dy_k B_k^T are the [T, ldz] low-rank intermediates.  The
// base product is launched once over all tasks' rows; the output tile is written once with the
// LoRA term already in it (no full-size intermediate for the LoRA part of dX exists).
#include "gemm_mfma_kernel.h"
#include "mlora_common.h"

namespace mlora {
namespace {

constexpr int BM = gemmk::BM, BN = gemmk::BN;

}  // namespace

bool gemm_mfma_ok(int M, int N, int Kd) { return M >= 1 && (N % 64) == 0 && (Kd % 64) == 0 && N >= 64 && Kd >= 64; }

namespace {

template <int NSEG>
double algorithmic_flops(const gemmk::GemmArgs<NSEG>& a) {
  double f = 0;
  for (int g = 0; g < NSEG; ++g) {
    f += 2.0 * a.M * (double)a.N * a.Kd[g];
    for (int k = 0; k < a.K; ++k) f += 2.0 * (a.off[k + 1] - a.off[k]) * (double)a.rank[g][k] * a.N;
  }
  return f;
}

template <bool NN, int NSEG>
hipError_t launch(const gemmk::GemmArgs<NSEG>& a, hipStream_t stream) {
  const dim3 grid(a.tiles_m * a.tiles_n);
  const int slot = profile_begin(kProfileGemm, algorithmic_flops(a), stream);
  hipLaunchKernelGGL((gemmk::k_gemm_mfma<2, 4, NN, NSEG>), grid, dim3(512), 0, stream, a);
  const hipError_t err = hipGetLastError();
  profile_end(slot, stream);
  return err;
}

template <int NSEG>
void fill_common(gemmk::GemmArgs<NSEG>* a, bf16* C, int M, int N, const SegTable& st) {
  a->C = C;
  a->M = M;
  a->N = N;
  a->tiles_n = (N + BN - 1) / BN;
  a->K = st.K;
  for (int k = 0; k <= kMaxK; ++k) a->off[k] = st.off[k];
  // rows of the virtual axis the grid tiles: every row range of the call (before the first
  // task, each task, after the last task) rounded up to whole 32-row MFMA fragments
  long long mv = 0;
  int prev = 0;
  for (int r = 0; r < st.K + 2; ++r) {
    const int b1 = r <= st.K ? st.off[r] : M;
    mv += (b1 - prev + 31) / 32 * 32;
    prev = b1;
  }
  a->tiles_m = (int)((mv + BM - 1) / BM);
}

template <int NSEG>
hipError_t launch_sum(const GemmOperands* ops, bf16* C, int M, int N, const SegTable& st, hipStream_t stream) {
  gemmk::GemmArgs<NSEG> a;
  fill_common(&a, C, M, N, st);
  for (int g = 0; g < NSEG; ++g) {
    a.A[g] = ops[g].A;
    a.Bm[g] = ops[g].Bm;
    a.L[g] = ops[g].L;
    a.Kd[g] = ops[g].Kd;
    a.ldz[g] = ops[g].ldz;
    for (int k = 0; k < kMaxK; ++k) a.rank[g][k] = (unsigned char)(k < st.K ? ops[g].rank[k] : 0);
    a.R[g] = *ops[g].R;
  }
  return launch<false, NSEG>(a, stream);
}

}  // namespace

// C[M,N] = A[M,Kd] * (nn ? Bm[Kd,N] : Bm[N,Kd]^T) + rows_k( L[rows_k, :r_k] * (nn ? R_k[r_k,N] : R_k[N,r_k]^T) )
hipError_t gemm_mfma(const bf16* A, const bf16* Bm, bf16* C, int M, int N, int Kd, bool nn, const bf16* L, int ldz,
                     const SegTable& st, const PtrTable& R, hipStream_t stream) {
  gemmk::GemmArgs<1> a;
  fill_common(&a, C, M, N, st);
  a.A[0] = A;
  a.Bm[0] = Bm;
  a.L[0] = L;
  a.Kd[0] = Kd;
  a.ldz[0] = ldz;
  for (int k = 0; k < kMaxK; ++k) a.rank[0][k] = (unsigned char)(k < st.K ? st.rank[k] : 0);
  a.R[0] = R;
  return nn ? launch<true, 1>(a, stream) : launch<false, 1>(a, stream);
}

// C[M,N] = sum_g ( A_g[M,Kd_g] * Bm_g[N,Kd_g]^T + rows_k( L_g[rows_k, :r_gk] * R_gk[N,r_gk]^T ) ), 1 <= n <= 4
hipError_t gemm_mfma_sum_nt(int n, const GemmOperands* ops, bf16* C, int M, int N, const SegTable& st,
                            hipStream_t stream) {
  switch (n) {
    case 1: return launch_sum<1>(ops, C, M, N, st, stream);
    case 2: return launch_sum<2>(ops, C, M, N, st, stream);
    case 3: return launch_sum<3>(ops, C, M, N, st, stream);
    case 4: return launch_sum<4>(ops, C, M, N, st, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace mlora
