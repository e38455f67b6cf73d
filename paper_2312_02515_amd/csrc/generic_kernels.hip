// Generic kernels: correct for every shape, segment layout and rank, in fp32 or
// bf16 storage with fp32 accumulation.  They carry the fp32 mode and every bf16
// problem whose shape the MFMA kernels do not take.  Plain VALU arithmetic.
//
// Steps (section 3.3.1 of the mLoRA paper, with the scaling s_k folded into the
// low-rank intermediates):
//   forward :  Z = s_k x_k A_k            (lowrank_rows)
//              Y = X W + Z B_k            (gemm_lora, B operand row-major [h,d])
//   backward:  G = s_k dy_k B_k^T         (lowrank_rows)
//              dB_k = Z^T dy_k            (grad_B)
//              dX = dY W^T + G A_k^T      (gemm_lora, B operand transposed)
//              dA_k = x_k^T G             (grad_A)
#include "mlora_common.h"

namespace mlora {
namespace {

// out[i, q] = s_k * sum_p In[i, p] * M_k(p, q) for q < r_k, 0 for r_k <= q < ldz;
// rows outside every segment are zero.  M_k(p, q) = M[p * sp + q * sq].
template <typename T>
__global__ void k_lowrank_rows(const T* __restrict__ In, int rows, int inner, T* __restrict__ Out, int ldz,
                               SegTable st, PtrTable M, int mode /*0: A_k [inner,r]; 1: B_k [r,inner]*/) {
  int i = blockIdx.x * blockDim.y + threadIdx.y;
  if (i >= rows) return;
  int k = find_segment(st, i);
  const T* in = In + (size_t)i * inner;
  for (int q = threadIdx.x; q < ldz; q += blockDim.x) {
    float acc = 0.f;
    if (k >= 0 && q < st.rank[k]) {
      const T* m = static_cast<const T*>(M.p[k]);
      int r = st.rank[k];
      if (mode == 0) {
        for (int p = 0; p < inner; ++p) acc += to_f32(in[p]) * to_f32(m[(size_t)p * r + q]);
      } else {
        const T* mq = m + (size_t)q * inner;
        for (int p = 0; p < inner; ++p) acc += to_f32(in[p]) * to_f32(mq[p]);
      }
      acc *= st.s[k];
    }
    Out[(size_t)i * ldz + q] = from_f32<T>(acc);
  }
}

// C[M,N] (+)= A[M,Kd] * op(Bm) + L[M,:r_k] * R_k   (64x64 tile, 16x16 threads, 4x4 each)
//   TRANSB = false: Bm is [Kd, N] row-major;  R_k(q, j) = Rk[q * N + j]   (forward:  W, B_k)
//   TRANSB = true : Bm is [N, Kd] row-major;  R_k(q, j) = Rk[j * r + q]   (backward: W, A_k)
template <typename T, bool TRANSB>
__global__ void k_gemm_lora(const T* __restrict__ A, const T* __restrict__ Bm, T* __restrict__ C, int M, int N,
                            int Kd, const T* __restrict__ L, int ldz, SegTable st, PtrTable R, int accumulate) {
  constexpr int TS = 64, BK = 16;
  __shared__ float As[BK][TS + 1];
  __shared__ float Bs[BK][TS + 1];
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  const int row0 = blockIdx.x * TS, col0 = blockIdx.y * TS;
  float acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = 0.f;

  for (int k0 = 0; k0 < Kd; k0 += BK) {
    // A tile: 64 rows x 16 k ; 1024 elements / 256 threads
    for (int e = threadIdx.x; e < TS * BK; e += 256) {
      int r = e / BK, kk = e % BK;
      int gr = row0 + r, gk = k0 + kk;
      As[kk][r] = (gr < M && gk < Kd) ? to_f32(A[(size_t)gr * Kd + gk]) : 0.f;
    }
    for (int e = threadIdx.x; e < TS * BK; e += 256) {
      int kk, c;
      if (TRANSB) { c = e / BK; kk = e % BK; } else { kk = e / TS; c = e % TS; }
      int gc = col0 + c, gk = k0 + kk;
      float v = 0.f;
      if (gc < N && gk < Kd) v = TRANSB ? to_f32(Bm[(size_t)gc * Kd + gk]) : to_f32(Bm[(size_t)gk * N + gc]);
      Bs[kk][c] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) { a[u] = As[kk][ty * 4 + u]; b[u] = Bs[kk][tx * 4 + u]; }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[u][v] += a[u] * b[v];
    }
    __syncthreads();
  }

  for (int u = 0; u < 4; ++u) {
    int gr = row0 + ty * 4 + u;
    if (gr >= M) continue;
    int k = find_segment(st, gr);
    int r = k >= 0 ? st.rank[k] : 0;
    const T* Rk = k >= 0 ? static_cast<const T*>(R.p[k]) : nullptr;
    for (int v = 0; v < 4; ++v) {
      int gc = col0 + tx * 4 + v;
      if (gc >= N) continue;
      float lo = 0.f;
      for (int q = 0; q < r; ++q) {
        float rv = TRANSB ? to_f32(Rk[(size_t)gc * r + q]) : to_f32(Rk[(size_t)q * N + gc]);
        lo += to_f32(L[(size_t)gr * ldz + q]) * rv;
      }
      T* dst = C + (size_t)gr * N + gc;
      *dst = from_f32<T>(acc[u][v] + lo + (accumulate ? to_f32(*dst) : 0.f));
    }
  }
}

// dB_k[q, j] (+)= sum_{i in seg k} Z[i, q] * dY[i, j]      grid (ceil(d/256), rmax, K)
template <typename T>
__global__ void k_grad_B(const T* __restrict__ Z, int ldz, const T* __restrict__ dY, int d, SegTable st,
                         OutTable dB, int accumulate) {
  int k = blockIdx.z, q = blockIdx.y;
  int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= st.rank[k] || j >= d) return;
  float acc = 0.f;
  for (int i = st.off[k]; i < st.off[k + 1]; ++i) acc += to_f32(Z[(size_t)i * ldz + q]) * to_f32(dY[(size_t)i * d + j]);
  float* out = dB.p[k] + (size_t)q * d + j;
  *out = accumulate ? *out + acc : acc;
}

// dA_k[p, q] (+)= sum_{i in seg k} X[i, p] * G[i, q]       grid (ceil(h/256), rmax, K)
template <typename T>
__global__ void k_grad_A(const T* __restrict__ X, int h, const T* __restrict__ G, int ldz, SegTable st,
                         OutTable dA, int accumulate) {
  int k = blockIdx.z, q = blockIdx.y;
  int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= st.rank[k] || p >= h) return;
  float acc = 0.f;
  for (int i = st.off[k]; i < st.off[k + 1]; ++i) acc += to_f32(X[(size_t)i * h + p]) * to_f32(G[(size_t)i * ldz + q]);
  float* out = dA.p[k] + (size_t)p * st.rank[k] + q;
  *out = accumulate ? *out + acc : acc;
}

template <typename T>
hipError_t lowrank_t(const CallCtx& c, const T* In, int inner, T* Out, const PtrTable& M, int mode) {
  if (c.K > 0 && c.T > 0)
    hipLaunchKernelGGL(k_lowrank_rows<T>, dim3((c.T + 7) / 8), dim3(32, 8), 0, c.stream, In, c.T, inner, Out, c.ldz,
                       c.st, M, mode);
  return hipGetLastError();
}

template <typename T, bool TRANSB>
hipError_t gemm_t(const CallCtx& c, const T* A, T* C, int N, int Kd, const T* L, const PtrTable& R, int accumulate = 0) {
  if (c.T > 0) {
    dim3 grid((c.T + 63) / 64, (N + 63) / 64);
    hipLaunchKernelGGL((k_gemm_lora<T, TRANSB>), grid, dim3(256), 0, c.stream, A, static_cast<const T*>(c.W), C, c.T,
                       N, Kd, L, c.ldz, c.st, R, accumulate);
  }
  return hipGetLastError();
}

int max_rank(const CallCtx& c) {
  int rmax = 0;
  for (int k = 0; k < c.K; ++k) rmax = c.st.rank[k] > rmax ? c.st.rank[k] : rmax;
  return rmax;
}

}  // namespace

#define DISPATCH(expr_f32, expr_bf16) ((c.dtype == MLORA_F32) ? (expr_f32) : (expr_bf16))

hipError_t generic_Z(const CallCtx& c, const void* X, void* Z) {
  return DISPATCH(lowrank_t<float>(c, (const float*)X, c.h, (float*)Z, c.A, 0),
                  lowrank_t<bf16>(c, (const bf16*)X, c.h, (bf16*)Z, c.A, 0));
}

hipError_t generic_G(const CallCtx& c, const void* dY, void* G) {
  return DISPATCH(lowrank_t<float>(c, (const float*)dY, c.d, (float*)G, c.B, 1),
                  lowrank_t<bf16>(c, (const bf16*)dY, c.d, (bf16*)G, c.B, 1));
}

hipError_t generic_gemm_fwd(const CallCtx& c, const void* X, void* Y, const void* Z) {
  return DISPATCH((gemm_t<float, false>(c, (const float*)X, (float*)Y, c.d, c.h, (const float*)Z, c.B)),
                  (gemm_t<bf16, false>(c, (const bf16*)X, (bf16*)Y, c.d, c.h, (const bf16*)Z, c.B)));
}

hipError_t generic_gemm_bwd(const CallCtx& c, const void* dY, void* dX, const void* G, int accumulate) {
  return DISPATCH((gemm_t<float, true>(c, (const float*)dY, (float*)dX, c.h, c.d, (const float*)G, c.A, accumulate)),
                  (gemm_t<bf16, true>(c, (const bf16*)dY, (bf16*)dX, c.h, c.d, (const bf16*)G, c.A, accumulate)));
}

hipError_t generic_dB(const CallCtx& c, const void* Z, const void* dY, const OutTable& dB, int accumulate) {
  if (c.K == 0) return hipSuccess;
  dim3 grid((c.d + 255) / 256, max_rank(c), c.K);
  if (c.dtype == MLORA_F32)
    hipLaunchKernelGGL(k_grad_B<float>, grid, dim3(256), 0, c.stream, (const float*)Z, c.ldz, (const float*)dY, c.d,
                       c.st, dB, accumulate);
  else
    hipLaunchKernelGGL(k_grad_B<bf16>, grid, dim3(256), 0, c.stream, (const bf16*)Z, c.ldz, (const bf16*)dY, c.d,
                       c.st, dB, accumulate);
  return hipGetLastError();
}

hipError_t generic_dA(const CallCtx& c, const void* X, const void* G, const OutTable& dA, int accumulate) {
  if (c.K == 0) return hipSuccess;
  dim3 grid((c.h + 255) / 256, max_rank(c), c.K);
  if (c.dtype == MLORA_F32)
    hipLaunchKernelGGL(k_grad_A<float>, grid, dim3(256), 0, c.stream, (const float*)X, c.h, (const float*)G, c.ldz,
                       c.st, dA, accumulate);
  else
    hipLaunchKernelGGL(k_grad_A<bf16>, grid, dim3(256), 0, c.stream, (const bf16*)X, c.h, (const bf16*)G, c.ldz,
                       c.st, dA, accumulate);
  return hipGetLastError();
}

}  // namespace mlora
