// Shared declarations of the HIP side of libmlora (gfx950 only).
// Notation follows section 3.3.1 of the mLoRA paper: X [T,h], W [h,d], A_k [h,r_k],
// B_k [r_k,d]; task k owns rows [off[k], off[k+1]) of X, Y, dY and dX.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/mlora.h"

namespace mlora {

constexpr int kMaxK = MLORA_MAX_ADAPTERS;
constexpr int kMaxRank = MLORA_MAX_RANK;

typedef __bf16 bf16;

// Split positions, ranks and scalings of one call, passed to kernels by value
// (they land in the kernel-argument segment and are read with scalar loads).
struct SegTable {
  int K;
  int off[kMaxK + 1];
  int rank[kMaxK];
  float s[kMaxK];
};

struct PtrTable {
  const void* p[kMaxK];
};

struct OutTable {
  float* p[kMaxK];
};

// Adapter that owns `row`, or -1 for rows outside every segment.
__device__ __forceinline__ int find_segment(const SegTable& st, int row) {
  int k = -1;
  for (int i = 0; i < st.K; ++i) {
    if (row >= st.off[i] && row < st.off[i + 1]) k = i;
  }
  return k;
}

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return static_cast<float>(v); }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
// fp32 -> bf16, round to nearest even, NaN/Inf propagate
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return static_cast<bf16>(v); }

// Row stride (in elements) of the saved intermediate Z and of G: the largest rank
// rounded up to a multiple of 16, so that rank-padded MFMA steps read zeros.
inline int lowrank_ld(const mlora_problem* p) {
  int rmax = 0;
  for (int k = 0; k < p->K; ++k) rmax = p->ranks[k] > rmax ? p->ranks[k] : rmax;
  return (rmax + 15) / 16 * 16;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Everything the launchers need, filled once per call from the validated problem.
struct CallCtx {
  int T, h, d, K, ldz;
  int dtype;
  SegTable st;
  PtrTable A, B;
  const void* W;
  hipStream_t stream;
};

// ---- launchers (each returns a hipError_t; all work goes to c.stream) ----
// generic_kernels.hip : any shape, fp32 or bf16 storage, plain VALU arithmetic
hipError_t generic_Z(const CallCtx& c, const void* X, void* Z);                        // Z = s x A
hipError_t generic_G(const CallCtx& c, const void* dY, void* G);                       // G = s dy B^T
hipError_t generic_gemm_fwd(const CallCtx& c, const void* X, void* Y, const void* Z);  // Y = X W + Z B
// dX (+)= dY W^T + G A^T; with `accumulate` the sum is added to what dX holds (in its storage type)
hipError_t generic_gemm_bwd(const CallCtx& c, const void* dY, void* dX, const void* G, int accumulate = 0);
hipError_t generic_dB(const CallCtx& c, const void* Z, const void* dY, const OutTable& dB, int accumulate);
hipError_t generic_dA(const CallCtx& c, const void* X, const void* G, const OutTable& dA, int accumulate);

// gemm_mfma.hip : bf16 MFMA GEMM with the LoRA term as extra contraction steps
bool gemm_mfma_ok(int M, int N, int Kd);
hipError_t gemm_mfma(const bf16* A, const bf16* Bm, bf16* C, int M, int N, int Kd, bool nn, const bf16* L, int ldz,
                     const SegTable& st, const PtrTable& R, hipStream_t stream);

// One operand pair of a summed contraction (the input gradient of projections that share X):
// A [M, Kd], Bm [N, Kd], L [M, ldz] with R_k [N, rank[k]].
struct GemmOperands {
  const bf16* A;
  const bf16* Bm;
  const bf16* L;
  int Kd, ldz;
  const int* rank;     // K entries
  const PtrTable* R;
};
hipError_t gemm_mfma_sum_nt(int n, const GemmOperands* ops, bf16* C, int M, int N, const SegTable& st,
                            hipStream_t stream);

// profile.hip : optional HIP-event timing of the MFMA kernels' launches, by kind
enum { kProfileGemm = 0, kProfileRows = 1, kProfileGrad = 2, kProfileKinds = 3 };
int profile_enable(int enable);
int profile_begin(int kind, double units, hipStream_t stream);
void profile_end(int slot, hipStream_t stream);
hipError_t profile_read(double* ms, double* units, int* launches);

// w8_kernels.hip : column-wise absmax code of the frozen weight and its decoder
hipError_t w8_quantize(const void* W, int dtype, int h, int d, int8_t* Wq, float* c, hipStream_t stream);
hipError_t w8_dequantize(const int8_t* Wq, const float* c, int dtype, int h, int d, void* Wh, hipStream_t stream);

// lowrank_mfma.hip : bf16 MFMA kernels for Z, G (row-local) and dA_k, dB_k (reduce over a task's tokens)
hipError_t lowrank_rows_mfma(const CallCtx& c, const bf16* In, int inner, bf16* Out, const PtrTable& M, bool a_major);
// `partial`: grad_partial_bytes(c.st, wide) bytes of scratch for calls whose tasks x column blocks
// do not fill the chip (the tokens of a task are then split over blocks); NULL = never split.
int grad_splits(const SegTable& st, int wide);
size_t grad_partial_bytes(const SegTable& st, int wide);
hipError_t grad_mfma(const CallCtx& c, const bf16* Big, int wide, const bf16* Small, const OutTable& out,
                     int accumulate, bool wide_first, float* partial);

// One projection of a group that shares its input, for the two shared-input kernels:
// rows: Z_p = s_pk x_k A_pk (M = A_pk, output rows_out [T, ldz]); grad: dA_pk = x_k^T G_p
// (grad_small = G_p [T, ldz], output table grad_out).
struct LowrankGroupItem {
  int ldz;
  const int* rank;      // K entries
  const float* s;       // K entries
  const PtrTable* M;
  bf16* rows_out;
  const bf16* grad_small;
  const OutTable* grad_out;
};
bool lowrank_group_ok(int np, int max_ldz);
hipError_t lowrank_rows_mfma_group(int np, const LowrankGroupItem* items, const SegTable& st, const bf16* X, int h,
                                   hipStream_t stream);
hipError_t grad_mfma_group(int np, const LowrankGroupItem* items, const SegTable& st, const bf16* X, int h, int T,
                           int accumulate, hipStream_t stream);

}  // namespace mlora
