// 8-bit frozen base weight (the single-GPU setup of section 4.1 keeps the pre-trained weights
// in 8 bits): column-wise absmax code of W [h, d],
//     c_j = max_i |W[i, j]| / 127,   Wq[i, j] = rint(W[i, j] / c_j),   W^[i, j] = Wq[i, j] c_j.
// Two streaming kernels: the coder (run once when a model is loaded) and the decoder that the
// w8 entry points run in front of the base products (1 byte read and one element written per
// weight; ~1 % of the product it feeds, which is bound by the matrix pipes and reads W through
// the L2 many times -- decoding inside the product would move the conversion into its inner
// loop and save none of its time).
#include "mlora_common.h"

namespace mlora {
namespace {

// One block: 64 columns of W, all h rows; 4 groups of 64 threads walk the rows, a row segment
// of 64 elements is one 128-byte (bf16) or 256-byte (fp32) piece.  The code is an integer
// decided by floating point: the maximum is exact, both divisions are IEEE fp32 divisions and
// rintf rounds halves to even, so the result is defined bit for bit.
template <typename T>
__global__ __launch_bounds__(256) void k_w8_quantize(const T* __restrict__ W, int h, int d,
                                                     int8_t* __restrict__ Wq, float* __restrict__ c) {
  __shared__ float s_max[4][64];
  const int cl = threadIdx.x & 63, rg = threadIdx.x >> 6;
  const int col = blockIdx.x * 64 + cl;
  float amax = 0.f;
  if (col < d) {
    for (int i = rg; i < h; i += 4) amax = fmaxf(amax, fabsf(to_f32(W[(size_t)i * d + col])));
  }
  s_max[rg][cl] = amax;
  __syncthreads();
  amax = fmaxf(fmaxf(s_max[0][cl], s_max[1][cl]), fmaxf(s_max[2][cl], s_max[3][cl]));
  const float cj = amax / 127.0f;
  if (col >= d) return;
  if (rg == 0) c[col] = cj;
  for (int i = rg; i < h; i += 4) {
    float q = 0.f;
    if (cj > 0.f) {
      q = rintf(to_f32(W[(size_t)i * d + col]) / cj);
      q = fminf(fmaxf(q, -127.f), 127.f);
    }
    Wq[(size_t)i * d + col] = (int8_t)(int)q;
  }
}

typedef int8_t i8x16 __attribute__((ext_vector_type(16)));
typedef float f32x4v __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8v __attribute__((ext_vector_type(8)));

// W^ = fl32(Wq * c_j), rounded to the storage type.
// Vector form (d a multiple of 16, 16-byte aligned buffers): a lane owns 16 consecutive columns,
// keeps their scales in registers and walks down the rows (blockIdx.y, stride gridDim.y); a wave
// reads 1 KiB and writes 2 or 4 KiB of contiguous memory per row.
template <typename T>
__global__ __launch_bounds__(64) void k_w8_dequantize_cols16(const int8_t* __restrict__ Wq, const float* __restrict__ c,
                                                             int h, int d, T* __restrict__ Wh) {
  const int j0 = (blockIdx.x * 64 + threadIdx.x) * 16;
  if (j0 >= d) return;
  float cs[16];
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    const f32x4v cg = *reinterpret_cast<const f32x4v*>(c + j0 + 4 * g);
#pragma unroll
    for (int e = 0; e < 4; ++e) cs[4 * g + e] = cg[e];
  }
#pragma unroll 4
  for (int i = blockIdx.y; i < h; i += gridDim.y) {
    const size_t o = (size_t)i * d + j0;
    const i8x16 q = __builtin_nontemporal_load(reinterpret_cast<const i8x16*>(Wq + o));
    float v[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) v[e] = (float)q[e] * cs[e];
    T* out = Wh + o;
    if constexpr (sizeof(T) == 2) {
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        bf16x8v w;
#pragma unroll
        for (int e = 0; e < 8; ++e) w[e] = from_f32<bf16>(v[8 * g + e]);
        *reinterpret_cast<bf16x8v*>(out + 8 * g) = w;
      }
    } else {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x4v w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = v[4 * g + e];
        *reinterpret_cast<f32x4v*>(out + 4 * g) = w;
      }
    }
  }
}

// Any d, any alignment: one element per thread.
template <typename T>
__global__ __launch_bounds__(256) void k_w8_dequantize_any(const int8_t* __restrict__ Wq, const float* __restrict__ c,
                                                           size_t n, int d, T* __restrict__ Wh) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x; t < n; t += stride)
    Wh[t] = from_f32<T>((float)Wq[t] * c[t % (size_t)d]);
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

hipError_t w8_quantize(const void* W, int dtype, int h, int d, int8_t* Wq, float* c, hipStream_t stream) {
  const dim3 grid((unsigned)((d + 63) / 64)), block(256);
  if (dtype == MLORA_F32)
    hipLaunchKernelGGL(k_w8_quantize<float>, grid, block, 0, stream, (const float*)W, h, d, Wq, c);
  else
    hipLaunchKernelGGL(k_w8_quantize<bf16>, grid, block, 0, stream, (const bf16*)W, h, d, Wq, c);
  return hipGetLastError();
}

hipError_t w8_dequantize(const int8_t* Wq, const float* c, int dtype, int h, int d, void* Wh, hipStream_t stream) {
  const size_t n = (size_t)h * (size_t)d;
  if (d % 16 == 0 && aligned16(Wq) && aligned16(c) && aligned16(Wh)) {
    const int gx = (d / 16 + 63) / 64;
    int gy = (256 * 16 + gx - 1) / gx;          // about 16 waves per CU over the whole grid
    gy = gy < h ? gy : h;
    const dim3 grid((unsigned)gx, (unsigned)gy), block(64);
    if (dtype == MLORA_F32)
      hipLaunchKernelGGL(k_w8_dequantize_cols16<float>, grid, block, 0, stream, Wq, c, h, d, (float*)Wh);
    else
      hipLaunchKernelGGL(k_w8_dequantize_cols16<bf16>, grid, block, 0, stream, Wq, c, h, d, (bf16*)Wh);
    return hipGetLastError();
  }
  size_t blocks = (n + 255) / 256;
  if (blocks > 256 * 64) blocks = 256 * 64;   // grid-stride beyond 64 blocks per CU
  const dim3 grid((unsigned)blocks), block(256);
  if (dtype == MLORA_F32)
    hipLaunchKernelGGL(k_w8_dequantize_any<float>, grid, block, 0, stream, Wq, c, n, d, (float*)Wh);
  else
    hipLaunchKernelGGL(k_w8_dequantize_any<bf16>, grid, block, 0, stream, Wq, c, n, d, (bf16*)Wh);
  return hipGetLastError();
}

}  // namespace mlora
