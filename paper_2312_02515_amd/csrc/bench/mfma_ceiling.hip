// Hardware characterisation for the base-product kernel (not a product kernel, not linked into
// libmlora): what one MI355X sustains on the inner loop of a 256 x 256 x 64 bf16 GEMM tile when
// the loop's ingredients are added one at a time.  256 blocks of 8 waves (one per CU), wave tile
// 128 x 64, fp32 accumulators in AccVGPRs, operand values drawn like the benchmark's
// (activations ~ N(0,1), weights ~ N(0, 0.02^2)): the board runs at its power cap under matrix
// work, and what it sustains there depends on the data and on everything else that draws power.
//
//   level 0  MFMAs on fragments held in registers
//   level 1  + every fragment re-read from LDS as the GEMM does (ds_read_b128, one MFMA step ahead)
//   level 2  + the tile's 64 KiB staged by direct global->LDS loads from an L2-resident matrix
//   level 3  + the loads follow the GEMM's addresses: an 8 x 4 patch of tiles per XCD over
//            A [32768, ld] and W [1024, ld], 128 B further along every row per tile
//
// Every address is in bounds by construction, every barrier is reached by all waves of a block,
// and nothing is read back from the staged data: the figures are rates, not results.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <type_traits>
#include <vector>

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
#define CK(x)                                                                         \
  do {                                                                                \
    hipError_t e_ = (x);                                                              \
    if (e_ != hipSuccess) {                                                           \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);           \
      exit(1);                                                                        \
    }                                                                                 \
  } while (0)

__device__ __forceinline__ void load_lds_16B(const void* g, char* lds_wave_base) {
  const unsigned lds = (unsigned)(size_t)(__attribute__((address_space(3))) char*)lds_wave_base;
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds) : "memory", "m0");
}

// SHAPE 0: v_mfma_f32_32x32x16_bf16 (4 x 2 fragments, 4 k-steps), 1: v_mfma_f32_16x16x32_bf16
// (8 x 4 fragments, 2 k-steps); 64 or 32 ... both 8.4 MFLOP per wave-tile step of 64.
template <int SHAPE, int LEVEL>
__global__ __launch_bounds__(512) void k_ceiling(const bf16* __restrict__ src, const char* __restrict__ A,
                                                 const char* __restrict__ W, float* __restrict__ out, int iters,
                                                 int ld, int kt) {
  constexpr int MF = SHAPE == 0 ? 32 : 16;
  constexpr int FM = 128 / MF, FN = 64 / MF;
  constexpr int KSTEPS = SHAPE == 0 ? 4 : 2;
  constexpr int NMF = FM * FN * KSTEPS;     // MFMAs per wave per tile
  constexpr int NLD = 8;                    // 1 KiB loads per wave per tile (64 KiB per block)
  __shared__ __attribute__((aligned(1024))) char lds[131072];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  for (int i = tid; i < 65536 / 16; i += 512) reinterpret_cast<uint4*>(lds)[i] = reinterpret_cast<const uint4*>(src)[i];
  __syncthreads();
  {
    float keep = 0.f;   // makes the compiler place the accumulators in AccVGPRs
    asm volatile("" : "+a"(keep));
  }
  typedef typename std::conditional<SHAPE == 0, f32x16, f32x4>::type accT;
  constexpr int NE = SHAPE == 0 ? 16 : 4;
  accT acc[FM][FN];
  for (int i = 0; i < FM; ++i)
    for (int j = 0; j < FN; ++j)
      for (int e = 0; e < NE; ++e) acc[i][j][e] = 0.f;
  bf16x8 af[FM], bfr[FN];
  const char* abase = lds + lane * 16 + (wave % 4) * (FM * 1024);          // activations: first 32 KiB
  const char* bbase = lds + 32768 + lane * 16 + (wave % 4) * (FN * 1024);  // weights: next 32 KiB
  for (int i = 0; i < FM; ++i) af[i] = *(const bf16x8*)(abase + i * 1024);
  for (int j = 0; j < FN; ++j) bfr[j] = *(const bf16x8*)(bbase + j * 1024);
  char* land = lds + 65536 + wave * NLD * 1024;   // where this wave's loads land (never read)
  const char* gsrc[NLD];
  const int b = blockIdx.x, x = b % 8, l = b / 8, pm = l % 8, pn = l / 8;
  for (int i = 0; i < NLD; ++i) {
    const int piece = wave + 8 * (i % 4);          // 1 KiB piece of the operand tile: 8 rows x 128 B
    const int row = 8 * piece + lane / 8, c = lane % 8;
    if (LEVEL == 3)
      gsrc[i] = i < 4 ? A + (size_t)((x * 8 + pm) * 256 + row) * ld + c * 16 : W + (size_t)(pn * 256 + row) * ld + c * 16;
    else
      gsrc[i] = (i < 4 ? A : W) + (size_t)row * ld + c * 16;
  }
  const size_t a_pass = LEVEL == 3 ? (size_t)64 * 256 * ld : 0;   // next pass over K: the other 64 row tiles of A
  unsigned koff = 0;
  int kcount = 0, pass = 0, foff = 0;
  for (int it = 0; it < iters; ++it) {
    int ldi = 0;
#pragma unroll
    for (int m = 0; m < NMF; ++m) {
      const int ks = m / (FM * FN), r = m % (FM * FN), i = r / FN, j = r % FN;
      if constexpr (SHAPE == 0)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
      else
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
      if (LEVEL >= 1 && r < FM + FN) {   // next k-step's fragments, one read behind each MFMA
        const int o = ((foff + (ks + 1) * 8192) & 16383) & ~1023;
        if (r < FN) bfr[r] = *(const bf16x8*)(bbase + (o & 8191) + r * 1024);
        else af[r - FN] = *(const bf16x8*)(abase + (o & 8191) + (r - FN) * 1024);
      }
      if (LEVEL >= 2 && m >= NMF - NLD) {   // next tile's loads behind the last MFMAs of this one
        const size_t po = ldi < 4 ? (size_t)(pass & 1) * a_pass : 0;
        load_lds_16B(gsrc[ldi] + koff + po, land + ldi * 1024);
        ++ldi;
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    foff = (foff + 8192) & 16383;
    koff += 128;
    if (++kcount == kt) { kcount = 0; koff = 0; ++pass; }
    if (LEVEL >= 2) {
      asm volatile("s_waitcnt vmcnt(8)" ::: "memory");   // the previous tile's loads have landed
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();                      // one barrier per tile, as in the GEMM
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  float s = (float)(unsigned char)land[lane];
  for (int i = 0; i < FM; ++i)
    for (int j = 0; j < FN; ++j)
      for (int e = 0; e < NE; ++e) s += acc[i][j][e];
  out[blockIdx.x * 512 + tid] = s;
}

typedef void (*kfn)(const bf16*, const char*, const char*, float*, int, int, int);
struct Variant { const char* mfma; const char* level; kfn f; int ld, kt; };

int main(int argc, char** argv) {
  const int iters = argc > 1 ? atoi(argv[1]) : 8000;   // tiles per block
  const int reps = argc > 2 ? atoi(argv[2]) : 4;       // the first repetition is a warm-up
  std::vector<bf16> h(32768);
  unsigned x = 12345u;
  auto rnd = [&]() { x = x * 1664525u + 1013904223u; return (x >> 8) * (1.0f / 16777216.0f); };
  for (int i = 0; i < 32768; ++i) {
    const float u1 = rnd() + 1e-7f, u2 = rnd();
    const float n = sqrtf(-2.f * logf(u1)) * cosf(6.2831853f * u2);
    h[i] = (bf16)(i < 16384 ? n : 0.02f * n);
  }
  bf16* src;
  float* out;
  char *A, *W;
  const size_t LD = 10240;   // bytes per row: 5120 bf16
  const size_t abytes = (size_t)32768 * LD + 65536, wbytes = (size_t)1024 * LD + 65536;
  CK(hipMalloc(&src, 65536));
  CK(hipMalloc(&out, 256 * 512 * 4));
  CK(hipMalloc(&A, abytes));
  CK(hipMalloc(&W, wbytes));
  CK(hipMemcpy(src, h.data(), 65536, hipMemcpyHostToDevice));
  CK(hipMemset(A, 0x3c, abytes));
  CK(hipMemset(W, 0x3c, wbytes));
  const std::vector<Variant> vs = {
      {"32x32x16", "0 registers only", k_ceiling<0, 0>, 4096, 16},
      {"32x32x16", "1 + LDS fragment reads", k_ceiling<0, 1>, 4096, 16},
      {"32x32x16", "2 + global->LDS loads, L2-resident", k_ceiling<0, 2>, 4096, 16},
      {"32x32x16", "3 + GEMM addresses (A 32768 x 5120, W 1024 x 5120)", k_ceiling<0, 3>, 10240, 80},
      {"16x16x32", "0 registers only", k_ceiling<1, 0>, 4096, 16},
      {"16x16x32", "1 + LDS fragment reads", k_ceiling<1, 1>, 4096, 16},
      {"16x16x32", "2 + global->LDS loads, L2-resident", k_ceiling<1, 2>, 4096, 16},
      {"16x16x32", "3 + GEMM addresses (A 32768 x 5120, W 1024 x 5120)", k_ceiling<1, 3>, 10240, 80},
  };
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  const double flops = 2.0 * 256 * 256 * 64 * (double)iters * 256;
  std::vector<double> sum(vs.size(), 0);
  for (int r = 0; r < reps; ++r)
    for (size_t i = 0; i < vs.size(); ++i) {
      CK(hipEventRecord(e0));
      hipLaunchKernelGGL(vs[i].f, dim3(256), dim3(512), 0, 0, src, A, W, out, iters, vs[i].ld, vs[i].kt);
      CK(hipGetLastError());
      CK(hipEventRecord(e1));
      CK(hipEventSynchronize(e1));
      float ms;
      CK(hipEventElapsedTime(&ms, e0, e1));
      if (r > 0) sum[i] += flops / ms / 1e9;
      printf("rep %d %s level %s: %.1f TFLOP/s\n", r, vs[i].mfma, vs[i].level, flops / ms / 1e9);
      fflush(stdout);
    }
  printf("| MFMA | inner loop | TFLOP/s | share of 2500 |\n|---|---|---|---|\n");
  for (size_t i = 0; i < vs.size(); ++i) {
    const double tf = sum[i] / (reps - 1);
    printf("| %s | %s | %.0f | %.3f |\n", vs[i].mfma, vs[i].level, tf, tf / 2500.0);
  }
  return 0;
}
