// Hardware characterisation for the base-product kernel (not a product kernel, not linked into
// libmlora): what one MI355X sustains on the inner loop of a 256 x 256 x 64 bf16 GEMM tile when
// the loop's ingredients are added one at a time.  256 blocks of 8 waves (one per CU), wave tile
// 128 x 64, fp32 accumulators in AccVGPRs updated in place, the same sub-step schedule as
// k_gemm_mfma (row fragments double-buffered and read one sub-step ahead, weight fragments
// re-read in place behind their last use, loads behind the MFMAs of the last sub-step, one
// barrier per tile) -- so every register that an MFMA reads was loaded at least 12 MFMAs earlier
// and no level stalls on a dependency the real kernel does not have.
//
//   level 0  MFMAs on fragments held in registers
//   level 1  + every fragment re-read from LDS as the GEMM does (24 ds_read_b128 per wave and tile)
//   level 2  + the tile's 64 KiB staged by direct global->LDS loads from an L2-resident matrix,
//            s_waitcnt vmcnt + one barrier per tile
//   level 3  + the loads follow the GEMM's addresses (an 8 x 4 patch of tiles per XCD over
//            A [rows, 5120] and W [1024, 5120], 128 B further along every row per tile), with A
//            small enough (168 MB) to stay in the 256 MB Infinity Cache from pass to pass
//   level 4  the same with twice the rows of A (336 MB, alternating halves): A streams from HBM.
//            Every XCD walks row strips of its own here, so A leaves HBM at five times the rate of
//            the GEMM, where the XCDs that work on one row group share its strips through the
//            Infinity Cache: the level bounds the effect from above
//   level 5  level 4 with k_gemm_mfma's load order and wait: the weight's loads first, then A's,
//            and the wait in front of the barrier leaves A's four loads in flight -- A has two
//            tiles of lead over its use (the kernel's three A stages), the weight one
//
// Each level runs twice: on operand values drawn like the benchmark's (activations ~ N(0,1),
// weights ~ N(0, 0.02^2)), where the board sits at its power cap, and on all-zero operands,
// where it does not -- the second column shows what the instruction stream and the memory
// system allow, the first what the power cap leaves of it.
//
// Every address is in bounds by construction (checked again on the host before the launches),
// every barrier is reached by all waves of a block, and nothing is read back from the staged
// data: the figures are rates, not results.
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

constexpr int kRowBytes = 10240;            // 5120 bf16 per row
constexpr int kStepsPerPass = 80;           // 80 x 128 B = one row
constexpr int kRowsA = 32768, kRowsW = 1024;

__device__ __forceinline__ void load_lds_16B(const void* g, char* lds_wave_base) {
  const unsigned lds = (unsigned)(size_t)(__attribute__((address_space(3))) char*)lds_wave_base;
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds) : "memory", "m0");
}
__device__ __forceinline__ void mfma16(f32x4& c, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma32(f32x16& c, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}

// Level 0 for the 32 x 32 x 16 shape: 4 x 2 fragments, 4 k-steps = 32 MFMAs per wave and tile.
__global__ __launch_bounds__(512) void k_regs_32x32x16(const bf16* __restrict__ src, float* __restrict__ out, int iters) {
  __shared__ __attribute__((aligned(1024))) char lds[65536];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < 65536 / 16; i += 512) reinterpret_cast<uint4*>(lds)[i] = reinterpret_cast<const uint4*>(src)[i];
  __syncthreads();
  f32x16 acc[4][2];
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 2; ++j)
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  bf16x8 af[4], bfr[2];
  for (int i = 0; i < 4; ++i) af[i] = *(const bf16x8*)(lds + lane * 16 + ((wave % 4) * 4 + i) * 1024);
  for (int j = 0; j < 2; ++j) bfr[j] = *(const bf16x8*)(lds + 32768 + lane * 16 + ((wave % 4) * 2 + j) * 1024);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < 32; ++m) {
      mfma32(acc[(m / 2) % 4][m % 2], bfr[m % 2], af[(m / 2) % 4]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  float s = 0.f;
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 2; ++j)
      for (int e = 0; e < 16; ++e) s += acc[i][j][e];
  out[blockIdx.x * 512 + tid] = s;
}

// Levels 0..5 for the 16 x 16 x 32 shape (8 x 4 fragments, 2 k-steps = 64 MFMAs per wave and tile).
template <int LEVEL>
__global__ __launch_bounds__(512) void k_ceiling(const bf16* __restrict__ src, const char* __restrict__ A,
                                                 const char* __restrict__ W, float* __restrict__ out, int iters) {
  constexpr int FM = 8, FN = 4, HM = 4;
  constexpr int NLD = 8;                    // 1 KiB loads per wave per tile (64 KiB per block)
  __shared__ __attribute__((aligned(1024))) char lds[131072];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  for (int i = tid; i < 65536 / 16; i += 512) reinterpret_cast<uint4*>(lds)[i] = reinterpret_cast<const uint4*>(src)[i];
  __syncthreads();
  f32x4 acc[FM][FN];
  for (int i = 0; i < FM; ++i)
    for (int j = 0; j < FN; ++j)
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;
  // fragment pool: activations in the first 32 KiB (32 pieces of 1 KiB), weights in the next 32 KiB
  const char* apool = lds + lane * 16;
  const char* bpool = lds + 32768 + lane * 16;
  bf16x8 af[2][HM], bfr[FN];
  for (int i = 0; i < HM; ++i) af[0][i] = *(const bf16x8*)(apool + ((wave % 4) * 8 + i) * 1024);
  for (int j = 0; j < FN; ++j) bfr[j] = *(const bf16x8*)(bpool + ((wave % 4) * 8 + j) * 1024);
  if (LEVEL == 0)
    for (int i = 0; i < HM; ++i) af[1][i] = *(const bf16x8*)(apool + ((wave % 4) * 8 + 4 + i) * 1024);
  char* land = lds + 65536 + wave * NLD * 1024;   // where this wave's loads land (never read)

  // per-lane source addresses of the wave's 8 loads (4 pieces of the A tile, 4 of the W tile;
  // a piece is 8 rows x 128 B)
  const char* gsrc[NLD];
  const int b = blockIdx.x, x = b % 8, l = b / 8, pm = l % 8, pn = l / 8;
  for (int i = 0; i < NLD; ++i) {
    const int piece = wave + 8 * (i % 4);
    const int row = 8 * piece + lane / 8, c = lane % 8;
    int arow = row, wrow = row;                                    // level 2: every block the same 256 + 256 rows
    if (LEVEL >= 3) { arow = (x * 8 + pm) * 256 + row; wrow = pn * 256 + row; }
    gsrc[i] = i < 4 ? A + (size_t)arow * kRowBytes + c * 16 : W + (size_t)wrow * kRowBytes + c * 16;
  }
  // level 2 walks 4 KiB of every row (1 MiB per operand: L2-resident); levels 3, 4 the whole row
  constexpr int KT = LEVEL == 2 ? 32 : kStepsPerPass;
  const size_t a_pass = LEVEL >= 4 ? (size_t)64 * 256 * kRowBytes : 0;   // odd passes: the other 16384 rows of A
  unsigned koff = 0;
  int kcount = 0, pass = 0;

  // sub-step S of a tile: 16 MFMAs on (k-half q = S / 2, row half h = S % 2), weight fragment by weight fragment
  auto substep = [&](auto S_, int frag_base) {
    constexpr int S = decltype(S_)::value;
    constexpr int h = S % 2, nh = (S + 1) % 2;
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      const int j = m / HM, i = m % HM;
      mfma16(acc[h * HM + i][j], bfr[j], af[h][i]);
      if (LEVEL >= 1) {
        // the next sub-step's row fragments behind the first four MFMAs; in the second sub-step of
        // a k-half, weight fragment j for the next k-half right behind its last MFMA
        if (m < HM) af[nh][m] = *(const bf16x8*)(apool + ((frag_base + 4 * ((S + 1) % 4) + m) & 31) * 1024);
        if (h == 1 && i == HM - 1) bfr[j] = *(const bf16x8*)(bpool + ((frag_base + 4 * ((S + 1) % 4) + j + 16) & 31) * 1024);
      }
      if (LEVEL >= 2 && S == 3 && m >= HM && i != HM - 1) {
        const int idx = (j - 1) * (HM - 1) + i;
        if (idx < NLD) {
          const int g = LEVEL >= 5 ? (idx + 4) % NLD : idx;   // level 5: the weight's four loads first
          const size_t po = g < 4 ? (size_t)(pass & 1) * a_pass : 0;
          load_lds_16B(gsrc[g] + koff + po, land + g * 1024);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  constexpr std::integral_constant<int, 0> S0{};
  constexpr std::integral_constant<int, 1> S1{};
  constexpr std::integral_constant<int, 2> S2{};
  constexpr std::integral_constant<int, 3> S3{};
  for (int it = 0; it < iters; ++it) {
    const int fb = (wave % 4) * 8 + (it & 1) * 2;
    substep(S0, fb);
    substep(S1, fb);
    substep(S2, fb);
    if (LEVEL >= 2) {
      if (LEVEL >= 5)
        asm volatile("s_waitcnt vmcnt(4)" ::: "memory");  // all but A's loads of a tile ago have landed
      else
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the loads issued a tile ago have landed
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
    }
    substep(S3, fb);
    koff += 128;
    if (++kcount == KT) { kcount = 0; koff = 0; ++pass; }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  float s = (float)(unsigned char)land[lane];
  for (int i = 0; i < FM; ++i)
    for (int j = 0; j < FN; ++j)
      for (int e = 0; e < 4; ++e) s += acc[i][j][e];
  out[blockIdx.x * 512 + tid] = s;
}

// The same levels for a block of 4 waves (one per SIMD), wave tile 128 x 128 = 8 x 8 fragments:
// a third fewer LDS fragment reads per flop (32 per wave and tile, 128 per block instead of 192).
// Schedule: a tile is two phases of 64 MFMAs (one per k-half); both operands' fragments are
// double-buffered by phase (2 x 16 fragments in registers), the 16 reads of the next phase ride
// behind the first 48 MFMAs of the current one, the tile's 16 loads behind the MFMAs of the
// second phase, the barrier sits between the phases.  (Level 5 as above: the weight's eight
// loads first, vmcnt(8) in front of the barrier.)
template <int LEVEL>
__global__ __launch_bounds__(256) void k_ceiling4(const bf16* __restrict__ src, const char* __restrict__ A,
                                                  const char* __restrict__ W, float* __restrict__ out, int iters) {
  constexpr int FM = 8, FN = 8, NLD = 16;
  __shared__ __attribute__((aligned(1024))) char lds[131072];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  for (int i = tid; i < 65536 / 16; i += 256) reinterpret_cast<uint4*>(lds)[i] = reinterpret_cast<const uint4*>(src)[i];
  __syncthreads();
  f32x4 acc[FM][FN];
  for (int i = 0; i < FM; ++i)
    for (int j = 0; j < FN; ++j)
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;
  const char* apool = lds + lane * 16;
  const char* bpool = lds + 32768 + lane * 16;
  bf16x8 fa[2][FM], fb[2][FN];
  for (int q = 0; q < 2; ++q) {
    for (int i = 0; i < FM; ++i) fa[q][i] = *(const bf16x8*)(apool + (((wave % 2) * 16 + q * 8 + i) & 31) * 1024);
    for (int j = 0; j < FN; ++j) fb[q][j] = *(const bf16x8*)(bpool + (((wave / 2) * 16 + q * 8 + j) & 31) * 1024);
  }
  char* land = lds + 65536 + wave * NLD * 1024;
  const char* gsrc[NLD];
  const int b = blockIdx.x, x = b % 8, l = b / 8, pm = l % 8, pn = l / 8;
  for (int i = 0; i < NLD; ++i) {
    const int piece = wave + 4 * (i % 8);                       // 32 pieces of 8 rows per operand tile
    const int row = 8 * piece + lane / 8, c = lane % 8;
    int arow = row, wrow = row;
    if (LEVEL >= 3) { arow = (x * 8 + pm) * 256 + row; wrow = pn * 256 + row; }
    gsrc[i] = i < 8 ? A + (size_t)arow * kRowBytes + c * 16 : W + (size_t)wrow * kRowBytes + c * 16;
  }
  constexpr int KT = LEVEL == 2 ? 32 : kStepsPerPass;
  const size_t a_pass = LEVEL >= 4 ? (size_t)64 * 256 * kRowBytes : 0;
  unsigned koff = 0;
  int kcount = 0, pass = 0;
  auto phase = [&](auto Q_, int frag_base) {
    constexpr int q = decltype(Q_)::value;
#pragma unroll
    for (int m = 0; m < 64; ++m) {
      const int j = m / FM, i = m % FM;
      mfma16(acc[i][j], fb[q][j], fa[q][i]);
      if (LEVEL >= 1 && m % 3 == 0 && m / 3 < 16) {
        // the other phase's fragments in the order its MFMAs need them: weight fragment 0, the 8 row
        // fragments, weight fragments 1..7
        const int n = m / 3;
        if (n == 0) fb[q ^ 1][0] = *(const bf16x8*)(bpool + ((frag_base + 16) & 31) * 1024);
        else if (n <= 8) fa[q ^ 1][n - 1] = *(const bf16x8*)(apool + ((frag_base + n) & 31) * 1024);
        else fb[q ^ 1][n - 8] = *(const bf16x8*)(bpool + ((frag_base + n + 8) & 31) * 1024);
      }
      if (LEVEL >= 2 && q == 1 && m % 3 == 1 && m / 3 < NLD) {
        const int idx = LEVEL >= 5 ? (m / 3 + 8) % NLD : m / 3;   // level 5: the weight's eight loads first
        const size_t po = idx < 8 ? (size_t)(pass & 1) * a_pass : 0;
        load_lds_16B(gsrc[idx] + koff + po, land + idx * 1024);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  constexpr std::integral_constant<int, 0> Q0{};
  constexpr std::integral_constant<int, 1> Q1{};
  for (int it = 0; it < iters; ++it) {
    const int fb_ = (wave % 2) * 16 + (it & 1) * 3;
    phase(Q0, fb_);
    if (LEVEL >= 2) {
      if (LEVEL >= 5)
        asm volatile("s_waitcnt vmcnt(8)" ::: "memory");   // A's loads of a tile ago stay in flight
      else
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
    }
    phase(Q1, fb_ + 5);
    koff += 128;
    if (++kcount == KT) { kcount = 0; koff = 0; ++pass; }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  float s = (float)(unsigned char)land[lane];
  for (int i = 0; i < FM; ++i)
    for (int j = 0; j < FN; ++j)
      for (int e = 0; e < 4; ++e) s += acc[i][j][e];
  out[blockIdx.x * 256 + tid] = s;
}

int main(int argc, char** argv) {
  const int iters = argc > 1 ? atoi(argv[1]) : 8000;   // tiles per block
  const int reps = argc > 2 ? atoi(argv[2]) : 4;       // the first repetition is a warm-up
  if (iters < 1 || reps < 2) return 1;
  std::vector<bf16> h(32768), zeros(32768, (bf16)0.f);
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
  const size_t abytes = (size_t)kRowsA * kRowBytes, wbytes = (size_t)kRowsW * kRowBytes;
  // host-side bound check of the kernels' address patterns: the largest row any lane reads is
  // (7 * 8 + 7) * 256 + 255 = 16383 (+ 16384 on odd passes of levels 4 and 5) of A and 3 * 256 + 255 of W,
  // the largest byte within a row 79 * 128 + 7 * 16 + 15
  {
    const size_t max_arow = (size_t)(7 * 8 + 7) * 256 + 255 + (size_t)64 * 256, max_wrow = 3 * 256 + 255;
    const size_t max_col = (size_t)(kStepsPerPass - 1) * 128 + 7 * 16 + 16;
    if (max_arow * kRowBytes + max_col > abytes || max_wrow * kRowBytes + max_col > wbytes) {
      printf("address pattern exceeds the buffers\n");
      return 1;
    }
  }
  CK(hipMalloc(&src, 65536));
  CK(hipMalloc(&out, 256 * 512 * 4));
  CK(hipMalloc(&A, abytes));
  CK(hipMalloc(&W, wbytes));
  CK(hipMemset(A, 0x3c, abytes));
  CK(hipMemset(W, 0x3c, wbytes));
  struct Variant { const char* name; int level; };   // level -1: the 32x32x16 register loop
  const Variant vs[] = {
      {"32x32x16, registers only", -1},
      {"16x16x32, 0 registers only", 0},
      {"16x16x32, 1 + LDS fragment reads", 1},
      {"16x16x32, 2 + global->LDS loads (L2-resident), barrier", 2},
      {"16x16x32, 3 + GEMM addresses, A in the Infinity Cache", 3},
      {"16x16x32, 4 + GEMM addresses, A streamed from HBM", 4},
      {"16x16x32, 5 = 4 with A's loads two tiles ahead of their use", 5},
      {"4 waves of 128 x 128: 1 + LDS fragment reads", 11},
      {"4 waves of 128 x 128: 2 + global->LDS loads (L2-resident), barrier", 12},
      {"4 waves of 128 x 128: 3 + GEMM addresses, A in the Infinity Cache", 13},
      {"4 waves of 128 x 128: 4 + GEMM addresses, A streamed from HBM", 14},
      {"4 waves of 128 x 128: 5 = 4 with A's loads two tiles ahead of their use", 15},
  };
  constexpr int NV = sizeof(vs) / sizeof(vs[0]);
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  const double flops = 2.0 * 256 * 256 * 64 * (double)iters * 256;
  double tf[2][NV] = {};
  for (int data = 0; data < 2; ++data) {
    CK(hipMemcpy(src, data == 0 ? h.data() : zeros.data(), 65536, hipMemcpyHostToDevice));
    for (int r = 0; r < reps; ++r)
      for (int i = 0; i < NV; ++i) {
        CK(hipEventRecord(e0));
        switch (vs[i].level) {
          case -1: hipLaunchKernelGGL(k_regs_32x32x16, dim3(256), dim3(512), 0, 0, src, out, iters); break;
          case 0: hipLaunchKernelGGL(k_ceiling<0>, dim3(256), dim3(512), 0, 0, src, A, W, out, iters); break;
          case 1: hipLaunchKernelGGL(k_ceiling<1>, dim3(256), dim3(512), 0, 0, src, A, W, out, iters); break;
          case 2: hipLaunchKernelGGL(k_ceiling<2>, dim3(256), dim3(512), 0, 0, src, A, W, out, iters); break;
          case 3: hipLaunchKernelGGL(k_ceiling<3>, dim3(256), dim3(512), 0, 0, src, A, W, out, iters); break;
          case 4: hipLaunchKernelGGL(k_ceiling<4>, dim3(256), dim3(512), 0, 0, src, A, W, out, iters); break;
          case 5: hipLaunchKernelGGL(k_ceiling<5>, dim3(256), dim3(512), 0, 0, src, A, W, out, iters); break;
          case 11: hipLaunchKernelGGL(k_ceiling4<1>, dim3(256), dim3(256), 0, 0, src, A, W, out, iters); break;
          case 12: hipLaunchKernelGGL(k_ceiling4<2>, dim3(256), dim3(256), 0, 0, src, A, W, out, iters); break;
          case 13: hipLaunchKernelGGL(k_ceiling4<3>, dim3(256), dim3(256), 0, 0, src, A, W, out, iters); break;
          case 14: hipLaunchKernelGGL(k_ceiling4<4>, dim3(256), dim3(256), 0, 0, src, A, W, out, iters); break;
          default: hipLaunchKernelGGL(k_ceiling4<5>, dim3(256), dim3(256), 0, 0, src, A, W, out, iters); break;
        }
        CK(hipGetLastError());
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        float ms;
        CK(hipEventElapsedTime(&ms, e0, e1));
        if (r > 0) tf[data][i] += flops / ms / 1e9 / (reps - 1);
        printf("%s rep %d %s: %.1f TFLOP/s\n", data == 0 ? "random" : "zeros", r, vs[i].name, flops / ms / 1e9);
        fflush(stdout);
      }
  }
  printf("| inner loop | TFLOP/s, N(0,1) x N(0,0.02^2) operands | share of 2500 | TFLOP/s, all-zero operands |\n|---|---|---|---|\n");
  for (int i = 0; i < NV; ++i) printf("| %s | %.0f | %.3f | %.0f |\n", vs[i].name, tf[0][i], tf[0][i] / 2500.0, tf[1][i]);
  return 0;
}
