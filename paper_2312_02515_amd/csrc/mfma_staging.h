// Staging primitives shared by the MFMA kernels (gfx950): direct global->LDS loads and the
// transposing LDS read.
#pragma once

#include "mlora_common.h"

namespace mlora {
namespace stage {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(8))) short short8v;

#define MLORA_AS3 __attribute__((address_space(3)))

#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"  // m0 is named as a clobber on purpose
// Direct global->LDS load of 16 B per lane: lane l's data lands at lds_wave_base + 16 l.
// Issued as inline assembly so that the compiler's wait-count insertion does not see an LDS
// write it would serialise the following LDS reads behind; the kernels place every
// s_waitcnt vmcnt for these loads themselves (wait_vmcnt).  M0 carries the LDS base.
__device__ __forceinline__ void load_lds_16B(const void* g, char* lds_wave_base) {
  const unsigned lds = (unsigned)(size_t)(MLORA_AS3 char*)lds_wave_base;
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds) : "memory", "m0");
}
// Same, with the address split into a wave-uniform 64-bit base (SGPR pair) and a 32-bit
// per-lane byte offset: issuing it reads one address VGPR per lane instead of two.
__device__ __forceinline__ void load_lds_16B_sbase(const void* base_uniform, unsigned lane_off, char* lds_wave_base) {
  const unsigned lds = (unsigned)(size_t)(MLORA_AS3 char*)lds_wave_base;
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(base_uniform), "s"(lds)
               : "memory", "m0");
}
#pragma clang diagnostic pop

template <int N> __device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Waits until every LDS read this wave has issued has returned its data.
__device__ __forceinline__ void wait_lds() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// ds_read_b64_tr_b16: within each group of 16 lanes, lane L supplies the address of 4 consecutive
// 16-bit elements of row L / 4 (columns 4 (L % 4) ..); lane i receives column i of that 4 x 16
// block, i.e. four consecutive rows of one column.
__device__ __forceinline__ short4v lds_read_tr(const char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLORA_AS3 short4v*)p);
}

__device__ __forceinline__ bf16x8 join(short4v lo, short4v hi) {
  short8v v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ bf16x8 lds_read_tr_pair(const char* p0, const char* p1) {
  return join(lds_read_tr(p0), lds_read_tr(p1));
}

}  // namespace stage
}  // namespace mlora
