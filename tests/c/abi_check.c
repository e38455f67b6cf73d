/* Plain C translation unit against include/mlora.h: the header must compile as C, and the
 * argument-checking entry points must be callable without a GPU.  Built and run by
 * tests/test_host_abi.py; prints one line per check and exits non-zero on a mismatch. */
#include <stdio.h>
#include <string.h>

#include "mlora.h"

static int fails = 0;
#define EXPECT(cond)                                          \
  do {                                                        \
    if (!(cond)) {                                            \
      printf("FAIL line %d: %s\n", __LINE__, #cond);          \
      ++fails;                                                \
    }                                                         \
  } while (0)

int main(void) {
  int64_t off[3] = {0, 32, 64};
  int32_t ranks[2] = {8, 4};
  float s[2] = {2.0f, 0.5f};
  const void* A[2] = {(const void*)0x1000, (const void*)0x2000};
  const void* B[2] = {(const void*)0x3000, (const void*)0x4000};
  mlora_problem p;
  memset(&p, 0, sizeof p);
  p.T = 64;
  p.h = 32;
  p.d = 48;
  p.K = 2;
  p.dtype = MLORA_BF16;
  p.seg_offsets = off;
  p.ranks = ranks;
  p.scalings = s;
  p.A = A;
  p.B = B;
  p.W = (const void*)0x5000;
  EXPECT(mlora_lora_validate(&p) == MLORA_OK);
  EXPECT(mlora_lora_saved_bytes(&p) >= 64 * 16 * 2);
  EXPECT(mlora_lora_workspace_bytes(&p) >= 64 * 16 * 2);
  EXPECT(mlora_lora_recompute_workspace_bytes(&p) >= 2 * 64 * 16 * 2);
  off[1] = 70;
  EXPECT(mlora_lora_validate(&p) == MLORA_ERR_SEGMENTS);
  off[1] = 32;
  ranks[1] = MLORA_MAX_RANK + 1;
  EXPECT(mlora_lora_validate(&p) == MLORA_ERR_RANK);
  ranks[1] = 4;
  p.W = NULL;
  EXPECT(mlora_lora_validate(&p) == MLORA_ERR_NULL);
  p.W = (const void*)0x5000;
  EXPECT(mlora_lora_fwd(&p, NULL, (void*)0x10, (void*)0x20, (void*)0x30, 1u << 20, NULL) == MLORA_ERR_NULL);
  {
    const mlora_problem* ps[2];
    ps[0] = &p;
    ps[1] = &p;
    EXPECT(mlora_lora_group_validate(ps, 2) == MLORA_OK);
    EXPECT(mlora_lora_group_validate(ps, MLORA_MAX_GROUP + 1) == MLORA_ERR_SHAPE);
    EXPECT(mlora_lora_group_workspace_bytes(ps, 2) == 2 * mlora_lora_workspace_bytes(&p));
  }
  /* the 8-bit-weight calls: p.W is not looked at; argument checks come before any GPU work */
  p.W = NULL;
  EXPECT(mlora_lora_w8_workspace_bytes(&p) > mlora_lora_saved_bytes(&p));
  EXPECT(mlora_lora_fwd_w8(&p, NULL, (const float*)0x70, (void*)0x10, (void*)0x20, (void*)0x30, (void*)0x40, 1u << 20,
                           NULL) == MLORA_ERR_NULL);
  EXPECT(mlora_lora_fwd_w8(&p, (const int8_t*)0x60, (const float*)0x70, (void*)0x10, (void*)0x20, (void*)0x30,
                           (void*)0x40, 16, NULL) == MLORA_ERR_WORKSPACE);
  EXPECT(mlora_w8_quantize((const void*)0x10, 7, 8, 8, (int8_t*)0x20, (float*)0x30, NULL) == MLORA_ERR_DTYPE);
  EXPECT(mlora_w8_dequantize((const int8_t*)0x10, (const float*)0x20, MLORA_BF16, 0, 8, (void*)0x30, NULL) ==
         MLORA_ERR_SHAPE);
  EXPECT(mlora_lora_kernel_path(&p) == -1);
  p.W = (const void*)0x5000;
  EXPECT(mlora_lora_kernel_path(&p) == 3);   /* h, d not multiples of 64: the generic kernels */
  EXPECT(mlora_lora_bwd_static(&p, (void*)0x10, NULL, (void*)0x20, (void*)0x30, NULL, NULL, 0, NULL) == MLORA_ERR_NULL);
  EXPECT(strlen(mlora_status_string(MLORA_ERR_WORKSPACE)) > 0);
  printf(fails ? "abi_check: %d failure(s)\n" : "abi_check: ok\n", fails);
  return fails ? 1 : 0;
}
