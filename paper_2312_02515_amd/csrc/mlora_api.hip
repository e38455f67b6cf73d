// C-ABI entry points of libmlora: argument validation, buffer layout, dispatch.
// No kernel lives here.
#include <atomic>
#include <mutex>

#include "../../include/mlora_testing.h"
#include "mlora_common.h"

// Scratch of mlora_lora_bwd_static: G and the gradient kernels' partial sums live here instead
// of in a caller's workspace.  One copy per GPU the library runs on, held until the process ends.
static __device__ __align__(256) unsigned char scratch[MLORA_STATIC_SCRATCH_BYTES];

namespace mlora {
namespace {

// `scratch` names a host-side stand-in, not device memory: the array's device address is looked
// up once per device (each GPU has its own copy at its own address) and only that pointer is
// ever handed to kernels.
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mu;

hipError_t static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (ptr == nullptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

thread_local int g_last_hip_error = 0;
std::atomic<int> g_kernel_path{0};

// `need_W` = false: for the queries and calls that never read p->W
mlora_status validate(const mlora_problem* p, bool need_W = true) {
  if (p == nullptr) return MLORA_ERR_NULL;
  if (p->dtype != MLORA_BF16 && p->dtype != MLORA_F32) return MLORA_ERR_DTYPE;
  if (p->T < 0 || p->h <= 0 || p->d <= 0) return MLORA_ERR_SHAPE;
  // row and feature indices are 32-bit inside the kernels, byte offsets within a 256-row tile
  // too (256 rows x 4 Mi features x 2 B = 2^31), and a grid holds fewer than 2^31 tiles
  if (p->T > 0x7fffffffLL - 1024 || p->h > (1 << 22) || p->d > (1 << 22)) return MLORA_ERR_SHAPE;
  {
    const int64_t wide = p->h > p->d ? p->h : p->d;
    if ((p->T / 256 + 1) * (wide / 256 + 1) > 0x7fffffffLL) return MLORA_ERR_SHAPE;
  }
  if (p->K < 0 || p->K > kMaxK) return MLORA_ERR_SHAPE;
  if (need_W && p->W == nullptr) return MLORA_ERR_NULL;
  if (p->K > 0) {
    if (!p->seg_offsets || !p->ranks || !p->scalings || !p->A || !p->B) return MLORA_ERR_NULL;
    int64_t prev = 0;
    for (int k = 0; k <= p->K; ++k) {
      int64_t o = p->seg_offsets[k];
      if (o < prev || o > p->T) return MLORA_ERR_SEGMENTS;
      prev = o;
    }
    for (int k = 0; k < p->K; ++k) {
      if (p->ranks[k] < 1 || p->ranks[k] > kMaxRank) return MLORA_ERR_RANK;
    }
    for (int k = 0; k < p->K; ++k) {
      if (p->A[k] == nullptr || p->B[k] == nullptr) return MLORA_ERR_NULL;
    }
  }
  return MLORA_OK;
}

size_t elem_size(const mlora_problem* p) { return p->dtype == MLORA_F32 ? 4 : 2; }

// bytes of one [T, ldz] low-rank intermediate (Z in `saved`, G at the head of the workspace)
size_t lowrank_bytes(const mlora_problem* p) {
  return align_up((size_t)p->T * (size_t)lowrank_ld(p) * elem_size(p), 256);
}

void fill_ctx(const mlora_problem* p, void* stream, CallCtx* c) {
  c->T = (int)p->T;
  c->h = (int)p->h;
  c->d = (int)p->d;
  c->K = p->K;
  c->ldz = lowrank_ld(p);
  c->dtype = p->dtype;
  c->W = p->W;
  c->stream = static_cast<hipStream_t>(stream);
  c->st.K = p->K;
  for (int k = 0; k < kMaxK; ++k) {
    bool live = k < p->K;
    c->st.off[k] = live ? (int)p->seg_offsets[k] : 0;
    c->st.rank[k] = live ? p->ranks[k] : 0;
    c->st.s[k] = live ? p->scalings[k] : 0.f;
    c->A.p[k] = live ? p->A[k] : nullptr;
    c->B.p[k] = live ? p->B[k] : nullptr;
  }
  c->st.off[kMaxK] = 0;
  if (p->K > 0) {
    for (int k = p->K; k <= kMaxK; ++k) c->st.off[k] = (int)p->seg_offsets[p->K];
  }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// The MFMA kernels take bf16 problems whose feature sizes are multiples of 64, whose ranks are
// multiples of 8 (mfma_sizes_ok) and whose buffers are 16-byte aligned; everything else runs the
// generic kernels.
bool mfma_sizes_ok(const mlora_problem* p) {
  if (p->dtype != MLORA_BF16 || p->T < 1) return false;
  if (!gemm_mfma_ok((int)p->T, (int)p->d, (int)p->h) || !gemm_mfma_ok((int)p->T, (int)p->h, (int)p->d)) return false;
  for (int k = 0; k < p->K; ++k)
    if (p->ranks[k] % 8 != 0) return false;
  return true;
}

bool mfma_shapes_ok(const mlora_problem* p) {
  if (!mfma_sizes_ok(p) || !aligned16(p->W)) return false;
  for (int k = 0; k < p->K; ++k)
    if (!aligned16(p->A[k]) || !aligned16(p->B[k])) return false;
  return true;
}

bool mfma_gemm_applies(const mlora_problem* p) { return !(g_kernel_path.load() & 1) && mfma_shapes_ok(p); }
bool mfma_lowrank_applies(const mlora_problem* p) { return !(g_kernel_path.load() & 2) && mfma_shapes_ok(p); }

// Scratch for the token-split form of the gradient kernels (0 when they do not split).  A
// function of the sizes alone: a size query must not change its answer with the addresses.
size_t grad_scratch_bytes(const mlora_problem* p) {
  if (!mfma_sizes_ok(p) || p->K == 0) return 0;
  CallCtx c;
  fill_ctx(p, nullptr, &c);
  const size_t a = grad_partial_bytes(c.st, c.h), b = grad_partial_bytes(c.st, c.d);
  return a > b ? a : b;
}

mlora_status hip_status(hipError_t e) {
  if (e == hipSuccess) return MLORA_OK;
  g_last_hip_error = (int)e;
  return MLORA_ERR_HIP;
}

// Z = s_k x_k A_k into `Z` ([T, ldz], layout of the `saved` buffer)
hipError_t compute_Z(const mlora_problem* p, const CallCtx& c, const void* X, void* Z) {
  if (mfma_lowrank_applies(p) && aligned16(X) && aligned16(Z))
    return lowrank_rows_mfma(c, (const bf16*)X, c.h, (bf16*)Z, c.A, true);
  return generic_Z(c, X, Z);
}

// Y = X W + Z B_k, given Z
hipError_t forward_gemm(const mlora_problem* p, const CallCtx& c, const void* X, void* Y, const void* Z) {
  if (mfma_gemm_applies(p) && aligned16(X) && aligned16(Y) && aligned16(Z))
    return gemm_mfma((const bf16*)X, (const bf16*)p->W, (bf16*)Y, c.T, c.d, c.h, true, (const bf16*)Z, c.ldz, c.st, c.B,
                     c.stream);
  return generic_gemm_fwd(c, X, Y, Z);
}

hipError_t forward_impl(const mlora_problem* p, const CallCtx& c, const void* X, void* Y, void* Z) {
  hipError_t e = compute_Z(p, c, X, Z);
  if (e != hipSuccess) return e;
  return forward_gemm(p, c, X, Y, Z);
}

mlora_status check_grad_tables(const mlora_problem* p, float* const* dA, float* const* dB) {
  if (p->K > 0) {
    if (dA == nullptr || dB == nullptr) return MLORA_ERR_NULL;
    for (int k = 0; k < p->K; ++k)
      if (dA[k] == nullptr || dB[k] == nullptr) return MLORA_ERR_NULL;
  }
  return MLORA_OK;
}

// G, dB_k and dA_k, given Z
// (with `skip_dA` the caller computes dA_k itself from G)
hipError_t adapter_grads_impl(const mlora_problem* p, const CallCtx& c, const void* X, const void* dY, const void* Z,
                              void* G, float* const* dA, float* const* dB, int accumulate, float* partial,
                              bool skip_dA = false) {
  OutTable ta, tb;
  for (int k = 0; k < kMaxK; ++k) {
    ta.p[k] = k < p->K ? dA[k] : nullptr;
    tb.p[k] = k < p->K ? dB[k] : nullptr;
  }
  hipError_t e;
  if (mfma_lowrank_applies(p) && aligned16(X) && aligned16(dY) && aligned16(Z) && aligned16(G)) {
    e = lowrank_rows_mfma(c, (const bf16*)dY, c.d, (bf16*)G, c.B, false);
    if (e == hipSuccess) e = grad_mfma(c, (const bf16*)dY, c.d, (const bf16*)Z, tb, accumulate ? 1 : 0, false, partial);
    if (e == hipSuccess && !skip_dA)
      e = grad_mfma(c, (const bf16*)X, c.h, (const bf16*)G, ta, accumulate ? 1 : 0, true, partial);
  } else {
    e = generic_G(c, dY, G);
    if (e == hipSuccess) e = generic_dB(c, Z, dY, tb, accumulate ? 1 : 0);
    if (e == hipSuccess && !skip_dA) e = generic_dA(c, X, G, ta, accumulate ? 1 : 0);
  }
  return e;
}

// G, dB_k, dA_k and (unless dX is NULL) dX, given Z
hipError_t backward_impl(const mlora_problem* p, const CallCtx& c, const void* X, const void* dY, const void* Z, void* G,
                         void* dX, float* const* dA, float* const* dB, int accumulate, float* partial) {
  hipError_t e = adapter_grads_impl(p, c, X, dY, Z, G, dA, dB, accumulate, partial);
  if (e == hipSuccess && dX != nullptr && p->T > 0) {
    if (mfma_gemm_applies(p) && aligned16(dY) && aligned16(dX) && aligned16(G))
      e = gemm_mfma((const bf16*)dY, (const bf16*)p->W, (bf16*)dX, c.T, c.h, c.d, false, (const bf16*)G, c.ldz, c.st, c.A,
                    c.stream);
    else
      e = generic_gemm_bwd(c, dY, dX, G);
  }
  return e;
}

// Whether the shared-input low-rank kernels (one pass over X for all projections) apply
bool group_lowrank_applies(const mlora_problem* const* ps, int P, const void* X) {
  if (P < 2 || !aligned16(X)) return false;
  int mx = 0;
  for (int p = 0; p < P; ++p) {
    if (!mfma_lowrank_applies(ps[p])) return false;
    const int l = lowrank_ld(ps[p]);
    mx = l > mx ? l : mx;
  }
  return lowrank_group_ok(P, mx);
}

// A group is valid when each member is and all share T, h, K, the dtype and the split positions.
mlora_status validate_group(const mlora_problem* const* ps, int P) {
  if (ps == nullptr) return MLORA_ERR_NULL;
  if (P < 1 || P > MLORA_MAX_GROUP) return MLORA_ERR_SHAPE;
  for (int p = 0; p < P; ++p) {
    mlora_status st = validate(ps[p]);
    if (st != MLORA_OK) return st;
  }
  for (int p = 1; p < P; ++p) {
    if (ps[p]->dtype != ps[0]->dtype) return MLORA_ERR_DTYPE;
    if (ps[p]->T != ps[0]->T || ps[p]->h != ps[0]->h || ps[p]->K != ps[0]->K) return MLORA_ERR_SHAPE;
    for (int k = 0; k <= ps[0]->K && ps[0]->K > 0; ++k)
      if (ps[p]->seg_offsets[k] != ps[0]->seg_offsets[k]) return MLORA_ERR_SEGMENTS;
  }
  return MLORA_OK;
}

}  // namespace
}  // namespace mlora

using namespace mlora;

extern "C" {

mlora_status mlora_lora_validate(const mlora_problem* p) { return validate(p); }

size_t mlora_lora_saved_bytes(const mlora_problem* p) {
  if (validate(p, false) != MLORA_OK) return 0;
  size_t b = lowrank_bytes(p);
  return b ? b : 256;
}

size_t mlora_lora_workspace_bytes(const mlora_problem* p) {
  if (validate(p) != MLORA_OK) return 0;
  size_t b = lowrank_bytes(p) + grad_scratch_bytes(p);  // G, partial sums of split gradient launches
  return b ? b : 256;
}

size_t mlora_lora_recompute_workspace_bytes(const mlora_problem* p) {
  if (validate(p) != MLORA_OK) return 0;
  size_t b = 2 * lowrank_bytes(p) + grad_scratch_bytes(p);  // G, Z, partial sums
  return b ? b : 256;
}

mlora_status mlora_lora_fwd(const mlora_problem* p, const void* X, void* Y, void* saved, void* workspace,
                            size_t workspace_bytes, void* hip_stream) {
  mlora_status st = validate(p);
  if (st != MLORA_OK) return st;
  if (p->T == 0) return MLORA_OK;
  if (X == nullptr || Y == nullptr || saved == nullptr) return MLORA_ERR_NULL;
  if (workspace == nullptr || workspace_bytes < mlora_lora_workspace_bytes(p)) return MLORA_ERR_WORKSPACE;
  CallCtx c;
  fill_ctx(p, hip_stream, &c);
  return hip_status(forward_impl(p, c, X, Y, saved));
}

mlora_status mlora_lora_fwd_nosave(const mlora_problem* p, const void* X, void* Y, void* workspace,
                                   size_t workspace_bytes, void* hip_stream) {
  mlora_status st = validate(p);
  if (st != MLORA_OK) return st;
  if (p->T == 0) return MLORA_OK;
  if (X == nullptr || Y == nullptr) return MLORA_ERR_NULL;
  if (workspace == nullptr || workspace_bytes < mlora_lora_recompute_workspace_bytes(p)) return MLORA_ERR_WORKSPACE;
  CallCtx c;
  fill_ctx(p, hip_stream, &c);
  void* Z = static_cast<char*>(workspace) + lowrank_bytes(p);
  return hip_status(forward_impl(p, c, X, Y, Z));
}

mlora_status mlora_lora_bwd(const mlora_problem* p, const void* X, const void* dY, const void* saved, void* dX,
                            float* const* dA, float* const* dB, int accumulate, void* workspace,
                            size_t workspace_bytes, void* hip_stream) {
  mlora_status st = validate(p);
  if (st != MLORA_OK) return st;
  if (p->T > 0 && (X == nullptr || dY == nullptr || saved == nullptr)) return MLORA_ERR_NULL;
  st = check_grad_tables(p, dA, dB);
  if (st != MLORA_OK) return st;
  if (workspace == nullptr || workspace_bytes < mlora_lora_workspace_bytes(p)) return MLORA_ERR_WORKSPACE;
  if (p->T == 0 && accumulate) return MLORA_OK;
  CallCtx c;
  fill_ctx(p, hip_stream, &c);
  float* partial = grad_scratch_bytes(p) ? reinterpret_cast<float*>(static_cast<char*>(workspace) + lowrank_bytes(p)) : nullptr;
  return hip_status(backward_impl(p, c, X, dY, saved, workspace, dX, dA, dB, accumulate, partial));
}

mlora_status mlora_lora_bwd_static(const mlora_problem* p, const void* X, const void* dY, const void* saved, void* dX,
                                   float* const* dA, float* const* dB, int accumulate, void* hip_stream) {
  mlora_status st = validate(p);
  if (st != MLORA_OK) return st;
  if (p->T > 0 && (X == nullptr || dY == nullptr || saved == nullptr)) return MLORA_ERR_NULL;
  st = check_grad_tables(p, dA, dB);
  if (st != MLORA_OK) return st;
  if (mlora_lora_workspace_bytes(p) > (size_t)MLORA_STATIC_SCRATCH_BYTES) return MLORA_ERR_WORKSPACE;
  if (p->T == 0 && accumulate) return MLORA_OK;
  void* ws = nullptr;
  const hipError_t e = static_scratch(&ws);
  if (e != hipSuccess) return hip_status(e);
  // Nothing in the scratch has to start at zero: G is written for every row that is read, the
  // partial sums are overwritten before the reduction reads them.
  return mlora_lora_bwd(p, X, dY, saved, dX, dA, dB, accumulate, ws, (size_t)MLORA_STATIC_SCRATCH_BYTES, hip_stream);
}

mlora_status mlora_lora_bwd_recompute(const mlora_problem* p, const void* X, const void* dY, void* dX,
                                      float* const* dA, float* const* dB, int accumulate, void* workspace,
                                      size_t workspace_bytes, void* hip_stream) {
  mlora_status st = validate(p);
  if (st != MLORA_OK) return st;
  if (p->T > 0 && (X == nullptr || dY == nullptr)) return MLORA_ERR_NULL;
  st = check_grad_tables(p, dA, dB);
  if (st != MLORA_OK) return st;
  if (workspace == nullptr || workspace_bytes < mlora_lora_recompute_workspace_bytes(p)) return MLORA_ERR_WORKSPACE;
  if (p->T == 0 && accumulate) return MLORA_OK;
  CallCtx c;
  fill_ctx(p, hip_stream, &c);
  void* Z = static_cast<char*>(workspace) + lowrank_bytes(p);
  hipError_t e = p->T > 0 ? compute_Z(p, c, X, Z) : hipSuccess;
  if (e != hipSuccess) return hip_status(e);
  float* partial =
      grad_scratch_bytes(p) ? reinterpret_cast<float*>(static_cast<char*>(workspace) + 2 * lowrank_bytes(p)) : nullptr;
  return hip_status(backward_impl(p, c, X, dY, Z, workspace, dX, dA, dB, accumulate, partial));
}

// ---- 8-bit frozen base weight: decode into the head of the workspace, then the plain path ----
namespace {

size_t w8_weight_bytes(const mlora_problem* p) { return align_up((size_t)p->h * (size_t)p->d * elem_size(p), 256); }

mlora_status w8_check_matrix(const void* a, const void* b, const void* c, int32_t dtype, int64_t h, int64_t d) {
  if (a == nullptr || b == nullptr || c == nullptr) return MLORA_ERR_NULL;
  if (dtype != MLORA_BF16 && dtype != MLORA_F32) return MLORA_ERR_DTYPE;
  if (h < 1 || d < 1 || h > (1 << 22) || d > (1 << 22)) return MLORA_ERR_SHAPE;
  return MLORA_OK;
}

// The problem as the plain entry points see it: W^ lives at the head of the workspace.
// (validate() only asks that W is not NULL, so any non-NULL stand-in serves for the checks.)
mlora_problem w8_plain_problem(const mlora_problem* p, const void* w_hat) {
  mlora_problem q = *p;
  q.W = w_hat;
  return q;
}

}  // namespace

mlora_status mlora_w8_quantize(const void* W, int32_t dtype, int64_t h, int64_t d, int8_t* Wq, float* c,
                               void* hip_stream) {
  const mlora_status st = w8_check_matrix(W, Wq, c, dtype, h, d);
  if (st != MLORA_OK) return st;
  return hip_status(w8_quantize(W, dtype, (int)h, (int)d, Wq, c, static_cast<hipStream_t>(hip_stream)));
}

mlora_status mlora_w8_dequantize(const int8_t* Wq, const float* c, int32_t dtype, int64_t h, int64_t d, void* W_hat,
                                 void* hip_stream) {
  const mlora_status st = w8_check_matrix(Wq, c, W_hat, dtype, h, d);
  if (st != MLORA_OK) return st;
  return hip_status(w8_dequantize(Wq, c, dtype, (int)h, (int)d, W_hat, static_cast<hipStream_t>(hip_stream)));
}

size_t mlora_lora_w8_workspace_bytes(const mlora_problem* p) {
  if (p == nullptr) return 0;
  static const char stand_in = 0;
  const mlora_problem q = w8_plain_problem(p, &stand_in);
  if (validate(&q) != MLORA_OK) return 0;
  return w8_weight_bytes(&q) + mlora_lora_workspace_bytes(&q);
}

mlora_status mlora_lora_fwd_w8(const mlora_problem* p, const int8_t* Wq, const float* c, const void* X, void* Y,
                               void* saved, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (p == nullptr) return MLORA_ERR_NULL;
  static const char stand_in = 0;
  mlora_problem q = w8_plain_problem(p, workspace ? workspace : &stand_in);
  mlora_status st = validate(&q);
  if (st != MLORA_OK) return st;
  if (Wq == nullptr || c == nullptr) return MLORA_ERR_NULL;
  if (q.T == 0) return MLORA_OK;
  if (X == nullptr || Y == nullptr || saved == nullptr) return MLORA_ERR_NULL;
  if (workspace == nullptr || workspace_bytes < mlora_lora_w8_workspace_bytes(p)) return MLORA_ERR_WORKSPACE;
  const hipError_t e = w8_dequantize(Wq, c, q.dtype, (int)q.h, (int)q.d, workspace, static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return hip_status(e);
  const size_t wb = w8_weight_bytes(&q);
  return mlora_lora_fwd(&q, X, Y, saved, static_cast<char*>(workspace) + wb, workspace_bytes - wb, hip_stream);
}

mlora_status mlora_lora_bwd_w8(const mlora_problem* p, const int8_t* Wq, const float* c, const void* X,
                               const void* dY, const void* saved, void* dX, float* const* dA, float* const* dB,
                               int accumulate, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (p == nullptr) return MLORA_ERR_NULL;
  static const char stand_in = 0;
  mlora_problem q = w8_plain_problem(p, workspace ? workspace : &stand_in);
  mlora_status st = validate(&q);
  if (st != MLORA_OK) return st;
  if (Wq == nullptr || c == nullptr) return MLORA_ERR_NULL;
  if (q.T > 0 && (X == nullptr || dY == nullptr || saved == nullptr)) return MLORA_ERR_NULL;
  st = check_grad_tables(&q, dA, dB);
  if (st != MLORA_OK) return st;
  if (workspace == nullptr || workspace_bytes < mlora_lora_w8_workspace_bytes(p)) return MLORA_ERR_WORKSPACE;
  if (q.T == 0 && accumulate) return MLORA_OK;
  if (dX != nullptr && q.T > 0) {   // only the input gradient reads the weight
    const hipError_t e =
        w8_dequantize(Wq, c, q.dtype, (int)q.h, (int)q.d, workspace, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return hip_status(e);
  }
  const size_t wb = w8_weight_bytes(&q);
  return mlora_lora_bwd(&q, X, dY, saved, dX, dA, dB, accumulate, static_cast<char*>(workspace) + wb,
                        workspace_bytes - wb, hip_stream);
}

mlora_status mlora_lora_group_validate(const mlora_problem* const* ps, int P) { return validate_group(ps, P); }

size_t mlora_lora_group_workspace_bytes(const mlora_problem* const* ps, int P) {
  if (validate_group(ps, P) != MLORA_OK) return 0;
  size_t b = 0;
  size_t scratch = 0;
  for (int p = 0; p < P; ++p) {
    b += lowrank_bytes(ps[p]);  // every G_p is live until dX is written
    const size_t g = grad_scratch_bytes(ps[p]);
    scratch = g > scratch ? g : scratch;  // shared: the projections' gradient launches run in turn
  }
  b += scratch;
  return b ? b : 256;
}

mlora_status mlora_lora_group_fwd(const mlora_problem* const* ps, int P, const void* X, void* const* Y,
                                  void* const* saved, void* workspace, size_t workspace_bytes, void* hip_stream) {
  mlora_status st = validate_group(ps, P);
  if (st != MLORA_OK) return st;
  if (ps[0]->T == 0) return MLORA_OK;
  if (X == nullptr || Y == nullptr || saved == nullptr) return MLORA_ERR_NULL;
  for (int p = 0; p < P; ++p)
    if (Y[p] == nullptr || saved[p] == nullptr) return MLORA_ERR_NULL;
  if (workspace == nullptr || workspace_bytes < mlora_lora_group_workspace_bytes(ps, P)) return MLORA_ERR_WORKSPACE;
  CallCtx c[MLORA_MAX_GROUP];
  bool fused = group_lowrank_applies(ps, P, X);
  for (int p = 0; p < P; ++p) {
    fill_ctx(ps[p], hip_stream, &c[p]);
    fused = fused && aligned16(saved[p]);
  }
  if (fused) {
    // every Z_p in one pass over X
    LowrankGroupItem it[MLORA_MAX_GROUP];
    for (int p = 0; p < P; ++p) {
      it[p] = LowrankGroupItem{c[p].ldz, c[p].st.rank, c[p].st.s, &c[p].A, (bf16*)saved[p], nullptr, nullptr};
    }
    hipError_t e = lowrank_rows_mfma_group(P, it, c[0].st, (const bf16*)X, c[0].h, c[0].stream);
    if (e != hipSuccess) return hip_status(e);
  }
  for (int p = 0; p < P; ++p) {
    hipError_t e = fused ? forward_gemm(ps[p], c[p], X, Y[p], saved[p]) : forward_impl(ps[p], c[p], X, Y[p], saved[p]);
    if (e != hipSuccess) return hip_status(e);
  }
  return MLORA_OK;
}

mlora_status mlora_lora_group_bwd(const mlora_problem* const* ps, int P, const void* X, const void* const* dY,
                                  const void* const* saved, void* dX, float* const* const* dA,
                                  float* const* const* dB, int accumulate, void* workspace, size_t workspace_bytes,
                                  void* hip_stream) {
  mlora_status st = validate_group(ps, P);
  if (st != MLORA_OK) return st;
  if (dY == nullptr || saved == nullptr) return MLORA_ERR_NULL;
  if (ps[0]->T > 0) {
    if (X == nullptr) return MLORA_ERR_NULL;
    for (int p = 0; p < P; ++p)
      if (dY[p] == nullptr || saved[p] == nullptr) return MLORA_ERR_NULL;
  }
  if (ps[0]->K > 0) {
    if (dA == nullptr || dB == nullptr) return MLORA_ERR_NULL;
    for (int p = 0; p < P; ++p) {
      st = check_grad_tables(ps[p], dA[p], dB[p]);
      if (st != MLORA_OK) return st;
    }
  }
  if (workspace == nullptr || workspace_bytes < mlora_lora_group_workspace_bytes(ps, P)) return MLORA_ERR_WORKSPACE;
  if (ps[0]->T == 0 && accumulate) return MLORA_OK;

  CallCtx c[MLORA_MAX_GROUP];
  void* G[MLORA_MAX_GROUP];
  char* w = static_cast<char*>(workspace);
  bool sum_kernel = dX != nullptr && aligned16(dX);
  for (int p = 0; p < P; ++p) {
    fill_ctx(ps[p], hip_stream, &c[p]);
    G[p] = w;
    w += lowrank_bytes(ps[p]);
    sum_kernel = sum_kernel && mfma_gemm_applies(ps[p]) && aligned16(dY[p]) && aligned16(G[p]);
  }
  bool fused = ps[0]->K > 0 && group_lowrank_applies(ps, P, X);
  for (int p = 0; p < P; ++p) fused = fused && aligned16(dY[p]) && aligned16(saved[p]) && aligned16(G[p]);
  for (int p = 0; p < P; ++p) {
    float* partial = grad_scratch_bytes(ps[p]) ? reinterpret_cast<float*>(w) : nullptr;  // behind the last G_p
    hipError_t e = adapter_grads_impl(ps[p], c[p], X, dY[p], saved[p], G[p], ps[0]->K > 0 ? dA[p] : nullptr,
                                      ps[0]->K > 0 ? dB[p] : nullptr, accumulate, partial, fused);
    if (e != hipSuccess) return hip_status(e);
  }
  if (fused) {
    // every dA_pk in one pass over X
    OutTable ta[MLORA_MAX_GROUP];
    LowrankGroupItem it[MLORA_MAX_GROUP];
    for (int p = 0; p < P; ++p) {
      for (int k = 0; k < kMaxK; ++k) ta[p].p[k] = k < ps[p]->K ? dA[p][k] : nullptr;
      it[p] = LowrankGroupItem{c[p].ldz, c[p].st.rank, c[p].st.s, &c[p].A, nullptr, (const bf16*)G[p], &ta[p]};
    }
    hipError_t e = grad_mfma_group(P, it, c[0].st, (const bf16*)X, c[0].h, c[0].T, accumulate ? 1 : 0, c[0].stream);
    if (e != hipSuccess) return hip_status(e);
  }
  if (dX == nullptr || ps[0]->T == 0) return MLORA_OK;
  hipError_t e = hipSuccess;
  if (sum_kernel) {
    // one kernel: the P products accumulate in fp32 in the same output tile, dX is written once
    GemmOperands ops[MLORA_MAX_GROUP];
    for (int p = 0; p < P; ++p) {
      ops[p].A = (const bf16*)dY[p];
      ops[p].Bm = (const bf16*)ps[p]->W;
      ops[p].L = (const bf16*)G[p];
      ops[p].Kd = c[p].d;
      ops[p].ldz = c[p].ldz;
      ops[p].rank = c[p].st.rank;
      ops[p].R = &c[p].A;
    }
    e = gemm_mfma_sum_nt(P, ops, (bf16*)dX, c[0].T, c[0].h, c[0].st, c[0].stream);
  } else {
    for (int p = 0; p < P && e == hipSuccess; ++p) e = generic_gemm_bwd(c[p], dY[p], dX, G[p], p > 0 ? 1 : 0);
  }
  return hip_status(e);
}

const char* mlora_status_string(mlora_status s) {
  switch (s) {
    case MLORA_OK: return "ok";
    case MLORA_ERR_NULL: return "a required pointer is NULL";
    case MLORA_ERR_SHAPE: return "bad shape (T, h, d or K out of range)";
    case MLORA_ERR_SEGMENTS: return "segment offsets not monotone within [0, T]";
    case MLORA_ERR_RANK: return "adapter rank out of range";
    case MLORA_ERR_DTYPE: return "unknown dtype";
    case MLORA_ERR_WORKSPACE: return "workspace missing or too small";
    case MLORA_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

int mlora_last_hip_error(void) { return g_last_hip_error; }

int mlora_lora_kernel_path(const mlora_problem* p) {
  if (validate(p) != MLORA_OK) return -1;
  return (mfma_gemm_applies(p) ? 0 : 1) | (mfma_lowrank_applies(p) ? 0 : 2);
}

int mlora_set_kernel_path(int path) { return g_kernel_path.exchange(path); }

int mlora_profile_kernels(int enable) { return profile_enable(enable); }

mlora_status mlora_profile_kernels_read(double* ms_total, double* units_total, int* launches) {
  double ms[kProfileKinds], un[kProfileKinds];
  int n[kProfileKinds];
  const hipError_t e = profile_read(ms, un, n);
  if (e != hipSuccess) return hip_status(e);
  for (int k = 0; k < kProfileKinds; ++k) {
    if (ms_total) ms_total[k] = ms[k];
    if (units_total) units_total[k] = un[k];
    if (launches) launches[k] = n[k];
  }
  return MLORA_OK;
}

}  // extern "C"
