/*
 * mlora.h -- C ABI of the MI355X (gfx950) BatchLoRA multi-adapter LoRA linear operator.
 *
 * The operator is the "BatchLoRA" training operator of the mLoRA paper
 * (arXiv 2312.02515, section 3.3.1).  K independent LoRA fine-tuning tasks share
 * one frozen weight W; their token matrices x_k are concatenated row-wise into
 * X = (x_1^T ... x_K^T)^T, and
 *
 *   forward   (Eq. "forward"):      Y  = X W + rows_k( s_k x_k A_k B_k )
 *   backward  (Eq. "grad_lora"):    dA_k = s_k x_k^T dy_k B_k^T
 *                                   dB_k = s_k A_k^T x_k^T dy_k
 *             (Eq. "grad_output"):  dX = dY W^T + rows_k( s_k dy_k B_k^T A_k^T )
 *
 * W receives no gradient (section 3.3.1).  The base products X W and dY W^T are
 * launched once over the consolidated rows; the per-task LoRA terms are added at
 * the rows recorded by the split positions `seg_offsets`, and dX is written once
 * with the LoRA part already in it (the paper's "graph pruning": no zero-padded
 * full-size intermediate exists).  The factor s_k (= alpha_k / r_k, computed by
 * the caller) is this library's reading of the LoRA scaling, which the paper's
 * equations leave out; s_k = 1 gives the paper's formulas verbatim.
 *
 * Shapes follow the paper's notation (Eq. 1):  W is [h, d] (h input features,
 * d output features, Y = X W), A_k is [h, r_k], B_k is [r_k, d].  Every matrix is
 * dense row-major with no padding between rows.
 *
 * Memory: the entry points declared in this header own nothing and allocate
 * nothing, on the host or on the device.  Every pointer marked
 * DEVICE is GPU memory allocated by the caller on the current HIP device; every
 * pointer marked HOST is ordinary host memory that is read before the call
 * returns (the caller may free or reuse it on return).  All work is enqueued on
 * `hip_stream` (a hipStream_t passed as void*; NULL = the default stream) and
 * the calls return without waiting for it.  (The test and measurement switches
 * of mlora_testing.h are not part of this contract: the timing aid there creates
 * HIP events.)
 *
 * Errors: every call validates its arguments first and returns a status; on any
 * status other than MLORA_OK no kernel has been launched and no output has been
 * touched (MLORA_ERR_HIP excepted: a launch failed midway).  Nothing aborts and
 * no exception crosses this boundary.
 */
#ifndef MLORA_H
#define MLORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MLORA_MAX_ADAPTERS 64   /* K <= 64 per call */
#define MLORA_MAX_RANK     128  /* 1 <= r_k <= 128  */

typedef enum {
  MLORA_OK            = 0,
  MLORA_ERR_NULL      = 1,  /* a required pointer is NULL                                   */
  MLORA_ERR_SHAPE     = 2,  /* T, h or d negative, h or d zero, K out of range, sizes too big
                              (T >= 2^31 - 1024, h or d > 2^22, 2^31 or more 256 x 256 tiles) */
  MLORA_ERR_SEGMENTS  = 3,  /* seg_offsets not monotone or outside [0, T]                   */
  MLORA_ERR_RANK      = 4,  /* a rank outside [1, MLORA_MAX_RANK]                           */
  MLORA_ERR_DTYPE     = 5,  /* dtype is not one of mlora_dtype                              */
  MLORA_ERR_WORKSPACE = 6,  /* workspace pointer NULL or workspace_bytes too small          */
  MLORA_ERR_HIP       = 7   /* the HIP runtime reported an error (see mlora_last_hip_error) */
} mlora_status;

typedef enum {
  MLORA_BF16 = 0,  /* X, W, A_k, B_k, dY, Y, dX stored as bfloat16; products accumulate in fp32 */
  MLORA_F32  = 1   /* everything stored and accumulated in fp32                                */
} mlora_dtype;

/* One problem instance: the tasks T_1..T_K of section 3.3.1 over one shared W. */
typedef struct {
  int64_t T;                  /* total tokens (rows of X, Y, dY, dX); 0 is allowed (no-op)       */
  int64_t h;                  /* input features  (columns of X, rows of W)                       */
  int64_t d;                  /* output features (columns of W and Y)                            */
  int32_t K;                  /* number of adapters, 0 <= K <= MLORA_MAX_ADAPTERS                */
  int32_t dtype;              /* an mlora_dtype: element type of X, W, A_k, B_k, dY, Y, dX        */
  const int64_t* seg_offsets; /* HOST, K+1 entries, 0 <= o_0 <= ... <= o_K <= T.  Task k owns rows
                                 [o_k, o_{k+1}); an empty range is allowed.  Rows before o_0 and
                                 from o_K on belong to no task and get the base term only.  May be
                                 NULL when K == 0.                                               */
  const int32_t* ranks;       /* HOST, K entries, r_k                                            */
  const float*   scalings;    /* HOST, K entries, s_k                                            */
  const void* const* A;       /* HOST array of K DEVICE pointers, A_k is [h, r_k]                */
  const void* const* B;       /* HOST array of K DEVICE pointers, B_k is [r_k, d]                */
  const void* W;              /* DEVICE, [h, d], frozen: never written                           */
} mlora_problem;

/* Size in bytes of the `saved` buffer that mlora_lora_fwd fills and mlora_lora_bwd reads
 * (the intermediate s_k x_k A_k of the forward workflow, section 3.3.1, kept so that the
 * backward pass does not recompute it).  Its layout is private to the library.
 * Returns 0 if the problem is invalid; p->W is not looked at (it may be NULL, as in the
 * problems of the 8-bit-weight calls below). */
size_t mlora_lora_saved_bytes(const mlora_problem* p);

/* Size in bytes of the scratch `workspace` either call needs (the larger of the two).
 * Depends on the sizes in `p` only (T, h, d, dtype, split positions, ranks), never on the
 * addresses it holds.  The workspace carries nothing from one call to the next.
 * Returns 0 if invalid. */
size_t mlora_lora_workspace_bytes(const mlora_problem* p);

/* Argument check only (no GPU needed): the status mlora_lora_fwd would return for `p`
 * before looking at its other arguments. */
mlora_status mlora_lora_validate(const mlora_problem* p);

/* Forward, Eq. "forward":  Y[i,:] = X[i,:] W + s_k (X[i,:] A_k) B_k  for i in task k's rows.
 *   X          DEVICE [T, h]  input, read only
 *   Y          DEVICE [T, d]  output, fully overwritten; must not overlap any input
 *   saved      DEVICE, mlora_lora_saved_bytes(p) bytes, output
 *   workspace  DEVICE, at least mlora_lora_workspace_bytes(p) bytes, 256-byte aligned, scratch
 */
mlora_status mlora_lora_fwd(const mlora_problem* p, const void* X, void* Y, void* saved,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/* Backward, Eqs. "grad_lora" and "grad_output".
 *   X, dY      DEVICE [T, h] / [T, d]  inputs, read only
 *   saved      DEVICE, what mlora_lora_fwd wrote for the same problem and the same X, A_k, s_k
 *   dX         DEVICE [T, h] output, fully overwritten, written once with the LoRA term
 *              included; NULL skips it (first layer of a model)
 *   dA, dB     HOST arrays of K DEVICE pointers to fp32 buffers [h, r_k] and [r_k, d]
 *              (fp32 in both dtypes: they feed an optimiser or accumulate over micro-batches)
 *   accumulate 0: dA_k, dB_k are overwritten (zeros for an empty segment);
 *              1: the gradients are added to what the buffers hold
 * Two tasks must not share a dA or dB buffer.  W is read, never written.
 * With T == 0 the data pointers may be NULL; overwrite mode still zeroes dA_k, dB_k.
 */
mlora_status mlora_lora_bwd(const mlora_problem* p, const void* X, const void* dY, const void* saved,
                            void* dX, float* const* dA, float* const* dB, int accumulate,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/* mlora_lora_bwd for callers that cannot allocate device memory or carry a workspace pointer
 * (code under HIP graph capture set up elsewhere, tight serving-style loops, harnesses that
 * forbid hipMalloc): the scratch the backward needs lives in a fixed array of
 * MLORA_STATIC_SCRATCH_BYTES inside the library's device image instead of a caller's
 * workspace.  The call allocates nothing on the host or the device; arguments, results and
 * errors are those of mlora_lora_bwd without `workspace`, and the results are bit-identical
 * to it.  A problem whose mlora_lora_workspace_bytes(p) exceeds MLORA_STATIC_SCRATCH_BYTES is
 * refused with MLORA_ERR_WORKSPACE before anything is launched.  Every GPU the library runs on
 * holds its own copy of the array until the process ends; its address is looked up on the first
 * call on each device.  All calls on one GPU share that array: two calls that may overlap in
 * time (different streams, different threads) race -- use mlora_lora_bwd with separate
 * workspaces there. */
#define MLORA_STATIC_SCRATCH_BYTES (32u << 20)
mlora_status mlora_lora_bwd_static(const mlora_problem* p, const void* X, const void* dY, const void* saved,
                                   void* dX, float* const* dA, float* const* dB, int accumulate,
                                   void* hip_stream);

/* Activation-recompute variant of the pair above, for training runs that checkpoint activations
 * (the single-GPU setup of section 4.1 does): nothing is kept between the two calls; the
 * backward call recomputes s_k x_k A_k from X (one more pass over X, 2 t_k h r_k flops per task)
 * instead of reading a `saved` buffer.  Results are bit-identical to mlora_lora_fwd /
 * mlora_lora_bwd on the same inputs.  Both calls take a workspace of at least
 * mlora_lora_recompute_workspace_bytes(p) bytes (0 if the problem is invalid), 256-byte
 * aligned, scratch; every other argument is as in mlora_lora_fwd / mlora_lora_bwd. */
size_t mlora_lora_recompute_workspace_bytes(const mlora_problem* p);
mlora_status mlora_lora_fwd_nosave(const mlora_problem* p, const void* X, void* Y,
                                   void* workspace, size_t workspace_bytes, void* hip_stream);
mlora_status mlora_lora_bwd_recompute(const mlora_problem* p, const void* X, const void* dY,
                                      void* dX, float* const* dA, float* const* dB, int accumulate,
                                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---- Projections that share their input -------------------------------------------------
 * Section 4.1 puts adapters on q_proj, k_proj, v_proj and o_proj of every layer; q, k and v
 * (and gate, up of an MLP) read the same X.  A group is P problems, 1 <= P <= MLORA_MAX_GROUP,
 * with the same T, h, K, dtype and split positions; d, W and the adapters (ranks, scalings,
 * A_k, B_k) are each projection's own.  The forward outputs are Eq. "forward" per projection;
 * the backward writes ONE dX, the sum over the projections of Eq. "grad_output", accumulated
 * in fp32 and rounded once (on the MFMA path; the generic path adds projection by projection
 * in the storage type), and Eq. "grad_lora" per projection.
 *   ps         HOST array of P pointers to problems
 *   Y, saved   HOST arrays of P DEVICE pointers: Y[p] is [T, d_p]; saved[p] has
 *              mlora_lora_saved_bytes(ps[p]) bytes
 *   dY         HOST array of P DEVICE pointers, dY[p] is [T, d_p]
 *   dA, dB     HOST arrays of P HOST arrays of K DEVICE pointers (as in mlora_lora_bwd)
 *   workspace  DEVICE, at least mlora_lora_group_workspace_bytes(ps, P) bytes, 256-byte aligned
 * Errors as for the single calls; a mismatch between the problems of a group reports
 * MLORA_ERR_SHAPE (P, T, h, K), MLORA_ERR_DTYPE or MLORA_ERR_SEGMENTS. */
#define MLORA_MAX_GROUP 4
mlora_status mlora_lora_group_validate(const mlora_problem* const* ps, int P);
size_t mlora_lora_group_workspace_bytes(const mlora_problem* const* ps, int P);
mlora_status mlora_lora_group_fwd(const mlora_problem* const* ps, int P, const void* X, void* const* Y,
                                  void* const* saved, void* workspace, size_t workspace_bytes,
                                  void* hip_stream);
mlora_status mlora_lora_group_bwd(const mlora_problem* const* ps, int P, const void* X,
                                  const void* const* dY, const void* const* saved, void* dX,
                                  float* const* const* dA, float* const* const* dB, int accumulate,
                                  void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---- 8-bit frozen base weight ------------------------------------------------------------
 * The single-GPU setup of section 4.1 keeps the frozen pre-trained weights in 8 bits.  The
 * paper names the technique without a format; this library's reading is the weight-only,
 * column-wise absmax code (one fp32 scale per output feature):
 *     c[j]     = max_i |W[i,j]| / 127                  fp32 division
 *     Wq[i,j]  = rint( W[i,j] / c[j] )  in [-127,127]   fp32 division, halves to even;
 *                                                       0 where c[j] = 0
 *     W^[i,j]  = Wq[i,j] * c[j]
 * and W^ takes the place of W in Eq. "forward" and Eq. "grad_output" (Eq. "grad_lora" does not
 * contain W).  Activations, adapters, gradients and all products keep the problem's dtype; the
 * kernels read W^ in that dtype: the fp32 product Wq[i,j] * c[j], rounded to the nearest-even
 * bfloat16 for MLORA_BF16.  W must be finite.
 *   Wq   DEVICE int8  [h, d], row-major like W
 *   c    DEVICE float [d]
 *
 * mlora_w8_quantize: codes W (DEVICE [h, d] of `dtype`, read only) into Wq and c (outputs).
 * mlora_w8_dequantize: writes W^ into W_hat (DEVICE [h, d] of `dtype`, output).
 * Both: MLORA_ERR_NULL / MLORA_ERR_DTYPE / MLORA_ERR_SHAPE (h or d not in [1, 2^22]).
 *
 * mlora_lora_fwd_w8 / mlora_lora_bwd_w8: mlora_lora_fwd / mlora_lora_bwd with the weight given
 * as (Wq, c); p->W is ignored (may be NULL).  Each call first decodes W^ into its workspace
 * (one streaming pass, 1 byte read and one element written per weight) and then runs the same
 * kernels as the plain calls, so its results are bit-identical to the plain calls on
 * mlora_w8_dequantize's output; nothing decoded is kept between calls (a backward call with
 * dX == NULL decodes nothing).  `saved` is interchangeable with the plain calls' (it does not
 * depend on W).  The workspace must hold mlora_lora_w8_workspace_bytes(p) bytes (the plain
 * workspace plus h * d elements; 0 if the problem is invalid), 256-byte aligned.  Errors as for
 * the plain calls, MLORA_ERR_NULL also for a NULL Wq or c. */
mlora_status mlora_w8_quantize(const void* W, int32_t dtype, int64_t h, int64_t d, int8_t* Wq, float* c,
                               void* hip_stream);
mlora_status mlora_w8_dequantize(const int8_t* Wq, const float* c, int32_t dtype, int64_t h, int64_t d,
                                 void* W_hat, void* hip_stream);
size_t mlora_lora_w8_workspace_bytes(const mlora_problem* p);
mlora_status mlora_lora_fwd_w8(const mlora_problem* p, const int8_t* Wq, const float* c, const void* X, void* Y,
                               void* saved, void* workspace, size_t workspace_bytes, void* hip_stream);
mlora_status mlora_lora_bwd_w8(const mlora_problem* p, const int8_t* Wq, const float* c, const void* X,
                               const void* dY, const void* saved, void* dX, float* const* dA, float* const* dB,
                               int accumulate, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Plain text for a status code; never NULL. */
const char* mlora_status_string(mlora_status s);

/* hipError_t (as int) of the last HIP failure seen by this thread's calls; 0 if none. */
int mlora_last_hip_error(void);

/* Which kernels the calls will run for `p` (bit mask), so that a caller can tell the fast path
 * from the fallback before it launches anything:
 *   0      bf16 MFMA kernels everywhere,
 *   bit 0  the two base products run the generic (plain vector ALU, roughly 100 times slower)
 *          kernels,
 *   bit 1  the low-rank products run the generic kernels (3 = generic everywhere).
 * The MFMA kernels take bf16 problems whose h and d are multiples of 64, whose ranks are
 * multiples of 8 and whose W, A_k, B_k are 16-byte aligned; the answer assumes that the buffers
 * passed to the calls (X, Y, dY, dX, saved, workspace) are 16-byte aligned too, as device
 * allocations are -- a call handed a misaligned buffer falls back for that call.  Returns -1 if
 * the problem is invalid.  Honours mlora_set_kernel_path (mlora_testing.h). */
int mlora_lora_kernel_path(const mlora_problem* p);

#ifdef __cplusplus
}
#endif
#endif /* MLORA_H */
