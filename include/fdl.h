/*
 * fdl -- fused dense-layer block for AMD MI355X (gfx950), C ABI.
 *
 *     Y = LayerNorm( GELU_erf( X W^T + b ) ) * gamma + beta          (forward)
 *     (dX, dW, db, dgamma, dbeta) for an upstream gradient dY         (backward)
 *
 * Operator conventions follow the paper's task definitions (appendix "Robust
 * Kernel Benchmark", linear backward task definition): the linear step is
 * torch's F.linear, y = x W^T + b with W stored [out_features, in_features];
 * the forward call keeps what backward needs; the backward call receives the
 * upstream gradient plus the saved tensors and returns the gradient of every
 * input.  A kernel counts as correct only if it reproduces the torch operator
 * (appendix "Kernel Evaluation Environment"), hence GELU is the exact erf form,
 * LayerNorm normalises over the last dimension with the biased variance, and
 * eps sits inside the square root.
 *
 * All pointers except where noted are DEVICE pointers owned by the caller.
 * Matrices are row-major and contiguous, with no padding between rows:
 *   X [M,K]   W [N,K]   Y, Zsave, dY [M,N]   dX [M,K]   dW [N,K]
 * and are stored in the type selected by `dt`.  Vectors b, gamma, beta, db,
 * dgamma, dbeta [N] and mean, rstd [M] are always fp32.  Every base pointer
 * (matrices and vectors) must be 16-byte aligned; row pitches need not be.
 *
 * The library allocates nothing and never synchronises: every call only
 * enqueues kernels on `hip_stream` (a hipStream_t passed as void*; NULL is the
 * default stream) and returns.  Scratch memory comes from the caller through
 * `workspace` (device memory, 256-byte aligned, at least
 * fdl_workspace_bytes(...) bytes, contents undefined before and after a call).
 * Outputs are overwritten, never accumulated into.  Input and output buffers
 * must not overlap.  Calls that share a workspace must be ordered on a stream.
 *
 * Errors are reported by return code; every argument check happens before any
 * device call, so a rejected call has touched nothing.  FDL_ERR_LAUNCH reports
 * a HIP launch error (hipGetLastError after the launches; the reason is printed
 * to stderr).  An accepted call first clears the calling thread's HIP last-error
 * state, so an error left behind by earlier, unrelated HIP calls is not reported.
 */
#ifndef FDL_H_
#define FDL_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The library is built with hidden symbol visibility; the entry points below are its only exports. */
#define FDL_API __attribute__((visibility("default")))

typedef enum {
  FDL_OK = 0,
  FDL_ERR_NULL = 1,       /* a required pointer is NULL                           */
  FDL_ERR_SHAPE = 2,      /* M, K or N < 1, or a product overflows the supported range */
  FDL_ERR_DTYPE = 3,      /* dt is not a member of fdl_dtype                      */
  FDL_ERR_EPS = 4,        /* eps is negative, NaN or infinite                     */
  FDL_ERR_WORKSPACE = 5,  /* workspace is NULL or smaller than fdl_workspace_bytes */
  FDL_ERR_ALIGN = 6,      /* a base pointer is not 16-byte aligned (workspace: 256) */
  FDL_ERR_LAUNCH = 7      /* HIP reported an error when launching                 */
} fdl_status;

typedef enum {
  FDL_F32 = 0,   /* matrices stored as fp32; contractions and reductions accumulate in fp64 */
  FDL_BF16 = 1   /* matrices stored as bf16; contractions and reductions accumulate in fp32 */
} fdl_dtype;

/* Human-readable name of a status code (host pointer to a static string). */
FDL_API const char* fdl_status_string(fdl_status s);

/*
 * Bytes of device scratch that fdl_forward and fdl_backward need for this
 * problem (the larger of the two, so one buffer serves both).  Returns 0 for
 * an invalid dtype or shape.  Host-only: touches no device.
 */
FDL_API size_t fdl_workspace_bytes(fdl_dtype dt, int64_t M, int64_t K, int64_t N);

/*
 * Forward:  Z = X W^T + b;  A = GELU_erf(Z) = Z * Phi(Z);
 *           mean_i = (1/N) sum_j A_ij;  var_i = (1/N) sum_j (A_ij - mean_i)^2;
 *           rstd_i = (var_i + eps)^(-1/2);
 *           Y_ij = (A_ij - mean_i) * rstd_i * gamma_j + beta_j.
 * (Linear step: linear task definition in the appendix "Robust Kernel
 * Benchmark"; LayerNorm as a two-step "row statistics, then normalise" pass:
 * appendix "Highlighted CUDA Kernels: Analysis", LayerNorm forward.)
 *
 * in : X [M,K], W [N,K] (dt);  b, gamma, beta [N] fp32;  eps >= 0.
 * out: Y [M,N] (dt);  Zsave [M,N] (dt) = Z rounded to dt, the pre-activation
 *      kept for backward;  mean, rstd [M] fp32 = row statistics of
 *      GELU_erf(Zsave) (i.e. of the stored, rounded pre-activation).
 */
FDL_API fdl_status fdl_forward(fdl_dtype dt, int64_t M, int64_t K, int64_t N,
                       const void* X, const void* W,
                       const float* b, const float* gamma, const float* beta, float eps,
                       void* Y, void* Zsave, float* mean, float* rstd,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * fdl_forward for callers that cannot allocate device memory or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and kernels as fdl_forward, but
 * the scratch is a fixed array of FDL_STATIC_SCRATCH_BYTES bytes inside the library's device code (one copy per
 * GPU, held from the moment the library is loaded there until the process ends).  The call allocates and frees
 * nothing; the first call on a GPU looks up the array's device address (a host-side query, no stream work).
 *
 * Limit: problems whose forward scratch exceeds the array are rejected with FDL_ERR_WORKSPACE before any device
 * call.  The forward scratch is 8 bytes per (row, column tile) of partial row statistics - none on the bf16 path
 * with K % 128 == 0, N % 256 == 0, N <= 8192, M >= 128, which normalises without partials - plus 512 K bytes when
 * that path sees a ragged M.  Every call on one GPU shares that GPU's array, so two calls that overlap in time on
 * one GPU (different streams, different host threads) race: order them on one stream or with events.
 */
#define FDL_STATIC_SCRATCH_BYTES (16 * 1024 * 1024)
FDL_API fdl_status fdl_forward_static(fdl_dtype dt, int64_t M, int64_t K, int64_t N,
                                      const void* X, const void* W,
                                      const float* b, const float* gamma, const float* beta, float eps,
                                      void* Y, void* Zsave, float* mean, float* rstd, void* hip_stream);

/*
 * Backward, given dY [M,N] and the tensors saved by fdl_forward:
 *   Ahat_ij = (GELU_erf(Z_ij) - mean_i) * rstd_i;     g_ij = dY_ij * gamma_j;
 *   c1_i = (1/N) sum_j g_ij;    c2_i = (1/N) sum_j g_ij * Ahat_ij;
 *   dA_ij = rstd_i * (g_ij - c1_i - Ahat_ij * c2_i);
 *   dZ_ij = dA_ij * (Phi(Z_ij) + Z_ij * phi(Z_ij));
 *   dbeta_j = sum_i dY_ij;   dgamma_j = sum_i dY_ij * Ahat_ij;   db_j = sum_i dZ_ij;
 *   dX = dZ W   [M,K];       dW = dZ^T X   [N,K].
 * (Gradient contract and the three linear-layer gradients: linear backward
 * task definition and the "MNIST Linear Backward Kernel" listing's operator;
 * recomputation of the activation from the saved pre-activation in backward:
 * "MNIST Linear-ReLU Backward Kernel".)
 *
 * in : dY [M,N], X [M,K], W [N,K], Zsave [M,N] (dt);  gamma [N], mean, rstd [M] fp32.
 * out: dX [M,K], dW [N,K] (dt);  db, dgamma, dbeta [N] fp32.
 */
FDL_API fdl_status fdl_backward(fdl_dtype dt, int64_t M, int64_t K, int64_t N,
                        const void* dY, const void* X, const void* W, const float* gamma,
                        const void* Zsave, const float* mean, const float* rstd,
                        void* dX, void* dW, float* db, float* dgamma, float* dbeta,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/* ----------------------------------------------------------------------------------------------------------------
 * Forward-only variant and sibling operators built on the same kernels.  Conventions as above: device pointers
 * owned by the caller, row-major contiguous matrices in the storage type `dt`, fp32 vectors, 16-byte aligned base
 * pointers, work enqueued on `hip_stream`, outputs overwritten, argument checks before any device call.
 * -------------------------------------------------------------------------------------------------------------- */

/*
 * Forward pass for inference (the paper's experiments are mostly forward kernels: section "Optimizing individual
 * operations", task table of the robust kernel benchmark): Y as fdl_forward computes it, and nothing saved for a
 * backward pass.  The pre-activation passes through Y itself and is normalised in place, so the workspace holds no
 * M x N tensor: row statistics, partial statistics where the contraction emits them, and for batches of 16384 rows
 * and more on the tuned bf16 kernels a transposed copy of W (2 N K bytes):
 * fdl_forward_inference_workspace_bytes bytes (0 for an invalid dtype or shape), 256-byte aligned.
 * in : X [M,K], W [N,K] (dt);  b, gamma, beta [N] fp32;  eps >= 0.     out: Y [M,N] (dt).
 */
FDL_API size_t fdl_forward_inference_workspace_bytes(fdl_dtype dt, int64_t M, int64_t K, int64_t N);
FDL_API fdl_status fdl_forward_inference(fdl_dtype dt, int64_t M, int64_t K, int64_t N,
                                         const void* X, const void* W,
                                         const float* b, const float* gamma, const float* beta, float eps,
                                         void* Y, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Linear + ReLU, forward and backward (appendix "Highlighted CUDA Kernels: Code": "MNIST Linear-ReLU" forward kernel
 * and "MNIST Linear-ReLU Backward Kernel"; task definition in the appendix "Robust Kernel Benchmark").
 *   forward :  Y = max(0, X W^T + b)
 *   backward:  the pre-activation Z = X W^T + b is recomputed from the inputs (only inputs are saved, as in the
 *              paper's task) and never stored;  G = dY where Z > 0, else 0 (the derivative at 0 is 0);
 *              dX = G W [M,K];  dW = G^T X [N,K];  db_j = sum_i G_ij.
 * in : X [M,K], W [N,K], dY [M,N] (dt);  b [N] fp32.     out: Y [M,N], dX [M,K], dW [N,K] (dt);  db [N] fp32.
 * One workspace size serves both calls (fdl_linear_relu_workspace_bytes; 0 for an invalid dtype or shape).
 * Where the exact pre-activation is within rounding of zero, the mask of that element is decided by the arithmetic
 * of the contraction (fp32 accumulation for bf16 storage, fp64 for fp32 storage).
 */
FDL_API size_t fdl_linear_relu_workspace_bytes(fdl_dtype dt, int64_t M, int64_t K, int64_t N);
FDL_API fdl_status fdl_linear_relu_forward(fdl_dtype dt, int64_t M, int64_t K, int64_t N,
                                           const void* X, const void* W, const float* b, void* Y,
                                           void* workspace, size_t workspace_bytes, void* hip_stream);
FDL_API fdl_status fdl_linear_relu_backward(fdl_dtype dt, int64_t M, int64_t K, int64_t N,
                                            const void* dY, const void* X, const void* W, const float* b,
                                            void* dX, void* dW, float* db,
                                            void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * LayerNorm forward over the last dimension (appendix "Highlighted CUDA Kernels: Analysis", Layernorm: row mean and
 * variance first, then normalise and apply the affine transform; torch semantics: biased variance, eps inside the
 * root):  Y_ij = (A_ij - mean_i) rstd_i gamma_j + beta_j.
 * in : A [M,N] (dt);  gamma, beta [N] fp32;  eps >= 0.     out: Y [M,N] (dt);  mean, rstd [M] fp32.
 * A and Y must not overlap.  No workspace.
 */
FDL_API fdl_status fdl_layernorm_forward(fdl_dtype dt, int64_t M, int64_t N,
                                         const void* A, const float* gamma, const float* beta, float eps,
                                         void* Y, float* mean, float* rstd, void* hip_stream);

/*
 * RMSNorm forward over the last dimension ("Llama RMSNorm Forward Kernel" listing):
 *   Y_ij = A_ij (mean_j A_ij^2 + eps)^(-1/2) weight_j.
 * in : A [M,N] (dt);  weight [N] fp32;  eps >= 0.     out: Y [M,N] (dt).  A and Y must not overlap.  No workspace.
 */
FDL_API fdl_status fdl_rmsnorm_forward(fdl_dtype dt, int64_t M, int64_t N,
                                       const void* A, const float* weight, float eps, void* Y, void* hip_stream);

/*
 * Llama feed-forward block, forward (task table of the robust kernel benchmark, Llama Feedforward; appendix
 * "Highlighted CUDA Kernels: Analysis", LlamaFFW: three matrix products and a fused SiLU-multiply, no biases):
 *   Y = ( SiLU(X Wg^T) * (X Wu^T) ) Wd^T,     SiLU(z) = z / (1 + exp(-z)).
 * in : X [M,D], Wg, Wu [H,D], Wd [D,H] (dt).     out: Y [M,D] (dt).
 * Workspace: fdl_llama_ffn_workspace_bytes bytes (the two M x H intermediates; 0 for an invalid dtype or shape).
 */
FDL_API size_t fdl_llama_ffn_workspace_bytes(fdl_dtype dt, int64_t M, int64_t D, int64_t H);
FDL_API fdl_status fdl_llama_ffn_forward(fdl_dtype dt, int64_t M, int64_t D, int64_t H,
                                         const void* X, const void* Wg, const void* Wu, const void* Wd, void* Y,
                                         void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Optional timing instrumentation (measurement protocol: the paper times kernels with warm-up runs
 * followed by many timed runs, appendix "Kernel Evaluation Environment"; this hook lets a harness time
 * each phase of a call with HIP events on the call's own stream).
 *
 * Phases: forward = F1 (GEMM + fused epilogue), FS (statistics merge), F2 (normalise);
 *         backward = B1 (row pass), B2 (column reduce), B3 (dX GEMM), B4 (dW GEMM).
 * `events` is a HOST array of 2*FDL_PHASE_COUNT hipEvent_t handles created by the caller (or NULL to switch
 * the instrumentation off, the default).  While set, fdl_forward / fdl_backward record events[2*p] just
 * before and events[2*p+1] just after the launches of phase p on the call's stream.  The array is copied;
 * the events stay owned by the caller.  This is a measurement hook, not part of the operator's contract: it is
 * process-wide state that changes what the other entry points enqueue, it is not thread-safe, and it must not be
 * switched while another thread is inside the library.  Benchmarks only.
 * Returns FDL_ERR_SHAPE if count != 2*FDL_PHASE_COUNT (and events != NULL).
 */
typedef enum {
  FDL_PHASE_F1 = 0, FDL_PHASE_FS = 1, FDL_PHASE_F2 = 2,
  FDL_PHASE_B1 = 3, FDL_PHASE_B2 = 4, FDL_PHASE_B3 = 5, FDL_PHASE_B4 = 6,
  FDL_PHASE_COUNT = 7
} fdl_phase;

FDL_API fdl_status fdl_set_phase_events(void* const* events, int count);

#ifdef __cplusplus
}
#endif
#endif /* FDL_H_ */
