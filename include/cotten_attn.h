/*
 * cotten_attn.h -- C ABI of the MI355X (gfx950) cosine-similarity attention library.
 *
 * The operation (Cotten4Rec, section "Model Description"): for every head-slice
 * (b,h) with per-head matrices Q, K, V of N rows and d_h columns,
 *
 *     xhat   = x / sqrt(sum_c x_c^2 + eps)        row-wise, for rows of Q and of K
 *                                                 (section "Cosine Similarity and
 *                                                  CUDA Kernel": eps inside the root)
 *     S      = sum_j m_j khat_j^T v_j             d_h x d_h state of the reordered
 *                                                 CosineAttention  Qhat (Khat^T V)
 *     O_i    = scale * qhat_i S                   scale = the scalar normaliser
 *                                                 1/n^m of the scaled CosineAttention
 *
 * m_j in {0,1} is a key-padding mask (1 = valid key).  The mask acts on keys
 * only: O and dQ are produced for all N query rows, and dO of every row flows
 * into the gradients.  The backward entry point returns the exact gradients of
 * the expression above,
 *
 *     dS   = scale * sum_i qhat_i^T dO_i
 *     dQ_i = (g_i - qhat_i (qhat_i . g_i)) / r(q_i),   g_i = scale * dO_i S^T
 *     dV_j = m_j * khat_j dS
 *     dK_j = m_j * (h_j - khat_j (khat_j . h_j)) / r(k_j),   h_j = v_j dS^T
 *
 * with r(x) = sqrt(sum_c x_c^2 + eps); dK and dV rows of masked keys are written
 * as exact zeros.  If a batch row has no valid key, O = 0 for it.
 *
 * Learnable normaliser (the scaled CosineAttention, scale = 1/n^m with a learnable
 * exponent).  Instead of one scalar the caller may pass one scale per slice,
 * params->slice_scale[b*H+h], and ask the backward for
 *
 *     dlog_scale[b*H+h] = d loss / d log(scale_bh) = sum_i dO_i . O_i  (= <S, dS>)
 *
 * which costs the kernels nothing extra in memory traffic.  cotten_normaliser_fwd
 * fills slice_scale from one exponent per head and one n per sequence,
 * scale_bh = n_b^(-m_h), and cotten_normaliser_bwd reduces dlog_scale to the
 * gradient of the exponents, dm_h = -sum_b ln(n_b) * dlog_scale[b*H+h].
 *
 * Memory.  Every pointer is a DEVICE pointer owned by the caller.  Q, K, V, O,
 * dO, dQ, dK, dV are [B, H, N, d_h] row-major and contiguous (each slice (b,h) is
 * one contiguous N x d_h block) or, with params->layout = COTTEN_BNHD, [B, N, H, d_h]
 * (the layout of the per-head split of a d_model-wide projection: no transposes
 * around the call); element type given by `dtype`; mask is [B, N]
 * bytes shared by the H heads, or NULL for "every key valid".  Tensor base
 * pointers must be 16-byte aligned.  Outputs must not overlap inputs or each
 * other.  Masked K/V rows are never dereferenced into arithmetic: they may hold
 * anything, NaN and Inf included.
 *
 * Arithmetic.  Row norms, the state and every accumulation are fp32 whatever
 * the I/O type (the paper keeps norms and partial sums in float32 under 16-bit
 * I/O).  Results are deterministic: reductions use a fixed order, no float
 * atomics, so two calls on the same inputs give identical bits.
 *
 * Execution.  Calls only enqueue kernels on `stream` (a hipStream_t passed as
 * void*; NULL = the default stream) and return; they never synchronise.  The
 * library runs on the device that is current in the calling thread.
 *
 * Workspace.  Long sequences are split over several workgroups per slice; the
 * partial d_h x d_h states travel through a workspace of
 * cotten_attn_workspace_bytes(...) bytes (0 when a shape needs none: every
 * sequence of at most 256 rows, and longer ones when B*H fills the device).  The
 * library never allocates, frees or synchronises: the caller brings the
 * workspace through cotten_params (its contents need no initialisation and mean
 * nothing afterwards; calls that share one must be ordered on one stream).  A
 * call whose shape needs a workspace and has none - params->workspace NULL, or
 * one of the plain entry points, which carry no params - returns
 * COTTEN_ERR_WORKSPACE_TOO_SMALL and enqueues nothing.
 *
 * Errors.  Every entry point returns a cotten_status; 0 is success, negative
 * values are listed below.  Argument validation happens on the host before any
 * device work and never touches the GPU, so a failed call has enqueued nothing.
 */
#ifndef COTTEN_ATTN_H_
#define COTTEN_ATTN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum cotten_dtype {
  COTTEN_F32 = 0,  /* float I/O                                   */
  COTTEN_BF16 = 1, /* bfloat16 I/O, fp32 norms and accumulation   */
  COTTEN_F16 = 2   /* IEEE half I/O, fp32 norms and accumulation (the mixed-precision mode
                      the paper trains in).  Results beyond +-65504 become Inf; the state
                      scale*S handed to the matrix cores is held in half as well, so
                      |scale * S| must stay in range (it does for scale ~ 1/N)           */
} cotten_dtype;

typedef enum cotten_layout {
  COTTEN_BHND = 0, /* [B, H, N, d_h]: every slice (b,h) is one contiguous block (default)   */
  COTTEN_BNHD = 1  /* [B, N, H, d_h]: what the Q/K/V projections of a transformer layer
                      write and what its output projection reads; the d_h elements of a
                      row stay contiguous, the rows of a slice are H*d_h elements apart   */
} cotten_layout;

typedef enum cotten_feature_map {
  COTTEN_MAP_COSINE = 0, /* rows of Q and K divided by sqrt(sum_c x_c^2 + eps): the cosine
                            attention of the paper (default)                                */
  COTTEN_MAP_ELU1 = 1    /* ELU(x) + 1 element-wise on Q and K (x + 1 above zero, exp(x) below):
                            the linear-attention comparison model of the paper's section
                            "Linear Attention Models", on the same two products
                            O = scale * phi(Q) (phi(K)^T V) and their exact gradients.  No
                            normalising denominator (the section names none), eps unused.
                            Every supported element type and d_h; not with causal
                            (COTTEN_ERR_BAD_PARAM)                                          */
} cotten_feature_map;

typedef enum cotten_status {
  COTTEN_OK = 0,
  COTTEN_ERR_NULL_POINTER = -1,         /* a required tensor pointer is NULL            */
  COTTEN_ERR_BAD_SHAPE = -2,            /* B, H or N < 1, sizes overflow the launch, or
                                           params->layout is not a cotten_layout         */
  COTTEN_ERR_UNSUPPORTED_HEAD_DIM = -3, /* d_h not in {16, 32, 64, 128}                 */
  COTTEN_ERR_BAD_DTYPE = -4,            /* dtype is not a cotten_dtype                  */
  COTTEN_ERR_MISALIGNED = -5,           /* a tensor or workspace pointer not 16-B aligned */
  COTTEN_ERR_WORKSPACE_TOO_SMALL = -6,  /* the shape needs a workspace and params->workspace is
                                           NULL or params->workspace_bytes is too small  */
  COTTEN_ERR_BAD_PARAM = -7,            /* params->scale or params->eps is NaN or Inf, or
                                           an option combination that is not available   */
  COTTEN_ERR_LAUNCH = -8,               /* the HIP runtime refused a launch             */
  COTTEN_ERR_STATIC_SCRATCH = -9        /* cotten_attn_bwd_static only: the call needs more than
                                           COTTEN_STATIC_SCRATCH_BYTES of scratch, or the
                                           address of the scratch array could not be obtained */
} cotten_status;

typedef struct cotten_params {
  int dtype;              /* a cotten_dtype                                             */
  float scale;            /* scalar normaliser s; <= 0 selects the default 1/N          */
  float eps;              /* epsilon inside the square root; < 0 selects 1e-6; 0 allowed */
  void* workspace;        /* device buffer, 16-byte aligned; may be NULL when
                             cotten_attn_workspace_bytes() is 0 for the call            */
  size_t workspace_bytes; /* size of `workspace` (ignored when it is NULL)              */
  const float* slice_scale; /* device, [B*H] floats, or NULL.  When given, slice (b,h) uses
                               slice_scale[b*H+h] (finite, > 0) and `scale` is ignored      */
  float* dlog_scale;      /* backward only: device, [B*H] floats, or NULL.  When given it
                             receives sum_i dO_i . O_i of every slice (see above)          */
  int layout;             /* a cotten_layout: applies to Q, K, V, O, dO, dQ, dK and dV     */
  int causal;             /* 0: bidirectional (the paper's model).  1: row i attends only the
                             valid keys j <= i (the variant the paper's model leaves out, "no
                             causal mask"): O_i = scale * qhat_i sum_{j<=i} m_j khat_j^T v_j
                             and its exact gradients.  d_h in {16, 32, 64}; sequences of more
                             than 208 rows need the workspace that
                             cotten_attn_workspace_bytes_ex() reports; dlog_scale is not
                             available (COTTEN_ERR_BAD_PARAM)                              */
  float* saved_state;     /* device, [B*H, d_h, d_h] floats, 16-byte aligned, or NULL.  The state
                             S = sum_j m_j khat_j^T v_j of every slice (row a, column c; without
                             the scale), kept by the caller from the forward call to the
                             backward call of the same K, V, mask and eps, as the chain rule
                             allows (the backward needs S again, nothing else of the forward).
                             Forward: written when given.  Backward: when given, read instead
                             of rebuilding S from K and V (one pass over K, V less); results
                             agree with the rebuilding call to fp32 rounding of S.  The
                             kernels for rows of 256 bytes and more (fp32 d_h = 64, d_h = 128),
                             the 16-bit backward
                             for N <= 208 (its slice sits in LDS, rebuilding costs no memory
                             traffic) and a backward call that also asks for dlog_scale rebuild
                             S all the same; the causal variant has no such state and ignores
                             the field                                                     */
  int feature_map;        /* a cotten_feature_map: what is done to the rows of Q and K    */
} cotten_params;

/* Forward (reordered CosineAttention with scalar normaliser, "Model Description"):
 * O = scale * Qhat (Khat^T V) under the key mask.  fp32 I/O, scale = 1/N, eps = 1e-6.
 * Shapes for which cotten_attn_workspace_bytes() is not 0 need the _ex form. */
int cotten_attn_fwd(const void* Q, const void* K, const void* V, const uint8_t* mask,
                    void* O, int B, int H, int N, int d_h, void* stream);

/* Backward of the same expression: given dO writes dQ, dK, dV (formulas above).
 * fp32 I/O, scale = 1/N, eps = 1e-6.  The state S is rebuilt from K, V; nothing
 * saved by the forward call is needed (cotten_params.saved_state offers the other way).
 * Shapes for which cotten_attn_workspace_bytes() is not 0 need the _ex form. */
int cotten_attn_bwd(const void* Q, const void* K, const void* V, const uint8_t* mask,
                    const void* dO, void* dQ, void* dK, void* dV, int B, int H, int N,
                    int d_h, void* stream);

/* Same operations with explicit dtype, scale, eps and workspace.  `params` must not
 * be NULL. */
int cotten_attn_fwd_ex(const void* Q, const void* K, const void* V, const uint8_t* mask,
                       void* O, int B, int H, int N, int d_h, void* stream,
                       const cotten_params* params);
int cotten_attn_bwd_ex(const void* Q, const void* K, const void* V, const uint8_t* mask,
                       const void* dO, void* dQ, void* dK, void* dV, int B, int H, int N,
                       int d_h, void* stream, const cotten_params* params);

/* For callers that cannot allocate device memory and so cannot bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same
 * operation, arguments and results (bit for bit) as cotten_attn_bwd_ex, except that the
 * partial states of long sequences go through a scratch array that is part of the library
 * image (a file-scope __device__ array of COTTEN_STATIC_SCRATCH_BYTES bytes; every GPU the
 * library runs on holds its own copy until the process ends) instead of params->workspace,
 * which is ignored together with params->workspace_bytes.  The call allocates, frees and
 * synchronises nothing.  A call that needs more scratch than the array holds
 * (cotten_attn_workspace_bytes(..., is_bwd = 1) > COTTEN_STATIC_SCRATCH_BYTES) returns
 * COTTEN_ERR_STATIC_SCRATCH and enqueues nothing; 32 MiB covers, for instance, 64 slices of
 * 4096 rows at d_h = 64 (16 MiB) and every shape that needs no workspace at all.  All calls on
 * one GPU share that GPU's array, which keeps the last call's contents (every element a
 * call reads it has written before, so nothing needs clearing): calls on the same GPU must be
 * ordered on one stream; calls that overlap on one GPU race. */
#define COTTEN_STATIC_SCRATCH_BYTES (32u << 20)
int cotten_attn_bwd_static(const void* Q, const void* K, const void* V, const uint8_t* mask,
                           const void* dO, void* dQ, void* dK, void* dV, int B, int H, int N,
                           int d_h, void* stream, const cotten_params* params);

/* Learnable normaliser 1/n^m of the scaled CosineAttention ("Model Description"), one
 * exponent per head:  slice_scale[b*H+h] = n_b^(-m_h).  m: device, [H] floats.  n: device,
 * [B] int32 with n_b >= 1 (for instance the valid length of each sequence), or NULL for
 * n_b = N, the padded length.  slice_scale: device, [B*H] floats, written. */
int cotten_normaliser_fwd(const float* m, const int32_t* n, float* slice_scale, int B, int H,
                          int N, void* stream);

/* Gradient of the exponents from the backward call's dlog_scale:
 * dm[h] = -sum_b ln(n_b) * dlog_scale[b*H+h], summed in a fixed order.  dm: device, [H]
 * floats, written.  n as above. */
int cotten_normaliser_bwd(const float* dlog_scale, const int32_t* n, float* dm, int B, int H,
                          int N, void* stream);

/* Bytes of workspace the given call would use (pure host arithmetic; 0 for an
 * unsupported shape).  Grows like B*H*d_h^2 times the number of sequence splits,
 * never like N*d_h or N^2: the method keeps only the d_h x d_h state ("Memory and
 * Compute Complexity"). */
size_t cotten_attn_workspace_bytes(int B, int H, int N, int d_h, int dtype, int is_bwd);

/* The same for a call with these params (dtype, causal and feature_map are looked at): what
 * params->workspace must hold.  Differs from the function above for the causal variant, whose
 * sequences of more than 208 rows pass one d x d state per 208-row chunk and slice through the
 * workspace (two in the backward call).  0 for invalid arguments or params == NULL.  Host
 * only, no device work. */
size_t cotten_attn_workspace_bytes_ex(int B, int H, int N, int d_h, int is_bwd,
                                      const cotten_params* params);

/* Static, NUL-terminated description of a status code. */
const char* cotten_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* COTTEN_ATTN_H_ */
