/* hbp.h -- C ABI of the Highway-BP backward pass for one MI355X (gfx950).
 *
 * The library computes, for a residual stack
 *       x_{l+1} = lambda_l (.) x_l + block_l(x_l),          l = 0 .. L-1
 *       block_l(x) = W2_l . act( W1_l . norm(x)  [+ U . xin_l] )
 * (paper, Section "Notations and assumptions": f_i = r_i(x, g_i(x)) with
 * r(x, z) = lambda (.) x + z, so K_i = diag(lambda) and J_i is the block's
 * Jacobian), the state-gradient estimates w^k of Theorem 2 by k iterations of
 *   (i)  v_l = g_{l+1} J_{l+1} for every block at once   ("Parallel computation", step 1)
 *   (ii) g_l = (e_l + v_l) + lambda_l (.) g_{l+1}, a reverse scan along the
 *        residual path                                    ("Parallel computation", step 2)
 * then the parameter gradients dL/dtheta_l = g_{l+1} . d block_l / d theta_l
 * (sentence after Theorem 2), and exact sequential backpropagation for
 * comparison.  kind = HBP_MLP: one weight pair per block, states along depth
 * (HBP_TRANSFORMER: attention and MLP sub-blocks in turn).
 * kind = HBP_RNN: one weight set shared by all L = T blocks, states along time,
 * block l maps state l to state l+1 and consumes xin[l].
 *
 * Conventions
 *  - Every pointer in hbp_buffers is DEVICE memory owned by the caller,
 *    contiguous, 16-byte aligned, row-major with the channel index fastest.
 *    "S" below is the storage type desc.dtype (fp32, or bf16 rounded to
 *    nearest-even at every store); all accumulation is fp32; rinv, the
 *    parameter gradients and a per-channel lambda (HBP_LAMBDA_CHANNEL) are
 *    always fp32, a per-token lambda (HBP_LAMBDA_TOKEN) is in S.  bf16 storage
 *    runs the contractions on the matrix cores (bf16 x bf16 -> fp32 MFMA); fp32
 *    storage runs them on the vector ALUs (an LDS-tiled FMA kernel, no fp32
 *    MFMA): that path is for small reference problems.
 *  - The library never allocates or frees device memory and never
 *    synchronises: kernels are enqueued on `stream` (a hipStream_t passed as
 *    void*; NULL = the default stream) and the call returns at once.  The
 *    backward calls can therefore be recorded into a HIP graph by stream
 *    capture and replayed (with timing by hbp_profile_enable off).
 *  - Inputs are read-only, with one exception: for HBP_GATED and HBP_LSTM
 *    hbp_forward WRITES the residual coefficients through `lambda`.  g, the
 *    workspace and the outputs must not alias the inputs or each other.
 *  - Errors are return codes, found before anything is launched: bad enum or
 *    struct_size, non-positive size, d / d_ff / d_in not a multiple of 8,
 *    d > 4096 with HBP_NORM_RMS, k < 0, a required pointer that is NULL, a
 *    workspace smaller than hbp_workspace_size() reports.  A failed launch
 *    gives HBP_E_DEVICE.
 *  - State between calls: none that changes results.  The library keeps (a) a
 *    flag per kernel and device saying that the kernel's shared-memory limit
 *    has been raised (set on the first launch, idempotent, safe from several
 *    threads) and (b) the process-wide timing switch and event lists of
 *    hbp_profile_enable / hbp_profile_read (mutex-protected).  Calls may be made
 *    from several threads; two calls that share g or the workspace must be
 *    ordered by the caller, and with timing on, hbp_profile_read returns the
 *    launches of all threads together.
 */
#ifndef HBP_H
#define HBP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  HBP_OK = 0,
  HBP_E_INVALID_ARG = 1,  /* bad enum, size, k or struct_size */
  HBP_E_UNSUPPORTED = 2,  /* sizes the kernels cannot take (see above) */
  HBP_E_WORKSPACE = 3,    /* workspace missing or too small */
  HBP_E_NULL = 4,         /* a required pointer is NULL */
  HBP_E_DEVICE = 5        /* a HIP call or launch failed */
} hbp_status;

typedef enum { HBP_F32 = 0, HBP_BF16 = 1 } hbp_dtype;
/* HBP_GATED: a recurrent cell whose residual coefficient is a function of the state (the GRU row of the table
 * of layer decompositions, f(x) = a(x) (.) x + b(x) with r(x, z) = z1 (.) x + z2):
 *   u = sigmoid(W_u x + U_u xin), c = tanh(W_c x + U_c xin), x' = (1 - u) (.) x + u (.) c,
 * so K = diag(1 - u) per token and the block VJP is [g (.) (c - x) u (1 - u) | g (.) u (1 - c^2)] . [W_u; W_c].
 * Shapes: d = H, d_ff = 2H, W1 = [W_u; W_c] [2H,H], U = [U_u; U_c] [2H,d_in]; W2, dW2, dphi, y, rinv unused.
 * z holds [u | c] as [L,N,2H].  lambda_kind must be HBP_LAMBDA_TOKEN: hbp_forward WRITES lambda = 1 - u there
 * ([L,N,H], storage type) and the backward calls read it.  act = HBP_ACT_TANH, norm = HBP_NORM_NONE. */
/* HBP_LSTM: the LSTM row of the same table.  The state is x = [c | h] (cell and hidden part, d = 2H); with
 * [i, f, o, gg] = [sigmoid, sigmoid, sigmoid, tanh](W h + U xin): c' = f (.) c + i (.) gg, h' = o (.) tanh(c').
 * K = diag([f | 0]): only the cell part has a residual path; everything else, h' depending on c included, is J.
 * Shapes: d = 2H, d_ff = 4H, W1 = [W_i; W_f; W_o; W_g] [4H,H] (acts on h), U likewise [4H,d_in]; z holds the
 * gates [i | f | o | gg] as [L,N,4H]; lambda ([L,N,2H], HBP_LAMBDA_TOKEN) is WRITTEN by hbp_forward as [f | 0].
 * dW1 is [4H,H].  Other rules as for HBP_GATED. */
/* HBP_GRU: the standard GRU, reset gate included (the GRU row of the table; the cell of the paper's RNN experiments):
 *   z = sigmoid(W_z x + U_z xin), r = sigmoid(W_r x + U_r xin), n = tanh(W_n (r (.) x) + U_n xin), x' = (1 - z) (.) x + z (.) n.
 * K = diag(1 - z); the block VJP is elementwise -> product with W_n -> elementwise -> product with [W_z; W_r].
 * Shapes: d = H, d_ff = 3H, W1 = [W_z; W_r; W_n] [3H,H], U [3H,d_in]; z holds [z | r | n] as [L,N,3H]; lambda
 * ([L,N,H], HBP_LAMBDA_TOKEN) is WRITTEN by hbp_forward as 1 - z.  Other rules as for HBP_GATED (which is this cell with the
 * reset gate held open). */
/* HBP_TRANSFORMER: the pre-norm transformer of the appendix (GPT-2 paragraph), every layer split into its self-attention
 * and feed-forward sub-layers, so that L = 2 x layers (L even).  Block l even: multi-head self-attention on the normed
 * state, [q | k | v] = norm(x_l) Wqkv_j^T (j = l/2), per sequence and head softmax(q k^T / sqrt(dh)) v (causal = 1: a
 * query sees keys up to its own position), heads side by side, times Wo_j^T.  Block l odd: the MLP of HBP_MLP with
 * W1_j, W2_j.  The N tokens are N / seq_len sequences of seq_len consecutive rows; head h is columns h dh .. (h+1) dh
 * (dh = d / heads) of each third of a [q | k | v] row.  The block Jacobian of an attention sub-block couples the rows of
 * a sequence; K stays diag(lambda), so steps (ii) and w^0 are unchanged, and gamma applies as for HBP_MLP (the paper
 * uses gamma = 0.2 on this stack).  Shapes: W1 [L/2,d_ff,d], W2 [L/2,d,d_ff], Wqkv [L/2,3d,d], Wo [L/2,d,d]; z, dphi
 * [L/2,N,d_ff]; qkv [L/2,N,3d], attn_o [L/2,N,d] (the attention's output before Wo) and lse [L/2, N heads] are
 * written by hbp_forward and read by the backward calls; x, y, rinv, lambda, e, g are per state / block as for
 * HBP_MLP.  post = HBP_POST_NONE, or HBP_POST_RMS with norm = HBP_NORM_NONE (post-norm layers, the RoBERTa paragraph of the
 * appendix: use gamma around 0.8); d_in = 0; dh a multiple of 8 (bf16 with dh = 64 runs on the matrix cores, any other
 * case on plain kernels that need seq_len <= 8192). */
typedef enum { HBP_MLP = 0, HBP_RNN = 1, HBP_GATED = 2, HBP_LSTM = 3, HBP_GRU = 4, HBP_TRANSFORMER = 5 } hbp_kind;
/* GELU is the exact erf form a*Phi(a); IDENTITY makes blocks linear (tests). */
typedef enum { HBP_ACT_GELU_ERF = 0, HBP_ACT_TANH = 1, HBP_ACT_IDENTITY = 2 } hbp_act;
/* RMS: y = x / sqrt(mean_c(x^2) + eps), no gain. */
typedef enum { HBP_NORM_NONE = 0, HBP_NORM_RMS = 1 } hbp_norm;
/* ONE: lambda = 1 (buffers.lambda ignored). CHANNEL: fp32 [L, d], shared by all tokens.
 * TOKEN: storage type S, [L, N, d]: a diagonal K_l that depends on the data (e.g. gates computed from
 * a recurrent cell's input), given as data: the backward calls treat it as constant. */
typedef enum { HBP_LAMBDA_ONE = 0, HBP_LAMBDA_CHANNEL = 1, HBP_LAMBDA_TOKEN = 2 } hbp_lambda;
/* What the residual function applies after the sum (Section "Notations and assumptions": r need not be
 * linear; table of layer decompositions, the original ResNet's row): NONE: x_{l+1} = lambda_l (.) x_l + block_l(x_l).
 * RELU: x_{l+1} = ReLU(lambda_l (.) x_l + block_l(x_l)); with m_l = 1[the sum > 0], K_l = diag(m_l lambda_l) and
 * J_l = diag(m_l) . d block_l / dx.  The backward calls then keep every state gradient already taken through
 * its ReLU: g[l] = m_{l-1} (.) dL/dx_l for l >= 1 (the gradient with respect to the sum that made x_l, which is
 * what the block VJP and the parameter gradients start from), g[0] = dL/dx_0.  HBP_MLP with gamma = 0 only. */
typedef enum { HBP_POST_NONE = 0, HBP_POST_RELU = 1, HBP_POST_RMS = 2 } hbp_post;
/* RMS: the post-norm row of the same table, x_{l+1} = RMSnorm(lambda_l (.) x_l + block_l(x_l)) (no gain; the block has
 * no norm of its own: norm = HBP_NORM_NONE).  With rho_l = 1/rms of the sum (one number per token, written to rinv by
 * hbp_forward): K_l = diag(lambda_l rho_l), J_l = the layer's Jacobian minus K_l.  As with RELU the backward calls
 * keep g[l] (l >= 1) taken through the norm that made x_l: g[l] = rho_{l-1} (G_l - x_l mean(G_l (.) x_l)), the
 * gradient with respect to the sum; g[0] = dL/dx_0.  HBP_MLP or HBP_TRANSFORMER, lambda ONE or CHANNEL, d <= 4096 (2048 with
 * gamma > 0).
 * On deep post-norm stacks the plain split (gamma = 0) diverges with k, as the paper reports for transformers: use
 * gamma around 0.5 .. 0.8. */

typedef struct {
  uint32_t struct_size;      /* = sizeof(hbp_desc) */
  int32_t kind;              /* hbp_kind   */
  int32_t dtype;             /* hbp_dtype  */
  int32_t act;               /* hbp_act    */
  int32_t norm;              /* hbp_norm   */
  int32_t lambda_kind;       /* hbp_lambda */
  int32_t loss_every_state;  /* 0: e = dL/dx_L only, [N,d]; 1: e = [L+1,N,d], one row block per state */
  float eps;                 /* RMS norm epsilon */
  int64_t L;                 /* blocks (RNN: time steps T) */
  int64_t N;                 /* tokens (RNN: batch rows per step) */
  int64_t d;                 /* state width (RNN: hidden size) */
  int64_t d_ff;              /* inner width of a block (RNN: hidden size of the cell) */
  int64_t d_in;              /* RNN input width; 0 for HBP_MLP */
  float gamma;               /* 0 <= gamma <= 1: share of the residual connection counted with the block in
                              * hbp_backward (appendix, the decomposition with gamma): the iteration then runs on
                              * K' = (1 - gamma) K and J' = J + gamma K.  0: the plain method; 1: fixed-point
                              * iteration.  The exact gradient and the other calls do not depend on it. */
  int32_t post;              /* hbp_post */
  /* HBP_TRANSFORMER only (ignored otherwise) */
  int32_t heads;             /* attention heads; d % heads == 0 */
  int32_t causal;            /* 1: keys after the query are masked out; 0: every query sees the whole sequence */
  int64_t seq_len;           /* rows per sequence; N % seq_len == 0 */
} hbp_desc;

typedef struct {
  uint32_t struct_size;      /* = sizeof(hbp_buffers) */
  /* parameters (S).  MLP: W1[L,d_ff,d], W2[L,d,d_ff].  RNN: W1 = W_h[d_ff,d],
   * W2 = W_o[d,d_ff], U[d_ff,d_in]. */
  const void* W1;
  const void* W2;
  const void* U;
  void* lambda;              /* CHANNEL: fp32 [L,d]; TOKEN: S [L,N,d].  Row (block) l carries state l+1 to state l.
                              * Read-only for the library, except HBP_GATED / HBP_LSTM: written by hbp_forward. */
  /* forward state: written by hbp_forward, read by the backward calls. */
  void* x;                   /* S [L+1,N,d]  states x_0..x_L (x[0] is the input) */
  void* y;                   /* S [L,N,d]    norm(x_l); unused (may be NULL) with HBP_NORM_NONE, where x is read */
  float* rinv;               /* [L,N]        1/sqrt(mean(x_l^2)+eps); unused with HBP_NORM_NONE, except with
                              *               HBP_POST_RMS, where it holds 1/rms of the sum that made x_{l+1} */
  void* z;                   /* S [L,N,d_ff] act(a_l) */
  void* dphi;                /* S [L,N,d_ff] act'(a_l); unused with TANH (1 - z^2) and IDENTITY (1) */
  const void* xin;           /* S [L,N,d_in] RNN inputs; NULL for MLP */
  uint8_t* mask;             /* [L,N,d/8] HBP_POST_RELU only (else unused, may be NULL): bit j of byte c of row
                              * (l, n) is 1 where the sum that made x_{l+1}[n, 8c+j] was positive; written by
                              * hbp_forward, read by the backward calls */
  /* loss gradients and results */
  const void* e;             /* S [N,d] or [L+1,N,d] (see loss_every_state) */
  void* g;                   /* S [L+1,N,d]  out: state-gradient estimates, g[L] = e_L */
  float* dW1;                /* out, fp32, shape of W1 */
  float* dW2;                /* out, fp32, shape of W2 */
  float* dU;                 /* out, fp32, shape of U (RNN) */
  void* workspace;
  size_t workspace_bytes;
  /* HBP_TRANSFORMER only (ignored otherwise, may be NULL) */
  const void* Wqkv;          /* S [L/2,3d,d]  rows [W_q; W_k; W_v] */
  const void* Wo;            /* S [L/2,d,d] */
  void* qkv;                 /* S [L/2,N,3d]  forward state */
  void* attn_o;              /* S [L/2,N,d]   forward state: attention output before Wo */
  float* lse;                /* [L/2, N heads] forward state: per (sequence, head, position) the base-2 logarithm of
                              * sum_j exp2(s_j log2 e), s the scaled scores the query sees */
  float* dWqkv;              /* out, fp32, shape of Wqkv */
  float* dWo;                /* out, fp32, shape of Wo */
} hbp_buffers;

/* Bytes of workspace that any of the calls below may need for this problem. */
hbp_status hbp_workspace_size(const hbp_desc* desc, size_t* bytes);

/* Validates a descriptor (and, when bufs is not NULL, the pointers the backward
 * calls need) without touching the device. */
hbp_status hbp_check(const hbp_desc* desc, const hbp_buffers* bufs);

/* Runs the stack forward from x[0] and fills x[1..L], y, rinv, z, dphi (the cells: z and lambda; HBP_TRANSFORMER: also
 * qkv, attn_o, lse): the state the backward calls read.  Part of hbp_train_step; otherwise support. */
hbp_status hbp_forward(const hbp_desc* desc, hbp_buffers* bufs, void* stream);

/* g := w^k, the sum of all gradient paths through at most k block Jacobians
 * (Theorem 2; with desc->gamma > 0, of the re-split pair J + gamma K and
 * (1 - gamma) K).  k = 0 gives the residual-path-only estimate; k >= L is exact.
 * Reads W1, W2, lambda, y (or x), rinv, z, dphi, e (HBP_TRANSFORMER: also Wqkv, Wo, qkv, attn_o, lse); writes g and the
 * workspace. */
hbp_status hbp_backward(const hbp_desc* desc, int k, hbp_buffers* bufs, void* stream);

/* The initial estimate alone, g := w^0 = CumSumProd(e, K) (Theorem 2; K scaled by 1 - gamma), by a
 * named form of the scan: what hbp_backward picks (AUTO), the sequential walk down the chain, the
 * chunked reduce / combine / apply form (every element read twice), the single-pass form (chunks that
 * hand their state down the chain through a chained look-back: every element read once; bf16 storage
 * only), or the Hillis-Steele sweeps of the paper's Algorithm 1 (kept for comparison: O(L log L)
 * elements moved).  Same result up to rounding order; each form is bitwise repeatable.  The workspace must
 * hold hbp_scan_workspace_size(desc, algorithm) bytes (CHUNKED and HILLIS_STEELE need more than the
 * backward calls; AUTO and SEQUENTIAL need hbp_workspace_size()).  Reads e, lambda; writes g. */
typedef enum {
  HBP_SCAN_AUTO = 0, HBP_SCAN_SEQUENTIAL = 1, HBP_SCAN_CHUNKED = 2, HBP_SCAN_HILLIS_STEELE = 3,
  HBP_SCAN_SINGLE_PASS = 4
} hbp_scan_algorithm;
hbp_status hbp_scan_workspace_size(const hbp_desc* desc, int algorithm, size_t* bytes);
hbp_status hbp_initial_estimate(const hbp_desc* desc, int algorithm, hbp_buffers* bufs, void* stream);

/* For callers that cannot allocate device memory or bring a workspace (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): hbp_initial_estimate(desc, HBP_SCAN_CHUNKED, ...) with the chunked
 * scan's scratch in a fixed array inside the library instead of bufs->workspace (which is ignored and may be NULL).
 * Same kernels, same result bit for bit.  Calls no hipMalloc / hipFree or any allocating routine.  Limit:
 * 16 * ceil(L / 64) * N * d bytes of scratch must fit HBP_STATIC_SCRATCH_BYTES (32 MiB: T = 4096 steps of 32 x 1024
 * chains just fit); larger problems return HBP_E_WORKSPACE, a residual function with a ReLU or norm after the sum
 * HBP_E_UNSUPPORTED.  Every GPU the library runs on holds one such array until the process ends, and every call on
 * a GPU shares it: it keeps the previous call's contents (each call writes what it reads, nothing needs clearing),
 * and two calls that overlap on one GPU (different streams or threads) race on it: the caller must order them. */
#define HBP_STATIC_SCRATCH_BYTES (32u << 20)
hbp_status hbp_initial_estimate_static(const hbp_desc* desc, hbp_buffers* bufs, void* stream);

/* g := the exact gradient by L sequential block steps, G_L = e_L,
 * G_l = e_l + lambda_l (.) G_{l+1} + G_{l+1} J_{l+1}: the chain rule through J + K that Section
 * "Backpropagation as a system of equations" writes as the system the method solves (first line of the proof
 * of Theorem 1).  The comparison baseline; same buffers as hbp_backward. */
hbp_status hbp_exact_backward(const hbp_desc* desc, hbp_buffers* bufs, void* stream);

/* The parameter gradients from the state-gradient estimate currently in bufs.g (sentence after Theorem 2:
 * dL/dtheta_l = w_{l+1} . d f_l / d theta_l, with the current estimate w^k in place of the exact gradient):
 * da_l = (g_{l+1} W2_l) (.) act'(a_l); dW2_l = sum_n g_{l+1}[n]^T z_l[n];
 * dW1_l = sum_n da_l[n]^T y_l[n]; dU = sum da^T xin; attention sub-blocks: dWo = sum_n g[n]^T o[n] and
 * dWqkv = sum_n d[q|k|v][n]^T y[n].  Shared weights sum over l too.  Long contractions over
 * tokens are computed in shares whose partial sums a second kernel adds in a fixed order (bitwise repeatable). */
hbp_status hbp_param_grads(const hbp_desc* desc, hbp_buffers* bufs, void* stream);

/* ---- the training step around the backward pass --------------------------------------------------------------
 * Section "Discussion and conclusion": the number of iterations is a knob that can be turned during training (few
 * iterations early, more later, exact backpropagation at the end); Section "Approximating backpropagation": a step
 * costs T_forward + (k / L) T_backward + O(k log L).  The calls below complete hbp_forward, hbp_backward /
 * hbp_exact_backward and hbp_param_grads into such a step: a stand-in loss, gradient clipping and the two
 * optimizers of the appendix "Training scheme" (SGD with momentum and weight decay; AdamW).  The schedule of k and
 * of the learning rate is the caller's loop. */
typedef enum { HBP_OPT_SGD = 0, HBP_OPT_ADAMW = 1 } hbp_opt_kind;
typedef struct {
  uint32_t struct_size;      /* = sizeof(hbp_optim) */
  int32_t kind;              /* hbp_opt_kind */
  float lr;
  float beta1;               /* SGD: the momentum; AdamW: beta1 */
  float beta2;               /* AdamW */
  float eps;                 /* AdamW */
  float weight_decay;        /* SGD: added to the gradient (L2); AdamW: decoupled */
  float clip_norm;           /* > 0: gradients scaled by min(1, clip_norm / (global L2 norm + 1e-6)); 0: off */
  int64_t step;              /* AdamW: number of this update, counted from 1 */
} hbp_optim;
typedef struct {
  uint32_t struct_size;      /* = sizeof(hbp_optim_state) */
  /* DEVICE, fp32, shapes of W1 / W2 / U (entries for weights the kind does not have are ignored).
   * master*: fp32 copies of the weights, updated and then rounded into W1 / W2 / U; may be NULL: the weights are
   * then kept in the storage type alone.  m*: momentum buffer (SGD) or first moment (AdamW); v*: second moment
   * (AdamW only).  The caller zeroes m and v before the first step and fills master with the weights. */
  float* master1; float* master2; float* masterU;
  float* m1; float* m2; float* mU;
  float* v1; float* v2; float* vU;
  float* scratch;            /* DEVICE, hbp_train_scratch_size() bytes: partial sums of the reductions */
  size_t scratch_bytes;
  /* HBP_TRANSFORMER only: the same for Wqkv and Wo */
  float* masterQ; float* masterO;
  float* mQ; float* mO;
  float* vQ; float* vO;
} hbp_optim_state;

hbp_status hbp_train_scratch_size(size_t* bytes);

/* The stand-in loss L = 1/(2N) sum |x - target|^2 over the last state (loss_every_state = 0: target [N,d]) or over
 * states 1..L (loss_every_state = 1: target [L+1,N,d], row 0 unused), N = desc->N: writes e_out = dL/dx in the
 * layout hbp_backward reads as bufs->e ([N,d] or [L+1,N,d] with e[0] = 0) and the loss value to loss_out[0] (DEVICE
 * float).  Reads bufs->x; scratch as in hbp_optim_state. */
hbp_status hbp_loss_mse(const hbp_desc* desc, const hbp_buffers* bufs, const void* target, void* e_out, float* loss_out,
                        float* scratch, size_t scratch_bytes, void* stream);

/* One optimizer update of W1, W2 (and U; Wqkv, Wo) from dW1, dW2 (and dU; dWqkv, dWo) in bufs. */
hbp_status hbp_optimizer_step(const hbp_desc* desc, hbp_buffers* bufs, const hbp_optim* opt, hbp_optim_state* state,
                              void* stream);

/* One training step: hbp_forward, hbp_loss_mse (writes bufs->e, which must be writable here), hbp_backward(k) or,
 * with k < 0, hbp_exact_backward, hbp_param_grads, hbp_optimizer_step. */
hbp_status hbp_train_step(const hbp_desc* desc, int k, hbp_buffers* bufs, const void* target, float* loss_out,
                          const hbp_optim* opt, hbp_optim_state* state, void* stream);

const char* hbp_status_string(hbp_status s);

/* Optional timing of the kernels the calls above enqueue, by class, with HIP
 * events recorded on the caller's stream around each launch (host-side objects
 * only; still no device allocation).  Off by default.  hbp_profile_read waits
 * for the recorded events, adds the elapsed milliseconds and launch counts per
 * class since the previous read into ms[HBP_PROF_CLASSES] and
 * launches[HBP_PROF_CLASSES] (both HOST arrays), and forgets them. */
enum {
  HBP_PROF_VJP1 = 0,    /* da = (g W2) (.) act'      (step (i), first contraction)  */
  HBP_PROF_VJP2 = 1,    /* dn = da W1                (step (i), second contraction) */
  HBP_PROF_SCAN = 2,    /* residual-path scan        (step (ii), and w^0)           */
  HBP_PROF_DW = 3,      /* parameter-gradient contractions over tokens              */
  HBP_PROF_FORWARD = 4, /* forward support kernels                                  */
  HBP_PROF_OTHER = 5,   /* copies, split-K reductions                               */
  HBP_PROF_ATTN = 6,    /* attention between its two matrices, forward and backward  */
  HBP_PROF_CLASSES = 7
};
hbp_status hbp_profile_enable(int on);
hbp_status hbp_profile_read(double* ms, int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* HBP_H */
