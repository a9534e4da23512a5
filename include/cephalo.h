/*
 * cephalo.h -- C ABI of the MI355X (gfx950) library for one GPU's share of a sharded
 * data-parallel transformer training step, after "Cephalo: Harnessing Heterogeneous GPU
 * Clusters for Training Transformer Models" (arXiv 2411.01075).
 *
 * The paper decouples what a GPU computes from what it stores:
 *   - Sec. 3.1 "Compute Partitioning" / Eq. 1: GPU i gets a batch share b_i and scales its
 *     local gradient by N*b_i/B.
 *   - Sec. 3.2: the share runs as l micro-batches of m samples, b = l*m, gradients
 *     accumulated; with layered accumulation every micro-batch passes through a layer
 *     before the next layer.
 *   - Sec. 3.1 "Training State Partitioning": GPU i owns a ratio r_i (anything from none to
 *     all, Sec. 1) of the flat parameter / gradient / Adam-moment buffers of an FSDP unit,
 *     and only that slice is updated there.  Sec. 3.3: 4+4+8 bytes of state per parameter.
 *
 * Conventions common to every call
 *   - Every pointer marked "device" is GPU memory owned by the caller; the library
 *     allocates nothing, keeps no state between calls and frees nothing.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work on it and return; there is no hidden synchronisation.  The offload and
 *     interleaved steps also enqueue on the further streams they are given, ordered by events
 *     that the call creates and releases; all of it is joined into `stream` before the call
 *     returns, so stream order on `stream` is all a caller needs.
 *   - Return value: 0 on success, a negative CEPHALO_E* code otherwise.  Arguments are
 *     validated on the host before anything is launched, so an error return means no
 *     kernel ran.  cephalo_last_error() gives a text for the calling thread's last error.
 *   - Device base pointers must be 16-byte aligned.
 *
 * Flat layout of one layer (an FSDP unit), element indices, no padding, matrices
 * [out_features, in_features] row-major (y = x W^T + b):
 *     ln1.gamma[H] ln1.beta[H] W_qkv[3H,H] b_qkv[3H] W_o[H,H] b_o[H]
 *     ln2.gamma[H] ln2.beta[H] W_fc1[F,H] b_fc1[F] W_fc2[H,F] b_fc2[H]
 * W_qkv rows [0,H) produce Q, [H,2H) K, [2H,3H) V; head a owns columns [a*d,(a+1)*d).
 * The paper fixes no order inside a unit; this one is the library's contract.
 */
#ifndef CEPHALO_H
#define CEPHALO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CEPHALO_OK            0
#define CEPHALO_EINVAL       (-1)  /* bad size, range, null or misaligned pointer          */
#define CEPHALO_EUNSUPPORTED (-2)  /* a shape the kernels do not cover (e.g. head dim)      */
#define CEPHALO_EWORKSPACE   (-3)  /* save / scratch buffer smaller than the query reports  */
#define CEPHALO_EHIP         (-4)  /* a HIP launch reported an error                        */

#define CEPHALO_F32   0  /* activations, parameters and arithmetic in fp32                  */
#define CEPHALO_BF16  1  /* bf16 parameter copy and bf16 operands of every projection and of
                            the attention; fp32 accumulation, statistics, softmax, GELU and
                            parameter gradients.  The residual stream -- a layer's x and y and
                            their gradients dy and dx -- is fp32 in both modes.               */

/* Layer kinds.  GPT-style: the layer described below.  Llama-style (five of the nine models of the paper's model table
 * are of this family): pre-RMSNorm residual blocks, no biases, rotary position embedding on queries and keys (pairs
 * (2i, 2i+1) of a head, angle position * 10000^(-2i/d), position = token index within the sample), gated feed-forward
 *     u = RMS1(x)  qkv = u Wqkv^T  q,k <- rotary  O = attention  x1 = x + O Wo^T
 *     u2 = RMS2(x1)  [g | up] = u2 Wgu^T  h = silu(g) * up  y = x1 + h Wdown^T,      RMS(x) = gamma x / sqrt(mean(x^2) + eps).
 * Its flat layout is  rms1.gamma[H] Wqkv[3H,H] Wo[H,H] rms2.gamma[H] Wgu[2F,H] Wdown[H,F]  (P = 4H^2 + 3HF + 2H): the
 * 12 offsets of cephalo_layer_param_offsets keep their order, the beta and bias slots are empty, slot 8 (W_fc1) is
 * Wgu with gate rows first, slot 10 (W_fc2) is Wdown.  The saved pre-activation is [g | up], 2F wide. */
#define CEPHALO_LAYER_GPT    0
#define CEPHALO_LAYER_LLAMA  1

/* A transformer layer: pre-LayerNorm residual blocks, exact (erf) GELU, biases on every
 * projection, scores scaled by 1/sqrt(d), optional causal mask, no dropout (Sec. 2.1 names
 * only "self-attention and feed-forward"; this form is the library's reading). */
typedef struct cephalo_layer_desc {
  int32_t hidden;   /* H, a multiple of heads; head dim d = H/heads <= 128, in BF16 mode a multiple of 8 (widths other than
                       64 and 128 run on the next of those two tiles with the further columns held at zero) */
  int32_t heads;    /* A */
  int32_t mlp;      /* F */
  int32_t seq;      /* S, tokens per sample */
  int32_t causal;   /* 0 or 1 */
  int32_t dtype;    /* CEPHALO_F32 or CEPHALO_BF16 */
  float   ln_eps;   /* added to the biased variance (GPT-style) or to the mean square (Llama-style) inside the square root */
  int32_t kind;     /* CEPHALO_LAYER_GPT (0) or CEPHALO_LAYER_LLAMA */
} cephalo_layer_desc;

/* Text of the calling thread's most recent error ("" if none). Host pointer, library-owned. */
const char* cephalo_last_error(void);

/* Number of bf16 GEMMs, since the library was loaded, that could not run on the matrix-core kernel (operand pitch or
 * alignment, or a layout / epilogue pair it does not implement) and took the general, much slower kernel instead.  The
 * results are the same; a caller that cares about speed checks that the count stays where it was. */
int64_t cephalo_gemm_general_count(void);

/* Tells the tile choice of the calling thread's later bf16 GEMM launches (cephalo_op_gemm and every call built on it)
 * how many kernels the caller runs side by side on different streams: each then plans for 256 / kernels compute units
 * (a GEMM with 128 output tiles of 256 x 256 fills half the device; two of them on two streams fill it).  1 is the
 * default; values below 1 count as 1.  Results do not depend on it.  Returns the previous value. */
int32_t cephalo_gemm_side_by_side(int32_t kernels);

/* Number of elements P of one layer's flat buffer, 4H^2 + 2HF + 9H + F (GPT-style) or 4H^2 + 3HF + 2H (Llama-style);
 * negative on a bad desc. */
int64_t cephalo_layer_param_count(const cephalo_layer_desc* desc);

/* Element offset of each of the 12 tensors inside the flat buffer, in layout order, written
 * to host array offsets[12]. */
int cephalo_layer_param_offsets(const cephalo_layer_desc* desc, int64_t* offsets);

/* Bytes of the per-micro-batch activation save area (written by layer_fwd, read by
 * layer_bwd) and of the scratch area, for micro-batch size m.  Neither depends on the
 * number of micro-batches l: compute memory is a function of m alone (Sec. 3.3, memory
 * utilization model).  Host pointers out. */
int cephalo_layer_workspace_bytes(const cephalo_layer_desc* desc, int32_t micro_batch,
                                  size_t* save_bytes, size_t* scratch_bytes);

/* The same for cephalo_share_layer_step, which keeps every micro-batch's saved activations and
 * weight-gradient operands until the share's single parameter-gradient pass (288 GB of HBM make
 * keeping cheaper than the recomputation and host offload the paper needs on 12-24 GB GPUs, Sec. 3.2
 * "Activation Checkpointing and Offloading").  batch_share must be a positive multiple of micro_batch. */
int cephalo_share_workspace_bytes(const cephalo_layer_desc* desc, int32_t batch_share, int32_t micro_batch,
                                  size_t* save_bytes_total, size_t* scratch_bytes);

/* Forward of one layer on one micro-batch of m samples (Sec. 3.2; the step timed as T_f(m)
 * in Sec. 3.3).
 *   flat_param  device, [P] in the compute dtype (fp32, or the bf16 copy of the fp32 master)
 *   x, y        device, [m, S, H] fp32 (the residual stream); y may not alias x
 *   save        device, save_bytes; holds what the backward needs (x itself is not copied:
 *               the caller keeps x alive and passes it to layer_bwd)
 *   scratch     device, scratch_bytes; contents undefined afterwards */
int cephalo_layer_fwd(const cephalo_layer_desc* desc, const void* flat_param,
                      const void* x, void* y, int32_t micro_batch,
                      void* save, size_t save_bytes,
                      void* scratch, size_t scratch_bytes, void* stream);

/* Backward of the same micro-batch (T_b(m) in Sec. 3.3) with the gradient accumulation of
 * Sec. 3.2 folded in:   flat_grad <- (accumulate ? flat_grad : 0) + grad_scale * g_j
 * where g_j is this micro-batch's parameter gradient summed over its tokens and grad_scale
 * is the caller's factor (Eq. 1's N*b_i/B and any 1/b_i mean).  Every element of flat_grad
 * is written by exactly one thread block in a fixed order, so results are reproducible.
 *   x           device, the forward input of this micro-batch
 *   dy, dx      device, [m, S, H] fp32; dx may not alias dy
 *   flat_grad   device, [P] fp32 */
int cephalo_layer_bwd(const cephalo_layer_desc* desc, const void* flat_param,
                      const void* x, const void* dy, void* dx, int32_t micro_batch,
                      const void* save, size_t save_bytes,
                      float* flat_grad, float grad_scale, int32_t accumulate,
                      void* scratch, size_t scratch_bytes, void* stream);

/* Whole share of one layer, micro-batches in order j = 0..l-1 (Sec. 3.2, b = l*m; the layered
 * order of Sec. 3.2 "Layered Gradient Accumulation": every micro-batch passes through the layer
 * before anything else runs): forward of every micro-batch, backward data path of every
 * micro-batch, then one parameter-gradient pass over all b*S tokens, in which the sum over
 * micro-batches is formed in the fp32 accumulators of the weight-gradient GEMMs and every element
 * of flat_grad is written exactly once:  flat_grad <- grad_scale * sum_j g_j.
 * Equal to l calls of layer_fwd and layer_bwd up to the order of the fp32 additions.
 * Fails with CEPHALO_EINVAL unless batch_share = l * micro_batch for a positive integer l.
 *   x, y, dy, dx  device, [b, S, H] fp32;  save, scratch: sizes from cephalo_share_workspace_bytes */
int cephalo_share_layer_step(const cephalo_layer_desc* desc, const void* flat_param,
                             const void* x, void* y, const void* dy, void* dx,
                             int32_t batch_share, int32_t micro_batch,
                             void* save, size_t save_bytes_total,
                             float* flat_grad, float grad_scale,
                             void* scratch, size_t scratch_bytes, void* stream);

/* The same with two micro-batches in flight: micro-batch j runs on stream j mod 2 (`stream` and `side_stream`, another
 * stream of the same device at the default priority), so that the bandwidth-bound kernels of one run under the
 * matrix-core kernels of the other and GEMMs with few output tiles share the compute units.  Every micro-batch's own
 * kernel order and every reduction order are those of cephalo_share_layer_step: same results bit for bit, same work
 * areas.  The call joins the streams before it returns: work enqueued on `stream` afterwards runs after the whole step. */
int cephalo_share_layer_step_interleaved(const cephalo_layer_desc* desc, const void* flat_param,
                                         const void* x, void* y, const void* dy, void* dx,
                                         int32_t batch_share, int32_t micro_batch,
                                         void* save, size_t save_bytes_total,
                                         float* flat_grad, float grad_scale,
                                         void* scratch, size_t scratch_bytes, void* stream, void* side_stream);

/* acc[i] <- acc[i] + scale * g[i], i in [0, n): gradient accumulation across micro-batches
 * (Sec. 3.2) as a stand-alone pass.  acc, g device fp32, n >= 0. */
int cephalo_grad_accum(float* acc, const float* g, float scale, int64_t n, void* stream);

/* Adam on this GPU's slice [offset, offset+len) of the flat training state (Sec. 3.1
 * "Training State Partitioning"; fp32 parameter, gradient and two moments, Sec. 3.3).
 *   g' = g + weight_decay p       (the decay joins the gradient: plain Adam's L2 term; 0 = none)
 *   m <- beta1 m + (1-beta1) g';  v <- beta2 v + (1-beta2) g'^2
 *   p <- p - lr * (m / (1-beta1^step)) / (sqrt(v / (1-beta2^step)) + eps)
 * p, g, m, v are device pointers to element 0 of the flat buffers and are indexed globally;
 * nothing outside the slice is read or written.  p_lowp, if not NULL, is a device bf16 [P]
 * buffer whose slice receives the rounded (nearest-even) new parameters for the next
 * step's compute.  len = 0 is a valid no-op; offset = 0, len = P is the unsharded update.
 * step is 1-based.  Each element's arithmetic is the same instruction sequence wherever
 * the slice starts, so updates over any partition of [0,P) concatenate to the unsharded
 * update bit for bit.  The four fp32 base pointers must be 16-byte aligned; the kernel runs
 * at its full rate when they are congruent modulo 256 bytes (it starts its vector body where
 * p's address is a multiple of 256; buffers that sit elsewhere are still correct, only slower).
 * Errors (nothing launched): slice outside [0, P), step < 1, beta outside [0, 1), eps < 0,
 * weight_decay < 0 or not finite, a NULL or misaligned buffer with len > 0. */
int cephalo_shard_adam(float* p, const float* g, float* m, float* v, void* p_lowp,
                       int64_t P, int64_t offset, int64_t len,
                       float lr, float beta1, float beta2, float eps, float weight_decay, int64_t step,
                       void* stream);

/* dst[i] <- bf16(src[i]) (nearest-even), i in [0, n): makes the compute copy of fp32 master
 * parameters (the mixed-precision workloads' rule; the paper itself trains in fp32). */
int cephalo_cast_bf16(void* dst_bf16, const float* src, int64_t n, void* stream);

/* ---------------------------------------------------------------------------------------
 * Building blocks of the layer, exported so that each kernel family can be checked against
 * the oracle and profiled on its own.  Same conventions as above.
 */

/* Epilogues of cephalo_op_gemm */
#define CEPHALO_EPI_NONE        0  /* C = acc                                              */
#define CEPHALO_EPI_BIAS        1  /* C = acc + bias[n]                                    */
#define CEPHALO_EPI_BIAS_RESID  2  /* C = acc + bias[n] + R[m,n]                           */
#define CEPHALO_EPI_BIAS_GELU   3  /* Z = acc + bias[n]; C = gelu(Z); both stored          */
#define CEPHALO_EPI_DGELU       4  /* C = acc * gelu'(Z[m,n])                              */
#define CEPHALO_EPI_GRAD        5  /* G = (accumulate ? G : 0) + scale * acc   (G fp32)    */
#define CEPHALO_EPI_NONE_F32    6  /* as NONE, C is fp32 [M,N] whatever dtype says          */
#define CEPHALO_EPI_BIAS_RESID_F32 7 /* as BIAS_RESID, R and C are fp32 [M,N] (the residual stream) */
#define CEPHALO_EPI_BIAS_GELU_DERIV 8 /* z = acc + bias[n]; C = gelu(z); Z = gelu'(z): what the layer's forward saves */
#define CEPHALO_EPI_MUL         9  /* C = acc * Z[m,n]: the layer's backward through GELU, with Z = gelu'(z) saved   */
/* For these two epilogues Z is a saved factor, not a matrix operand: with bf16 operands it is an [M,N] array of IEEE
 * half values (two bytes like bf16, three more significand bits), with fp32 operands an fp32 array. */

/* C[M,N] = sum_k A(m,k) * B(n,k) with a fused epilogue; the contraction of a linear layer's
 * forward (both operands k-contiguous), input gradient (B n-contiguous) and weight gradient
 * (both operands contiguous along their own rows, strided along k = tokens).
 * Element (m,k) of A is A[m*a_rs + k*a_cs], (n,k) of B is B[n*b_rs + k*b_cs]; one stride of
 * each operand is 1.  dtype selects fp32 or bf16 operands/outputs (accumulation is fp32 either
 * way).  C, R, Z are [M,N] row-major in dtype; bias [N] in dtype; G [M,N] fp32.  Unused
 * pointers may be NULL.  All device memory. */
int cephalo_op_gemm(int32_t dtype, const void* A, int64_t a_rs, int64_t a_cs,
                    const void* B, int64_t b_rs, int64_t b_cs, int32_t M, int32_t N, int32_t K,
                    int32_t epilogue, void* C, const void* bias, const void* R, void* Z,
                    float* G, float scale, int32_t accumulate, void* stream);

/* Weight gradient of a linear layer y = x W^T over T tokens, as the layer's backward computes it:
 *   G[N,K] <- (accumulate ? G : 0) + scale * sum_t dY[t,n] X[t,k]        (dY [T,N], X [T,K] row-major in dtype, G fp32)
 * Both operands are read as they lie (no transposed copy).  In bf16 mode, when the output has few tiles, the token axis
 * is cut into pieces whose partial sums are added in a fixed order (reproducible).  workspace: device, at least
 * cephalo_op_linear_wgrad_workspace(dtype, T, N, K) bytes. */
size_t cephalo_op_linear_wgrad_workspace(int32_t dtype, int32_t T, int32_t N, int32_t K);
int cephalo_op_linear_wgrad(int32_t dtype, const void* dY, const void* X, int32_t T, int32_t N, int32_t K,
                            float* G, float scale, int32_t accumulate, void* workspace, size_t workspace_bytes, void* stream);

/* The same weight gradient together with the bias gradient of the projection (Sec. 3.2: both belong to the gradient
 * the share accumulates over its micro-batches):
 *   gb[N] <- (accumulate ? gb : 0) + scale * sum_t dY[t,n]                 (fp32)
 * In bf16 mode the GEMM forms the column sums on the way: dY's tiles pass through its registers anyway, every tile is
 * summed by exactly one wavefront, and the pieces are added in a fixed order (reproducible).  With fp32 operands, or
 * a token axis so long that the GEMM runs in several calls (operands beyond 2 GiB), a column-sum kernel runs after
 * the GEMM on the same stream.  N must be a multiple of 8; buffers 16-byte aligned, all device memory.
 * workspace: at least cephalo_op_linear_wgrad_bias_workspace(dtype, T, N, K) bytes. */
size_t cephalo_op_linear_wgrad_bias_workspace(int32_t dtype, int32_t T, int32_t N, int32_t K);
int cephalo_op_linear_wgrad_bias(int32_t dtype, const void* dY, const void* X, int32_t T, int32_t N, int32_t K,
                                 float* G, float* gb, float scale, int32_t accumulate, void* workspace,
                                 size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory and have no work area to hand over (code under HIP graph capture,
 * tight serving loops, harnesses that forbid allocation): cephalo_op_linear_wgrad with the partial sums of a split
 * token axis kept in a fixed device array of CEPHALO_NOALLOC_SCRATCH_BYTES that the library's code object carries
 * (each GPU the library is used on holds one copy until the process ends).  Same arguments without the work area, same
 * kernels, bit-identical G.  The call allocates and frees nothing (no device memory, no events); its first use on a
 * GPU looks the array's address up once.  A problem whose partial sums (pieces x N x K x 4 bytes, for bf16 outputs
 * with few tiles and T >= 2048 only) exceed the array is refused with CEPHALO_EWORKSPACE before anything is launched.
 * Every call on a GPU uses that GPU's one array: two calls that overlap in time on the same GPU (different streams or
 * threads) race on it; calls on one stream are ordered and safe.  Nothing in the array has to be cleared between
 * calls.  Call it with the GPU of `stream` current. */
#define CEPHALO_NOALLOC_SCRATCH_BYTES (64u << 20)
int cephalo_op_linear_wgrad_static(int32_t dtype, const void* dY, const void* X, int32_t T, int32_t N, int32_t K,
                                   float* G, float scale, int32_t accumulate, void* stream);

/* The bandwidth-bound pieces of the layer and of the stack's head, one call each (one wavefront per row; fp32
 * statistics).  dtype selects the activation type (fp32, or bf16 for u / gamma / beta / dx_lowp / dlogits); the
 * residual stream x, the incoming gradient du, the result dx and every parameter gradient are fp32 in both modes.
 *
 * norm_fwd: u[r] = gamma * (x[r] - mean_r) * rstd_r + beta over the H columns of each of `rows` rows, biased variance,
 *   eps inside the square root; mean, rstd: fp32 [rows], saved for the backward.  rms != 0: root-mean-square norm,
 *   u = gamma * x / sqrt(mean(x^2) + eps); beta is not read and may be NULL.  H a multiple of 8, at most 8192 (4096 in
 *   fp32 mode).
 * norm_bwd: dx = resid + rstd * (g - mean_h(g) - xhat * mean_h(g * xhat)),  g = du * gamma  (resid may be NULL: none;
 *   rms: the mean_h(g) term is absent); dx_lowp, if not NULL, receives dx in the activation type as well;
 *   dgamma[h] = sum_r du * xhat, dbeta[h] = sum_r du (rms: dbeta untouched, may be NULL), summed in a fixed order.
 *   workspace: device, cephalo_op_norm_bwd_workspace(rows, H) bytes.
 * norm_bwd_sums: norm_bwd in the LayerNorm form (no rms) that also returns dx_colsum[h] = sum_r dx[r][h] (fp32, fixed
 *   order): dx is a gradient of the residual stream, and its column sum is the bias gradient of the projection whose
 *   output was added to the stream there (Sec. 3.2's accumulated gradient holds it), so the kernel that writes dx sums
 *   it on the way.  dx, dx_lowp, dgamma, dbeta are bit-identical to norm_bwd's.  workspace:
 *   cephalo_op_norm_bwd_sums_workspace(rows, H) bytes.
 * colsum: g[n] = (accumulate ? g[n] : 0) + scale * sum_r X[r][n], X [rows, N] in dtype (a bias gradient), fixed order.
 * cross_entropy: for each row of fp32 logits [rows, ld] (V valid columns, ld >= V a multiple of 8):
 *   loss_rows[r] = logsumexp(row) - row[target],  dlogits[r] = coef * (softmax(row) - onehot(target)) in dtype, columns
 *   V..ld-1 zero; targets int32 [rows], clamped to [0, V).
 * Errors as elsewhere: nothing is launched when an argument is refused. */
int cephalo_op_norm_fwd(int32_t dtype, int32_t rms, const float* x, const void* gamma, const void* beta, void* u,
                        float* mean, float* rstd, int32_t rows, int32_t H, float eps, void* stream);
size_t cephalo_op_norm_bwd_workspace(int32_t rows, int32_t H);
int cephalo_op_norm_bwd(int32_t dtype, int32_t rms, const float* du, const float* x, const float* mean, const float* rstd,
                        const void* gamma, const float* resid, float* dx, void* dx_lowp, float* dgamma, float* dbeta,
                        int32_t rows, int32_t H, void* workspace, size_t workspace_bytes, void* stream);
size_t cephalo_op_norm_bwd_sums_workspace(int32_t rows, int32_t H);
int cephalo_op_norm_bwd_sums(int32_t dtype, const float* du, const float* x, const float* mean, const float* rstd,
                             const void* gamma, const float* resid, float* dx, void* dx_lowp, float* dgamma, float* dbeta,
                             float* dx_colsum, int32_t rows, int32_t H, void* workspace, size_t workspace_bytes, void* stream);
size_t cephalo_op_colsum_workspace(int32_t rows, int32_t N);
int cephalo_op_colsum(int32_t dtype, const void* X, int32_t rows, int32_t N, float* g, float scale, int32_t accumulate,
                      void* workspace, size_t workspace_bytes, void* stream);
int cephalo_op_cross_entropy(int32_t dtype, const float* logits, int32_t ld, const int32_t* targets, void* dlogits,
                             float* loss_rows, int32_t rows, int32_t V, float coef, void* stream);

/* Attention of one micro-batch on the packed projection qkv [m*S, 3H] (column blocks Q | K | V).
 * Forward writes O [m*S, H] (dtype) and lse [m, A, S] fp32, the log-sum-exp of each query row's
 * scaled, masked scores.  Backward writes dqkv [m*S, 3H]; dvec [m, A, S] fp32 is scratch. */
int cephalo_op_attention_fwd(const cephalo_layer_desc* desc, const void* qkv, void* O, float* lse,
                             int32_t micro_batch, void* stream);
int cephalo_op_attention_bwd(const cephalo_layer_desc* desc, const void* qkv, const void* O, const void* dO,
                             const float* lse, float* dvec, void* dqkv, int32_t micro_batch, void* stream);

/* ---------------------------------------------------------------------------------------
 * A whole stack on one GPU's batch share, in the layered order of Sec. 3.2 ("Layered Gradient
 * Accumulation": all micro-batches pass through a layer before the next layer, forward and backward).
 * The paper trains such models (Table 2) without describing their pieces; the form here: learned token
 * and position embeddings x0 = wte[id] + wpe[pos], `layers` layers as above, final LayerNorm, logits =
 * lnf(x) wte^T (tied, no bias), loss = mean cross-entropy over all b*S tokens.
 * Flat layout: wte[V,H] wpe[S,H] layer 0 .. layer L-1 (each as above) lnf.gamma[H] lnf.beta[H].
 * With Llama-style layers (layer.kind = CEPHALO_LAYER_LLAMA; five of the nine models of Sec. 5.1's table): x0 = wte[id]
 * (positions enter through the rotation inside the layers), a final RMSNorm, logits = normf(x) w_head^T with a head
 * of its own.  Flat layout: wte[V,H] layer 0 .. layer L-1 normf.gamma[H] w_head[V,H].
 */
typedef struct cephalo_stack_desc {
  cephalo_layer_desc layer;
  int32_t layers;      /* L */
  int32_t vocab;       /* V */
  int32_t checkpoint;  /* 0: every layer's internal activations are kept from forward to backward (the default on a
                          288 GB device).  1: activation checkpointing at layer boundaries (Sec. 3.2 "Activation
                          Checkpointing and Offloading"): only the layer-boundary activations are kept, and the backward
                          of a layer first runs that layer's forward again for all micro-batches.  Same results bit for
                          bit; the work area holds one layer's internals instead of L; costs one extra forward. */
  int32_t offload;     /* 0, or 1 (needs checkpoint = 1): the layer-boundary activations live in pinned host memory instead
                          of the work area (the same section, and the supplementary figure on activation offloading): a
                          micro-batch's boundary activation is copied out on a second stream while the next micro-batch
                          runs and is fetched back ahead of its use, in the forward as the next layer's input and in the
                          backward for the recomputation; the device holds four micro-batches of them.  Same results bit
                          for bit.  (The gradient of the residual stream, two [b*S, H] buffers, stays on the device; the
                          paper moves that to the host too.)  Goes with cephalo_stack_step_offload. */
  int32_t interleave;  /* 0, or 1 (not with offload): two micro-batches are in flight at once, micro-batch j on stream j mod 2
                          (the caller's compute stream and a side stream), so that the bandwidth-bound kernels of one
                          overlap the matrix-core kernels of the other and GEMMs with few output tiles share the compute
                          units.  The order of a micro-batch's own kernels, and every reduction order, are unchanged: same
                          results bit for bit.  The work area holds the per-micro-batch buffers twice.  Goes with
                          cephalo_stack_step_interleaved. */
} cephalo_stack_desc;

/* V*H + S*H + L*P_layer + 2H (GPT-style) or 2*V*H + L*P_layer + H (Llama-style); negative on a bad desc. */
int64_t cephalo_stack_param_count(const cephalo_stack_desc* desc);

/* Element offsets inside the stack's flat buffer, written to host array offsets[5]: token embedding, learned positions
 * (an empty range, equal to the next offset, where the stack has none), layer 0 (layer i follows at i * P_layer), the
 * final norm's parameters, the head (the token embedding's offset where the head is tied to it). */
int cephalo_stack_param_offsets(const cephalo_stack_desc* desc, int64_t* offsets);

/* Bytes of the single work area of cephalo_stack_step (layer-boundary activations and saved activations of
 * every layer and micro-batch, one micro-batch of logits and the share's logit gradients, backward buffers).
 * Host pointer out.  Without offload the area begins with the layer-boundary activations, fp32 [layers+1][b*S][H]:
 * entry 0 is the embedding output, entry i the output of layer i-1; they are valid after cephalo_stack_step returns. */
int cephalo_stack_workspace_bytes(const cephalo_stack_desc* desc, int32_t batch_share, int32_t micro_batch, size_t* bytes);

/* Where three things lie in that work area once a step has returned, as byte offsets written to host array
 * offsets[3], so that a layer of a full-size stack can be checked on its own (Sec. 3.2's layered order: the backward
 * of layer 0 is the last thing that ran, over every micro-batch):
 *   [0] the layer-boundary activations (as above; meaningful without offload only),
 *   [1] the gradient of the loss with respect to layer 0's input,  fp32 [b*S][H], times grad_scale,
 *   [2] the gradient of the loss with respect to layer 0's output, fp32 [b*S][H], times grad_scale
 *       (a one-layer stack: with respect to the final norm's input). */
int cephalo_stack_workspace_regions(const cephalo_stack_desc* desc, int32_t batch_share, int32_t micro_batch, size_t* offsets);

/* Forward, loss and backward of the whole share (b = l*m, Sec. 3.2):
 *   loss[0]   <- mean over the b*S tokens of the cross-entropy (device, one float)
 *   flat_grad <- grad_scale * d(loss)/d(parameters), every element written (device, [P] fp32); grad_scale is
 *                Eq. 1's factor.  The sum over micro-batches is formed inside the weight-gradient GEMMs.
 *   flat_param   device, [P] in the compute dtype;  ids, targets  device, int32 [b, S]; values outside [0, V)
 *                are clamped into range.
 * Reproducible: no atomics; token-embedding rows are summed in ascending token order (rows of ids that do not occur get
 * the head's part where the head is tied, zero otherwise). */
int cephalo_stack_step(const cephalo_stack_desc* desc, const void* flat_param,
                       const int32_t* ids, const int32_t* targets, int32_t batch_share, int32_t micro_batch,
                       float* flat_grad, float grad_scale, float* loss,
                       void* workspace, size_t workspace_bytes, void* stream);

/* The same step for a desc with offload = 1 (Sec. 3.2 "Activation Checkpointing and Offloading").
 *   host_area    HOST memory, page-locked (pinned) so that the copies run asynchronously, at least
 *                cephalo_stack_host_bytes(...) bytes; afterwards it holds the layer-boundary activations, fp32
 *                [layers+1][b*S][H] as described for the work area above.  Caller-owned.
 *   copy_in_stream, copy_out_stream   HIP streams other than `stream` on which the library enqueues the copies to the
 *                device and to the host (two streams keep both directions of the link busy; the same stream may be
 *                given for both); events order them against `stream`.  When the call returns everything is enqueued
 *                and `stream` ends behind the last copy: synchronising `stream` is enough before the host area is
 *                read or released.
 * The library creates and destroys a handful of HIP events per call (no device memory). */
int cephalo_stack_host_bytes(const cephalo_stack_desc* desc, int32_t batch_share, int32_t micro_batch, size_t* bytes);
int cephalo_stack_step_offload(const cephalo_stack_desc* desc, const void* flat_param,
                               const int32_t* ids, const int32_t* targets, int32_t batch_share, int32_t micro_batch,
                               float* flat_grad, float grad_scale, float* loss,
                               void* workspace, size_t workspace_bytes, void* host_area, size_t host_bytes,
                               void* stream, void* copy_in_stream, void* copy_out_stream);

/* The same step for a desc with interleave = 1 (Sec. 3.2's layered order leaves the micro-batches of a layer independent
 * of each other; here two of them run side by side).  side_stream: a second stream of the same device, other than
 * `stream`, at the default priority.  The call joins the streams before it returns: work enqueued on `stream`
 * afterwards runs after the whole step; the side stream may be reused at once.  Arguments otherwise as for
 * cephalo_stack_step; workspace size from cephalo_stack_workspace_bytes with the same desc. */
int cephalo_stack_step_interleaved(const cephalo_stack_desc* desc, const void* flat_param,
                                   const int32_t* ids, const int32_t* targets, int32_t batch_share, int32_t micro_batch,
                                   float* flat_grad, float grad_scale, float* loss,
                                   void* workspace, size_t workspace_bytes, void* stream, void* side_stream);

/* ---------------------------------------------------------------------------------------
 * Measurement probes (bench.py --peaks): what this device sustains, to be quoted beside the published peaks.
 *
 * probe_mfma: `blocks` blocks of eight wavefronts, each issuing iters x 32 products v_mfma_f32_16x16x32_bf16 on operands
 *   held in registers (the GEMM kernel's wavefront tile without any LDS or memory traffic).  seed_bf16: device, 64 KiB of
 *   bf16 values the operands are taken from (the sustained rate depends on the data: fill it with random values);
 *   sink: device, one float; flops_out (host, may be NULL) receives the flops of the launch.
 * probe_stream: mode 0 reads `bytes` of src, 1 writes `bytes` of dst, 2 copies src to dst, with streaming 16-byte
 *   accesses (bytes a multiple of 16; both buffers device memory, 16-byte aligned).
 * Both only enqueue on `stream`; the caller times them. */
int cephalo_probe_mfma(const void* seed_bf16, int32_t blocks, int32_t iters, float* sink, double* flops_out, void* stream);
int cephalo_probe_stream(int32_t mode, void* dst, const void* src, int64_t bytes, float* sink, void* stream);

/* ---------------------------------------------------------------------------------------
 * Planning on the host (no device involved): how the global batch and the training state are divided over the
 * N GPUs of a cluster (Sec. 3.4 "Optimizer" and the supplementary Algorithm 1).
 *
 * The paper's notation table calls N, B "number of layers and GPUs"; the text and the algorithm use N = number of
 * GPUs and B = global batch size, which is the reading here.  Its algorithm starts the search for the best final
 * entry from 0 instead of infinity and writes the compute memory as M(m, l) although Sec. 3.3 makes it a function of
 * m alone; this library starts from infinity, uses M(m) = mem_base + mem_per_sample * m, and keeps only those totals
 * k of the micro-batch sizes whose cluster-wide memory fits (constraint III), as the text says.
 */
typedef struct cephalo_gpu_perf {
  const double* t_fwd;   /* host, [max_m + 1]: forward latency of one micro-batch of m samples at index m (index 0 unused) */
  const double* t_bwd;   /* likewise for the backward; sizes beyond max_m are extended linearly through the last two points */
  int32_t max_m;
  double  mem_cap;       /* bytes this GPU may use */
} cephalo_gpu_perf;

typedef struct cephalo_cluster_model {
  double allgather, reducescatter;                /* latency of the even collectives of one unit            */
  double allgather_uneven, reducescatter_uneven;  /* and with uneven inputs (Sec. 3.3: assumed 15 % slower)  */
  double mem_base, mem_per_sample;                /* compute memory M(m) = mem_base + mem_per_sample * m     */
  double state_bytes;                             /* training state of the model, 16 bytes per parameter     */
} cephalo_cluster_model;

/* Compute partition: micro-batch size m_i and micro-batch count l_i per GPU with sum_i m_i l_i = batch, minimising
 *   max_i [ max(l_i T_f^i(m_i), AG') + max(l_i T_b^i(m_i), AG' + RS') ]
 * where AG', RS' are the uneven latencies for a GPU whose compute memory plus an even state share exceeds its
 * capacity; M(m_i) <= capacity_i for every GPU and the cluster-wide memory must fit; every GPU takes at least one
 * sample.  Solved as a bottleneck problem: bisection over the candidate latencies, and for a candidate a dynamic
 * programme over (GPU, batch so far) that keeps the least sum of micro-batch sizes, which is all the cluster-wide
 * memory depends on: O(N B^2 log(N B)) time, tables of N x B entries (the supplementary algorithm spends N B^4 steps
 * on a table of N x B x B).  m_out, l_out: host, [n_gpus]; latency_out (may be NULL): the minimised layer latency.
 * CEPHALO_EUNSUPPORTED if nothing fits, if batch < n_gpus, or if n_gpus x batch exceeds 2^26. */
int cephalo_plan_compute(int32_t n_gpus, const cephalo_gpu_perf* gpus, int32_t batch, const cephalo_cluster_model* cluster,
                         int32_t* m_out, int32_t* l_out, double* latency_out);

/* Training-state partition for given micro-batch sizes: ratios r_i (sum 1) that minimise the largest memory
 * utilisation (compute memory + r_i * state) / capacity_i, by handing state to the least utilised GPU first.
 * ratio_out: host, [n_gpus]. */
int cephalo_plan_state(int32_t n_gpus, const cephalo_gpu_perf* gpus, const int32_t* m, const cephalo_cluster_model* cluster,
                       double* ratio_out);

/* Per-unit shards for given training-state ratios (Sec. 4 "Uneven Parameter Sharding": uneven collectives cost up to
 * 15 % whatever the skew, so as few units as possible are sharded unevenly; the paper's example: two units and a 3:1
 * ratio over two GPUs give one unit split 1:1 and one split 1:0).  n_units identical units of unit_len elements;
 * GPU i is to hold ratio[i] (>= 0, sum 1) of all n_units * unit_len elements (targets rounded to whole elements by
 * largest remainder).  The first n_even units are sharded evenly, GPU i holding [floor(i L / N), floor((i+1) L / N));
 * n_even is the largest count every GPU's target can carry.  The other units are one flat run that the GPUs divide
 * in order, each taking what its target still lacks, so a GPU's part of a unit is one slice (possibly empty).
 * offset_out, len_out: host, [n_units][n_gpus], unit-major: GPU i's slice of unit u is [offset, offset + len) -- the
 * (offset, len) that cephalo_shard_adam takes for that unit.  n_even_out: host, may be NULL. */
int cephalo_plan_units(int32_t n_gpus, const double* ratio, int32_t n_units, int64_t unit_len,
                       int64_t* offset_out, int64_t* len_out, int32_t* n_even_out);

#ifdef __cplusplus
}
#endif
#endif /* CEPHALO_H */
