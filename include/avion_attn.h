/*
 * avion_attn.h -- C ABI of the MI355X (gfx950) exact, O(N)-memory multi-head self-attention.
 *
 * The operation is the attention core of the plain joint space-time ViT of the paper (Sec. 3,
 * "Video Transformer": N = T/t * H/h * W/w tokens; each encoder layer holds one multi-head
 * self-attention), made memory efficient as in Sec. 3, "Flash Attention": the softmax weights are
 * never stored (memory O(N) instead of O(N^2)) and the work is done block by block out of on-chip
 * memory, the block results being combined into the exact final output (Sec. 1).
 *
 * Per (batch b, head h), with s_ij = scale * <q_i, k_j>, P = row-softmax(S):
 *     forward :  O = P V ,  LSE_i = ln sum_j exp(s_ij)
 *     backward:  dV = P^T dO ; dP = dO V^T ; dS = P o (dP - rowsum(dO o O)) ;
 *                dQ = scale * dS K ; dK = scale * dS^T Q
 * Non-causal, no mask, no dropout, same N for queries and keys.
 *
 * Common rules for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library never allocates,
 *     frees or keeps them.  q, k, v, o, dO, dq, dk, dv are bf16 in the layout [B, N, H, d],
 *     contiguous (token stride H*d elements, head stride d).  lse is fp32 in the layout [B, H, N]
 *     (natural logarithm of the sum of exponentials of the *scaled* scores).
 *   - Every tensor pointer must be 16-byte aligned.  Outputs must not alias inputs or each other.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls only enqueue work
 *     on that stream and return; they never synchronise.
 *   - Supported head dims: d = 64 and d = 80.  Any B, H, N >= 1 with N <= 2^24, B*H <= 2^24,
 *     (N + 256) * H*d * 2 bytes < 2^31 and fewer than 2^31 workgroups (else AVION_EUNSUPPORTED).
 *   - Return value: AVION_OK (0) or a negative AVION_E* code.  On an argument error nothing is
 *     launched and no output is touched.  No exception crosses the boundary.
 *   - NaN/Inf in the inputs are not checked and propagate.
 *   - Arithmetic: bf16 MFMA contractions with fp32 accumulation; softmax statistics, LSE and the
 *     row sums of dO o O in fp32; P and dS are rounded to bf16 (nearest even) before they enter a
 *     contraction; outputs are rounded to bf16 once, at the final store.
 *   - Results are bit-reproducible from run to run (no atomics anywhere).
 */
#ifndef AVION_ATTN_H
#define AVION_ATTN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AVION_OK 0
#define AVION_EINVAL (-1)       /* null pointer; B, H or N < 1; scale not finite or < 2^-60         */
#define AVION_EUNSUPPORTED (-2) /* d not in {64, 80}; misaligned pointer; N > 2^24; B*H > 2^24     */
#define AVION_EWORKSPACE (-3)   /* workspace NULL, misaligned (256 B) or smaller than required      */
#define AVION_EHIP (-4)         /* a HIP launch failed; avion_last_hip_error() has the runtime text */
#define AVION_ESCRATCH (-5)     /* avion_attn_bwd_noalloc: problem exceeds the built-in scratch     */

/* Library version as major*10000 + minor*100 + patch. */
int avion_version(void);

/* Static text for a return code (never NULL). */
const char *avion_strerror(int code);

/* Text of the last HIP runtime error seen by this thread inside the library ("" if none). */
const char *avion_last_hip_error(void);

/*
 * Forward (Sec. 3, "Flash Attention"; Sec. 1 for the exactness of the block-wise combination).
 *   q, k, v : in,  bf16 [B,N,H,d]
 *   o       : out, bf16 [B,N,H,d], fully overwritten
 *   lse     : out, fp32 [B,H,N],   fully overwritten; needed by avion_attn_bwd
 *   scale   : multiplies the dot products (1/sqrt(d) in a ViT); must be finite and >= 2^-60
 *             (keys outside a ragged tile or a causal mask are removed by a score of -1e30 times
 *             scale, which must stay far below every real score)
 * Extra device memory used: none.
 */
int avion_attn_fwd(const void *q, const void *k, const void *v, void *o, float *lse,
                   int B, int H, int N, int d, float scale, void *stream);

/*
 * Bytes of device workspace avion_attn_bwd needs for this shape: two fp32 per (batch, head, query)
 * (the row sums of dO o O and a rescaled copy of lse), with N rounded up to a multiple of 64 and
 * the total to 256 bytes -- linear in N, never N^2.  Returns 0 for an unsupported shape.
 */
size_t avion_attn_bwd_workspace_bytes(int B, int H, int N, int d);

/*
 * Backward.  P is rebuilt block by block from q, k and the saved lse, so no N x N matrix is read
 * or written (Sec. 3: the weights stay implicit; Sec. 4.1: the attention memory is removed).
 *   q, k, v     : in,  bf16 [B,N,H,d]  (the forward's inputs)
 *   o, lse      : in,  exactly as avion_attn_fwd wrote them
 *   dO          : in,  bf16 [B,N,H,d]  gradient of the loss with respect to o
 *   dq, dk, dv  : out, bf16 [B,N,H,d], fully overwritten
 *   workspace   : device scratch, 256-byte aligned, at least avion_attn_bwd_workspace_bytes(...)
 *                 bytes; contents on entry are ignored, contents on return are unspecified.
 *                 Two calls that overlap in time on the GPU must not share a workspace.
 */
int avion_attn_bwd(const void *q, const void *k, const void *v, const void *o, const float *lse,
                   const void *dO, void *dq, void *dk, void *dv,
                   int B, int H, int N, int d, float scale,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * The two phases of avion_attn_bwd, callable on their own (same argument rules as above).
 * For N > 32, avion_attn_bwd(...) gives exactly the bits of avion_attn_bwd_dq(...) followed by
 * avion_attn_bwd_dkdv(...) on the same stream with the same workspace; for N <= 128 it runs both
 * phases in one launch (one workgroup then covers a whole (batch, head)), otherwise as two.
 * Sequences of at most 32 tokens (temporal attention over a few frames, Sec. 4.1; very short
 * captions) take another route in avion_attn_fwd / avion_attn_bwd and all their variants: one
 * wavefront computes a window of floor(32 / N) whole problems at once, forward and backward each
 * in one pass with no workspace traffic; same formulas and rounding points, another summation
 * order, so those results agree with the two phases within the tolerances, not bit for bit.
 *
 *   avion_attn_bwd_dq   : query-stationary pass.  Computes the row sums delta = rowsum(dO o O) and
 *                         dQ = scale * (P o (dO V^T - delta)) K.  Writes dq (fully) and leaves
 *                         delta and lse, in the form the second pass consumes, in `workspace`.
 *   avion_attn_bwd_dkdv : key-stationary pass.  Reads delta and lse from `workspace` (as left there
 *                         by avion_attn_bwd_dq for the same q, k, v, o, lse, dO; the `lse` argument
 *                         is only checked) and computes dV = P^T dO and dK = scale * dS^T Q.
 *                         Writes dk, dv (fully).
 * Both rebuild P from q, k and lse block by block (Sec. 3: the weights stay implicit).
 */
int avion_attn_bwd_dq(const void *q, const void *k, const void *v, const void *o, const float *lse,
                      const void *dO, void *dq, int B, int H, int N, int d, float scale,
                      void *workspace, size_t workspace_bytes, void *stream);

int avion_attn_bwd_dkdv(const void *q, const void *k, const void *v, const float *lse,
                        const void *dO, void *dk, void *dv, int B, int H, int N, int d, float scale,
                        const void *workspace, size_t workspace_bytes, void *stream);

/*
 * Packed-QKV variants: the attention of an encoder layer sits right after the layer's joint
 * query/key/value projection (Sec. 3, "Video Transformer": each layer is a multi-head
 * self-attention on the N tokens), whose output is one tensor.  These take that tensor as it is,
 * so no copy splits it first, and return the gradient in the same packing, ready for the
 * projection's backward.
 *   qkv   : in,  bf16 [B,N,3,H,d] contiguous: plane 0 = queries, 1 = keys, 2 = values
 *           (token stride 3*H*d elements, plane stride H*d, head stride d)
 *   o, dO : bf16 [B,N,H,d];  lse : fp32 [B,H,N]   (as in the unpacked calls)
 *   dqkv  : out, bf16 [B,N,3,H,d], fully overwritten (planes dQ, dK, dV); must not alias qkv
 * Everything else -- alignment, workspace (same size as avion_attn_bwd_workspace_bytes), stream,
 * errors, arithmetic -- is as in avion_attn_fwd / avion_attn_bwd; the same kernels run, with a
 * token stride of 3*H*d for the packed tensors, and give bit-identical results.  The shape limit
 * becomes (N + 256) * 3*H*d * 2 bytes < 2^31.
 */
int avion_attn_fwd_qkvpacked(const void *qkv, void *o, float *lse,
                             int B, int H, int N, int d, float scale, void *stream);

int avion_attn_bwd_qkvpacked(const void *qkv, const void *o, const float *lse, const void *dO,
                             void *dqkv, int B, int H, int N, int d, float scale,
                             void *workspace, size_t workspace_bytes, void *stream);

/*
 * fp16 variants: the same operation on IEEE half-precision tensors, the type the paper's
 * throughput and maximum-batch-size figure was measured in (its caption names torch.float16; the
 * training setup in the implementation details uses automatic mixed precision).  Every tensor that is bf16 above is
 * fp16 here (q, k, v, o, dO, dq, dk, dv); lse and the workspace are unchanged.  Same kernels with
 * the fp16 MFMA; P and dS are rounded to fp16 before they enter a contraction, outputs once at the
 * final store; accumulation and statistics stay fp32.  fp16 has 5 exponent bits: the caller's
 * values must be representable (|x| <= 65504, gradients not below ~6e-8 in magnitude unless loss
 * scaling has lifted them), as with any fp16 attention; inside the kernels the softmax weights
 * are kept below 2^15 (a row that would exceed it takes the running-maximum path), P <= 1 in the
 * backward pass.
 */
int avion_attn_fwd_f16(const void *q, const void *k, const void *v, void *o, float *lse,
                       int B, int H, int N, int d, float scale, void *stream);

int avion_attn_bwd_f16(const void *q, const void *k, const void *v, const void *o, const float *lse,
                       const void *dO, void *dq, void *dk, void *dv,
                       int B, int H, int N, int d, float scale,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * Causal variants, for the text side of the paper's video-language model: its text encoder is a
 * GPT-like Transformer over at most 77 tokens (implementation details of the video-language model),
 * i.e. token i attends to tokens 0..i.  Same tensors, layouts, workspace and rules as
 * avion_attn_fwd / avion_attn_bwd (bf16); the softmax of query i runs over keys j <= i only:
 *     P_ij = exp(s_ij - LSE_i) for j <= i, 0 otherwise;  LSE_i = ln sum_{j<=i} exp(s_ij)
 * and every formula of the header's first comment holds with that P.  Blocks of keys that no query
 * of a wavefront sees are skipped, blocks on the diagonal are masked; nothing N x N is stored.
 */
int avion_attn_fwd_causal(const void *q, const void *k, const void *v, void *o, float *lse,
                          int B, int H, int N, int d, float scale, void *stream);

int avion_attn_bwd_causal(const void *q, const void *k, const void *v, const void *o,
                          const float *lse, const void *dO, void *dq, void *dk, void *dv,
                          int B, int H, int N, int d, float scale,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * General forms: every combination of element format, masking and tensor packing that the kernels
 * are instantiated for (the entry points above are the common cases of these two).  `flags` is a
 * bitwise OR of:
 *   AVION_FLAG_F16       tensors are fp16 instead of bf16 (as avion_attn_*_f16: the precision of the
 *                        paper's throughput figure)
 *   AVION_FLAG_CAUSAL    query i attends to keys 0..i (as avion_attn_*_causal: the GPT-like text
 *                        encoder of the video-language model)
 *   AVION_FLAG_QKVPACKED `q` is the [B,N,3,H,d] output of the joint projection (Sec. 3, "Video
 *                        Transformer") and `dq` receives the gradient in the same packing; k, v,
 *                        dk, dv must then be NULL (AVION_EINVAL otherwise)
 * Any other bit set returns AVION_EINVAL.  All other arguments, limits, workspace size and error
 * behaviour are those of avion_attn_fwd / avion_attn_bwd; the results are bit-identical to the
 * specific entry point where one exists.
 */
#define AVION_FLAG_F16 1u
#define AVION_FLAG_CAUSAL 2u
#define AVION_FLAG_QKVPACKED 4u

int avion_attn_fwd_ex(const void *q, const void *k, const void *v, void *o, float *lse,
                      int B, int H, int N, int d, float scale, unsigned flags, void *stream);

int avion_attn_bwd_ex(const void *q, const void *k, const void *v, const void *o, const float *lse,
                      const void *dO, void *dq, void *dk, void *dv,
                      int B, int H, int N, int d, float scale, unsigned flags,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * Layer normalisation over the channel axis, forward and backward: the per-token normalisation in
 * front of the attention and of the MLP of every encoder layer (Sec. 3, "Video Transformer"), and
 * one of the three entries of the paper's memory profile (Sec. 4.1).  Per token row x in R^D:
 *     mu = mean(x), var = mean((x - mu)^2), rstd = 1/sqrt(var + eps),
 *     y = (x - mu) * rstd * gamma + beta
 *     dbeta = sum_rows dy;  dgamma = sum_rows dy * xhat;  g = dy * gamma;
 *     dx = rstd * (g - mean(g) - xhat * mean(g * xhat)),      xhat = (x - mu) * rstd
 *   x, y, dy, dx   : bf16 (fp16 with AVION_FLAG_F16, the only flag accepted) [M, D] contiguous, device
 *   gamma, beta, dgamma, dbeta : fp32 [D], device;  mean, rstd : fp32 [M], device
 *   M >= 1 rows (tokens of all clips); D a multiple of 8, at most 2048; eps finite and >= 0
 *   workspace (backward): 256-byte aligned, avion_layernorm_bwd_workspace_bytes(M, D) bytes (the
 *   workgroups' partial sums of dgamma and dbeta: at most 1024 * 2 * D floats, independent of M)
 * What the backward needs from the forward is x and two floats per row -- the O(N D) activation
 * memory the paper's profile lists for this layer.  Pointers 16-byte aligned; same stream, error
 * and ownership rules as every entry point above.  Statistics and sums in fp32, outputs rounded
 * once; no atomics, results are bit-reproducible.
 */
int avion_layernorm_fwd(const void *x, const float *gamma, const float *beta, void *y,
                        float *mean, float *rstd, long long M, int D, float eps,
                        unsigned flags, void *stream);

size_t avion_layernorm_bwd_workspace_bytes(long long M, int D);

int avion_layernorm_bwd(const void *x, const float *gamma, const float *mean, const float *rstd,
                        const void *dy, void *dx, float *dgamma, float *dbeta,
                        long long M, int D, unsigned flags,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * Bias + GELU, forward and backward: the elementwise step between the two matrix products of the
 * encoder's 2-layer MLP (Sec. 3, "Video Transformer"), the third entry of the paper's memory
 * profile (Sec. 4.1, figure "memory footprint").  The paper names no activation; this is the
 * exact (erf) GELU of the plain ViT.  Per element, with h = x + bias_c:
 *     y  = h * Phi(h)                       Phi = standard normal distribution function
 *     dx = dy * (Phi(h) + h * phi(h))       phi = its density
 *     dbias_c = sum over rows of dx_c       (from the fp32 dx, before it is rounded)
 *   x, dy    : in,  bf16 (fp16 with AVION_FLAG_F16, the only flag accepted) [M, F] contiguous;
 *              x is the first matrix product's output WITHOUT the bias
 *   bias     : in,  fp32 [F];   dbias : out, fp32 [F], fully overwritten
 *   y, dx    : out, same format and shape as x, fully overwritten; may not alias the inputs
 *   M >= 1 rows (tokens); F % 8 == 0, F <= 65536 (else AVION_EUNSUPPORTED)
 *   workspace (backward): 256-byte aligned, avion_bias_gelu_bwd_workspace_bytes(M, F) bytes
 *   (partial sums of dbias: at most 4096 * 1024 floats, independent of M)
 * The backward rebuilds Phi and phi from x and bias, so the activation's output need not be kept
 * for it: with it the MLP keeps F * 2 bytes per token for this step instead of 2 * F * 2 (the
 * second matrix product's own input is rebuilt by one more avion_bias_gelu_fwd when its weight
 * gradient is formed).  erf by a five-term rational approximation with absolute error < 1.5e-7,
 * arithmetic in fp32, outputs rounded once; no atomics, results are bit-reproducible.
 * Pointers 16-byte aligned; same stream, error and ownership rules as every entry point above.
 */
int avion_bias_gelu_fwd(const void *x, const float *bias, void *y, long long M, int F,
                        unsigned flags, void *stream);

size_t avion_bias_gelu_bwd_workspace_bytes(long long M, int F);

int avion_bias_gelu_bwd(const void *x, const float *bias, const void *dy, void *dx, float *dbias,
                        long long M, int F, unsigned flags,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * Allocation-free backward, for callers that cannot provide device scratch of their own: code
 * under HIP graph capture, tight serving or training loops, harnesses that forbid hipMalloc.
 * Same operation, arguments, rules and bits as avion_attn_bwd (bf16, not causal), without the
 * workspace: the per-query scalars that the two passes exchange live in a 32 MiB array that is
 * part of the library's device image (one copy per GPU, held until the process ends).
 *   - Limit: avion_attn_bwd_workspace_bytes(B, H, N, d) <= 32 MiB, i.e.
 *     B*H*ceil(N/64)*64 <= 4 194 304 rows; larger problems return AVION_ESCRATCH and launch nothing.
 *   - Calls no hipMalloc, hipFree or other allocating routine.  The first call on a device looks
 *     up the array's address on that device (hipGetSymbolAddress) and keeps it; make that first
 *     call outside a graph capture.
 *   - All calls on one GPU share that GPU's array: two calls that overlap in time on the same GPU
 *     (different streams, different threads) race on it.  Calls on one stream are ordered and safe.
 *     Nothing in the array has to survive between calls and nothing needs clearing: each call
 *     writes every entry it later reads.
 */
int avion_attn_bwd_noalloc(const void *q, const void *k, const void *v, const void *o,
                           const float *lse, const void *dO, void *dq, void *dk, void *dv,
                           int B, int H, int N, int d, float scale, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* AVION_ATTN_H */
