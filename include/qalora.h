/*
 * qalora.h -- C ABI of the MI355X (gfx950) QA-LoRA adapted linear layer.
 *
 * The layer (arXiv 2309.14717, Sec. 3.3, Alg. 1, App. B), 0-based indices:
 *
 *   W~[i,j] = alpha[i/g, j] * code[i,j] + beta[i/g, j]            (Eq. 1 per group)
 *   y       = x W~ + s * (pool_g(x) A) B                          (Alg. 1 forward)
 *   pool_g(x)[t,l] = (1/g) * sum_{q<g} x[t, l*g+q]                (group AVERAGE)
 *
 * W is [d_in x d_out]; every column is cut into L = d_in/g groups of g consecutive
 * input rows, each with its own scaling factor alpha and zero factor beta.  A is
 * [L x rank], B is [rank x d_out].  The paper pools by SUM; a caller who wants that
 * passes s*g as s.  beta is Eq. 1's zero FACTOR in weight units (beta = group
 * minimum after quantize), not the zero point of Alg. 1 / App. B.1; the two are
 * related by z = -beta/alpha.
 *
 * Conventions for every entry point
 *   - All pointers are DEVICE pointers unless marked "host".  All matrices are dense
 *     row-major with no padding.  The descriptor is a host struct, read during the call.
 *   - The caller owns every buffer.  The library allocates nothing, frees nothing and
 *     never synchronises: work is enqueued on `stream` (a hipStream_t passed as void*;
 *     NULL = the default stream) and the results are ready when that stream reaches the
 *     end of the enqueued work.  No state that affects a result is kept between calls
 *     (the only process state is a call counter that tags flags in the workspace, one bit
 *     per kernel and device noting that its dynamic-LDS attribute has been set, the device
 *     address of qalora_forward_noalloc's built-in scratch array, and whatever the
 *     qalora_profile_* measurement aids armed).
 *   - Scratch memory comes from the caller through (ws, ws_bytes); ask
 *     qalora_workspace_bytes for the size (forward and backward always need some, at least
 *     8 bytes per token).  ws contents are undefined afterwards.  Two calls that may run
 *     at the same time (different streams) must not share a workspace.
 *   - Stream capture: forward, backward and merge -- and the _keep / _kept, _shared,
 *     _deployed and _noalloc forms -- may be captured into a HIP graph and
 *     replayed (they enqueue kernels only: no memset, copy, allocation or event unless
 *     qalora_profile_arm armed one).  Make one eager call of the same shape first: the
 *     first use of a kernel sets its dynamic-LDS attribute, which is not stream work.  The
 *     workspace passed at capture is used by every replay.
 *   - Inputs are read-only.  Outputs must not alias inputs unless stated.
 *   - Device pointers must be 16-byte aligned (QALORA_EALIGN otherwise).
 *   - Every entry returns a status (0 = QALORA_OK, negative = error).  Argument errors
 *     are detected on the host before anything is launched; no partial work is
 *     enqueued in that case.  Nothing throws.
 *   - Supported shapes: bits in {2,3,4}; group dividing d_in and a multiple of 8 (4-bit),
 *     16 (2-bit) or 32 (3-bit); d_out a multiple of 8; rank at most 128; for forward and
 *     backward, the packed codes, alpha (beta), and tokens (rounded up to 256) x
 *     max(d_in, d_out) x 2 bytes each below 0xf0000000 bytes (the kernels use 32-bit byte
 *     offsets).  Anything else that is well-formed returns QALORA_EUNSUPPORTED -- there is
 *     no fallback path.
 *   - Results are deterministic: a rerun on the same inputs is bit-identical.
 */
#ifndef QALORA_H_
#define QALORA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* One QA-LoRA linear layer (header of Alg. 1).  Plain data, caller-owned, host. */
typedef struct qalora_desc {
  int32_t d_in;  /* input features  D_in  (rows of W)                      */
  int32_t d_out; /* output features D_out (columns of W)                   */
  int32_t bits;  /* N, code width: codes are in {0 .. 2^N - 1}   (Eq. 1)   */
  int32_t group; /* g = D_in / L, rows per quantization group (Sec. 3.3)   */
  int32_t rank;  /* D_int, adapter rank; 0 = no adapter                    */
  float s;       /* adapter coefficient (Sec. 3.1), with average pooling   */
} qalora_desc;

enum qalora_status {
  QALORA_OK = 0,
  QALORA_EINVAL = -1,       /* null pointer, bad enum, bits/group/rank/tokens out of range,
                               group does not divide d_in, exactly one of A/B null */
  QALORA_EALIGN = -2,       /* a device pointer is not 16-byte aligned              */
  QALORA_EWORKSPACE = -3,   /* ws is null or smaller than qalora_workspace_bytes    */
  QALORA_EUNSUPPORTED = -4, /* well-formed, but outside the supported shapes        */
  QALORA_EHIP = -5          /* a launch failed; hipGetLastError() is left in place  */
};

enum qalora_dtype { QALORA_F32 = 0, QALORA_BF16 = 1 };

enum qalora_op {
  QALORA_OP_QUANTIZE = 0,
  QALORA_OP_FORWARD = 1,
  QALORA_OP_BACKWARD = 2,
  QALORA_OP_MERGE = 3,
  QALORA_OP_FORWARD_FACTORS16 = 4,
  QALORA_OP_QUANTIZE_COMPENSATED = 5
};

/* Human-readable name of a status code (static string, host). */
const char* qalora_status_string(int status);

/* Validate a descriptor on the host.  Returns QALORA_OK, QALORA_EINVAL or
 * QALORA_EUNSUPPORTED exactly as the compute entry points would. */
int qalora_check_desc(const qalora_desc* desc);

/* Size in bytes of the packed-code buffer for this layer (0 if the descriptor is
 * invalid).  The packed format is private to the library (codes are bit-packed
 * N bits each, eight consecutive input rows of one column per field); its meaning is
 * defined by qalora_unpack. */
size_t qalora_packed_bytes(const qalora_desc* desc);

/* Scratch bytes the given operation needs for `tokens` tokens (tokens is ignored by
 * QUANTIZE and MERGE).  Returns 0 for an invalid descriptor or op. */
size_t qalora_workspace_bytes(const qalora_desc* desc, int tokens, int op);

/* Group-wise min-max quantization: Eq. 1 applied to each group of g consecutive rows
 * of each column (Sec. 3.3).  In fp32, in this order:
 *   beta = min, alpha = (max - min) / (2^N - 1)   (one subtract, one IEEE divide),
 *   code = clamp(rint((w - beta) / alpha), 0, 2^N - 1)   (ties to even);
 *   a group whose alpha is not > 0 (constant group) gets alpha = 2^-60 and codes 0.
 * in : W      fp32 [d_in, d_out]
 * out: packed  qalora_packed_bytes(desc) bytes
 *      alpha, beta  fp32 [L, d_out]
 * rank and s of the descriptor are ignored.  Non-finite W gives unspecified codes. */
int qalora_quantize(const qalora_desc* desc, const float* W, void* packed, float* alpha,
                    float* beta, void* ws, size_t ws_bytes, void* stream);

/* Error-compensated code selection, the role the post-training quantizer plays in the paper's
 * experiments (Sec. 4.1, quantization settings; App. B.1): same outputs as qalora_quantize, but
 * the codes are chosen to reduce the layer's OUTPUT error tr((W - W~)^T H (W - W~)) under a given
 * input Hessian H instead of rounding every weight to its nearest level.
 * in : W fp32 [d_in, d_out]; hinv_chol fp32 [d_in, d_in] row-major, the upper-triangular
 *      Cholesky factor U of the inverse Hessian (H^-1 = U^T U; only the upper triangle is read).
 *      Computing H from calibration inputs and factorising it is the caller's business.
 * The input rows are quantized in order; at the first row of a group beta = min and
 * alpha = (max - min) / (2^N - 1) are taken from the group's rows as they then stand (Eq. 1's
 * recipe); code = clamp(rint((w - beta) / alpha)); e = (w - (alpha code + beta)) / U[i,i]; every
 * later row r receives w_r -= U[i,r] e, rows beyond the current block of 128 in one lazy
 * update per block (sums in ascending row order, fused multiply-adds, fp32): with this order
 * fixed the result is reproducible bit for bit.  U = identity gives qalora_quantize's result.
 * group must divide 128 (QALORA_EUNSUPPORTED otherwise).
 * Workspace: qalora_workspace_bytes(.., QALORA_OP_QUANTIZE_COMPENSATED) = 5 bytes per weight. */
int qalora_quantize_compensated(const qalora_desc* desc, const float* W, const float* hinv_chol,
                                void* packed, float* alpha, float* beta, void* ws, size_t ws_bytes,
                                void* stream);

/* packed -> canonical codes, uint8 [d_in, d_out] row-major, one code per byte.
 * This is the definition of the packed format ("bit-exact codes" means equal here). */
int qalora_unpack(const qalora_desc* desc, const void* packed, uint8_t* codes, void* stream);

/* canonical codes -> packed; imports codes chosen by any other quantizer (the layer
 * accepts any (codes, alpha, beta) triple).  Codes above 2^N - 1 are masked to N bits. */
int qalora_pack(const qalora_desc* desc, const uint8_t* codes, void* packed, void* stream);

/* Adapted forward, Alg. 1 / App. B.2:   y = x W~ + s (pool_g(x) A) B.
 * in : x bf16 [tokens, d_in]; packed; alpha, beta fp32 [L, d_out];
 *      A fp32 [L, rank], B fp32 [rank, d_out] -- both NULL (or rank 0) for the
 *      adapter-free layer, e.g. after qalora_merge (then s is ignored).
 * out: y [tokens, d_out], fp32 or bf16 per y_dtype (bf16 = round-to-nearest-even of the
 *      fp32 result).
 * Precision: x is used exactly (each token row is scaled by a power of two and converted to
 * fp16); accumulation is fp32.  The adapter is folded into the zero factors for the call,
 * beta' = beta + (s/g) A B (App. B.3, fp32), and the weight is rebuilt around the mid code
 * mid = 2^(N-1) from two fp16 factors per (group, column), scaled by a power of two so that
 * the conversion keeps 11 significant bits at any magnitude:
 *     W~' = fp16(alpha) (code - mid) + fp16(beta' + mid alpha),
 * so per element |error| <= 2^-11 (|beta' + mid alpha| + |alpha (code - mid)|).  For min-max
 * triples (qalora_quantize, qalora_quantize_compensated) that is 2^-11 of the group's largest
 * |W~|; for imported triples whose used codes sit far from the mid code (say codes all 0,
 * alpha = 1, beta = v) the bound is what it says: 2^-11 |v + mid|, not 2^-11 |v|.  The
 * adapter's contribution passes through the same constant: with alpha = beta = 0 it is
 * evaluated to 2^-11 relative.  Without an adapter, for
 * tokens <= 16 (<= 32 for 4-bit codes), group 32/64/128 and d_in a multiple of 128, a
 * streaming kernel takes over (one column per lane for tokens <= 4 and for the 2- and 3-bit
 * codes, a sixteen-token tile -- two of them beyond sixteen tokens -- for 4-bit codes) whose
 * operands are exact (only the fp32 accumulation
 * order differs from the definition); its cross-block sum waits on flags with a bound -- should a
 * wait ever run out (another kernel holding the compute units for ~0.3 s) the affected outputs
 * are NaN and the kernel sets the 64-bit word at byte QALORA_WS_STATUS_OFFSET of ws to a non-zero
 * value.  The library only ever sets that word: a caller who wants the status zeroes it once
 * (e.g. when allocating ws) and reads it after the stream has completed; after a non-zero
 * status the first QALORA_WS_STATUS_OFFSET bytes of ws must be zeroed before ws is used again
 * (a late flag of the failed call may still be there). */
#define QALORA_WS_STATUS_OFFSET 2048
int qalora_forward(const qalora_desc* desc, int tokens, const void* x, const void* packed,
                   const float* alpha, const float* beta, const float* A, const float* B,
                   void* y, int y_dtype, void* ws, size_t ws_bytes, void* stream);

/* For callers that cannot allocate or carry a workspace -- code under HIP graph capture, tight
 * decode loops, harnesses that forbid hipMalloc: qalora_forward for the adapter-free few-token
 * regime (A = B = NULL; tokens <= QALORA_NOALLOC_MAX_TOKENS; shapes of the streaming kernel:
 * group 32/64/128, d_in a multiple of 128) with the flags and partial sums of the cross-block
 * sum in a device array built into the library (QALORA_NOALLOC_SCRATCH_BYTES per GPU, held from
 * first use until the process ends) instead of a caller workspace.  Anything beyond that
 * returns QALORA_EUNSUPPORTED; nothing is allocated, freed or synchronised.  Same kernels and
 * results, bit for bit, as qalora_forward.  All calls on one GPU share that array: calls that
 * may overlap on one GPU (different streams or threads) race -- serialise them or use
 * qalora_forward with a workspace per stream.  The first call on each device looks up the
 * array's address (not stream work: make it outside graph capture, like the first call of any
 * kernel here).  A wait that runs out gives NaN outputs, as above. */
#define QALORA_NOALLOC_MAX_TOKENS 16
#define QALORA_NOALLOC_SCRATCH_BYTES (2304 + 256 * 16 * 512 * 4)
int qalora_forward_noalloc(const qalora_desc* desc, int tokens, const void* x, const void* packed,
                           const float* alpha, const float* beta, void* y, int y_dtype,
                           void* stream);

/* Backward of qalora_forward with W~ frozen: only A and B are parameters (Alg. 1),
 * so with G = dy, P = pool_g(x), U = P A:
 *   dU = s G B^T,  dB = s U^T G,  dA = P^T dU,
 *   dx[t,i] = sum_j G[t,j] W~[i,j] + (dU A^T)[t, i/g] / g.
 * in : dy bf16 [tokens, d_out]; x bf16 [tokens, d_in]; packed, alpha, beta, A, B as above
 *      (A = B = NULL: only dx is produced, dA and dB are not touched).
 * out: dx [tokens, d_in] fp32 or bf16 per dx_dtype, or NULL to skip it;
 *      dA fp32 [L, rank], dB fp32 [rank, d_out]; accumulate = 0 overwrites them,
 *      accumulate = 1 adds to their current contents (gradient accumulation). */
int qalora_backward(const qalora_desc* desc, int tokens, const void* dy, const void* x,
                    const void* packed, const float* alpha, const float* beta,
                    const float* A, const float* B, void* dx, int dx_dtype, float* dA,
                    float* dB, int accumulate, void* ws, size_t ws_bytes, void* stream);

/* The pair above for training loops that keep the pooled activations instead of x.  The
 * backward needs x only through P = pool_g(x) and U = P A (Alg. 1; App. B.2: the adapter sees
 * the group averages, never x itself), which are g times smaller than x.
 * qalora_forward_keep is qalora_forward (adapter required) that also leaves them in `kept`:
 * device memory of qalora_kept_bytes(desc, tokens) bytes, 16-byte aligned, contents private to
 * the library and valid for a backward call with the same desc, tokens, A and B.
 * qalora_backward_kept is qalora_backward reading `kept` in place of x: same results bit for
 * bit, one read of x less, and the caller may release x after the forward.
 * qalora_kept_bytes returns 0 for an invalid descriptor, tokens <= 0 or rank 0.
 * Workspace sizes are those of QALORA_OP_FORWARD and QALORA_OP_BACKWARD. */
size_t qalora_kept_bytes(const qalora_desc* desc, int tokens);
int qalora_forward_keep(const qalora_desc* desc, int tokens, const void* x, const void* packed,
                        const float* alpha, const float* beta, const float* A, const float* B,
                        void* y, int y_dtype, void* kept, void* ws, size_t ws_bytes,
                        void* stream);
int qalora_backward_kept(const qalora_desc* desc, int tokens, const void* dy, const void* kept,
                         const void* packed, const float* alpha, const float* beta,
                         const float* A, const float* B, void* dx, int dx_dtype, float* dA,
                         float* dB, int accumulate, void* ws, size_t ws_bytes, void* stream);

/* Several adapted linears that share their input x (q/k/v of an attention block; gate/up of a
 * SwiGLU MLP), evaluated as ONE wide layer: one pass over x (row scales, conversion, pooling --
 * pool_g(x) is the same for all of them), one dense launch over the concatenated columns, and
 * in the backward one contraction dx = dy W~'^T over all of them, which IS the sum of the
 * linears' input gradients.  Each linear keeps its own adapter (Alg. 1: A, B and s per layer),
 * folded into its own columns of the zero factors.
 * The wide layer: desc (d_out = sum of the parts' widths; rank and s of desc are ignored);
 * packed, alpha, beta of the column-wise concatenation [W_0 | W_1 | ...] -- quantization is per
 * column (Eq. 1 per group of a column), so quantizing the concatenation is concatenating the
 * quantizations; y and dy are [tokens, d_out] with part p at columns [col0_p, col0_p + d_out_p).
 * parts: HOST array of n_parts (1 .. QALORA_MAX_PARTS) entries; A [L, rank], B [rank, d_out],
 * dA, dB are device pointers (dA, dB only used, and required, by the backward).  Every width
 * must be a multiple of 32 and every rank in 1..128 (QALORA_EUNSUPPORTED otherwise); the widths
 * must add up to desc->d_out (QALORA_EINVAL).
 * kept: as in qalora_forward_keep / qalora_backward_kept (qalora_shared_kept_bytes); NULL in
 * the forward keeps nothing, NULL in the backward re-reads x (then required).
 * Results per part are those of the single-layer calls on that part, to rounding order: the
 * forward's words are scaled per column either way (bit-identical y), the backward's one scale
 * per call is taken over the wide layer. */
#define QALORA_MAX_PARTS 4
typedef struct qalora_part {
  int32_t d_out; /* width of this linear (columns of the wide layer, in order)   */
  int32_t rank;  /* its adapter rank                                             */
  float s;       /* its adapter coefficient                                      */
  const float* A;
  const float* B;
  float* dA;
  float* dB;
} qalora_part;
size_t qalora_shared_kept_bytes(const qalora_desc* desc, int tokens, int n_parts, const qalora_part* parts);
size_t qalora_shared_workspace_bytes(const qalora_desc* desc, int tokens, int op, int n_parts,
                                     const qalora_part* parts);
int qalora_forward_shared(const qalora_desc* desc, int tokens, const void* x, const void* packed,
                          const float* alpha, const float* beta, int n_parts, const qalora_part* parts,
                          void* y, int y_dtype, void* kept, void* ws, size_t ws_bytes, void* stream);
int qalora_backward_shared(const qalora_desc* desc, int tokens, const void* dy, const void* x,
                           const void* kept, const void* packed, const float* alpha, const float* beta,
                           int n_parts, const qalora_part* parts, void* dx, int dx_dtype, int accumulate,
                           void* ws, size_t ws_bytes, void* stream);

/* Merge the adapter into the zero factors (Alg. 1 merge, App. B.3, in Eq. 1's
 * convention):  beta_out[l,j] = beta[l,j] + (s/g) * sum_k A[l,k] B[k,j].
 * Codes and alpha are untouched, so the merged layer is still N-bit.
 * beta_out may alias beta.  Needs no workspace. */
int qalora_merge(const qalora_desc* desc, const float* beta, const float* A, const float* B,
                 float* beta_out, void* stream);

/* Deployment of the merged model (Sec. 3.3: after the merge the layer is a plain N-bit layer
 * again, and static; App. B.3).  qalora_deploy derives, once, what every later call would
 * otherwise rebuild or gather, into `deployed` (qalora_deployed_bytes; about 1.17 x the size of
 * packed + alpha + beta):
 *   - a decode stream: the codes and fp32 factors of every 64 columns x 128 rows together, in
 *     the order the decode kernel consumes them (16-byte accesses over contiguous records);
 *   - the dense kernel's fp16 factor words and their column scales.
 * qalora_forward_deployed is the adapter-free forward from it: up to
 * QALORA_DEPLOYED_STREAM_TOKENS tokens the decode kernel on the stream (`packed` is not read
 * and may be NULL; same arithmetic and results, bit for bit, as qalora_forward on the triple);
 * beyond that the dense contraction on `packed` (required) with the prepared words (results
 * as qalora_forward, bit for bit, without its per-call factor pass).  Five to thirty-two
 * tokens are served faster by qalora_forward on the original triple, which has a streaming
 * kernel for them.  Supported: bits 4, group 32/64/128, d_in a multiple of 128; otherwise
 * QALORA_EUNSUPPORTED (qalora_deployed_bytes returns 0).  Workspace: that of
 * QALORA_OP_FORWARD; status word as for qalora_forward. */
#define QALORA_DEPLOYED_STREAM_TOKENS 4
size_t qalora_deployed_bytes(const qalora_desc* desc);
int qalora_deploy(const qalora_desc* desc, const void* packed, const float* alpha, const float* beta,
                  void* deployed, void* stream);
int qalora_forward_deployed(const qalora_desc* desc, int tokens, const void* x, const void* packed,
                            const void* deployed, void* y, int y_dtype, void* ws, size_t ws_bytes,
                            void* stream);

/* 16-bit storage of the quantization factors for inference on the merged model, where every
 * call streams the whole weight (Sec. 3.3 deployment; App. B.3): one 32-bit word per
 * (group, column), fp16(alpha) in the low half and fp16(beta) in the high half, each rounded to
 * nearest even.  At INT4, g = 32 this takes a quarter off the bytes of a call.  It is a lossy
 * re-encoding of the layer (11 significant bits per factor): the layer it defines is
 * W~ = fp16(alpha) code + fp16(beta), and that is what qalora_forward_factors16 computes.
 * in : alpha, beta fp32 [L, d_out]      out: factors16, 4 * L * d_out bytes. */
int qalora_pack_factors16(const qalora_desc* desc, const float* alpha, const float* beta,
                          void* factors16, void* stream);

/* Adapter-free forward y = x W~ of a layer whose factors are stored as above; otherwise as
 * qalora_forward with A = B = NULL.  In the few-token regime (conditions as for qalora_forward) the
 * streaming kernel reads the 16-bit factors directly; beyond that they are expanded to fp32
 * in the workspace first.  Workspace: qalora_workspace_bytes(.., QALORA_OP_FORWARD_FACTORS16). */
int qalora_forward_factors16(const qalora_desc* desc, int tokens, const void* x,
                             const void* packed, const void* factors16, void* y, int y_dtype,
                             void* ws, size_t ws_bytes, void* stream);

/* Zero-point interchange.  Alg. 1 (`pre_quantization`, `merge_with_quantization`) and App. B.1
 * write the de-quantized weight as W~ = alpha (code - z) with a zero POINT z in code units
 * (an integer out of a post-training quantizer, real-valued after a merge); this library
 * keeps Eq. 1's zero FACTOR beta, W~ = alpha code + beta.  They name the same weights iff
 *   beta = -(alpha z)          (qalora_beta_from_zero_point: import a (codes, scales, zeros) model)
 *   z    = -(beta / alpha)     (qalora_zero_point_from_beta: export; applied to the beta' of
 *                               qalora_merge it yields App. B.3's z' = z - (s/g) (A B) / alpha)
 * one IEEE fp32 operation per element, so import then export returns z to within 2 ulp.
 * in / out: fp32 [L, d_out]; the output may alias the input it is computed from.
 * alpha = 0 gives a non-finite z (qalora_quantize never produces it).  No workspace. */
int qalora_beta_from_zero_point(const qalora_desc* desc, const float* alpha, const float* z,
                                float* beta, void* stream);
int qalora_zero_point_from_beta(const qalora_desc* desc, const float* alpha, const float* beta,
                                float* z, void* stream);

/* The optimiser step that follows qalora_backward in the fine-tuning loop (Sec. 4.1, training
 * details: AdamW, a maximum gradient norm of 0.3, a constant learning rate; only A and B are
 * parameters, Sec. 3.1), fused over up to QALORA_ADAMW_MAX_TENSORS tensors -- e.g. the A and B
 * of every linear of a decoder layer -- in two launches.  With t = step (counted from 1):
 *   norm = joint L2 norm of all grads;  clip = min(1, max_grad_norm / (norm + 1e-6)), or 1 if
 *   max_grad_norm <= 0;  g = clip * grad;
 *   m = beta1 m + (1 - beta1) g;   v = beta2 v + (1 - beta2) g^2;
 *   p = p (1 - lr weight_decay) - lr (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps).
 * params, grads, exp_avg, exp_avg_sq: HOST arrays of n_tensors DEVICE pointers (fp32, numel[i]
 * elements each, 16-byte aligned); params, exp_avg, exp_avg_sq are updated in place; grads are
 * read, and set to zero afterwards if zero_grads != 0 (so that the next qalora_backward can
 * accumulate).  grad_norm: optional device float receiving the norm before clipping.
 * ws: qalora_adamw_workspace_bytes(n_tensors, numel) bytes (needed when clipping or when the
 * norm is asked for).  fp32 arithmetic, sums in a fixed order: a step is bit-reproducible. */
#define QALORA_ADAMW_MAX_TENSORS 32
typedef struct qalora_adamw {
  float lr, beta1, beta2, eps, weight_decay, max_grad_norm;
} qalora_adamw;
size_t qalora_adamw_workspace_bytes(int n_tensors, const size_t* numel);
int qalora_adamw_step(const qalora_adamw* hp, int step, int n_tensors, float* const* params,
                      float* const* grads, float* const* exp_avg, float* const* exp_avg_sq,
                      const size_t* numel, int zero_grads, float* grad_norm, void* ws,
                      size_t ws_bytes, void* stream);

/* Measurement aid (used by the benchmark, not part of the layer): arm a pair of HIP events
 * (hipEvent_t passed as void*, created by the caller with timing enabled).  The next dense
 * contraction kernel of the given direction (0 = the y = x W~ kernel of qalora_forward,
 * 1 = the dx = dy W~^T kernel of qalora_backward) launched by this process records `start`
 * right before and `stop` right after itself on its stream, then disarms.  Passing NULLs
 * disarms.  Process-wide and not thread safe; returns QALORA_EINVAL for a bad direction. */
int qalora_profile_arm(int direction, void* start_event, void* stop_event);

/* Measurement aid: which clock did the chip run the kernel at?  Call after qalora_profile_arm
 * for the same direction (arming events clears it): the armed dense contraction kernel then
 * also stores four 64-bit counts to `counts` (device, 32 bytes, 16-byte aligned) from its first
 * block: shader-clock cycles and constant-rate wall-clock ticks when the block starts, and both
 * again when it ends.  (cycles_end - cycles_start) / (ticks_end - ticks_start) x the wall-clock
 * rate (qalora_profile_wall_clock_khz; 100 MHz on this hardware) is the average shader clock
 * over that block's life -- under load well below the nominal 2.4 GHz that the published
 * matrix-core peak assumes.  The small-token kernel does not report.  NULL disarms. */
int qalora_profile_arm_clock(int direction, void* counts);

/* Measurement aid: the time line of a launch.  Call after qalora_profile_arm for the same
 * direction: every block b < capacity of the armed dense contraction kernel then stores four
 * 64-bit values to times[4b .. 4b+3] (device, 32 * capacity bytes, 16-byte aligned): wall-clock
 * ticks when it started, when it left the K loop and when it ended, and the id (0..7) of the
 * XCD it ran on.  Blocks >= capacity store nothing; slices of a split-K launch other than the
 * first store nothing.  NULL disarms; capacity <= 0 with a buffer is QALORA_EINVAL. */
int qalora_profile_arm_blocks(int direction, void* times, int capacity);
int qalora_profile_wall_clock_khz(int* khz /* host */);

/* Create / time / destroy timing events for qalora_profile_arm (thin wrappers over
 * hipEventCreate, hipEventElapsedTime, hipEventDestroy so that a caller without HIP
 * headers can use the aid).  elapsed_ms requires both events to have completed. */
int qalora_profile_event_create(void** event);
int qalora_profile_event_elapsed_ms(void* start_event, void* stop_event, float* ms);
int qalora_profile_event_destroy(void* event);

/* Measurement aid: a plain device-to-device copy kernel of `bytes` bytes (a multiple of 16; both
 * pointers 16-byte aligned, buffers must not overlap).  It reads and writes exactly `bytes` of
 * HBM once, which makes it the yardstick the hardware traffic counters are scaled by. */
int qalora_profile_copy(void* dst, const void* src, size_t bytes, void* stream);

/* Measurement aid: an issue-rate probe of the matrix cores.  `blocks` blocks each run `iters` K
 * steps (64 deep) of the inner loop of a dense contraction with only the instruction mix left:
 * v_mfma_f32_32x32x16_f16 on register accumulators, with (lds_reads = 1) or without the operand
 * fragment reads from LDS, and valu_per_mfma ordinary vector instructions behind every matrix
 * instruction.  shape 0: eight wavefronts of 4 x 2 tiles per block (valu_per_mfma in
 * {0,1,2,3,4,6,8}, and 102 / 104: two / four per matrix instruction issued as one burst behind
 * the eight matrix instructions of a K-16 slice; 0 only without LDS reads); shape 1: four
 * wavefronts of 4 x 4 tiles (valu in {0,2,4,6,8}); shape 2: shape 0 with the accumulators held
 * in AGPRs (valu in {0,2,4}).  Other combinations return QALORA_EINVAL.  Block b stores its shader cycles and
 * wall-clock ticks over the loop to counts[2b], counts[2b+1] (device, 16 * blocks bytes); sink
 * is device scratch of 2048 * blocks bytes.  A block issues iters * 32 (shape 0: per wavefront,
 * two wavefronts per SIMD; shape 1: iters * 64, one wavefront per SIMD) matrix instructions per
 * wavefront. */
int qalora_profile_mfma_probe(int shape, int lds_reads, int valu_per_mfma, int iters, int blocks,
                              void* sink, void* counts, void* stream);

/* Benchmark-harness glue, not part of the QA-LoRA layer: the elementwise part of a LLaMA
 * SwiGLU MLP block around three adapted linears (the MLP-block workload of the benchmark).
 *   forward : h[i] = silu(gate[i]) * up[i],  silu(v) = v / (1 + exp(-v))
 *   backward: dgate[i] = dh[i] * up[i] * d silu(gate[i]),  dup[i] = dh[i] * silu(gate[i])
 * All arrays bf16, n elements (n a multiple of 8, pointers 16-byte aligned); arithmetic in
 * fp32, results rounded to bf16.  Outputs must not alias inputs. */
int qalora_swiglu_forward(const void* gate, const void* up, void* h, size_t n, void* stream);
int qalora_swiglu_backward(const void* dh, const void* gate, const void* up, void* dgate,
                           void* dup, size_t n, void* stream);
/* The same glue on gu = [gate | up], one bf16 tensor [rows, 2 cols] as a wide gate/up layer
 * (qalora_forward_shared) produces it: h [rows, cols]; dgu = [dgate | dup] [rows, 2 cols], which
 * is the dy of qalora_backward_shared.  cols a multiple of 8. */
int qalora_swiglu_forward_wide(const void* gu, void* h, size_t rows, size_t cols, void* stream);
int qalora_swiglu_backward_wide(const void* dh, const void* gu, void* dgu, size_t rows, size_t cols,
                                void* stream);

#ifdef __cplusplus
}
#endif
#endif /* QALORA_H_ */
