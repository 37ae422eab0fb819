// Host-side launchers of the gfx950 kernels.  Everything here takes raw device pointers
// and a stream; argument validation and workspace carving happen in api.hip.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qalora {

// --- quantize.hip -------------------------------------------------------------------
void launch_quantize(int bits, const float* W, void* packed, float* alpha, float* beta, int d_in,
                     int d_out, int g, hipStream_t st);
void launch_unpack(int bits, const void* packed, uint8_t* codes, int d_in, int d_out,
                   hipStream_t st);
// fac16[i] = fp16(alpha[i]) | fp16(beta[i]) << 16 over n = L * d_out elements, and back
hipError_t launch_pack_factors(const float* alpha, const float* beta, void* fac16, size_t n, hipStream_t st);
hipError_t launch_unpack_factors(const void* fac16, float* alpha, float* beta, size_t n, hipStream_t st);
void launch_pack(int bits, const uint8_t* codes, void* packed, int d_in, int d_out,
                 hipStream_t st);

// --- compensate.hip: error-compensated code selection on a given inverse-Hessian factor ------
// work: d_in * d_out fp32 scratch; codes: canonical, one code per byte.  g must divide 128.
hipError_t launch_compensate(const float* W, const float* U, int d_in, int d_out, int bits, int g,
                             float* work, uint8_t* codes, float* alpha, float* beta, hipStream_t st);

// --- gemm_dq.hip --------------------------------------------------------------------
struct GemmArgs {
  const uint16_t* a_main;  // fp16 [M, K_main]: x (forward) or dy (backward), each row already
                           // multiplied by its power-of-two row scale
  int lda_main;
  int a_main_padded_rows;   // rows a_main may be read for (>= M; the rest holds anything)
  const uint16_t* a_tail;  // bf16 [M, K_tail]: first operand of a plain product (no main part)
  int lda_tail;
  const uint32_t* plane0;  // packed codes
  const uint32_t* plane1;
  const uint32_t* fac;     // [L, d_out] factor words: fp16(alpha S) | fp16((beta' + mid alpha) S) << 16
  const float* n_scale;    // 1 / S: [d_out] (forward, per column) or [1] (backward)
  const uint16_t* b_tail;  // bf16 [N, K_tail]: second operand of a plain product
  const float2* row_scale; // [M] (scale, 1/scale): power-of-two row scales of a_main
  void* out;               // [ksplit][M, N] fp32, or [M, N] bf16
  int out_bf16;
  float* partial;          // [ksplit][M, N] fp32 when ksplit > 1 (dequantising product)
  int ksplit;              // K slices of the dequantising product (0 or 1: none)
  int M, N;                // tokens; d_out (forward) or d_in (backward)
  int K_main;              // d_in (forward) or d_out (backward); 0 for a plain product
  int K_tail;              // multiple of 64 (zero padded), may be 0
  int d_in, d_out, group;
  unsigned long long* clock_probe;  // measurement aid (may be null): block 0 stores its shader
                                    // cycle and wall-clock tick counts at start and end, [4]
  unsigned long long* block_times;  // measurement aid (may be null): block b < block_times_cap
  int block_times_cap;              // stores wall-clock ticks at start, K loop end and end, and
                                    // the id of the XCD it ran on, [4 b .. 4 b + 3]
};
hipError_t launch_gemm_dq(int bits, bool bwd, const GemmArgs& a, hipStream_t st);
// K slices the dequantising product should use for an [M x K_main] x [K_main x N] problem.
int gemm_dq_ksplit(int M, int N, int K_main);
// Measurement aid: events recorded around the next launch_gemm_dq of each direction.
struct ProfileHook {
  hipEvent_t start, stop;
  unsigned long long* clock_probe;  // device, 4 x u64, or null
  unsigned long long* block_times;  // device, 4 x u64 per block, or null
  int block_times_cap;
};
extern ProfileHook g_profile_hook[2];
hipError_t launch_gemm_plain(const GemmArgs& a, int ksplit, hipStream_t st);
int gemm_plain_tile_rows(int K);  // row tile launch_gemm_plain uses for a K of this length

// --- smallt.hip ---------------------------------------------------------------------
// Adapter-free forward for T <= 16 tokens, INT4, group 32 / 64 / 128 (memory-bound path).
constexpr int ST_MAX_BLOCKS = 256; // one block per compute unit
constexpr int ST_PARTIAL_FLOATS = 16 * 512;  // one [16 tokens x widest slab] tile per block
// Head of the small-token workspace: one 64-bit flag per block, then one 64-bit status word that
// a kernel sets (and never clears) when a bounded wait for a flag ran out; partials follow.
constexpr size_t ST_STATUS_OFFSET = (size_t)ST_MAX_BLOCKS * 8;
constexpr size_t ST_HEAD_BYTES = ((ST_STATUS_OFFSET + 8 + 255) / 256) * 256;
struct SmallTArgs {
  const uint16_t* x;       // bf16 [T, d_in]
  const uint32_t* plane0;  // packed codes (INT3: the low two bits)
  const uint32_t* plane1;  // INT3: the plane of high bits; otherwise unused
  const float* alpha;      // [L, d_out]
  const float* beta;       // [L, d_out]
  const uint32_t* fac16;   // or, instead of both: [L, d_out] words fp16 alpha | fp16 beta << 16
  const void* stream;      // or, instead of planes and factors: the deployment stream (launch_deploy)
  void* out;               // [T, d_out] fp32 or bf16
  float* partial;          // [blocks][ST_PARTIAL_FLOATS] fp32: each block's [token][slab column] tile
  unsigned long long* flags;  // [blocks]: set to `nonce` once the block's partial is complete
  unsigned long long* status; // one word: set to a non-zero value if a wait for a flag ran out
  unsigned long long nonce;   // filled in by the launcher, unique per call
  int out_bf16;
  int T, d_in, d_out, group;
  int bits;  // 4, 3 or 2
};
// Launch shape: blocks = slabs * parts; `halves` (1 or 2) is how many ways a block splits its
// own chunks, which sets the slab width (512 or 256 columns).
struct SmallTPlan {
  int halves, slab_cols, slabs, parts, blocks;
};
SmallTPlan smallt_plan(int d_in, int d_out, int tokens);
hipError_t launch_smallt(const SmallTArgs& a, hipStream_t st);  // dispatches on T
unsigned long long smallt_next_nonce();  // unique per call of this process, never zero
// Deployment stream of a 4-bit layer (the static, merged model of Sec. 3.3 / App. B.3): for
// every group of 64 columns and every 128-row chunk one contiguous record of 16-byte units,
// unit u of lane (= column) at byte 1024 u + 16 lane: units 0..3 the column's sixteen code words
// of the chunk in row order, then the chunk's fp32 factors -- group 32: alpha of its four
// groups, beta of its four groups; group 64: alpha0 alpha1 beta0 beta1; group 128: alpha beta
// 0 0.  Records are ordered [chunk][column group]: the chip's wavefronts advance through the
// chunks together, so at any moment they sweep one contiguous region.
__host__ __device__ constexpr int s4_dep_units(int sub) { return sub == 1 ? 6 : 5; }
inline size_t deploy_stream_bytes(int d_in, int d_out, int group) {
  return (size_t)((d_out + 63) / 64) * (size_t)(d_in / 128) * (size_t)s4_dep_units(group / 32) * 1024;
}
hipError_t launch_deploy(const uint32_t* plane0, const float* alpha, const float* beta, int d_in, int d_out,
                         int group, void* stream_out, hipStream_t st);
hipError_t launch_smallt4_deployed(const SmallTArgs& a, hipStream_t st);  // nonce set here

// --- smallt4.hip: one column per lane on the 4x4x4 MFMA: T <= 4 for every code width, and
// INT3 / INT2 up to sixteen tokens -------------------------------------------------------
SmallTPlan smallt4_plan(int d_in, int d_out, int tokens);
hipError_t launch_smallt4(const SmallTArgs& a, hipStream_t st);  // nonce set by the caller
hipError_t launch_smallt4_f16(const SmallTArgs& a, hipStream_t st);  // the 16-bit-factor instantiations

// --- adapter.hip --------------------------------------------------------------------
// Rows of the hi (and of the lo) section of a bf16 hi/lo split of a [rank, *] matrix.
__host__ __device__ inline int rank_pad32(int rank) { return ((rank + 31) / 32) * 32; }

// The adapters of up to MAX_PARTS linears that share their input x and are evaluated as one
// wide layer (q/k/v; gate/up): part p owns columns [col0, col0 + d_out) of it.  A single layer
// is one part covering all columns; n = 0 means no adapter.
constexpr int MAX_PARTS = 4;
struct AdapterParts {
  int n;
  const float* A[MAX_PARTS];  // [L, rank]
  const float* B[MAX_PARTS];  // [rank, d_out of the part]
  float s[MAX_PARTS];
  int rank[MAX_PARTS], col0[MAX_PARTS], d_out[MAX_PARTS];
};

// The factor job of a front launch: folds the adapters into the zero factors for this call,
// beta' = beta + (s/g) A B (App. B.3), and writes the dense kernels' factor words
// fp16(alpha S) | fp16((beta' + 2^(N-1) alpha) S) << 16.
//   forward : words + inv_scale[d_out] (S per column, decided inside the job); optionally
//             block_max[factor_job_blocks], the per-block bounds on |W~'|
//   backward: the scale may not vary along the contraction index, which is the column there,
//             so one S serves the call.  Either cst fp32 [L, d_out] + block_max -- then
//             launch_factor_scale finishes the words -- or, given known_max (the block_max of
//             an earlier launch on the same alpha, beta, A, B), words + inv_scale[1] at once.
struct FactorJob {
  const float* alpha;   // [L, d_out]; null: no factor job in this launch
  const float* beta;    // [L, d_out]
  AdapterParts parts;   // what to fold in (n = 0: nothing)
  int g, bits, L, d_out;
  uint32_t* words;      // forward
  float* inv_scale;     // forward
  float* cst;           // backward, two-stage form
  float* block_max;     // [factor_job_blocks], optional in the forward
  const float* known_max;  // backward, one-stage form
};
int factor_job_blocks(int L, int d_out);
int factor_job_cols(int L);  // columns per block of the folding job: part widths must be multiples
hipError_t launch_factor_job(const FactorJob& f, hipStream_t st);  // the job as a launch of its own
hipError_t launch_factor_scale(const float* alpha, const float* cst, const float* block_max, int nmax,
                               size_t n, uint32_t* words, float* inv_scale, hipStream_t st);

// Forward front launch: x -> rs (row scales), x16 = fp16(x * scale), the factor job, and, when
// given, P_keep fp32 [T, L] = pool_g(x) and per part u_keep fp32 [T, rank] = s pool_g(x) A, from
// which the backward front launch below can work without x (its u_kept argument).
hipError_t launch_front_forward(const uint16_t* x, int T, int d_in, float2* rs, uint16_t* x16,
                                const AdapterParts& parts, int g, float* P_keep,
                                float* const* u_keep, const FactorJob& fac, hipStream_t st);
// Backward front launch: dy -> rs_dy, dy16; the factor job (first stage); and per adapter part
//   P       fp32 [T, L]          = pool_g(x)  (shared by the parts)
//   us_t    bf16 [2*rp, t_pad]   = rows hi(sU)^T then lo(sU)^T (token-contiguous, zero padded)
//   b_hl    bf16 [2*rp, d_out]   = hi(B) rows then lo(B) rows
// With u_kept (the forward's u_keep) x is not read: P is not written (the caller passes the
// forward's P_keep on to the gradient kernels) and us_t is transposed from u_kept.
hipError_t launch_front_backward(const uint16_t* dy, int T, int d_out, float2* rs_dy,
                                 uint16_t* dy16, const uint16_t* x, int d_in,
                                 const AdapterParts& parts, int g, float* P, uint16_t* const* us_t,
                                 int t_pad, uint16_t* const* b_hl, const float* const* u_kept,
                                 const FactorJob& fac, hipStream_t st);
// Both adapter-gradient jobs in one launch (neither depends on the other):
//   dB partials over token slices: db_part[z][rank][d_out] = sum_{t in slice z} sU[t,:]^T dy[t,:]
//   (dy: rows dy_ld elements apart, so that a part's columns of a wider dy can be passed)
//   dA partials over token slices: da_part[z][L][rank] = sum_{t in slice z} P[t,:]^T dU[t,:], with
//   dU = s * sum_q (raw[q][:, :rp] + raw[q][:, rp:]) rebuilt from the split-K partials of the dU
//   product
hipError_t launch_adapter_grads(const uint16_t* us_t, int t_pad, const uint16_t* dy, int dy_ld, int T,
                                int d_out, int rank, int tsplit_b, float* db_part, const float* P,
                                const float* raw, int ksplit, float s, int L, int tsplit_a,
                                float* da_part, hipStream_t st);
// out = (accumulate ? out : 0) + sum_z part[z], fixed order, for two outputs in one launch
hipError_t launch_reduce2(const float* part_a, int nparts_a, size_t n_a, float* out_a,
                          const float* part_b, int nparts_b, size_t n_b, float* out_b,
                          int accumulate, hipStream_t st);
// beta_out = beta + (s/g) A B
hipError_t launch_merge(const float* beta, const float* A, const float* B, int L, int d_out,
                        int rank, int g, float s, float* beta_out, hipStream_t st);

// out = -(alpha * in) (zero point -> zero factor) or -(in / alpha) (the reverse), n elements
hipError_t launch_zero_point(const float* alpha, const float* in, float* out, size_t n, bool to_zero_point,
                             hipStream_t st);

// --- optim.hip: fused AdamW step with a joint gradient-norm clip over up to 32 tensors ----
constexpr int OPT_MAX_TENSORS = 32;
constexpr int OPT_CHUNK = 4096;  // elements per block; a block never straddles two tensors
struct OptTensors {
  float* p[OPT_MAX_TENSORS];
  float* g[OPT_MAX_TENSORS];
  float* m[OPT_MAX_TENSORS];
  float* v[OPT_MAX_TENSORS];
  unsigned long long numel[OPT_MAX_TENSORS];
  unsigned chunk_start[OPT_MAX_TENSORS + 1];  // first block of each tensor; [n] = blocks in all
  int n;
};
struct OptHyper {
  float beta1, one_minus_beta1, beta2, one_minus_beta2, eps;
  float decay;           // 1 - lr * weight_decay
  float step_size;       // lr / (1 - beta1^t)
  float inv_sqrt_bias2;  // 1 / sqrt(1 - beta2^t)
  float max_norm;
  int zero_grads;
};
hipError_t launch_adamw(const OptTensors& t, const OptHyper& h, float* partial, float* norm_out, hipStream_t st);

// --- probe.hip (measurement aid): issue-rate probe of the matrix cores ----------------------
hipError_t launch_mfma_probe(int shape, int lds_reads, int valu_per_mfma, float* sink,
                             unsigned long long* counts, int iters, int blocks, hipStream_t st);

// --- glue.hip (benchmark-harness glue, not part of the layer) --------------------------
// h = silu(gate) * up over n bf16 elements (n a multiple of 8), and its backward.
hipError_t launch_swiglu_forward(const void* gate, const void* up, void* h, size_t n, hipStream_t st);
hipError_t launch_swiglu_backward(const void* dh, const void* gate, const void* up, void* dgate,
                                  void* dup, size_t n, hipStream_t st);
// the same on gu = [gate | up] of shape [rows, 2 cols], gradients to dgu = [dgate | dup]
hipError_t launch_swiglu_forward_wide(const void* gu, void* h, size_t rows, size_t cols, hipStream_t st);
hipError_t launch_swiglu_backward_wide(const void* dh, const void* gu, void* dgu, size_t rows, size_t cols,
                                       hipStream_t st);

}  // namespace qalora
