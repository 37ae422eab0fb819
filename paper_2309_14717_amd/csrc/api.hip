// extern "C" entry points of the QA-LoRA library: host-side argument validation,
// workspace carving and kernel sequencing.  No allocation, no synchronisation, no state.
#include "../../include/qalora.h"

#include "common.hpp"
#include "kernels.hpp"

#include <cmath>

using namespace qalora;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int row_align_for_bits(int bits) { return bits == 4 ? 8 : (bits == 2 ? 16 : 32); }

// Workspace plans.  Offsets are a pure function of (desc, tokens), so the size query and
// the compute call always agree.
struct FwdPlan {
  int gsplit;
  size_t rs, a16, fac, inv, gpart, total;
};
// One adapter among those sharing x (a single layer is one part over all columns).
struct PartSpec {
  int n;
  AdapterParts ap;
  float* dA[MAX_PARTS];
  float* dB[MAX_PARTS];
};
struct BwdPartPlan {
  int rp, ksplit, tsplit_b, tsplit_a;
  size_t us_t, b_hl, du_raw, db_part, da_part;
};
struct BwdPlan {
  int t_pad, gsplit, nmax;
  size_t rs, a16, fac, cst, bmax, inv, P, gpart, total;
  BwdPartPlan part[MAX_PARTS];
};

// forward workspace: row scales, the fp16 copy of x, the factor words and their column scales,
// then the split-K partials if any.  Independent of the adapter: the factor job folds it in.
FwdPlan plan_forward(const qalora_desc& d, int T) {
  FwdPlan p{};
  const size_t L = (size_t)(d.d_in / d.group);
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t o = off;
    off += align_up(bytes);
    return o;
  };
  p.rs = take((size_t)T * sizeof(float2));
  p.a16 = take((size_t)round_up(T, 256) * d.d_in * 2);
  p.fac = take(L * d.d_out * 4);
  p.inv = take((size_t)d.d_out * 4);
  p.gsplit = gemm_dq_ksplit(T, d.d_out, d.d_in);
  if (p.gsplit > 1) p.gpart = take((size_t)p.gsplit * T * d.d_out * 4);
  p.total = off;
  return p;
}

// backward workspace: what the dx contraction needs (row scales, fp16 copy of dy, factor words
// and their first stage), then P = pool(x) and per adapter part the operands and partial sums
// of its gradient kernels.  n_parts = 0: adapter-free, only dx.
BwdPlan plan_backward(const qalora_desc& d, int T, int n_parts, const int* part_rank, const int* part_dout) {
  BwdPlan p{};
  const int L = d.d_in / d.group;
  p.t_pad = round_up(T, 64);
  p.nmax = factor_job_blocks(L, d.d_out);
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t o = off;
    off += align_up(bytes);
    return o;
  };
  p.rs = take((size_t)T * sizeof(float2));
  p.a16 = take((size_t)round_up(T, 256) * d.d_out * 2);
  p.fac = take((size_t)L * d.d_out * 4);
  p.cst = take((size_t)L * d.d_out * 4);
  p.bmax = take((size_t)p.nmax * 4);
  p.inv = take(16);
  p.gsplit = gemm_dq_ksplit(T, d.d_in, d.d_out);
  if (p.gsplit > 1) p.gpart = take((size_t)p.gsplit * T * d.d_in * 4);
  if (n_parts <= 0) {
    p.total = off;
    return p;
  }
  p.P = take((size_t)T * L * 4);
  for (int q = 0; q < n_parts; ++q) {
    BwdPartPlan& pp = p.part[q];
    const int rank = part_rank[q], dout = part_dout[q];
    pp.rp = rank_pad32(rank);
    // dU product: [T, 2rp] output tiles of plain_tile_rows x 128 (the taller tile pays when K
    // is long: half the K steps per block for the same number of blocks); split K = d_out to
    // fill the chip.
    {
      const int tiles = ceil_div(T, gemm_plain_tile_rows(dout)) * ceil_div(2 * pp.rp, 128);
      const int nk = ceil_div(dout, 64);
      int ks = ceil_div(256, tiles);
      ks = ks < 1 ? 1 : (ks > 16 ? 16 : ks);
      const int by_steps = nk / 12;  // a slice shorter than about twelve K steps is all prologue
      if (ks > by_steps) ks = by_steps < 1 ? 1 : by_steps;
      pp.ksplit = ks;
    }
    {
      const int blocks = ceil_div(dout, 128);
      int ts = ceil_div(256, blocks);  // about one block per compute unit
      ts = ts > 32 ? 32 : ts;
      const int steps = p.t_pad / 64;
      pp.tsplit_b = ts > steps ? steps : ts;
    }
    {
      // one 16-token chunk per block where possible: the work is tiny and latency-bound, so
      // maximise the number of independent blocks
      const int steps = ceil_div(T, 16);
      pp.tsplit_a = steps > 256 ? 256 : steps;
    }
    pp.us_t = take((size_t)2 * pp.rp * p.t_pad * 2);
    pp.b_hl = take((size_t)2 * pp.rp * dout * 2);
    pp.du_raw = take((size_t)pp.ksplit * T * 2 * pp.rp * 4);
    pp.db_part = take((size_t)pp.tsplit_b * rank * dout * 4);
    pp.da_part = take((size_t)pp.tsplit_a * L * rank * 4);
  }
  p.total = off;
  return p;
}
BwdPlan plan_backward(const qalora_desc& d, int T) {
  return plan_backward(d, T, d.rank > 0 ? 1 : 0, &d.rank, &d.d_out);
}

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

// The contraction kernels address their operands through buffer resources with 32-bit byte
// offsets (and keep a range of offsets above kAddressable for "reads as zero"): the packed
// planes, the factor matrices and the fp16 copy of the activations must each stay below it.
constexpr size_t kAddressable = 0xf0000000ull;
inline bool addressable(const qalora_desc& d, int tokens) {
  const size_t L = (size_t)(d.d_in / d.group);
  const size_t wide = (size_t)(d.d_in > d.d_out ? d.d_in : d.d_out);
  return plane0_words(d.bits, d.d_in, d.d_out) * 4 < kAddressable &&
         L * (size_t)d.d_out * 4 < kAddressable &&
         (size_t)round_up(tokens, 256) * wide * 2 < kAddressable;
}

// The small-token streaming path covers groups of 32, 64 or 128 rows, input widths that are
// whole 128-row chunks, and operands its 32-bit buffer offsets can address: every code width
// up to sixteen tokens, 4-bit codes up to thirty-two.
inline bool use_smallt(const qalora_desc& d, int tokens) {
  if (tokens > (d.bits == 4 ? 32 : 16)) return false;
  if (d.group != 32 && d.group != 64 && d.group != 128) return false;
  if (d.d_in % 128 != 0) return false;
  return plane0_words(d.bits, d.d_in, d.d_out) * 4 < kAddressable;
}

// Workspace of the small-token path: one flag and one [16 x slab] fp32 partial per block.
inline size_t smallt_workspace(const qalora_desc& d, int tokens) {
  const int blocks = (tokens <= 4 || d.bits != 4) ? smallt4_plan(d.d_in, d.d_out, tokens).blocks
                                                  : smallt_plan(d.d_in, d.d_out, tokens).blocks;
  const size_t per_block = (size_t)(tokens > 16 ? 2 : 1) * ST_PARTIAL_FLOATS;  // two groups of sixteen tokens
  return ST_HEAD_BYTES + align_up((size_t)blocks * per_block * 4);
}

static_assert(MAX_PARTS == QALORA_MAX_PARTS, "the header documents this limit");
static_assert(ST_STATUS_OFFSET == QALORA_WS_STATUS_OFFSET, "the header documents this offset");

// Scratch of qalora_forward_noalloc: the streaming kernels' flags, status word and per-block
// partial sums for up to sixteen tokens.  Host code never uses this name as an address; the
// device address is looked up once per device (scratch_on_current_device).
constexpr size_t kScratchBytes = ST_HEAD_BYTES + (size_t)ST_MAX_BLOCKS * ST_PARTIAL_FLOATS * 4;
static_assert(kScratchBytes == QALORA_NOALLOC_SCRATCH_BYTES, "the header documents this size");
}  // namespace

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];  // device address of `scratch`, per device

// Device address of this device's copy of the scratch array (every device holds its own, at
// its own address); looked up on the first call with that device current.
hipError_t scratch_on_current_device(void** out) {
  int dev = 0;
  if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    if (hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)); e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);
  }
  *out = ptr;
  return hipSuccess;
}
}  // namespace

// Plain copy of known size: the yardstick the HBM traffic counters are scaled by.
__global__ __launch_bounds__(256) void profile_copy_kernel(const uint4* __restrict__ src,
                                                           uint4* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

extern "C" {

const char* qalora_status_string(int status) {
  switch (status) {
    case QALORA_OK: return "QALORA_OK";
    case QALORA_EINVAL: return "QALORA_EINVAL: invalid argument";
    case QALORA_EALIGN: return "QALORA_EALIGN: device pointer not 16-byte aligned";
    case QALORA_EWORKSPACE: return "QALORA_EWORKSPACE: workspace missing or too small";
    case QALORA_EUNSUPPORTED: return "QALORA_EUNSUPPORTED: shape outside the supported set";
    case QALORA_EHIP: return "QALORA_EHIP: kernel launch failed";
    default: return "unknown status";
  }
}

int qalora_check_desc(const qalora_desc* d) {
  if (!d) return QALORA_EINVAL;
  if (d->d_in <= 0 || d->d_out <= 0) return QALORA_EINVAL;
  if (d->bits < 2 || d->bits > 4) return QALORA_EINVAL;
  if (d->group <= 0 || d->d_in % d->group != 0) return QALORA_EINVAL;
  if (d->rank < 0) return QALORA_EINVAL;
  if (d->group % row_align_for_bits(d->bits) != 0) return QALORA_EUNSUPPORTED;
  if (d->d_out % 8 != 0) return QALORA_EUNSUPPORTED;
  if (d->rank > 128) return QALORA_EUNSUPPORTED;
  return QALORA_OK;
}

size_t qalora_packed_bytes(const qalora_desc* d) {
  if (qalora_check_desc(d) != QALORA_OK) return 0;
  return 4 * (plane0_words(d->bits, d->d_in, d->d_out) + plane1_words(d->bits, d->d_in, d->d_out));
}

size_t qalora_workspace_bytes(const qalora_desc* d, int tokens, int op) {
  if (qalora_check_desc(d) != QALORA_OK) return 0;
  switch (op) {
    case QALORA_OP_QUANTIZE:
    case QALORA_OP_MERGE: return 0;
    case QALORA_OP_QUANTIZE_COMPENSATED: {
      const size_t n = (size_t)d->d_in * d->d_out;
      return align_up(n * 4) + align_up(n);
    }
    case QALORA_OP_FORWARD: {
      if (tokens <= 0) return 0;
      size_t need = plan_forward(*d, tokens).total;
      if (use_smallt(*d, tokens)) {
        const size_t st = smallt_workspace(*d, tokens);
        if (st > need) need = st;
      }
      return need;
    }
    case QALORA_OP_FORWARD_FACTORS16: {
      if (tokens <= 0) return 0;
      if (use_smallt(*d, tokens)) return smallt_workspace(*d, tokens);
      // matrix path: the adapter-free forward's workspace, then alpha and beta expanded to fp32
      qalora_desc plain = *d;
      plain.rank = 0;
      return align_up(qalora_workspace_bytes(&plain, tokens, QALORA_OP_FORWARD)) +
             2 * align_up((size_t)(d->d_in / d->group) * d->d_out * 4);
    }
    case QALORA_OP_BACKWARD: return tokens > 0 ? plan_backward(*d, tokens).total : 0;
    default: return 0;
  }
}

int qalora_quantize(const qalora_desc* d, const float* W, void* packed, float* alpha, float* beta,
                    void* ws, size_t ws_bytes, void* stream) {
  (void)ws;
  (void)ws_bytes;
  const int rc = qalora_check_desc(d);
  if (rc != QALORA_OK) return rc;
  if (!W || !packed || !alpha || !beta) return QALORA_EINVAL;
  if (misaligned(W) || misaligned(packed) || misaligned(alpha) || misaligned(beta))
    return QALORA_EALIGN;
  launch_quantize(d->bits, W, packed, alpha, beta, d->d_in, d->d_out, d->group, as_stream(stream));
  return hipGetLastError() == hipSuccess ? QALORA_OK : QALORA_EHIP;
}

int qalora_quantize_compensated(const qalora_desc* d, const float* W, const float* hinv_chol, void* packed,
                                float* alpha, float* beta, void* ws, size_t ws_bytes, void* stream) {
  const int rc = qalora_check_desc(d);
  if (rc != QALORA_OK) return rc;
  if (!W || !hinv_chol || !packed || !alpha || !beta) return QALORA_EINVAL;
  if (misaligned(W) || misaligned(hinv_chol) || misaligned(packed) || misaligned(alpha) || misaligned(beta) ||
      misaligned(ws))
    return QALORA_EALIGN;
  if (128 % d->group != 0) return QALORA_EUNSUPPORTED;  // groups must not straddle the lazy blocks
  const size_t n = (size_t)d->d_in * d->d_out;
  if (!ws || ws_bytes < align_up(n * 4) + align_up(n)) return QALORA_EWORKSPACE;
  float* work = static_cast<float*>(ws);
  uint8_t* codes = static_cast<uint8_t*>(ws) + align_up(n * 4);
  if (launch_compensate(W, hinv_chol, d->d_in, d->d_out, d->bits, d->group, work, codes, alpha, beta,
                        as_stream(stream)) != hipSuccess)
    return QALORA_EHIP;
  // the codes enter the packed format the way any other quantizer's would
  launch_pack(d->bits, codes, packed, d->d_in, d->d_out, as_stream(stream));
  return hipGetLastError() == hipSuccess ? QALORA_OK : QALORA_EHIP;
}

int qalora_unpack(const qalora_desc* d, const void* packed, uint8_t* codes, void* stream) {
  const int rc = qalora_check_desc(d);
  if (rc != QALORA_OK) return rc;
  if (!packed || !codes) return QALORA_EINVAL;
  if (misaligned(packed) || misaligned(codes)) return QALORA_EALIGN;
  launch_unpack(d->bits, packed, codes, d->d_in, d->d_out, as_stream(stream));
  return hipGetLastError() == hipSuccess ? QALORA_OK : QALORA_EHIP;
}

int qalora_pack(const qalora_desc* d, const uint8_t* codes, void* packed, void* stream) {
  const int rc = qalora_check_desc(d);
  if (rc != QALORA_OK) return rc;
  if (!packed || !codes) return QALORA_EINVAL;
  if (misaligned(packed) || misaligned(codes)) return QALORA_EALIGN;
  launch_pack(d->bits, codes, packed, d->d_in, d->d_out, as_stream(stream));
  return hipGetLastError() == hipSuccess ? QALORA_OK : QALORA_EHIP;
}

// What the forward leaves for the backward when asked to: P = pool_g(x) [T, L] and
// s P A [T, rank], both fp32.
struct KeptLayout {
  size_t P, U[MAX_PARTS], bmax, total;
};
static KeptLayout kept_layout(const qalora_desc& d, int T, int n_parts, const int* part_rank) {
  KeptLayout k{};
  k.P = 0;
  size_t off = align_up((size_t)T * (d.d_in / d.group) * 4);
  for (int q = 0; q < n_parts; ++q) {
    k.U[q] = off;
    off += align_up((size_t)T * part_rank[q] * 4);
  }
  k.bmax = off;
  k.total = k.bmax + align_up((size_t)factor_job_blocks(d.d_in / d.group, d.d_out) * 4);
  return k;
}

struct PreparedFactors {  // factor words and column scales made ahead of the call (deployment)
  const uint32_t* words;
  const float* inv_scale;
};
static int forward_impl(const qalora_desc* d, int tokens, const void* x, const void* packed,
                        const float* alpha, const float* beta, const PartSpec& ps, void* y, int y_dtype,
                        void* kept, bool keep, void* ws, size_t ws_bytes, void* stream,
                        const PreparedFactors* pre = nullptr);
static int backward_impl(const qalora_desc* d, int tokens, const void* dy, const void* x,
                         const void* kept, bool use_kept, const void* packed, const float* alpha,
                         const float* beta, const PartSpec& ps, void* dx, int dx_dtype, int accumulate,
                         void* ws, size_t ws_bytes, void* stream);

// A single layer as one part over all its columns; exactly one of A, B null is an error the
// caller has checked for.
static PartSpec single_part(const qalora_desc* d, const float* A, const float* B, float* dA, float* dB) {
  PartSpec ps{};
  if (d && A && B && d->rank > 0) {
    ps.n = ps.ap.n = 1;
    ps.ap.A[0] = A;
    ps.ap.B[0] = B;
    ps.ap.s[0] = d->s;
    ps.ap.rank[0] = d->rank;
    ps.ap.col0[0] = 0;
    ps.ap.d_out[0] = d->d_out;
    ps.dA[0] = dA;
    ps.dB[0] = dB;
  }
  return ps;
}

int qalora_forward(const qalora_desc* d, int tokens, const void* x, const void* packed,
                   const float* alpha, const float* beta, const float* A, const float* B, void* y,
                   int y_dtype, void* ws, size_t ws_bytes, void* stream) {
  if ((A == nullptr) != (B == nullptr)) return QALORA_EINVAL;
  return forward_impl(d, tokens, x, packed, alpha, beta, single_part(d, A, B, nullptr, nullptr), y, y_dtype,
                      nullptr, false, ws, ws_bytes, stream);
}

size_t qalora_kept_bytes(const qalora_desc* d, int tokens) {
  if (qalora_check_desc(d) != QALORA_OK || tokens <= 0 || d->rank <= 0) return 0;
  return kept_layout(*d, tokens, 1, &d->rank).total;
}

int qalora_forward_keep(const qalora_desc* d, int tokens, const void* x, const void* packed,
                        const float* alpha, const float* beta, const float* A, const float* B,
                        void* y, int y_dtype, void* kept, void* ws, size_t ws_bytes, void* stream) {
  if (!A || !B || !kept || !d || d->rank <= 0) return QALORA_EINVAL;  // only an adapter has anything to keep
  return forward_impl(d, tokens, x, packed, alpha, beta, single_part(d, A, B, nullptr, nullptr), y, y_dtype,
                      kept, true, ws, ws_bytes, stream);
}

int qalora_backward(const qalora_desc* d, int tokens, const void* dy, const void* x,
                    const void* packed, const float* alpha, const float* beta, const float* A,
                    const float* B, void* dx, int dx_dtype, float* dA, float* dB, int accumulate,
                    void* ws, size_t ws_bytes, void* stream) {
  if ((A == nullptr) != (B == nullptr)) return QALORA_EINVAL;
  if (A && d && d->rank > 0 && (!dA || !dB || !x)) return QALORA_EINVAL;
  return backward_impl(d, tokens, dy, x, nullptr, false, packed, alpha, beta, single_part(d, A, B, dA, dB),
                       dx, dx_dtype, accumulate, ws, ws_bytes, stream);
}

int qalora_backward_kept(const qalora_desc* d, int tokens, const void* dy, const void* kept,
                         const void* packed, const float* alpha, const float* beta, const float* A,
                         const float* B, void* dx, int dx_dtype, float* dA, float* dB,
                         int accumulate, void* ws, size_t ws_bytes, void* stream) {
  if (!A || !B || !kept || !dA || !dB || !d || d->rank <= 0) return QALORA_EINVAL;
  return backward_impl(d, tokens, dy, nullptr, kept, true, packed, alpha, beta, single_part(d, A, B, dA, dB),
                       dx, dx_dtype, accumulate, ws, ws_bytes, stream);
}

// ---- several linears that share x, as one wide layer -----------------------------------
static int shared_parts(const qalora_desc* d, int n_parts, const qalora_part* parts, bool backward,
                        PartSpec& ps) {
  const int rc = qalora_check_desc(d);
  if (rc != QALORA_OK) return rc;
  if (n_parts < 1 || n_parts > MAX_PARTS || !parts) return QALORA_EINVAL;
  ps = PartSpec{};
  int col = 0;
  for (int q = 0; q < n_parts; ++q) {
    const qalora_part& pt = parts[q];
    if (pt.d_out <= 0 || pt.rank <= 0 || !pt.A || !pt.B) return QALORA_EINVAL;
    if (backward && (!pt.dA || !pt.dB)) return QALORA_EINVAL;
    if (misaligned(pt.A) || misaligned(pt.B) || misaligned(pt.dA) || misaligned(pt.dB)) return QALORA_EALIGN;
    if (pt.rank > 128 || pt.d_out % 32 != 0) return QALORA_EUNSUPPORTED;
    ps.ap.A[q] = pt.A;
    ps.ap.B[q] = pt.B;
    ps.ap.s[q] = pt.s;
    ps.ap.rank[q] = pt.rank;
    ps.ap.col0[q] = col;
    ps.ap.d_out[q] = pt.d_out;
    ps.dA[q] = pt.dA;
    ps.dB[q] = pt.dB;
    col += pt.d_out;
  }
  if (col != d->d_out) return QALORA_EINVAL;
  ps.n = ps.ap.n = n_parts;
  return QALORA_OK;
}

size_t qalora_shared_kept_bytes(const qalora_desc* d, int tokens, int n_parts, const qalora_part* parts) {
  PartSpec ps;
  if (tokens <= 0 || shared_parts(d, n_parts, parts, false, ps) != QALORA_OK) return 0;
  return kept_layout(*d, tokens, ps.n, ps.ap.rank).total;
}

size_t qalora_shared_workspace_bytes(const qalora_desc* d, int tokens, int op, int n_parts,
                                     const qalora_part* parts) {
  PartSpec ps;
  if (tokens <= 0 || shared_parts(d, n_parts, parts, false, ps) != QALORA_OK) return 0;
  if (op == QALORA_OP_FORWARD) return plan_forward(*d, tokens).total;
  if (op == QALORA_OP_BACKWARD) return plan_backward(*d, tokens, ps.n, ps.ap.rank, ps.ap.d_out).total;
  return 0;
}

int qalora_forward_shared(const qalora_desc* d, int tokens, const void* x, const void* packed,
                          const float* alpha, const float* beta, int n_parts, const qalora_part* parts,
                          void* y, int y_dtype, void* kept, void* ws, size_t ws_bytes, void* stream) {
  PartSpec ps;
  if (const int rc = shared_parts(d, n_parts, parts, false, ps); rc != QALORA_OK) return rc;
  return forward_impl(d, tokens, x, packed, alpha, beta, ps, y, y_dtype, kept, kept != nullptr, ws, ws_bytes,
                      stream);
}

int qalora_backward_shared(const qalora_desc* d, int tokens, const void* dy, const void* x,
                           const void* kept, const void* packed, const float* alpha, const float* beta,
                           int n_parts, const qalora_part* parts, void* dx, int dx_dtype, int accumulate,
                           void* ws, size_t ws_bytes, void* stream) {
  PartSpec ps;
  if (const int rc = shared_parts(d, n_parts, parts, true, ps); rc != QALORA_OK) return rc;
  if (!kept && !x) return QALORA_EINVAL;
  return backward_impl(d, tokens, dy, kept ? nullptr : x, kept, kept != nullptr, packed, alpha, beta, ps, dx,
                       dx_dtype, accumulate, ws, ws_bytes, stream);
}

static int forward_impl(const qalora_desc* d, int tokens, const void* x, const void* packed,
                        const float* alpha, const float* beta, const PartSpec& ps, void* y, int y_dtype,
                        void* kept, bool keep, void* ws, size_t ws_bytes, void* stream,
                        const PreparedFactors* pre) {
  const int rc = qalora_check_desc(d);
  if (rc != QALORA_OK) return rc;
  if (tokens <= 0 || !x || !packed || !y) return QALORA_EINVAL;
  if (!pre && (!alpha || !beta)) return QALORA_EINVAL;
  if (y_dtype != QALORA_F32 && y_dtype != QALORA_BF16) return QALORA_EINVAL;
  const bool adapter = ps.n > 0;
  if (keep && (!kept || !adapter)) return QALORA_EINVAL;  // only an adapter has anything to keep
  if (misaligned(x) || misaligned(packed) || misaligned(alpha) || misaligned(beta) || misaligned(y) ||
      misaligned(ws) || misaligned(kept))
    return QALORA_EALIGN;
  for (int q = 0; q < ps.n; ++q)
    if (misaligned(ps.ap.A[q]) || misaligned(ps.ap.B[q])) return QALORA_EALIGN;
  if (!addressable(*d, tokens)) return QALORA_EUNSUPPORTED;
  // the folding job owns whole column blocks: every part's width must be a multiple of them
  if (ps.n > 1)
    for (int q = 0; q < ps.n; ++q)
      if (ps.ap.d_out[q] % factor_job_cols(d->d_in / d->group) != 0) return QALORA_EUNSUPPORTED;
  if (!adapter && !pre && use_smallt(*d, tokens)) {
    // memory-bound regime: stream the weight once on the exact-operand path
    const size_t need = smallt_workspace(*d, tokens);
    if (!ws || ws_bytes < need) return QALORA_EWORKSPACE;
    SmallTArgs a{};
    a.x = static_cast<const uint16_t*>(x);
    a.plane0 = static_cast<const uint32_t*>(packed);
    a.plane1 = a.plane0 + plane0_words(d->bits, d->d_in, d->d_out);
    a.bits = d->bits;
    a.alpha = alpha;
    a.beta = beta;
    a.out = y;
    a.flags = static_cast<unsigned long long*>(ws);
    a.status = a.flags + ST_MAX_BLOCKS;
    a.partial = reinterpret_cast<float*>(static_cast<char*>(ws) + ST_HEAD_BYTES);
    a.out_bf16 = (y_dtype == QALORA_BF16);
    a.T = tokens;
    a.d_in = d->d_in;
    a.d_out = d->d_out;
    a.group = d->group;
    return launch_smallt(a, as_stream(stream)) == hipSuccess ? QALORA_OK : QALORA_EHIP;
  }
  const FwdPlan plan = plan_forward(*d, tokens);
  if (!ws || ws_bytes < plan.total) return QALORA_EWORKSPACE;
  hipStream_t st = as_stream(stream);
  char* w = static_cast<char*>(ws);
  float2* rs = reinterpret_cast<float2*>(w + plan.rs);
  uint16_t* x16 = reinterpret_cast<uint16_t*>(w + plan.a16);
  const int L = d->d_in / d->group;

  // front launch: row scales and the fp16 copy of x; the adapter folded into the zero factors
  // and the factor words of the dense kernel; P and s P A for the backward when asked for
  FactorJob fj{};
  fj.alpha = alpha;
  fj.beta = beta;
  fj.parts = ps.ap;
  fj.g = d->group;
  fj.bits = d->bits;
  fj.L = L;
  fj.d_out = d->d_out;
  fj.words = reinterpret_cast<uint32_t*>(w + plan.fac);
  fj.inv_scale = reinterpret_cast<float*>(w + plan.inv);
  if (pre) fj.alpha = nullptr;  // the words exist already: no factor job
  float* P_keep = nullptr;
  float* u_keep[MAX_PARTS] = {};
  if (keep) {
    const KeptLayout k = kept_layout(*d, tokens, ps.n, ps.ap.rank);
    P_keep = reinterpret_cast<float*>(static_cast<char*>(kept) + k.P);
    for (int q = 0; q < ps.n; ++q) u_keep[q] = reinterpret_cast<float*>(static_cast<char*>(kept) + k.U[q]);
    // the bounds on |W~'| the factor job finds anyway: with them the backward knows its scale
    fj.block_max = reinterpret_cast<float*>(static_cast<char*>(kept) + k.bmax);
  }
  if (launch_front_forward(static_cast<const uint16_t*>(x), tokens, d->d_in, rs, x16, ps.ap, d->group,
                           P_keep, u_keep, fj, st) != hipSuccess)
    return QALORA_EHIP;

  GemmArgs g{};
  g.a_main = x16;
  g.lda_main = d->d_in;
  g.a_main_padded_rows = round_up(tokens, 256);
  g.plane0 = static_cast<const uint32_t*>(packed);
  g.plane1 = g.plane0 + plane0_words(d->bits, d->d_in, d->d_out);
  g.fac = pre ? pre->words : fj.words;
  g.n_scale = pre ? pre->inv_scale : fj.inv_scale;
  g.out = y;
  g.out_bf16 = (y_dtype == QALORA_BF16);
  g.M = tokens;
  g.N = d->d_out;
  g.K_main = d->d_in;
  g.d_in = d->d_in;
  g.d_out = d->d_out;
  g.group = d->group;
  g.row_scale = rs;
  g.ksplit = plan.gsplit;
  g.partial = plan.gsplit > 1 ? reinterpret_cast<float*>(w + plan.gpart) : nullptr;
  return launch_gemm_dq(d->bits, false, g, st) == hipSuccess ? QALORA_OK : QALORA_EHIP;
}

static int backward_impl(const qalora_desc* d, int tokens, const void* dy, const void* x,
                         const void* kept, bool use_kept, const void* packed, const float* alpha,
                         const float* beta, const PartSpec& ps, void* dx, int dx_dtype, int accumulate,
                         void* ws, size_t ws_bytes, void* stream) {
  const int rc = qalora_check_desc(d);
  if (rc != QALORA_OK) return rc;
  if (tokens <= 0 || !dy || !packed || !alpha || !beta) return QALORA_EINVAL;
  const bool adapter = ps.n > 0;
  if (use_kept && (!kept || !adapter)) return QALORA_EINVAL;
  if (adapter && !use_kept && !x) return QALORA_EINVAL;
  for (int q = 0; q < ps.n; ++q)
    if (!ps.dA[q] || !ps.dB[q]) return QALORA_EINVAL;
  if (misaligned(kept)) return QALORA_EALIGN;
  if (dx && dx_dtype != QALORA_F32 && dx_dtype != QALORA_BF16) return QALORA_EINVAL;
  if (accumulate != 0 && accumulate != 1) return QALORA_EINVAL;
  if (misaligned(dy) || misaligned(x) || misaligned(packed) || misaligned(alpha) || misaligned(beta) ||
      misaligned(dx) || misaligned(ws))
    return QALORA_EALIGN;
  for (int q = 0; q < ps.n; ++q)
    if (misaligned(ps.ap.A[q]) || misaligned(ps.ap.B[q]) || misaligned(ps.dA[q]) || misaligned(ps.dB[q]))
      return QALORA_EALIGN;
  if (!addressable(*d, tokens)) return QALORA_EUNSUPPORTED;
  if (ps.n > 1)
    for (int q = 0; q < ps.n; ++q)
      if (ps.ap.d_out[q] % factor_job_cols(d->d_in / d->group) != 0) return QALORA_EUNSUPPORTED;
  const BwdPlan plan = plan_backward(*d, tokens, ps.n, ps.ap.rank, ps.ap.d_out);
  for (int q = 0; q < ps.n; ++q)
    if ((size_t)plan.part[q].ksplit * tokens * 2 * plan.part[q].rp * 4 >= kAddressable)
      return QALORA_EUNSUPPORTED;  // the split-K partials of dU are read with 32-bit byte offsets
  if (!ws || ws_bytes < plan.total) return QALORA_EWORKSPACE;
  hipStream_t st = as_stream(stream);
  char* w = static_cast<char*>(ws);
  const int L = d->d_in / d->group;
  const uint16_t* dy16 = static_cast<const uint16_t*>(dy);  // bf16 bits
  float2* rs = reinterpret_cast<float2*>(w + plan.rs);
  uint16_t* dyh = reinterpret_cast<uint16_t*>(w + plan.a16);  // fp16 scaled copy of dy

  // dx = dy W~'^T with beta' = beta + (s/g) A B: the pooled-LoRA term of dx is the adapter's
  // share of W~' (App. B.3), so the factor job folds it in and the contraction needs no extra
  // operand.  Skipped when dx is not wanted.
  FactorJob fj{};
  uint32_t* words = reinterpret_cast<uint32_t*>(w + plan.fac);
  float* inv_scale = reinterpret_cast<float*>(w + plan.inv);
  KeptLayout kl{};
  if (use_kept) kl = kept_layout(*d, tokens, ps.n, ps.ap.rank);
  if (dx) {
    fj.alpha = alpha;
    fj.beta = beta;
    fj.parts = ps.ap;
    fj.g = d->group;
    fj.bits = d->bits;
    fj.L = L;
    fj.d_out = d->d_out;
    if (use_kept) {  // the forward left the bounds: one stage
      fj.known_max = reinterpret_cast<const float*>(static_cast<const char*>(kept) + kl.bmax);
      fj.words = words;
      fj.inv_scale = inv_scale;
    } else {
      fj.cst = reinterpret_cast<float*>(w + plan.cst);
      fj.block_max = reinterpret_cast<float*>(w + plan.bmax);
    }
  }
  float* P = nullptr;
  uint16_t* us_t[MAX_PARTS] = {};
  uint16_t* b_hl[MAX_PARTS] = {};
  const float* u_kept[MAX_PARTS] = {};
  if (adapter) {
    P = reinterpret_cast<float*>(w + plan.P);
    for (int q = 0; q < ps.n; ++q) {
      us_t[q] = reinterpret_cast<uint16_t*>(w + plan.part[q].us_t);
      b_hl[q] = reinterpret_cast<uint16_t*>(w + plan.part[q].b_hl);
    }
    if (use_kept) {  // written by the forward: the front launch below then skips x altogether
      char* kp = const_cast<char*>(static_cast<const char*>(kept));
      P = reinterpret_cast<float*>(kp + kl.P);
      for (int q = 0; q < ps.n; ++q) u_kept[q] = reinterpret_cast<const float*>(kp + kl.U[q]);
    }
  }
  // row scales + fp16 copy of dy; first stage of the factor words; P = pool(x), sU^T hi/lo and
  // the hi/lo rows of B for the adapter gradients
  if (launch_front_backward(dy16, tokens, d->d_out, rs, dyh,
                            (adapter && !use_kept) ? static_cast<const uint16_t*>(x) : nullptr, d->d_in,
                            ps.ap, d->group, P, us_t, plan.t_pad, b_hl, use_kept ? u_kept : nullptr, fj,
                            st) != hipSuccess)
    return QALORA_EHIP;
  if (dx) {
    if (!use_kept && launch_factor_scale(alpha, fj.cst, fj.block_max, plan.nmax, (size_t)L * d->d_out,
                                         words, inv_scale, st) != hipSuccess)
      return QALORA_EHIP;
    GemmArgs g{};
    g.a_main = dyh;
    g.lda_main = d->d_out;
    g.a_main_padded_rows = round_up(tokens, 256);
    g.plane0 = static_cast<const uint32_t*>(packed);
    g.plane1 = g.plane0 + plane0_words(d->bits, d->d_in, d->d_out);
    g.fac = words;
    g.n_scale = inv_scale;
    g.out = dx;
    g.out_bf16 = (dx_dtype == QALORA_BF16);
    g.M = tokens;
    g.N = d->d_in;
    g.K_main = d->d_out;
    g.d_in = d->d_in;
    g.d_out = d->d_out;
    g.group = d->group;
    g.row_scale = rs;
    g.ksplit = plan.gsplit;
    g.partial = plan.gsplit > 1 ? reinterpret_cast<float*>(w + plan.gpart) : nullptr;
    if (launch_gemm_dq(d->bits, true, g, st) != hipSuccess) return QALORA_EHIP;
  }
  for (int q = 0; q < ps.n; ++q) {  // the adapter gradients of every part, on its columns of dy
    const BwdPartPlan& pp = plan.part[q];
    const int rank = ps.ap.rank[q], dout = ps.ap.d_out[q];
    const uint16_t* dyq = dy16 + ps.ap.col0[q];
    float* du_raw = reinterpret_cast<float*>(w + pp.du_raw);
    float* db_part = reinterpret_cast<float*>(w + pp.db_part);
    float* da_part = reinterpret_cast<float*>(w + pp.da_part);
    // dU = s dy B^T : plain bf16 product against the hi/lo rows of B, split over K = d_out
    GemmArgs g{};
    g.a_tail = dyq;
    g.lda_tail = d->d_out;
    g.b_tail = b_hl[q];
    g.K_tail = dout;
    g.out = du_raw;
    g.M = tokens;
    g.N = 2 * pp.rp;
    g.group = 1;
    if (launch_gemm_plain(g, pp.ksplit, st) != hipSuccess) return QALORA_EHIP;
    // dB = (sU)^T dy and dA = P^T dU as partials over token slices, one launch; the dA job
    // finalises dU on the fly
    if (launch_adapter_grads(us_t[q], plan.t_pad, dyq, d->d_out, tokens, dout, rank, pp.tsplit_b, db_part, P,
                             du_raw, pp.ksplit, ps.ap.s[q], L, pp.tsplit_a, da_part, st) != hipSuccess)
      return QALORA_EHIP;
    if (launch_reduce2(da_part, pp.tsplit_a, (size_t)L * rank, ps.dA[q], db_part, pp.tsplit_b,
                       (size_t)rank * dout, ps.dB[q], accumulate, st) != hipSuccess)
      return QALORA_EHIP;
  }
  return QALORA_OK;
}

int qalora_merge(const qalora_desc* d, const float* beta, const float* A, const float* B,
                 float* beta_out, void* stream) {
  const int rc = qalora_check_desc(d);
  if (rc != QALORA_OK) return rc;
  if (!beta || !A || !B || !beta_out || d->rank <= 0) return QALORA_EINVAL;
  if (misaligned(beta) || misaligned(A) || misaligned(B) || misaligned(beta_out))
    return QALORA_EALIGN;
  return launch_merge(beta, A, B, d->d_in / d->group, d->d_out, d->rank, d->group, d->s, beta_out,
                      as_stream(stream)) == hipSuccess
             ? QALORA_OK
             : QALORA_EHIP;
}

int qalora_forward_noalloc(const qalora_desc* d, int tokens, const void* x, const void* packed,
                           const float* alpha, const float* beta, void* y, int y_dtype, void* stream) {
  const int rc = qalora_check_desc(d);
  if (rc != QALORA_OK) return rc;
  if (tokens <= 0 || !x || !packed || !alpha || !beta || !y) return QALORA_EINVAL;
  if (y_dtype != QALORA_F32 && y_dtype != QALORA_BF16) return QALORA_EINVAL;
  if (misaligned(x) || misaligned(packed) || misaligned(alpha) || misaligned(beta) || misaligned(y))
    return QALORA_EALIGN;
  // beyond what the built-in scratch holds, or outside the streaming kernels' shapes
  if (tokens > QALORA_NOALLOC_MAX_TOKENS || !use_smallt(*d, tokens)) return QALORA_EUNSUPPORTED;
  if (smallt_workspace(*d, tokens) > kScratchBytes) return QALORA_EUNSUPPORTED;
  void* ptr = nullptr;
  if (scratch_on_current_device(&ptr) != hipSuccess) return QALORA_EHIP;
  SmallTArgs a{};
  a.x = static_cast<const uint16_t*>(x);
  a.plane0 = static_cast<const uint32_t*>(packed);
  a.plane1 = a.plane0 + plane0_words(d->bits, d->d_in, d->d_out);
  a.bits = d->bits;
  a.alpha = alpha;
  a.beta = beta;
  a.out = y;
  a.flags = static_cast<unsigned long long*>(ptr);
  a.status = a.flags + ST_MAX_BLOCKS;
  a.partial = reinterpret_cast<float*>(static_cast<char*>(ptr) + ST_HEAD_BYTES);
  a.out_bf16 = (y_dtype == QALORA_BF16);
  a.T = tokens;
  a.d_in = d->d_in;
  a.d_out = d->d_out;
  a.group = d->group;
  return launch_smallt(a, as_stream(stream)) == hipSuccess ? QALORA_OK : QALORA_EHIP;
}

// The deployment stream covers what the one-column-per-lane streaming kernel covers at 4 bits.
static bool deployable(const qalora_desc& d) {
  return d.bits == 4 && (d.group == 32 || d.group == 64 || d.group == 128) && d.d_in % 128 == 0 &&
         deploy_stream_bytes(d.d_in, d.d_out, d.group) < kAddressable;
}

// deployed = [decode stream][dense-kernel factor words][their column scales]
struct DeployLayout {
  size_t words, inv, total;
};
static DeployLayout deploy_layout(const qalora_desc& d) {
  DeployLayout l{};
  l.words = align_up(deploy_stream_bytes(d.d_in, d.d_out, d.group));
  l.inv = l.words + align_up((size_t)(d.d_in / d.group) * d.d_out * 4);
  l.total = l.inv + align_up((size_t)d.d_out * 4);
  return l;
}

size_t qalora_deployed_bytes(const qalora_desc* d) {
  if (qalora_check_desc(d) != QALORA_OK || !deployable(*d)) return 0;
  return deploy_layout(*d).total;
}

int qalora_deploy(const qalora_desc* d, const void* packed, const float* alpha, const float* beta,
                  void* deployed, void* stream) {
  const int rc = qalora_check_desc(d);
  if (rc != QALORA_OK) return rc;
  if (!packed || !alpha || !beta || !deployed) return QALORA_EINVAL;
  if (misaligned(packed) || misaligned(alpha) || misaligned(beta) || misaligned(deployed)) return QALORA_EALIGN;
  if (!deployable(*d)) return QALORA_EUNSUPPORTED;
  if (launch_deploy(static_cast<const uint32_t*>(packed), alpha, beta, d->d_in, d->d_out, d->group, deployed,
                    as_stream(stream)) != hipSuccess)
    return QALORA_EHIP;
  // the dense kernel's factor words of the static layer, so that no call has to make them
  const DeployLayout l = deploy_layout(*d);
  FactorJob fj{};
  fj.alpha = alpha;
  fj.beta = beta;
  fj.g = d->group;
  fj.bits = d->bits;
  fj.L = d->d_in / d->group;
  fj.d_out = d->d_out;
  fj.words = reinterpret_cast<uint32_t*>(static_cast<char*>(deployed) + l.words);
  fj.inv_scale = reinterpret_cast<float*>(static_cast<char*>(deployed) + l.inv);
  return launch_factor_job(fj, as_stream(stream)) == hipSuccess ? QALORA_OK : QALORA_EHIP;
}

int qalora_forward_deployed(const qalora_desc* d, int tokens, const void* x, const void* packed,
                            const void* deployed, void* y, int y_dtype, void* ws, size_t ws_bytes,
                            void* stream) {
  const int rc = qalora_check_desc(d);
  if (rc != QALORA_OK) return rc;
  if (tokens <= 0 || !x || !deployed || !y) return QALORA_EINVAL;
  if (y_dtype != QALORA_F32 && y_dtype != QALORA_BF16) return QALORA_EINVAL;
  if (misaligned(x) || misaligned(deployed) || misaligned(y) || misaligned(ws) || misaligned(packed))
    return QALORA_EALIGN;
  if (!deployable(*d)) return QALORA_EUNSUPPORTED;
  if (tokens > QALORA_DEPLOYED_STREAM_TOKENS) {
    // beyond the decode kernel: the dense contraction on the codes as packed, with the factor
    // words the deployment prepared
    if (!packed) return QALORA_EINVAL;
    const DeployLayout l = deploy_layout(*d);
    const PreparedFactors pre{reinterpret_cast<const uint32_t*>(static_cast<const char*>(deployed) + l.words),
                              reinterpret_cast<const float*>(static_cast<const char*>(deployed) + l.inv)};
    return forward_impl(d, tokens, x, packed, nullptr, nullptr, PartSpec{}, y, y_dtype, nullptr, false, ws,
                        ws_bytes, stream, &pre);
  }
  const size_t need = smallt_workspace(*d, tokens);
  if (!ws || ws_bytes < need) return QALORA_EWORKSPACE;
  SmallTArgs a{};
  a.x = static_cast<const uint16_t*>(x);
  a.stream = deployed;
  a.bits = d->bits;
  a.out = y;
  a.flags = static_cast<unsigned long long*>(ws);
  a.status = a.flags + ST_MAX_BLOCKS;
  a.partial = reinterpret_cast<float*>(static_cast<char*>(ws) + ST_HEAD_BYTES);
  a.out_bf16 = (y_dtype == QALORA_BF16);
  a.T = tokens;
  a.d_in = d->d_in;
  a.d_out = d->d_out;
  a.group = d->group;
  return launch_smallt4_deployed(a, as_stream(stream)) == hipSuccess ? QALORA_OK : QALORA_EHIP;
}

int qalora_pack_factors16(const qalora_desc* d, const float* alpha, const float* beta, void* factors16,
                          void* stream) {
  const int rc = qalora_check_desc(d);
  if (rc != QALORA_OK) return rc;
  if (!alpha || !beta || !factors16) return QALORA_EINVAL;
  if (misaligned(alpha) || misaligned(beta) || misaligned(factors16)) return QALORA_EALIGN;
  const size_t n = (size_t)(d->d_in / d->group) * d->d_out;
  return launch_pack_factors(alpha, beta, factors16, n, as_stream(stream)) == hipSuccess ? QALORA_OK
                                                                                          : QALORA_EHIP;
}

int qalora_forward_factors16(const qalora_desc* d, int tokens, const void* x, const void* packed,
                             const void* factors16, void* y, int y_dtype, void* ws, size_t ws_bytes,
                             void* stream) {
  const int rc = qalora_check_desc(d);
  if (rc != QALORA_OK) return rc;
  if (tokens <= 0 || !x || !packed || !factors16 || !y) return QALORA_EINVAL;
  if (y_dtype != QALORA_F32 && y_dtype != QALORA_BF16) return QALORA_EINVAL;
  if (misaligned(x) || misaligned(packed) || misaligned(factors16) || misaligned(y) || misaligned(ws))
    return QALORA_EALIGN;
  if (!addressable(*d, tokens)) return QALORA_EUNSUPPORTED;
  const size_t need = qalora_workspace_bytes(d, tokens, QALORA_OP_FORWARD_FACTORS16);
  if (!ws || ws_bytes < need) return QALORA_EWORKSPACE;
  if (use_smallt(*d, tokens)) {
    SmallTArgs a{};
    a.x = static_cast<const uint16_t*>(x);
    a.plane0 = static_cast<const uint32_t*>(packed);
    a.plane1 = a.plane0 + plane0_words(d->bits, d->d_in, d->d_out);
    a.bits = d->bits;
    a.fac16 = static_cast<const uint32_t*>(factors16);
    a.out = y;
    a.flags = static_cast<unsigned long long*>(ws);
    a.status = a.flags + ST_MAX_BLOCKS;
    a.partial = reinterpret_cast<float*>(static_cast<char*>(ws) + ST_HEAD_BYTES);
    a.out_bf16 = (y_dtype == QALORA_BF16);
    a.T = tokens;
    a.d_in = d->d_in;
    a.d_out = d->d_out;
    a.group = d->group;
    return launch_smallt(a, as_stream(stream)) == hipSuccess ? QALORA_OK : QALORA_EHIP;
  }
  // matrix path: expand the factors behind the forward's own workspace and run it
  qalora_desc plain = *d;
  plain.rank = 0;
  const size_t fwd_ws = align_up(qalora_workspace_bytes(&plain, tokens, QALORA_OP_FORWARD));
  const size_t n = (size_t)(d->d_in / d->group) * d->d_out;
  float* alpha = reinterpret_cast<float*>(static_cast<char*>(ws) + fwd_ws);
  float* beta = reinterpret_cast<float*>(static_cast<char*>(ws) + fwd_ws + align_up(n * 4));
  if (launch_unpack_factors(factors16, alpha, beta, n, as_stream(stream)) != hipSuccess) return QALORA_EHIP;
  return qalora_forward(&plain, tokens, x, packed, alpha, beta, nullptr, nullptr, y, y_dtype, ws, fwd_ws,
                        stream);
}

int qalora_beta_from_zero_point(const qalora_desc* d, const float* alpha, const float* z, float* beta,
                                void* stream) {
  const int rc = qalora_check_desc(d);
  if (rc != QALORA_OK) return rc;
  if (!alpha || !z || !beta) return QALORA_EINVAL;
  if (misaligned(alpha) || misaligned(z) || misaligned(beta)) return QALORA_EALIGN;
  const size_t n = (size_t)(d->d_in / d->group) * d->d_out;
  return launch_zero_point(alpha, z, beta, n, false, as_stream(stream)) == hipSuccess ? QALORA_OK : QALORA_EHIP;
}

int qalora_zero_point_from_beta(const qalora_desc* d, const float* alpha, const float* beta, float* z,
                                void* stream) {
  const int rc = qalora_check_desc(d);
  if (rc != QALORA_OK) return rc;
  if (!alpha || !beta || !z) return QALORA_EINVAL;
  if (misaligned(alpha) || misaligned(beta) || misaligned(z)) return QALORA_EALIGN;
  const size_t n = (size_t)(d->d_in / d->group) * d->d_out;
  return launch_zero_point(alpha, beta, z, n, true, as_stream(stream)) == hipSuccess ? QALORA_OK : QALORA_EHIP;
}

namespace {
// Block table of a tensor list; false if the list is not acceptable.
bool adamw_table(int n, const size_t* numel, OptTensors& t) {
  if (n < 1 || n > OPT_MAX_TENSORS || !numel) return false;
  unsigned long long blocks = 0;
  for (int i = 0; i < n; ++i) {
    if (numel[i] == 0) return false;
    t.numel[i] = numel[i];
    t.chunk_start[i] = (unsigned)blocks;
    blocks += (numel[i] + OPT_CHUNK - 1) / OPT_CHUNK;
    if (blocks > 0x7fffffffull) return false;
  }
  t.chunk_start[n] = (unsigned)blocks;
  t.n = n;
  return true;
}
}  // namespace

size_t qalora_adamw_workspace_bytes(int n_tensors, const size_t* numel) {
  OptTensors t{};
  if (!adamw_table(n_tensors, numel, t)) return 0;
  return align_up((size_t)t.chunk_start[t.n] * sizeof(float));
}

int qalora_adamw_step(const qalora_adamw* hp, int step, int n_tensors, float* const* params,
                      float* const* grads, float* const* exp_avg, float* const* exp_avg_sq,
                      const size_t* numel, int zero_grads, float* grad_norm, void* ws, size_t ws_bytes,
                      void* stream) {
  if (!hp || step < 1 || !params || !grads || !exp_avg || !exp_avg_sq) return QALORA_EINVAL;
  if (!(hp->beta1 >= 0.0f && hp->beta1 < 1.0f && hp->beta2 >= 0.0f && hp->beta2 < 1.0f) ||
      !(hp->eps >= 0.0f) || !(hp->lr >= 0.0f) || !(hp->weight_decay >= 0.0f))
    return QALORA_EINVAL;
  OptTensors t{};
  if (!adamw_table(n_tensors, numel, t)) return QALORA_EINVAL;
  for (int i = 0; i < n_tensors; ++i) {
    if (!params[i] || !grads[i] || !exp_avg[i] || !exp_avg_sq[i]) return QALORA_EINVAL;
    if (misaligned(params[i]) || misaligned(grads[i]) || misaligned(exp_avg[i]) || misaligned(exp_avg_sq[i]))
      return QALORA_EALIGN;
    t.p[i] = params[i];
    t.g[i] = grads[i];
    t.m[i] = exp_avg[i];
    t.v[i] = exp_avg_sq[i];
  }
  if (misaligned(grad_norm) || misaligned(ws)) return QALORA_EALIGN;
  const bool need_norm = hp->max_grad_norm > 0.0f || grad_norm;
  if (need_norm && (!ws || ws_bytes < (size_t)t.chunk_start[t.n] * sizeof(float))) return QALORA_EWORKSPACE;
  OptHyper h{};
  const double b1 = hp->beta1, b2 = hp->beta2;
  h.beta1 = hp->beta1;
  h.one_minus_beta1 = (float)(1.0 - b1);
  h.beta2 = hp->beta2;
  h.one_minus_beta2 = (float)(1.0 - b2);
  h.eps = hp->eps;
  h.decay = (float)(1.0 - (double)hp->lr * (double)hp->weight_decay);
  h.step_size = (float)((double)hp->lr / (1.0 - pow(b1, (double)step)));
  h.inv_sqrt_bias2 = (float)(1.0 / sqrt(1.0 - pow(b2, (double)step)));
  h.max_norm = hp->max_grad_norm;
  h.zero_grads = zero_grads ? 1 : 0;
  return launch_adamw(t, h, need_norm ? static_cast<float*>(ws) : nullptr, grad_norm, as_stream(stream)) ==
                 hipSuccess
             ? QALORA_OK
             : QALORA_EHIP;
}

int qalora_profile_arm(int direction, void* start_event, void* stop_event) {
  if (direction != 0 && direction != 1) return QALORA_EINVAL;
  g_profile_hook[direction] = ProfileHook{static_cast<hipEvent_t>(start_event),
                                          static_cast<hipEvent_t>(stop_event), nullptr, nullptr, 0};
  return QALORA_OK;
}

int qalora_profile_arm_blocks(int direction, void* times, int capacity) {
  if (direction != 0 && direction != 1) return QALORA_EINVAL;
  if (times && (misaligned(times) || capacity <= 0)) return times && capacity <= 0 ? QALORA_EINVAL : QALORA_EALIGN;
  g_profile_hook[direction].block_times = static_cast<unsigned long long*>(times);
  g_profile_hook[direction].block_times_cap = times ? capacity : 0;
  return QALORA_OK;
}

int qalora_profile_arm_clock(int direction, void* counts) {
  if (direction != 0 && direction != 1) return QALORA_EINVAL;
  if (counts && misaligned(counts)) return QALORA_EALIGN;
  g_profile_hook[direction].clock_probe = static_cast<unsigned long long*>(counts);
  return QALORA_OK;
}

int qalora_profile_wall_clock_khz(int* khz) {
  if (!khz) return QALORA_EINVAL;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return QALORA_EHIP;
  if (hipDeviceGetAttribute(khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess) return QALORA_EHIP;
  return QALORA_OK;
}

int qalora_profile_event_create(void** event) {
  if (!event) return QALORA_EINVAL;
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return QALORA_EHIP;
  *event = e;
  return QALORA_OK;
}

int qalora_profile_event_elapsed_ms(void* start_event, void* stop_event, float* ms) {
  if (!start_event || !stop_event || !ms) return QALORA_EINVAL;
  return hipEventElapsedTime(ms, static_cast<hipEvent_t>(start_event),
                             static_cast<hipEvent_t>(stop_event)) == hipSuccess
             ? QALORA_OK
             : QALORA_EHIP;
}

int qalora_profile_event_destroy(void* event) {
  if (!event) return QALORA_EINVAL;
  return hipEventDestroy(static_cast<hipEvent_t>(event)) == hipSuccess ? QALORA_OK : QALORA_EHIP;
}

int qalora_profile_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || bytes == 0 || bytes % 16 != 0) return QALORA_EINVAL;
  if (misaligned(dst) || misaligned(src)) return QALORA_EALIGN;
  const size_t n16 = bytes / 16;
  const unsigned blocks = (unsigned)((n16 + 1023) / 1024 < 8192 ? (n16 + 1023) / 1024 : 8192);
  profile_copy_kernel<<<blocks, 256, 0, as_stream(stream)>>>(static_cast<const uint4*>(src),
                                                              static_cast<uint4*>(dst), n16);
  return hipGetLastError() == hipSuccess ? QALORA_OK : QALORA_EHIP;
}

int qalora_profile_mfma_probe(int shape, int lds_reads, int valu_per_mfma, int iters, int blocks,
                              void* sink, void* counts, void* stream) {
  if (!sink || !counts || iters <= 0 || blocks <= 0 || blocks > 65536) return QALORA_EINVAL;
  if (misaligned(sink) || misaligned(counts)) return QALORA_EALIGN;
  const hipError_t e = launch_mfma_probe(shape, lds_reads, valu_per_mfma, static_cast<float*>(sink),
                                         static_cast<unsigned long long*>(counts), iters, blocks,
                                         as_stream(stream));
  if (e == hipErrorInvalidValue) return QALORA_EINVAL;
  return e == hipSuccess ? QALORA_OK : QALORA_EHIP;
}

int qalora_swiglu_forward(const void* gate, const void* up, void* h, size_t n, void* stream) {
  if (!gate || !up || !h || n == 0 || n % 8 != 0) return QALORA_EINVAL;
  if (misaligned(gate) || misaligned(up) || misaligned(h)) return QALORA_EALIGN;
  return launch_swiglu_forward(gate, up, h, n, as_stream(stream)) == hipSuccess ? QALORA_OK
                                                                                 : QALORA_EHIP;
}

int qalora_swiglu_backward(const void* dh, const void* gate, const void* up, void* dgate,
                           void* dup, size_t n, void* stream) {
  if (!dh || !gate || !up || !dgate || !dup || n == 0 || n % 8 != 0) return QALORA_EINVAL;
  if (misaligned(dh) || misaligned(gate) || misaligned(up) || misaligned(dgate) || misaligned(dup))
    return QALORA_EALIGN;
  return launch_swiglu_backward(dh, gate, up, dgate, dup, n, as_stream(stream)) == hipSuccess
             ? QALORA_OK
             : QALORA_EHIP;
}

int qalora_swiglu_forward_wide(const void* gu, void* h, size_t rows, size_t cols, void* stream) {
  if (!gu || !h || rows == 0 || cols == 0 || cols % 8 != 0) return QALORA_EINVAL;
  if (misaligned(gu) || misaligned(h)) return QALORA_EALIGN;
  return launch_swiglu_forward_wide(gu, h, rows, cols, as_stream(stream)) == hipSuccess ? QALORA_OK : QALORA_EHIP;
}

int qalora_swiglu_backward_wide(const void* dh, const void* gu, void* dgu, size_t rows, size_t cols,
                                void* stream) {
  if (!dh || !gu || !dgu || rows == 0 || cols == 0 || cols % 8 != 0) return QALORA_EINVAL;
  if (misaligned(dh) || misaligned(gu) || misaligned(dgu)) return QALORA_EALIGN;
  return launch_swiglu_backward_wide(dh, gu, dgu, rows, cols, as_stream(stream)) == hipSuccess ? QALORA_OK
                                                                                              : QALORA_EHIP;
}

}  // extern "C"
