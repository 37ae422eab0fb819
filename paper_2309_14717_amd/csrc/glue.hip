// Benchmark-harness glue, NOT part of the QA-LoRA layer: the elementwise part of a LLaMA
// SwiGLU MLP block, h = silu(gate) * up, and its backward.  It exists so that the MLP-block
// workload (three adapted linears around this function) is timed without a dozen framework
// elementwise launches in between.  bf16 in and out, fp32 arithmetic, 16-byte accesses.
#include "common.hpp"
#include "kernels.hpp"

namespace qalora {

namespace {
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float lo_f(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi_f(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float sigmoidf_(float v) { return 1.0f / (1.0f + __expf(-v)); }
}  // namespace

// Element i of the flat index space is 16-byte piece i % c8 of row i / c8; gate, up (and their
// gradients) have rows ld8 pieces apart, h (and dh) c8: ld8 = c8 for separate tensors, 2 c8 for
// the two halves of one [gate | up] tensor.
__global__ __launch_bounds__(256) void swiglu_fwd_kernel(const u32x4* __restrict__ gate,
                                                         const u32x4* __restrict__ up,
                                                         u32x4* __restrict__ h, size_t n8, size_t c8,
                                                         size_t ld8) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n8; i += stride) {
    const size_t gi = (i / c8) * ld8 + i % c8;
    const u32x4 g = gate[gi], u = up[gi];
    u32x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float g0 = lo_f(g[e]), g1 = hi_f(g[e]);
      o[e] = pack_bf16x2(g0 * sigmoidf_(g0) * lo_f(u[e]), g1 * sigmoidf_(g1) * hi_f(u[e]));
    }
    h[i] = o;
  }
}

// dgate = dh * up * d/dg[g sigmoid(g)] = dh * up * sig * (1 + g (1 - sig));  dup = dh * g * sig
__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const u32x4* __restrict__ dh,
                                                         const u32x4* __restrict__ gate,
                                                         const u32x4* __restrict__ up,
                                                         u32x4* __restrict__ dgate,
                                                         u32x4* __restrict__ dup, size_t n8, size_t c8,
                                                         size_t ld8) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n8; i += stride) {
    const size_t gi = (i / c8) * ld8 + i % c8;
    const u32x4 d = dh[i], g = gate[gi], u = up[gi];
    u32x4 og, ou;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float dg[2], du[2];
#pragma unroll
      for (int hsel = 0; hsel < 2; ++hsel) {
        const float dv = hsel ? hi_f(d[e]) : lo_f(d[e]);
        const float gv = hsel ? hi_f(g[e]) : lo_f(g[e]);
        const float uv = hsel ? hi_f(u[e]) : lo_f(u[e]);
        const float sg = sigmoidf_(gv);
        dg[hsel] = dv * uv * (sg * (1.0f + gv * (1.0f - sg)));
        du[hsel] = dv * gv * sg;
      }
      og[e] = pack_bf16x2(dg[0], dg[1]);
      ou[e] = pack_bf16x2(du[0], du[1]);
    }
    dgate[gi] = og;
    dup[gi] = ou;
  }
}

hipError_t launch_swiglu_forward(const void* gate, const void* up, void* h, size_t n, hipStream_t st) {
  const size_t n8 = n / 8;
  const unsigned blocks = (unsigned)((n8 + 255) / 256 < 4096 ? (n8 + 255) / 256 : 4096);
  swiglu_fwd_kernel<<<blocks, 256, 0, st>>>(static_cast<const u32x4*>(gate), static_cast<const u32x4*>(up),
                                            static_cast<u32x4*>(h), n8, n8, n8);
  return hipGetLastError();
}

hipError_t launch_swiglu_backward(const void* dh, const void* gate, const void* up, void* dgate,
                                  void* dup, size_t n, hipStream_t st) {
  const size_t n8 = n / 8;
  const unsigned blocks = (unsigned)((n8 + 255) / 256 < 4096 ? (n8 + 255) / 256 : 4096);
  swiglu_bwd_kernel<<<blocks, 256, 0, st>>>(static_cast<const u32x4*>(dh), static_cast<const u32x4*>(gate),
                                            static_cast<const u32x4*>(up), static_cast<u32x4*>(dgate),
                                            static_cast<u32x4*>(dup), n8, n8, n8);
  return hipGetLastError();
}

// The same on one [rows, 2 cols] tensor gu = [gate | up] (what a wide gate/up layer produces),
// with the gradients written to dgu = [dgate | dup].
hipError_t launch_swiglu_forward_wide(const void* gu, void* h, size_t rows, size_t cols, hipStream_t st) {
  const size_t c8 = cols / 8, n8 = rows * c8;
  const unsigned blocks = (unsigned)((n8 + 255) / 256 < 4096 ? (n8 + 255) / 256 : 4096);
  const u32x4* g = static_cast<const u32x4*>(gu);
  swiglu_fwd_kernel<<<blocks, 256, 0, st>>>(g, g + c8, static_cast<u32x4*>(h), n8, c8, 2 * c8);
  return hipGetLastError();
}

hipError_t launch_swiglu_backward_wide(const void* dh, const void* gu, void* dgu, size_t rows, size_t cols,
                                       hipStream_t st) {
  const size_t c8 = cols / 8, n8 = rows * c8;
  const unsigned blocks = (unsigned)((n8 + 255) / 256 < 4096 ? (n8 + 255) / 256 : 4096);
  const u32x4* g = static_cast<const u32x4*>(gu);
  u32x4* dg = static_cast<u32x4*>(dgu);
  swiglu_bwd_kernel<<<blocks, 256, 0, st>>>(static_cast<const u32x4*>(dh), g, g + c8, dg, dg + c8, n8, c8, 2 * c8);
  return hipGetLastError();
}

}  // namespace qalora
