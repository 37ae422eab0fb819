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

__global__ __launch_bounds__(256) void swiglu_fwd_kernel(const u32x4* __restrict__ gate,
                                                         const u32x4* __restrict__ up,
                                                         u32x4* __restrict__ h, size_t n8) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n8; i += stride) {
    const u32x4 g = gate[i], u = up[i];
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
                                                         u32x4* __restrict__ dup, size_t n8) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n8; i += stride) {
    const u32x4 d = dh[i], g = gate[i], u = up[i];
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
    dgate[i] = og;
    dup[i] = ou;
  }
}

hipError_t launch_swiglu_forward(const void* gate, const void* up, void* h, size_t n, hipStream_t st) {
  const size_t n8 = n / 8;
  const unsigned blocks = (unsigned)((n8 + 255) / 256 < 4096 ? (n8 + 255) / 256 : 4096);
  swiglu_fwd_kernel<<<blocks, 256, 0, st>>>(static_cast<const u32x4*>(gate), static_cast<const u32x4*>(up),
                                            static_cast<u32x4*>(h), n8);
  return hipGetLastError();
}

hipError_t launch_swiglu_backward(const void* dh, const void* gate, const void* up, void* dgate,
                                  void* dup, size_t n, hipStream_t st) {
  const size_t n8 = n / 8;
  const unsigned blocks = (unsigned)((n8 + 255) / 256 < 4096 ? (n8 + 255) / 256 : 4096);
  swiglu_bwd_kernel<<<blocks, 256, 0, st>>>(static_cast<const u32x4*>(dh), static_cast<const u32x4*>(gate),
                                            static_cast<const u32x4*>(up), static_cast<u32x4*>(dgate),
                                            static_cast<u32x4*>(dup), n8);
  return hipGetLastError();
}

}  // namespace qalora
