// The optimiser step that follows the backward in the fine-tuning loop (Sec. 4.1, training
// details: AdamW, a maximum gradient norm, a constant learning rate), fused over all adapter
// tensors of a decoder layer: only A and B are parameters (Sec. 3.1), a few hundred thousand
// values per linear, so one launch per tensor would be nothing but launch latency.
//
//   norm  = || all gradients ||_2                     (joint over the tensors)
//   clip  = min(1, max_norm / (norm + 1e-6))          (1 when max_norm <= 0)
//   g     = clip * grad
//   m     = beta1 m + (1 - beta1) g
//   v     = beta2 v + (1 - beta2) g^2
//   p     = p (1 - lr wd) - (lr / (1 - beta1^t)) m / (sqrt(v) / sqrt(1 - beta2^t) + eps)
//
// Two launches: per-block sums of squares, then the update, whose blocks each add the block
// sums in the same fixed order (fp64) -- no atomics, so a step is bit-reproducible.  The
// tensor table travels by value in the kernel arguments: the library allocates nothing.
#include "common.hpp"
#include "kernels.hpp"

namespace qalora {

namespace {

constexpr int OPT_THREADS = 256;
constexpr int OPT_PER_THREAD = OPT_CHUNK / OPT_THREADS;  // 16

__device__ __forceinline__ int opt_find_tensor(const OptTensors& t, unsigned b) {
  int ti = 0;
  while (ti + 1 < t.n && b >= t.chunk_start[ti + 1]) ++ti;  // at most 31 steps, uniform per block
  return ti;
}

// fixed-order sum over the block; every thread gets the result
template <typename T>
__device__ __forceinline__ T opt_block_sum(T v, T* lds) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) lds[wave] = v;
  __syncthreads();
  const T r = ((lds[0] + lds[1]) + lds[2]) + lds[3];
  __syncthreads();
  return r;
}

}  // namespace

// One element of the update.
__device__ __forceinline__ void opt_update_one(float& p, float g, float& m, float& v, float clip, const OptHyper& h) {
  const float gv = clip * g;
  m = __builtin_fmaf(h.beta1, m, h.one_minus_beta1 * gv);
  v = __builtin_fmaf(h.beta2, v, h.one_minus_beta2 * gv * gv);
  const float denom = __fsqrt_rn(v) * h.inv_sqrt_bias2 + h.eps;
  p = __builtin_fmaf(p, h.decay, -h.step_size * __fdiv_rn(m, denom));
}

// A block owns OPT_CHUNK consecutive elements of one tensor: 16-byte accesses when the tensor's
// length is a multiple of four (every adapter matrix of a supported layer), 4-byte ones otherwise.
__global__ __launch_bounds__(OPT_THREADS) void opt_sumsq_kernel(const OptTensors t, float* __restrict__ partial) {
  __shared__ float lds[4];
  const int ti = opt_find_tensor(t, blockIdx.x);
  const unsigned long long base = (unsigned long long)(blockIdx.x - t.chunk_start[ti]) * OPT_CHUNK;
  const unsigned long long n = t.numel[ti];
  const float* g = t.g[ti];
  float acc = 0.0f;
  if ((n & 3) == 0) {
#pragma unroll
    for (int k = 0; k < OPT_PER_THREAD / 4; ++k) {
      const unsigned long long i = base + 4ull * (threadIdx.x + (unsigned long long)k * OPT_THREADS);
      if (i < n) {
        const f32x4 gv = *reinterpret_cast<const f32x4*>(g + i);
#pragma unroll
        for (int c = 0; c < 4; ++c) acc = __builtin_fmaf(gv[c], gv[c], acc);
      }
    }
  } else {
#pragma unroll 4
    for (int k = 0; k < OPT_PER_THREAD; ++k) {
      const unsigned long long i = base + threadIdx.x + (unsigned long long)k * OPT_THREADS;
      const float gv = i < n ? g[i] : 0.0f;
      acc = __builtin_fmaf(gv, gv, acc);
    }
  }
  acc = opt_block_sum(acc, lds);
  if (threadIdx.x == 0) partial[blockIdx.x] = acc;
}

__global__ __launch_bounds__(OPT_THREADS) void opt_update_kernel(const OptTensors t, const OptHyper h,
                                                                 const float* __restrict__ partial,
                                                                 float* __restrict__ norm_out) {
  __shared__ double lds[4];
  float clip = 1.0f;
  if (partial) {
    double acc = 0.0;
    for (unsigned i = threadIdx.x; i < gridDim.x; i += OPT_THREADS) acc += (double)partial[i];
    const double norm = sqrt(opt_block_sum(acc, lds));
    if (h.max_norm > 0.0f) clip = (float)fmin(1.0, (double)h.max_norm / (norm + 1e-6));
    if (norm_out && blockIdx.x == 0 && threadIdx.x == 0) *norm_out = (float)norm;
  }
  const int ti = opt_find_tensor(t, blockIdx.x);
  const unsigned long long base = (unsigned long long)(blockIdx.x - t.chunk_start[ti]) * OPT_CHUNK;
  const unsigned long long n = t.numel[ti];
  float* __restrict__ p = t.p[ti];
  float* __restrict__ g = t.g[ti];
  float* __restrict__ m = t.m[ti];
  float* __restrict__ v = t.v[ti];
  if ((n & 3) == 0) {
#pragma unroll
    for (int k = 0; k < OPT_PER_THREAD / 4; ++k) {
      const unsigned long long i = base + 4ull * (threadIdx.x + (unsigned long long)k * OPT_THREADS);
      if (i < n) {
        f32x4 pv = *reinterpret_cast<f32x4*>(p + i), mv = *reinterpret_cast<f32x4*>(m + i),
              vv = *reinterpret_cast<f32x4*>(v + i);
        const f32x4 gv = *reinterpret_cast<const f32x4*>(g + i);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          float pc = pv[c], mc = mv[c], vc = vv[c];
          opt_update_one(pc, gv[c], mc, vc, clip, h);
          pv[c] = pc;
          mv[c] = mc;
          vv[c] = vc;
        }
        *reinterpret_cast<f32x4*>(p + i) = pv;
        *reinterpret_cast<f32x4*>(m + i) = mv;
        *reinterpret_cast<f32x4*>(v + i) = vv;
        if (h.zero_grads) *reinterpret_cast<f32x4*>(g + i) = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
      }
    }
  } else {
#pragma unroll 4
    for (int k = 0; k < OPT_PER_THREAD; ++k) {
      const unsigned long long i = base + threadIdx.x + (unsigned long long)k * OPT_THREADS;
      if (i < n) {
        float pv = p[i], mv = m[i], vv = v[i];
        opt_update_one(pv, g[i], mv, vv, clip, h);
        p[i] = pv;
        m[i] = mv;
        v[i] = vv;
        if (h.zero_grads) g[i] = 0.0f;
      }
    }
  }
}

// `partial` may be null when neither the clip nor the norm is wanted.
hipError_t launch_adamw(const OptTensors& t, const OptHyper& h, float* partial, float* norm_out, hipStream_t st) {
  const unsigned blocks = t.chunk_start[t.n];
  if (blocks == 0) return hipSuccess;
  if (partial) {
    opt_sumsq_kernel<<<blocks, OPT_THREADS, 0, st>>>(t, partial);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  }
  opt_update_kernel<<<blocks, OPT_THREADS, 0, st>>>(t, h, partial, norm_out);
  return hipGetLastError();
}

}  // namespace qalora
