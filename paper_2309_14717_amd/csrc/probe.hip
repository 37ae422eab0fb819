// Measurement aid, not part of the layer: issue-rate probes for the matrix cores of gfx950.
//
// A block runs the inner loop of a dense contraction with everything but the instruction mix
// taken away -- v_mfma_f32_32x32x16_f16 on accumulators that live in registers, optionally the
// operand-fragment reads from LDS that feed them, optionally n ordinary vector instructions
// behind every matrix instruction -- and its first thread reports how many shader cycles and
// wall-clock ticks the loop took.  cycles / (matrix instructions per SIMD) is the issue
// interval; cycles / ticks the clock the chip held under that mix.  The numbers say what the
// dequantising contraction kernel can reach at best: what the matrix cores sustain when all
// compute units run them, what the fragment reads cost, and whether vector work hides under
// matrix work on the same SIMD.
#include "common.hpp"
#include "kernels.hpp"

namespace qalora {

namespace {

typedef uint32_t pu32x4 __attribute__((ext_vector_type(4)));

// WAVES x 64 threads; every wavefront owns TM x TN accumulator tiles of 32 x 32.
//   (8, 4, 2): the contraction kernel's shape, two wavefronts per SIMD, 6 fragment reads per 8 MFMAs
//   (4, 4, 4): one wavefront per SIMD, 8 fragment reads per 16 MFMAs
// LDS : fetch the fragments of the next K-16 slice from LDS under the current slice's MFMAs
// NV  : vector instructions (v_and_or_b32 on private registers) issued behind every MFMA;
//       100 + n: n per MFMA, issued as one burst behind the MFMAs of a K-16 slice
// ACC : keep the accumulators in the accumulation registers (AGPRs).  With eight wavefronts per
//       block the compiler otherwise keeps them in ordinary vector registers.
template <int WAVES, int TM, int TN, bool LDS, int NV, bool ACC = false>
__global__ __launch_bounds__(WAVES * 64) void mfma_probe_kernel(float* sink, unsigned long long* counts,
                                                                int iters) {
  // 64 KB of fp16 values of either sign with magnitudes in [0.5, 2) and hashed mantissas:
  // operands that toggle the data paths the way real tiles do (constant operands would let the
  // chip hold a clock it does not hold on real data)
  __shared__ pu32x4 lds[4096];
  for (int i = threadIdx.x; i < 4096; i += WAVES * 64) {
    pu32x4 v;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      uint32_t h = (uint32_t)(i * 4 + c) * 0x9e3779b9u + blockIdx.x * 0x85ebca6bu;
      h ^= h >> 15;
      h *= 0x2c1b3c6du;
      h ^= h >> 12;
      // per half-word: sign, exponent 14 or 15 (0.5 .. 2), ten mantissa bits
      v[c] = (h & 0x87ff87ffu) | 0x38003800u;
    }
    lds[i] = v;
  }
  __syncthreads();
  if constexpr (ACC) {  // one use of the register class makes the compiler place MFMA results there
    float hint = 0.0f;
    asm volatile("" : "+a"(hint));
  }
  f32x16 acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;
  pu32x4 af[TM], bf[TN];
#pragma unroll
  for (int a = 0; a < TM; ++a) af[a] = lds[(threadIdx.x + a * 512) & 4095];
#pragma unroll
  for (int b = 0; b < TN; ++b) bf[b] = lds[(threadIdx.x + 2048 + b * 512) & 4095];
  uint32_t jj[8];
#pragma unroll
  for (int v = 0; v < 8; ++v) jj[v] = threadIdx.x + v;
  const unsigned long long c0 = clock64(), w0 = wall_clock64();
#pragma nounroll
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {  // four K-16 slices = one K step of 64
      pu32x4 na[TM], nb[TN];
      if constexpr (LDS) {
#pragma unroll
        for (int a = 0; a < TM; ++a) na[a] = lds[(threadIdx.x + a * 512 + kk * 64 + it) & 4095];
#pragma unroll
        for (int b = 0; b < TN; ++b) nb[b] = lds[(threadIdx.x + 2048 + b * 512 + kk * 64 + it) & 4095];
      }
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) {
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, af[a]),
                                                             __builtin_bit_cast(f16x8, bf[b]), acc[a][b], 0, 0, 0);
#pragma unroll
          for (int v = 0; v < NV % 100; ++v)
            asm volatile("v_and_or_b32 %0, %1, %2, %3"
                         : "=v"(jj[v & 7])
                         : "v"(jj[(v + 1) & 7]), "s"(0x0f0f0f0f), "v"(jj[(v + 3) & 7]));
        }
      if constexpr (LDS) {
#pragma unroll
        for (int a = 0; a < TM; ++a) af[a] = na[a];
#pragma unroll
        for (int b = 0; b < TN; ++b) bf[b] = nb[b];
        if constexpr (NV >= 100) {  // all matrix instructions of the slice, then all vector work
          __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, TM * TN, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, (NV % 100) * TM * TN, 0);
        } else {
#pragma unroll
          for (int i = 0; i < TM * TN; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // LDS read
            if constexpr (NV > 0) __builtin_amdgcn_sched_group_barrier(0x002, NV, 0);
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  // the block is done when its last wavefront is: the issue arbiter favours the oldest
  // wavefront of a SIMD, so the first one alone would report the rate of a SIMD it does not share
  __syncthreads();
  const unsigned long long c1 = clock64(), w1 = wall_clock64();
  float s = 0.0f;
#pragma unroll
  for (int v = 0; v < 8; ++v) s += (float)jj[v];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) s += acc[a][b][r];
  sink[blockIdx.x * (WAVES * 64) + threadIdx.x] = s;
  if (threadIdx.x == 0) {
    counts[2 * blockIdx.x] = c1 - c0;
    counts[2 * blockIdx.x + 1] = w1 - w0;
  }
}

template <int WAVES, int TM, int TN, bool LDS, int NV, bool ACC = false>
hipError_t run(float* sink, unsigned long long* counts, int iters, int blocks, hipStream_t st) {
  mfma_probe_kernel<WAVES, TM, TN, LDS, NV, ACC><<<blocks, WAVES * 64, 0, st>>>(sink, counts, iters);
  return hipGetLastError();
}

}  // namespace

// shape 0: eight wavefronts x (4 x 2) tiles; shape 1: four wavefronts x (4 x 4) tiles; shape 2:
// shape 0 with the accumulators in AGPRs.
// Returns hipErrorInvalidValue for a combination that is not built.
hipError_t launch_mfma_probe(int shape, int lds_reads, int valu_per_mfma, float* sink,
                             unsigned long long* counts, int iters, int blocks, hipStream_t st) {
  if (shape == 0) {
    if (!lds_reads) return valu_per_mfma == 0 ? run<8, 4, 2, false, 0>(sink, counts, iters, blocks, st)
                                              : hipErrorInvalidValue;
    switch (valu_per_mfma) {
      case 0: return run<8, 4, 2, true, 0>(sink, counts, iters, blocks, st);
      case 1: return run<8, 4, 2, true, 1>(sink, counts, iters, blocks, st);
      case 2: return run<8, 4, 2, true, 2>(sink, counts, iters, blocks, st);
      case 3: return run<8, 4, 2, true, 3>(sink, counts, iters, blocks, st);
      case 102: return run<8, 4, 2, true, 102>(sink, counts, iters, blocks, st);
      case 104: return run<8, 4, 2, true, 104>(sink, counts, iters, blocks, st);
      case 4: return run<8, 4, 2, true, 4>(sink, counts, iters, blocks, st);
      case 6: return run<8, 4, 2, true, 6>(sink, counts, iters, blocks, st);
      case 8: return run<8, 4, 2, true, 8>(sink, counts, iters, blocks, st);
      default: return hipErrorInvalidValue;
    }
  }
  if (shape == 1) {
    if (!lds_reads) return valu_per_mfma == 0 ? run<4, 4, 4, false, 0>(sink, counts, iters, blocks, st)
                                              : hipErrorInvalidValue;
    switch (valu_per_mfma) {
      case 0: return run<4, 4, 4, true, 0>(sink, counts, iters, blocks, st);
      case 2: return run<4, 4, 4, true, 2>(sink, counts, iters, blocks, st);
      case 4: return run<4, 4, 4, true, 4>(sink, counts, iters, blocks, st);
      case 6: return run<4, 4, 4, true, 6>(sink, counts, iters, blocks, st);
      case 8: return run<4, 4, 4, true, 8>(sink, counts, iters, blocks, st);
      default: return hipErrorInvalidValue;
    }
  }
  if (shape == 2) {
    if (!lds_reads) return valu_per_mfma == 0 ? run<8, 4, 2, false, 0, true>(sink, counts, iters, blocks, st)
                                              : hipErrorInvalidValue;
    switch (valu_per_mfma) {
      case 0: return run<8, 4, 2, true, 0, true>(sink, counts, iters, blocks, st);
      case 2: return run<8, 4, 2, true, 2, true>(sink, counts, iters, blocks, st);
      case 4: return run<8, 4, 2, true, 4, true>(sink, counts, iters, blocks, st);
      default: return hipErrorInvalidValue;
    }
  }
  return hipErrorInvalidValue;
}

}  // namespace qalora
