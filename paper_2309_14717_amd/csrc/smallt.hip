// Adapter-free forward for a handful of tokens (T <= 16): the memory-bound regime of
// post-merge inference, where every call streams the whole quantized weight once.
//
//   y[t,j] = sum_l ( alpha[l,j] * sum_{i in group l} x[t,i] code[i,j]  +  beta[l,j] * sum_{i in l} x[t,i] )
//
// (Eq. 1 per group pulled out of the inner sum.)  The inner sums run on the matrix cores with
// EXACT operands: x is bf16 already, and a 4-bit code c becomes the bf16 number 128 + c by
// OR-ing it into the mantissa of 0x4300 -- no int->float conversion, no rounding.  The extra
// 128 * sum(x) is folded into beta.  One more MFMA against a matrix of ones yields the group
// sums of x in exactly the accumulator layout the update needs.  alpha and beta are applied in
// fp32 once per group, so this path is more accurate than the large-T one.
//
// Streaming: a wavefront owns 64 output columns and a range of groups; per group it issues
// three 16-byte loads per lane (codes, alpha, beta: 1 KB + 256 B + 256 B contiguous pieces) and
// one for x.  The eight wavefronts of a block split the groups of one 64-column slab and
// combine through LDS in fixed order; blocks may further split K (partials reduced by a
// second small kernel, fixed order).
#include "common.hpp"
#include "kernels.hpp"

namespace qalora {

constexpr int ST_WAVES = 8;

__global__ __launch_bounds__(64 * ST_WAVES) void smallt_kernel(const SmallTArgs p) {
  __shared__ float red[ST_WAVES][16][64];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 15, kb = lane >> 4;
  const int j0 = blockIdx.x * 64 + 4 * n;  // this lane's 4 columns
  const bool col_ok = j0 < p.d_out;
  const int L = p.d_in / p.group;
  const int sub = p.group / 32;  // 32-row MFMA blocks per group

  // groups of this block, then of this wavefront
  const int per_block = ceil_div(L, (int)gridDim.y);
  const int gb = blockIdx.y * per_block, ge = min(L, gb + per_block);
  const int per_wave = ceil_div(max(ge - gb, 0), ST_WAVES);
  const int l_begin = gb + wave * per_wave, l_end = min(ge, l_begin + per_wave);

  f32x4 acc[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) acc[q] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

  const uint32_t kMask = 0x000f000fu;
  const bf16x8 ones = __builtin_bit_cast(bf16x8, uint4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u});
  const bool row_ok = n < p.T;  // A operand row = token n
  const uint16_t* xrow = p.x + (size_t)(row_ok ? n : 0) * p.d_in + 8 * kb;
  const uint32_t* wcol = p.plane0 + (size_t)kb * p.d_out + (col_ok ? j0 : 0);

#pragma unroll 2
  for (int l = l_begin; l < l_end; ++l) {
    f32x4 d[4], dsx = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int q = 0; q < 4; ++q) d[q] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    for (int sb = 0; sb < sub; ++sb) {
      const int i0 = l * p.group + 32 * sb;
      uint4 w = *reinterpret_cast<const uint4*>(wcol + (size_t)(i0 / 8) * p.d_out);
      uint4 xa = *reinterpret_cast<const uint4*>(xrow + i0);
      if (!row_ok) xa = uint4{0, 0, 0, 0};
      if (!col_ok) w = uint4{0, 0, 0, 0};
      const bf16x8 a = __builtin_bit_cast(bf16x8, xa);
      const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        uint4 b;
        b.x = (ww[q] & kMask) | 0x43004300u;
        b.y = ((ww[q] >> 4) & kMask) | 0x43004300u;
        b.z = ((ww[q] >> 8) & kMask) | 0x43004300u;
        b.w = ((ww[q] >> 12) & kMask) | 0x43004300u;
        d[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, b), d[q], 0, 0, 0);
      }
      dsx = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, ones, dsx, 0, 0, 0);
    }
    f32x4 al = f32x4{0.0f, 0.0f, 0.0f, 0.0f}, be = al;
    if (col_ok) {
      al = *reinterpret_cast<const f32x4*>(p.alpha + (size_t)l * p.d_out + j0);
      be = *reinterpret_cast<const f32x4*>(p.beta + (size_t)l * p.d_out + j0);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float bp = __builtin_fmaf(-128.0f, al[q], be[q]);  // codes carry a +128 offset
#pragma unroll
      for (int r = 0; r < 4; ++r)
        acc[q][r] = __builtin_fmaf(al[q], d[q][r], __builtin_fmaf(bp, dsx[r], acc[q][r]));
    }
  }

  // combine the wavefronts of the block in fixed order
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int r = 0; r < 4; ++r) red[wave][4 * q + r][lane] = acc[q][r];
  __syncthreads();
  // wavefront w finishes accumulator registers 2w and 2w+1
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const int reg = 2 * wave + e;
    float v = 0.0f;
#pragma unroll
    for (int w = 0; w < ST_WAVES; ++w) v += red[w][reg][lane];
    const int q = reg >> 2, r = reg & 3;
    const int row = 4 * kb + r, col = j0 + q;  // D layout: lane (n, kb) holds rows 4*kb + r
    if (row < p.T && col_ok) {
      if (gridDim.y > 1) {
        p.partial[((size_t)blockIdx.y * p.T + row) * p.d_out + col] = v;
      } else if (p.out_bf16) {
        static_cast<uint16_t*>(p.out)[(size_t)row * p.d_out + col] = f32_to_bf16_bits(v);
      } else {
        static_cast<float*>(p.out)[(size_t)row * p.d_out + col] = v;
      }
    }
  }
}

__global__ __launch_bounds__(256) void smallt_reduce_kernel(const float* __restrict__ partial,
                                                            int nparts, size_t n, void* out,
                                                            int out_bf16) {
  const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i >= n) return;
  float v = 0.0f;
  for (int z = 0; z < nparts; ++z) v += partial[(size_t)z * n + i];
  if (out_bf16)
    static_cast<uint16_t*>(out)[i] = f32_to_bf16_bits(v);
  else
    static_cast<float*>(out)[i] = v;
}

int smallt_ksplit(int d_in, int d_out, int group) {
  const int slabs = ceil_div(d_out, 64);
  const int L = d_in / group;
  int ks = ceil_div(640, slabs);            // aim for a few blocks per compute unit
  const int max_ks = L / (ST_WAVES * 4);    // but keep >= 4 groups per wavefront
  if (ks > max_ks) ks = max_ks;
  if (ks > 16) ks = 16;
  return ks < 1 ? 1 : ks;
}

hipError_t launch_smallt(const SmallTArgs& a, int ksplit, hipStream_t st) {
  dim3 grid(ceil_div(a.d_out, 64), ksplit);
  smallt_kernel<<<grid, 64 * ST_WAVES, 0, st>>>(a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || ksplit == 1) return e;
  const size_t n = (size_t)a.T * a.d_out;
  smallt_reduce_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(a.partial, ksplit, n, a.out,
                                                                    a.out_bf16);
  return hipGetLastError();
}

}  // namespace qalora
