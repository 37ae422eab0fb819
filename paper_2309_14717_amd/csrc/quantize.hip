// Group-wise min-max quantization (Eq. 1 of the paper applied to each group of g
// consecutive rows of each column, Sec. 3.3), and pack / unpack between the canonical
// one-code-per-byte matrix and the private bit-packed format.
//
// HBM-bound, one pass over W plus a second pass that hits L2: a thread owns four adjacent
// columns of one group, adjacent threads own adjacent column quads, so every load and store
// is a coalesced 16-byte access along D_out.
#include <type_traits>

#include "common.hpp"
#include "kernels.hpp"

namespace qalora {

// The arithmetic below is the fp32 recipe of the C ABI, operation by operation, with
// explicit round-to-nearest intrinsics so that no contraction or reciprocal sneaks in.
// A thread owns four adjacent columns of one group: 16-byte loads and stores, and four
// independent min/max and code chains per thread to keep loads in flight.
// GKEEP = 32: the group has 32 rows and they stay in registers between the two passes (W is
// then read exactly once); GKEEP = 0: any group size, the code pass reads the rows again.
template <int NBITS, int GKEEP>
__global__ __launch_bounds__(256) void quantize_kernel(const float* __restrict__ W,
                                                       uint32_t* __restrict__ plane0,
                                                       uint32_t* __restrict__ plane1,
                                                       float* __restrict__ alpha,
                                                       float* __restrict__ beta, int d_in,
                                                       int d_out, int g) {
  const int j = 4 * (blockIdx.x * blockDim.x + threadIdx.x);  // d_out is a multiple of 8
  const int l = blockIdx.y;
  if (j >= d_out) return;
  const int i0 = l * g;
  const float* col = W + (size_t)i0 * d_out + j;
  f32x4 mn = *reinterpret_cast<const f32x4*>(col);
  f32x4 mx = mn;
  constexpr int KEEP_N = GKEEP > 0 ? GKEEP : 1;
  f32x4 keep[KEEP_N];
  if constexpr (GKEEP > 0) {
#pragma unroll
    for (int q = 0; q < GKEEP; ++q) keep[q] = *reinterpret_cast<const f32x4*>(col + (size_t)q * d_out);
#pragma unroll
    for (int q = 0; q < GKEEP; ++q)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if (keep[q][c] < mn[c]) mn[c] = keep[q][c];
        if (keep[q][c] > mx[c]) mx[c] = keep[q][c];
      }
  } else {
    for (int q0 = 0; q0 < g; q0 += 8) {  // g is a multiple of 8: eight rows' loads in flight
      f32x4 w[8];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        w[u] = *reinterpret_cast<const f32x4*>(col + (size_t)(q0 + u) * d_out);
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          if (w[u][c] < mn[c]) mn[c] = w[u][c];
          if (w[u][c] > mx[c]) mx[c] = w[u][c];
        }
    }
  }
  constexpr int QMAX = (1 << NBITS) - 1;
  f32x4 a;
  bool degenerate[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const float range = __fsub_rn(mx[c], mn[c]);
    a[c] = __fdiv_rn(range, (float)QMAX);
    degenerate[c] = !(a[c] > 0.0f);
    if (degenerate[c]) a[c] = 0x1p-60f;
  }
  *reinterpret_cast<f32x4*>(alpha + (size_t)l * d_out + j) = a;
  *reinterpret_cast<f32x4*>(beta + (size_t)l * d_out + j) = mn;

  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  constexpr int RB0 = PackFmt<NBITS>::kRowsPerWord0;
  constexpr int LOW_BITS = (NBITS == 3) ? 2 : NBITS;
  constexpr int ROWS = (NBITS == 3) ? 32 : RB0;  // rows handled per outer step
  auto code_rows = [&](int q0, auto in_regs) {
    u32x4 hiword = {0, 0, 0, 0};
#pragma unroll
    for (int h = 0; h < ROWS / RB0; ++h) {
      u32x4 word = {0, 0, 0, 0};
#pragma unroll
      for (int p = 0; p < RB0; ++p) {
        f32x4 w;
        if constexpr (decltype(in_regs)::value)
          w = keep[q0 + h * RB0 + p];  // a constant index once the caller's loop is unrolled
        else
          w = *reinterpret_cast<const f32x4*>(col + (size_t)(q0 + h * RB0 + p) * d_out);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          int code = 0;
          if (!degenerate[c]) {
            const float d = __fsub_rn(w[c], mn[c]);
            const float r = rintf(__fdiv_rn(d, a[c]));
            code = (int)r;
            code = code < 0 ? 0 : (code > QMAX ? QMAX : code);
          }
          word[c] |= (uint32_t)(code & ((1 << LOW_BITS) - 1)) << (LOW_BITS * (p >> 1) + 16 * (p & 1));
          if constexpr (NBITS == 3) {
            const int pp = h * RB0 + p;
            hiword[c] |= (uint32_t)(code >> 2) << ((pp >> 1) + 16 * (pp & 1));
          }
        }
      }
      *reinterpret_cast<u32x4*>(plane0 + (size_t)((i0 + q0) / RB0 + h) * d_out + j) = word;
    }
    if constexpr (NBITS == 3)
      *reinterpret_cast<u32x4*>(plane1 + (size_t)((i0 + q0) / 32) * d_out + j) = hiword;
  };
  if constexpr (GKEEP > 0) {
    static_assert(GKEEP % ROWS == 0 || GKEEP == 0, "whole words");
#pragma unroll
    for (int w = 0; w < GKEEP / ROWS; ++w) code_rows(w * ROWS, std::true_type{});
  } else {
    for (int q0 = 0; q0 < g; q0 += ROWS) code_rows(q0, std::false_type{});
  }
}

// One thread rebuilds the codes of 8 rows of one column.
template <int NBITS>
__global__ __launch_bounds__(256) void unpack_kernel(const uint32_t* __restrict__ plane0,
                                                     const uint32_t* __restrict__ plane1,
                                                     uint8_t* __restrict__ codes, int d_in,
                                                     int d_out) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  const int i0 = blockIdx.y * 8;
  if (j >= d_out || i0 >= d_in) return;
  constexpr int RB0 = PackFmt<NBITS>::kRowsPerWord0;
  uint32_t w0 = plane0[(size_t)(i0 / RB0) * d_out + j] >> patch_preshift0<NBITS>(i0);
  uint32_t w1 = 0;
  if constexpr (NBITS == 3) w1 = plane1[(size_t)(i0 / 32) * d_out + j] >> patch_preshift1(i0);
#pragma unroll
  for (int p = 0; p < 8; ++p)
    codes[(size_t)(i0 + p) * d_out + j] = (uint8_t)patch_code<NBITS>(w0, w1, p);
}

// One thread builds the word(s) of ROWS consecutive rows of one column.
template <int NBITS>
__global__ __launch_bounds__(256) void pack_kernel(const uint8_t* __restrict__ codes,
                                                   uint32_t* __restrict__ plane0,
                                                   uint32_t* __restrict__ plane1, int d_in,
                                                   int d_out) {
  constexpr int RB0 = PackFmt<NBITS>::kRowsPerWord0;
  constexpr int LOW_BITS = (NBITS == 3) ? 2 : NBITS;
  constexpr int ROWS = (NBITS == 3) ? 32 : RB0;
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  const int i0 = blockIdx.y * ROWS;
  if (j >= d_out || i0 >= d_in) return;
  uint32_t hiword = 0;
#pragma unroll
  for (int h = 0; h < ROWS / RB0; ++h) {
    uint32_t word = 0;
#pragma unroll
    for (int p = 0; p < RB0; ++p) {
      const uint32_t c = codes[(size_t)(i0 + h * RB0 + p) * d_out + j] & ((1u << NBITS) - 1);
      word |= (c & ((1u << LOW_BITS) - 1)) << (LOW_BITS * (p >> 1) + 16 * (p & 1));
      if constexpr (NBITS == 3) {
        const int pp = h * RB0 + p;
        hiword |= (c >> 2) << ((pp >> 1) + 16 * (pp & 1));
      }
    }
    plane0[(size_t)(i0 / RB0 + h) * d_out + j] = word;
  }
  if constexpr (NBITS == 3) plane1[(size_t)(i0 / 32) * d_out + j] = hiword;
}

template <int NBITS>
static void quantize_n(const float* W, uint32_t* p0, uint32_t* p1, float* alpha, float* beta,
                       int d_in, int d_out, int g, hipStream_t st) {
  dim3 grid(ceil_div(d_out, 4 * 256), d_in / g);
  if (g == 32)
    quantize_kernel<NBITS, 32><<<grid, 256, 0, st>>>(W, p0, p1, alpha, beta, d_in, d_out, g);
  else
    quantize_kernel<NBITS, 0><<<grid, 256, 0, st>>>(W, p0, p1, alpha, beta, d_in, d_out, g);
}
template <int NBITS>
static void unpack_n(const uint32_t* p0, const uint32_t* p1, uint8_t* codes, int d_in, int d_out,
                     hipStream_t st) {
  dim3 grid(ceil_div(d_out, 256), d_in / 8);
  unpack_kernel<NBITS><<<grid, 256, 0, st>>>(p0, p1, codes, d_in, d_out);
}
template <int NBITS>
static void pack_n(const uint8_t* codes, uint32_t* p0, uint32_t* p1, int d_in, int d_out,
                   hipStream_t st) {
  constexpr int ROWS = (NBITS == 3) ? 32 : PackFmt<NBITS>::kRowsPerWord0;
  dim3 grid(ceil_div(d_out, 256), d_in / ROWS);
  pack_kernel<NBITS><<<grid, 256, 0, st>>>(codes, p0, p1, d_in, d_out);
}

void launch_quantize(int bits, const float* W, void* packed, float* alpha, float* beta, int d_in,
                     int d_out, int g, hipStream_t st) {
  uint32_t* p0 = static_cast<uint32_t*>(packed);
  uint32_t* p1 = p0 + plane0_words(bits, d_in, d_out);
  if (bits == 4) quantize_n<4>(W, p0, p1, alpha, beta, d_in, d_out, g, st);
  else if (bits == 3) quantize_n<3>(W, p0, p1, alpha, beta, d_in, d_out, g, st);
  else quantize_n<2>(W, p0, p1, alpha, beta, d_in, d_out, g, st);
}

void launch_unpack(int bits, const void* packed, uint8_t* codes, int d_in, int d_out,
                   hipStream_t st) {
  const uint32_t* p0 = static_cast<const uint32_t*>(packed);
  const uint32_t* p1 = p0 + plane0_words(bits, d_in, d_out);
  if (bits == 4) unpack_n<4>(p0, p1, codes, d_in, d_out, st);
  else if (bits == 3) unpack_n<3>(p0, p1, codes, d_in, d_out, st);
  else unpack_n<2>(p0, p1, codes, d_in, d_out, st);
}

void launch_pack(int bits, const uint8_t* codes, void* packed, int d_in, int d_out,
                 hipStream_t st) {
  uint32_t* p0 = static_cast<uint32_t*>(packed);
  uint32_t* p1 = p0 + plane0_words(bits, d_in, d_out);
  if (bits == 4) pack_n<4>(codes, p0, p1, d_in, d_out, st);
  else if (bits == 3) pack_n<3>(codes, p0, p1, d_in, d_out, st);
  else pack_n<2>(codes, p0, p1, d_in, d_out, st);
}

// ---------------------------------------------------------------------------------------
// 16-bit storage of the factors for the memory-bound forward: one word per (group, column),
// fp16(alpha) | fp16(beta) << 16, round-to-nearest-even; and back to two fp32 matrices.
// ---------------------------------------------------------------------------------------
typedef uint32_t qz_u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void pack_factors_kernel(const f32x4* __restrict__ alpha,
                                                           const f32x4* __restrict__ beta,
                                                           qz_u32x4* __restrict__ out, size_t n4) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  const f32x4 a = alpha[i], b = beta[i];
  qz_u32x4 o;
#pragma unroll
  for (int c = 0; c < 4; ++c)
    o[c] = (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)a[c]) |
           ((uint32_t)__builtin_bit_cast(uint16_t, (_Float16)b[c]) << 16);
  out[i] = o;
}

__global__ __launch_bounds__(256) void unpack_factors_kernel(const qz_u32x4* __restrict__ in,
                                                             f32x4* __restrict__ alpha,
                                                             f32x4* __restrict__ beta, size_t n4) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  const qz_u32x4 w = in[i];
  f32x4 a, b;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    a[c] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[c] & 0xffffu));
    b[c] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[c] >> 16));
  }
  alpha[i] = a;
  beta[i] = b;
}

hipError_t launch_pack_factors(const float* alpha, const float* beta, void* fac16, size_t n, hipStream_t st) {
  const size_t n4 = n / 4;  // d_out is a multiple of 8
  pack_factors_kernel<<<(unsigned)((n4 + 255) / 256), 256, 0, st>>>(
      reinterpret_cast<const f32x4*>(alpha), reinterpret_cast<const f32x4*>(beta),
      static_cast<qz_u32x4*>(fac16), n4);
  return hipGetLastError();
}

hipError_t launch_unpack_factors(const void* fac16, float* alpha, float* beta, size_t n, hipStream_t st) {
  const size_t n4 = n / 4;
  unpack_factors_kernel<<<(unsigned)((n4 + 255) / 256), 256, 0, st>>>(
      static_cast<const qz_u32x4*>(fac16), reinterpret_cast<f32x4*>(alpha), reinterpret_cast<f32x4*>(beta), n4);
  return hipGetLastError();
}

}  // namespace qalora
