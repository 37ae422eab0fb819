// Shared device-side helpers for the gfx950 QA-LoRA kernels: vector types, bf16
// conversion, and the private bit-packed code format.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace qalora {

// Dynamic LDS beyond 48 KB has to be granted to a kernel once per device.  `granted` (one
// per kernel instantiation) remembers the devices that have it, so that the library works on
// whichever device is current and from any thread.
inline hipError_t grant_dynamic_lds(const void* kernel, int bytes, std::atomic<uint64_t>& granted) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = 1ull << (dev & 63);
  if (granted.load(std::memory_order_acquire) & bit) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) granted.fetch_or(bit, std::memory_order_release);
  return e;
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;
// bf16 elements per LDS row of a 64-wide K tile: 64 data + 8 pad (144 bytes), which keeps
// 128-bit reads of 16 consecutive rows and 128-bit writes of 8 chunks x 2 rows conflict free.
constexpr int LDS_ROW_72 = 72;

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// Round-to-nearest-even fp32 -> bf16 pair, packed lo | hi << 16 (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 b = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, b);
}
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  return (uint16_t)(pack_bf16x2(f, 0.0f) & 0xffffu);
}
// hi + lo split of an fp32 value into two bf16 (v ~= hi + lo to about 2^-17 relative).
__device__ __forceinline__ void split_bf16(float v, uint16_t& hi, uint16_t& lo) {
  hi = f32_to_bf16_bits(v);
  lo = f32_to_bf16_bits(v - bf16_bits_to_f32(hi));
}

__host__ __device__ constexpr int ceil_div(int a, int b) { return (a + b - 1) / b; }
__host__ __device__ constexpr int round_up(int a, int b) { return ceil_div(a, b) * b; }

// ---------------------------------------------------------------------------
// Private packed-code format.
//
// Codes of one column are packed down the input rows into 32-bit words; a word holds
// the N-bit codes of RB consecutive rows of one column, and words are stored row-major
// [d_in / RB][d_out] ("plane").  Inside a word, row p sits at bit
//     N * (p >> 1) + 16 * (p & 1)
// i.e. even rows fill the low half-word and odd rows the high half-word, so that
// (word >> N*m) & (mask | mask << 16) yields rows 2m and 2m+1 as a pair of 16-bit
// lanes -- the shape a packed-bf16 matrix operand wants.
//   N = 4: one plane, RB = 8.      N = 2: one plane, RB = 16.
//   N = 3: plane 0 holds the low two bits of every code in the N = 2 layout,
//          plane 1 (right behind it) the high bit, RB = 32, row p at bit (p>>1) + 16*(p&1).
// ---------------------------------------------------------------------------
template <int NBITS>
struct PackFmt;
template <>
struct PackFmt<4> {
  static constexpr int kRowsPerWord0 = 8;
  static constexpr int kRowAlign = 8;  // d_in must be a multiple of this
};
template <>
struct PackFmt<2> {
  static constexpr int kRowsPerWord0 = 16;
  static constexpr int kRowAlign = 16;
};
template <>
struct PackFmt<3> {
  static constexpr int kRowsPerWord0 = 16;
  static constexpr int kRowAlign = 32;
};

__host__ __device__ inline size_t plane0_words(int bits, int d_in, int d_out) {
  const int rb = (bits == 4) ? 8 : 16;
  return (size_t)(d_in / rb) * (size_t)d_out;
}
__host__ __device__ inline size_t plane1_words(int bits, int d_in, int d_out) {
  return bits == 3 ? (size_t)(d_in / 32) * (size_t)d_out : 0;
}

// Load the column words a thread needs to rebuild the 8x8 patch of codes whose top-left
// corner is (i0, j0), i0 and j0 multiples of 8: plane-0 words of columns j0..j0+7 into
// (a0, a1), plane-1 words (N = 3 only) into (b0, b1).
template <int NBITS>
__device__ __forceinline__ void load_patch_words(const uint32_t* __restrict__ plane0,
                                                 const uint32_t* __restrict__ plane1, int d_out,
                                                 int i0, int j0, uint4& a0, uint4& a1, uint4& b0,
                                                 uint4& b1) {
  constexpr int RB0 = PackFmt<NBITS>::kRowsPerWord0;
  const uint4* p = reinterpret_cast<const uint4*>(plane0 + (size_t)(i0 / RB0) * d_out + j0);
  a0 = p[0];
  a1 = p[1];
  if constexpr (NBITS == 3) {
    const uint4* q = reinterpret_cast<const uint4*>(plane1 + (size_t)(i0 / 32) * d_out + j0);
    b0 = q[0];
    b1 = q[1];
  }
}

// Code of row p (0..7) of the patch from the words of one column.  `sh0` / `sh1` are the
// run-time pre-shifts that select the patch's eight rows inside a wider word.
template <int NBITS>
__device__ __forceinline__ int patch_preshift0(int i0) {
  if constexpr (NBITS == 4) return 0;
  return (i0 & 8) ? 8 : 0;  // rows 8..15 of a 16-row word start 4 pairs (8 bits) up
}
__device__ __forceinline__ int patch_preshift1(int i0) { return ((i0 >> 3) & 3) * 4; }

template <int NBITS>
__device__ __forceinline__ uint32_t patch_code(uint32_t w0s, uint32_t w1s, int p) {
  // w0s, w1s: words already shifted right by the pre-shifts above; p is a constant.
  if constexpr (NBITS == 4) {
    return (w0s >> (4 * (p >> 1) + 16 * (p & 1))) & 15u;
  } else if constexpr (NBITS == 2) {
    return (w0s >> (2 * (p >> 1) + 16 * (p & 1))) & 3u;
  } else {
    const uint32_t lo = (w0s >> (2 * (p >> 1) + 16 * (p & 1))) & 3u;
    const uint32_t hi = (w1s >> ((p >> 1) + 16 * (p & 1))) & 1u;
    return lo | (hi << 2);
  }
}

// The codes of rows 2m and 2m+1 (m = 0..3) of the patch, for one column, less the mid code
// 2^(N-1), as an exact pair of fp16 integers (low half = even row).  0x6400 is fp16 1024.0, whose
// mantissa unit is 1, so (0x6400 | c) - (1024 + mid) == c - mid for c < 1024 without any
// int->float conversion.  The caller adds mid * alpha to beta (code_center<NBITS>()).
// `mask` and `magic` are the constants (2^LB - 1) * 0x00010001 and 0x64006400 handed in by the
// caller: a kernel that keeps them in registers gets "(w >> k) & mask | magic" as one shift and
// one v_and_or_b32 (a VOP3 instruction cannot carry a 32-bit literal on gfx9-class targets).
template <int NBITS>
__device__ __forceinline__ f16x2 patch_code_pair_f16(uint32_t w0s, uint32_t w1s, int m,
                                                     uint32_t mask, uint32_t magic) {
  constexpr int LB = (NBITS == 3) ? 2 : NBITS;  // code bits held in plane 0
  uint32_t u;
  if constexpr (NBITS == 3) {
    u = ((w0s >> (LB * m)) & mask) | (((w1s >> m) & 0x00010001u) << 2);
    u |= magic;
  } else {
    u = ((w0s >> (LB * m)) & mask) | magic;
  }
  constexpr float kOff = 1024.0f + float(1 << (NBITS - 1));
  const f16x2 off = {(_Float16)kOff, (_Float16)kOff};
  return __builtin_bit_cast(f16x2, u) - off;
}
template <int NBITS>
__host__ __device__ constexpr float code_center() {
  return float(1 << (NBITS - 1));
}
template <int NBITS>
__host__ __device__ constexpr uint32_t patch_code_mask() {
  return ((1u << ((NBITS == 3) ? 2 : NBITS)) - 1u) * 0x00010001u;
}

}  // namespace qalora
