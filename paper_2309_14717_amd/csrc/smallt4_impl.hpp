// Adapter-free forward for one to four tokens: the decode step of post-merge inference.
//
//   y[t,j] = sum_l ( alpha[l,j] * sum_{i in group l} x[t,i] code[i,j]  +  beta[l,j] * sum_{i in l} x[t,i] )
//
// Same arithmetic as the sixteen-token kernel (Eq. 1 per group pulled out of the inner sum,
// exact bf16 operands: a code c is the bf16 number 128 + c), on a tile shape that fits four
// tokens: v_mfma_f32_4x4x4 (sixteen independent 4 x 4 blocks, K = 4) with the four tokens as
// the rows of every block and ONE output column per lane.  A lane then owns a whole column:
// its codes, alpha and beta come from its own loads (no exchange between lanes), the fp32
// update `acc += alpha d + (beta - 128 alpha) sum(x)` is four FMAs pairs per group instead of
// sixteen, and the group sums of x -- the same for every column -- are computed once per block
// when x is staged in LDS.  The vector work per weight byte is a little over half that of the
// sixteen-token kernel, which is what bounds a compute unit's streaming rate there.
//
// INT2 and INT3 take the same route with the code bits OR-ed higher into the bf16 mantissa, so
// that the bias of 128 weighs less against the codes: an INT2 code c becomes 128 + 32 c, an INT3
// code -- low two bits from plane 0, high bit from plane 1, both OR-ed into ONE operand --
// 128 + 16 c; the per-group update undoes the scale and the bias exactly (powers of two).
//
// Decomposition, partial sums, flags and their bounded waits are those of the sixteen-token
// kernel: slabs of 512 or 256 columns (eight or four 64-column wavefronts, the block's chunks
// split two or four ways over the remaining factor of wavefronts) x m parts of the 128-row
// chunks; parts 0 .. m-2 publish a partial and a flag, the last part adds them in part order.
#pragma once
#include "common.hpp"
#include "kernels.hpp"

#include <atomic>
#include <type_traits>

namespace qalora {

namespace {

constexpr int S4_WAVES = 16;
constexpr int S4_THREADS = 64 * S4_WAVES;
constexpr int S4_WCOLS = 64;                      // columns per wavefront: one per lane
constexpr int S4_XCHUNKS = 32;                    // chunks of x staged in LDS at a time
constexpr int S4_XROW = S4_XCHUNKS * 256 + 16;    // bytes per token row in LDS (+16: bank spread)
constexpr int S4_GS_BYTES = S4_XCHUNKS * 4 * 16;  // group sums per 4 tokens: [chunk][group in chunk][tokens] fp32
constexpr int s4_lds_bytes(int tg) { return tg * (4 * S4_XROW + S4_GS_BYTES); }  // tg: groups of four tokens
constexpr uint32_t S4_SPIN_LIMIT = 1u << 18;      // bounded wait: the kernel always terminates
constexpr uint32_t kS4Oob = 0xffff0000u;          // beyond every buffer: the range check returns zero
constexpr int S4_NT = 2;                          // cache policy "nontemporal": streamed once

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef short bf16x4_bits __attribute__((ext_vector_type(4)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t s4_rsrc(const void* base, size_t bytes) {
  const uint32_t n = bytes > 0xffffffffull ? 0xffffffffu : (uint32_t)bytes;
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)n, 0x00020000);
}

// LDS-only barrier: does not wait for the global loads that are in flight.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Words of one 128-row chunk of a column: plane 0 holds 8 (INT4) or 16 (INT2, low bits of INT3)
// rows per word, plane 1 (INT3 only) 32 rows per word.
template <int NBITS>
struct S4Fmt {
  static constexpr int W0 = NBITS == 4 ? 16 : 8;
  static constexpr int W1 = NBITS == 3 ? 4 : 0;
  // operand = 128 + kStep * code;  sum x code = d / kStep - (128 / kStep) sum x
  static constexpr float kInvStep = NBITS == 4 ? 1.0f : (NBITS == 2 ? 1.0f / 32.0f : 1.0f / 16.0f);
  static constexpr float kOff = NBITS == 4 ? 128.0f : (NBITS == 2 ? 4.0f : 8.0f);
  static constexpr uint32_t kMask0 = NBITS == 4 ? 0x000f000fu : (NBITS == 2 ? 0x00600060u : 0x00300030u);
  static constexpr int kTop0 = NBITS == 4 ? 0 : (NBITS == 2 ? 5 : 4);  // mantissa bit of the code's bit 0
};

// One 128-row chunk of a lane's column, as loaded: its code words and the factors of the
// chunk's 4 / SUB groups.
template <int NBITS, int SUB>
struct Chunk4 {
  uint32_t w[S4Fmt<NBITS>::W0];
  uint32_t h[S4Fmt<NBITS>::W1 > 0 ? S4Fmt<NBITS>::W1 : 1];
  uint32_t al[4 / SUB], be[4 / SUB];
};

// f(integral_constant<I>), ..., f(integral_constant<N - 1>): a loop whose index is a constant
// expression (instruction immediates need one)
template <int I, int N, typename Fn>
__device__ __forceinline__ void s4_static_for(Fn&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    s4_static_for<I + 1, N>(f);
  }
}

// word << sh for sh >= 0, word >> -sh otherwise (sh is a compile-time constant at every use)
__device__ __forceinline__ uint32_t shift_to(uint32_t word, int sh) { return sh >= 0 ? word << sh : word >> -sh; }

}  // namespace

// NBITS : code width (4, 3, 2)
// SUB   : 32-row steps per quantization group (group = 32 * SUB; 1, 2 or 4)
// KH    : ways a block splits its own chunks (2, 4: slab of 512, 256 columns)
// TG    : groups of four tokens (1, 2, 4): every group reuses the code operand a lane has built,
//         with its own rows of x and its own accumulators
// F16   : the factors of a (group, column) come as ONE word, fp16 alpha | fp16 beta << 16
// DEP   : the weight comes as the deployment stream (see s4_dep_units): per 64 columns and
//         128-row chunk one contiguous record of 16-byte units, a lane's four code units and its
//         factor unit(s), so that a wavefront streams one contiguous range with 16-byte loads
//         instead of twenty-four strided 4-byte ones (4-bit codes, fp32 factors, up to 4 tokens)
template <int NBITS, int SUB, int KH, int TG, bool F16, bool DEP = false>
__global__ __launch_bounds__(S4_THREADS) void smallt4_kernel(const SmallTArgs p) {
  using F = S4Fmt<NBITS>;
  static_assert(!DEP || (NBITS == 4 && !F16 && TG == 1), "the deployment stream holds 4-bit codes and fp32 factors");
  constexpr int NTOK = 4 * TG;             // token rows held in LDS
  constexpr int WPR = S4_WAVES / NTOK;     // wavefronts that share the staging of one token row
  constexpr int NBUF = TG == 1 ? 3 : 2;    // chunk buffers in rotation
  extern __shared__ __align__(16) unsigned char xs[];  // [NTOK][S4_XROW] x, then the group sums
  __shared__ int poison;
  constexpr int NG = 4 / SUB;              // groups per chunk
  constexpr int DEP_UNITS = s4_dep_units(SUB);             // 16-byte units per lane and chunk
  constexpr int NLOADS = DEP ? DEP_UNITS : F::W0 + F::W1 + (F16 ? 1 : 2) * NG;  // vector-memory loads of one chunk
  constexpr int NCG = S4_WAVES / KH;       // column groups (64 columns each)
  constexpr int SLAB_COLS = NCG * S4_WCOLS;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int cg = wave % NCG;
  const int kh = wave / NCG;               // which share of every staged piece's chunks
  const int L = p.d_in / p.group;
  const int C = p.d_in / 128;                   // chunks per slab
  const int S = ceil_div(p.d_out, SLAB_COLS);   // slabs
  const int m = gridDim.x / S;                  // parts per slab
  const int b = blockIdx.x, s = b / m, part = b - s * m;
  const int ca = (int)((long)C * part / m), ce = (int)((long)C * (part + 1) / m);

  const __amdgpu_buffer_rsrc_t rs_w =
      DEP ? s4_rsrc(p.stream, (size_t)ceil_div(p.d_out, 64) * (p.d_in / 128) * (DEP_UNITS * 1024))
          : s4_rsrc(p.plane0, (size_t)(p.d_in / 128) * F::W0 * p.d_out * 4);
  const __amdgpu_buffer_rsrc_t rs_h = s4_rsrc(p.plane1, (size_t)(p.d_in / 32) * p.d_out * 4);  // INT3 only
  const __amdgpu_buffer_rsrc_t rs_x = s4_rsrc(p.x, (size_t)p.T * p.d_in * 2);
  const __amdgpu_buffer_rsrc_t rs_al = s4_rsrc(F16 ? (const void*)p.fac16 : (const void*)p.alpha, (size_t)L * p.d_out * 4);
  const __amdgpu_buffer_rsrc_t rs_be = s4_rsrc(p.beta, F16 ? 0 : (size_t)L * p.d_out * 4);
  const uint32_t row_b = (uint32_t)p.d_out * 4u;  // one packed row, or one row of factors
  // Mask and bias live in registers (not literals) so that "(w >> k) & mask | bias" is one
  // shift and one v_and_or_b32: a VOP3 instruction cannot carry a 32-bit literal on this target.
  uint32_t kMask, kMaskH, kBias;
  asm volatile("s_mov_b32 %0, %1" : "=s"(kMask) : "n"(F::kMask0));
  asm volatile("s_mov_b32 %0, 0x00400040" : "=s"(kMaskH));  // INT3: the high bit, mantissa bit 6
  asm volatile("v_mov_b32 %0, 0x43004300" : "=v"(kBias));
  const f32x4 zero4 = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  // MFMA A operand: lane supplies four k values of token (lane & 3)
  // MFMA A operand.  The sixteen 4 x 4 blocks of an instruction all multiply the same tokens,
  // so only one block has to supply them: with the broadcast controls (CBSZ = 4, ABID = i) the
  // A rows held by the four lanes of block i serve every block.  Lane l therefore keeps the
  // 8-row slice l / 4 of token l % 4 -- ONE 16-byte LDS read per chunk and token group holds all
  // sixteen slices of the chunk across the wavefront, and slice i is used with ABID = i.
  // (Layout checked on the device: D[lane l][r] = sum_k A(lane 4 ABID + r)[k] B(lane l)[k].)
  const unsigned char* xs_lane = xs + (lane & 3) * S4_XROW + (lane >> 2) * 16;  // token group t: + 4 t rows
  const unsigned char* gs = xs + NTOK * S4_XROW;             // [chunk][group][NTOK] fp32

  const int j = s * SLAB_COLS + cg * S4_WCOLS + lane;  // this lane's column
  const bool col_ok = j < p.d_out;
  const uint32_t voff = col_ok ? (DEP ? (uint32_t)lane * 16u : (uint32_t)j * 4u) : kS4Oob;
  // deployment stream: the records of a chunk lie side by side for all column groups, so that
  // the wavefronts of the chip, which advance through the chunks together, sweep one contiguous
  // region at any moment (every memory channel busy) -- a wavefront's own records are one
  // chunk row of records apart
  const uint32_t dep_base = (uint32_t)(s * NCG + cg) * (uint32_t)(DEP_UNITS * 1024);
  const uint32_t dep_chunk = (uint32_t)ceil_div(p.d_out, 64) * (uint32_t)(DEP_UNITS * 1024);

  // Loads of chunk c, or -- past the end `lim` of the wavefront's share -- the same number of
  // loads aimed outside the buffers: they return zeros without touching memory, and the
  // count of loads in flight (which the waits rely on) stays the same.
  auto load_chunk = [&](Chunk4<NBITS, SUB>& ch, int c, int lim) {
    const uint32_t v = c < lim ? voff : kS4Oob;
    c = min(c, C - 1);
    if constexpr (DEP) {
      const uint32_t rec = dep_base + (uint32_t)c * dep_chunk;
      u32x4 q[DEP_UNITS];
#pragma unroll
      for (int i = 0; i < DEP_UNITS; ++i)
        q[i] = __builtin_amdgcn_raw_buffer_load_b128(rs_w, (int)v, (int)(rec + (uint32_t)i * 1024u), S4_NT);
#pragma unroll
      for (int i = 0; i < 16; ++i) ch.w[i] = q[i >> 2][i & 3];
      if constexpr (SUB == 1) {  // alpha of the four groups, then beta
#pragma unroll
        for (int u = 0; u < 4; ++u) ch.al[u] = q[4][u], ch.be[u] = q[5][u];
      } else if constexpr (SUB == 2) {  // alpha0, alpha1, beta0, beta1
        ch.al[0] = q[4][0], ch.al[1] = q[4][1], ch.be[0] = q[4][2], ch.be[1] = q[4][3];
      } else {  // alpha, beta, -, -
        ch.al[0] = q[4][0], ch.be[0] = q[4][1];
      }
      return;
    }
#pragma unroll
    for (int i = 0; i < F::W0; ++i)
      ch.w[i] = __builtin_amdgcn_raw_buffer_load_b32(rs_w, (int)v, (int)((uint32_t)(F::W0 * c + i) * row_b), S4_NT);
#pragma unroll
    for (int i = 0; i < F::W1; ++i)
      ch.h[i] = __builtin_amdgcn_raw_buffer_load_b32(rs_h, (int)v, (int)((uint32_t)(F::W1 * c + i) * row_b), S4_NT);
#pragma unroll
    for (int u = 0; u < NG; ++u) {
      const uint32_t so = (uint32_t)(NG * c + u) * row_b;
      ch.al[u] = __builtin_amdgcn_raw_buffer_load_b32(rs_al, (int)v, (int)so, S4_NT);
      if constexpr (!F16) ch.be[u] = __builtin_amdgcn_raw_buffer_load_b32(rs_be, (int)v, (int)so, S4_NT);
    }
  };

  f32x4 acc[TG];  // rows = tokens 4 t .. 4 t + 3 of this lane's column
#pragma unroll
  for (int t = 0; t < TG; ++t) acc[t] = zero4;

  // The bf16 pair (rows 2i, 2i+1 of 8-row slice k of 32-row step st) of a chunk: code bits
  // OR-ed into the mantissa of 128.0.  All indices are compile-time constants at every use.
  auto pair_bits = [&](const Chunk4<NBITS, SUB>& ch, int st, int k, int i) -> uint32_t {
    if constexpr (NBITS == 4) {
      return ((ch.w[4 * st + k] >> (4 * i)) & kMask) | kBias;
    } else {
      const int m = 4 * (k & 1) + i;  // pair inside the 16-row word of plane 0
      uint32_t v = (shift_to(ch.w[2 * st + (k >> 1)], F::kTop0 - 2 * m) & kMask) | kBias;
      if constexpr (NBITS == 3) v = (shift_to(ch.h[st], 6 - (4 * k + i)) & kMaskH) | v;
      return v;
    }
  };

  // xrel: chunk index relative to the staged piece
  auto compute_chunk = [&](const Chunk4<NBITS, SUB>& ch, int xrel) {
    u32x4 xa[TG];  // the chunk's x: slice lane / 4 of token lane % 4 (+ 4 t)
#pragma unroll
    for (int t = 0; t < TG; ++t)
      xa[t] = *reinterpret_cast<const u32x4*>(xs_lane + 4 * t * S4_XROW + xrel * 256);
    s4_static_for<0, NG>([&](auto u_c) {
      constexpr int u = decltype(u_c)::value;
      f32x4 d[TG];
#pragma unroll
      for (int t = 0; t < TG; ++t) d[t] = zero4;
      s4_static_for<0, 4 * SUB>([&](auto i_c) {
        constexpr int ks = u * 4 * SUB + decltype(i_c)::value;  // 8-row slice of the chunk
        constexpr int st = ks / 4, k = ks % 4;                  // 32-row step, slice inside it
        const u32x2 b01 = {pair_bits(ch, st, k, 0), pair_bits(ch, st, k, 1)};
        const u32x2 b23 = {pair_bits(ch, st, k, 2), pair_bits(ch, st, k, 3)};
#pragma unroll
        for (int t = 0; t < TG; ++t) {
          d[t] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(bf16x4_bits, u32x2{xa[t].x, xa[t].y}),
                                                        __builtin_bit_cast(bf16x4_bits, b01), d[t], 4, ks, 0);
          d[t] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(bf16x4_bits, u32x2{xa[t].z, xa[t].w}),
                                                        __builtin_bit_cast(bf16x4_bits, b23), d[t], 4, ks, 0);
        }
      });
      // sum x code = d * kInvStep - kOff * sum x  (the operand was 128 + code / kInvStep)
      float a0, b0;
      if constexpr (F16) {
        a0 = (float)__builtin_bit_cast(_Float16, (uint16_t)(ch.al[u] & 0xffffu));
        b0 = (float)__builtin_bit_cast(_Float16, (uint16_t)(ch.al[u] >> 16));
      } else {
        a0 = __uint_as_float(ch.al[u]);
        b0 = __uint_as_float(ch.be[u]);
      }
      const float bp = __builtin_fmaf(-F::kOff, a0, b0);
      const float al = F::kInvStep * a0;
#pragma unroll
      for (int t = 0; t < TG; ++t) {
        const f32x4 sx = *reinterpret_cast<const f32x4*>(gs + ((xrel * NG + u) * TG + t) * 16);
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[t][r] = __builtin_fmaf(al, d[t][r], __builtin_fmaf(bp, sx[r], acc[t][r]));
      }
    });
  };

  for (int pa = ca; pa < ce; pa += S4_XCHUNKS) {  // pieces of at most S4_XCHUNKS chunks
    const int pe = min(ce, pa + S4_XCHUNKS);
    const int np = (pe - pa) * 16;  // 16-byte pieces per token row
    if (pa != ca) lds_barrier();    // every wavefront is done reading the previous piece
    // x of this piece: the WPR wavefronts of a token row copy its 1 KB runs (four chunks each)
    // straight into LDS (no registers), turn and turn about.  The copies are issued BEFORE the
    // weight prefetch, so waiting for them leaves it in flight.
    {
      const int row = wave % NTOK, q0 = wave / NTOK;
      if (row < p.T) {
        const uint32_t xoff = ((uint32_t)row * p.d_in + (uint32_t)pa * 128) * 2u + lane * 16u;
#pragma unroll
        for (int k = 0; k < S4_XCHUNKS / 4 / WPR; ++k) {
          const int run = q0 + WPR * k;
          if (lane + 64 * run < np)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rs_x, (__attribute__((address_space(3))) void*)(xs + row * S4_XROW + run * 1024), 16,
                (int)xoff, run * 1024, 0, 0);
        }
      }
    }
    // this wavefront's share of the piece: a contiguous KH-th of its chunks
    const int wa = pa + (int)((long)(pe - pa) * kh / KH), we = pa + (int)((long)(pe - pa) * (kh + 1) / KH);
    Chunk4<NBITS, SUB> b0, b1, b2;  // b2 unused with two buffers
    load_chunk(b0, wa, we);
    if constexpr (NBUF == 3) load_chunk(b1, wa + 1, we);
    __builtin_amdgcn_sched_barrier(0);
    if (pa == ca) {
      // first piece: with the loads above already in flight, clear what must start at zero --
      // the token rows that do not exist (they stay zero for the whole kernel)
      if (tid == 0) poison = 0;
      const int row = wave % NTOK, q0 = wave / NTOK;
      if (row >= p.T) {
        for (int o = lane + 64 * q0; o < S4_XROW / 16; o += 64 * WPR)
          *reinterpret_cast<u32x4*>(xs + row * S4_XROW + o * 16) = u32x4{0, 0, 0, 0};
      }
    }
    // (NBUF - 1) * NLOADS weight loads were issued after the copies: once at most that many
    // are outstanding, the copies have landed
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NBUF - 1) * NLOADS) : "memory");
    lds_barrier();
    // group sums of x for the piece, one (group, token) pair per thread, element order
    for (int idx = tid; idx < (pe - pa) * NG * NTOK; idx += S4_THREADS) {
      const int grp = idx / NTOK, tok = idx % NTOK;
      const unsigned char* src = xs + tok * S4_XROW + grp * (64 * SUB);
      float sum = 0.0f;
#pragma unroll
      for (int q = 0; q < 4 * SUB; ++q) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(src + 16 * q);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          sum += __uint_as_float(v[e] << 16);
          sum += __uint_as_float(v[e] & 0xffff0000u);
        }
      }
      *reinterpret_cast<float*>(xs + NTOK * S4_XROW + grp * (4 * NTOK) + tok * 4) = sum;
    }
    lds_barrier();

    int c = wa;
    if constexpr (NBUF == 3) {
#pragma nounroll
      for (; c + 2 < we; c += 3) {
        load_chunk(b2, c + 2, we);
        __builtin_amdgcn_sched_barrier(0);
        compute_chunk(b0, c - pa);
        __builtin_amdgcn_sched_barrier(0);
        load_chunk(b0, c + 3, we);
        __builtin_amdgcn_sched_barrier(0);
        compute_chunk(b1, c + 1 - pa);
        __builtin_amdgcn_sched_barrier(0);
        load_chunk(b1, c + 4, we);
        __builtin_amdgcn_sched_barrier(0);
        compute_chunk(b2, c + 2 - pa);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (c < we) compute_chunk(b0, c - pa);
      if (c + 1 < we) compute_chunk(b1, c + 1 - pa);
    } else {
#pragma nounroll
      for (; c + 1 < we; c += 2) {
        load_chunk(b1, c + 1, we);
        __builtin_amdgcn_sched_barrier(0);
        compute_chunk(b0, c - pa);
        __builtin_amdgcn_sched_barrier(0);
        load_chunk(b0, c + 2, we);
        __builtin_amdgcn_sched_barrier(0);
        compute_chunk(b1, c + 1 - pa);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (c < we) compute_chunk(b0, c - pa);
    }
  }

  // ---- the KH shares of the block meet in LDS (fixed order: share 0 + 1 + 2 + 3) ----------
  if constexpr (KH > 1) {
    float* red = reinterpret_cast<float*>(xs);  // [KH - 1][NCG][NTOK rows][64 lanes]
    lds_barrier();                              // x is no longer needed
    if (kh > 0) {
#pragma unroll
      for (int t = 0; t < TG; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[(((kh - 1) * NCG + cg) * NTOK + 4 * t + r) * 64 + lane] = acc[t][r];
    }
    lds_barrier();
    if (kh == 0) {
#pragma unroll
      for (int h = 1; h < KH; ++h)
#pragma unroll
        for (int t = 0; t < TG; ++t)
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[t][r] += red[(((h - 1) * NCG + cg) * NTOK + 4 * t + r) * 64 + lane];
    }
  }

  // ---- hand over, or finish the slab (wavefronts of share 0 hold the sums) ------------------
  // The block's sums are first laid out in LDS as a [token][column] tile, so that they travel
  // as 16-byte accesses, one (token, four columns) item per thread: a partial leaves the block
  // in a quarter of the memory instructions the one-column-per-lane registers would need, and
  // the cost of the hand-over goes with the number of these cache-bypassing accesses.
  // They carry the cache policy of a device-scope atomic (coherent at the level all compute
  // units share), so no cache write-back or invalidate is needed.
  float* tile = reinterpret_cast<float*>(xs);  // [NTOK][SLAB_COLS]
  constexpr int kDeviceCoherent = 16;          // "sc1"
  constexpr int C4 = SLAB_COLS / 4;            // items per token row
  constexpr int ITEMS_PER_THREAD = (NTOK * C4 + S4_THREADS - 1) / S4_THREADS;
  static_assert(NTOK * SLAB_COLS <= ST_PARTIAL_FLOATS, "a partial holds the whole tile");
  lds_barrier();  // x and the meeting area of the shares are no longer needed
  if (kh == 0) {
#pragma unroll
    for (int t = 0; t < TG; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) tile[(4 * t + r) * SLAB_COLS + cg * S4_WCOLS + lane] = acc[t][r];
  }
  lds_barrier();
  const int items = p.T * C4;
  const __amdgpu_buffer_rsrc_t rs_p = s4_rsrc(p.partial, (size_t)gridDim.x * ST_PARTIAL_FLOATS * 4);
  if (part < m - 1) {
#pragma unroll
    for (int k = 0; k < ITEMS_PER_THREAD; ++k) {
      const int it = tid + k * S4_THREADS;
      if (it < items) {
        const int r = it / C4, c4 = it - r * C4;
        const u32x4 v = *reinterpret_cast<const u32x4*>(tile + r * SLAB_COLS + 4 * c4);
        __builtin_amdgcn_raw_buffer_store_b128(v, rs_p, (r * SLAB_COLS + 4 * c4) * 4,
                                               (int)((uint32_t)b * (ST_PARTIAL_FLOATS * 4u)), kDeviceCoherent);
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // every store of this wavefront has landed
    __syncthreads();
    if (tid == 0)
      __hip_atomic_store(p.flags + b, p.nonce, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  } else {
    f32x4 tot[ITEMS_PER_THREAD];
#pragma unroll
    for (int k = 0; k < ITEMS_PER_THREAD; ++k) tot[k] = zero4;
    if (m > 1) {
      const int bf = b - (m - 1);  // block of part 0 of this slab
      // one thread per flag, all polling at once
      for (int i = tid; i < m - 1; i += S4_THREADS) {
        uint32_t spins = 0;
        bool timed_out = false;
        while (__hip_atomic_load(p.flags + bf + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != p.nonce) {
          if (++spins > S4_SPIN_LIMIT) {
            poison = 1;
            timed_out = true;
            break;
          }
          __builtin_amdgcn_s_sleep(8);
        }
        // Consumed: clear it, so that a replay of this very launch (a captured graph repeats
        // the nonce) waits for its own producers instead of seeing this launch's flags.  A flag
        // that never came is left alone and reported: its producer may still write it, and a
        // workspace in that state must be cleared by the caller before it is used again.
        if (!timed_out)
          __hip_atomic_store(p.flags + bf + i, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else
          __hip_atomic_store(p.status, p.nonce | 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      __syncthreads();
      // partials in part order, PB blocks' loads in flight at a time
      constexpr int PB = 8 / ITEMS_PER_THREAD;
#pragma unroll
      for (int k = 0; k < ITEMS_PER_THREAD; ++k) {
        const int it = tid + k * S4_THREADS;
        if (it < items) {
          const int r = it / C4, c4 = it - r * C4;
          for (int i0 = 0; i0 < m - 1; i0 += PB) {
            u32x4 v[PB];
#pragma unroll
            for (int i = 0; i < PB; ++i) {
              v[i] = u32x4{0, 0, 0, 0};
              if (i0 + i < m - 1)
                v[i] = __builtin_amdgcn_raw_buffer_load_b128(
                    rs_p, (r * SLAB_COLS + 4 * c4) * 4,
                    (int)((uint32_t)(bf + i0 + i) * (ST_PARTIAL_FLOATS * 4u)), kDeviceCoherent);
            }
#pragma unroll
            for (int i = 0; i < PB; ++i) tot[k] += __builtin_bit_cast(f32x4, v[i]);
          }
        }
      }
    }
    const bool bad = (m > 1) && poison != 0;
#pragma unroll
    for (int k = 0; k < ITEMS_PER_THREAD; ++k) {
      const int it = tid + k * S4_THREADS;
      if (it < items) {
        const int r = it / C4, c4 = it - r * C4;
        const int jj = s * SLAB_COLS + 4 * c4;  // d_out is a multiple of 8: four columns are all in or all out
        if (jj < p.d_out) {
          f32x4 v = tot[k] + *reinterpret_cast<const f32x4*>(tile + r * SLAB_COLS + 4 * c4);
          if (bad) v = f32x4{__builtin_nanf(""), __builtin_nanf(""), __builtin_nanf(""), __builtin_nanf("")};  // a wait ran out: make it loud
          const size_t o = (size_t)r * p.d_out + jj;
          if (p.out_bf16)
            *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(p.out) + o) =
                u32x2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
          else
            *reinterpret_cast<f32x4*>(static_cast<float*>(p.out) + o) = v;
        }
      }
    }
  }
}

template <int NBITS, int SUB, int KH, int TG, bool F16, bool DEP = false>
static hipError_t launch_sub4(const SmallTArgs& a, int grid, hipStream_t st) {
  static std::atomic<uint64_t> granted{0};  // per instantiation
  constexpr int lds = s4_lds_bytes(TG);
  if (hipError_t e = grant_dynamic_lds(reinterpret_cast<const void*>(smallt4_kernel<NBITS, SUB, KH, TG, F16, DEP>), lds, granted);
      e != hipSuccess)
    return e;
  smallt4_kernel<NBITS, SUB, KH, TG, F16, DEP><<<grid, S4_THREADS, lds, st>>>(a);
  return hipGetLastError();
}

// the deployment-stream form: 4-bit codes, fp32 factors, up to four tokens
template <int SUB>
static hipError_t launch_dep4(const SmallTArgs& a, const SmallTPlan& pl, hipStream_t st) {
  if (pl.halves == 4) return launch_sub4<4, SUB, 4, 1, false, true>(a, pl.blocks, st);
  if (pl.halves == 2) return launch_sub4<4, SUB, 2, 1, false, true>(a, pl.blocks, st);
  return hipErrorInvalidValue;
}

template <int NBITS, int SUB, int TG, bool F16>
static hipError_t launch_halves4(const SmallTArgs& a, const SmallTPlan& pl, hipStream_t st) {
  if (pl.halves == 4) return launch_sub4<NBITS, SUB, 4, TG, F16>(a, pl.blocks, st);
  if (pl.halves == 2) return launch_sub4<NBITS, SUB, 2, TG, F16>(a, pl.blocks, st);
  return hipErrorInvalidValue;
}

template <int NBITS, int TG, bool F16>
static hipError_t launch_group4(const SmallTArgs& a, const SmallTPlan& pl, hipStream_t st) {
  const int sub = a.group / 32;
  if (sub == 1) return launch_halves4<NBITS, 1, TG, F16>(a, pl, st);
  if (sub == 2) return launch_halves4<NBITS, 2, TG, F16>(a, pl, st);
  if (sub == 4) return launch_halves4<NBITS, 4, TG, F16>(a, pl, st);
  return hipErrorInvalidValue;
}

// INT4 beyond four tokens belongs to the sixteen-token kernel; INT3 and INT2 stay here.
template <int NBITS, bool F16>
static hipError_t launch_tokens4(const SmallTArgs& a, const SmallTPlan& pl, hipStream_t st) {
  if (a.T <= 4) return launch_group4<NBITS, 1, F16>(a, pl, st);
  if constexpr (NBITS != 4) {
    if (a.T <= 8) return launch_group4<NBITS, 2, F16>(a, pl, st);
    return launch_group4<NBITS, 4, F16>(a, pl, st);
  }
  return hipErrorInvalidValue;
}

// F16: the factors come as one 32-bit word per (group, column), fp16 alpha | fp16 beta << 16.
template <bool F16>
static hipError_t launch_smallt4_impl(const SmallTArgs& a, hipStream_t st) {
  if (a.T < 1 || a.T > 16 || a.d_in % 128 != 0) return hipErrorInvalidValue;
  const SmallTPlan pl = smallt4_plan(a.d_in, a.d_out, a.T);
  if (a.bits == 4) return launch_tokens4<4, F16>(a, pl, st);
  if (a.bits == 3) return launch_tokens4<3, F16>(a, pl, st);
  if (a.bits == 2) return launch_tokens4<2, F16>(a, pl, st);
  return hipErrorInvalidValue;
}

}  // namespace qalora
