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
// Decomposition, partial sums, flags and their bounded waits are those of the sixteen-token
// kernel: slabs of 1024, 512 or 256 columns (sixteen, eight or four 64-column wavefronts, the
// block's chunks split over the remaining factor of wavefronts) x m parts of the 128-row
// chunks; parts 0 .. m-2 publish a partial and a flag, the last part adds them in part order.
#include "common.hpp"
#include "kernels.hpp"

#include <atomic>

namespace qalora {

namespace {

constexpr int S4_WAVES = 16;
constexpr int S4_THREADS = 64 * S4_WAVES;
constexpr int S4_WCOLS = 64;                      // columns per wavefront: one per lane
constexpr int S4_XCHUNKS = 32;                    // chunks of x staged in LDS at a time
constexpr int S4_XROW = S4_XCHUNKS * 256 + 16;    // bytes per token row in LDS (+16: bank spread)
constexpr int S4_GS_BYTES = S4_XCHUNKS * 4 * 16;  // group sums: [chunk][group in chunk][4 tokens] fp32
constexpr int S4_LDS = 4 * S4_XROW + S4_GS_BYTES;
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

// One 128-row chunk of a lane's column, as loaded: sixteen code words (eight rows each) and the
// factors of the chunk's 4 / SUB groups.
template <int SUB>
struct Chunk4 {
  uint32_t w[16];
  uint32_t al[4 / SUB], be[4 / SUB];
};

}  // namespace

// SUB : 32-row steps per quantization group (group = 32 * SUB; 1, 2 or 4)
// KH  : ways a block splits its own chunks (1, 2, 4: slab of 1024, 512, 256 columns)
template <int SUB, int KH>
__global__ __launch_bounds__(S4_THREADS) void smallt4_kernel(const SmallTArgs p) {
  extern __shared__ __align__(16) unsigned char xs[];  // [4][S4_XROW] x, then the group sums
  __shared__ int poison;
  constexpr int NG = 4 / SUB;              // groups per chunk
  constexpr int NLOADS = 16 + 2 * NG;      // vector-memory loads of one chunk
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

  const __amdgpu_buffer_rsrc_t rs_w = s4_rsrc(p.plane0, (size_t)(p.d_in / 8) * p.d_out * 4);
  const __amdgpu_buffer_rsrc_t rs_x = s4_rsrc(p.x, (size_t)p.T * p.d_in * 2);
  const __amdgpu_buffer_rsrc_t rs_al = s4_rsrc(p.alpha, (size_t)L * p.d_out * 4);
  const __amdgpu_buffer_rsrc_t rs_be = s4_rsrc(p.beta, (size_t)L * p.d_out * 4);
  const uint32_t row_b = (uint32_t)p.d_out * 4u;  // one packed row, or one row of factors
  // Mask and bias live in registers (not literals) so that "(w >> k) & mask | bias" is one
  // shift and one v_and_or_b32: a VOP3 instruction cannot carry a 32-bit literal on this target.
  uint32_t kMask, kBias;
  asm volatile("s_mov_b32 %0, 0x000f000f" : "=s"(kMask));
  asm volatile("v_mov_b32 %0, 0x43004300" : "=v"(kBias));
  const f32x4 zero4 = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  // MFMA A operand: lane supplies four k values of token (lane & 3)
  const unsigned char* xs_lane = xs + (lane & 3) * S4_XROW;
  const unsigned char* gs = xs + 4 * S4_XROW;

  const int j = s * SLAB_COLS + cg * S4_WCOLS + lane;  // this lane's column
  const bool col_ok = j < p.d_out;
  const uint32_t voff = col_ok ? (uint32_t)j * 4u : kS4Oob;

  // Loads of chunk c, or -- past the end `lim` of the wavefront's share -- the same number of
  // loads aimed outside the buffers: they return zeros without touching memory, and the
  // count of loads in flight (which the waits rely on) stays the same.
  auto load_chunk = [&](Chunk4<SUB>& ch, int c, int lim) {
    const uint32_t v = c < lim ? voff : kS4Oob;
    c = min(c, C - 1);
#pragma unroll
    for (int i = 0; i < 16; ++i)
      ch.w[i] = __builtin_amdgcn_raw_buffer_load_b32(rs_w, (int)v, (int)((uint32_t)(16 * c + i) * row_b), S4_NT);
#pragma unroll
    for (int u = 0; u < NG; ++u) {
      const uint32_t so = (uint32_t)(NG * c + u) * row_b;
      ch.al[u] = __builtin_amdgcn_raw_buffer_load_b32(rs_al, (int)v, (int)so, S4_NT);
      ch.be[u] = __builtin_amdgcn_raw_buffer_load_b32(rs_be, (int)v, (int)so, S4_NT);
    }
  };

  f32x4 acc = zero4;  // rows = tokens 0..3 of this lane's column

  // xrel: chunk index relative to the staged piece
  auto compute_chunk = [&](const Chunk4<SUB>& ch, int xrel) {
#pragma unroll
    for (int u = 0; u < NG; ++u) {
      f32x4 d = zero4;
#pragma unroll
      for (int ii = 0; ii < 4 * SUB; ++ii) {
        const int wi = u * 4 * SUB + ii;  // word of the chunk: rows 8 wi .. 8 wi + 7
        const u32x4 xa = *reinterpret_cast<const u32x4*>(xs_lane + xrel * 256 + wi * 16);
        const uint32_t w = ch.w[wi];
        const u32x2 b01 = {(w & kMask) | kBias, ((w >> 4) & kMask) | kBias};
        const u32x2 b23 = {((w >> 8) & kMask) | kBias, ((w >> 12) & kMask) | kBias};
        d = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(bf16x4_bits, u32x2{xa.x, xa.y}),
                                                   __builtin_bit_cast(bf16x4_bits, b01), d, 0, 0, 0);
        d = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(bf16x4_bits, u32x2{xa.z, xa.w}),
                                                   __builtin_bit_cast(bf16x4_bits, b23), d, 0, 0, 0);
      }
      const float al = __uint_as_float(ch.al[u]);
      const float bp = __builtin_fmaf(-128.0f, al, __uint_as_float(ch.be[u]));  // codes carry +128
      const f32x4 sx = *reinterpret_cast<const f32x4*>(gs + (xrel * NG + u) * 16);
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[r] = __builtin_fmaf(al, d[r], __builtin_fmaf(bp, sx[r], acc[r]));
    }
  };

  for (int pa = ca; pa < ce; pa += S4_XCHUNKS) {  // pieces of at most S4_XCHUNKS chunks
    const int pe = min(ce, pa + S4_XCHUNKS);
    const int np = (pe - pa) * 16;  // 16-byte pieces per token row
    if (pa != ca) lds_barrier();    // every wavefront is done reading the previous piece
    // x of this piece: wavefront w copies every fourth 1 KB run of token row w & 3 straight into
    // LDS (no registers).  The copies are issued BEFORE the weight prefetch, so waiting for them
    // leaves it in flight.
    {
      const int row = wave & 3, q0 = wave >> 2;
      if (row < p.T) {
        const uint32_t xoff = ((uint32_t)row * p.d_in + (uint32_t)pa * 128) * 2u + lane * 16u;
#pragma unroll
        for (int k = 0; k < S4_XCHUNKS / 16; ++k) {
          const int run = q0 + 4 * k;  // 1 KB = four chunks of the row
          if (lane + 64 * run < np)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rs_x, (__attribute__((address_space(3))) void*)(xs + row * S4_XROW + run * 1024), 16,
                (int)xoff, run * 1024, 0, 0);
        }
      }
    }
    // this wavefront's share of the piece: a contiguous KH-th of its chunks
    const int wa = pa + (int)((long)(pe - pa) * kh / KH), we = pa + (int)((long)(pe - pa) * (kh + 1) / KH);
    Chunk4<SUB> b0, b1, b2;
    load_chunk(b0, wa, we);
    load_chunk(b1, wa + 1, we);
    __builtin_amdgcn_sched_barrier(0);
    if (pa == ca) {
      // first piece: with the loads above already in flight, clear what must start at zero --
      // the token rows that do not exist (they stay zero for the whole kernel)
      if (tid == 0) poison = 0;
      const int row = wave & 3, q0 = wave >> 2;
      if (row >= p.T) {
        for (int o = lane + 64 * q0; o < S4_XROW / 16; o += 256)
          *reinterpret_cast<u32x4*>(xs + row * S4_XROW + o * 16) = u32x4{0, 0, 0, 0};
      }
    }
    // 2 * NLOADS weight loads were issued after the copies: once at most that many are
    // outstanding, the copies have landed
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * NLOADS) : "memory");
    lds_barrier();
    // group sums of x for the piece, one (group, token) pair per thread, element order
    for (int idx = tid; idx < (pe - pa) * NG * 4; idx += S4_THREADS) {
      const int grp = idx >> 2, tok = idx & 3;
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
      *reinterpret_cast<float*>(xs + 4 * S4_XROW + grp * 16 + tok * 4) = sum;
    }
    lds_barrier();

    int c = wa;
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
  }

  // ---- the KH shares of the block meet in LDS (fixed order: share 0 + 1 + 2 + 3) ----------
  if constexpr (KH > 1) {
    float* red = reinterpret_cast<float*>(xs);  // [KH - 1][NCG][4 rows][64 lanes]
    lds_barrier();                              // x is no longer needed
    if (kh > 0) {
#pragma unroll
      for (int r = 0; r < 4; ++r) red[(((kh - 1) * NCG + cg) * 4 + r) * 64 + lane] = acc[r];
    }
    lds_barrier();
    if (kh == 0) {
#pragma unroll
      for (int h = 1; h < KH; ++h)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[r] += red[(((h - 1) * NCG + cg) * 4 + r) * 64 + lane];
    }
  }

  // ---- hand over, or finish the slab (wavefronts of share 0 hold the sums) ------------------
  // A partial is [column group][row pair][lane] x 8 bytes: every store and load is 512
  // contiguous bytes.
  if (part < m - 1) {
    // The partial and the flag are written with device-scope atomic stores (write-through to
    // the level all compute units share), so no cache write-back or invalidate is needed.
    unsigned long long* dst =
        reinterpret_cast<unsigned long long*>(p.partial + (size_t)b * ST_PARTIAL_FLOATS) + cg * 128 + lane;
    if (kh == 0) {
      __hip_atomic_store(dst, __builtin_bit_cast(unsigned long long, f32x2{acc[0], acc[1]}),
                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (p.T > 2)
        __hip_atomic_store(dst + 64, __builtin_bit_cast(unsigned long long, f32x2{acc[2], acc[3]}),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // every store of this wavefront has landed
    __syncthreads();
    if (tid == 0)
      __hip_atomic_store(p.flags + b, p.nonce, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  } else {
    f32x4 tot = zero4;
    if (m > 1) {
      const int bf = b - (m - 1);  // block of part 0 of this slab
      // one thread per flag, all polling at once
      for (int i = tid; i < m - 1; i += S4_THREADS) {
        uint32_t spins = 0;
        while (__hip_atomic_load(p.flags + bf + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != p.nonce) {
          if (++spins > S4_SPIN_LIMIT) {
            poison = 1;
            break;
          }
          __builtin_amdgcn_s_sleep(8);
        }
        // Consumed: clear it, so that a replay of this very launch (a captured graph repeats
        // the nonce) waits for its own producers instead of seeing this launch's flags.
        __hip_atomic_store(p.flags + bf + i, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      __syncthreads();
      // partials in part order, eight blocks' loads in flight at a time
      if (kh == 0) {
        for (int i0 = 0; i0 < m - 1; i0 += 8) {
          f32x2 v[8][2];
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const unsigned long long* src =
                reinterpret_cast<const unsigned long long*>(p.partial + (size_t)(bf + i0 + i) * ST_PARTIAL_FLOATS) +
                cg * 128 + lane;
            v[i][0] = v[i][1] = f32x2{0.0f, 0.0f};
            if (i0 + i < m - 1) {
              v[i][0] = __builtin_bit_cast(
                  f32x2, __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
              if (p.T > 2)
                v[i][1] = __builtin_bit_cast(
                    f32x2, __hip_atomic_load(src + 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            }
          }
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            tot[0] += v[i][0][0];
            tot[1] += v[i][0][1];
            tot[2] += v[i][1][0];
            tot[3] += v[i][1][1];
          }
        }
      }
    }
    const bool bad = (m > 1) && poison != 0;
    if (kh == 0 && col_ok) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float v = tot[r] + acc[r];
        if (bad) v = __builtin_nanf("");  // a wait ran out: make it loud
        if (r < p.T) {
          if (p.out_bf16)
            static_cast<uint16_t*>(p.out)[(size_t)r * p.d_out + j] = f32_to_bf16_bits(v);
          else
            static_cast<float*>(p.out)[(size_t)r * p.d_out + j] = v;
        }
      }
    }
  }
}

// Launch shape: slabs x parts with parts chosen to fill the compute units (at least one chunk
// per part); of the three slab widths, the one that occupies most compute units (ties: the
// narrower slab, which has fewer partials to add).
SmallTPlan smallt4_plan(int d_in, int d_out) {
  const int chunks = d_in / 128;
  SmallTPlan best{};
  for (int halves = 4; halves >= 1; halves /= 2) {
    SmallTPlan pl;
    pl.halves = halves;
    pl.slab_cols = (S4_WAVES / halves) * S4_WCOLS;
    pl.slabs = ceil_div(d_out, pl.slab_cols);
    int m = ST_MAX_BLOCKS / pl.slabs;
    if (m > chunks) m = chunks;
    if (m < 1) m = 1;
    pl.parts = m;
    pl.blocks = pl.slabs * m;
    const int busy = pl.blocks < ST_MAX_BLOCKS ? pl.blocks : ST_MAX_BLOCKS;
    const int best_busy = best.blocks < ST_MAX_BLOCKS ? best.blocks : ST_MAX_BLOCKS;
    if (halves == 4 || busy > best_busy) best = pl;
  }
  return best;
}

template <int SUB, int KH>
static hipError_t launch_sub4(const SmallTArgs& a, int grid, hipStream_t st) {
  static bool attr_set = false;  // per instantiation
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(smallt4_kernel<SUB, KH>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, S4_LDS);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  smallt4_kernel<SUB, KH><<<grid, S4_THREADS, S4_LDS, st>>>(a);
  return hipGetLastError();
}

template <int SUB>
static hipError_t launch_halves4(const SmallTArgs& a, const SmallTPlan& pl, hipStream_t st) {
  if (pl.halves == 4) return launch_sub4<SUB, 4>(a, pl.blocks, st);
  if (pl.halves == 2) return launch_sub4<SUB, 2>(a, pl.blocks, st);
  return launch_sub4<SUB, 1>(a, pl.blocks, st);
}

// `args.nonce` is set by the caller (launch_smallt), which also owns the measurement hook.
hipError_t launch_smallt4(const SmallTArgs& a, hipStream_t st) {
  const SmallTPlan pl = smallt4_plan(a.d_in, a.d_out);
  const int sub = a.group / 32;
  if (sub == 1) return launch_halves4<1>(a, pl, st);
  if (sub == 2) return launch_halves4<2>(a, pl, st);
  if (sub == 4) return launch_halves4<4>(a, pl, st);
  return hipErrorInvalidValue;
}

}  // namespace qalora
