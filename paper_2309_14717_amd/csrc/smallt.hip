// Adapter-free forward for a handful of tokens (T <= 16): the memory-bound regime of
// post-merge inference, where every call streams the whole quantized weight once.
//
//   y[t,j] = sum_l ( alpha[l,j] * sum_{i in group l} x[t,i] code[i,j]  +  beta[l,j] * sum_{i in l} x[t,i] )
//
// (Eq. 1 per group pulled out of the inner sum.)  The inner sums run on the matrix cores with
// EXACT operands: x is bf16 already, and a 4-bit code c becomes the bf16 number 128 + c by
// OR-ing it into the mantissa of 0x4300 -- no int->float conversion, no rounding.  The extra
// 128 * sum(x) is folded into beta.  alpha is applied in fp32 once per group; the beta term of a
// chunk, sum_groups beta'[group, col] sum(x)[token, group], is a small product of its own and
// runs on the fp32 matrix instruction, with the group sums of x taken from a table made when x
// is staged.  Nothing is rounded before the fp32 accumulation, so this path is more accurate
// than the large-T one.
//
// Decomposition.  The weight is cut into slabs of 256 or 512 output columns, and the 128-row
// chunks of each slab into m equal parts, m chosen so that slabs x m fills the 256 compute units
// with one block each; every block streams the same number of bytes.  Parts 0 .. m-2 leave
// their partial result in the workspace and raise a flag; the block of the last part (the
// highest-numbered one, so the others are already running or finished) waits for the flags,
// adds the partials in part order, then its own, and writes y.  The order of every sum is
// fixed by the shape alone: reruns are bit-identical.  The waits are bounded; if one ever ran
// out the block would write NaN instead of a wrong number.
//
// Inside a block the sixteen wavefronts are column groups of 32 columns each: sixteen of them
// (512-column slab), or eight times two halves of the block's chunks (256-column slab; the
// halves meet in LDS at the end).  x for the block's rows is staged once in LDS (one token
// row per wavefront) and read from there as MFMA operands, so the only traffic through the
// texture path is the weight itself.  Per chunk a lane issues four 8-byte code loads (2 columns
// x 8 rows each) and ONE alpha and ONE beta load: lane group kb = lane / 16 fetches the factors
// of the chunk's kb-th quantization group and the wavefront hands them round with ds_bpermute.
// All of them are buffer loads whose per-lane offset is fixed (the running position lives in
// the scalar offset); lanes outside the matrix read zeros from the range check.  Three chunk
// buffers rotate, so two chunks of loads are always in flight behind the one being multiplied.
#include <atomic>

#include "common.hpp"
#include "kernels.hpp"

namespace qalora {

namespace {

constexpr int ST_WAVES = 16;
constexpr int ST_THREADS = 64 * ST_WAVES;
constexpr int ST_CW = 2;                         // columns per lane
constexpr int ST_WCOLS = 16 * ST_CW;             // columns per wavefront
// tgs = groups of sixteen tokens (1 or 2): chunks of x staged in LDS at a time, and the bytes
// per token row in LDS (+16: bank spread)
constexpr int st_xchunks(int tgs) { return 32 / tgs; }
constexpr int st_xrow(int tgs) { return st_xchunks(tgs) * 256 + 16; }
constexpr uint32_t ST_SPIN_LIMIT = 1u << 18;     // bounded wait: the kernel always terminates
constexpr uint32_t kStOob = 0xffff0000u;         // beyond every buffer: the range check returns zero
constexpr int ST_NT = 2;                         // cache policy "nontemporal": streamed once


typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t st_rsrc(const void* base, size_t bytes) {
  const uint32_t n = bytes > 0xffffffffull ? 0xffffffffu : (uint32_t)bytes;
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)n, 0x00020000);
}

// One 128-row chunk of a wavefront's weight operands, as loaded.
struct Chunk {
  u32x2 w[4];    // codes: step st = rows 32*st + 8*kb .. +7 of the lane's 2 columns
  u32x2 al, be;  // factors of group (first group of the chunk) + kb
};

// LDS-only barrier: does not wait for the global loads that are in flight.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

}  // namespace

// SUB : 32-row steps per quantization group (group = 32 * SUB; 1, 2 or 4)
// KH  : ways a block splits its own chunks (1: sixteen column groups, slab of 512 columns;
//       2: eight column groups x two halves, slab of 256 columns)
// F16 : the factors of a (group, column) come as ONE word, fp16 alpha | fp16 beta << 16
// TGS : groups of sixteen tokens (1, 2): the second group reuses the code operand a lane has
//       built, with its own rows of x and its own accumulators
template <int SUB, int KH, bool F16, int TGS>
__global__ __launch_bounds__(ST_THREADS) void smallt_kernel(const SmallTArgs p) {
  extern __shared__ __align__(16) unsigned char xs[];  // [NTOK][ST_XROW], then the group sums
  __shared__ int poison;
  constexpr int CW = ST_CW;
  constexpr int NTOK = 16 * TGS;
  constexpr int ST_XCHUNKS = st_xchunks(TGS), ST_XROW = st_xrow(TGS);
  constexpr int ST_XPIECES = ST_XCHUNKS * 16 / 64;  // 1 KB wavefront copies per staged token row
  constexpr int NBUF = TGS == 1 ? 3 : 2;            // chunk buffers in rotation (registers)
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 15, kb = lane >> 4;
  constexpr int NCG = ST_WAVES / KH;   // column groups (32 columns each)
  constexpr int ST_SLAB_COLS = NCG * ST_WCOLS;
  const int cg = wave % NCG;
  const int kh = wave / NCG;           // which share of every staged piece's chunks
  const int L = p.d_in / p.group;
  const int C = p.d_in / 128;                      // chunks per slab
  const int S = ceil_div(p.d_out, ST_SLAB_COLS);   // slabs
  const int m = gridDim.x / S;                     // parts per slab
  const int b = blockIdx.x, s = b / m, part = b - s * m;
  const int ca = (int)((long)C * part / m), ce = (int)((long)C * (part + 1) / m);

  const __amdgpu_buffer_rsrc_t rs_w = st_rsrc(p.plane0, (size_t)(p.d_in / 8) * p.d_out * 4);
  const __amdgpu_buffer_rsrc_t rs_x = st_rsrc(p.x, (size_t)p.T * p.d_in * 2);
  const __amdgpu_buffer_rsrc_t rs_al = st_rsrc(F16 ? (const void*)p.fac16 : (const void*)p.alpha, (size_t)L * p.d_out * 4);
  const __amdgpu_buffer_rsrc_t rs_be = st_rsrc(p.beta, F16 ? 0 : (size_t)L * p.d_out * 4);
  constexpr int NLOADS = F16 ? 5 : 6;  // vector-memory loads of one chunk
  const uint32_t step_w = 4u * p.d_out * 4u;  // four packed rows per 32-row step
  const uint32_t row_ab = (uint32_t)p.d_out * 4u;
  // Mask and bias live in registers (not literals) so that "(w >> k) & mask | bias" is one
  // shift and one v_and_or_b32: a VOP3 instruction cannot carry a 32-bit literal on this target.
  uint32_t kMask, kBias;
  asm volatile("s_mov_b32 %0, 0x000f000f" : "=s"(kMask));
  asm volatile("v_mov_b32 %0, 0x43004300" : "=v"(kBias));
  const f32x4 zero4 = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  const unsigned char* xs_lane = xs + n * ST_XROW + 16 * kb;
  constexpr int NG = 4 / SUB;  // quantization groups per chunk
  float* gs = reinterpret_cast<float*>(xs + NTOK * ST_XROW);  // [chunk of the piece][group][NTOK tokens]

  {
    const int jw = cg * ST_WCOLS + CW * n;  // column inside the slab
    const int j0 = s * ST_SLAB_COLS + jw;
    const bool col_ok = j0 < p.d_out;
    const uint32_t voff_w = col_ok ? ((uint32_t)kb * p.d_out + j0) * 4u : kStOob;
    const uint32_t voff_ab = (col_ok && kb < 4 / SUB) ? ((uint32_t)kb * p.d_out + j0) * 4u : kStOob;

    // Loads of chunk c, or -- past the end `lim` of the wavefront's share -- the same number of
    // loads aimed outside the buffers: they return zeros without touching memory, and the
    // count of loads in flight (which the waits rely on) stays the same.
    auto load_chunk = [&](Chunk& ch, int c, int lim) {
      const bool live = c < lim;
      const uint32_t vw = live ? voff_w : kStOob, vab = live ? voff_ab : kStOob;
      c = min(c, C - 1);
#pragma unroll
      for (int st = 0; st < 4; ++st)
        ch.w[st] = __builtin_amdgcn_raw_buffer_load_b64(rs_w, (int)vw,
                                                        (int)((uint32_t)(4 * c + st) * step_w), ST_NT);
      const uint32_t so = (uint32_t)(4 * c / SUB) * row_ab;
      ch.al = __builtin_amdgcn_raw_buffer_load_b64(rs_al, (int)vab, (int)so, ST_NT);
      if constexpr (!F16) ch.be = __builtin_amdgcn_raw_buffer_load_b64(rs_be, (int)vab, (int)so, ST_NT);
    };

    f32x4 acc[TGS][CW];
#pragma unroll
    for (int tg = 0; tg < TGS; ++tg)
#pragma unroll
      for (int q = 0; q < CW; ++q) acc[tg][q] = zero4;

    // xrel: chunk index relative to the staged piece
    auto compute_chunk = [&](const Chunk& ch, int xrel) {
      // The beta term of the whole chunk, sum_groups beta'[group, col] * sum(x)[token, group], is
      // itself a small product [16 tokens x 4 groups] x [4 groups x columns]: one fp32 MFMA per
      // 16 columns.  Its B operand wants lane (n, kb) to supply beta' of group kb for column n --
      // exactly how the factors were LOADED (lane group kb fetched group kb), so beta needs no
      // hand-round at all; its A operand is the table of group sums made when x was staged.
      float sx[TGS];
#pragma unroll
      for (int tg = 0; tg < TGS; ++tg) sx[tg] = kb < NG ? gs[(xrel * NG + kb) * NTOK + 16 * tg + n] : 0.0f;
#pragma unroll
      for (int q = 0; q < CW; ++q) {
        float al_own, be_own;  // group kb of the chunk (zero for kb >= NG: the loads aimed outside)
        if constexpr (F16) {
          al_own = (float)__builtin_bit_cast(_Float16, (uint16_t)(ch.al[q] & 0xffffu));
          be_own = (float)__builtin_bit_cast(_Float16, (uint16_t)(ch.al[q] >> 16));
        } else {
          al_own = __uint_as_float(ch.al[q]);
          be_own = __uint_as_float(ch.be[q]);
        }
        const float bp = __builtin_fmaf(-128.0f, al_own, be_own);  // codes carry a +128 offset
#pragma unroll
        for (int tg = 0; tg < TGS; ++tg)
          acc[tg][q] = __builtin_amdgcn_mfma_f32_16x16x4f32(sx[tg], bp, acc[tg][q], 0, 0, 0);
      }
      f32x4 d[TGS][CW];
#pragma unroll
      for (int st = 0; st < 4; ++st) {
        const bool first = (st % SUB) == 0, last = (st % SUB) == SUB - 1;
        u32x4 xa[TGS];  // x of this 32-row step (read here, not a chunk ahead: registers)
#pragma unroll
        for (int tg = 0; tg < TGS; ++tg)
          xa[tg] = *reinterpret_cast<const u32x4*>(xs_lane + tg * 16 * ST_XROW + xrel * 256 + st * 64);
#pragma unroll
        for (int q = 0; q < CW; ++q) {
          const uint32_t w = ch.w[st][q];
          u32x4 bv;
          bv.x = (w & kMask) | kBias;
          bv.y = ((w >> 4) & kMask) | kBias;
          bv.z = ((w >> 8) & kMask) | kBias;
          bv.w = ((w >> 12) & kMask) | kBias;
#pragma unroll
          for (int tg = 0; tg < TGS; ++tg)
            d[tg][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xa[tg]),
                                                               __builtin_bit_cast(bf16x8, bv),
                                                               first ? zero4 : d[tg][q], 0, 0, 0);
        }
        if (last) {
          const int src = (n + 16 * (st / SUB)) * 4;  // the lane group holding this group's factors
#pragma unroll
          for (int q = 0; q < CW; ++q) {
            const uint32_t ab = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)ch.al[q]);
            const float al = F16 ? (float)__builtin_bit_cast(_Float16, (uint16_t)(ab & 0xffffu)) : __uint_as_float(ab);
#pragma unroll
            for (int tg = 0; tg < TGS; ++tg)
#pragma unroll
              for (int r = 0; r < 4; ++r) acc[tg][q][r] = __builtin_fmaf(al, d[tg][q][r], acc[tg][q][r]);
          }
        }
      }
    };

    for (int pa = ca; pa < ce; pa += ST_XCHUNKS) {  // pieces of at most ST_XCHUNKS chunks
      const int pe = min(ce, pa + ST_XCHUNKS);
      const int np = (pe - pa) * 16;  // 16-byte pieces per token row
      if (pa != ca) lds_barrier();  // every wavefront is done reading the previous piece
      // x of this piece: wavefront w copies token rows w (and w + 16) straight into LDS (no
      // registers).  The copies are issued BEFORE the weight prefetch, so waiting for them
      // leaves it in flight.
#pragma unroll
      for (int tg = 0; tg < TGS; ++tg) {
        const int row = wave + 16 * tg;
        if (row < p.T) {
          const uint32_t xoff = ((uint32_t)row * p.d_in + (uint32_t)pa * 128) * 2u + lane * 16u;
#pragma unroll
          for (int k = 0; k < ST_XPIECES; ++k)
            if (lane + 64 * k < np)
              __builtin_amdgcn_raw_ptr_buffer_load_lds(
                  rs_x, (__attribute__((address_space(3))) void*)(xs + row * ST_XROW + k * 1024), 16,
                  (int)xoff, k * 1024, 0, 0);
        }
      }
      // this wavefront's share of the piece: the first or the second half of its chunks
      const int pm = KH == 2 ? pa + (pe - pa + 1) / 2 : pe;
      const int wa = kh ? pm : pa, we = kh ? pe : pm;
      Chunk b0, b1, b2;  // b2 unused with two buffers
      load_chunk(b0, wa, we);
      if constexpr (NBUF == 3) load_chunk(b1, wa + 1, we);
      __builtin_amdgcn_sched_barrier(0);
      if (pa == ca) {
        // first piece: with the loads above already in flight, clear what must start at zero --
        // the token rows that do not exist (they stay zero for the whole kernel)
        if (tid == 0) poison = 0;
#pragma unroll
        for (int tg = 0; tg < TGS; ++tg) {
          const int row = wave + 16 * tg;
          if (row >= p.T) {
            for (int o = lane; o < ST_XROW / 16; o += 64)
              *reinterpret_cast<u32x4*>(xs + row * ST_XROW + o * 16) = u32x4{0, 0, 0, 0};
          }
        }
      }
      // two chunks of weight loads were issued after the copies: once at most that many are outstanding,
      // the copies have landed
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NBUF - 1) * NLOADS) : "memory");
      lds_barrier();
      // group sums of x for the piece, one (group, token) pair per thread, element order
      for (int idx = tid; idx < (pe - pa) * NG * NTOK; idx += ST_THREADS) {
        const int grp = idx / NTOK, tok = idx % NTOK;
        const unsigned char* src = xs + tok * ST_XROW + grp * (64 * SUB);
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
        gs[grp * NTOK + tok] = sum;
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

    // ---- the two halves of the block meet in LDS (fixed order: first half + second half) ----
    if constexpr (KH == 2) {
      float* red = reinterpret_cast<float*>(xs);  // [8 column groups][8 TGS registers][64 lanes]
      lds_barrier();                              // x is no longer needed
      if (kh == 1) {
#pragma unroll
        for (int tg = 0; tg < TGS; ++tg)
#pragma unroll
          for (int q = 0; q < CW; ++q)
#pragma unroll
            for (int r = 0; r < 4; ++r) red[((cg * TGS + tg) * 8 + 4 * q + r) * 64 + lane] = acc[tg][q][r];
      }
      lds_barrier();
      if (kh == 0) {
#pragma unroll
        for (int tg = 0; tg < TGS; ++tg)
#pragma unroll
          for (int q = 0; q < CW; ++q)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[tg][q][r] += red[((cg * TGS + tg) * 8 + 4 * q + r) * 64 + lane];
      }
    }

    // ---- hand over, or finish the slab (wavefronts of the first half hold the sums) --------
    // D layout: lane (n, kb) holds rows 4*kb + r of columns 2n, 2n+1.  The block's sums are
    // first laid out in LDS as a [token][column] tile, so that they travel as 16-byte accesses,
    // one (token, four columns) item per thread: a partial leaves the block in far fewer memory
    // instructions than the accumulator layout would need, and the cost of the hand-over goes
    // with the number of these cache-bypassing accesses.  They carry the cache policy of a
    // device-scope atomic (coherent at the level all compute units share), so no cache
    // write-back or invalidate is needed -- those walk a whole L2 and cost far more than the
    // few KB moved here.
    float* tile = reinterpret_cast<float*>(xs);  // [NTOK][ST_SLAB_COLS]
    constexpr int kDeviceCoherent = 16;          // "sc1"
    constexpr int C4 = ST_SLAB_COLS / 4;         // items per token row
    constexpr int ITEMS_PER_THREAD = (NTOK * C4 + ST_THREADS - 1) / ST_THREADS;
    constexpr int PART_FLOATS = TGS * ST_PARTIAL_FLOATS;  // a block's partial: the [NTOK][512] tile at most
    static_assert(NTOK * ST_SLAB_COLS <= PART_FLOATS, "a partial holds the whole tile");
    lds_barrier();  // x and the meeting area of the halves are no longer needed
    if (kh == 0) {
#pragma unroll
      for (int tg = 0; tg < TGS; ++tg)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          *reinterpret_cast<f32x2*>(tile + (16 * tg + 4 * kb + r) * ST_SLAB_COLS + cg * ST_WCOLS + CW * n) =
              f32x2{acc[tg][0][r], acc[tg][1][r]};
    }
    lds_barrier();
    const int items = p.T * C4;
    const __amdgpu_buffer_rsrc_t rs_p = st_rsrc(p.partial, (size_t)gridDim.x * PART_FLOATS * 4);
    if (part < m - 1) {
#pragma unroll
      for (int k = 0; k < ITEMS_PER_THREAD; ++k) {
        const int it = tid + k * ST_THREADS;
        if (it < items) {
          const int r = it / C4, c4 = it - r * C4;
          const u32x4 v = *reinterpret_cast<const u32x4*>(tile + r * ST_SLAB_COLS + 4 * c4);
          __builtin_amdgcn_raw_buffer_store_b128(v, rs_p, (r * ST_SLAB_COLS + 4 * c4) * 4,
                                                 (int)((uint32_t)b * (PART_FLOATS * 4u)), kDeviceCoherent);
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
        for (int i = tid; i < m - 1; i += ST_THREADS) {
          uint32_t spins = 0;
          bool timed_out = false;
          while (__hip_atomic_load(p.flags + bf + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != p.nonce) {
            if (++spins > ST_SPIN_LIMIT) {
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
          const int it = tid + k * ST_THREADS;
          if (it < items) {
            const int r = it / C4, c4 = it - r * C4;
            for (int i0 = 0; i0 < m - 1; i0 += PB) {
              u32x4 v[PB];
#pragma unroll
              for (int i = 0; i < PB; ++i) {
                v[i] = u32x4{0, 0, 0, 0};
                if (i0 + i < m - 1)
                  v[i] = __builtin_amdgcn_raw_buffer_load_b128(
                      rs_p, (r * ST_SLAB_COLS + 4 * c4) * 4,
                      (int)((uint32_t)(bf + i0 + i) * (PART_FLOATS * 4u)), kDeviceCoherent);
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
        const int it = tid + k * ST_THREADS;
        if (it < items) {
          const int r = it / C4, c4 = it - r * C4;
          const int jj = s * ST_SLAB_COLS + 4 * c4;  // d_out is a multiple of 8: four columns are all in or all out
          if (jj < p.d_out) {
            f32x4 v = tot[k] + *reinterpret_cast<const f32x4*>(tile + r * ST_SLAB_COLS + 4 * c4);
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
}

// Launch shape: slabs x parts with parts chosen to fill the compute units (at least one chunk
// per part).  Of the two slab widths, the one with fewer parts to add if both keep at least
// kEnoughBlocks compute units streaming (HBM is saturated from about four fifths of the chip
// on, and every further part costs a hand-over: 4096 x 11008 at sixteen tokens takes 18.6 us
// as 22 slabs x 11 parts and 14.8 us as 43 x 5), otherwise the one that occupies more units.
SmallTPlan smallt_plan(int d_in, int d_out, int tokens) {
  constexpr int kEnoughBlocks = 200;
  const int chunks = d_in / 128;
  SmallTPlan best{};
  bool have = false;
  (void)tokens;  // both widths serve every token count (a partial of the two-group form is twice the size)
  for (int halves = 2; halves >= 1; --halves) {
    SmallTPlan pl;
    pl.halves = halves;
    pl.slab_cols = (ST_WAVES / halves) * ST_WCOLS;
    pl.slabs = ceil_div(d_out, pl.slab_cols);
    int m = ST_MAX_BLOCKS / pl.slabs;
    if (m > chunks) m = chunks;
    if (m < 1) m = 1;
    pl.parts = m;
    pl.blocks = pl.slabs * m;
    const int busy = pl.blocks < ST_MAX_BLOCKS ? pl.blocks : ST_MAX_BLOCKS;
    const int best_busy = best.blocks < ST_MAX_BLOCKS ? best.blocks : ST_MAX_BLOCKS;
    bool better;
    if (!have) better = true;
    else if (busy >= kEnoughBlocks && best_busy >= kEnoughBlocks)
      better = pl.parts < best.parts || (pl.parts == best.parts && busy > best_busy);
    else
      better = busy > best_busy;
    if (better) {
      best = pl;
      have = true;
    }
  }
  return best;
}

template <int SUB, int KH, bool F16, int TGS>
static hipError_t launch_tgs(const SmallTArgs& a, int grid, hipStream_t st) {
  constexpr size_t smem = 16 * TGS * st_xrow(TGS) + st_xchunks(TGS) * 4 * 16 * TGS * sizeof(float);
  static std::atomic<uint64_t> granted{0};  // per instantiation
  if (hipError_t e = grant_dynamic_lds(reinterpret_cast<const void*>(smallt_kernel<SUB, KH, F16, TGS>), (int)smem, granted);
      e != hipSuccess)
    return e;
  smallt_kernel<SUB, KH, F16, TGS><<<grid, ST_THREADS, smem, st>>>(a);
  return hipGetLastError();
}

// seventeen to thirty-two tokens take the two-group form
template <int SUB, int KH, bool F16>
static hipError_t launch_sub(const SmallTArgs& a, int grid, hipStream_t st) {
  if (a.T <= 16) return launch_tgs<SUB, KH, F16, 1>(a, grid, st);
  return launch_tgs<SUB, KH, F16, 2>(a, grid, st);
}

// A value no earlier call of this process has written to the flags (and never zero).
unsigned long long smallt_next_nonce() {
  static std::atomic<unsigned long long> calls{0};
  unsigned long long z = (calls.fetch_add(1) + 1) * 0x9e3779b97f4a7c15ull;
  z ^= z >> 31;  // both steps are bijections that fix zero, and the count is never zero
  return z;
}

hipError_t launch_smallt(const SmallTArgs& args, hipStream_t st) {
  SmallTArgs a = args;
  a.nonce = smallt_next_nonce();
  const SmallTPlan pl = smallt_plan(a.d_in, a.d_out, a.T);
  const int sub = a.group / 32;
  auto run = [&]() -> hipError_t {
    // decode shapes and the narrower codes: the one-column-per-lane kernel
    if (a.T <= 4 || a.bits != 4) return launch_smallt4(a, st);
    if (pl.halves == 2) {
      if (sub == 1) return a.fac16 ? launch_sub<1, 2, true>(a, pl.blocks, st) : launch_sub<1, 2, false>(a, pl.blocks, st);
      if (sub == 2) return a.fac16 ? launch_sub<2, 2, true>(a, pl.blocks, st) : launch_sub<2, 2, false>(a, pl.blocks, st);
      if (sub == 4) return a.fac16 ? launch_sub<4, 2, true>(a, pl.blocks, st) : launch_sub<4, 2, false>(a, pl.blocks, st);
    } else {
      if (sub == 1) return a.fac16 ? launch_sub<1, 1, true>(a, pl.blocks, st) : launch_sub<1, 1, false>(a, pl.blocks, st);
      if (sub == 2) return a.fac16 ? launch_sub<2, 1, true>(a, pl.blocks, st) : launch_sub<2, 1, false>(a, pl.blocks, st);
      if (sub == 4) return a.fac16 ? launch_sub<4, 1, true>(a, pl.blocks, st) : launch_sub<4, 1, false>(a, pl.blocks, st);
    }
    return hipErrorInvalidValue;
  };
  // measurement aid: this kernel is the forward contraction of the small-token regime
  ProfileHook hook = g_profile_hook[0];
  g_profile_hook[0] = ProfileHook{nullptr, nullptr, nullptr};
  if (hook.start) (void)hipEventRecord(hook.start, st);
  const hipError_t e = run();
  if (hook.stop) (void)hipEventRecord(hook.stop, st);
  return e;
}

}  // namespace qalora
