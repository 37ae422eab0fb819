// The dense contractions of the QA-LoRA linear on the matrix cores of gfx950:
//
//   forward   y  = [x | s U~] . [W~ ; B~]        K = D_in  (+ adapter tail), N = D_out
//   backward  dx = [dy | dU~] . [W~^T ; A~/g]    K = D_out (+ adapter tail), N = D_in
//
// with W~[i,j] = alpha[i/g,j] * code[i,j] + beta[i/g,j] (Eq. 1 per group, Sec. 3.3)
// rebuilt on the fly: packed codes are read with 128-bit loads, dequantised in registers
// with packed 16-bit fma, staged in LDS and fed to v_mfma_f32_32x32x16 with fp32
// accumulation.
//
// Operand precision.  The main K steps run the matrix cores in fp16 (same rate as bf16 on
// gfx950): W~ keeps 11 significant bits instead of 8, which is what keeps the result inside
// the 2e-3 parity bar for every bit width (with bf16 operands the 4-level INT2 grids land
// on 2.1e-3).  The activations arrive here already converted: every token row scaled by a
// power of two that brings its largest magnitude into [2^14, 2^15) and written as fp16
// (exact for bf16 inputs); the output row is scaled back in the epilogue.
//
// The low-rank branch of Alg. 1, s (pool(x) A) B, rides along as a few extra K steps in
// bf16: the small factors are split into bf16 hi + lo parts (hi*hi + lo*hi + hi*lo), which
// keeps fp32-level accuracy and bf16's range for gradients.
//
// One kernel serves both directions from ONE packed copy of the codes: a thread owns half
// of an 8x8 patch of codes, from which it emits four K-contiguous operand fragments along
// either axis -- down the rows (forward, K = input rows) or across the columns (backward,
// K = output columns).
//
// Tiling: 512 threads = 8 wavefronts (two per SIMD, so one can dequantise while the other
// feeds the matrix core), block tile BM x BN x 64, double-buffered in LDS.  The A tile goes
// global -> LDS directly (128-bit LDS-DMA loads, no registers); the B tile goes through
// registers for dequantisation.  LDS rows are 128 bytes, XOR-swizzled so that operand reads
// (16 consecutive rows, one 16-byte chunk) and both producers' writes are bank-conflict free.
#include <type_traits>

#include "common.hpp"
#include "kernels.hpp"

namespace qalora {

constexpr int BK = 64;
constexpr int NT = 512;  // threads per block

__device__ __forceinline__ uint4 ldg128(const void* p) {
  return *reinterpret_cast<const uint4*>(p);
}

// Byte offset inside a [rows][64 x 16-bit] tile of the 16-byte chunk `c` of row `n`.
// Two rows share a 256-byte line (half = which 128 bytes); the chunk slot is XORed with row
// bits.  With n = b7..b0:  half = b0^b3^b4,  slot = c ^ (b1^b5 | b2<<1 | b3<<2).
// Distinct (half, slot) for: 16 consecutive rows at one chunk (operand reads), 16 rows of
// stride 4 at one chunk (forward producer), rows n and n+8 over all chunks (backward
// producer), rows n and n+1 over all chunks (plain copies).
__device__ __forceinline__ int swz_offset(int n, int c) {
  const int half = (n ^ (n >> 3) ^ (n >> 4)) & 1;
  const int f = (((n >> 1) ^ (n >> 5)) & 1) | (((n >> 2) & 3) << 1);
  return ((n >> 1) << 8) | (half << 7) | ((c ^ f) << 4);
}
// Inverse for the LDS-DMA path: which (row, chunk) lives at byte offset `o` (multiple of 16).
__device__ __forceinline__ void swz_inverse(int o, int& n, int& c) {
  const int pair = o >> 8, half = (o >> 7) & 1, slot = (o >> 4) & 7;
  const int b3 = (pair >> 2) & 1, b4 = (pair >> 3) & 1;
  n = 2 * pair + (half ^ b3 ^ b4);
  const int f = ((pair ^ (pair >> 4)) & 1) | (((pair >> 1) & 3) << 1);
  c = slot ^ f;
}

// Block-index -> tile-index map.  Consecutive block ids are dealt round-robin to the 8
// XCDs, each with its own L2; give every XCD a contiguous run of tiles (tile_m fastest)
// so that the weight panels and activation rows it touches stay in that L2.
__device__ __forceinline__ int xcd_remap(int bid, int nblocks) {
  if (nblocks % 8 != 0) return bid;
  return (bid % 8) * (nblocks / 8) + bid / 8;
}

// HAS_MAIN = false: a plain bf16 x bf16^T product over the "tail" operands only (used for
// dU = s dy B^T), optionally split along K over blockIdx.y.
template <int NBITS, bool BWD, int BM, int BN, int WAVES_M, int WAVES_N, bool HAS_MAIN>
__global__ __launch_bounds__(NT) void gemm_dq_kernel(const GemmArgs p) {
  static_assert(WAVES_M * WAVES_N == 8, "eight wavefronts per block");
  static_assert(!HAS_MAIN || BN == 256, "the dequantising producer assumes 256 columns");
  constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  static_assert(TM >= 1 && TN >= 1, "wave tile must hold at least one 32x32 MFMA tile");
  constexpr int A_LOADS = BM * 8 / NT;                           // LDS-DMA loads per thread
  constexpr int B_CHUNKS = (BN * 8 / NT) > 0 ? BN * 8 / NT : 1;  // plain B tile, per thread
  static_assert(A_LOADS >= 1, "BM too small for 512 threads");
  constexpr int A_TILE = BM * 64;  // 16-bit elements per A buffer
  constexpr int B_TILE = BN * 64;

  extern __shared__ __align__(1024) uint16_t smem[];
  uint16_t* As = smem;               // [2][BM][64] swizzled
  uint16_t* Bs = smem + 2 * A_TILE;  // [2][BN][64] swizzled

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;

  const int tiles_m = ceil_div(p.M, BM);
  const int tiles_n = ceil_div(p.N, BN);
  const int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n);
  const int m0 = (tile % tiles_m) * BM;
  const int n0 = (tile / tiles_m) * BN;

  const int nk_main = HAS_MAIN ? ceil_div(p.K_main, BK) : 0;
  const int nk_tail = ceil_div(p.K_tail, BK);
  int it_begin = 0, it_end = nk_main + nk_tail;
  if (!HAS_MAIN && gridDim.y > 1) {
    const int per = ceil_div(nk_tail, (int)gridDim.y);
    it_begin = blockIdx.y * per;
    it_end = min(nk_tail, it_begin + per);
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;

  // Step kinds: a K step is either a MAIN step (fp16: converted activations x dequantised
  // codes) or a TAIL step (bf16 hi/lo adapter operands, plain copies).  The pipeline below is
  // instantiated per (current kind, next kind) so that the hot loop carries no branches.
  using MainK = std::integral_constant<int, 0>;
  using TailK = std::integral_constant<int, 1>;
  using NoneK = std::integral_constant<int, 2>;

  // ---- A tile: global -> LDS by LDS-DMA.  Load q of wave w fills the 1 KB block q*8+w;
  // lane i lands at byte 16*i of it, so it fetches the (row, chunk) the swizzle puts there.
  // Rows past M are clamped to the last row (their results are never stored); K chunks past
  // the end re-read chunk 0 (the B tile is zero there, any finite data will do).
  const uint16_t* a_src_main[A_LOADS];
  const uint16_t* a_src_tail[A_LOADS];
  int a_chunk8[A_LOADS];
#pragma unroll
  for (int q = 0; q < A_LOADS; ++q) {
    int n, c;
    swz_inverse((q * 8 + wave) * 1024 + lane * 16, n, c);
    const int row = min(m0 + n, p.M - 1);
    a_chunk8[q] = 8 * c;
    a_src_main[q] = HAS_MAIN ? p.a_main + (size_t)row * p.lda_main : nullptr;
    a_src_tail[q] = p.a_tail + (size_t)row * p.lda_tail;
  }
  auto issue_a = [&](auto kind, int it, int buf) {
    constexpr bool kMain = decltype(kind)::value == 0;
    const int k0 = kMain ? it * BK : (it - nk_main) * BK;
    const int klim = kMain ? p.K_main : p.K_tail;
#pragma unroll
    for (int q = 0; q < A_LOADS; ++q) {
      int k = k0 + a_chunk8[q];
      k = (k < klim) ? k : 0;
      const uint16_t* src = (kMain ? a_src_main[q] : a_src_tail[q]) + k;
      uint16_t* dst = As + buf * A_TILE + (q * 8 + wave) * 512;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                       (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
    }
  };

  // ---- B tile through registers --------------------------------------------------------
  // MAIN steps: half an 8x8 patch of codes per thread.
  //   forward : wave = K chunk u0, lane -> column quad (coalesced 1 KB rows of words)
  //   backward: u0 = K chunk (column octet), u1 = row block, hb = which two row pairs
  // Out-of-range patches are read from a clamped address and get alpha = beta = 0.
  const int f_u0 = wave, f_cq = lane;
  const int b_u0 = tid & 7, b_u1 = (tid >> 3) & 31, b_hb = tid >> 8;
  constexpr int RB0 = PackFmt<NBITS>::kRowsPerWord0;
  // the K-invariant coordinate of this thread's patch, clamped, and its validity
  const int f_j0 = n0 + 4 * f_cq;
  const int b_i0 = n0 + 8 * b_u1;
  const bool n_valid = BWD ? (b_i0 < p.d_in) : (f_j0 < p.d_out);
  const int f_j0c = min(f_j0, p.d_out - 4);
  const int b_i0c = min(b_i0, p.d_in - 8);

  uint4 breg[6];   // fwd: codes, alpha, beta, plane-1 codes | bwd: 2 codes, 2 alpha, 2 beta
  uint4 breg1[2];  // bwd, N = 3: plane-1 words
  uint4 btail[B_CHUNKS];
  uint32_t bmask = 0;  // all-ones when the patch being staged is inside the matrix

  auto gload_b = [&](auto kind, int it) {
    constexpr bool kMain = decltype(kind)::value == 0;
    if constexpr (kMain) {
      const int k0 = it * BK;
      if constexpr (!BWD) {
        const int i0 = k0 + 8 * f_u0;
        const int i0c = min(i0, p.d_in - 8);
        bmask = (n_valid && i0 < p.d_in) ? 0xffffffffu : 0u;
        breg[0] = ldg128(p.plane0 + (size_t)(i0c / RB0) * p.d_out + f_j0c);
        if constexpr (NBITS == 3)
          breg[3] = ldg128(p.plane1 + (size_t)(i0c / 32) * p.d_out + f_j0c);
        const size_t ab = (size_t)(i0c / p.group) * p.d_out + f_j0c;
        breg[1] = ldg128(p.alpha + ab);
        breg[2] = ldg128(p.beta + ab);
      } else {
        const int j0 = k0 + 8 * b_u0;
        const int j0c = min(j0, p.d_out - 8);
        bmask = (n_valid && j0 < p.d_out) ? 0xffffffffu : 0u;
        const uint32_t* w = p.plane0 + (size_t)(b_i0c / RB0) * p.d_out + j0c;
        breg[0] = ldg128(w);
        breg[1] = ldg128(w + 4);
        if constexpr (NBITS == 3) {
          const uint32_t* w1 = p.plane1 + (size_t)(b_i0c / 32) * p.d_out + j0c;
          breg1[0] = ldg128(w1);
          breg1[1] = ldg128(w1 + 4);
        }
        const size_t ab = (size_t)(b_i0c / p.group) * p.d_out + j0c;
        breg[2] = ldg128(p.alpha + ab);
        breg[3] = ldg128(p.alpha + ab + 4);
        breg[4] = ldg128(p.beta + ab);
        breg[5] = ldg128(p.beta + ab + 4);
      }
    } else {
      const int k0 = (it - nk_main) * BK;
#pragma unroll
      for (int q = 0; q < B_CHUNKS; ++q) {
        const int idx = tid + NT * q;
        const int row = idx >> 3, ch = idx & 7;
        const int n = n0 + row;
        // forward tail: row n of B~^T; backward tail: row n/g of A~ (the unpooling of
        // the pooled gradient is this broadcast over the g rows of a group)
        const int src_row = BWD ? n / p.group : n;
        btail[q] = (row < BN && n < p.N && k0 + 8 * ch < p.K_tail)
                       ? ldg128(p.b_tail + (size_t)src_row * p.K_tail + k0 + 8 * ch)
                       : uint4{0, 0, 0, 0};
      }
    }
  };

  // alpha * code + beta for the row pair m of one column, as a packed fp16 pair
  auto ab_pair = [&](uint32_t a_bits, uint32_t b_bits) {
    const f32x2 abf = {__uint_as_float(a_bits & bmask), __uint_as_float(b_bits & bmask)};
    return __builtin_convertvector(abf, f16x2);
  };
  auto dq_pair = [&](uint32_t w0s, uint32_t w1s, f16x2 ab, int m) {
    const f16x2 a2 = {ab.x, ab.x};
    const f16x2 b2 = {ab.y, ab.y};
    const f16x2 cc = patch_code_pair_f16<NBITS>(w0s, w1s, m);
    return __builtin_bit_cast(uint32_t, cc * a2 + b2);
  };

  auto store_b = [&](auto kind, int it, int buf) {
    constexpr bool kMain = decltype(kind)::value == 0;
    char* bs = reinterpret_cast<char*>(Bs + buf * B_TILE);
    if constexpr (kMain) {
      if constexpr (!BWD) {
        const int i0 = it * BK + 8 * f_u0;
        const int sh0 = patch_preshift0<NBITS>(i0), sh1 = patch_preshift1(i0);
        const uint32_t w0[4] = {breg[0].x, breg[0].y, breg[0].z, breg[0].w};
        const uint32_t w1[4] = {breg[3].x, breg[3].y, breg[3].z, breg[3].w};
        const uint32_t al[4] = {breg[1].x, breg[1].y, breg[1].z, breg[1].w};
        const uint32_t be[4] = {breg[2].x, breg[2].y, breg[2].z, breg[2].w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const uint32_t w0s = w0[c] >> sh0;
          const uint32_t w1s = (NBITS == 3) ? (w1[c] >> sh1) : 0u;
          const f16x2 ab = ab_pair(al[c], be[c]);
          uint4 frag;
          frag.x = dq_pair(w0s, w1s, ab, 0);
          frag.y = dq_pair(w0s, w1s, ab, 1);
          frag.z = dq_pair(w0s, w1s, ab, 2);
          frag.w = dq_pair(w0s, w1s, ab, 3);
          *reinterpret_cast<uint4*>(bs + swz_offset(4 * f_cq + c, f_u0)) = frag;
        }
      } else {
        constexpr int LB = (NBITS == 3) ? 2 : NBITS;
        // pre-shift so that this thread's two row pairs (2*hb, 2*hb+1) sit at pairs 0, 1
        const int sh0 = patch_preshift0<NBITS>(b_i0) + LB * 2 * b_hb;
        const int sh1 = patch_preshift1(b_i0) + 2 * b_hb;
        const uint32_t w0[8] = {breg[0].x, breg[0].y, breg[0].z, breg[0].w,
                                breg[1].x, breg[1].y, breg[1].z, breg[1].w};
        const uint32_t w1[8] = {breg1[0].x, breg1[0].y, breg1[0].z, breg1[0].w,
                                breg1[1].x, breg1[1].y, breg1[1].z, breg1[1].w};
        const uint32_t al[8] = {breg[2].x, breg[2].y, breg[2].z, breg[2].w,
                                breg[3].x, breg[3].y, breg[3].z, breg[3].w};
        const uint32_t be[8] = {breg[4].x, breg[4].y, breg[4].z, breg[4].w,
                                breg[5].x, breg[5].y, breg[5].z, breg[5].w};
        uint32_t wt[8][2];  // [column][row pair]: (W~[2m][c], W~[2m+1][c])
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          const uint32_t w0s = w0[c] >> sh0;
          const uint32_t w1s = (NBITS == 3) ? (w1[c] >> sh1) : 0u;
          const f16x2 ab = ab_pair(al[c], be[c]);
          wt[c][0] = dq_pair(w0s, w1s, ab, 0);
          wt[c][1] = dq_pair(w0s, w1s, ab, 1);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {  // row 4*hb + r of the patch: gather the 8 columns
          uint32_t o[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const uint32_t lo = wt[2 * q][r >> 1], hi = wt[2 * q + 1][r >> 1];
            o[q] = (r & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u)
                           : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
          }
          *reinterpret_cast<uint4*>(bs + swz_offset(8 * b_u1 + 4 * b_hb + r, b_u0)) =
              uint4{o[0], o[1], o[2], o[3]};
        }
      }
    } else {
#pragma unroll
      for (int q = 0; q < B_CHUNKS; ++q) {
        const int idx = tid + NT * q;
        const int row = idx >> 3, ch = idx & 7;
        if (row < BN) *reinterpret_cast<uint4*>(bs + swz_offset(row, ch)) = btail[q];
      }
    }
  };

  // ---- LDS -> matrix cores ---------------------------------------------------------
  // lane (r = lane % 32, kb = lane / 32) reads chunk 2*kk + kb of row base + r; the swizzled
  // offset of chunk c is offset(row, 0) ^ (c << 4).
  int a_off[TM], b_off[TN];
#pragma unroll
  for (int a = 0; a < TM; ++a) a_off[a] = swz_offset(wm * WTM + a * 32 + (lane & 31), 0);
#pragma unroll
  for (int b = 0; b < TN; ++b) b_off[b] = swz_offset(wn * WTN + b * 32 + (lane & 31), 0);

  auto compute = [&](auto kind, int buf) {
    constexpr bool kMain = decltype(kind)::value == 0;
    const char* as = reinterpret_cast<const char*>(As + buf * A_TILE);
    const char* bs = reinterpret_cast<const char*>(Bs + buf * B_TILE);
    uint4 af[2][TM], bf[2][TN];
    auto load_frags = [&](int kk, int slot) {
      const int cx = (2 * kk + (lane >> 5)) << 4;
#pragma unroll
      for (int a = 0; a < TM; ++a)
        af[slot][a] = *reinterpret_cast<const uint4*>(as + (a_off[a] ^ cx));
#pragma unroll
      for (int b = 0; b < TN; ++b)
        bf[slot][b] = *reinterpret_cast<const uint4*>(bs + (b_off[b] ^ cx));
    };
    load_frags(0, 0);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      const int cur = kk & 1;
      if (kk + 1 < BK / 16) load_frags(kk + 1, cur ^ 1);  // fragments of the next step in flight
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) {
          if constexpr (kMain)
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                __builtin_bit_cast(f16x8, af[cur][a]), __builtin_bit_cast(f16x8, bf[cur][b]),
                acc[a][b], 0, 0, 0);
          else
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                __builtin_bit_cast(bf16x8, af[cur][a]), __builtin_bit_cast(bf16x8, bf[cur][b]),
                acc[a][b], 0, 0, 0);
        }
      __builtin_amdgcn_sched_barrier(0);  // keep the fragment prefetch depth at one step
    }
  };

  // One pipelined K step: start the loads of step it+1, run the matrix cores on step it,
  // then dequantise / stage step it+1.
  auto step = [&](auto cur, auto next, int it, int buf) {
    constexpr bool kHasNext = decltype(next)::value != 2;
    if constexpr (kHasNext) {
      issue_a(next, it + 1, buf ^ 1);
      gload_b(next, it + 1);
    }
    __builtin_amdgcn_sched_barrier(0);
    compute(cur, buf);
    if constexpr (kHasNext) store_b(next, it + 1, buf ^ 1);
    __syncthreads();  // also waits for the LDS-DMA loads of the next A tile
  };

  if (it_begin < it_end) {
    int it = it_begin, buf = 0;
    if (HAS_MAIN && nk_main > 0) {
      issue_a(MainK{}, it, 0);
      gload_b(MainK{}, it);
      store_b(MainK{}, it, 0);
      __syncthreads();
      for (; it + 1 < nk_main; ++it, buf ^= 1) step(MainK{}, MainK{}, it, buf);
      if (nk_tail > 0) {
        step(MainK{}, TailK{}, it, buf);
        ++it, buf ^= 1;
        for (; it + 1 < it_end; ++it, buf ^= 1) step(TailK{}, TailK{}, it, buf);
        step(TailK{}, NoneK{}, it, buf);
      } else {
        step(MainK{}, NoneK{}, it, buf);
      }
    } else {
      issue_a(TailK{}, it, 0);
      gload_b(TailK{}, it);
      store_b(TailK{}, it, 0);
      __syncthreads();
      for (; it + 1 < it_end; ++it, buf ^= 1) step(TailK{}, TailK{}, it, buf);
      step(TailK{}, NoneK{}, it, buf);
    }
  }

  // ---- epilogue: D[m][n] lives at lane n%32, register 4*(m/8) + m%4, half (m/4)%2 ----
  const size_t zoff = (size_t)blockIdx.y * (size_t)p.M * (size_t)p.N;
#pragma unroll
  for (int a = 0; a < TM; ++a) {
    float inv[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = m0 + wm * WTM + a * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      inv[r] = (HAS_MAIN && row < p.M) ? p.row_scale[row].y : 1.0f;
    }
#pragma unroll
    for (int b = 0; b < TN; ++b) {
      const int col = n0 + wn * WTN + b * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * WTM + a * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < p.M && col < p.N) {
          const size_t o = zoff + (size_t)row * p.N + col;
          const float v = acc[a][b][r] * inv[r];
          if (p.out_bf16)
            static_cast<uint16_t*>(p.out)[o] = f32_to_bf16_bits(v);
          else
            static_cast<float*>(p.out)[o] = v;
        }
      }
    }
  }
}

template <int NBITS, bool BWD, int BM, int BN, int WAVES_M, int WAVES_N, bool HAS_MAIN>
static hipError_t launch_cfg(const GemmArgs& a, int ksplit, hipStream_t st) {
  auto kern = gemm_dq_kernel<NBITS, BWD, BM, BN, WAVES_M, WAVES_N, HAS_MAIN>;
  const size_t smem = (size_t)2 * (BM + BN) * 64 * sizeof(uint16_t);
  static bool attr_set = false;  // per instantiation
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  dim3 grid(ceil_div(a.M, BM) * ceil_div(a.N, BN), ksplit);
  kern<<<grid, NT, smem, st>>>(a);
  return hipGetLastError();
}

template <int NBITS, bool BWD>
static hipError_t launch_dir(const GemmArgs& a, hipStream_t st) {
  if (a.M > 128) return launch_cfg<NBITS, BWD, 256, 256, 2, 4, true>(a, 1, st);
  if (a.M > 64) return launch_cfg<NBITS, BWD, 128, 256, 2, 4, true>(a, 1, st);
  return launch_cfg<NBITS, BWD, 64, 256, 1, 8, true>(a, 1, st);
}

ProfileHook g_profile_hook[2] = {{nullptr, nullptr}, {nullptr, nullptr}};

static hipError_t launch_bits(int bits, bool bwd, const GemmArgs& a, hipStream_t st) {
  if (bits == 4) return bwd ? launch_dir<4, true>(a, st) : launch_dir<4, false>(a, st);
  if (bits == 3) return bwd ? launch_dir<3, true>(a, st) : launch_dir<3, false>(a, st);
  return bwd ? launch_dir<2, true>(a, st) : launch_dir<2, false>(a, st);
}

hipError_t launch_gemm_dq(int bits, bool bwd, const GemmArgs& a, hipStream_t st) {
  ProfileHook hook = g_profile_hook[bwd ? 1 : 0];
  g_profile_hook[bwd ? 1 : 0] = ProfileHook{nullptr, nullptr};
  if (hook.start) (void)hipEventRecord(hook.start, st);
  const hipError_t e = launch_bits(bits, bwd, a, st);
  if (hook.stop) (void)hipEventRecord(hook.stop, st);
  return e;
}

// Plain bf16 x bf16^T product  out[z][M][N] = a_tail[M, Kz] . b_tail[N, Kz]^T  with the K
// range split over `ksplit` slices (partial sums, reduced by the caller in a fixed order).
hipError_t launch_gemm_plain(const GemmArgs& a, int ksplit, hipStream_t st) {
  return launch_cfg<4, false, 64, 128, 2, 4, false>(a, ksplit, st);
}

}  // namespace qalora
