// The dense contractions of the QA-LoRA linear on the matrix cores of gfx950:
//
//   forward   y  = x  . W~'        K = D_in,  N = D_out
//   backward  dx = dy . W~'^T      K = D_out, N = D_in
//
// with W~'[i,j] = alpha[i/g,j] * code[i,j] + beta'[i/g,j] (Eq. 1 per group, Sec. 3.3)
// rebuilt on the fly: packed codes are read with 128-bit loads, dequantised in registers
// with packed 16-bit fma, staged in LDS and fed to v_mfma_f32_32x32x16 with fp32
// accumulation.
//
// The factors arrive as one 32-bit word per (group, column), prepared once per call by the
// front launch: fp16(alpha S) in the low half and fp16((beta' + mid alpha) S) in the high half,
// where beta' = beta + (s/g) A B already holds the adapter (App. B.3: the adapted layer IS the
// quantized layer with these zero factors, so the dense kernels need no separate low-rank
// branch), mid = 2^(N-1) is the code the weight is evaluated around, and S is a power of two
// -- per output column in the forward direction, one for the call in the backward direction --
// that brings the largest factor to about 2^13, so that the fp16 conversion keeps 11
// significant bits whatever the magnitude of the weights.  The epilogue divides it out again.
//
// Operand precision.  The main K steps run the matrix cores in fp16 (same rate as bf16 on
// gfx950): W~ keeps 11 significant bits instead of 8, which is what keeps the result inside
// the 2e-3 parity bar for every bit width (with bf16 operands the 4-level INT2 grids land
// on 2.1e-3).  The activations arrive here already converted: every token row scaled by a
// power of two that brings its largest magnitude into [2^14, 2^15) and written as fp16
// (exact for bf16 inputs); the output row is scaled back in the epilogue.
//
// The same kernel without the dequantising part (HAS_MAIN = false) is a plain bf16 product over
// "tail" operands; the adapter gradients use it for dU = s dy B^T with B split into bf16 hi + lo
// parts, which keeps fp32-level accuracy and bf16's range for gradients.
//
// One kernel serves both directions from ONE packed copy of the codes: a thread owns half
// of an 8x8 patch of codes, from which it emits four K-contiguous operand fragments along
// either axis -- down the rows (forward, K = input rows) or across the columns (backward,
// K = output columns).
//
// Tiling: 512 threads = 8 wavefronts (two per SIMD), block tile BM x BN x 64.  The A tile
// goes global -> LDS directly (128-bit buffer LDS-DMA loads, no registers), three stages deep;
// the B tile goes through two alternating register sets for dequantisation into two LDS
// stages.  Vector instructions do not hide under matrix instructions on this target (they
// share the issue cycles of the SIMD), so the producer is kept as short as it can be and is
// spread between the matrix instructions of the step before; one barrier per step, placed
// so that the next step's first operand fragments are already in registers when it starts.
// Loads stay in flight across the barrier (counted s_waitcnt).  LDS rows are 128 bytes,
// XOR-swizzled so that operand reads (16 consecutive rows, one 16-byte chunk) and all
// producers' writes are bank-conflict free.  The epilogue transposes through LDS.
#include <type_traits>

#include <hip/hip_ext.h>

#include "common.hpp"
#include "kernels.hpp"

namespace qalora {

constexpr int BK = 64;
constexpr int NT = 512;  // threads per block

// Measurement aid: -DQALORA_ABLATE=n builds the dequantising kernels with one part of their work
// taken away, to see what that part costs.  The results are WRONG on purpose; every access stays
// in bounds and every wait still ends.  (Such a build is for the benchmark's --library option,
// never for the tests.)
//   1  the producer dequantises every second column only (half the vector work, half the B writes)
//   2  a quarter of the A tile's LDS-DMA loads
//   3  the A tile always comes from the first 256 elements of K (served by L2 after the first pass)
//   4  half of the A operand fragments are read from LDS, the others reuse them
//   5  as 4, and one B fragment is read instead of all
//   6  no block barrier in the K step
//   7  no wait for the A tile in the K step
#ifndef QALORA_ABLATE
#define QALORA_ABLATE 0
#endif

// Raw buffer resources: loads through them return zero past `bytes`, which is how every
// ragged edge (rows past M, patches past the matrix) is zero-filled without branches.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, size_t bytes) {
  const uint32_t n = bytes > 0xffffffffull ? 0xffffffffu : (uint32_t)bytes;
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)n, 0x00020000);
}
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));  // register-resident 128-bit values
__device__ __forceinline__ u32x4_t buf_load128(__amdgpu_buffer_rsrc_t r, uint32_t byte_off) {
  return __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, 0);
}
constexpr uint32_t kOobOffset = 0xffff0000u;  // past any buffer (also after a small add): reads zero

// Byte offset inside a [rows][64 x 16-bit] tile of the 16-byte chunk `c` of row `n`.
// Two rows share a 256-byte line (half = which 128 bytes); the chunk slot is XORed with row
// bits.  With n = b7..b0:  half = b0^b2^b3^b4,  slot = c ^ (b1 | b2<<1 | b3<<2).
// Operand reads (16 consecutive rows at one chunk) see 16 distinct (half, slot); every
// producer writes whole 128-byte rows from 8 adjacent lanes, with the next 8 lanes (row n+1,
// n+4 or n+8) landing in the other half.  Rows 32 apart share the pattern, so the fragment
// reads of a wave differ only by an immediate offset.
__device__ __forceinline__ int swz_offset(int n, int c) {
  const int half = (n ^ (n >> 2) ^ (n >> 3) ^ (n >> 4)) & 1;
  const int f = (n >> 1) & 7;
  return ((n >> 1) << 8) | (half << 7) | ((c ^ f) << 4);
}
// Inverse for the LDS-DMA path: which (row, chunk) lives at byte offset `o` (multiple of 16).
__device__ __forceinline__ void swz_inverse(int o, int& n, int& c) {
  const int pair = o >> 8, half = (o >> 7) & 1, slot = (o >> 4) & 7;
  const int b2 = (pair >> 1) & 1, b3 = (pair >> 2) & 1, b4 = (pair >> 3) & 1;
  n = 2 * pair + (half ^ b2 ^ b3 ^ b4);
  c = slot ^ (pair & 7);
}

// Block-index -> tile-index map.  Consecutive block ids are dealt round-robin to the 8
// XCDs, each with its own L2; give every XCD a contiguous run of tiles (tile_m fastest)
// so that the weight panels and activation rows it touches stay in that L2.
__device__ __forceinline__ int xcd_remap(int bid, int nblocks) {
  if (nblocks % 8 != 0) return bid;
  return (bid % 8) * (nblocks / 8) + bid / 8;
}

// LDS-DMA loads stay in flight across barriers (three A stages), so the barrier is issued
// raw -- the compiler would otherwise drain every counter in front of it -- with explicit
// waits: all of this wave's LDS writes, and all but the newest `VM_KEEP` vector-memory ops.
template <int VM_KEEP>
__device__ __forceinline__ void wait_and_barrier() {
  static_assert(VM_KEEP >= 0 && VM_KEEP < 64, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(VM_KEEP) : "memory");
}

// Calls f with the four LDS regions of one pipeline step as restrict-qualified parameters:
// the region the LDS-DMA is filling, the A and B regions being read, and the B region being
// written never overlap within a step, and saying so keeps the compiler from draining the
// LDS-DMA loads before every LDS read.
template <typename F>
__device__ __forceinline__ void with_step_regions(uint16_t* __restrict__ a_dma,
                                                  const uint16_t* __restrict__ a_rd,
                                                  const uint16_t* __restrict__ b_rd,
                                                  uint16_t* __restrict__ b_wr, F&& f) {
  f(a_dma, a_rd, b_rd, b_wr);
}
// Main pipeline: additionally the A stage of the next step (read at the end of the step).
template <typename F>
__device__ __forceinline__ void with_step_regions(uint16_t* __restrict__ a_dma,
                                                  const uint16_t* __restrict__ a_rd,
                                                  const uint16_t* __restrict__ a_nx,
                                                  const uint16_t* __restrict__ b_rd,
                                                  uint16_t* __restrict__ b_wr, F&& f) {
  f(a_dma, a_rd, a_nx, b_rd, b_wr);
}

// A stages of the LDS-DMA pipeline.  Three (the tile of step it+3 is requested as soon as step it
// has released its stage), except for the 64-row tile of the dequantising product: with two
// stages its LDS is 80 KB, so that two blocks fit a compute unit and cover each other's waits
// -- a K step of that tile is mostly producer work and synchronisation, not matrix work.
constexpr int gemm_a_stages(int bm, bool has_main) { return (has_main && bm == 64) ? 2 : 3; }
// wavefronts per SIMD the kernel is compiled for (two blocks of the 64-row tile: four, i.e. 128
// registers; the 3-bit backward producer with per-step edge handling does not fit them and
// stays at one block per unit)
constexpr int gemm_min_waves(int bm, bool has_main, int nbits, bool bwd, bool fast) {
  return (has_main && bm == 64 && !(nbits == 3 && bwd && !fast)) ? 4 : 1;
}

// HAS_MAIN = false: a plain bf16 x bf16^T product over the "tail" operands only (used for
// dU = s dy B^T), optionally split along K over blockIdx.y.
//
// FAST = true (main K a multiple of 64, group size dividing or divisible by 64, activation
// copies padded to whole row tiles): every per-lane global offset is a kernel-lifetime
// constant and the K advance lives in scalar offsets, so the hot loop carries no vector
// address arithmetic.  FAST = false keeps per-step, per-lane offsets with full edge handling.
template <int NBITS, bool BWD, int BM, int BN, int WAVES_M, int WAVES_N, bool HAS_MAIN, bool FAST>
__global__ __launch_bounds__(NT, gemm_min_waves(BM, HAS_MAIN, NBITS, BWD, FAST)) void gemm_dq_kernel(const GemmArgs p) {
  static_assert(!FAST || HAS_MAIN, "the fast addressing path is for the dequantising product");
  static_assert(WAVES_M * WAVES_N == 8, "eight wavefronts per block");
  static_assert(!HAS_MAIN || BN == 256, "the dequantising producer assumes 256 columns");
  constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  static_assert(TM >= 1 && TN >= 1, "wave tile must hold at least one 32x32 MFMA tile");
  constexpr int A_LOADS = (QALORA_ABLATE == 2 && HAS_MAIN) ? 1 : BM * 8 / NT;  // LDS-DMA loads per thread
  constexpr int B_CHUNKS = (BN * 8 / NT) > 0 ? BN * 8 / NT : 1;  // plain B tile, per thread
  static_assert(A_LOADS >= 1, "BM too small for 512 threads");
  constexpr int A_TILE = BM * 64;  // 16-bit elements per A buffer
  constexpr int B_TILE = BN * 64;
  constexpr int A_STAGES = gemm_a_stages(BM, HAS_MAIN);  // LDS-DMA prefetch runs A_STAGES - 1 K steps ahead

  extern __shared__ __align__(1024) uint16_t smem[];
  // The B stages sit at the bottom: their offsets then fit the 16-bit immediate of the LDS
  // instructions for either parity, so the producer's writes and the operand reads of B need no
  // address arithmetic in the loop (the A stage rotates through three, so its base is a register).
  uint16_t* Bs = smem;               // [2][BN][64] swizzled
  uint16_t* As = smem + 2 * B_TILE;  // [A_STAGES][BM][64] swizzled

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, lives in an SGPR
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;

  const int tiles_m = ceil_div(p.M, BM);
  const int tiles_n = ceil_div(p.N, BN);
  // Each XCD gets a contiguous run of tile ids, and ids walk bands of kGroupM row tiles across
  // all column tiles: the 32 blocks resident on one XCD then share kGroupM activation row
  // panels and 32 / kGroupM weight column panels in that XCD's L2.
  const int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n);
  constexpr int kGroupM = 4;
  const int band = tile / (kGroupM * tiles_n);
  const int band_rows = min(kGroupM, tiles_m - band * kGroupM);
  const int in_band = tile - band * kGroupM * tiles_n;
  const int m0 = (band * kGroupM + in_band % band_rows) * BM;
  const int n0 = (in_band / band_rows) * BN;

  const int nk_main = HAS_MAIN ? ceil_div(p.K_main, BK) : 0;
  const int nk_tail = HAS_MAIN ? 0 : ceil_div(p.K_tail, BK);  // a plain product has only these
  // blockIdx.y splits the K range (partial sums, added by a later launch in a fixed order)
  int it_begin = 0, it_end = nk_main + nk_tail;
  if (gridDim.y > 1) {
    const int per = ceil_div(it_end, (int)gridDim.y);
    it_begin = blockIdx.y * per;
    it_end = min(it_end, it_begin + per);
  }

  // measurement aid: the first block reports how many shader cycles and wall-clock ticks it
  // lived for (their ratio is the clock the chip actually ran this kernel at)
  const bool probe = HAS_MAIN && p.clock_probe != nullptr && blockIdx.x == 0 && blockIdx.y == 0 &&
                     tid == 0;
  if (probe) {
    p.clock_probe[0] = (unsigned long long)clock64();
    p.clock_probe[1] = (unsigned long long)wall_clock64();
  }
  // measurement aid: every block reports when it started, left the K loop and ended, and on
  // which XCD (register XCC_ID, bits 3:0), so that the launch can be laid out on a time line
  const bool timeline = HAS_MAIN && p.block_times != nullptr && blockIdx.y == 0 && tid == 0 &&
                        (int)blockIdx.x < p.block_times_cap;
  if (timeline) {
    p.block_times[4 * blockIdx.x + 0] = (unsigned long long)wall_clock64();
    p.block_times[4 * blockIdx.x + 3] = (unsigned long long)__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11));
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
  const __amdgpu_buffer_rsrc_t rs_a_main = make_rsrc(
      p.a_main, HAS_MAIN ? (size_t)(FAST ? round_up(p.M, BM) : p.M) * p.lda_main * 2 : 0);
  const __amdgpu_buffer_rsrc_t rs_a_tail = make_rsrc(p.a_tail, (size_t)p.M * p.lda_tail * 2);
  uint32_t a_row[A_LOADS];  // global row of each load (rows past M read as zero)
  int a_chunk8[A_LOADS];
#pragma unroll
  for (int q = 0; q < A_LOADS; ++q) {
    int n, c;
    swz_inverse((q * 8 + wave) * 1024 + lane * 16, n, c);
    a_row[q] = (uint32_t)(m0 + n);
    a_chunk8[q] = 8 * c;
  }
  // fast path: one lane offset for all loads of the kernel (rows of later loads are 64*q
  // further down; the copies are padded to whole tiles, so no row check is needed)
  const uint32_t a_voff_main = (a_row[0] * (uint32_t)p.lda_main + (uint32_t)a_chunk8[0]) * 2u;
  // `live` = false (a step past the end of the K range): same number of loads, aimed outside
  // the buffer, so the in-flight count the waits rely on does not depend on the position.
  auto issue_a = [&](auto kind, int it, uint16_t* a_dst, bool live) {
    constexpr bool kMain = decltype(kind)::value == 0;
    const int k0 = kMain ? (it - nk_tail) * BK : it * BK;
    if constexpr (FAST && kMain) {
      // branch-free on purpose: OR-ing the mask into a valid offset puts it past any buffer
      // (the range check looks at the vector offset alone, whatever the scalar offset is).
      // A branch around a load would make the compiler's count of loads in flight -- and with
      // it every wait it inserts for the code registers -- one too strict.
      const uint32_t voff = a_voff_main | (live ? 0u : kOobOffset);
#pragma unroll
      for (int q = 0; q < A_LOADS; ++q) {
        const uint32_t soff = (uint32_t)(QALORA_ABLATE == 3 ? (k0 & 255) : k0) * 2u +
                              (uint32_t)q * 64u * (uint32_t)p.lda_main * 2u;
        uint16_t* dst = a_dst + (q * 8 + wave) * 512;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_a_main,
                                                 (__attribute__((address_space(3))) void*)dst, 16,
                                                 (int)voff, (int)soff, 0, 0);
      }
      return;
    }
    const int klim = kMain ? p.K_main : p.K_tail;
    const uint32_t lda = kMain ? p.lda_main : p.lda_tail;
#pragma unroll
    for (int q = 0; q < A_LOADS; ++q) {
      const int k = k0 + a_chunk8[q];
      const uint32_t off = (live && k < klim && a_row[q] < (uint32_t)p.M)
                               ? (a_row[q] * lda + (uint32_t)k) * 2u
                               : kOobOffset;
      uint16_t* dst = a_dst + (q * 8 + wave) * 512;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(kMain ? rs_a_main : rs_a_tail,
                                               (__attribute__((address_space(3))) void*)dst, 16,
                                               (int)off, 0, 0, 0);
    }
  };

  // ---- B tile through registers --------------------------------------------------------
  // MAIN steps: half an 8x8 patch of codes per thread.
  //   forward : u0 = K chunk, cq = column quad (8 adjacent lanes fill one 128-byte LDS row)
  //   backward: u0 = K chunk (column octet), u1 = row block, hb = which two row pairs
  // Out-of-range patches are read from a clamped address and get alpha = beta = 0.
  const int f_u0 = tid & 7, f_cq = tid >> 3;
  const int b_u0 = tid & 7, b_u1 = (tid >> 3) & 31, b_hb = tid >> 8;
  constexpr int RB0 = PackFmt<NBITS>::kRowsPerWord0;
  // Codes, alpha and beta come through buffer loads; a patch outside the matrix gets
  // alpha = beta = 0 (so W~ = 0) by pointing its factor loads past the buffer.
  const size_t n_groups = (size_t)(p.d_in / (p.group > 0 ? p.group : 1));
  const __amdgpu_buffer_rsrc_t rs_p0 =
      make_rsrc(p.plane0, HAS_MAIN ? plane0_words(NBITS, p.d_in, p.d_out) * 4 : 0);
  const __amdgpu_buffer_rsrc_t rs_p1 =
      make_rsrc(p.plane1, HAS_MAIN ? plane1_words(NBITS, p.d_in, p.d_out) * 4 : 0);
  const __amdgpu_buffer_rsrc_t rs_fc = make_rsrc(p.fac, HAS_MAIN ? n_groups * p.d_out * 4 : 0);
  const __amdgpu_buffer_rsrc_t rs_bt = make_rsrc(
      p.b_tail, (size_t)(BWD ? (int)n_groups : p.N) * p.K_tail * 2);
  const int f_j0 = n0 + 4 * f_cq;   // forward: this thread's 4 columns
  const int b_i0 = n0 + 8 * b_u1;   // backward: this thread's row block
  const bool n_valid = BWD ? (b_i0 < p.d_in) : (f_j0 < p.d_out);

  // Two register sets: the set of step it+1 is being dequantised while the set of step it+2
  // is loading (its loads then have a whole K step to land).
  u32x4_t bregs[2][4];   // fwd: codes, factor words, -, plane-1 codes | bwd: 2 codes, 2 factor words
  u32x4_t bregs1[2][2];  // bwd, N = 3: plane-1 words
  u32x4_t btail[B_CHUNKS];
  using Set0 = std::integral_constant<int, 0>;
  using Set1 = std::integral_constant<int, 1>;

  // fast path: lane-constant offsets (patches outside the matrix point past the buffers)
  uint32_t fb_voff_p0_c = 0, fb_voff_p1_c = 0, fb_voff_ab_c = 0;
  int fb_grp_small = 0;  // forward, g < 64: groups per K step; else 0
  if constexpr (FAST) {
    if constexpr (!BWD) {
      fb_voff_p0_c = n_valid ? ((uint32_t)((8 * f_u0) / RB0) * p.d_out + f_j0) * 4u : kOobOffset;
      fb_voff_p1_c = n_valid ? ((uint32_t)((8 * f_u0) / 32) * p.d_out + f_j0) * 4u : kOobOffset;
      fb_grp_small = p.group < BK ? BK / p.group : 0;
      const uint32_t lane_grp = p.group < BK ? (uint32_t)(8 * f_u0) / (uint32_t)p.group : 0u;
      fb_voff_ab_c = n_valid ? (lane_grp * p.d_out + f_j0) * 4u : kOobOffset;
    } else {
      fb_voff_p0_c = n_valid ? ((uint32_t)(b_i0 / RB0) * p.d_out + 8 * b_u0) * 4u : kOobOffset;
      fb_voff_p1_c = n_valid ? ((uint32_t)(b_i0 / 32) * p.d_out + 8 * b_u0) * 4u : kOobOffset;
      fb_voff_ab_c = n_valid ? ((uint32_t)(b_i0 / p.group) * p.d_out + 8 * b_u0) * 4u : kOobOffset;
    }
  }
  auto buf_load128_s = [&](__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) -> u32x4_t {
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, (int)soff, 0);
  };

  auto gload_b = [&](auto kind, int it, auto set, bool live) {
    constexpr bool kMain = decltype(kind)::value == 0;
    u32x4_t(&breg)[4] = bregs[decltype(set)::value];
    u32x4_t(&breg1)[2] = bregs1[decltype(set)::value];
    if constexpr (kMain && FAST) {
      const uint32_t km = (uint32_t)(it - nk_tail);  // main step index (uniform)
      const uint32_t dead = live ? 0u : kOobOffset;   // branch-free, as for the A tile
      const uint32_t fb_voff_p0 = fb_voff_p0_c | dead;
      const uint32_t fb_voff_p1 = fb_voff_p1_c | dead;
      const uint32_t fb_voff_ab = fb_voff_ab_c | dead;
      if constexpr (!BWD) {
        // scalar parts: word rows advance by 64/RB per step, group rows by 64/g (or 1 per g/64)
        const uint32_t s_p0 = km * (uint32_t)(BK / RB0) * p.d_out * 4u;
        const uint32_t grp = fb_grp_small ? km * (uint32_t)fb_grp_small
                                          : km / (uint32_t)(p.group / BK);
        const uint32_t s_ab = grp * p.d_out * 4u;
        breg[0] = buf_load128_s(rs_p0, fb_voff_p0, s_p0);
        if constexpr (NBITS == 3)
          breg[3] = buf_load128_s(rs_p1, fb_voff_p1, km * (uint32_t)(BK / 32) * p.d_out * 4u);
        breg[1] = buf_load128_s(rs_fc, fb_voff_ab, s_ab);
      } else {
        const uint32_t s_k = km * (uint32_t)BK * 4u;  // 64 columns further along the row
        breg[0] = buf_load128_s(rs_p0, fb_voff_p0, s_k);
        breg[1] = buf_load128_s(rs_p0, fb_voff_p0 + 16, s_k);
        if constexpr (NBITS == 3) {
          breg1[0] = buf_load128_s(rs_p1, fb_voff_p1, s_k);
          breg1[1] = buf_load128_s(rs_p1, fb_voff_p1 + 16, s_k);
        }
        breg[2] = buf_load128_s(rs_fc, fb_voff_ab, s_k);
        breg[3] = buf_load128_s(rs_fc, fb_voff_ab + 16, s_k);
      }
    } else if constexpr (kMain) {
      const int k0 = (it - nk_tail) * BK;
      if constexpr (!BWD) {
        const int i0 = k0 + 8 * f_u0;
        const bool ok = live && n_valid && i0 < p.d_in;
        breg[0] = buf_load128(rs_p0, ok ? ((uint32_t)(i0 / RB0) * p.d_out + f_j0) * 4u : kOobOffset);
        if constexpr (NBITS == 3)
          breg[3] = buf_load128(rs_p1, ok ? ((uint32_t)(i0 / 32) * p.d_out + f_j0) * 4u : kOobOffset);
        const uint32_t ab = ok ? ((uint32_t)(i0 / p.group) * p.d_out + f_j0) * 4u : kOobOffset;
        breg[1] = buf_load128(rs_fc, ab);
      } else {
        const int j0 = k0 + 8 * b_u0;
        const bool ok = live && n_valid && j0 < p.d_out;
        const uint32_t w = ok ? ((uint32_t)(b_i0 / RB0) * p.d_out + j0) * 4u : kOobOffset;
        breg[0] = buf_load128(rs_p0, w);
        breg[1] = buf_load128(rs_p0, w + 16);
        if constexpr (NBITS == 3) {
          const uint32_t w1 = ok ? ((uint32_t)(b_i0 / 32) * p.d_out + j0) * 4u : kOobOffset;
          breg1[0] = buf_load128(rs_p1, w1);
          breg1[1] = buf_load128(rs_p1, w1 + 16);
        }
        const uint32_t ab = ok ? ((uint32_t)(b_i0 / p.group) * p.d_out + j0) * 4u : kOobOffset;
        breg[2] = buf_load128(rs_fc, ab);
        breg[3] = buf_load128(rs_fc, ab + 16);
      }
    } else {
      const int k0 = it * BK;
#pragma unroll
      for (int q = 0; q < B_CHUNKS; ++q) {
        const int idx = tid + NT * q;
        const int row = idx >> 3, ch = idx & 7;
        const int n = n0 + row;
        // forward tail: row n of B~^T; backward tail: row n/g of A~ (the unpooling of
        // the pooled gradient is this broadcast over the g rows of a group)
        const int src_row = BWD ? n / p.group : n;
        const int k = k0 + 8 * ch;
        const bool ok = live && row < BN && n < p.N && k < p.K_tail;
        btail[q] = buf_load128(rs_bt, ok ? ((uint32_t)src_row * p.K_tail + k) * 2u : kOobOffset);
      }
    }
  };

  // The fp16 factors of one (group, column), as the front launch left them: W~ S = (alpha S) *
  // (c - mid) + (beta' + mid alpha) S with mid = 2^(N-1).  Written around the mid code, the
  // constant term is the group's mid value instead of its minimum: it is several times smaller
  // for a group that straddles zero, and so is its fp16 rounding error, the one error of this
  // path that is the same for every row of a group and therefore adds up along K instead of
  // averaging out.
  auto ab_pair = [&](uint32_t word) { return __builtin_bit_cast(f16x2, word); };
  // extraction constants held in registers (see patch_code_pair_f16)
  uint32_t dq_mask = patch_code_mask<NBITS>(), dq_magic = 0x64006400u;
  if constexpr (NBITS != 3) {  // (the 3-bit extraction has a second plane and no such fusion)
    asm volatile("s_mov_b32 %0, %1" : "=s"(dq_mask) : "n"(patch_code_mask<NBITS>()));
    asm volatile("v_mov_b32 %0, 0x64006400" : "=v"(dq_magic));
  }
  auto dq_pair = [&](uint32_t w0s, uint32_t w1s, f16x2 ab, int m) {
    const f16x2 a2 = {ab.x, ab.x};
    const f16x2 b2 = {ab.y, ab.y};
    const f16x2 cc = patch_code_pair_f16<NBITS>(w0s, w1s, m, dq_mask, dq_magic);
    return __builtin_bit_cast(uint32_t, cc * a2 + b2);
  };

  // Dequantise the register set `set` of step `it` into the B stage b_dst.  The work is cut in
  // three pieces (piece = 0..2, or -1 for all of it) so that it can be spread over the first
  // three K-16 slices of the matrix-core work of the step before.
  uint32_t wt[8][2];  // backward: [column][row pair] (W~[2m][c], W~[2m+1][c]), kept across pieces
  auto store_b = [&](auto kind, int it, uint16_t* b_dst, auto set, auto piece_c) {
    constexpr bool kMain = decltype(kind)::value == 0;
    constexpr int piece = decltype(piece_c)::value;
    u32x4_t(&breg)[4] = bregs[decltype(set)::value];
    u32x4_t(&breg1)[2] = bregs1[decltype(set)::value];
    char* bs = reinterpret_cast<char*>(b_dst);
    if constexpr (kMain) {
      if constexpr (!BWD) {
        const int i0 = (it - nk_tail) * BK + 8 * f_u0;
        const int sh0 = patch_preshift0<NBITS>(i0), sh1 = patch_preshift1(i0);
        const uint32_t w0[4] = {breg[0].x, breg[0].y, breg[0].z, breg[0].w};
        const uint32_t w1[4] = {breg[3].x, breg[3].y, breg[3].z, breg[3].w};
        const uint32_t fc[4] = {breg[1].x, breg[1].y, breg[1].z, breg[1].w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          if (piece >= 0 && (piece == 2 ? c < 2 : c != piece)) continue;  // columns {0}, {1}, {2, 3}
          if (QALORA_ABLATE == 1 && (c & 1)) continue;
          const uint32_t w0s = w0[c] >> sh0;
          const uint32_t w1s = (NBITS == 3) ? (w1[c] >> sh1) : 0u;
          const f16x2 ab = ab_pair(fc[c]);
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
        const uint32_t fc[8] = {breg[2].x, breg[2].y, breg[2].z, breg[2].w,
                                breg[3].x, breg[3].y, breg[3].z, breg[3].w};
        // pieces 0 and 1 dequantise columns 0-3 and 4-7; piece 2 gathers and writes
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          if (piece >= 0 && c / 4 != piece) continue;
          if (QALORA_ABLATE == 1 && (c & 1)) {
            wt[c][0] = wt[c - 1][0];
            wt[c][1] = wt[c - 1][1];
            continue;
          }
          const uint32_t w0s = w0[c] >> sh0;
          const uint32_t w1s = (NBITS == 3) ? (w1[c] >> sh1) : 0u;
          const f16x2 ab = ab_pair(fc[c]);
          wt[c][0] = dq_pair(w0s, w1s, ab, 0);
          wt[c][1] = dq_pair(w0s, w1s, ab, 1);
        }
        if (piece >= 0 && piece != 2) return;
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
      static_assert(piece < 0, "tail tiles are copied in one go");
#pragma unroll
      for (int q = 0; q < B_CHUNKS; ++q) {
        const int idx = tid + NT * q;
        const int row = idx >> 3, ch = idx & 7;
        if (row < BN) *reinterpret_cast<u32x4_t*>(bs + swz_offset(row, ch)) = btail[q];
      }
    }
  };
  using AllPieces = std::integral_constant<int, -1>;

  // ---- LDS -> matrix cores ---------------------------------------------------------
  // lane (r = lane % 32, kb = lane / 32) reads chunk 2*kk + kb of rows base + 32*t + r.  The
  // swizzle repeats every 32 rows, so one lane offset (XORed with the chunk) serves every
  // 32-row tile of the wave through the instruction's immediate offset.
  static_assert(BK == 64, "four K-16 slices per step");
  constexpr int kSideValuPerMfma = 5;  // side-work VALU instructions slotted behind each MFMA
  const int a_lane = swz_offset(wm * WTM + (lane & 31), 0);
  const int b_lane = swz_offset(wn * WTN + (lane & 31), 0);

  // `side(kk)` is extra work issued in the shadow of the matrix-core instructions of slice kk.
  auto compute = [&](auto kind, const uint16_t* a_src, const uint16_t* b_src, auto&& side) {
    constexpr bool kMain = decltype(kind)::value == 0;
    const char* as = reinterpret_cast<const char*>(a_src);
    const char* bs = reinterpret_cast<const char*>(b_src);
    uint4 af[2][TM], bf[2][TN];
    auto load_frags = [&](int kk, int slot) {
      const int cx = (2 * kk + (lane >> 5)) << 4;
      const char* ap = as + (a_lane ^ cx);
      const char* bp = bs + (b_lane ^ cx);
#pragma unroll
      for (int a = 0; a < TM; ++a) af[slot][a] = *reinterpret_cast<const uint4*>(ap + a * 4096);
#pragma unroll
      for (int b = 0; b < TN; ++b) bf[slot][b] = *reinterpret_cast<const uint4*>(bp + b * 4096);
    };
    load_frags(0, 0);
    auto slice = [&](auto kk_c) {
      constexpr int kk = decltype(kk_c)::value;
      constexpr int cur = kk & 1;
      if (kk + 1 < BK / 16) load_frags(kk + 1, cur ^ 1);  // next slice in flight under the MFMAs
      side(kk_c);
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
      // one matrix-core instruction, then whatever else is ready (LDS reads of the next
      // slice, the side work), eight times over; nothing crosses into the next slice
#pragma unroll
      for (int i = 0; i < TM * TN; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // LDS read
        __builtin_amdgcn_sched_group_barrier(0x002, kSideValuPerMfma, 0);  // VALU
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    slice(std::integral_constant<int, 0>{});
    slice(std::integral_constant<int, 1>{});
    slice(std::integral_constant<int, 2>{});
    slice(std::integral_constant<int, 3>{});
  };
  auto no_side = [](auto) {};

  // Main-pipeline variant.  The fragment registers live across steps: slices 0-2 carry the
  // side work (the dequantisation of the next step, one piece each), then the block
  // synchronises, and slice 3 runs while the first fragments of the NEXT step are fetched
  // from the stages that barrier has just published -- so a step starts on the matrix cores
  // at once instead of waiting for an LDS round trip.
  constexpr int kMainB = BWD ? (NBITS == 3 ? 6 : 4) : (NBITS == 3 ? 3 : 2);
  // see the main step below (two stages: only the registers of it+2 were requested after A(it+1))
  constexpr int kMidKeep = A_STAGES == 2 ? kMainB : kMainB + A_LOADS + kMainB;
  uint4 maf[2][TM], mbf[2][TN];
  auto load_frags_main = [&](const uint16_t* a_src, const uint16_t* b_src, int kk, auto slot_c) {
    constexpr int slot = decltype(slot_c)::value;
    const int cx = (2 * kk + (lane >> 5)) << 4;
    const char* ap = reinterpret_cast<const char*>(a_src) + (a_lane ^ cx);
    const char* bp = reinterpret_cast<const char*>(b_src) + (b_lane ^ cx);
    constexpr int kReadA = (QALORA_ABLATE == 4 || QALORA_ABLATE == 5) ? (TM + 1) / 2 : TM;
    constexpr int kReadB = (QALORA_ABLATE == 5) ? 1 : TN;
#pragma unroll
    for (int a = 0; a < TM; ++a)
      maf[slot][a] = a < kReadA ? *reinterpret_cast<const uint4*>(ap + a * 4096) : maf[slot][a - kReadA];
#pragma unroll
    for (int b = 0; b < TN; ++b)
      mbf[slot][b] = b < kReadB ? *reinterpret_cast<const uint4*>(bp + b * 4096) : mbf[slot][0];
  };
  auto compute_main = [&](const uint16_t* a_rd, const uint16_t* b_rd, const uint16_t* a_nx,
                          const uint16_t* b_nx, auto&& side, auto&& after_barrier) {
    auto slice = [&](auto kk_c) {
      constexpr int kk = decltype(kk_c)::value;
      constexpr int cur = kk & 1;
      using Nxt = std::integral_constant<int, cur ^ 1>;
      if constexpr (kk < 3) {
        load_frags_main(a_rd, b_rd, kk + 1, Nxt{});
        side(kk_c);
      } else {
        load_frags_main(a_nx, b_nx, 0, Nxt{});
      }
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
              __builtin_bit_cast(f16x8, maf[cur][a]), __builtin_bit_cast(f16x8, mbf[cur][b]),
              acc[a][b], 0, 0, 0);
#pragma unroll
      for (int i = 0; i < TM * TN; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // LDS read
        __builtin_amdgcn_sched_group_barrier(0x002, kSideValuPerMfma, 0);  // VALU
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    slice(std::integral_constant<int, 0>{});
    slice(std::integral_constant<int, 1>{});
    slice(std::integral_constant<int, 2>{});
    // this wave's LDS writes (next B stage) and reads (fragments of slice 3) are done
    // ... and its share of A(it+1) has landed: the loads issued since (registers of it+2, A(it+2),
    // registers... see the step) may stay in flight
    if constexpr (QALORA_ABLATE == 6)
      asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(kMidKeep) : "memory");
    else if constexpr (QALORA_ABLATE == 7)
      asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else
      asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(kMidKeep) : "memory");
    after_barrier();
    __builtin_amdgcn_sched_barrier(0);
    slice(std::integral_constant<int, 3>{});
  };

  // Vector-memory ops per thread of one B-register load, per step kind (for the waits).
  constexpr int kBLoadsMain = BWD ? (NBITS == 3 ? 6 : 4) : (NBITS == 3 ? 3 : 2);
  constexpr int kBLoadsTail = B_CHUNKS;

  if constexpr (HAS_MAIN) {
    // Main steps.  K step `it` in pipeline slot `slot` (A stage slot % 3, B stage and register
    // set slot % 2, the parity `par` being a compile-time constant):
    //   entry : A(it), B(it) visible in LDS; the LDS-DMA of A(it+1), A(it+2) and the register
    //           loads of step it+1 (set par^1) are in flight or done
    //   1. start the register loads of step it+2 (set par)
    //   2. slices 0-2 on the matrix cores; between them, piece by piece, the registers of it+1
    //      (the compiler waits for exactly those) are dequantised into the other B stage
    //   3. wait until A(it+1) has landed -- issued since: registers it+1... the three newest
    //      groups (registers of it+1's successor, A(it+2), registers of it+2) may stay in
    //      flight -- then barrier
    //   4. start the LDS-DMA of A(it+3) into the stage of A(it), which nobody reads any more
    //   5. slice 3, fetching the first fragments of step it+1
    const int pb = it_begin, pe = it_end;
    // (The 3-bit backward producer of the 256-row tile holds two code planes and has no
    // registers left for a second set: it keeps ONE set and reloads it in slice 2, as soon as
    // the dequantisation has read it -- half a step of lead instead of a whole one.)
    constexpr bool kSingleSet = (NBITS == 3 && BWD && BM == 256);
    // Steps past the end of the K range still issue their loads (the waits count them).  On the
    // fast path they re-read the last step, which is valid memory and never used; elsewhere they
    // are aimed outside the buffers.
    auto at = [&](int i) { return FAST ? min(i, pe - 1) : i; };
    auto live = [&](int i) { return FAST ? true : i < pe; };
    // a_cur / a_next / a_dma2: the A stages holding steps it, it+1 and it+2 (the caller rotates them)
    auto step = [&](int it, uint16_t* a_cur, uint16_t* a_next, uint16_t* a_dma2, auto par) {
      constexpr int kPar = decltype(par)::value;
      using SetCur = std::integral_constant<int, kSingleSet ? 0 : kPar>;
      using SetNext = std::integral_constant<int, kSingleSet ? 0 : (kPar ^ 1)>;
      with_step_regions(
          a_dma2, a_cur, a_next, Bs + kPar * B_TILE,
          Bs + (kPar ^ 1) * B_TILE,
          [&](uint16_t*, const uint16_t* a_rd, const uint16_t* a_nx, const uint16_t* b_rd,
              uint16_t* b_wr) {
            if constexpr (!kSingleSet) gload_b(MainK{}, at(it + 2), SetCur{}, live(it + 2));
            __builtin_amdgcn_sched_barrier(0);
            compute_main(
                a_rd, b_rd, a_nx, b_wr,
                [&](auto kk) {
                  store_b(MainK{}, it + 1, b_wr, SetNext{}, kk);
                  if constexpr (kSingleSet && decltype(kk)::value == 2)
                    gload_b(MainK{}, at(it + 2), SetCur{}, live(it + 2));
                },
                [&]() { issue_a(MainK{}, at(it + A_STAGES), a_cur, live(it + A_STAGES)); });
          });
    };
    if (pe > pb) {
      // prologue: A(pb), A(pb+1), A(pb+2) in flight, registers of pb (set 0) and pb+1 (set 1)
      // loading; B(pb) dequantised into stage 0
      issue_a(MainK{}, pb, As, true);
      gload_b(MainK{}, pb, Set0{}, true);
      issue_a(MainK{}, at(pb + 1), As + A_TILE, live(pb + 1));
      if constexpr (!kSingleSet) gload_b(MainK{}, at(pb + 1), Set1{}, live(pb + 1));
      if constexpr (A_STAGES == 3) issue_a(MainK{}, at(pb + 2), As + 2 * A_TILE, live(pb + 2));
      __builtin_amdgcn_sched_barrier(0);
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((A_STAGES - 1) * A_LOADS + (kSingleSet ? 0 : kBLoadsMain))
                   : "memory");
      store_b(MainK{}, pb, Bs, Set0{}, AllPieces{});
      if constexpr (kSingleSet) gload_b(MainK{}, at(pb + 1), Set0{}, live(pb + 1));
      asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
      load_frags_main(As, Bs, 0, Set0{});
      int it = pb;
      if constexpr (A_STAGES == 3) {
        uint16_t *a0 = As, *a1 = As + A_TILE, *a2 = As + 2 * A_TILE;  // stages of it, it+1, it+2
#pragma nounroll
        for (; it + 1 < pe; it += 2) {  // hot loop: two steps, one per parity
          step(it, a0, a1, a2, Set0{});
          step(it + 1, a1, a2, a0, Set1{});
          uint16_t* t = a0;  // two steps on: the stage of it+2 is the current one
          a0 = a2;
          a2 = a1;
          a1 = t;
        }
        if (it < pe) step(it, a0, a1, a2, Set0{});
      } else {  // two stages: they alternate with the parity
        uint16_t *a0 = As, *a1 = As + A_TILE;
#pragma nounroll
        for (; it + 1 < pe; it += 2) {
          step(it, a0, a1, Bs, Set0{});
          step(it + 1, a1, a0, Bs, Set1{});
        }
        if (it < pe) step(it, a0, a1, Bs, Set0{});
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the out-of-range loads of the last steps
    }
  } else {
    // Plain product over the tail operands: one register set, so the copy of step it+1 into
    // LDS and the loads of step it+2 follow the matrix-core work of step it.
    //   entry : A(it), B(it) visible in LDS; A(it+1) LDS-DMA in flight; registers hold it+1
    auto step = [&](auto n1, auto n2, int it, int slot) {
      constexpr bool kHas1 = decltype(n1)::value != 2;
      constexpr bool kHas2 = decltype(n2)::value != 2;
      const int sa = slot % 3, sa2 = (slot + 2) % 3, sb = slot & 1;
      with_step_regions(
          As + sa2 * A_TILE, As + sa * A_TILE, Bs + sb * B_TILE, Bs + (sb ^ 1) * B_TILE,
          [&](uint16_t* a_dma, const uint16_t* a_rd, const uint16_t* b_rd, uint16_t* b_wr) {
            if constexpr (kHas2) issue_a(TailK{}, it + 2, a_dma, true);
            __builtin_amdgcn_sched_barrier(0);
            compute(TailK{}, a_rd, b_rd, no_side);
            if constexpr (kHas1) store_b(TailK{}, it + 1, b_wr, Set0{}, AllPieces{});
            if constexpr (kHas2) gload_b(TailK{}, it + 2, Set0{}, true);
          });
      constexpr int kKeepT = kHas2 ? A_LOADS + kBLoadsTail : 0;
      wait_and_barrier<kKeepT>();
    };
    const int pb = it_begin, pe = it_end;
    const int n = pe - pb;
    if (n > 0) {
      issue_a(TailK{}, pb, As, true);
      gload_b(TailK{}, pb, Set0{}, true);
      if (n > 1) issue_a(TailK{}, pb + 1, As + A_TILE, true);
      store_b(TailK{}, pb, Bs, Set0{}, AllPieces{});
      if (n > 1) gload_b(TailK{}, pb + 1, Set0{}, true);
      wait_and_barrier<0>();  // prologue only: drain everything
      int it = pb, slot = 0;
#pragma nounroll
      for (; it + 2 < pe; ++it, ++slot) step(TailK{}, TailK{}, it, slot);  // hot loop
      if (it + 1 < pe) {
        step(TailK{}, NoneK{}, it, slot);
        ++it, ++slot;
      }
      step(NoneK{}, NoneK{}, it, slot);
    }
  }

  // ---- epilogue: D[m][n] lives at lane n%32, register 4*(m/8) + m%4, half (m/4)%2 ----
  // The tile is rescaled, converted and transposed through LDS (free by now), so that global
  // memory sees 16-byte stores covering whole 512- or 1024-byte rows of the tile.  The row
  // scales are fetched once into LDS first.  (Thread coordinates are re-derived here so that
  // nothing but the accumulators has to stay live across the K loop.)
  if (timeline) p.block_times[4 * blockIdx.x + 1] = (unsigned long long)wall_clock64();
  int e_tid = threadIdx.x;
  asm volatile("" : "+v"(e_tid));
  const int e_lane = e_tid & 63, e_wave = e_tid >> 6;
  const int e_wm = e_wave % WAVES_M, e_wn = e_wave / WAVES_M;
  const size_t zoff = (size_t)blockIdx.y * (size_t)p.M * (size_t)p.N;
  float* inv_s = reinterpret_cast<float*>(smem);  // [BM]
  char* stage = reinterpret_cast<char*>(smem) + BM * 4;
  __syncthreads();  // every wave is past its last LDS read of the K loop
  if (e_tid < BM)
    inv_s[e_tid] = (HAS_MAIN && m0 + e_tid < p.M) ? p.row_scale[m0 + e_tid].y : 1.0f;
  // 1 / S of the factor words for this lane's output columns: per column (forward), one value
  // for the call (backward)
  float inv_n[TN];
#pragma unroll
  for (int b = 0; b < TN; ++b) {
    inv_n[b] = 1.0f;
    if constexpr (HAS_MAIN) {
      const int n = n0 + e_wn * WTN + b * 32 + (e_lane & 31);
      inv_n[b] = BWD ? p.n_scale[0] : (n < p.N ? p.n_scale[n] : 1.0f);
    }
  }
  auto epilogue = [&](auto as_bf16) {
    constexpr bool kBf16 = decltype(as_bf16)::value;
    constexpr int ES = kBf16 ? 2 : 4;
    constexpr int ROW = BN * ES + 16;  // staged row stride (+16: spreads rows over banks)
    constexpr int kLds = (A_STAGES * BM + 2 * BN) * 64 * 2;
    constexpr int kPasses = (BM * ROW + BM * 4 > kLds) ? 2 : 1;
    constexpr int RP = BM / kPasses;  // rows staged per pass
    static_assert(RP % WTM == 0 && RP * ROW + BM * 4 <= kLds, "a pass is whole wave row-bands");
    constexpr int CPR = BN * ES / 16;  // 16-byte chunks per row
    static_assert(NT % CPR == 0, "threads tile the rows of a pass");
    __syncthreads();  // row scales visible
#pragma unroll
    for (int pass = 0; pass < kPasses; ++pass) {
      if (pass > 0) __syncthreads();  // the previous pass has been read out
      if ((e_wm * WTM) / RP == pass) {
        const int rbase = e_wm * WTM - pass * RP;
#pragma unroll
        for (int a = 0; a < TM; ++a) {
          f32x4 inv[4];
#pragma unroll
          for (int g4 = 0; g4 < 4; ++g4)
            inv[g4] = *reinterpret_cast<const f32x4*>(inv_s + e_wm * WTM + a * 32 + 8 * g4 + 4 * (e_lane >> 5));
#pragma unroll
          for (int b = 0; b < TN; ++b) {
            const int cl = e_wn * WTN + b * 32 + (e_lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int rl = rbase + a * 32 + 8 * (r >> 2) + 4 * (e_lane >> 5) + (r & 3);
              const float v = acc[a][b][r] * inv[r >> 2][r & 3] * inv_n[b];
              if constexpr (kBf16)
                *reinterpret_cast<uint16_t*>(stage + rl * ROW + cl * 2) = f32_to_bf16_bits(v);
              else
                *reinterpret_cast<float*>(stage + rl * ROW + cl * 4) = v;
            }
          }
        }
      }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < RP * CPR / NT; ++k) {
        const int idx = e_tid + NT * k;
        const int rl = idx / CPR, ch = idx % CPR;
        const int row = m0 + pass * RP + rl, col = n0 + ch * (16 / ES);
        if (row < p.M && col < p.N) {
          const uint4 v = *reinterpret_cast<const uint4*>(stage + rl * ROW + ch * 16);
          char* o = static_cast<char*>(p.out) + (zoff + (size_t)row * p.N + col) * ES;
          *reinterpret_cast<uint4*>(o) = v;
        }
      }
    }
  };
  if (p.out_bf16)
    epilogue(std::true_type{});
  else
    epilogue(std::false_type{});
  if (probe) {
    p.clock_probe[2] = (unsigned long long)clock64();
    p.clock_probe[3] = (unsigned long long)wall_clock64();
  }
  if (timeline) p.block_times[4 * blockIdx.x + 2] = (unsigned long long)wall_clock64();
}

template <int NBITS, bool BWD, int BM, int BN, int WAVES_M, int WAVES_N, bool HAS_MAIN, bool FAST>
static hipError_t launch_cfg(const GemmArgs& a, int ksplit, hipStream_t st, hipEvent_t ev_start = nullptr,
                             hipEvent_t ev_stop = nullptr) {
  auto kern = gemm_dq_kernel<NBITS, BWD, BM, BN, WAVES_M, WAVES_N, HAS_MAIN, FAST>;
  const size_t smem = (size_t)(gemm_a_stages(BM, HAS_MAIN) * BM + 2 * BN) * 64 * sizeof(uint16_t);
  static std::atomic<uint64_t> granted{0};  // per instantiation
  if (hipError_t e = grant_dynamic_lds(reinterpret_cast<const void*>(kern), (int)smem, granted); e != hipSuccess)
    return e;
  dim3 grid(ceil_div(a.M, BM) * ceil_div(a.N, BN), ksplit);
  if (ev_start || ev_stop) {
    // measurement aid: the events take the dispatch's own begin and end timestamps, which costs
    // the stream nothing (events recorded around the launch cost it a few microseconds each)
    hipExtLaunchKernelGGL(kern, grid, dim3(NT), (unsigned)smem, st, ev_start, ev_stop, 0, a);
  } else {
    kern<<<grid, NT, smem, st>>>(a);
  }
  return hipGetLastError();
}

template <int NBITS, bool BWD>
static hipError_t launch_dir(const GemmArgs& a, hipStream_t st, hipEvent_t e0, hipEvent_t e1) {
  const int ks = a.ksplit > 1 ? a.ksplit : 1;
  const bool fast = a.a_main_padded_rows >= round_up(a.M, 256) && a.K_main % BK == 0 &&
                    (BK % a.group == 0 || a.group % BK == 0);
  if (a.M > 128) {
    if (fast) return launch_cfg<NBITS, BWD, 256, 256, 2, 4, true, true>(a, ks, st, e0, e1);
    return launch_cfg<NBITS, BWD, 128, 256, 2, 4, true, false>(a, ks, st, e0, e1);
  }
  if (a.M > 64) {
    if (fast) return launch_cfg<NBITS, BWD, 128, 256, 2, 4, true, true>(a, ks, st, e0, e1);
    return launch_cfg<NBITS, BWD, 128, 256, 2, 4, true, false>(a, ks, st, e0, e1);
  }
  if (fast) return launch_cfg<NBITS, BWD, 64, 256, 1, 8, true, true>(a, ks, st, e0, e1);
  return launch_cfg<NBITS, BWD, 64, 256, 1, 8, true, false>(a, ks, st, e0, e1);
}

// K splits of the dequantising product.  One block runs per compute unit, so a launch takes
// rounds(tiles x splits) x (steps per block + a fixed cost per block); splitting K pays when it
// fills compute units that a short or ragged last round leaves idle (few tokens; 160 tiles on
// 256 units) by more than the fp32 partial sums cost: `splits` copies of the output written
// here and read again by the sum, priced at 4 TB/s against the ~2 us of a 256-row K step.
// At least eight K steps per slice.
int gemm_dq_ksplit(int M, int N, int K_main) {
  constexpr double kBlockSteps = 7;  // prologue + epilogue of a block, in K steps
  const int bm = M > 128 ? 256 : (M > 64 ? 128 : 64);
  const int kUnits = bm == 64 ? 512 : 256;  // resident blocks: one per compute unit, two of the 64-row tile
  const long tiles = (long)ceil_div(M, bm) * ceil_div(N, 256);
  const int nk = ceil_div(K_main, BK);
  const double step_us = 2.0 * bm / 256;
  auto cost = [&](int ks) {
    const long rounds = (tiles * ks + kUnits - 1) / kUnits;
    const double sum_us = ks > 1 ? (double)M * N * (8.0 * ks + 2.0) / 4e6 : 0.0;
    return rounds * (ceil_div(nk, ks) + kBlockSteps) + sum_us / step_us;
  };
  int best = 1;
  double best_cost = cost(1);
  for (int ks = 2; ks <= 16 && nk / ks >= 8; ++ks) {
    const double c = cost(ks);
    if (c < best_cost) {
      best_cost = c;
      best = ks;
    }
  }
  return best;
}

// out = sum over the K slices of the partial products, slice order, converted on the way out
__global__ __launch_bounds__(256) void split_reduce_kernel(const float* __restrict__ part,
                                                           int nparts, size_t n4, void* out,
                                                           int out_bf16) {
  const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;  // group of 4 elements
  if (i >= n4) return;
  f32x4 v = reinterpret_cast<const f32x4*>(part)[i];
  for (int z = 1; z < nparts; ++z) v += reinterpret_cast<const f32x4*>(part)[(size_t)z * n4 + i];
  if (out_bf16)
    reinterpret_cast<uint2*>(out)[i] = uint2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
  else
    reinterpret_cast<f32x4*>(out)[i] = v;
}

ProfileHook g_profile_hook[2] = {{nullptr, nullptr, nullptr}, {nullptr, nullptr, nullptr}};

static hipError_t launch_bits(int bits, bool bwd, const GemmArgs& a, hipStream_t st, hipEvent_t e0,
                              hipEvent_t e1) {
  if (bits == 4) return bwd ? launch_dir<4, true>(a, st, e0, e1) : launch_dir<4, false>(a, st, e0, e1);
  if (bits == 3) return bwd ? launch_dir<3, true>(a, st, e0, e1) : launch_dir<3, false>(a, st, e0, e1);
  return bwd ? launch_dir<2, true>(a, st, e0, e1) : launch_dir<2, false>(a, st, e0, e1);
}

hipError_t launch_gemm_dq(int bits, bool bwd, const GemmArgs& args, hipStream_t st) {
  GemmArgs a = args;
  const bool split = a.ksplit > 1;
  if (split) {  // slices write fp32 partials; the sum is converted afterwards
    a.out = a.partial;
    a.out_bf16 = 0;
  }
  ProfileHook hook = g_profile_hook[bwd ? 1 : 0];
  g_profile_hook[bwd ? 1 : 0] = ProfileHook{nullptr, nullptr, nullptr, nullptr, 0};
  a.clock_probe = hook.clock_probe;
  a.block_times = hook.block_times;
  a.block_times_cap = hook.block_times_cap;
  // without a split the events ride on the dispatch itself; with one they bracket both launches
  const bool ride = !split && hook.start && hook.stop;
  if (hook.start && !ride) (void)hipEventRecord(hook.start, st);
  hipError_t e = launch_bits(bits, bwd, a, st, ride ? hook.start : nullptr, ride ? hook.stop : nullptr);
  if (e == hipSuccess && split) {
    const size_t n4 = (size_t)a.M * a.N / 4;  // N is a multiple of 8
    split_reduce_kernel<<<(unsigned)((n4 + 255) / 256), 256, 0, st>>>(a.partial, a.ksplit, n4,
                                                                      args.out, args.out_bf16);
    e = hipGetLastError();
  }
  if (hook.stop && !ride) (void)hipEventRecord(hook.stop, st);
  return e;
}

// Plain bf16 x bf16^T product  out[z][M][N] = a_tail[M, Kz] . b_tail[N, Kz]^T  with the K
// range split over `ksplit` slices (partial sums, reduced by the caller in a fixed order).
// Row tile of the plain product by its K length: 128 rows from 128 K steps on (measured: the
// dU product of a layer with D_out = 11008 runs 35 -> 24 us on the taller tile, the one with
// D_out = 4096 14 -> 16 us).
int gemm_plain_tile_rows(int K) { return K >= 128 * BK ? 128 : 64; }

hipError_t launch_gemm_plain(const GemmArgs& a, int ksplit, hipStream_t st) {
  if (gemm_plain_tile_rows(a.K_tail) == 128)
    return launch_cfg<4, false, 128, 128, 2, 4, false, false>(a, ksplit, st);
  return launch_cfg<4, false, 64, 128, 2, 4, false, false>(a, ksplit, st);
}

}  // namespace qalora
