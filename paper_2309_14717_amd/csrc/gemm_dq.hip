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
// on 2.1e-3).  The bf16 activations are converted exactly: every token row is first scaled
// by a power of two that brings its largest magnitude into [2^14, 2^15) (fp16's range is
// narrower than bf16's), and the output row is scaled back in the epilogue.
//
// The low-rank branch of Alg. 1, s (pool(x) A) B, rides along as a few extra K steps in
// bf16: the small factors are split into bf16 hi + lo parts (hi*hi + lo*hi + hi*lo), which
// keeps fp32-level accuracy and bf16's range for gradients.
//
// One kernel serves both directions from ONE packed copy of the codes: a thread owns an
// 8x8 patch of codes (eight 32-bit column words), from which it emits eight K-contiguous
// operand fragments along either axis -- down the rows (forward, K = input rows) or across
// the columns (backward, K = output columns).
//
// Tiling: 256 threads = 4 wavefronts of 64, block tile BM x BN x 64, double-buffered in
// LDS (rows padded to 144 bytes so that both the 128-bit fragment writes and the 128-bit
// operand reads are bank-conflict free), global->register prefetch of the next K step
// issued before the MFMAs of the current one.
#include "common.hpp"
#include "kernels.hpp"

namespace qalora {

constexpr int BK = 64;
constexpr int LDS_ROW = LDS_ROW_72;

__device__ __forceinline__ uint4 ldg128(const void* p) {
  return *reinterpret_cast<const uint4*>(p);
}

// 8 bf16 -> 8 fp16 after scaling by `sc` (a power of two chosen so nothing overflows).
__device__ __forceinline__ uint4 bf16x8_to_f16x8_scaled(uint4 v, float sc) {
  uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const f32x2 f = {__uint_as_float(w[e] << 16) * sc, __uint_as_float(w[e] & 0xffff0000u) * sc};
    w[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, f16x2));
  }
  return uint4{w[0], w[1], w[2], w[3]};
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
__global__ __launch_bounds__(256) void gemm_dq_kernel(const GemmArgs p) {
  static_assert(WAVES_M * WAVES_N == 4, "four wavefronts per block");
  static_assert(!HAS_MAIN || BN == 256, "the dequantising producer assumes 256 columns");
  constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int A_CHUNKS = BM / 32;  // 16-byte chunks of the A tile per thread
  constexpr int B_CHUNKS = BN / 32;  // same for a plain (already 16-bit) B tile

  extern __shared__ __align__(16) uint16_t smem[];
  uint16_t* As = smem;                     // [2][BM][LDS_ROW]
  uint16_t* Bs = smem + 2 * BM * LDS_ROW;  // [2][BN][LDS_ROW]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;

  const int tiles_m = ceil_div(p.M, BM);
  const int tiles_n = ceil_div(p.N, BN);
  const int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n);
  const int m0 = (tile % tiles_m) * BM;
  const int n0 = (tile / tiles_m) * BN;

  // K range of this block: all main steps, then the tail steps; split over blockIdx.y
  // only for tail-only launches.
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

  uint4 areg[A_CHUNKS];
  uint4 breg[8 > B_CHUNKS ? 8 : B_CHUNKS];

  // Power-of-two scale of each A row this thread stages (the rows do not change with k).
  float ascale[A_CHUNKS];
  if constexpr (HAS_MAIN) {
#pragma unroll
    for (int q = 0; q < A_CHUNKS; ++q) {
      const int m = m0 + ((tid + 256 * q) >> 3);
      ascale[q] = (m < p.M) ? p.row_scale[m].x : 1.0f;
    }
  }

  // ---- global -> registers for K step `it` ---------------------------------------
  auto gload = [&](int it) {
    const bool main_step = HAS_MAIN && it < nk_main;
    const uint16_t* a_base = main_step ? p.a_main : p.a_tail;
    const int lda = main_step ? p.lda_main : p.lda_tail;
    const int k0 = main_step ? it * BK : (it - nk_main) * BK;
    const int klim = main_step ? p.K_main : p.K_tail;
#pragma unroll
    for (int q = 0; q < A_CHUNKS; ++q) {
      const int idx = tid + 256 * q;
      const int row = idx >> 3, ch = idx & 7;
      const int m = m0 + row, k = k0 + 8 * ch;
      areg[q] = (m < p.M && k < klim) ? ldg128(a_base + (size_t)m * lda + k) : uint4{0, 0, 0, 0};
    }
    if (main_step) {
      if constexpr (HAS_MAIN) {
        const int u0 = tid & 7, u1 = tid >> 3;
        const int i0 = BWD ? n0 + 8 * u1 : k0 + 8 * u0;
        const int j0 = BWD ? k0 + 8 * u0 : n0 + 8 * u1;
        if (i0 < p.d_in && j0 < p.d_out) {
          load_patch_words<NBITS>(p.plane0, p.plane1, p.d_out, i0, j0, breg[0], breg[1], breg[6],
                                  breg[7]);
          const size_t ab = (size_t)(i0 / p.group) * p.d_out + j0;
          breg[2] = ldg128(p.alpha + ab);
          breg[3] = ldg128(p.alpha + ab + 4);
          breg[4] = ldg128(p.beta + ab);
          breg[5] = ldg128(p.beta + ab + 4);
        } else {
#pragma unroll
          for (int q = 0; q < 8; ++q) breg[q] = uint4{0, 0, 0, 0};
        }
      }
    } else {
#pragma unroll
      for (int q = 0; q < B_CHUNKS; ++q) {
        const int idx = tid + 256 * q;
        const int row = idx >> 3, ch = idx & 7;
        const int n = n0 + row;
        // forward tail: row n of B~^T; backward tail: row n/g of A~ (the unpooling of
        // the pooled gradient is this broadcast over the g rows of a group)
        const int src_row = BWD ? n / p.group : n;
        breg[q] = (n < p.N && k0 + 8 * ch < p.K_tail)
                      ? ldg128(p.b_tail + (size_t)src_row * p.K_tail + k0 + 8 * ch)
                      : uint4{0, 0, 0, 0};
      }
    }
  };

  // ---- registers -> LDS (converting / dequantising on the way for main steps) -------
  auto lds_store = [&](int it, int buf) {
    const bool main_step = HAS_MAIN && it < nk_main;
    uint16_t* as = As + buf * BM * LDS_ROW;
    uint16_t* bs = Bs + buf * BN * LDS_ROW;
    if (main_step) {
      if constexpr (HAS_MAIN) {
#pragma unroll
        for (int q = 0; q < A_CHUNKS; ++q) {
          const int idx = tid + 256 * q;
          const int row = idx >> 3, ch = idx & 7;
          *reinterpret_cast<uint4*>(as + row * LDS_ROW + 8 * ch) =
              bf16x8_to_f16x8_scaled(areg[q], ascale[q]);
        }
        const int u0 = tid & 7, u1 = tid >> 3;
        const int i0 = BWD ? n0 + 8 * u1 : (it * BK) + 8 * u0;
        uint32_t w0[8] = {breg[0].x, breg[0].y, breg[0].z, breg[0].w,
                          breg[1].x, breg[1].y, breg[1].z, breg[1].w};
        uint32_t w1[8] = {breg[6].x, breg[6].y, breg[6].z, breg[6].w,
                          breg[7].x, breg[7].y, breg[7].z, breg[7].w};
        const float al[8] = {__uint_as_float(breg[2].x), __uint_as_float(breg[2].y),
                             __uint_as_float(breg[2].z), __uint_as_float(breg[2].w),
                             __uint_as_float(breg[3].x), __uint_as_float(breg[3].y),
                             __uint_as_float(breg[3].z), __uint_as_float(breg[3].w)};
        const float be[8] = {__uint_as_float(breg[4].x), __uint_as_float(breg[4].y),
                             __uint_as_float(breg[4].z), __uint_as_float(breg[4].w),
                             __uint_as_float(breg[5].x), __uint_as_float(breg[5].y),
                             __uint_as_float(breg[5].z), __uint_as_float(breg[5].w)};
        const int sh0 = patch_preshift0<NBITS>(i0);
        const int sh1 = patch_preshift1(i0);
        // wt[c][m] = (W~[2m][c], W~[2m+1][c]) as an fp16 pair: alpha * code + beta in one
        // packed fma per pair of rows.
        uint32_t wt[8][4];
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          const uint32_t w0s = w0[c] >> sh0;
          const uint32_t w1s = (NBITS == 3) ? (w1[c] >> sh1) : 0u;
          const f32x2 abf = {al[c], be[c]};
          const f16x2 ab = __builtin_convertvector(abf, f16x2);
          const f16x2 a2 = {ab.x, ab.x};
          const f16x2 b2 = {ab.y, ab.y};
#pragma unroll
          for (int m = 0; m < 4; ++m) {
            const f16x2 cc = patch_code_pair_f16<NBITS>(w0s, w1s, m);
            wt[c][m] = __builtin_bit_cast(uint32_t, cc * a2 + b2);
          }
        }
        if constexpr (!BWD) {
          // fragment c = column c, its 8 rows are already K-contiguous
#pragma unroll
          for (int c = 0; c < 8; ++c)
            *reinterpret_cast<uint4*>(bs + (8 * u1 + c) * LDS_ROW + 8 * u0) =
                uint4{wt[c][0], wt[c][1], wt[c][2], wt[c][3]};
        } else {
          // fragment r = row r: gather the matching halves of the eight columns
#pragma unroll
          for (int r = 0; r < 8; ++r) {
            uint32_t o[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const uint32_t lo = wt[2 * q][r >> 1], hi = wt[2 * q + 1][r >> 1];
              o[q] = (r & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u)
                             : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
            }
            *reinterpret_cast<uint4*>(bs + (8 * u1 + r) * LDS_ROW + 8 * u0) =
                uint4{o[0], o[1], o[2], o[3]};
          }
        }
      }
    } else {
#pragma unroll
      for (int q = 0; q < A_CHUNKS; ++q) {
        const int idx = tid + 256 * q;
        const int row = idx >> 3, ch = idx & 7;
        *reinterpret_cast<uint4*>(as + row * LDS_ROW + 8 * ch) = areg[q];
      }
#pragma unroll
      for (int q = 0; q < B_CHUNKS; ++q) {
        const int idx = tid + 256 * q;
        const int row = idx >> 3, ch = idx & 7;
        *reinterpret_cast<uint4*>(bs + row * LDS_ROW + 8 * ch) = breg[q];
      }
    }
  };

  // ---- LDS -> matrix cores ---------------------------------------------------------
  auto compute = [&](int buf, bool main_step) {
    const uint16_t* as = As + buf * BM * LDS_ROW + (wm * WTM + (lane & 31)) * LDS_ROW + 8 * (lane >> 5);
    const uint16_t* bs = Bs + buf * BN * LDS_ROW + (wn * WTN + (lane & 31)) * LDS_ROW + 8 * (lane >> 5);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      uint4 af[TM], bf[TN];
#pragma unroll
      for (int a = 0; a < TM; ++a)
        af[a] = *reinterpret_cast<const uint4*>(as + a * 32 * LDS_ROW + kk * 16);
#pragma unroll
      for (int b = 0; b < TN; ++b)
        bf[b] = *reinterpret_cast<const uint4*>(bs + b * 32 * LDS_ROW + kk * 16);
      if (HAS_MAIN && main_step) {
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
          for (int b = 0; b < TN; ++b)
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                __builtin_bit_cast(f16x8, af[a]), __builtin_bit_cast(f16x8, bf[b]), acc[a][b], 0, 0, 0);
      } else {
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
          for (int b = 0; b < TN; ++b)
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                __builtin_bit_cast(bf16x8, af[a]), __builtin_bit_cast(bf16x8, bf[b]), acc[a][b], 0, 0, 0);
      }
    }
  };

  if (it_begin < it_end) {
    gload(it_begin);
    lds_store(it_begin, 0);
    __syncthreads();
    for (int it = it_begin; it < it_end; ++it) {
      const int buf = (it - it_begin) & 1;
      if (it + 1 < it_end) gload(it + 1);
      compute(buf, it < nk_main);
      if (it + 1 < it_end) lds_store(it + 1, buf ^ 1);
      __syncthreads();
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
  const size_t smem = (size_t)2 * (BM + BN) * LDS_ROW * sizeof(uint16_t);
  static bool attr_set = false;  // per instantiation
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  dim3 grid(ceil_div(a.M, BM) * ceil_div(a.N, BN), ksplit);
  kern<<<grid, 256, smem, st>>>(a);
  return hipGetLastError();
}

template <int NBITS, bool BWD>
static hipError_t launch_dir(const GemmArgs& a, hipStream_t st) {
  if (a.M > 64) return launch_cfg<NBITS, BWD, 128, 256, 2, 2, true>(a, 1, st);
  return launch_cfg<NBITS, BWD, 64, 256, 1, 4, true>(a, 1, st);
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
  return launch_cfg<4, false, 64, 128, 2, 2, false>(a, ksplit, st);
}

}  // namespace qalora
