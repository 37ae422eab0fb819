// The dense contractions of the QA-LoRA linear on the bf16 matrix cores of gfx950:
//
//   forward   y  = [x | s U~] . [W~ ; B~]        K = D_in  (+ adapter tail), N = D_out
//   backward  dx = [dy | dU~] . [W~^T ; A~/g]    K = D_out (+ adapter tail), N = D_in
//
// with W~[i,j] = alpha[i/g,j] * code[i,j] + beta[i/g,j] (Eq. 1 per group, Sec. 3.3)
// rebuilt on the fly: packed codes are read from HBM with 128-bit loads, dequantised in
// registers (fp32 fma, one rounding to bf16), staged in LDS and fed to
// v_mfma_f32_32x32x16_bf16 with fp32 accumulation.  The low-rank branch of Alg. 1,
// s (pool(x) A) B, rides along as a few extra K steps: the small factors are split into
// bf16 hi + lo parts (three products hi*hi + lo*hi + hi*lo) so the adapter keeps fp32-level
// accuracy while staying on the matrix cores.
//
// One kernel serves both directions from ONE packed copy of the codes: a thread owns an
// 8x8 patch of codes (eight 32-bit column words), from which it can emit eight K-contiguous
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

// Dequantise one column's worth (forward) or one row's worth (backward) of an 8x8 patch
// into eight bf16 values packed in a uint4.
template <int NBITS, bool BWD>
__device__ __forceinline__ uint4 dequant_fragment(const uint32_t (&w0)[8], const uint32_t (&w1)[8],
                                                  const float (&al)[8], const float (&be)[8],
                                                  int f) {
  float v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    // forward: fragment f = column f, element e = row e; backward: fragment f = row f,
    // element e = column e.
    const int col = BWD ? e : f;
    const int row = BWD ? f : e;
    const float c = (float)patch_code<NBITS>(w0[col], w1[col], row);
    v[e] = __builtin_fmaf(al[col], c, be[col]);
  }
  uint4 r;
  r.x = pack_bf16x2(v[0], v[1]);
  r.y = pack_bf16x2(v[2], v[3]);
  r.z = pack_bf16x2(v[4], v[5]);
  r.w = pack_bf16x2(v[6], v[7]);
  return r;
}

// Block-index -> tile-index map.  Consecutive block ids are dealt round-robin to the 8
// XCDs, each with its own L2; give every XCD a contiguous run of tiles (tile_m fastest)
// so that the weight panels and activation rows it touches stay in that L2.
__device__ __forceinline__ int xcd_remap(int bid, int nblocks) {
  if (nblocks % 8 != 0) return bid;
  return (bid % 8) * (nblocks / 8) + bid / 8;
}

template <int NBITS, bool BWD, int BM, int BN, int WAVES_M, int WAVES_N, bool HAS_MAIN>
__global__ __launch_bounds__(256) void gemm_dq_kernel(const GemmArgs p) {
  static_assert(WAVES_M * WAVES_N == 4, "four wavefronts per block");
  static_assert(!HAS_MAIN || BN == 256, "the dequantising producer assumes 256 columns");
  constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int A_CHUNKS = BM / 32;  // 16-byte chunks of the A tile per thread
  constexpr int B_CHUNKS = BN / 32;  // same for a plain (already bf16) B tile

  extern __shared__ __align__(16) uint16_t smem[];
  uint16_t* As = smem;                      // [2][BM][LDS_ROW]
  uint16_t* Bs = smem + 2 * BM * LDS_ROW;   // [2][BN][LDS_ROW]

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
  // only for tail-only launches (plain bf16 x bf16 products with a short M).
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

  // ---- registers -> LDS (dequantising on the way for main steps) -------------------
  auto lds_store = [&](int it, int buf) {
    const bool main_step = HAS_MAIN && it < nk_main;
    uint16_t* as = As + buf * BM * LDS_ROW;
    uint16_t* bs = Bs + buf * BN * LDS_ROW;
#pragma unroll
    for (int q = 0; q < A_CHUNKS; ++q) {
      const int idx = tid + 256 * q;
      const int row = idx >> 3, ch = idx & 7;
      *reinterpret_cast<uint4*>(as + row * LDS_ROW + 8 * ch) = areg[q];
    }
    if (main_step) {
      if constexpr (HAS_MAIN) {
        const int u0 = tid & 7, u1 = tid >> 3;
        const int i0 = BWD ? n0 + 8 * u1 : (it * BK) + 8 * u0;
        uint32_t w0[8] = {breg[0].x, breg[0].y, breg[0].z, breg[0].w,
                          breg[1].x, breg[1].y, breg[1].z, breg[1].w};
        uint32_t w1[8] = {breg[6].x, breg[6].y, breg[6].z, breg[6].w,
                          breg[7].x, breg[7].y, breg[7].z, breg[7].w};
        const int sh0 = patch_preshift0<NBITS>(i0);
        const int sh1 = patch_preshift1(i0);
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          w0[c] >>= sh0;
          if constexpr (NBITS == 3) w1[c] >>= sh1;
        }
        const float al[8] = {__uint_as_float(breg[2].x), __uint_as_float(breg[2].y),
                             __uint_as_float(breg[2].z), __uint_as_float(breg[2].w),
                             __uint_as_float(breg[3].x), __uint_as_float(breg[3].y),
                             __uint_as_float(breg[3].z), __uint_as_float(breg[3].w)};
        const float be[8] = {__uint_as_float(breg[4].x), __uint_as_float(breg[4].y),
                             __uint_as_float(breg[4].z), __uint_as_float(breg[4].w),
                             __uint_as_float(breg[5].x), __uint_as_float(breg[5].y),
                             __uint_as_float(breg[5].z), __uint_as_float(breg[5].w)};
#pragma unroll
        for (int f = 0; f < 8; ++f) {
          const uint4 frag = dequant_fragment<NBITS, BWD>(w0, w1, al, be, f);
          *reinterpret_cast<uint4*>(bs + (8 * u1 + f) * LDS_ROW + 8 * u0) = frag;
        }
      }
    } else {
#pragma unroll
      for (int q = 0; q < B_CHUNKS; ++q) {
        const int idx = tid + 256 * q;
        const int row = idx >> 3, ch = idx & 7;
        *reinterpret_cast<uint4*>(bs + row * LDS_ROW + 8 * ch) = breg[q];
      }
    }
  };

  // ---- LDS -> matrix cores ---------------------------------------------------------
  auto compute = [&](int buf) {
    const uint16_t* as = As + buf * BM * LDS_ROW + (wm * WTM + (lane & 31)) * LDS_ROW + 8 * (lane >> 5);
    const uint16_t* bs = Bs + buf * BN * LDS_ROW + (wn * WTN + (lane & 31)) * LDS_ROW + 8 * (lane >> 5);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 af[TM], bf[TN];
#pragma unroll
      for (int a = 0; a < TM; ++a)
        af[a] = *reinterpret_cast<const bf16x8*>(as + a * 32 * LDS_ROW + kk * 16);
#pragma unroll
      for (int b = 0; b < TN; ++b)
        bf[b] = *reinterpret_cast<const bf16x8*>(bs + b * 32 * LDS_ROW + kk * 16);
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bf[b], acc[a][b], 0, 0, 0);
    }
  };

  if (it_begin < it_end) {
    gload(it_begin);
    lds_store(it_begin, 0);
    __syncthreads();
    for (int it = it_begin; it < it_end; ++it) {
      const int buf = (it - it_begin) & 1;
      if (it + 1 < it_end) gload(it + 1);
      compute(buf);
      if (it + 1 < it_end) lds_store(it + 1, buf ^ 1);
      __syncthreads();
    }
  }

  // ---- epilogue: D[m][n] lives at lane n%32, register 4*(m/8) + m%4, half (m/4)%2 ----
  const size_t zoff = (size_t)blockIdx.y * (size_t)p.M * (size_t)p.N;
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b) {
      const int col = n0 + wn * WTN + b * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * WTM + a * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < p.M && col < p.N) {
          const size_t o = zoff + (size_t)row * p.N + col;
          if (p.out_bf16)
            static_cast<uint16_t*>(p.out)[o] = f32_to_bf16_bits(acc[a][b][r]);
          else
            static_cast<float*>(p.out)[o] = acc[a][b][r];
        }
      }
    }
}

template <int NBITS, bool BWD, int BM, int BN, int WAVES_M, int WAVES_N, bool HAS_MAIN>
static hipError_t launch_cfg(const GemmArgs& a, int ksplit, hipStream_t st) {
  auto kern = gemm_dq_kernel<NBITS, BWD, BM, BN, WAVES_M, WAVES_N, HAS_MAIN>;
  const size_t smem = (size_t)2 * (BM + BN) * LDS_ROW * sizeof(uint16_t);
  static bool attr_set = false;  // per instantiation; setting it again is harmless
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
  if (a.M > 128) return launch_cfg<NBITS, BWD, 256, 256, 2, 2, true>(a, 1, st);
  if (a.M > 64) return launch_cfg<NBITS, BWD, 128, 256, 2, 2, true>(a, 1, st);
  return launch_cfg<NBITS, BWD, 64, 256, 1, 4, true>(a, 1, st);
}

hipError_t launch_gemm_dq(int bits, bool bwd, const GemmArgs& a, hipStream_t st) {
  if (bits == 4) return bwd ? launch_dir<4, true>(a, st) : launch_dir<4, false>(a, st);
  if (bits == 3) return bwd ? launch_dir<3, true>(a, st) : launch_dir<3, false>(a, st);
  return bwd ? launch_dir<2, true>(a, st) : launch_dir<2, false>(a, st);
}

// Plain bf16 x bf16^T product  out[z][M][N] = a_tail[M, Kz] . b_tail[N, Kz]^T  with the K
// range split over `ksplit` slices (partial sums, reduced by the caller in a fixed order).
hipError_t launch_gemm_plain(const GemmArgs& a, int ksplit, hipStream_t st) {
  return launch_cfg<4, false, 64, 128, 2, 2, false>(a, ksplit, st);
}

}  // namespace qalora
