// The low-rank branch of the QA-LoRA linear (Alg. 1; Sec. 3.3): group pooling of the
// input, the small products with A and B, their gradients, and the merge of the adapter
// into the zero factors (App. B.3).  All of it is tiny next to the two dense contractions;
// the kernels here are shaped for latency and for deterministic (fixed-order) reductions.
//
// Small fp32 factors that must go through the bf16 matrix cores are split as hi + lo
// (hi = bf16(v), lo = bf16(v - hi)); a product U.B is then evaluated as
// hi.hi + lo.hi + hi.lo, which is accurate to about 2^-16.
#include "common.hpp"
#include "kernels.hpp"

namespace qalora {

// ---------------------------------------------------------------------------------------
// Per-row power-of-two scale for the fp16 matrix-core path: scale = 2^(14 - e) where e is the
// unbiased exponent of the row's largest magnitude, so the scaled row peaks in [2^14, 2^15).
// (.x = scale, .y = 1/scale).  Rows that are all zero (or hold inf/nan) get 1.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float2 scale_from_maxbits(uint32_t maxbits) {
  const int e = (int)(maxbits >> 7);  // biased exponent of the largest |bf16|
  if (e < 15 || e >= 255) return float2{1.0f, 1.0f};
  return float2{__uint_as_float((uint32_t)(268 - e) << 23), __uint_as_float((uint32_t)(e - 14) << 23)};
}

__device__ __forceinline__ uint32_t max_abs_bits(uint4 q, uint32_t m) {
  const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    m = max(m, w[e] & 0x7fffu);
    m = max(m, (w[e] >> 16) & 0x7fffu);
  }
  return m;
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) v = max(v, (uint32_t)__shfl_xor((int)v, off, 64));
  return v;
}

// 8 bf16 -> 8 fp16 after scaling by `sc` (a power of two chosen so nothing overflows; exact
// unless an element is more than 2^31 below the row maximum).
__device__ __forceinline__ uint4 bf16x8_to_f16x8_scaled(uint4 v, float sc) {
  uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const f32x2 f = {__uint_as_float(w[e] << 16) * sc, __uint_as_float(w[e] & 0xffff0000u) * sc};
    w[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, f16x2));
  }
  return uint4{w[0], w[1], w[2], w[3]};
}

// a bf16 [rows, cols] -> a16 fp16 [rows, cols] = a * rs[row].x, and rs.  One wavefront per
// row: a first sweep finds the row maximum, a second (served by L2) converts.
__global__ __launch_bounds__(256) void convert_rows_kernel(const uint16_t* __restrict__ a,
                                                           int rows, int cols,
                                                           float2* __restrict__ rs,
                                                           uint16_t* __restrict__ a16) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const uint16_t* src = a + (size_t)row * cols;
  uint32_t m = 0;
  for (int ch = lane; ch < cols / 8; ch += 64)
    m = max_abs_bits(*reinterpret_cast<const uint4*>(src + 8 * ch), m);
  m = wave_max_u32(m);
  const float2 sc = scale_from_maxbits(m);
  if (lane == 0) rs[row] = sc;
  uint16_t* dst = a16 + (size_t)row * cols;
  for (int ch = lane; ch < cols / 8; ch += 64)
    *reinterpret_cast<uint4*>(dst + 8 * ch) =
        bf16x8_to_f16x8_scaled(*reinterpret_cast<const uint4*>(src + 8 * ch), sc.x);
}

hipError_t launch_convert_rows(const uint16_t* a, int rows, int cols, float2* rs, uint16_t* a16,
                               hipStream_t st) {
  convert_rows_kernel<<<ceil_div(rows, 4), 256, 0, st>>>(a, rows, cols, rs, a16);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// pool_g(x) and U = pool_g(x) A.   One block = 8 tokens, one wavefront = 2 of them.
// The group average uses a wavefront butterfly: each lane sums 8 consecutive bf16 inputs
// (one 128-bit load), then lanes of the same group (g/8 of them) combine with xor-shuffles.
// The same sweep over the row yields its largest magnitude, hence its power-of-two scale.
// ---------------------------------------------------------------------------------------
constexpr int POOL_TB = 8;

__global__ __launch_bounds__(256) void pool_down_kernel(const uint16_t* __restrict__ x,
                                                        const float* __restrict__ A, float s,
                                                        int T, int d_in, int g, int rank,
                                                        float* __restrict__ P_out,
                                                        float2* __restrict__ rs_out,
                                                        uint16_t* __restrict__ x16,
                                                        uint16_t* __restrict__ u_ext, int ktail,
                                                        uint16_t* __restrict__ us_t, int t_pad) {
  extern __shared__ float P_s[];  // [POOL_TB][L]
  __shared__ float sc_s[POOL_TB];
  const int L = d_in / g;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t0 = blockIdx.x * POOL_TB;
  const int lpg = g / 8;  // lanes per group
  const bool butterfly = (lpg <= 64) && ((lpg & (lpg - 1)) == 0);
  const float inv_g = 1.0f / (float)g;
  const int nchunks = d_in / 8;

  for (int tt = wave * 2; tt < wave * 2 + 2; ++tt) {
    const int t = t0 + tt;
    uint32_t amax = 0;
    for (int c0 = 0; c0 < nchunks; c0 += 64) {
      const int ch = c0 + lane;
      float v = 0.0f;
      if (t < T && ch < nchunks) {
        const uint4 q = *reinterpret_cast<const uint4*>(x + (size_t)t * d_in + 8 * ch);
        amax = max_abs_bits(q, amax);
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          v += bf16_bits_to_f32(w[e] & 0xffffu);
          v += __uint_as_float(w[e] & 0xffff0000u);
        }
      }
      if (butterfly) {
        for (int off = 1; off < lpg; off <<= 1) v += __shfl_xor(v, off, 64);
        if (ch < nchunks && (lane & (lpg - 1)) == 0) P_s[tt * L + ch / lpg] = v * inv_g;
      }
    }
    amax = wave_max_u32(amax);
    const float2 sc = scale_from_maxbits(amax);
    if (lane == 0) {
      sc_s[tt] = sc.x;
      if (rs_out && t < T) rs_out[t] = sc;
    }
    if (x16 && t < T) {  // second sweep over the row (L2): scaled fp16 copy for the matrix cores
      for (int ch = lane; ch < nchunks; ch += 64)
        *reinterpret_cast<uint4*>(x16 + (size_t)t * d_in + 8 * ch) = bf16x8_to_f16x8_scaled(
            *reinterpret_cast<const uint4*>(x + (size_t)t * d_in + 8 * ch), sc.x);
    }
  }
  if (!butterfly) {
    for (int o = tid; o < POOL_TB * L; o += 256) {
      const int tt = o / L, l = o % L;
      const int t = t0 + tt;
      float v = 0.0f;
      if (t < T)
        for (int q = 0; q < g; ++q) v += bf16_bits_to_f32(x[(size_t)t * d_in + l * g + q]);
      P_s[o] = v * inv_g;
    }
  }
  __syncthreads();

  if (P_out) {
    for (int o = tid; o < POOL_TB * L; o += 256) {
      const int t = t0 + o / L;
      if (t < T) P_out[(size_t)t * L + o % L] = P_s[o];
    }
  }
  const int rp = rank_pad32(rank);
  for (int o = tid; o < POOL_TB * rank; o += 256) {
    const int tt = o / rank, k = o % rank;
    const int t = t0 + tt;
    if (t >= T) continue;
    float u = 0.0f;
    for (int l = 0; l < L; ++l) u = __builtin_fmaf(P_s[tt * L + l], A[(size_t)l * rank + k], u);
    u *= s;
    uint16_t hi, lo;
    if (u_ext) {
      // the forward tail shares the accumulator of the scaled main product
      split_bf16(u * sc_s[tt], hi, lo);
      uint16_t* row = u_ext + (size_t)t * ktail;
      row[k] = hi;
      row[rank + k] = lo;
      row[2 * rank + k] = hi;
    }
    if (us_t) {
      split_bf16(u, hi, lo);
      us_t[(size_t)k * t_pad + t] = hi;
      us_t[(size_t)(rp + k) * t_pad + t] = lo;
    }
  }
  if (u_ext) {
    const int npad = ktail - 3 * rank;
    for (int o = tid; o < POOL_TB * npad; o += 256) {
      const int t = t0 + o / npad;
      if (t < T) u_ext[(size_t)t * ktail + 3 * rank + o % npad] = 0;
    }
  }
}

__global__ void fill_zero_kernel(uint4* __restrict__ p, size_t n16) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n16;
       i += (size_t)gridDim.x * blockDim.x)
    p[i] = uint4{0, 0, 0, 0};
}

hipError_t launch_pool_down(const uint16_t* x, const float* A, float s, int T, int d_in, int g,
                            int rank, float* P_out, float2* rs_out, uint16_t* x16,
                            uint16_t* u_ext, int ktail, uint16_t* us_t, int t_pad,
                            hipStream_t st) {
  const int L = d_in / g;
  const size_t smem = (size_t)POOL_TB * L * sizeof(float);
  static size_t smem_limit = 48 * 1024;
  if (smem > smem_limit) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(pool_down_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    smem_limit = smem;
  }
  if (us_t) {
    // padding rows / columns of the transposed operand must read as zero
    const size_t n16 = (size_t)2 * rank_pad32(rank) * t_pad * sizeof(uint16_t) / 16;
    const size_t nblk = (n16 + 255) / 256;
    fill_zero_kernel<<<(int)(nblk < 1024 ? nblk : 1024), 256, 0, st>>>(
        reinterpret_cast<uint4*>(us_t), n16);
  }
  pool_down_kernel<<<ceil_div(T, POOL_TB), 256, smem, st>>>(
      x, A, s, T, d_in, g, rank, P_out, rs_out, x16, u_ext, ktail, us_t, t_pad);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Operand preparation (elementwise hi/lo splits).
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prep_b_fwd_kernel(const float* __restrict__ B, int rank,
                                                         int d_out, uint16_t* __restrict__ bt,
                                                         int ktail) {
  const size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (idx >= (size_t)d_out * ktail) return;
  const int j = (int)(idx / ktail), c = (int)(idx % ktail);
  uint16_t v = 0;
  if (c < 3 * rank) {
    const int k = c % rank;
    uint16_t hi, lo;
    split_bf16(B[(size_t)k * d_out + j], hi, lo);
    v = (c < 2 * rank) ? hi : lo;
  }
  bt[idx] = v;
}

hipError_t launch_prep_b_fwd(const float* B, int rank, int d_out, uint16_t* b_ext_t, int ktail,
                             hipStream_t st) {
  const size_t n = (size_t)d_out * ktail;
  prep_b_fwd_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(B, rank, d_out, b_ext_t, ktail);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void prep_bwd_kernel(const float* __restrict__ A,
                                                       const float* __restrict__ B, int L,
                                                       int rank, int d_out, int g,
                                                       uint16_t* __restrict__ b_hl,
                                                       uint16_t* __restrict__ a_ext_t,
                                                       int ktail) {
  const int rp = rank_pad32(rank);
  const size_t nb = (size_t)2 * rp * d_out;
  const size_t na = (size_t)L * ktail;
  const size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (idx < nb) {
    const int row = (int)(idx / d_out), j = (int)(idx % d_out);
    const int k = row % rp;
    uint16_t v = 0;
    if (k < rank) {
      uint16_t hi, lo;
      split_bf16(B[(size_t)k * d_out + j], hi, lo);
      v = (row < rp) ? hi : lo;
    }
    b_hl[idx] = v;
  } else if (idx < nb + na) {
    const size_t o = idx - nb;
    const int l = (int)(o / ktail), c = (int)(o % ktail);
    uint16_t v = 0;
    if (c < 3 * rank) {
      uint16_t hi, lo;
      split_bf16(A[(size_t)l * rank + c % rank] / (float)g, hi, lo);
      v = (c < 2 * rank) ? hi : lo;
    }
    a_ext_t[o] = v;
  }
}

hipError_t launch_prep_bwd(const float* A, const float* B, int L, int rank, int d_out, int g,
                           uint16_t* b_hl, uint16_t* a_ext_t, int ktail, hipStream_t st) {
  const size_t n = (size_t)2 * rank_pad32(rank) * d_out + (size_t)L * ktail;
  prep_bwd_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(A, B, L, rank, d_out, g, b_hl,
                                                               a_ext_t, ktail);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void du_finalize_kernel(const float* __restrict__ raw,
                                                          int ksplit, int T, int rank, float s,
                                                          const float2* __restrict__ rs,
                                                          float* __restrict__ dU,
                                                          uint16_t* __restrict__ du_ext,
                                                          int ktail) {
  const int rp = rank_pad32(rank);
  const size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (idx >= (size_t)T * ktail) return;
  const int t = (int)(idx / ktail), c = (int)(idx % ktail);
  uint16_t out = 0;
  if (c < 3 * rank) {
    const int k = c % rank;
    float v = 0.0f;
    for (int z = 0; z < ksplit; ++z) {
      const float* r = raw + ((size_t)z * T + t) * (2 * rp);
      v += r[k] + r[rp + k];
    }
    v *= s;
    if (c < rank) dU[(size_t)t * rank + k] = v;
    uint16_t hi, lo;
    split_bf16(v * rs[t].x, hi, lo);  // the backward tail rides on the scaled main product
    out = (c >= rank && c < 2 * rank) ? lo : hi;
  }
  du_ext[idx] = out;
}

hipError_t launch_du_finalize(const float* raw, int ksplit, int T, int rank, float s,
                              const float2* rs, float* dU, uint16_t* du_ext, int ktail,
                              hipStream_t st) {
  const size_t n = (size_t)T * ktail;
  du_finalize_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(raw, ksplit, T, rank, s, rs, dU,
                                                                  du_ext, ktail);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// dB = (sU)^T dy : contraction over tokens with a tiny output, on the bf16 matrix cores.
// A operand = (sU)^T hi/lo rows (token-contiguous in memory); B operand = dy, whose
// contraction index (token) is the strided one, so the 8-token fragments are gathered
// from the LDS tile with 16-bit reads.  Block = 128 output columns x one token slice;
// wavefront w owns columns [32w, 32w+32) and all hi/lo rows.
// ---------------------------------------------------------------------------------------
constexpr int DB_BN = 128;
constexpr int DB_DY_ROW = 136;  // bf16 per LDS row of the dy tile (128 + 8 pad)

template <int MT>  // number of 32-row tiles of the hi/lo operand = 2*rp/32
__global__ __launch_bounds__(256) void db_partial_kernel(const uint16_t* __restrict__ us_t,
                                                         int t_pad,
                                                         const uint16_t* __restrict__ dy, int T,
                                                         int d_out, int rank, int tsplit,
                                                         float* __restrict__ part) {
  constexpr int ROWS = 32 * MT;
  __shared__ __align__(16) uint16_t us_s[ROWS * LDS_ROW_72];
  __shared__ __align__(16) uint16_t dy_s[64 * DB_DY_ROW];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j0 = blockIdx.x * DB_BN;
  const int z = blockIdx.y;
  const int steps = ceil_div(t_pad / 64, tsplit);
  const int step_begin = z * steps, step_end = min(t_pad / 64, step_begin + steps);

  f32x16 acc[MT];
#pragma unroll
  for (int a = 0; a < MT; ++a)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[a][r] = 0.0f;

  for (int step = step_begin; step < step_end; ++step) {
    const int t0 = step * 64;
    for (int idx = tid; idx < ROWS * 8; idx += 256) {
      const int row = idx >> 3, ch = idx & 7;
      *reinterpret_cast<uint4*>(us_s + row * LDS_ROW_72 + 8 * ch) =
          *reinterpret_cast<const uint4*>(us_t + (size_t)row * t_pad + t0 + 8 * ch);
    }
    for (int idx = tid; idx < 64 * 16; idx += 256) {
      const int row = idx >> 4, ch = idx & 15;
      const int t = t0 + row, j = j0 + 8 * ch;
      uint4 v = {0, 0, 0, 0};
      if (t < T && j < d_out) v = *reinterpret_cast<const uint4*>(dy + (size_t)t * d_out + j);
      *reinterpret_cast<uint4*>(dy_s + row * DB_DY_ROW + 8 * ch) = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      union {
        bf16x8 v;
        uint16_t h[8];
      } bfrag;
      const uint16_t* src = dy_s + (kk * 16 + 8 * (lane >> 5)) * DB_DY_ROW + 32 * wave + (lane & 31);
#pragma unroll
      for (int e = 0; e < 8; ++e) bfrag.h[e] = src[e * DB_DY_ROW];
#pragma unroll
      for (int a = 0; a < MT; ++a) {
        const bf16x8 af = *reinterpret_cast<const bf16x8*>(
            us_s + (32 * a + (lane & 31)) * LDS_ROW_72 + kk * 16 + 8 * (lane >> 5));
        acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfrag.v, acc[a], 0, 0, 0);
      }
    }
    __syncthreads();
  }

  const int j = j0 + 32 * wave + (lane & 31);
  if (j < d_out) {
#pragma unroll
    for (int a = 0; a < MT / 2; ++a)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int k = 32 * a + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (k < rank)
          part[((size_t)z * rank + k) * d_out + j] = acc[a][r] + acc[a + MT / 2][r];
      }
  }
}

hipError_t launch_db_partial(const uint16_t* us_t, int t_pad, const uint16_t* dy, int T, int d_out,
                             int rank, int tsplit, float* part, hipStream_t st) {
  const int mt = 2 * rank_pad32(rank) / 32;
  dim3 grid(ceil_div(d_out, DB_BN), tsplit);
  if (mt == 2) db_partial_kernel<2><<<grid, 256, 0, st>>>(us_t, t_pad, dy, T, d_out, rank, tsplit, part);
  else if (mt == 4) db_partial_kernel<4><<<grid, 256, 0, st>>>(us_t, t_pad, dy, T, d_out, rank, tsplit, part);
  else if (mt == 6) db_partial_kernel<6><<<grid, 256, 0, st>>>(us_t, t_pad, dy, T, d_out, rank, tsplit, part);
  else if (mt == 8) db_partial_kernel<8><<<grid, 256, 0, st>>>(us_t, t_pad, dy, T, d_out, rank, tsplit, part);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// dA = P^T dU over a token slice, fp32 on the vector units (67 MFLOP at LLaMA-7B shapes).
// Block = 64 groups x all ranks; thread = 4 groups x up to 8 ranks (rank <= 128).
// ---------------------------------------------------------------------------------------
constexpr int DA_TT = 16;

__global__ __launch_bounds__(256) void da_partial_kernel(const float* __restrict__ P,
                                                         const float* __restrict__ dU, int T,
                                                         int L, int rank, int tsplit,
                                                         float* __restrict__ part) {
  __shared__ float p_s[DA_TT][64];
  __shared__ float du_s[DA_TT][128];
  const int tid = threadIdx.x;
  const int lq = tid >> 4, kq = tid & 15;
  const int l0 = blockIdx.x * 64;
  const int z = blockIdx.y;
  const int per = ceil_div(ceil_div(T, DA_TT), tsplit) * DA_TT;
  const int t_begin = z * per, t_end = min(T, t_begin + per);

  float acc[4][8];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[a][c] = 0.0f;

  for (int t0 = t_begin; t0 < t_end; t0 += DA_TT) {
    for (int idx = tid; idx < DA_TT * 64; idx += 256) {
      const int tt = idx >> 6, l = l0 + (idx & 63);
      p_s[tt][idx & 63] = (t0 + tt < t_end && l < L) ? P[(size_t)(t0 + tt) * L + l] : 0.0f;
    }
    for (int idx = tid; idx < DA_TT * 128; idx += 256) {
      const int tt = idx >> 7, k = idx & 127;
      du_s[tt][k] = (t0 + tt < t_end && k < rank) ? dU[(size_t)(t0 + tt) * rank + k] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int tt = 0; tt < DA_TT; ++tt) {
      float pv[4], dv[8];
#pragma unroll
      for (int a = 0; a < 4; ++a) pv[a] = p_s[tt][4 * lq + a];
#pragma unroll
      for (int c = 0; c < 8; ++c) dv[c] = du_s[tt][kq + 16 * c];
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[a][c] = __builtin_fmaf(pv[a], dv[c], acc[a][c]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int l = l0 + 4 * lq + a;
    if (l >= L) continue;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const int k = kq + 16 * c;
      if (k < rank) part[((size_t)z * L + l) * rank + k] = acc[a][c];
    }
  }
}

hipError_t launch_da_partial(const float* P, const float* dU, int T, int L, int rank, int tsplit,
                             float* part, hipStream_t st) {
  dim3 grid(ceil_div(L, 64), tsplit);
  da_partial_kernel<<<grid, 256, 0, st>>>(P, dU, T, L, rank, tsplit, part);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ part,
                                                              int nparts, size_t n,
                                                              float* __restrict__ out,
                                                              int accumulate) {
  const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i >= n) return;
  float v = accumulate ? out[i] : 0.0f;
  for (int z = 0; z < nparts; ++z) v += part[(size_t)z * n + i];
  out[i] = v;
}

hipError_t launch_reduce_partials(const float* part, int nparts, size_t n, float* out,
                                  int accumulate, hipStream_t st) {
  reduce_partials_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(part, nparts, n, out,
                                                                      accumulate);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Merge (Alg. 1 merge / App. B.3 in Eq. 1's zero-factor convention):
//   beta'[l,j] = beta[l,j] + (s/g) sum_k A[l,k] B[k,j]
// One thread per (group, 4 columns); row l of A is uniform over the block.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void merge_kernel(const float* beta,  // may alias beta_out
                                                    const float* __restrict__ A,
                                                    const float* __restrict__ B, int d_out,
                                                    int rank, float scale, float* beta_out) {
  const int l = blockIdx.y;
  const int j = (blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (j >= d_out) return;  // d_out is a multiple of 8
  const float* a = A + (size_t)l * rank;
  f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
  for (int k = 0; k < rank; ++k) {
    const float av = a[k];
    const f32x4 b = *reinterpret_cast<const f32x4*>(B + (size_t)k * d_out + j);
    acc.x = __builtin_fmaf(av, b.x, acc.x);
    acc.y = __builtin_fmaf(av, b.y, acc.y);
    acc.z = __builtin_fmaf(av, b.z, acc.z);
    acc.w = __builtin_fmaf(av, b.w, acc.w);
  }
  const f32x4 bt = *reinterpret_cast<const f32x4*>(beta + (size_t)l * d_out + j);
  f32x4 o;
  o.x = __builtin_fmaf(scale, acc.x, bt.x);
  o.y = __builtin_fmaf(scale, acc.y, bt.y);
  o.z = __builtin_fmaf(scale, acc.z, bt.z);
  o.w = __builtin_fmaf(scale, acc.w, bt.w);
  *reinterpret_cast<f32x4*>(beta_out + (size_t)l * d_out + j) = o;
}

hipError_t launch_merge(const float* beta, const float* A, const float* B, int L, int d_out,
                        int rank, int g, float s, float* beta_out, hipStream_t st) {
  dim3 grid(ceil_div(d_out / 4, 256), L);
  merge_kernel<<<grid, 256, 0, st>>>(beta, A, B, d_out, rank, s / (float)g, beta_out);
  return hipGetLastError();
}

}  // namespace qalora
