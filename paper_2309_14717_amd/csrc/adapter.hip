// The low-rank branch of the QA-LoRA linear (Alg. 1; Sec. 3.3): group pooling of the
// input, the small products with A and B, their gradients, and the merge of the adapter
// into the zero factors (App. B.3).  All of it is tiny next to the two dense contractions;
// the kernels here are shaped for latency and for deterministic (fixed-order) reductions.
//
// Small fp32 factors that must go through the bf16 matrix cores are split as hi + lo
// (hi = bf16(v), lo = bf16(v - hi)); a product U.B is then evaluated as
// hi.hi + lo.hi + hi.lo, which is accurate to about 2^-16.
#include <algorithm>

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

// ---------------------------------------------------------------------------------------
// The "front" launch: every row-wise and elementwise preparation step of a forward or a
// backward call, as independent jobs of ONE kernel (the steps are tiny; launches are not).
//   rows job 1 : x -> row scale, fp16 scaled copy (forward), P = pool_g(x), U = P A (kept for
//                the backward, or transposed into us_t).  One wavefront per token, the row held in registers: a single
//                sweep of 128-bit loads gives the maximum (scale), the group sums (wavefront
//                butterfly over the g/8 lanes of a group) and the converted copy.
//   rows job 2 : dy -> row scale + fp16 scaled copy (backward)
//   factor job : the adapter folded into the zero factors, as the dense kernels' factor words
//   prep job   : hi/lo split of B into the operand layout of the dU product
// ---------------------------------------------------------------------------------------
constexpr int ROWS_PER_BLOCK = 4;  // one wavefront each
// 128-bit chunks per lane of a row that a wavefront holds in registers (64 lanes x 8 elements
// each): 8 covers rows of 4096 elements.  The launch is built for 8, 16 and 28 and takes the
// smallest that holds its longest row, so that rows up to 14336 elements are read once; the
// larger forms cost the launch occupancy, which is why they are not the only one.
constexpr int ROW_BATCH = 8;
constexpr int TR_TOK = 32;         // tokens per block of the transpose job

// One linear's adapter among those that share the input x (a single layer is one part).
struct FrontPart {
  const float* A;       // [L, rank]
  const float* B;       // [rank, d_out]
  float s;
  int rank;
  int col0, d_out;      // its columns [col0, col0 + d_out) of the (wide) layer
  float* u_keep;        // optional [T, rank]: s U in fp32, for a later launch's transpose job
  const float* u_kept;  // transpose job: the [T, rank] rows an earlier launch kept
  uint16_t* us_t;       // optional [2*rp, t_pad]
  uint16_t* b_hl;       // backward: [2*rp, d_out]
  int prep_block0;      // first block of its share of the prep job
};

struct FrontArgs {
  // rows job 1 (x)
  const uint16_t* x;
  int T, d_in;
  float2* rs_x;         // optional
  uint16_t* x16;        // optional, [T, d_in]
  int pool;             // rows job 1 also pools x and forms U = P A of every part
  int g;
  float* P_out;         // optional [T, L]
  int t_pad;
  FrontPart part[MAX_PARTS];
  int n_parts;
  int tr_blocks;        // transpose job: blocks per part (t_pad / TR_TOK), or 0
  // rows job 2 (dy): scale + convert only
  const uint16_t* y;
  int Ty, d_y;
  float2* rs_y;
  uint16_t* y16;
  // factor job (see factor_block): the dense kernels' factor words
  const float* f_alpha; // [L, d_out]
  const float* f_beta;  // [L, d_out]
  int f_fold;           // fold the parts' adapters in
  float f_inv_g, f_mid; // 1 / g; 2^(N-1)
  int f_L, f_dout, f_cols;  // f_cols: columns per block, a power of two <= 16
  int f_cw;             // columns per block of the adapter-free form: 32 or 64
  uint32_t* f_words;    // forward: [L, d_out] words at the per-column scale
  float* f_inv;         // forward: [d_out] 1 / S of each column
  float* f_const;       // backward: [L, d_out] beta' + mid alpha, fp32 (scaled by a later launch)
  float* f_max;         // optional [nb_fac]: bound on |W~'| over each block's columns
  const float* f_known; // backward, optional [nb_fac]: those bounds as an earlier launch on the
                        // same operands left them -- the call's S is then known here, and the
                        // words are written at once (f_words, f_inv[0]; no f_const)
  int nb_rows1, nb_rows2, nb_tr, nb_prep, nb_fac;
};

// Power of two S = 2^e that brings a magnitude bound m to [2^13, 2^14), as (S, 1/S); (1, 1) for
// m = 0 or a non-finite m.  Every |W~'| S then stays below 2^14 in fp16, its largest factor keeps
// 11 significant bits, and the products with activations scaled to below 2^15 leave the fp32
// accumulator ample room.
__device__ __forceinline__ float2 factor_scale(float m) {
  const int E = (int)(__float_as_uint(m) >> 23) & 255;
  if (m == 0.0f || E == 255) return float2{1.0f, 1.0f};
  int e = 140 - E;  // m in [2^(E-127), 2^(E-126))
  e = e > 100 ? 100 : (e < -100 ? -100 : e);
  return float2{__uint_as_float((uint32_t)(127 + e) << 23), __uint_as_float((uint32_t)(127 - e) << 23)};
}

// The factor job.  The adapted layer is the quantized layer with the zero factors
//   beta'[l,j] = beta[l,j] + (s/g) sum_k A[l,k] B[k,j]                  (App. B.3)
// so the dense kernels need no low-rank branch of their own: this job folds the adapter into
// the zero factors for the call at hand (fp32, k in order) and hands them over in the form the
// kernels multiply with: one word per (group, column), fp16(alpha S) | fp16(c S) << 16, where
// c = beta' + mid alpha is the weight at the mid code mid = 2^(N-1) and S a power of two taken
// from the bound |c| + mid |alpha| >= |W~'|.
// A block owns f_cols columns and every group: thread (c, lg) takes column c and groups lg,
// lg + 256 / f_cols, ...; B's columns sit in LDS, the rows of A come as broadcast loads, and c
// is parked in LDS until the column's bound is known.  Forward: S per column, decided here.
// Backward (the scale must not vary along the output columns, which are the contraction index
// there): c goes out in fp32 with the block's bound, and a later launch scales by the call's S.
// Without an adapter there is nothing to fold: the job is elementwise plus the bounds, and a
// block takes 64 or 32 columns (whole 128-byte lines of alpha and beta) and makes two sweeps
// over them, the second served by the cache, instead of parking c in LDS.  It fills the same f_cols-wide slots
// of f_max as the folding form would.
__device__ __forceinline__ void factor_block_plain(const FrontArgs& a, int bid, float* red, int tid) {
  const int CW = a.f_cw, NLG = 256 / CW;  // columns per block; threads per column
  const int c = tid & (CW - 1), lg = tid / CW;
  const int L = a.f_L, dout = a.f_dout;
  const int j = bid * CW + c;
  const bool col_ok = j < dout;
  const float mid = a.f_mid;
  float m = 0.0f;
  constexpr int NB = 8;  // rows of alpha and of beta in flight per thread
  if (col_ok) {
    for (int l0 = lg; l0 < L; l0 += NLG * NB) {
      float al[NB], be[NB];
#pragma unroll
      for (int q = 0; q < NB; ++q) {
        const int l = min(l0 + NLG * q, L - 1);
        al[q] = a.f_alpha[(size_t)l * dout + j];
        be[q] = a.f_beta[(size_t)l * dout + j];
      }
#pragma unroll
      for (int q = 0; q < NB; ++q) {
        const int l = l0 + NLG * q;
        if (l < L) {
          const float cst = __builtin_fmaf(mid, al[q], be[q]);
          m = fmaxf(m, fabsf(cst) + mid * fabsf(al[q]));
          if (a.f_const) a.f_const[(size_t)l * dout + j] = cst;
        }
      }
    }
  }
  red[tid] = m;
  __syncthreads();
  float cm = 0.0f;  // column bound
  for (int q = 0; q < NLG; ++q) cm = fmaxf(cm, red[q * CW + c]);
  if (a.f_max) {
    __syncthreads();
    red[tid] = cm;
    __syncthreads();
    const int per = CW / a.f_cols, slots = ceil_div(dout, a.f_cols);  // f_cols-wide slots of this block
    if (tid < per && bid * per + tid < slots) {
      float bm = 0.0f;
      for (int q = 0; q < a.f_cols; ++q) bm = fmaxf(bm, red[tid * a.f_cols + q]);
      a.f_max[bid * per + tid] = bm;
    }
  }
  if (a.f_known) {
    __syncthreads();
    float km = 0.0f;
    const int slots = ceil_div(dout, a.f_cols);
    for (int i = tid; i < slots; i += 256) km = fmaxf(km, a.f_known[i]);
    red[tid] = km;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
      if (tid < off) red[tid] = fmaxf(red[tid], red[tid + off]);
      __syncthreads();
    }
    cm = red[0];
  }
  if (!a.f_words) return;
  const float2 sc = factor_scale(cm);
  if (a.f_known) {
    if (bid == 0 && tid == 0) a.f_inv[0] = sc.y;
  } else if (lg == 0 && col_ok) {
    a.f_inv[j] = sc.y;
  }
  if (col_ok) {
    for (int l0 = lg; l0 < L; l0 += NLG * NB) {
      float al[NB], be[NB];
#pragma unroll
      for (int q = 0; q < NB; ++q) {
        const int l = min(l0 + NLG * q, L - 1);
        al[q] = a.f_alpha[(size_t)l * dout + j];
        be[q] = a.f_beta[(size_t)l * dout + j];
      }
#pragma unroll
      for (int q = 0; q < NB; ++q) {
        const int l = l0 + NLG * q;
        if (l < L) {
          const f32x2 v = {al[q] * sc.x, __builtin_fmaf(mid, al[q], be[q]) * sc.x};
          a.f_words[(size_t)l * dout + j] = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
        }
      }
    }
  }
}

__device__ __forceinline__ void factor_block(const FrontArgs& a, int bid, float* lds, int tid) {
  if (!a.f_fold) {
    factor_block_plain(a, bid, lds, tid);
    return;
  }
  const int FC = a.f_cols, NLG = 256 / FC;
  const int c = tid & (FC - 1), lg = tid / FC;
  const int L = a.f_L, dout = a.f_dout;
  const int j0 = bid * FC, j = j0 + c;
  // the part this block's columns belong to (part widths are multiples of the block's width)
  int pi = 0;
  for (int q = 1; q < a.n_parts; ++q)
    if (j0 >= a.part[q].col0) pi = q;
  const FrontPart& pt = a.part[pi];
  const int rank = pt.rank, pj0 = j0 - pt.col0, pdout = pt.d_out;
  const float* __restrict__ pA = pt.A;
  const float sg = pt.s * a.f_inv_g;
  const bool col_ok = j < dout;
  const int bs = rank + 4;          // floats per staged column of B
  float* tile = lds;                // [L][FC]
  float* Bs = tile + (size_t)L * FC;  // [FC][bs]
  float* red = Bs + FC * bs;        // [256]
  float m = 0.0f;
  // what a thread does with one element of A B once it has it: the constant of the factor word
  // into the LDS tile, its bound into the thread's running maximum
  auto finish = [&](int l, float ab, float al, float be) {
    float cst = 0.0f, bound = 0.0f;
    if (col_ok) {
      const float bp = __builtin_fmaf(sg, ab, be);
      cst = __builtin_fmaf(a.f_mid, al, bp);
      bound = fabsf(cst) + a.f_mid * fabsf(al);
    }
    tile[(size_t)l * FC + c] = cst;
    m = fmaxf(m, bound);
  };
  if (FC == 16) {
    // 16 columns: A B on the matrix cores in fp32 (v_mfma_f32_16x16x4_f32), a 16-group tile per
    // wavefront at a time.  Lane (n, kb) = (lane % 16, lane / 16) supplies row n of the A tile and
    // column n of B for the k values kb kq .. kb kq + kq - 1 (kq = a quarter of the rank, rounded
    // up: the instruction's four k slots are four contiguous runs of k, so a lane's operands are
    // contiguous in memory), and receives rows 4 kb .. 4 kb + 3 of column n -- the thread's
    // column c, as in the plain form.
    const int lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, kb = lane >> 4;
    const int kq = (rank + 3) >> 2;  // <= 32
    const bool vec4 = (rank & 3) == 0 && (kq & 3) == 0;
    const int kbase = kb * kq;
    const uint32_t bcol = (uint32_t)kbase * (uint32_t)pdout + (uint32_t)(pj0 + n);  // element index in B
    const bool bcol_ok = pj0 + n < pdout;
    // operands in chunks of eight k values (whole fragments in registers would cost the row jobs
    // of the same launch their occupancy; the other wavefronts of the unit cover the latency)
    constexpr int KC = 8;
    float bres[16];
#pragma unroll
    for (int q = 0; q < 16; ++q)
      bres[q] = (kq <= 16 && bcol_ok && q < kq && kbase + q < rank) ? pt.B[bcol + (uint32_t)q * (uint32_t)pdout] : 0.0f;
    for (int l0 = 16 * wave; l0 < L; l0 += 64) {
      const uint32_t arow = (uint32_t)min(l0 + n, L - 1) * (uint32_t)rank + (uint32_t)kbase;  // rows past the end repeat the last one, unused
      // alpha and beta of the four elements this lane will receive: requested now, used after
      // the product
      float al4[4], be4[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const size_t o = (size_t)min(l0 + 4 * kb + r, L - 1) * dout + (col_ok ? j : 0);
        al4[r] = a.f_alpha[o];
        be4[r] = a.f_beta[o];
      }
      f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
      if (kq <= 16) {
        // rank <= 64: the lane's share of B is sixteen values held for the whole block, its share
        // of the tile's rows of A sixteen more, requested together with alpha and beta -- one
        // round trip to memory per tile
        float af[16];
        if (vec4) {
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            f32x4 v = {0.0f, 0.0f, 0.0f, 0.0f};
            if (4 * q4 < kq) v = *reinterpret_cast<const f32x4*>(pA + arow + 4 * q4);
#pragma unroll
            for (int q = 0; q < 4; ++q) af[4 * q4 + q] = v[q];
          }
        } else {
#pragma unroll
          for (int q = 0; q < 16; ++q) af[q] = (q < kq && kbase + q < rank) ? pA[arow + q] : 0.0f;
        }
#pragma unroll
        for (int q = 0; q < 16; ++q)
          if (q < kq) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(af[q], bres[q], acc, 0, 0, 0);
      } else
      for (int i0 = 0; i0 < kq; i0 += KC) {
        float av[KC], bv[KC];
        if (vec4 && i0 + KC <= kq) {
          const f32x4 v0 = *reinterpret_cast<const f32x4*>(pA + arow + i0);
          const f32x4 v1 = *reinterpret_cast<const f32x4*>(pA + arow + i0 + 4);
#pragma unroll
          for (int q = 0; q < 4; ++q) av[q] = v0[q], av[4 + q] = v1[q];
        } else {
#pragma unroll
          for (int q = 0; q < KC; ++q) av[q] = (i0 + q < kq && kbase + i0 + q < rank) ? pA[arow + i0 + q] : 0.0f;
        }
#pragma unroll
        for (int q = 0; q < KC; ++q)
          bv[q] = (bcol_ok && i0 + q < kq && kbase + i0 + q < rank) ? pt.B[bcol + (uint32_t)(i0 + q) * (uint32_t)pdout] : 0.0f;
#pragma unroll
        for (int q = 0; q < KC; ++q) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[q], bv[q], acc, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int l = l0 + 4 * kb + r;
        if (l < L) finish(l, acc[r], al4[r], be4[r]);
      }
    }
  } else {
  for (int idx = tid; idx < FC * rank; idx += 256) {
    const int cc = idx & (FC - 1), k = idx / FC;
    Bs[cc * bs + k] = (pj0 + cc < pdout) ? pt.B[(size_t)k * pdout + pj0 + cc] : 0.0f;
  }
  __syncthreads();
  constexpr int GB = 4;  // groups per thread in flight
  const bool vec = (rank & 3) == 0;
  for (int lb = lg; lb < L; lb += NLG * GB) {
    float acc[GB];
#pragma unroll
    for (int i = 0; i < GB; ++i) acc[i] = 0.0f;
    if (vec) {
#pragma unroll 2
      for (int k = 0; k < rank; k += 4) {
        const f32x4 b = *reinterpret_cast<const f32x4*>(Bs + c * bs + k);
#pragma unroll
        for (int i = 0; i < GB; ++i) {
          const int l = min(lb + i * NLG, L - 1);  // rows past the end repeat the last one, unused
          const f32x4 av = *reinterpret_cast<const f32x4*>(pA + (size_t)l * rank + k);
#pragma unroll
          for (int q = 0; q < 4; ++q) acc[i] = __builtin_fmaf(av[q], b[q], acc[i]);
        }
      }
    } else {
      for (int k = 0; k < rank; ++k) {
        const float b = Bs[c * bs + k];
#pragma unroll
        for (int i = 0; i < GB; ++i) {
          const int l = min(lb + i * NLG, L - 1);
          acc[i] = __builtin_fmaf(pA[(size_t)l * rank + k], b, acc[i]);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < GB; ++i) {
      const int l = lb + i * NLG;
      if (l < L) {
        const size_t o = (size_t)l * dout + (col_ok ? j : 0);
        finish(l, acc[i], a.f_alpha[o], a.f_beta[o]);
      }
    }
  }
  }
  red[tid] = m;
  __syncthreads();
  float cm = 0.0f;  // bound of column c over all groups
  for (int q = 0; q < NLG; ++q) cm = fmaxf(cm, red[q * FC + c]);
  if (a.f_max) {  // the block's bound, for a launch that needs one scale for the whole matrix
    __syncthreads();
    red[tid] = cm;
    __syncthreads();
    if (tid == 0) {
      float bm = 0.0f;
      for (int q = 0; q < FC; ++q) bm = fmaxf(bm, red[q]);
      a.f_max[bid] = bm;
    }
  }
  if (a.f_known) {  // one scale for the call, from the bounds an earlier launch left
    __syncthreads();
    float km = 0.0f;
    for (int i = tid; i < ceil_div(dout, FC); i += 256) km = fmaxf(km, a.f_known[i]);
    red[tid] = km;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
      if (tid < off) red[tid] = fmaxf(red[tid], red[tid + off]);
      __syncthreads();
    }
    cm = red[0];
  }
  if (a.f_words) {
    const float2 sc = factor_scale(cm);
    if (a.f_known) {
      if (bid == 0 && tid == 0) a.f_inv[0] = sc.y;
    } else if (lg == 0 && col_ok) {
      a.f_inv[j] = sc.y;
    }
    if (col_ok) {
      constexpr int WB = 8;  // groups per batch: their alpha loads go out together
      for (int lb = lg; lb < L; lb += NLG * WB) {
        float al[WB];
#pragma unroll
        for (int q = 0; q < WB; ++q) al[q] = a.f_alpha[(size_t)min(lb + q * NLG, L - 1) * dout + j];
#pragma unroll
        for (int q = 0; q < WB; ++q) {
          const int l = lb + q * NLG;
          if (l < L) {
            const f32x2 v = {al[q] * sc.x, tile[(size_t)l * FC + c] * sc.x};
            a.f_words[(size_t)l * dout + j] = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
          }
        }
      }
    }
  } else if (col_ok) {
    for (int l = lg; l < L; l += NLG) a.f_const[(size_t)l * dout + j] = tile[(size_t)l * FC + c];
  }
}

// One wavefront processes one bf16 row: returns the row scale; optionally writes the fp16
// scaled copy and the group averages (to P_s, LDS, [L]).
template <int RB>
__device__ __forceinline__ float2 process_row(const uint16_t* __restrict__ src, int cols,
                                              uint16_t* __restrict__ dst16, float* P_s, int g,
                                              int lane) {
  const int nch = cols / 8;
  const int lpg = g > 0 ? g / 8 : 0;
  const bool butterfly = P_s && lpg <= 64 && (lpg & (lpg - 1)) == 0;
  const float inv_g = g > 0 ? 1.0f / (float)g : 0.0f;
  uint32_t amax = 0;
  uint4 v[RB];
  const bool resident = nch <= 64 * RB;  // whole row fits the register batch
  for (int base = 0; base < nch; base += 64 * RB) {
#pragma unroll
    for (int c = 0; c < RB; ++c) {
      const int ch = base + c * 64 + lane;
      v[c] = ch < nch ? *reinterpret_cast<const uint4*>(src + 8 * ch) : uint4{0, 0, 0, 0};
    }
#pragma unroll
    for (int c = 0; c < RB; ++c) {
      amax = max_abs_bits(v[c], amax);
      if (butterfly) {
        const int ch = base + c * 64 + lane;
        const uint32_t w[4] = {v[c].x, v[c].y, v[c].z, v[c].w};
        float sum = 0.0f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          sum += bf16_bits_to_f32(w[e] & 0xffffu);
          sum += __uint_as_float(w[e] & 0xffff0000u);
        }
        for (int off = 1; off < lpg; off <<= 1) sum += __shfl_xor(sum, off, 64);
        if (ch < nch && (lane & (lpg - 1)) == 0) P_s[ch / lpg] = sum * inv_g;
      }
    }
  }
  amax = wave_max_u32(amax);
  const float2 sc = scale_from_maxbits(amax);
  if (dst16) {
    if (resident) {
#pragma unroll
      for (int c = 0; c < RB; ++c) {
        const int ch = c * 64 + lane;
        if (ch < nch)
          *reinterpret_cast<uint4*>(dst16 + 8 * ch) = bf16x8_to_f16x8_scaled(v[c], sc.x);
      }
    } else {  // second sweep, served by L2
      for (int ch = lane; ch < nch; ch += 64)
        *reinterpret_cast<uint4*>(dst16 + 8 * ch) =
            bf16x8_to_f16x8_scaled(*reinterpret_cast<const uint4*>(src + 8 * ch), sc.x);
    }
  }
  if (P_s && !butterfly) {  // group sizes the butterfly does not cover: plain loop
    const int L = cols / g;
    for (int l = lane; l < L; l += 64) {
      float sum = 0.0f;
      for (int q = 0; q < g; ++q) sum += bf16_bits_to_f32(src[l * g + q]);
      P_s[l] = sum * inv_g;
    }
  }
  return sc;
}

template <int RB>
__global__ __launch_bounds__(256) void front_kernel(const FrontArgs a) {
  extern __shared__ float P_all[];  // [ROWS_PER_BLOCK][L] when pooling
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int bid = blockIdx.x;
  // The factor job's blocks are the longest-running ones: started last they would finish after
  // everything else instead of under it.  But all of them first would hold most of the chip's
  // block slots while the row jobs, which carry the launch's memory traffic, wait; so the two
  // kinds alternate until one runs out.
  {
    const int n_other = (int)gridDim.x - a.nb_fac;
    const int m = min(a.nb_fac, n_other);
    if (bid < 2 * m)
      bid = (bid & 1) ? a.nb_fac + (bid >> 1) : (bid >> 1);
    else
      bid = (a.nb_fac > m) ? bid - m : bid;  // the rest of the longer kind, in order
  }
  if (bid < a.nb_fac) {
    // Block ids are dealt round-robin to the 8 XCDs, each with its own L2.  The folding form
    // works on 64-byte pieces of the 128-byte lines of alpha, beta and the words, so column
    // blocks that share a line go to the same XCD: XCD x takes a contiguous run of them.
    const int q = a.nb_fac >> 3, rem = a.nb_fac & 7, x = bid & 7;
    const int fid = a.f_fold ? x * q + min(x, rem) + (bid >> 3) : bid;
    factor_block(a, fid, P_all, tid);
    return;
  }
  bid -= a.nb_fac;
  if (bid < a.nb_rows1) {
    // ---- rows job 1: x ---------------------------------------------------------------
    const int t = bid * ROWS_PER_BLOCK + wave;
    const int L = a.pool ? a.d_in / a.g : 0;
    float* P_s = a.pool ? P_all + wave * L : nullptr;
    float2 sc = float2{1.0f, 1.0f};
    if (t < a.T) {
      sc = process_row<RB>(a.x + (size_t)t * a.d_in, a.d_in,
                       a.x16 ? a.x16 + (size_t)t * a.d_in : nullptr, P_s, a.g, lane);
      if (lane == 0 && a.rs_x) a.rs_x[t] = sc;
    } else if (a.pool) {
      for (int l = lane; l < L; l += 64) P_s[l] = 0.0f;
    }
    if (!a.pool) return;
    __syncthreads();
    if (t < a.T && a.P_out)
      for (int l = lane; l < L; l += 64) a.P_out[(size_t)t * L + l] = P_s[l];
    // U = P A of every part for the block's 4 tokens, cooperatively: thread (k, q) covers a
    // quarter of the groups for all 4 tokens (each A element is loaded once per block), then
    // the quarters are added in fixed order.
    float* part = P_all + ROWS_PER_BLOCK * L;  // [4 quarters][4 tokens][128]
    const int lq0 = (L * wave) / 4, lq1 = (L * (wave + 1)) / 4;
    for (int pi = 0; pi < a.n_parts; ++pi) {
      const FrontPart& pt = a.part[pi];
      const int rank = pt.rank, rp = rank_pad32(rank);
      if (pi > 0) __syncthreads();  // the previous part's sums have been read
      for (int k = lane; k < rank; k += 64) {
        float u[ROWS_PER_BLOCK] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll 4
        for (int l = lq0; l < lq1; ++l) {
          const float av = pt.A[(size_t)l * rank + k];
#pragma unroll
          for (int r = 0; r < ROWS_PER_BLOCK; ++r) u[r] = __builtin_fmaf(P_all[r * L + l], av, u[r]);
        }
#pragma unroll
        for (int r = 0; r < ROWS_PER_BLOCK; ++r) part[(wave * ROWS_PER_BLOCK + r) * 128 + k] = u[r];
      }
      __syncthreads();
      if (t < a.T) {
        for (int k = lane; k < rp; k += 64) {
          float u = 0.0f;
          if (k < rank) {
            u = ((part[(0 * ROWS_PER_BLOCK + wave) * 128 + k] + part[(1 * ROWS_PER_BLOCK + wave) * 128 + k]) +
                 part[(2 * ROWS_PER_BLOCK + wave) * 128 + k]) +
                part[(3 * ROWS_PER_BLOCK + wave) * 128 + k];
            u *= pt.s;
          }
          uint16_t hi, lo;
          if (pt.u_keep && k < rank) pt.u_keep[(size_t)t * rank + k] = u;
          if (pt.us_t) {
            split_bf16(u, hi, lo);  // zero for the padding rows k >= rank
            pt.us_t[(size_t)k * a.t_pad + t] = hi;
            pt.us_t[(size_t)(rp + k) * a.t_pad + t] = lo;
          }
        }
      } else if (pt.us_t && t < a.t_pad) {
        // token padding of the transposed operand must read as zero
        for (int k = lane; k < 2 * rp; k += 64) pt.us_t[(size_t)k * a.t_pad + t] = 0;
      }
    }
    return;
  }
  bid -= a.nb_rows1;
  if (bid < a.nb_rows2) {
    // ---- rows job 2: dy -> scale + fp16 copy ----------------------------------------------
    const int t = bid * ROWS_PER_BLOCK + wave;
    if (t < a.Ty) {
      const float2 sc = process_row<RB>(a.y + (size_t)t * a.d_y, a.d_y, a.y16 + (size_t)t * a.d_y,
                                    nullptr, 0, lane);
      if (lane == 0) a.rs_y[t] = sc;
    }
    return;
  }
  bid -= a.nb_rows2;
  if (bid < a.nb_tr) {
    // ---- transpose job: TR_TOK tokens of the kept s U -> token-contiguous hi/lo rows --------
    // (the same values and the same split as rows job 1 writes when it computes U itself).
    // The loads go out in batches of eight per thread before any is used: the launch is
    // memory-saturated by the row jobs, and a round trip per element would outlast them.
    float* tile = P_all;  // [TR_TOK][rank + 1]
    const FrontPart& pt = a.part[bid / a.tr_blocks];
    const int t0 = (bid % a.tr_blocks) * TR_TOK, rank = pt.rank, rp = rank_pad32(rank), ld = rank + 1;
    const int n = TR_TOK * rank;
    for (int e0 = 0; e0 < n; e0 += 8 * 256) {
      float r[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int e = e0 + j * 256 + tid;
        const int t = e / rank;
        r[j] = (e < n && t0 + t < a.T) ? pt.u_kept[(size_t)t0 * rank + e] : 0.0f;
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int e = e0 + j * 256 + tid;
        const int t = e / rank;
        if (e < n) tile[t * ld + (e - t * rank)] = r[j];
      }
    }
    __syncthreads();
    const int tl = lane & (TR_TOK - 1);
    for (int k = 2 * wave + (lane >> 5); k < rp; k += 8) {
      uint16_t hi, lo;
      split_bf16(k < rank ? tile[tl * ld + k] : 0.0f, hi, lo);  // zero for padding rows and tokens
      pt.us_t[(size_t)k * a.t_pad + t0 + tl] = hi;
      pt.us_t[(size_t)(rp + k) * a.t_pad + t0 + tl] = lo;
    }
    return;
  }
  bid -= a.nb_tr;
  // ---- prep job: hi/lo split of every part's B for its dU product -----------------------
  int pi = 0;
  for (int q = 1; q < a.n_parts; ++q)
    if (bid >= a.part[q].prep_block0) pi = q;
  const FrontPart& pt = a.part[pi];
  const size_t idx = (size_t)(bid - pt.prep_block0) * 256 + tid;
  const int rp = rank_pad32(pt.rank);
  const size_t nb = (size_t)2 * rp * pt.d_out;
  if (idx < nb) {
    // b_hl rows = hi(B) then lo(B) (rows padded to rp with zeros)
    const int row = (int)(idx / pt.d_out), j = (int)(idx % pt.d_out);
    const int k = row % rp;
    uint16_t v = 0;
    if (k < pt.rank) {
      uint16_t hi, lo;
      split_bf16(pt.B[(size_t)k * pt.d_out + j], hi, lo);
      v = (row < rp) ? hi : lo;
    }
    pt.b_hl[idx] = v;
  }
}

// Few rows, no adapter work (the post-merge forward of a small batch): with one wavefront per
// row the launch is a handful of wavefronts walking 16-44 KB each, batch after batch, at the
// latency of a single wavefront.  Here a whole block takes a row: every thread holds its share
// of it in registers (up to WIDE_BATCH 16-byte pieces: rows of up to 32768 elements), the four
// wavefronts' maxima meet in LDS, and the row is converted from the registers -- one pass, one
// memory round trip.  Same scale and same conversion as process_row, bit for bit.
constexpr int WIDE_BATCH = 16;
constexpr int kWideRows = 1024;  // beyond this the one-wavefront-per-row launch fills the chip
__global__ __launch_bounds__(256) void front_wide_kernel(const uint16_t* __restrict__ src, int cols,
                                                         float2* __restrict__ rs,
                                                         uint16_t* __restrict__ dst16) {
  __shared__ uint32_t wave_amax[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const size_t row = (size_t)blockIdx.x * cols;
  const int nch = cols / 8;
  uint4 v[WIDE_BATCH];
#pragma unroll
  for (int c = 0; c < WIDE_BATCH; ++c) {
    const int ch = c * 256 + tid;
    v[c] = ch < nch ? *reinterpret_cast<const uint4*>(src + row + 8 * ch) : uint4{0, 0, 0, 0};
  }
  uint32_t amax = 0;
#pragma unroll
  for (int c = 0; c < WIDE_BATCH; ++c) amax = max_abs_bits(v[c], amax);
  amax = wave_max_u32(amax);
  if (lane == 0) wave_amax[wave] = amax;
  __syncthreads();
  amax = max(max(wave_amax[0], wave_amax[1]), max(wave_amax[2], wave_amax[3]));
  const float2 sc = scale_from_maxbits(amax);
  if (tid == 0 && rs) rs[blockIdx.x] = sc;
  if (dst16) {
#pragma unroll
    for (int c = 0; c < WIDE_BATCH; ++c) {
      const int ch = c * 256 + tid;
      if (ch < nch) *reinterpret_cast<uint4*>(dst16 + row + 8 * ch) = bf16x8_to_f16x8_scaled(v[c], sc.x);
    }
  }
}

// Columns per block of the factor job: as many (up to 16) as keep its LDS tile of L x columns
// fp32 values within 32 KB, so that the row jobs of the same launch keep their occupancy.
static int factor_cols(int L) {
  int fc = 16;
  while (fc > 1 && (size_t)L * fc * 4 > 32 * 1024) fc >>= 1;
  return fc;
}

static hipError_t launch_front(FrontArgs a, hipStream_t st) {
  const bool prep = a.n_parts > 0 && a.part[0].b_hl;
  const bool transposes = a.n_parts > 0 && a.part[0].u_kept;
  if (a.x && !a.pool && !a.y && !prep && !transposes && a.T <= kWideRows && a.d_in % 8 == 0 &&
      a.d_in <= 256 * 8 * WIDE_BATCH) {
    // few rows: a block per row; the factor job (if any) follows as a launch of its own
    front_wide_kernel<<<a.T, 256, 0, st>>>(a.x, a.d_in, a.rs_x, a.x16);
    if (hipError_t e = hipGetLastError(); e != hipSuccess || !a.f_alpha) return e;
    a.x = nullptr;
  }
  int max_rank = 0;
  for (int p = 0; p < a.n_parts; ++p) max_rank = a.part[p].rank > max_rank ? a.part[p].rank : max_rank;
  a.nb_rows1 = a.x ? ceil_div((a.pool && a.part[0].us_t) ? a.t_pad : a.T, ROWS_PER_BLOCK) : 0;
  a.nb_rows2 = a.y ? ceil_div(a.Ty, ROWS_PER_BLOCK) : 0;
  a.nb_prep = 0;
  if (prep)
    for (int p = 0; p < a.n_parts; ++p) {
      a.part[p].prep_block0 = a.nb_prep;
      a.nb_prep += (int)(((size_t)2 * rank_pad32(a.part[p].rank) * a.part[p].d_out + 255) / 256);
    }
  a.tr_blocks = transposes ? a.t_pad / TR_TOK : 0;
  a.nb_tr = a.tr_blocks * a.n_parts;
  size_t smem =
      (a.x && a.pool) ? ((size_t)ROWS_PER_BLOCK * (a.d_in / a.g) + 4 * ROWS_PER_BLOCK * 128) * sizeof(float) : 0;
  const size_t tr_smem = (size_t)TR_TOK * (max_rank + 1) * sizeof(float);
  if (a.nb_tr > 0 && smem < tr_smem) smem = tr_smem;
  a.nb_fac = 0;
  if (a.f_alpha) {
    a.f_cols = factor_cols(a.f_L);
    // adapter-free form: the widest column tile that still leaves more blocks than compute units
    a.f_cw = a.f_dout / 64 >= 384 ? 64 : 32;
    a.nb_fac = a.f_fold ? ceil_div(a.f_dout, a.f_cols) : ceil_div(a.f_dout, a.f_cw);
    const size_t f_smem =
        a.f_fold ? ((size_t)a.f_L * a.f_cols + (size_t)a.f_cols * (max_rank + 4) + 256 + 4) * sizeof(float)
                 : 256 * sizeof(float);
    if (smem < f_smem) smem = f_smem;
  }
  constexpr size_t kFrontLdsMax = 160 * 1024;  // a compute unit's LDS
  if (smem > kFrontLdsMax) return hipErrorInvalidValue;
  const int nblocks = a.nb_rows1 + a.nb_rows2 + a.nb_tr + a.nb_fac + a.nb_prep;
  if (nblocks == 0) return hipSuccess;
  // the register batch that holds the launch's longest row (two sweeps beyond 14336 elements)
  const int longest = std::max(a.x ? a.d_in : 0, a.y ? a.d_y : 0);
  auto launch = [&](auto rb) -> hipError_t {
    constexpr int RB = decltype(rb)::value;
    if (smem > 48 * 1024) {
      static std::atomic<uint64_t> granted{0};  // per instantiation
      if (hipError_t e = grant_dynamic_lds(reinterpret_cast<const void*>(front_kernel<RB>), (int)kFrontLdsMax,
                                           granted);
          e != hipSuccess)
        return e;
    }
    front_kernel<RB><<<nblocks, 256, smem, st>>>(a);
    return hipGetLastError();
  };
  // ... when the rows are most of the launch: the larger batches cost occupancy, which a launch
  // whose factor job is the longer part pays back with interest (measured at 5120 x 13824 with
  // 2048 tokens: 36.0 us with two sweeps, 40.9 us with one)
  const size_t row_bytes = ((a.x ? (size_t)a.T * a.d_in : 0) + (a.y ? (size_t)a.Ty * a.d_y : 0)) * 4;
  const size_t fac_bytes = a.f_alpha ? (size_t)a.f_L * a.f_dout * 12 : 0;
  if (row_bytes >= 8 * fac_bytes) {
    if (longest > 512 * 8 && longest <= 512 * 16) return launch(std::integral_constant<int, 16>{});
    if (longest > 512 * 16 && longest <= 512 * 28) return launch(std::integral_constant<int, 28>{});
  }
  return launch(std::integral_constant<int, ROW_BATCH>{});
}

static void set_parts(FrontArgs& a, const AdapterParts& ap) {
  a.n_parts = ap.n;
  for (int p = 0; p < ap.n; ++p) {
    a.part[p].A = ap.A[p];
    a.part[p].B = ap.B[p];
    a.part[p].s = ap.s[p];
    a.part[p].rank = ap.rank[p];
    a.part[p].col0 = ap.col0[p];
    a.part[p].d_out = ap.d_out[p];
  }
}

static void set_factor_job(FrontArgs& a, const FactorJob& f) {
  a.f_alpha = f.alpha; a.f_beta = f.beta; a.f_fold = f.parts.n > 0;
  if (a.n_parts == 0) set_parts(a, f.parts);
  a.f_inv_g = 1.0f / (float)f.g; a.f_mid = (float)(1 << (f.bits - 1));
  a.f_L = f.L; a.f_dout = f.d_out;
  a.f_words = f.words; a.f_inv = f.inv_scale; a.f_const = f.cst; a.f_max = f.block_max;
  a.f_known = f.known_max;
}

int factor_job_blocks(int L, int d_out) { return ceil_div(d_out, factor_cols(L)); }
int factor_job_cols(int L) { return factor_cols(L); }

hipError_t launch_factor_job(const FactorJob& f, hipStream_t st) {
  FrontArgs a{};
  set_factor_job(a, f);
  return launch_front(a, st);
}

hipError_t launch_front_forward(const uint16_t* x, int T, int d_in, float2* rs, uint16_t* x16,
                                const AdapterParts& parts, int g, float* P_keep,
                                float* const* u_keep, const FactorJob& fac, hipStream_t st) {
  FrontArgs a{};
  a.x = x; a.T = T; a.d_in = d_in; a.rs_x = rs; a.x16 = x16; a.g = g;
  if (parts.n > 0 && P_keep) {  // only a caller that keeps them needs P and s P A here
    set_parts(a, parts);
    a.pool = 1;
    a.P_out = P_keep;
    for (int p = 0; p < parts.n; ++p) a.part[p].u_keep = u_keep[p];
  }
  set_factor_job(a, fac);
  return launch_front(a, st);
}

hipError_t launch_front_backward(const uint16_t* dy, int T, int d_out, float2* rs_dy,
                                 uint16_t* dy16, const uint16_t* x, int d_in,
                                 const AdapterParts& parts, int g, float* P, uint16_t* const* us_t,
                                 int t_pad, uint16_t* const* b_hl, const float* const* u_kept,
                                 const FactorJob& fac, hipStream_t st) {
  FrontArgs a{};
  a.y = dy; a.Ty = T; a.d_y = d_out; a.rs_y = rs_dy; a.y16 = dy16; a.g = g;
  if (parts.n > 0) {
    set_parts(a, parts);
    const bool kept = u_kept != nullptr;
    a.x = kept ? nullptr : x;  // with the kept rows, P is the caller's and us_t is a transpose
    a.pool = kept ? 0 : 1;
    a.T = T; a.d_in = d_in;
    a.P_out = P; a.t_pad = t_pad;
    for (int p = 0; p < parts.n; ++p) {
      a.part[p].us_t = us_t[p];
      a.part[p].b_hl = b_hl[p];
      a.part[p].u_kept = kept ? u_kept[p] : nullptr;
    }
  }
  if (fac.alpha) set_factor_job(a, fac);
  return launch_front(a, st);
}

// Second stage of the backward direction's factor words: S for the call from the first
// stage's per-block bounds (every block reduces them itself: a few hundred values), then
// words[i] = fp16(alpha[i] S) | fp16(c[i] S) << 16.  Block 0 leaves 1 / S for the epilogue.
__global__ __launch_bounds__(256) void factor_scale_kernel(const f32x4* __restrict__ alpha,
                                                           const f32x4* __restrict__ cst,
                                                           const float* __restrict__ block_max,
                                                           int nmax, size_t n4,
                                                           uint32_t* __restrict__ words,
                                                           float* __restrict__ inv_scale) {
  __shared__ float red[256];
  float m = 0.0f;
  for (int i = threadIdx.x; i < nmax; i += 256) m = fmaxf(m, block_max[i]);
  red[threadIdx.x] = m;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + off]);
    __syncthreads();
  }
  const float2 sc = factor_scale(red[0]);
  if (blockIdx.x == 0 && threadIdx.x == 0) inv_scale[0] = sc.y;
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
    const f32x4 al = alpha[i], c = cst[i];
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    u32x4 w;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const f32x2 v = {al[q] * sc.x, c[q] * sc.x};
      w[q] = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
    }
    reinterpret_cast<u32x4*>(words)[i] = w;
  }
}

hipError_t launch_factor_scale(const float* alpha, const float* cst, const float* block_max, int nmax,
                               size_t n, uint32_t* words, float* inv_scale, hipStream_t st) {
  const size_t n4 = n / 4;  // d_out is a multiple of 8
  const unsigned blocks = (unsigned)((n4 + 1023) / 1024 < 1024 ? (n4 + 1023) / 1024 : 1024);
  factor_scale_kernel<<<blocks, 256, 0, st>>>(reinterpret_cast<const f32x4*>(alpha),
                                              reinterpret_cast<const f32x4*>(cst), block_max, nmax, n4,
                                              words, inv_scale);
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

struct DbArgs {
  const uint16_t* us_t;  // bf16 [2*rp, t_pad]: hi rows, then lo rows, of (s U)^T
  int t_pad;
  const uint16_t* dy;    // bf16 [T, d_out], rows dy_ld elements apart (a column slice of a wider dy)
  int dy_ld;
  int T, d_out, rank, tsplit;
  float* part;           // [tsplit][rank, d_out]
};
template <int MT>
constexpr int db_lds_bytes() { return (32 * MT * LDS_ROW_72 + 64 * DB_DY_ROW) * 2; }

template <int MT>  // number of 32-row tiles of the hi/lo operand = 2*rp/32
__device__ __forceinline__ void db_partial_block(const DbArgs& a, int bx, int z,
                                                 unsigned char* lds) {
  constexpr int ROWS = 32 * MT;
  const uint16_t* __restrict__ us_t = a.us_t;
  const uint16_t* __restrict__ dy = a.dy;
  float* __restrict__ part = a.part;
  const int t_pad = a.t_pad, T = a.T, d_out = a.d_out, rank = a.rank, tsplit = a.tsplit;
  uint16_t* us_s = reinterpret_cast<uint16_t*>(lds);  // [ROWS][LDS_ROW_72]
  uint16_t* dy_s = us_s + ROWS * LDS_ROW_72;          // [64][DB_DY_ROW]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j0 = bx * DB_BN;
  const int steps = ceil_div(t_pad / 64, tsplit);
  const int step_begin = z * steps, step_end = min(t_pad / 64, step_begin + steps);

  f32x16 acc[MT];
#pragma unroll
  for (int a = 0; a < MT; ++a)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[a][r] = 0.0f;

  // The tiles of step+1 are fetched into registers while step runs on the matrix cores (one
  // loop body with the three phases guarded, so that each phase is written once and the
  // staging registers stay plain registers).
  constexpr int US_LOADS = ROWS * 8 / 256, DY_LOADS = 64 * 16 / 256;
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4 us_r[US_LOADS], dy_r[DY_LOADS];
  for (int step = step_begin - 1; step < step_end; ++step) {
    const bool have = step >= step_begin;  // registers hold the tiles of `step`
    if (have) {
#pragma unroll
      for (int q = 0; q < US_LOADS; ++q) {
        const int idx = tid + 256 * q, row = idx >> 3, ch = idx & 7;
        *reinterpret_cast<u32x4*>(us_s + row * LDS_ROW_72 + 8 * ch) = us_r[q];
      }
#pragma unroll
      for (int q = 0; q < DY_LOADS; ++q) {
        const int idx = tid + 256 * q, row = idx >> 4, ch = idx & 15;
        *reinterpret_cast<u32x4*>(dy_s + row * DB_DY_ROW + 8 * ch) = dy_r[q];
      }
      __syncthreads();
    }
    if (step + 1 < step_end) {
      const int t0 = (step + 1) * 64;
#pragma unroll
      for (int q = 0; q < US_LOADS; ++q) {
        const int idx = tid + 256 * q, row = idx >> 3, ch = idx & 7;
        us_r[q] = *reinterpret_cast<const u32x4*>(us_t + (size_t)row * t_pad + t0 + 8 * ch);
      }
#pragma unroll
      for (int q = 0; q < DY_LOADS; ++q) {
        const int idx = tid + 256 * q, row = idx >> 4, ch = idx & 15;
        const int t = t0 + row, j = j0 + 8 * ch;
        dy_r[q] = u32x4{0, 0, 0, 0};
        if (t < T && j < d_out) dy_r[q] = *reinterpret_cast<const u32x4*>(dy + (size_t)t * a.dy_ld + j);
      }
    }
    if (have) {
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        // B fragment: eight tokens of one column, gathered with 16-bit reads and packed in pairs
        const uint16_t* src = dy_s + (kk * 16 + 8 * (lane >> 5)) * DB_DY_ROW + 32 * wave + (lane & 31);
        uint32_t h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = src[e * DB_DY_ROW];
        const u32x4 packed = {h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
        const bf16x8 bfrag = __builtin_bit_cast(bf16x8, packed);
#pragma unroll
        for (int a = 0; a < MT; ++a) {
          const bf16x8 af = *reinterpret_cast<const bf16x8*>(
              us_s + (32 * a + (lane & 31)) * LDS_ROW_72 + kk * 16 + 8 * (lane >> 5));
          acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfrag, acc[a], 0, 0, 0);
        }
      }
      __syncthreads();
    }
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

// ---------------------------------------------------------------------------------------
// dA = P^T dU over a token slice, fp32 on the vector units (67 MFLOP at LLaMA-7B shapes),
// fused with the finalisation of dU: dU[t,k] = s * sum_z (raw[z][t][k] + raw[z][t][rp+k]) is
// rebuilt from the split-K partials of the dU product while staging.
// Block = 64 groups x all ranks; thread = 4 groups x up to 8 ranks.
// ---------------------------------------------------------------------------------------
constexpr int DA_TT = 16;

struct DaArgs {
  const float* P;    // [T, L] group averages of x
  const float* raw;  // [ksplit][T, 2*rp] split-K partials of dy [B_hi | B_lo]^T
  int ksplit;
  float s;
  int T, L, rank, tsplit;
  float* part;       // [tsplit][L, rank]
};
constexpr int da_lds_bytes() { return DA_TT * (64 + 128) * 4; }

__device__ __forceinline__ void da_partial_block(const DaArgs& a, int bx, int z,
                                                 unsigned char* lds) {
  const float* __restrict__ P = a.P;
  const float* __restrict__ raw = a.raw;
  float* __restrict__ part = a.part;
  const int ksplit = a.ksplit, T = a.T, L = a.L, rank = a.rank, tsplit = a.tsplit;
  const float s = a.s;
  float (*p_s)[64] = reinterpret_cast<float (*)[64]>(lds);                        // [DA_TT][64]
  float (*du_s)[128] = reinterpret_cast<float (*)[128]>(lds + DA_TT * 64 * 4);    // [DA_TT][128]
  const int tid = threadIdx.x;
  const int lq = tid >> 4, kq = tid & 15;
  const int l0 = bx * 64;
  const int rp = rank_pad32(rank);
  // The split-K partials are read through a buffer resource: the lane offset is fixed per
  // (token, rank) element and the partial index lives in the scalar offset, so the four
  // partials' loads in flight together cost no address registers.  (The host refuses token
  // counts for which the partials exceed 32-bit byte offsets.)
  constexpr uint32_t kDaOob = 0xffff0000u;
  const uint32_t q_stride = (uint32_t)T * (uint32_t)(2 * rp) * 4u;
  const __amdgpu_buffer_rsrc_t rs_raw = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<float*>(raw), 0, (int)((uint32_t)ksplit * q_stride), 0x00020000);
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
    // dU of this thread's eight (token, rank) elements: the loads of one split-K partial are
    // all issued before any is used (element loop unrolled inside the partial loop)
    constexpr int DU_E = DA_TT * 128 / 256;
    float duv[DU_E];
    uint32_t voff[DU_E];  // byte offset of (t, k) inside one split-K partial; elements that do
                          // not exist point past the buffer and read as zero
#pragma unroll
    for (int e = 0; e < DU_E; ++e) {
      const int idx = tid + 256 * e;
      const int t = t0 + (idx >> 7), k = idx & 127;
      duv[e] = 0.0f;
      voff[e] = (t < t_end && k < rank) ? ((uint32_t)t * (uint32_t)(2 * rp) + (uint32_t)k) * 4u : kDaOob;
    }
    constexpr int QB = 2;  // split-K partials whose loads are in flight together
    for (int q0 = 0; q0 < ksplit; q0 += QB) {
      float ld[QB][DU_E][2];
#pragma unroll
      for (int j = 0; j < QB; ++j) {
        const bool live = q0 + j < ksplit;  // uniform
        const uint32_t so = live ? (uint32_t)(q0 + j) * q_stride : 0u;
#pragma unroll
        for (int e = 0; e < DU_E; ++e) {
          const uint32_t v = live ? voff[e] : kDaOob;
          ld[j][e][0] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_raw, (int)v, (int)so, 0));
          ld[j][e][1] = __builtin_bit_cast(
              float, __builtin_amdgcn_raw_buffer_load_b32(rs_raw, (int)v, (int)(so + (uint32_t)rp * 4u), 0));
        }
      }
#pragma unroll
      for (int j = 0; j < QB; ++j)  // partial order, as a plain loop over q would add them
#pragma unroll
        for (int e = 0; e < DU_E; ++e)
          if (q0 + j < ksplit) duv[e] += ld[j][e][0] + ld[j][e][1];
    }
#pragma unroll
    for (int e = 0; e < DU_E; ++e) {
      const int idx = tid + 256 * e;
      const int tt = idx >> 7, k = idx & 127;
      du_s[tt][k] = duv[e] * s;
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

// Both gradient jobs in ONE launch (neither needs the other; the dB blocks, the longer job,
// come first): blocks [0, db_blocks) are (column block, token slice) pairs of dB, the rest
// (group block, token slice) pairs of dA.
// (Three wavefronts per SIMD fit in registers up to rank 64; the larger ranks' accumulators
// need the room of one.)
template <int MT>
__global__ __launch_bounds__(256, MT <= 4 ? 3 : 1) void adapter_grads_kernel(const DbArgs db, const DaArgs da,
                                                            int db_bx, int db_blocks, int da_bx) {
  constexpr int kLds = db_lds_bytes<MT>() > da_lds_bytes() ? db_lds_bytes<MT>() : da_lds_bytes();
  __shared__ __align__(16) unsigned char lds[kLds];
  const int b = blockIdx.x;
  if (b < db_blocks) {
    db_partial_block<MT>(db, b % db_bx, b / db_bx, lds);
  } else {
    const int c = b - db_blocks;
    da_partial_block(da, c % da_bx, c / da_bx, lds);
  }
}

hipError_t launch_adapter_grads(const uint16_t* us_t, int t_pad, const uint16_t* dy, int dy_ld, int T,
                                int d_out, int rank, int tsplit_b, float* db_part, const float* P,
                                const float* raw, int ksplit, float s, int L, int tsplit_a,
                                float* da_part, hipStream_t st) {
  const DbArgs db{us_t, t_pad, dy, dy_ld, T, d_out, rank, tsplit_b, db_part};
  const DaArgs da{P, raw, ksplit, s, T, L, rank, tsplit_a, da_part};
  const int db_bx = ceil_div(d_out, DB_BN), db_blocks = db_bx * tsplit_b;
  const int da_bx = ceil_div(L, 64), da_blocks = da_bx * tsplit_a;
  const int mt = 2 * rank_pad32(rank) / 32;
  const dim3 grid(db_blocks + da_blocks);
  if (mt == 2) adapter_grads_kernel<2><<<grid, 256, 0, st>>>(db, da, db_bx, db_blocks, da_bx);
  else if (mt == 4) adapter_grads_kernel<4><<<grid, 256, 0, st>>>(db, da, db_bx, db_blocks, da_bx);
  else if (mt == 6) adapter_grads_kernel<6><<<grid, 256, 0, st>>>(db, da, db_bx, db_blocks, da_bx);
  else if (mt == 8) adapter_grads_kernel<8><<<grid, 256, 0, st>>>(db, da, db_bx, db_blocks, da_bx);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

// out[i] = (accumulate ? out[i] : 0) + sum_z part[z][i] in a fixed order, for two outputs in
// one launch.  Block = 64 outputs x 4 part groups: thread (o, q) adds parts q, q+4, q+8, ...
// (coalesced across o, loads independent so they pipeline), then the four group sums are
// added in order 0..3.
__global__ __launch_bounds__(256) void reduce2_kernel(const float* __restrict__ part_a,
                                                      int nparts_a, size_t n_a,
                                                      float* __restrict__ out_a,
                                                      const float* __restrict__ part_b,
                                                      int nparts_b, size_t n_b,
                                                      float* __restrict__ out_b, int accumulate,
                                                      int blocks_a) {
  __shared__ float sums[4][64];
  const int o = threadIdx.x & 63, q = threadIdx.x >> 6;
  const bool second = (int)blockIdx.x >= blocks_a;
  const float* part = second ? part_b : part_a;
  const int nparts = second ? nparts_b : nparts_a;
  const size_t n = second ? n_b : n_a;
  float* out = second ? out_b : out_a;
  const size_t i = (size_t)(second ? blockIdx.x - blocks_a : blockIdx.x) * 64 + o;
  float v = 0.0f;
  if (i < n) {
#pragma unroll 8
    for (int z = q; z < nparts; z += 4) v += part[(size_t)z * n + i];
  }
  sums[q][o] = v;
  __syncthreads();
  if (q == 0 && i < n) {
    float r = accumulate ? out[i] : 0.0f;
    r += ((sums[0][o] + sums[1][o]) + sums[2][o]) + sums[3][o];
    out[i] = r;
  }
}

hipError_t launch_reduce2(const float* part_a, int nparts_a, size_t n_a, float* out_a,
                          const float* part_b, int nparts_b, size_t n_b, float* out_b,
                          int accumulate, hipStream_t st) {
  const int blocks_a = (int)((n_a + 63) / 64), blocks_b = (int)((n_b + 63) / 64);
  reduce2_kernel<<<blocks_a + blocks_b, 256, 0, st>>>(part_a, nparts_a, n_a, out_a, part_b,
                                                       nparts_b, n_b, out_b, accumulate, blocks_a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Merge (Alg. 1 merge / App. B.3 in Eq. 1's zero-factor convention):
//   beta'[l,j] = beta[l,j] + (s/g) sum_k A[l,k] B[k,j]
// One thread per (GL groups, 4 columns): a row of B fetched for one k serves GL groups, so the
// L2 traffic for B is 1/GL of what one group per thread would draw; the GL rows of A are
// uniform over the block.  The sum over k runs in k order for every output.
// ---------------------------------------------------------------------------------------
template <int GL>
__global__ __launch_bounds__(256) void merge_kernel(const float* beta,  // may alias beta_out
                                                    const float* __restrict__ A,
                                                    const float* __restrict__ B, int L, int d_out,
                                                    int rank, float scale, float* beta_out) {
  const int l0 = blockIdx.y * GL;
  const int j = (blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (j >= d_out) return;  // d_out is a multiple of 8
  // beta of this thread's elements is requested first and used last: its trip to HBM runs
  // under the whole product
  f32x4 bt[GL];
#pragma unroll
  for (int u = 0; u < GL; ++u)
    bt[u] = *reinterpret_cast<const f32x4*>(beta + (size_t)min(l0 + u, L - 1) * d_out + j);
  f32x4 acc[GL];
#pragma unroll
  for (int u = 0; u < GL; ++u) acc[u] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  auto step = [&](int k, const f32x4 b) {
#pragma unroll
    for (int u = 0; u < GL; ++u) {
      const int l = min(l0 + u, L - 1);  // rows past the end repeat the last one, unused
      const float av = A[(size_t)l * rank + k];
#pragma unroll
      for (int c = 0; c < 4; ++c) acc[u][c] = __builtin_fmaf(av, b[c], acc[u][c]);
    }
  };
  // rows of B in batches of eight, the next batch in flight while the current one is used
  constexpr int KB = 8;
  const int nb = rank / KB;
  f32x4 cur[KB], nxt[KB];
  auto fetch = [&](f32x4 (&dst)[KB], int k) {
#pragma unroll
    for (int q = 0; q < KB; ++q) dst[q] = *reinterpret_cast<const f32x4*>(B + (size_t)(k + q) * d_out + j);
  };
  if (nb > 0) fetch(cur, 0);
  for (int ib = 0; ib < nb; ++ib) {
    if (ib + 1 < nb) fetch(nxt, (ib + 1) * KB);
#pragma unroll
    for (int q = 0; q < KB; ++q) step(ib * KB + q, cur[q]);
    if (ib + 1 < nb) {
#pragma unroll
      for (int q = 0; q < KB; ++q) cur[q] = nxt[q];
    }
  }
  for (int k = nb * KB; k < rank; ++k) step(k, *reinterpret_cast<const f32x4*>(B + (size_t)k * d_out + j));
#pragma unroll
  for (int u = 0; u < GL; ++u) {
    const int l = l0 + u;
    if (l >= L) break;
    f32x4 o;
#pragma unroll
    for (int c = 0; c < 4; ++c) o[c] = __builtin_fmaf(scale, acc[u][c], bt[u][c]);
    *reinterpret_cast<f32x4*>(beta_out + (size_t)l * d_out + j) = o;
  }
}

hipError_t launch_merge(const float* beta, const float* A, const float* B, int L, int d_out,
                        int rank, int g, float s, float* beta_out, hipStream_t st) {
  const int bx = ceil_div(d_out / 4, 256);
  const float scale = s / (float)g;
  if (bx * ceil_div(L, 8) >= 200) {  // enough blocks for the chip at eight groups per thread
    merge_kernel<8><<<dim3(bx, ceil_div(L, 8)), 256, 0, st>>>(beta, A, B, L, d_out, rank, scale, beta_out);
  } else {
    merge_kernel<2><<<dim3(bx, ceil_div(L, 2)), 256, 0, st>>>(beta, A, B, L, d_out, rank, scale, beta_out);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Zero-point interchange (App. B.1 / Alg. 1 write W~ = alpha (code - z); Eq. 1 writes
// W~ = alpha code + beta): beta = -(alpha z), z = -(beta / alpha), one IEEE operation each.
// ---------------------------------------------------------------------------------------
template <bool TO_ZERO_POINT>
__global__ __launch_bounds__(256) void zero_point_kernel(const f32x4* __restrict__ alpha,
                                                         const f32x4* __restrict__ in,
                                                         f32x4* __restrict__ out, size_t n4) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  const f32x4 a = alpha[i], v = in[i];
  f32x4 o;
#pragma unroll
  for (int c = 0; c < 4; ++c) o[c] = TO_ZERO_POINT ? -__fdiv_rn(v[c], a[c]) : -__fmul_rn(a[c], v[c]);
  out[i] = o;
}

hipError_t launch_zero_point(const float* alpha, const float* in, float* out, size_t n, bool to_zero_point,
                             hipStream_t st) {
  const size_t n4 = n / 4;  // d_out is a multiple of 8
  const unsigned blocks = (unsigned)((n4 + 255) / 256);
  if (to_zero_point)
    zero_point_kernel<true><<<blocks, 256, 0, st>>>(reinterpret_cast<const f32x4*>(alpha),
                                                    reinterpret_cast<const f32x4*>(in),
                                                    reinterpret_cast<f32x4*>(out), n4);
  else
    zero_point_kernel<false><<<blocks, 256, 0, st>>>(reinterpret_cast<const f32x4*>(alpha),
                                                     reinterpret_cast<const f32x4*>(in),
                                                     reinterpret_cast<f32x4*>(out), n4);
  return hipGetLastError();
}

}  // namespace qalora
