// Error-compensated code selection: the role the post-training quantizer plays in the paper's
// experiments (Sec. 4.1, quantization settings; App. B.1: the layer takes whatever codes, scales
// and zeros that quantizer hands over).  The published procedure, restated for W [d_in x d_out]
// with groups down the input rows: the rows are quantized in order; the error a row leaves,
// divided by the diagonal of U (the upper Cholesky factor of the inverse input Hessian,
// H^-1 = U^T U), is spread over the rows not yet quantized with the weights U[i, r], so that
// the output error tr((W - W~)^T H (W - W~)) shrinks; a group's beta and alpha are taken, by
// Eq. 1's min-max recipe, from the group's rows as they stand when its first row is reached;
// rows beyond the current block of kBlock rows receive the block's errors in one lazy update.
//
// Columns are independent, rows strictly sequential.  A block of 1024 threads owns 16 columns:
// thread (c, rl) is column c and row lane rl (64 of them).  Per block of rows: the 128 x 16
// tile of weights and the 128 x 128 diagonal block of U sit in LDS; every thread follows its
// column's row i redundantly (code, error), then the 64 row lanes update the tile rows behind
// i -- one barrier per row; afterwards the rows behind the block are updated 64 at a time from
// a staged 128 x 64 piece of U.  fp32 throughout, every sum in ascending row order with fused
// multiply-adds: the operation order is part of the definition, so the codes are reproducible
// bit for bit.
#include "common.hpp"
#include "kernels.hpp"

namespace qalora {

namespace {
constexpr int kBlock = 128;   // rows per lazy block (a multiple of every supported group size <= 128)
constexpr int kCols = 16;     // columns per thread block
constexpr int kLanes = 64;    // row lanes
constexpr int kThreads = kCols * kLanes;
constexpr int kLds = (kBlock * kCols * 2 + kBlock * kBlock) * 4;
}  // namespace

__global__ __launch_bounds__(kThreads) void compensate_kernel(const float* __restrict__ W,
                                                              const float* __restrict__ U, int d_in,
                                                              int d_out, int bits, int g,
                                                              float* __restrict__ work,
                                                              uint8_t* __restrict__ codes,
                                                              float* __restrict__ alpha,
                                                              float* __restrict__ beta) {
  extern __shared__ __align__(16) float lds[];
  float* tile = lds;                          // [kBlock][kCols] current weights of the block's rows
  float* err = tile + kBlock * kCols;         // [kBlock][kCols] errors of the block's rows
  float* Us = err + kBlock * kCols;           // [kBlock][kBlock] diagonal block of U, or [kBlock][kLanes]
  const int tid = threadIdx.x, c = tid & (kCols - 1), rl = tid >> 4;
  const int j = blockIdx.x * kCols + c;
  const bool col_ok = j < d_out;
  const float levels = (float)((1 << bits) - 1);

  // the block's columns of W become its working copy
  for (int r = rl; r < d_in; r += kLanes)
    if (col_ok) work[(size_t)r * d_out + j] = W[(size_t)r * d_out + j];
  __syncthreads();

  for (int i1 = 0; i1 < d_in; i1 += kBlock) {
    const int n = min(kBlock, d_in - i1);
    for (int r = rl; r < n; r += kLanes) tile[r * kCols + c] = col_ok ? work[(size_t)(i1 + r) * d_out + j] : 0.0f;
    for (int idx = tid; idx < n * kBlock; idx += kThreads) {
      const int i = idx / kBlock, r = idx - i * kBlock;
      Us[i * kBlock + r] = r < n ? U[(size_t)(i1 + i) * d_in + i1 + r] : 0.0f;
    }
    __syncthreads();
    float a = 1.0f, b = 0.0f;  // factors of the column's current group
    for (int i = 0; i < n; ++i) {
      if ((i1 + i) % g == 0) {  // a new group: min-max of its rows as they stand now (Eq. 1)
        float mn = tile[i * kCols + c], mx = mn;
        for (int q = i + 1; q < i + g; ++q) {
          const float w = tile[q * kCols + c];
          mn = w < mn ? w : mn;
          mx = w > mx ? w : mx;
        }
        a = __fdiv_rn(__fsub_rn(mx, mn), levels);
        if (!(a > 0.0f)) a = 0x1p-60f;
        b = mn;
        if (rl == 0 && col_ok) {
          const size_t o = (size_t)((i1 + i) / g) * d_out + j;
          alpha[o] = a;
          beta[o] = b;
        }
        // every row lane has read the group's rows before any lane updates them below (the
        // condition is uniform over the block)
        __syncthreads();
      }
      const float w = tile[i * kCols + c];
      float rq = rintf(__fdiv_rn(__fsub_rn(w, b), a));
      if (!(rq >= 0.0f)) rq = 0.0f;
      if (rq > levels) rq = levels;
      const float e = __fdiv_rn(__fsub_rn(w, __fmaf_rn(a, rq, b)), Us[i * kBlock + i]);
      if (rl == 0) {
        err[i * kCols + c] = e;
        if (col_ok) codes[(size_t)(i1 + i) * d_out + j] = (uint8_t)(int)rq;
      }
      for (int r = i + 1 + rl; r < n; r += kLanes)
        tile[r * kCols + c] = __fmaf_rn(-Us[i * kBlock + r], e, tile[r * kCols + c]);
      __syncthreads();  // row i + 1 is complete
    }
    // the block's errors onto the rows behind it, kLanes rows at a time
    for (int r0 = i1 + n; r0 < d_in; r0 += kLanes) {
      __syncthreads();  // the previous piece of U (or its diagonal block) has been used
      for (int idx = tid; idx < n * kLanes; idx += kThreads) {
        const int i = idx / kLanes, rr = idx - i * kLanes;
        Us[i * kLanes + rr] = r0 + rr < d_in ? U[(size_t)(i1 + i) * d_in + r0 + rr] : 0.0f;
      }
      __syncthreads();
      float acc = 0.0f;
      for (int i = 0; i < n; ++i) acc = __fmaf_rn(Us[i * kLanes + rl], err[i * kCols + c], acc);
      const int r = r0 + rl;
      if (r < d_in && col_ok) {
        const size_t o = (size_t)r * d_out + j;
        work[o] = __fsub_rn(work[o], acc);
      }
    }
    __syncthreads();  // this thread block's updates of `work` are visible to its next load
  }
}

// work: d_in * d_out fp32; codes: d_in * d_out bytes (canonical, one code per byte)
hipError_t launch_compensate(const float* W, const float* U, int d_in, int d_out, int bits, int g,
                             float* work, uint8_t* codes, float* alpha, float* beta, hipStream_t st) {
  if (kBlock % g != 0) return hipErrorInvalidValue;
  static std::atomic<uint64_t> granted{0};
  if (hipError_t e = grant_dynamic_lds(reinterpret_cast<const void*>(compensate_kernel), kLds, granted);
      e != hipSuccess)
    return e;
  compensate_kernel<<<ceil_div(d_out, kCols), kThreads, kLds, st>>>(W, U, d_in, d_out, bits, g, work, codes,
                                                                    alpha, beta);
  return hipGetLastError();
}

}  // namespace qalora
