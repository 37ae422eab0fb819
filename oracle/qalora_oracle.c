/*
 * QA-LoRA CPU oracle  --  TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, obviously-correct statement of the quantization-aware adapted
 * linear layer, written from the paper (arXiv 2309.14717).  Only the tests, the
 * smoke check and the benchmark's "cpu_baseline" leg may call it.  It shares no
 * source, header, table or helper with the HIP path and never touches a GPU.
 *
 * Conventions (0-based): W is [D_in x D_out]; group l of column j covers rows
 * i in [l*g, (l+1)*g), l = i / g (Sec. 3.3; App. B.1).  Codes are integers in
 * {0..2^N-1}; alpha, beta are the scaling / zero factors of Eq. 1, one pair per
 * (group, column), stored [L x D_out] row-major.  A is [L x r], B is [r x D_out].
 * Pooling is the group AVERAGE; Alg. 1 / App. B.2 use the group SUM, which is the
 * same family with s replaced by s*g (the *_zp_sum twins below use the paper's
 * literal zero-point + sum convention and are tested to agree).
 *
 * Precision: quantize follows a fixed fp32 recipe (so codes/alpha/beta can be
 * compared bit for bit); everything else accumulates in fp64 from the exact
 * input values.
 *
 * Pins (tests/test_oracle_*.py): brute force on tiny inputs with an independent
 * exact-rational implementation, the min-max bound |W - W~| <= alpha/2, code
 * range and extremes, integer round trip, the merge invariant of App. B.3,
 * reduction to ordinary LoRA (Sec. 3.1) through a library matmul, finite
 * differences for the backward (which the paper does not print), the L = 1
 * rank-one special case (Sec. 3.3), and Table 2's parameter counts.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int qo_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Round a double to the nearest bfloat16 value (ties to even), returned as double.
 * Used only by the "declared precision" mode, which mimics operand rounding of a
 * bf16 matrix unit; the definition mode never calls it. */
static double round_to_bf16(double v) {
  float f = (float)v;
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7f800000u) == 0x7f800000u) return (double)f; /* inf / nan unchanged */
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  u &= 0xffff0000u;
  memcpy(&f, &u, 4);
  return (double)f;
}

/* ------------------------------------------------------------------------- */
/* Eq. 1 applied per group of g consecutive rows of each column (Sec. 3.3).   */
/* fp32 recipe, in this exact order:                                          */
/*   mn, mx  : running strict-compare min / max down the group's rows         */
/*   beta    = mn                                                             */
/*   alpha   = (mx - mn) / (2^N - 1)      one subtract, one IEEE divide       */
/*   alpha not > 0 (constant group, or underflow): alpha = 2^-60, all codes 0 */
/*     (Eq. 1 gives alpha = 0 and 0/0 codes there; any alpha > 0 with codes 0  */
/*     dequantises to beta exactly, and one far below every real step keeps   */
/*     alpha * code negligible however the product is later evaluated)        */
/*   code    = clamp(rint((w - beta) / alpha), 0, 2^N - 1)   ties to even     */
/* Returns 0, or -1 on bad arguments.                                         */
/* ------------------------------------------------------------------------- */
int qo_quantize(const float* W, int d_in, int d_out, int bits, int g,
                uint8_t* codes, float* alpha, float* beta) {
  if (!W || !codes || !alpha || !beta) return -1;
  if (d_in <= 0 || d_out <= 0 || bits < 1 || bits > 8 || g <= 0 || d_in % g) return -1;
  const int L = d_in / g;
  const int qmax = (1 << bits) - 1;
  const float levels = (float)qmax;
#pragma omp parallel for schedule(static)
  for (int j = 0; j < d_out; ++j) {
    for (int l = 0; l < L; ++l) {
      const int i0 = l * g;
      float mn = W[(size_t)i0 * d_out + j];
      float mx = mn;
      for (int i = i0 + 1; i < i0 + g; ++i) {
        const float w = W[(size_t)i * d_out + j];
        if (w < mn) mn = w;
        if (w > mx) mx = w;
      }
      const float range = mx - mn;
      float a = range / levels;
      const int degenerate = !(a > 0.0f);
      if (degenerate) a = 0x1p-60f;
      alpha[(size_t)l * d_out + j] = a;
      beta[(size_t)l * d_out + j] = mn;
      for (int i = i0; i < i0 + g; ++i) {
        int c = 0;
        if (!degenerate) {
          const float d = W[(size_t)i * d_out + j] - mn;
          const float q = d / a;
          const float r = rintf(q);
          c = (int)r;
          if (c < 0) c = 0;
          if (c > qmax) c = qmax;
        }
        codes[(size_t)i * d_out + j] = (uint8_t)c;
      }
    }
  }
  return 0;
}

/* ------------------------------------------------------------------------- */
/* Error-compensated code selection: the role the post-training quantizer of   */
/* the paper's experiments plays (Sec. 4.1, quantization settings; App. B.1:   */
/* the layer takes whatever (codes, scales, zeros) that quantizer produced).    */
/* The published procedure, restated: the input rows of W are quantized one     */
/* after the other, and the error each row leaves is spread over the rows not   */
/* yet quantized, weighted by the upper Cholesky factor U of the inverse of the */
/* layer's input Hessian H (H^-1 = U^T U), so that the OUTPUT error under the   */
/* calibration inputs, tr((W - W~)^T H (W - W~)), is reduced.  Per column j:    */
/*   at the first row of a group: beta, alpha from the group's CURRENT rows,    */
/*                                by the recipe of qo_quantize                   */
/*   c   = clamp(rint((w_i - beta) / alpha), 0, 2^N - 1)                          */
/*   e   = (w_i - (alpha c + beta)) / U[i,i]                                      */
/*   w_r -= U[i,r] e     for the rows r > i                                       */
/* with the updates of rows beyond the current block of `block` rows applied    */
/* lazily, once per block, as the published procedure does.  fp32 throughout,   */
/* every sum in ascending row order, products fused (fmaf): this order IS the   */
/* definition both sides implement, so codes can be compared bit for bit.       */
/* `block` must be a multiple of g.  U = identity gives qo_quantize exactly.     */
/* Returns 0, or -1 on bad arguments.                                           */
/* ------------------------------------------------------------------------- */
int qo_quantize_compensated(const float* W, int d_in, int d_out, int bits, int g, const float* U,
                            int block, uint8_t* codes, float* alpha, float* beta) {
  if (!W || !U || !codes || !alpha || !beta) return -1;
  if (d_in <= 0 || d_out <= 0 || bits < 1 || bits > 8 || g <= 0 || d_in % g) return -1;
  if (block <= 0 || block % g) return -1;
  const int qmax = (1 << bits) - 1;
  const float levels = (float)qmax;
  float* work = (float*)malloc((size_t)d_in * d_out * sizeof(float));
  float* err = (float*)malloc((size_t)block * d_out * sizeof(float));
  if (!work || !err) {
    free(work);
    free(err);
    return -1;
  }
  memcpy(work, W, (size_t)d_in * d_out * sizeof(float));
  for (int i1 = 0; i1 < d_in; i1 += block) {
    const int i2 = i1 + block < d_in ? i1 + block : d_in;
#pragma omp parallel for schedule(static)
    for (int j = 0; j < d_out; ++j) {  /* columns are independent */
      for (int i = i1; i < i2; ++i) {
        const int l = i / g;
        if (i % g == 0) {
          float mn = work[(size_t)i * d_out + j];
          float mx = mn;
          for (int q = i + 1; q < i + g; ++q) {
            const float w = work[(size_t)q * d_out + j];
            if (w < mn) mn = w;
            if (w > mx) mx = w;
          }
          float a = (mx - mn) / levels;
          if (!(a > 0.0f)) a = 0x1p-60f;
          alpha[(size_t)l * d_out + j] = a;
          beta[(size_t)l * d_out + j] = mn;
        }
        const float a = alpha[(size_t)l * d_out + j], b = beta[(size_t)l * d_out + j];
        const float w = work[(size_t)i * d_out + j];
        const float d = w - b;
        const float q = d / a;
        float rq = rintf(q);
        if (!(rq >= 0.0f)) rq = 0.0f;  /* clamp before the conversion (also catches NaN) */
        if (rq > levels) rq = levels;
        const int c = (int)rq;
        codes[(size_t)i * d_out + j] = (uint8_t)c;
        const float wq = fmaf(a, (float)c, b);
        const float e = (w - wq) / U[(size_t)i * d_in + i];
        err[(size_t)(i - i1) * d_out + j] = e;
        for (int r = i + 1; r < i2; ++r)
          work[(size_t)r * d_out + j] = fmaf(-U[(size_t)i * d_in + r], e, work[(size_t)r * d_out + j]);
      }
    }
#pragma omp parallel for schedule(static)
    for (int r = i2; r < d_in; ++r) {  /* the block's errors, onto the rows behind it */
      for (int j = 0; j < d_out; ++j) {
        float acc = 0.0f;
        for (int i = i1; i < i2; ++i)
          acc = fmaf(U[(size_t)i * d_in + r], err[(size_t)(i - i1) * d_out + j], acc);
        work[(size_t)r * d_out + j] -= acc;
      }
    }
  }
  free(work);
  free(err);
  return 0;
}

/* W~[i,j] = alpha[i/g, j] * code[i,j] + beta[i/g, j]      (Eq. 1)             */
/* lrow = (i / g) * d_out is the offset of row i's group in alpha / beta.         */
static inline double wtilde(const uint8_t* codes, const float* alpha, const float* beta,
                            int d_out, size_t lrow, int i, int j, int round_bf16) {
  double w = (double)alpha[lrow + j] * (double)codes[(size_t)i * d_out + j] +
             (double)beta[lrow + j];
  return round_bf16 ? round_to_bf16(w) : w;
}

void qo_dequantize(const uint8_t* codes, const float* alpha, const float* beta,
                   int d_in, int d_out, int g, double* Wt) {
#pragma omp parallel for schedule(static)
  for (int i = 0; i < d_in; ++i) {
    const size_t lrow = (size_t)(i / g) * d_out;
    for (int j = 0; j < d_out; ++j)
      Wt[(size_t)i * d_out + j] = wtilde(codes, alpha, beta, d_out, lrow, i, j, 0);
  }
}

/* P[t,l] = (1/g) * sum_{q<g} x[t, l*g + q]   (Sec. 3.3; App. B.2 with the 1/g) */
void qo_pool(const float* x, int T, int d_in, int g, double* P) {
  const int L = d_in / g;
#pragma omp parallel for schedule(static)
  for (int t = 0; t < T; ++t)
    for (int l = 0; l < L; ++l) {
      double sum = 0.0;
      for (int q = 0; q < g; ++q) sum += (double)x[(size_t)t * d_in + l * g + q];
      P[(size_t)t * L + l] = sum / (double)g;
    }
}

/* y = x W~ + s (pool(x) A) B        (Alg. 1 forward; App. B.2)                 */
/* A == NULL or r == 0: the adapter branch is absent (post-merge inference).    */
void qo_forward(const float* x, int T, const uint8_t* codes, const float* alpha,
                const float* beta, int d_in, int d_out, int g, const float* A,
                const float* B, int r, double s, int round_wt_bf16, double* y) {
  const int L = d_in / g;
  const int adapter = (A && B && r > 0);
#pragma omp parallel for schedule(dynamic, 1)
  for (int t = 0; t < T; ++t) {
    double* acc = y + (size_t)t * d_out;
    for (int j = 0; j < d_out; ++j) acc[j] = 0.0;
    for (int i = 0; i < d_in; ++i) {
      const double xv = (double)x[(size_t)t * d_in + i];
      const size_t lrow = (size_t)(i / g) * d_out;
      for (int j = 0; j < d_out; ++j)
        acc[j] += xv * wtilde(codes, alpha, beta, d_out, lrow, i, j, round_wt_bf16);
    }
    if (adapter) {
      double* P = (double*)malloc(sizeof(double) * (size_t)L);
      double* U = (double*)malloc(sizeof(double) * (size_t)r);
      for (int l = 0; l < L; ++l) {
        double sum = 0.0;
        for (int q = 0; q < g; ++q) sum += (double)x[(size_t)t * d_in + l * g + q];
        P[l] = sum / (double)g;
      }
      for (int k = 0; k < r; ++k) {
        double u = 0.0;
        for (int l = 0; l < L; ++l) u += P[l] * (double)A[(size_t)l * r + k];
        U[k] = u;
      }
      for (int j = 0; j < d_out; ++j) {
        double v = 0.0;
        for (int k = 0; k < r; ++k) v += U[k] * (double)B[(size_t)k * d_out + j];
        acc[j] += s * v;
      }
      free(P);
      free(U);
    }
  }
}

/* Backward of the forward above with W~ frozen (only A and B are parameters,   */
/* Alg. 1; Sec. 3.1).  With G = dy:                                             */
/*   dU = s G B^T ; dB = s U^T G ; dA = P^T dU ; dP = dU A^T                     */
/*   dx[t,i] = sum_j G[t,j] W~[i,j] + dP[t, i/g] / g                             */
/* dx may be NULL.  dA, dB may be NULL (then only dx is produced, which lets a   */
/* caller evaluate dx on a subset of token rows).  A == NULL: no adapter.        */
void qo_backward(const float* dy, const float* x, int T, const uint8_t* codes,
                 const float* alpha, const float* beta, int d_in, int d_out, int g,
                 const float* A, const float* B, int r, double s, int round_wt_bf16,
                 double* dx, double* dA, double* dB) {
  const int L = d_in / g;
  const int adapter = (A && B && r > 0);
  double *P = NULL, *U = NULL, *dU = NULL, *dP = NULL;
  if (adapter) {
    P = (double*)malloc(sizeof(double) * (size_t)T * L);
    U = (double*)malloc(sizeof(double) * (size_t)T * r);
    dU = (double*)malloc(sizeof(double) * (size_t)T * r);
    dP = (double*)malloc(sizeof(double) * (size_t)T * L);
    qo_pool(x, T, d_in, g, P);
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
      for (int k = 0; k < r; ++k) {
        double u = 0.0;
        for (int l = 0; l < L; ++l) u += P[(size_t)t * L + l] * (double)A[(size_t)l * r + k];
        U[(size_t)t * r + k] = u;
        double d = 0.0;
        for (int j = 0; j < d_out; ++j)
          d += (double)dy[(size_t)t * d_out + j] * (double)B[(size_t)k * d_out + j];
        dU[(size_t)t * r + k] = s * d;
      }
      for (int l = 0; l < L; ++l) {
        double d = 0.0;
        for (int k = 0; k < r; ++k) d += dU[(size_t)t * r + k] * (double)A[(size_t)l * r + k];
        dP[(size_t)t * L + l] = d;
      }
    }
    if (dB) {
#pragma omp parallel for schedule(static)
      for (int k = 0; k < r; ++k)
        for (int j = 0; j < d_out; ++j) {
          double d = 0.0;
          for (int t = 0; t < T; ++t)
            d += U[(size_t)t * r + k] * (double)dy[(size_t)t * d_out + j];
          dB[(size_t)k * d_out + j] = s * d;
        }
    }
    if (dA) {
#pragma omp parallel for schedule(static)
      for (int l = 0; l < L; ++l)
        for (int k = 0; k < r; ++k) {
          double d = 0.0;
          for (int t = 0; t < T; ++t) d += P[(size_t)t * L + l] * dU[(size_t)t * r + k];
          dA[(size_t)l * r + k] = d;
        }
    }
  }
  if (dx) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int t = 0; t < T; ++t)
      for (int i = 0; i < d_in; ++i) {
        double acc = 0.0;
        const size_t lrow = (size_t)(i / g) * d_out;
        for (int j = 0; j < d_out; ++j)
          acc += (double)dy[(size_t)t * d_out + j] *
                 wtilde(codes, alpha, beta, d_out, lrow, i, j, round_wt_bf16);
        if (adapter) acc += dP[(size_t)t * L + i / g] / (double)g;
        dx[(size_t)t * d_in + i] = acc;
      }
  }
  free(P);
  free(U);
  free(dU);
  free(dP);
}

/* beta'[l,j] = beta[l,j] + (s/g) sum_k A[l,k] B[k,j]                           */
/* (Alg. 1 merge and App. B.3, moved to Eq. 1's zero-factor convention and to   */
/* average pooling: no division by alpha and no sign flip are left.)            */
void qo_merge(const float* beta, const float* A, const float* B, int L, int d_out,
              int r, int g, double s, float* beta_out) {
#pragma omp parallel for schedule(static)
  for (int l = 0; l < L; ++l)
    for (int j = 0; j < d_out; ++j) {
      double ab = 0.0;
      for (int k = 0; k < r; ++k)
        ab += (double)A[(size_t)l * r + k] * (double)B[(size_t)k * d_out + j];
      beta_out[(size_t)l * d_out + j] =
          (float)((double)beta[(size_t)l * d_out + j] + (s / (double)g) * ab);
    }
}

/* ------------------------------------------------------------------------- */
/* The paper's literal convention (Alg. 1, App. B): de-quantization            */
/* W~ = alpha (code - z) with a real zero POINT z in code units, SUM pooling   */
/* with coefficient s_sum, merge z' = z - s_sum (A B) / alpha.                  */
/* Kept as an independent twin so the tests can show both conventions agree.   */
/* ------------------------------------------------------------------------- */
void qo_forward_zp_sum(const float* x, int T, const uint8_t* codes, const float* alpha,
                       const double* z, int d_in, int d_out, int g, const float* A,
                       const float* B, int r, double s_sum, double* y) {
  const int L = d_in / g;
  const int adapter = (A && B && r > 0);
#pragma omp parallel for schedule(dynamic, 1)
  for (int t = 0; t < T; ++t) {
    double* acc = y + (size_t)t * d_out;
    for (int j = 0; j < d_out; ++j) acc[j] = 0.0;
    for (int i = 0; i < d_in; ++i) {
      const double xv = (double)x[(size_t)t * d_in + i];
      const size_t p = (size_t)(i / g) * d_out;
      for (int j = 0; j < d_out; ++j)
        acc[j] += xv * ((double)alpha[p + j] * ((double)codes[(size_t)i * d_out + j] - z[p + j]));
    }
    if (adapter) {
      for (int j = 0; j < d_out; ++j) {
        double v = 0.0;
        for (int l = 0; l < L; ++l) {
          double h = 0.0; /* aggregated input, App. B.2 */
          for (int q = 0; q < g; ++q) h += (double)x[(size_t)t * d_in + l * g + q];
          double ab = 0.0;
          for (int k = 0; k < r; ++k)
            ab += (double)A[(size_t)l * r + k] * (double)B[(size_t)k * d_out + j];
          v += h * ab;
        }
        acc[j] += s_sum * v;
      }
    }
  }
}

void qo_merge_zp_sum(const double* z, const float* alpha, const float* A, const float* B,
                     int L, int d_out, int r, double s_sum, double* z_out) {
#pragma omp parallel for schedule(static)
  for (int l = 0; l < L; ++l)
    for (int j = 0; j < d_out; ++j) {
      double ab = 0.0;
      for (int k = 0; k < r; ++k)
        ab += (double)A[(size_t)l * r + k] * (double)B[(size_t)k * d_out + j];
      z_out[(size_t)l * d_out + j] =
          z[(size_t)l * d_out + j] - s_sum * ab / (double)alpha[(size_t)l * d_out + j];
    }
}

/* The two zero conventions name the same weight: alpha (code - z) = alpha code  */
/* + beta  iff  beta = -alpha z  (App. B.1 against Eq. 1).  Interchange in fp64. */
void qo_beta_from_zero_point(const float* alpha, const double* z, size_t n, double* beta) {
  for (size_t i = 0; i < n; ++i) beta[i] = -(double)alpha[i] * z[i];
}
void qo_zero_point_from_beta(const float* alpha, const float* beta, size_t n, double* z) {
  for (size_t i = 0; i < n; ++i) z[i] = -(double)beta[i] / (double)alpha[i];
}

/* ------------------------------------------------------------------------- */
/* The optimiser step that follows the backward in the fine-tuning recipe      */
/* (Sec. 4.1, training details: AdamW, a maximum gradient norm, a constant     */
/* learning rate; only A and B are parameters, Sec. 3.1).  AdamW is Adam with  */
/* decoupled weight decay; the clip rescales ALL gradients by one factor when  */
/* their joint L2 norm exceeds the maximum.  fp64 from fp32 inputs.            */
/* ------------------------------------------------------------------------- */
double qo_sum_squares(const float* g, size_t n) {
  double acc = 0.0;
  for (size_t i = 0; i < n; ++i) acc += (double)g[i] * (double)g[i];
  return acc;
}

/* step counts from 1.  clip is the factor applied to the raw gradient.         */
void qo_adamw_update(const float* p, const float* g, const float* m, const float* v, size_t n,
                     double clip, double lr, double beta1, double beta2, double eps,
                     double weight_decay, int step, double* p_out, double* m_out, double* v_out) {
  const double bias1 = 1.0 - pow(beta1, (double)step);
  const double bias2 = 1.0 - pow(beta2, (double)step);
  for (size_t i = 0; i < n; ++i) {
    const double gi = clip * (double)g[i];
    const double mi = beta1 * (double)m[i] + (1.0 - beta1) * gi;        /* first moment  */
    const double vi = beta2 * (double)v[i] + (1.0 - beta2) * gi * gi;   /* second moment */
    const double decayed = (double)p[i] * (1.0 - lr * weight_decay);    /* decoupled decay */
    const double m_hat = mi / bias1, v_hat = vi / bias2;
    p_out[i] = decayed - lr * m_hat / (sqrt(v_hat) + eps);
    m_out[i] = mi;
    v_out[i] = vi;
  }
}

/* Storage bookkeeping of Sec. 3.3: a QA-LoRA linear carries L*D_out pairs of   */
/* quantization factors and L*r + r*D_out adapter parameters (ordinary LoRA:    */
/* D_in*r + r*D_out).                                                           */
long long qo_adapter_params(int d_in, int d_out, int g, int r) {
  return (long long)(d_in / g) * r + (long long)r * d_out;
}
long long qo_lora_params(int d_in, int d_out, int r) {
  return (long long)d_in * r + (long long)r * d_out;
}
long long qo_quant_factor_pairs(int d_in, int d_out, int g) {
  return (long long)(d_in / g) * d_out;
}
