/*
 * CPU oracle for the quantized GEMM  C_u8 = requant(A_u8 * B_s8)  and the
 * group-wise convolution built on it.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct
 * statement of what the GPU library must compute.  Only the tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it.  It shares no
 * header, helper, table or constant with the HIP code and neither side
 * includes the other.
 *
 * What each function follows (paper = "FBGEMM: Enabling High-Performance
 * Low-Precision Deep Learning Inference", arXiv 2101.05615):
 *   - affine quantization X = alpha_X (X^q - theta_X): Sec. 2.1, Eq. (1);
 *   - expansion of the quantized product into dot product, row offset,
 *     column offset and the constant K*theta_A*theta_B: Sec. 2.1, Eq. (2);
 *     the sums run over k = 0..K-1 (K terms, as the constant K*theta_A*theta_B
 *     in the same equation requires);
 *   - row offset / column offset definitions and the remark that the constant
 *     can be folded into the offsets of the constant matrix: Sec. 2.1, the
 *     list after Eq. (2);
 *   - requantization C^q = multiplier * C_int32 + theta_C: same list, third
 *     item.  The combined multiplier alpha_A*alpha_B/alpha_C is passed in as
 *     one fp32 number per tensor or per output channel.
 * Readings where the paper is silent (rounding = nearest-even, saturation to
 * [0,255], bias added in the int32 domain before scaling, ReLU = lower clamp
 * at theta_C) are fixed here and must be mirrored bit for bit by the GPU.
 *
 *   - the other ends of the pipeline (Appendix B: any packing routine for A,
 *     any output processing): activations given in fp32 and quantized by
 *     Eq. (1) solved for X^q, and the result left in fp32, i.e. the real-domain
 *     product alpha_A alpha_B * x of Eq. (2) without the division by alpha_C.
 *     Readings fixed here: the caller passes 1/alpha_A and alpha_A*alpha_B as
 *     fp32 numbers and each is applied with ONE fp32 multiply; rounding is to
 *     nearest even; quantized activations saturate to [0,255]; ReLU on the fp32
 *     result is max(., 0).
 *   - outlier-aware split of the constant matrix (Sec. 2.2, "sample end-to-end
 *     pipeline"): B = B' + B_sparse with only small-magnitude numbers in B',
 *     the few big ones in B_sparse in compressed sparse column form, and
 *     A B = A B' + A B_sparse.  "Small" is fixed here as lo <= b <= hi for a
 *     caller-chosen range (the GPU library stores B' in 4 bits: -8..7).
 *
 * Pins (tests/test_oracle_pins.py): brute force in Python integers, the
 * identity x - bias == sum_k (A - theta_A)(B - theta_B), fp64
 * dequantize->GEMM->quantize, closed forms for all-0 / all-255 inputs,
 * hand-worked rounding and clamp examples, torch conv2d for the convolution;
 * for the fp32 ends: hand-worked ties and saturation, exact round trips of
 * Eq. (1) on power-of-two scales, the half-step error bound of rounding, and
 * the fp64 real-domain product within two fp32 roundings.
 * No function here is "parity unpinned".
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -fno-fast-math -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_EOVERFLOW (-2) /* the corrected accumulator does not fit int32 */
#define ORC_ENOMEM (-3)

int orc_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* column offset before folding: colsum[j] = sum_k B[k][j]   (Sec. 2.1) */
int orc_colsum(const int8_t* B, int K, int N, int ldb, int32_t* colsum) {
  if (!B || !colsum || K <= 0 || N <= 0 || ldb < N) return ORC_EINVAL;
  for (int j = 0; j < N; ++j) {
    int64_t s = 0;
    for (int k = 0; k < K; ++k) s += B[(size_t)k * ldb + j];
    colsum[j] = (int32_t)s;
  }
  return ORC_OK;
}

/* row offset: rowsum[i] = sum_k A[i][k]   (Sec. 2.1) */
int orc_rowsum(const uint8_t* A, int M, int K, int lda, int32_t* rowsum) {
  if (!A || !rowsum || M <= 0 || K <= 0 || lda < K) return ORC_EINVAL;
  for (int i = 0; i < M; ++i) {
    int64_t s = 0;
    for (int k = 0; k < K; ++k) s += A[(size_t)i * lda + k];
    rowsum[i] = (int32_t)s;
  }
  return ORC_OK;
}

/* Column offsets with the constant of Eq. (2) folded in, possible because B is
 * the constant matrix:  col_offsets[j] = colsum[j] - K * theta_B[j].
 * b_zp has 1 entry (per tensor) or N entries (per output channel). */
int orc_col_offsets(const int8_t* B, int K, int N, int ldb, const int32_t* b_zp,
                    int n_b_zp, int32_t* col_offsets) {
  if (!b_zp || (n_b_zp != 1 && n_b_zp != N)) return ORC_EINVAL;
  int rc = orc_colsum(B, K, N, ldb, col_offsets);
  if (rc) return rc;
  for (int j = 0; j < N; ++j) {
    int64_t zp = b_zp[n_b_zp == 1 ? 0 : j];
    col_offsets[j] = (int32_t)((int64_t)col_offsets[j] - (int64_t)K * zp);
  }
  return ORC_OK;
}

/* Raw accumulator  acc[i][j] = sum_{k<K} A[i][k] * B[k][j]  in int32: the first
 * term of Eq. (2).  Three nested loops, nothing blocked or packed; the loop
 * order i,k,j only lets the inner loop run along memory. */
int orc_acc32(const uint8_t* A, int M, int K, int lda, const int8_t* B, int N,
              int ldb, int32_t* C32, int ldc) {
  if (!A || !B || !C32 || M <= 0 || N <= 0 || K <= 0 || lda < K || ldb < N ||
      ldc < N)
    return ORC_EINVAL;
#pragma omp parallel for schedule(static)
  for (int i = 0; i < M; ++i) {
    int32_t* restrict row = C32 + (size_t)i * ldc;
    for (int j = 0; j < N; ++j) row[j] = 0;
    for (int k = 0; k < K; ++k) {
      const int32_t a = A[(size_t)i * lda + k];
      const int8_t* restrict b = B + (size_t)k * ldb;
      for (int j = 0; j < N; ++j) row[j] += a * (int32_t)b[j];
    }
  }
  return ORC_OK;
}

/* Requantization of one corrected accumulator x (third item after Eq. (2)):
 *   f = (float)x            int32 -> fp32, round to nearest even
 *   p = f * scale           one IEEE fp32 multiply
 *   r = nearbyintf(p)       round to nearest even
 *   clamp r to [lo - theta_C, 255 - theta_C], lo = theta_C with ReLU else 0
 *   result = (int)r + theta_C
 * The clamp is done in float, before the conversion to integer, so no
 * out-of-range float->int conversion can happen. */
uint8_t orc_requant_one(int32_t x, float scale, int32_t c_zp, int relu) {
  volatile float f = (float)x;
  volatile float p = f * scale;
  float r = nearbyintf(p);
  const int32_t lo = relu ? c_zp : 0;
  r = fminf(fmaxf(r, (float)(lo - c_zp)), (float)(255 - c_zp));
  return (uint8_t)((int32_t)r + c_zp);
}

/* fp32 output of one corrected accumulator: the real-domain value of Eq. (2),
 * alpha_A*alpha_B*x, with the product alpha_A*alpha_B passed as one fp32
 * number.  Fixed sequence: int32 -> fp32 (nearest even), ONE fp32 multiply,
 * then max(., 0) if relu. */
float orc_dequant_one(int32_t x, float scale, int relu) {
  volatile float f = (float)x;
  volatile float p = f * scale;
  float r = p;
  if (relu && r < 0.0f) r = 0.0f;
  return r;
}

/* out[i][j] = orc_dequant_one(x[i][j], scales[j or 0], relu); x and out are
 * M x N row-major with leading dimension N. */
int orc_dequant_f32(const int32_t* x, int M, int N, const float* scales,
                    int n_scales, int relu, float* out) {
  if (!x || !scales || !out || M <= 0 || N <= 0) return ORC_EINVAL;
  if (n_scales != 1 && n_scales != N) return ORC_EINVAL;
  for (int i = 0; i < M; ++i)
    for (int j = 0; j < N; ++j)
      out[(size_t)i * N + j] = orc_dequant_one(
          x[(size_t)i * N + j], scales[n_scales == 1 ? 0 : j], relu);
  return ORC_OK;
}

/* Quantization of one fp32 activation, Eq. (1) solved for the quantized value:
 * X^q = X / alpha + theta.  The caller passes inv_scale = 1/alpha as fp32.
 * Fixed sequence (the mirror image of the requantization above):
 *   p = a * inv_scale        ONE fp32 multiply
 *   r = nearbyintf(p)        round to nearest even
 *   clamp r to [-theta, 255 - theta]   (in float, before the conversion)
 *   result = (int)r + theta
 * a must not be NaN. */
uint8_t orc_quantize_one(float a, float inv_scale, int32_t zp) {
  volatile float p = a * inv_scale;
  float r = nearbyintf(p);
  r = fminf(fmaxf(r, (float)(0 - zp)), (float)(255 - zp));
  return (uint8_t)((int32_t)r + zp);
}

/* Aq[i][k] = orc_quantize_one(A[i][k], inv_scale, zp) for an M x K matrix. */
int orc_quantize_f32(const float* A, int M, int K, int lda, float inv_scale,
                     int32_t zp, uint8_t* Aq, int ldq) {
  if (!A || !Aq || M <= 0 || K <= 0 || lda < K || ldq < K) return ORC_EINVAL;
  if (zp < 0 || zp > 255) return ORC_EINVAL;
  for (int i = 0; i < M; ++i)
    for (int k = 0; k < K; ++k)
      Aq[(size_t)i * ldq + k] =
          orc_quantize_one(A[(size_t)i * lda + k], inv_scale, zp);
  return ORC_OK;
}

/* Outlier split (Sec. 2.2): B' keeps the entries with lo <= b <= hi and is zero
 * elsewhere; B_sparse = B - B' keeps the others.  Both are written densely
 * (K x N, leading dimension N); returns the number of outliers, or a negative
 * ORC_E* code. */
long orc_split_outliers(const int8_t* B, int K, int N, int ldb, int lo, int hi,
                        int8_t* B_small, int8_t* B_sparse) {
  if (!B || !B_small || !B_sparse || K <= 0 || N <= 0 || ldb < N || lo > hi)
    return ORC_EINVAL;
  long nnz = 0;
  for (int k = 0; k < K; ++k)
    for (int j = 0; j < N; ++j) {
      const int8_t b = B[(size_t)k * ldb + j];
      const int small = (b >= lo && b <= hi);
      B_small[(size_t)k * N + j] = small ? b : 0;
      B_sparse[(size_t)k * N + j] = small ? 0 : b;
      nnz += !small;
    }
  return nnz;
}

/* Compressed sparse column form of a dense K x N matrix (leading dimension N):
 * col_ptr has N+1 entries; the nonzeros of column j are row_idx/val[col_ptr[j]
 * .. col_ptr[j+1]) in increasing row order.  cap = capacity of row_idx/val. */
int orc_csc_from_dense(const int8_t* S, int K, int N, int32_t* col_ptr,
                       int32_t* row_idx, int8_t* val, long cap) {
  if (!S || !col_ptr || K <= 0 || N <= 0) return ORC_EINVAL;
  long n = 0;
  for (int j = 0; j < N; ++j) {
    col_ptr[j] = (int32_t)n;
    for (int k = 0; k < K; ++k) {
      const int8_t v = S[(size_t)k * N + j];
      if (v != 0) {
        if (n >= cap || !row_idx || !val) return ORC_EINVAL;
        row_idx[n] = k;
        val[n] = v;
        ++n;
      }
    }
  }
  col_ptr[N] = (int32_t)n;
  return ORC_OK;
}

/* Accumulator of the split product, term by term as the paper writes it:
 *   C32 = A B_small  (dense, plain triple loop)  +  A B_sparse  (CSC, one
 *   multiply-add per stored nonzero and row of A). */
int orc_acc32_split(const uint8_t* A, int M, int K, int lda, const int8_t* B_small,
                    int N, const int32_t* col_ptr, const int32_t* row_idx,
                    const int8_t* val, int32_t* C32) {
  if (!A || !B_small || !col_ptr || !C32 || M <= 0 || N <= 0 || K <= 0 || lda < K)
    return ORC_EINVAL;
  for (int i = 0; i < M; ++i)
    for (int j = 0; j < N; ++j) {
      int32_t acc = 0;
      for (int k = 0; k < K; ++k)
        acc += (int32_t)A[(size_t)i * lda + k] * (int32_t)B_small[(size_t)k * N + j];
      for (int32_t e = col_ptr[j]; e < col_ptr[j + 1]; ++e)
        acc += (int32_t)A[(size_t)i * lda + row_idx[e]] * (int32_t)val[e];
      C32[(size_t)i * N + j] = acc;
    }
  return ORC_OK;
}

/* The whole path.  For every (i,j):
 *   acc = sum_k A[i][k]*B[k][j]
 *   x   = acc - theta_A*colsum[j] - theta_B[j]*rowsum[i] + K*theta_A*theta_B[j]
 *         (+ bias[j])                                  -- Eq. (2), four terms
 *   C[i][j] = requant(x, scale[j])
 * x is formed in int64 and must fit int32, otherwise ORC_EOVERFLOW.
 * x_out (optional, M*N, row-major, ld = N) receives x.
 * b_zp: 1 or N entries; scales: 1 or N entries; bias: N entries or NULL. */
int orc_gemm_u8s8_requant(const uint8_t* A, int M, int K, int lda, int32_t a_zp,
                          const int8_t* B, int N, int ldb, const int32_t* b_zp,
                          int n_b_zp, const int32_t* bias, const float* scales,
                          int n_scales, int32_t c_zp, int relu, uint8_t* C,
                          int ldc, int32_t* x_out) {
  if (!A || !B || !C || !b_zp || !scales || M <= 0 || N <= 0 || K <= 0 ||
      lda < K || ldb < N || ldc < N)
    return ORC_EINVAL;
  if ((n_b_zp != 1 && n_b_zp != N) || (n_scales != 1 && n_scales != N))
    return ORC_EINVAL;
  if (a_zp < 0 || a_zp > 255 || c_zp < 0 || c_zp > 255) return ORC_EINVAL;

  int32_t* colsum = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
  int32_t* rowsum = (int32_t*)malloc(sizeof(int32_t) * (size_t)M);
  if (!colsum || !rowsum) {
    free(colsum);
    free(rowsum);
    return ORC_ENOMEM;
  }
  orc_colsum(B, K, N, ldb, colsum);
  orc_rowsum(A, M, K, lda, rowsum);

  long overflow = 0;
  int nomem = 0;
#pragma omp parallel reduction(+ : overflow) reduction(| : nomem)
  {
    int32_t* acc = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
    if (!acc) nomem = 1;
#pragma omp for schedule(static)
    for (int i = 0; i < M; ++i) {
      if (!acc) continue;
      for (int j = 0; j < N; ++j) acc[j] = 0;
      for (int k = 0; k < K; ++k) {
        const int32_t a = A[(size_t)i * lda + k];
        const int8_t* restrict b = B + (size_t)k * ldb;
        for (int j = 0; j < N; ++j) acc[j] += a * (int32_t)b[j];
      }
      for (int j = 0; j < N; ++j) {
        const int64_t zb = b_zp[n_b_zp == 1 ? 0 : j];
        int64_t x64 = (int64_t)acc[j] - (int64_t)a_zp * colsum[j] -
                      zb * (int64_t)rowsum[i] + (int64_t)K * a_zp * zb;
        if (bias) x64 += bias[j];
        if (x64 < INT32_MIN || x64 > INT32_MAX) {
          ++overflow;
          x64 = 0;
        }
        const int32_t x = (int32_t)x64;
        if (x_out) x_out[(size_t)i * N + j] = x;
        C[(size_t)i * ldc + j] =
            orc_requant_one(x, scales[n_scales == 1 ? 0 : j], c_zp, relu);
      }
    }
    free(acc);
  }
  free(colsum);
  free(rowsum);
  if (nomem) return ORC_ENOMEM;
  return overflow ? ORC_EOVERFLOW : ORC_OK;
}

/* ------------------------------------------------------------------------ */
/* Group-wise convolution.  The paper names convolution but gives no
 * algorithm, so the definition is the real-domain one implied by Eq. (1):
 * the input is NHWC uint8 with zero point theta_A, padding is real zero,
 * weights are int8 [G][R][S][Cin/G][Cout/G] with zero point theta_B per tensor
 * or per output channel, and
 *   x[n,ho,wo,oc] = sum over in-image taps (kh,kw,ci) of
 *        (in[n,hi,wi,g*Cg+ci] - theta_A) * (w[g][kh][kw][ci][co] - theta_B[oc])
 *        + bias[oc],          oc = g*Og + co
 * followed by the same requantization.  Out-of-image taps contribute nothing
 * (real zero), which is what "padding with theta_A" means in the quantized
 * domain. */
int orc_conv_groupwise_direct(const uint8_t* in, int Nb, int H, int W, int C,
                              int G, int Cout, int R, int S, int pad,
                              int stride, int32_t a_zp, const int8_t* wgt,
                              const int32_t* b_zp, int n_b_zp,
                              const int32_t* bias, const float* scales,
                              int n_scales, int32_t c_zp, int relu,
                              uint8_t* out, int32_t* x_out) {
  if (!in || !wgt || !out || !b_zp || !scales) return ORC_EINVAL;
  if (Nb <= 0 || H <= 0 || W <= 0 || C <= 0 || G <= 0 || Cout <= 0 || R <= 0 ||
      S <= 0 || pad < 0 || stride <= 0 || C % G || Cout % G)
    return ORC_EINVAL;
  if ((n_b_zp != 1 && n_b_zp != Cout) || (n_scales != 1 && n_scales != Cout))
    return ORC_EINVAL;
  const int Cg = C / G, Og = Cout / G;
  const int Ho = (H + 2 * pad - R) / stride + 1;
  const int Wo = (W + 2 * pad - S) / stride + 1;
  if (Ho <= 0 || Wo <= 0) return ORC_EINVAL;
  long overflow = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(+ : overflow)
  for (int n = 0; n < Nb; ++n)
    for (int ho = 0; ho < Ho; ++ho)
      for (int wo = 0; wo < Wo; ++wo)
        for (int g = 0; g < G; ++g)
          for (int co = 0; co < Og; ++co) {
            const int oc = g * Og + co;
            const int64_t zb = b_zp[n_b_zp == 1 ? 0 : oc];
            int64_t x64 = bias ? bias[oc] : 0;
            for (int kh = 0; kh < R; ++kh)
              for (int kw = 0; kw < S; ++kw) {
                const int hi = ho * stride + kh - pad;
                const int wi = wo * stride + kw - pad;
                if (hi < 0 || hi >= H || wi < 0 || wi >= W) continue;
                for (int ci = 0; ci < Cg; ++ci) {
                  const int64_t a =
                      in[(((size_t)n * H + hi) * W + wi) * C + g * Cg + ci];
                  const int64_t b =
                      wgt[((((size_t)g * R + kh) * S + kw) * Cg + ci) * Og + co];
                  x64 += (a - a_zp) * (b - zb);
                }
              }
            if (x64 < INT32_MIN || x64 > INT32_MAX) {
              ++overflow;
              x64 = 0;
            }
            const size_t o = (((size_t)n * Ho + ho) * Wo + wo) * Cout + oc;
            if (x_out) x_out[o] = (int32_t)x64;
            out[o] = orc_requant_one((int32_t)x64,
                                     scales[n_scales == 1 ? 0 : oc], c_zp, relu);
          }
  return overflow ? ORC_EOVERFLOW : ORC_OK;
}

/* im2col of one group: rows = output pixels (n,ho,wo), columns ordered
 * (kh,kw,ci) with ci fastest; out-of-image taps are filled with theta_A (the
 * quantized value of real zero).  Pure data movement; lets a test express the
 * convolution as one orc_gemm_u8s8_requant per group. */
int orc_im2col_group(const uint8_t* in, int Nb, int H, int W, int C, int G,
                     int g, int R, int S, int pad, int stride, int32_t a_zp,
                     uint8_t* cols) {
  if (!in || !cols || G <= 0 || C % G || g < 0 || g >= G || stride <= 0)
    return ORC_EINVAL;
  const int Cg = C / G;
  const int Ho = (H + 2 * pad - R) / stride + 1;
  const int Wo = (W + 2 * pad - S) / stride + 1;
  const int Kc = R * S * Cg;
  size_t row = 0;
  for (int n = 0; n < Nb; ++n)
    for (int ho = 0; ho < Ho; ++ho)
      for (int wo = 0; wo < Wo; ++wo, ++row)
        for (int kh = 0; kh < R; ++kh)
          for (int kw = 0; kw < S; ++kw)
            for (int ci = 0; ci < Cg; ++ci) {
              const int hi = ho * stride + kh - pad;
              const int wi = wo * stride + kw - pad;
              uint8_t v = (uint8_t)a_zp;
              if (hi >= 0 && hi < H && wi >= 0 && wi < W)
                v = in[(((size_t)n * H + hi) * W + wi) * C + g * Cg + ci];
              cols[row * Kc + (kh * S + kw) * Cg + ci] = v;
            }
  return ORC_OK;
}
