/*
 * CPU oracle for the HOT linear-layer backward pass (arxiv 2503.21261).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP kernels are compared against.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it; the product path never does, and
 * this file shares no code, header, table or helper with the HIP path.
 *
 * HOT is an approximation (a quantised, rank-reduced backward pass), so the
 * oracle is the algorithm taken step by step in the paper's order and
 * notation (Sec. 3.1-3.3, Sec. 5.1-5.2): x [L x I], w [O x I], g_y [L x O],
 * g_x = g_y . w  [L x I],  g_w = g_y^T . x  [O x I]  (Eq. 7-8), row-major.
 * Every fp32 operation that decides an integer code is written out in a fixed
 * order (one rounding per add / sub / mul / div, no contraction), integer
 * products are accumulated in int64, and dequantisation / error statistics
 * are done in double.
 *
 * Readings of points the paper leaves open (each is a definition here):
 *   - H is used unnormalised (entries +-1, H.H^T = n.I); the 1/sqrt(2) per
 *     stage of Eq. 2 is applied once, exactly, as a division by n when the
 *     integer product is dequantised (the product of two rotated operands
 *     carries the factor n).
 *   - "min-max" quantiser (Sec. 5.1) = symmetric abs-max, no zero point,
 *     codes in [-qmax, qmax], qmax = 2^(bits-1) - 1.
 *   - pseudo-stochastic rounding (Sec. 5.1): the low 11 bits of the fp32
 *     pattern of the scaled value, read as a fraction in [0,1), are the
 *     threshold the fractional part is compared against.
 *   - HLA keeps, per block of n tokens, the r rows of H of lowest sequency
 *     (number of sign changes), listed by increasing sequency, unless an
 *     explicit index list is given (Sec. 3.3).  The LP_L1 list of Supp. B is
 *     defined in another paper; hot_oracle_lowpass_l1_index states the reading
 *     taken of it (2-D sequency of the block read as a token grid).
 *   - the per-token / per-tensor choice (Sec. 5.2.2) applies to the INT4
 *     quantiser of the rotated g_y on the g_x path, where a token-wise scale
 *     factors out of the product row (Sec. 4.3); operands of the g_w path
 *     (tokens already mixed by HLA) use one scale per tensor.
 *   - selection rule (Sec. 5.2.2): per-token iff the per-tensor MSE is
 *     positive and (MSE_tensor - MSE_token) >= threshold * MSE_tensor.
 *
 * Parity status: the fast transform, the quantiser bounds, the integer GEMMs,
 * full-rank HLA, and the end-points of the selection rule are pinned by the
 * CPU tests against closed forms / brute force.  The exact form of the
 * pseudo-stochastic threshold, the default low-pass row choice, the LP_L1 row
 * order, and the meaning of "difference of 50 %" are fixed by no value in the
 * paper: "parity unpinned" for those four readings.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define HOT_ORACLE_ROUND_NEAREST_EVEN 0
#define HOT_ORACLE_ROUND_PSEUDO_STOCHASTIC 1

int hot_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Sec. 3.1, Eq. 2 without the 1/sqrt(2): H_1 = [[1,1],[1,-1]], H_n = H_1 (x) H_{n/2}.
 * Written from the Kronecker recurrence itself: the top-left, top-right and
 * bottom-left quadrants repeat the half-size matrix, the bottom-right negates it. */
void hot_oracle_hadamard(int n, int8_t* H /* [n*n] */) {
  H[0] = 1;
  for (int m = 1; m < n; m *= 2) {
    /* grow the m x m matrix stored with row pitch n into 2m x 2m */
    for (int i = 0; i < m; ++i)
      for (int j = 0; j < m; ++j) {
        int8_t h = H[i * n + j];
        H[i * n + (j + m)] = h;
        H[(i + m) * n + j] = h;
        H[(i + m) * n + (j + m)] = (int8_t)-h;
      }
  }
}

/* Sec. 3.1: fast Walsh-Hadamard transform of one length-n block, additions and
 * subtractions only.  Stage h pairs element j (bit h clear) with j+h:
 * (a, b) -> (a+b, a-b), h = 1, 2, 4, ..., n/2.  Result is H_u.v in natural
 * (Sylvester) order; each add/sub rounds once in fp32. */
void hot_oracle_fwht(float* v, int n) {
  for (int h = 1; h < n; h *= 2)
    for (int j = 0; j < n; ++j)
      if ((j & h) == 0) {
        float a = v[j], b = v[j + h];
        v[j] = a + b;
        v[j + h] = a - b;
      }
}

/* Number of sign changes along row k of H_u (its "sequency"), by inspection of
 * the explicit matrix. */
int hot_oracle_sequency(int n, int k) {
  int8_t* H = (int8_t*)malloc((size_t)n * n);
  hot_oracle_hadamard(n, H);
  int c = 0;
  for (int j = 1; j < n; ++j) c += (H[k * n + j] != H[k * n + j - 1]);
  free(H);
  return c;
}

/* Sec. 3.3: default low-pass selection, the r natural-order row indices of
 * lowest sequency, listed by increasing sequency. */
void hot_oracle_lowpass_index(int n, int r, int32_t* idx /* [r] */) {
  for (int want = 0, got = 0; got < r && want < n; ++want)
    for (int k = 0; k < n; ++k)
      if (hot_oracle_sequency(n, k) == want) { idx[got++] = k; break; }
}

/* Supp. B ("Hyper-parameter of HLA"): the low-pass rows by the LP_L1 criterion of the 2-D
 * transform the paper takes from earlier work.  Reading taken here (the criterion itself is
 * defined in that other paper; parity unpinned): the n tokens of a block are a gh x gw grid
 * in raster order (token t at row t / gw, column t % gw; gw = gh = sqrt(n) for n = 16, 64;
 * gh = 4, gw = 8 for n = 32), row k of H_u is read as a gh x gw image, sv(k) and sh(k) are
 * its sign changes going down a column and along a row, and rows are listed by increasing
 * sv + sh (the L1 norm of the 2-D sequency), ties by increasing max(sv, sh), then by
 * increasing sv.  Everything is counted on the explicit matrix. */
void hot_oracle_lowpass_l1_index(int n, int r, int32_t* idx /* [r] */) {
  const int gw = n == 32 ? 8 : (n == 16 ? 4 : 8), gh = n / gw;
  int8_t* H = (int8_t*)malloc((size_t)n * n);
  int* key = (int*)malloc(sizeof(int) * (size_t)n);
  hot_oracle_hadamard(n, H);
  for (int k = 0; k < n; ++k) {
    const int8_t* img = H + (size_t)k * n;
    int sv = 0, sh = 0;
    for (int y = 1; y < gh; ++y) sv += (img[y * gw] != img[(y - 1) * gw]);          /* down column 0 */
    for (int x = 1; x < gw; ++x) sh += (img[x] != img[x - 1]);                      /* along row 0 */
    /* H_u(k, .) is a product of a function of y and a function of x, so every column and
     * every row of the image changes sign at the same places: checked, not assumed */
    for (int x = 0; x < gw; ++x) {
      int c = 0;
      for (int y = 1; y < gh; ++y) c += (img[y * gw + x] != img[(y - 1) * gw + x]);
      if (c != sv) abort();
    }
    for (int y = 0; y < gh; ++y) {
      int c = 0;
      for (int x = 1; x < gw; ++x) c += (img[y * gw + x] != img[y * gw + x - 1]);
      if (c != sh) abort();
    }
    const int mx = sv > sh ? sv : sh;
    key[k] = ((sv + sh) * 64 + mx) * 64 + sv;
  }
  for (int got = 0; got < r; ++got) {       /* selection sort: r smallest keys, in order */
    int bestk = -1;
    for (int k = 0; k < n; ++k) {
      int taken = 0;
      for (int j = 0; j < got; ++j) taken |= (idx[j] == k);
      if (!taken && (bestk < 0 || key[k] < key[bestk])) bestk = k;
    }
    idx[got] = bestk;
  }
  free(key);
  free(H);
}

/* Sec. 5.1: HT of a [rows x cols] matrix along its columns index (the
 * contiguous one): each row is cut into cols/n blocks, each block transformed. */
void hot_oracle_transform_rows(const float* g, int64_t rows, int64_t cols, int n, float* T) {
#pragma omp parallel for schedule(static)
  for (int64_t l = 0; l < rows; ++l) {
    float blk[64];
    for (int64_t b = 0; b < cols / n; ++b) {
      for (int j = 0; j < n; ++j) blk[j] = g[l * cols + b * n + j];
      hot_oracle_fwht(blk, n);
      for (int j = 0; j < n; ++j) T[l * cols + b * n + j] = blk[j];
    }
  }
}

/* Sec. 3.3 Eq. 5 / Sec. 5.2: block transform along the row index (tokens, or
 * the O index of w) of x [R x C], keeping r outputs per block: block b takes
 * rows b*n .. b*n+n-1 of every column, output row b*r + j is transformed
 * element keep[j].  r = n with keep = 0..n-1 is the plain HT along that index. */
void hot_oracle_hla(const float* x, int64_t R, int64_t C, int n, int r, const int32_t* keep,
                    float* out /* [R/n*r x C] */) {
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < R / n; ++b) {
    float blk[64];
    for (int64_t c = 0; c < C; ++c) {
      for (int j = 0; j < n; ++j) blk[j] = x[(b * n + j) * C + c];
      hot_oracle_fwht(blk, n);
      for (int j = 0; j < r; ++j) out[(b * r + j) * C + c] = blk[keep[j]];
    }
  }
}

static float absmax_range(const float* t, int64_t count) {
  float m = 0.0f;
  for (int64_t i = 0; i < count; ++i) {
    float a = fabsf(t[i]);
    if (a > m) m = a;
  }
  return m;
}

static int8_t quantize_one(float t, float inv, int qmax, int rounding) {
  float v = t * inv; /* one fp32 multiply */
  int q;
  if (rounding == HOT_ORACLE_ROUND_NEAREST_EVEN) {
    q = (int)rintf(v);
  } else {
    float f = floorf(v);
    float frac = v - f;
    uint32_t bits;
    memcpy(&bits, &v, 4);
    float rnd = (float)(bits & 0x7FFu) * (1.0f / 2048.0f);
    q = (int)f + (frac > rnd ? 1 : 0);
  }
  if (q > qmax) q = qmax;
  if (q < -qmax) q = -qmax;
  return (int8_t)q;
}

/* Sec. 5.1 quantiser over a [rows x cols] matrix.  per_token = 1: one scale per
 * row (token), scales[rows]; per_token = 0: one scale for the tensor, scales[1].
 * scale = amax / qmax and inv = qmax / amax are fp32 divisions; an all-zero
 * group has scale 0 and codes 0. */
void hot_oracle_quantize(const float* t, int64_t rows, int64_t cols, int bits, int per_token,
                         int rounding, int8_t* codes, float* scales) {
  const int qmax = (1 << (bits - 1)) - 1;
  float amax_all = 0.0f;
  if (!per_token) {
    amax_all = absmax_range(t, rows * cols);
    scales[0] = amax_all / (float)qmax;
  }
#pragma omp parallel for schedule(static)
  for (int64_t l = 0; l < rows; ++l) {
    float amax = per_token ? absmax_range(t + l * cols, cols) : amax_all;
    if (per_token) scales[l] = amax / (float)qmax;
    float inv = 0.0f;
    if (amax > 0.0f) inv = (float)qmax / amax;
    for (int64_t c = 0; c < cols; ++c)
      codes[l * cols + c] = quantize_one(t[l * cols + c], inv, qmax, rounding);
  }
}

/* acc[m, j] = sum_k A[m, k] * B[k, j]; A [M x K], B [K x N]; exact in int64.
 * Returns the number of accumulators whose magnitude does not fit int32. */
int64_t hot_oracle_igemm_nn(const int8_t* A, const int8_t* B, int64_t M, int64_t N, int64_t K,
                            int64_t* acc) {
  int64_t bad = 0;
#pragma omp parallel for schedule(static) reduction(+ : bad)
  for (int64_t m = 0; m < M; ++m) {
    int64_t* row = acc + m * N;
    for (int64_t j = 0; j < N; ++j) row[j] = 0;
    for (int64_t k = 0; k < K; ++k) {
      int64_t a = A[m * K + k];
      for (int64_t j = 0; j < N; ++j) row[j] += a * (int64_t)B[k * N + j];
    }
    for (int64_t j = 0; j < N; ++j)
      if (row[j] > 2147483647LL || row[j] < -2147483647LL - 1) ++bad;
  }
  return bad;
}

/* acc[m, j] = sum_k A[k, m] * B[k, j]; A [K x M], B [K x N] (g_w = g_y^T . x). */
int64_t hot_oracle_igemm_tn(const int8_t* A, const int8_t* B, int64_t M, int64_t N, int64_t K,
                            int64_t* acc) {
  int64_t bad = 0;
#pragma omp parallel for schedule(static) reduction(+ : bad)
  for (int64_t m = 0; m < M; ++m) {
    int64_t* row = acc + m * N;
    for (int64_t j = 0; j < N; ++j) row[j] = 0;
    for (int64_t k = 0; k < K; ++k) {
      int64_t a = A[k * M + m];
      for (int64_t j = 0; j < N; ++j) row[j] += a * (int64_t)B[k * N + j];
    }
    for (int64_t j = 0; j < N; ++j)
      if (row[j] > 2147483647LL || row[j] < -2147483647LL - 1) ++bad;
  }
  return bad;
}

/* Sec. 4.3 / Supp. F dequantisation: out[m, j] = acc[m, j] * s_row[m] * s_col / n in
 * double.  row_stride 1 = token-wise scales, 0 = a single scale. */
void hot_oracle_dequant(const int64_t* acc, int64_t M, int64_t N, const float* s_row,
                        int row_stride, float s_col, int n, double* out) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m) {
    double s = (double)s_row[m * row_stride] * (double)s_col / (double)n;
    for (int64_t j = 0; j < N; ++j) out[m * N + j] = (double)acc[m * N + j] * s;
  }
}

/* Sec. 5.1: the whole g_x path.  Optional taps (may be NULL) expose every
 * intermediate the HIP path is compared against bit by bit. */
int64_t hot_oracle_backward_gx(const float* g_y, const float* w, int64_t L, int64_t O, int64_t I,
                               int n, int bits, int per_token, int rounding, double* g_x,
                               int8_t* tap_qg /* [L x O] */, float* tap_sg /* [L] or [1] */,
                               int8_t* tap_qw /* [O x I] */, float* tap_sw /* [1] */,
                               int64_t* tap_acc /* [L x I] */) {
  float* T = (float*)malloc(sizeof(float) * L * O);
  float* U = (float*)malloc(sizeof(float) * O * I);
  int8_t* qg = tap_qg ? tap_qg : (int8_t*)malloc((size_t)L * O);
  int8_t* qw = tap_qw ? tap_qw : (int8_t*)malloc((size_t)O * I);
  float* sg = tap_sg ? tap_sg : (float*)malloc(sizeof(float) * (per_token ? L : 1));
  float sw_local;
  float* sw = tap_sw ? tap_sw : &sw_local;
  int64_t* acc = tap_acc ? tap_acc : (int64_t*)malloc(sizeof(int64_t) * L * I);
  int32_t ident[64];
  for (int j = 0; j < n; ++j) ident[j] = j;

  hot_oracle_transform_rows(g_y, L, O, n, T);        /* g_y . H^T, along O          */
  hot_oracle_hla(w, O, I, n, n, ident, U);           /* H . w, along O, full rank   */
  hot_oracle_quantize(T, L, O, bits, per_token, rounding, qg, sg);
  hot_oracle_quantize(U, O, I, bits, 0, rounding, qw, sw);
  int64_t bad = hot_oracle_igemm_nn(qg, qw, L, I, O, acc);
  hot_oracle_dequant(acc, L, I, sg, per_token ? 1 : 0, sw[0], n, g_x);

  free(T);
  free(U);
  if (!tap_qg) free(qg);
  if (!tap_qw) free(qw);
  if (!tap_sg) free(sg);
  if (!tap_acc) free(acc);
  return bad;
}

/* Sec. 5.2.1 (ABC): x_hat = HLA(x) along L, INT8, one scale. codes [L*r/n x I]. */
void hot_oracle_compress_activation(const float* x, int64_t L, int64_t I, int n, int r,
                                    const int32_t* keep, int bits, int rounding, int8_t* codes,
                                    float* scale) {
  int64_t Lr = L / n * r;
  float* xh = (float*)malloc(sizeof(float) * Lr * I);
  hot_oracle_hla(x, L, I, n, r, keep, xh);
  hot_oracle_quantize(xh, Lr, I, bits, 0, rounding, codes, scale);
  free(xh);
}

/* Sec. 5.2: the g_w path from the stored compressed activation. */
int64_t hot_oracle_backward_gw(const float* g_y, const int8_t* x_codes, float x_scale, int64_t L,
                               int64_t O, int64_t I, int n, int r, const int32_t* keep, int bits,
                               int rounding, double* g_w, int8_t* tap_qg /* [L*r/n x O] */,
                               float* tap_sg /* [1] */, int64_t* tap_acc /* [O x I] */) {
  int64_t Lr = L / n * r;
  float* gh = (float*)malloc(sizeof(float) * Lr * O);
  int8_t* qg = tap_qg ? tap_qg : (int8_t*)malloc((size_t)Lr * O);
  float sg_local;
  float* sg = tap_sg ? tap_sg : &sg_local;
  int64_t* acc = tap_acc ? tap_acc : (int64_t*)malloc(sizeof(int64_t) * O * I);

  hot_oracle_hla(g_y, L, O, n, r, keep, gh);
  hot_oracle_quantize(gh, Lr, O, bits, 0, rounding, qg, sg);
  int64_t bad = hot_oracle_igemm_tn(qg, x_codes, O, I, Lr, acc);
  hot_oracle_dequant(acc, O, I, sg, 0, x_scale, n, g_w);

  free(gh);
  if (!tap_qg) free(qg);
  if (!tap_acc) free(acc);
  return bad;
}

/* Sec. 5.2.2 (LQS): MSE between g_y and its per-token / per-tensor quantised
 * version.  Computed on the rotated tensor T = g_y . H_u^T; with the orthonormal
 * H = H_u / sqrt(n) the squared error of the rotated tensor equals that of the
 * original, so the sums over T are divided by n.  Returns 1 for per-token. */
int hot_oracle_select_quantizer(const float* g_y, int64_t L, int64_t O, int n, int bits,
                                int rounding, double threshold, double* mse_token,
                                double* mse_tensor) {
  float* T = (float*)malloc(sizeof(float) * L * O);
  int8_t* q = (int8_t*)malloc((size_t)L * O);
  float* s = (float*)malloc(sizeof(float) * L);
  hot_oracle_transform_rows(g_y, L, O, n, T);
  double mse[2];
  for (int per_token = 0; per_token < 2; ++per_token) {
    hot_oracle_quantize(T, L, O, bits, per_token, rounding, q, s);
    double sum = 0.0;
    for (int64_t l = 0; l < L; ++l) {
      double sc = (double)s[per_token ? l : 0];
      for (int64_t o = 0; o < O; ++o) {
        double e = (double)T[l * O + o] - (double)q[l * O + o] * sc;
        sum += e * e;
      }
    }
    mse[per_token] = sum / ((double)n * (double)L * (double)O);
  }
  free(T);
  free(q);
  free(s);
  *mse_tensor = mse[0];
  *mse_token = mse[1];
  return (mse[0] > 0.0 && (mse[0] - mse[1]) >= threshold * mse[0]) ? 1 : 0;
}

/* Eq. 8 in double precision: the un-approximated backward, used only to report
 * the method's error as a statistic. */
void hot_oracle_exact_backward(const float* g_y, const float* x, const float* w, int64_t L,
                               int64_t O, int64_t I, double* g_x, double* g_w) {
  if (g_x) {
#pragma omp parallel for schedule(static)
    for (int64_t l = 0; l < L; ++l) {
      double* row = g_x + l * I;
      for (int64_t i = 0; i < I; ++i) row[i] = 0.0;
      for (int64_t o = 0; o < O; ++o) {
        double a = g_y[l * O + o];
        for (int64_t i = 0; i < I; ++i) row[i] += a * (double)w[o * I + i];
      }
    }
  }
  if (g_w) {
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < O; ++o) {
      double* row = g_w + o * I;
      for (int64_t i = 0; i < I; ++i) row[i] = 0.0;
      for (int64_t l = 0; l < L; ++l) {
        double a = g_y[l * O + o];
        for (int64_t i = 0; i < I; ++i) row[i] += a * (double)x[l * I + i];
      }
    }
  }
}
