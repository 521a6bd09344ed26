/* CPU oracle, naive C form -- TEST INFRASTRUCTURE ONLY.
 *
 * The GlowQ group forward straight from the stored bytes, with triple loops and
 * float64 accumulation.  It is used by tests/, by __graft_entry__.smoke() and by
 * the cpu_baseline leg of bench.py; it shares no code with the HIP library.
 *
 *   R[t][j]   = sum_k X[t][k] B[j][k]                              Sec. 3.3, Eq. 8
 *   Y_i[t][o] = sum_k X[t][k] What_i[o][k] + sum_j R[t][j] A_i[o][j]   Eq. 9
 *   What[o][k] = round_act((q[o][k] - z[o][k/G]) * s[o][k/G])      W4A16, Sec. 4.1
 *
 * Memory is token-major; 16-bit operands arrive as their bit patterns
 * (act: 0 = IEEE binary16, 1 = bfloat16; scales and zero-points are always
 * binary16).  q is packed eight to a 32-bit word, element 8j+e in bits 4e..4e+3.
 * Loops over independent output elements are split over OpenMP threads; nothing
 * is blocked, fused or reordered beyond that.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* value of a 16-bit float pattern: sign, exponent field, fraction field */
static double widen16(uint16_t b, int act) {
  int ebits = act ? 8 : 5, fbits = 15 - ebits, bias = (1 << (ebits - 1)) - 1;
  int sign = (b >> 15) & 1;
  int e = (b >> fbits) & ((1 << ebits) - 1);
  int f = b & ((1 << fbits) - 1);
  double v;
  if (e == (1 << ebits) - 1) v = f ? NAN : INFINITY;
  else if (e == 0) v = ldexp((double)f, 1 - bias - fbits);
  else v = ldexp((double)(f + (1 << fbits)), e - bias - fbits);
  return sign ? -v : v;
}

/* nearest-even rounding of a double to the 16-bit format, returned widened */
static double round16(double x, int act) {
  int sig = act ? 8 : 11, emin = act ? -126 : -14, emax = act ? 127 : 15;
  if (x == 0.0 || isnan(x) || isinf(x)) return x;
  int e;
  frexp(fabs(x), &e);
  e -= 1;
  if (e < emin) e = emin;
  double quantum = ldexp(1.0, e - (sig - 1));
  double n = nearbyint(fabs(x) / quantum); /* default mode: half to even */
  double v = n * quantum;
  if (v >= ldexp(1.0, emax + 1)) v = INFINITY;
  return x < 0 ? -v : v;
}

static inline int nibble(const uint32_t* wq, int64_t row, int64_t k, int64_t d_in) {
  uint32_t w = wq[row * (d_in / 8) + k / 8];
  return (int)((w >> (4 * (k % 8))) & 15u);
}

int glowq_oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* q[o][k] as bytes */
int glowq_oracle_unpack(const uint32_t* wq, int d_out, int d_in, uint8_t* q) {
  if (!wq || !q || d_in % 8) return -1;
  for (int64_t o = 0; o < d_out; ++o)
    for (int64_t k = 0; k < d_in; ++k) q[o * d_in + k] = (uint8_t)nibble(wq, o, k, d_in);
  return 0;
}

/* What[o][k] as float64 (already rounded to the activation type) */
int glowq_oracle_dequant(const uint32_t* wq, const uint16_t* scales, const uint16_t* zeros,
                         int d_out, int d_in, int G, int act, double* what) {
  if (!wq || !scales || !zeros || !what || G <= 0 || d_in % G || d_in % 8) return -1;
  int64_t ng = d_in / G;
#pragma omp parallel for schedule(static)
  for (int64_t o = 0; o < d_out; ++o)
    for (int64_t k = 0; k < d_in; ++k) {
      double s = widen16(scales[o * ng + k / G], 0);
      double z = widen16(zeros[o * ng + k / G], 0);
      what[o * d_in + k] = round16(((double)nibble(wq, o, k, d_in) - z) * s, act);
    }
  return 0;
}

/* Eq. 8 */
int glowq_oracle_shared_proj(const uint16_t* X, const uint16_t* B, int T, int d_in, int r,
                             int act, double* R) {
  if (!X || !B || !R) return -1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t t = 0; t < T; ++t)
    for (int64_t j = 0; j < r; ++j) {
      double acc = 0.0;
      for (int64_t k = 0; k < d_in; ++k)
        acc += widen16(X[t * d_in + k], act) * widen16(B[j * d_in + k], act);
      R[t * r + j] = acc;
    }
  return 0;
}

/* Eq. 9 for the listed output rows of one module (rows == NULL: all d_out rows).
 * R == NULL (unit not restored, or r == 0): the correction sum is absent.
 * Y is [T][n_rows] float64, column c holding output row rows[c]. */
int glowq_oracle_module_forward(const uint32_t* wq, const uint16_t* scales,
                                const uint16_t* zeros, const uint16_t* A, const uint16_t* X,
                                const double* R, int T, int d_in, int d_out, int r, int G,
                                int act, const int32_t* rows, int n_rows, double* Y) {
  if (!wq || !scales || !zeros || !X || !Y || G <= 0 || d_in % G || d_in % 8) return -1;
  if (R && !A) return -1;
  if (!rows) n_rows = d_out;
  int64_t ng = d_in / G;
  /* the stored activations, widened once */
  double* Xd = (double*)malloc(sizeof(double) * (size_t)T * (size_t)d_in);
  if (!Xd) return -2;
  for (int64_t i = 0; i < (int64_t)T * d_in; ++i) Xd[i] = widen16(X[i], act);
#pragma omp parallel
  {
    double* what = (double*)malloc(sizeof(double) * (size_t)d_in);
    double* arow = (double*)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
#pragma omp for schedule(dynamic, 4)
    for (int64_t c = 0; c < n_rows; ++c) {
      int64_t o = rows ? rows[c] : c;
      for (int64_t k = 0; k < d_in; ++k) {
        double s = widen16(scales[o * ng + k / G], 0);
        double z = widen16(zeros[o * ng + k / G], 0);
        what[k] = round16(((double)nibble(wq, o, k, d_in) - z) * s, act);
      }
      if (R)
        for (int64_t j = 0; j < r; ++j) arow[j] = widen16(A[o * r + j], act);
      for (int64_t t = 0; t < T; ++t) {
        double acc = 0.0;
        for (int64_t k = 0; k < d_in; ++k) acc += Xd[t * d_in + k] * what[k];
        if (R) {
          double corr = 0.0;
          for (int64_t j = 0; j < r; ++j) corr += R[t * r + j] * arow[j];
          acc += corr;
        }
        Y[t * (int64_t)n_rows + c] = acc;
      }
    }
    free(what);
    free(arow);
  }
  free(Xd);
  return 0;
}
