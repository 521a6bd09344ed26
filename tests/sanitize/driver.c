/* Sanitizer driver (AddressSanitizer + UndefinedBehaviorSanitizer, CPU only).
 *
 * Part 1 runs the naive C oracle on exact-size heap buffers with ragged shapes, so that
 * any read or write past an operand shows up; its results are also compared with a
 * second, independently written evaluation of the same sums (plain doubles, no bit
 * tricks) to make sure the instrumented build computes what the normal build computes.
 * Part 2 (only when built with -DWITH_GLOWQ_ABI) walks the host-side argument checks of
 * the C ABI: every call must come back with its status code and touch no GPU.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int glowq_oracle_unpack(const uint32_t* wq, int d_out, int d_in, uint8_t* q);
int glowq_oracle_dequant(const uint32_t* wq, const uint16_t* scales, const uint16_t* zeros,
                         int d_out, int d_in, int G, int act, double* what);
int glowq_oracle_shared_proj(const uint16_t* X, const uint16_t* B, int T, int d_in, int r, int act,
                             double* R);
int glowq_oracle_module_forward(const uint32_t* wq, const uint16_t* scales, const uint16_t* zeros,
                                const uint16_t* A, const uint16_t* X, const double* R, int T,
                                int d_in, int d_out, int r, int G, int act, const int32_t* rows,
                                int n_rows, double* Y);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void) {
  rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
  return (uint32_t)(rng_state >> 32);
}
/* small integers as binary16 / bfloat16 bit patterns: exact in both formats */
static uint16_t small_int_bits(int v, int act) {
  if (v == 0) return 0;
  int s = v < 0, a = s ? -v : v, e = 0;
  while ((a >> (e + 1)) != 0) ++e;                 /* a in [2^e, 2^(e+1)), a <= 15 here */
  int fbits = act ? 7 : 10, bias = act ? 127 : 15;
  int frac = (a - (1 << e)) << (fbits - e);
  return (uint16_t)((s << 15) | ((e + bias) << fbits) | frac);
}
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "FAILED %s:%d: %s\n", __FILE__, __LINE__, #c); exit(1); } } while (0)

static void oracle_case(int T, int d_in, int d_out, int r, int G, int act) {
  int ng = d_in / G;
  uint32_t* wq = malloc(sizeof(uint32_t) * d_out * (d_in / 8));
  uint16_t* sc = malloc(sizeof(uint16_t) * d_out * ng);
  uint16_t* zp = malloc(sizeof(uint16_t) * d_out * ng);
  uint16_t* A = malloc(sizeof(uint16_t) * d_out * (r ? r : 1));
  uint16_t* B = malloc(sizeof(uint16_t) * (r ? r : 1) * d_in);
  uint16_t* X = malloc(sizeof(uint16_t) * T * d_in);
  int* si = malloc(sizeof(int) * d_out * ng);      /* scales are powers of two: exact products */
  int* zi = malloc(sizeof(int) * d_out * ng);
  int* xi = malloc(sizeof(int) * T * d_in);
  int* ai = malloc(sizeof(int) * d_out * (r ? r : 1));
  int* bi = malloc(sizeof(int) * (r ? r : 1) * d_in);
  for (int i = 0; i < d_out * (d_in / 8); ++i) wq[i] = rnd();
  for (int i = 0; i < d_out * ng; ++i) { si[i] = 1 << (rnd() % 3); zi[i] = rnd() % 16;
    sc[i] = small_int_bits(si[i], 0); zp[i] = small_int_bits(zi[i], 0); }
  for (int i = 0; i < T * d_in; ++i) { xi[i] = (int)(rnd() % 7) - 3; X[i] = small_int_bits(xi[i], act); }
  for (int i = 0; i < d_out * r; ++i) { ai[i] = (int)(rnd() % 5) - 2; A[i] = small_int_bits(ai[i], act); }
  for (int i = 0; i < r * d_in; ++i) { bi[i] = (int)(rnd() % 5) - 2; B[i] = small_int_bits(bi[i], act); }

  uint8_t* q = malloc((size_t)d_out * d_in);
  CHECK(glowq_oracle_unpack(wq, d_out, d_in, q) == 0);
  double* what = malloc(sizeof(double) * d_out * d_in);
  CHECK(glowq_oracle_dequant(wq, sc, zp, d_out, d_in, G, act, what) == 0);
  for (int o = 0; o < d_out; ++o)
    for (int k = 0; k < d_in; ++k) {
      int qq = (int)((wq[o * (d_in / 8) + k / 8] >> (4 * (k % 8))) & 15u);
      CHECK(q[o * d_in + k] == qq);
      CHECK(what[o * d_in + k] == (double)((qq - zi[o * ng + k / G]) * si[o * ng + k / G]));
    }
  double* R = malloc(sizeof(double) * T * (r ? r : 1));
  if (r) CHECK(glowq_oracle_shared_proj(X, B, T, d_in, r, act, R) == 0);
  /* every second row, in reverse order, then all rows */
  int n_sel = (d_out + 1) / 2;
  int32_t* rows = malloc(sizeof(int32_t) * n_sel);
  for (int i = 0; i < n_sel; ++i) rows[i] = d_out - 1 - 2 * i;
  double* Ys = malloc(sizeof(double) * T * n_sel);
  double* Ya = malloc(sizeof(double) * T * d_out);
  CHECK(glowq_oracle_module_forward(wq, sc, zp, r ? A : NULL, X, r ? R : NULL, T, d_in, d_out, r, G,
                                    act, rows, n_sel, Ys) == 0);
  CHECK(glowq_oracle_module_forward(wq, sc, zp, r ? A : NULL, X, r ? R : NULL, T, d_in, d_out, r, G,
                                    act, NULL, 0, Ya) == 0);
  for (int t = 0; t < T; ++t)
    for (int o = 0; o < d_out; ++o) {
      long long acc = 0;                            /* everything is a small integer: exact */
      for (int k = 0; k < d_in; ++k)
        acc += (long long)xi[t * d_in + k] * (q[o * d_in + k] - zi[o * ng + k / G]) * si[o * ng + k / G];
      for (int j = 0; j < r; ++j) {
        long long rr = 0;
        for (int k = 0; k < d_in; ++k) rr += (long long)xi[t * d_in + k] * bi[j * d_in + k];
        CHECK(R[t * r + j] == (double)rr);
        acc += rr * ai[o * r + j];
      }
      CHECK(Ya[t * d_out + o] == (double)acc);
    }
  for (int t = 0; t < T; ++t)
    for (int i = 0; i < n_sel; ++i) CHECK(Ys[t * n_sel + i] == Ya[t * d_out + rows[i]]);
  free(wq); free(sc); free(zp); free(A); free(B); free(X); free(si); free(zi); free(xi); free(ai);
  free(bi); free(q); free(what); free(R); free(rows); free(Ys); free(Ya);
}

#ifdef WITH_GLOWQ_ABI
#include "../../include/glowq.h"
static glowq_unit make_unit(glowq_module* m, int T, int d_in, int r, int G) {
  glowq_unit u;
  memset(&u, 0, sizeof u);
  u.X = (void*)0x1000; u.B = (void*)0x2000; u.modules = m; u.n_modules = 1;
  u.T = T; u.d_in = d_in; u.r = r; u.group_size = G; u.act_dtype = GLOWQ_F16; u.out_dtype = GLOWQ_F32;
  return u;
}
static void abi_checks(void) {
  glowq_module m = {(void*)0x3000, (void*)0x4000, (void*)0x5000, 64, 64};
  glowq_unit u = make_unit(&m, 4, 256, 16, 64);
  size_t bytes = 0;
  CHECK(glowq_validate_unit(&u, 1) == GLOWQ_OK);
  CHECK(glowq_validate_unit(NULL, 1) == GLOWQ_ERR_NULL);
  CHECK(glowq_workspace_bytes(&u, 1, &bytes) == GLOWQ_OK && bytes > 0 && bytes % 256 == 0);
  CHECK(glowq_workspace_bytes(&u, 0, &bytes) == GLOWQ_ERR_SHAPE);
  CHECK(glowq_workspace_bytes(NULL, 1, &bytes) == GLOWQ_ERR_NULL);
  /* every size the planner is asked about: token counts of every kernel class, long
     contractions, every rank, many modules */
  static const int Ts[] = {1, 2, 3, 4, 5, 16, 17, 32, 33, 64, 65, 130, 512, 2048, 1 << 20};
  static const int Ks[] = {128, 256, 2048, 2176, 4096, 8192, 14336, 65536};
  glowq_module ms[GLOWQ_MAX_MODULES];
  for (int i = 0; i < GLOWQ_MAX_MODULES; ++i) { ms[i] = m; ms[i].d_out = 8 * (i + 1) * (i + 1); ms[i].ldy = ms[i].d_out + 8; }
  for (unsigned a = 0; a < sizeof Ts / sizeof *Ts; ++a)
    for (unsigned b = 0; b < sizeof Ks / sizeof *Ks; ++b)
      for (int r = 0; r <= GLOWQ_MAX_RANK; r += 8)
        for (int nm = 1; nm <= GLOWQ_MAX_MODULES; nm += 7) {
          glowq_unit v = make_unit(ms, Ts[a], Ks[b], r, 128);
          v.n_modules = nm;
          CHECK(glowq_workspace_bytes(&v, 1, &bytes) == GLOWQ_OK);
          CHECK(glowq_validate_unit(&v, 1) == GLOWQ_OK);
        }
  /* rejected before anything is enqueued (no GPU in this process) */
  glowq_unit bad = u; bad.d_in = 192;
  CHECK(glowq_group_forward(&bad, 1, (void*)0x9000, 1 << 20, NULL) == GLOWQ_ERR_UNSUPPORTED);
  bad = u; bad.T = 0;
  CHECK(glowq_group_forward(&bad, 1, (void*)0x9000, 1 << 20, NULL) == GLOWQ_ERR_SHAPE);
  bad = u; bad.X = (void*)0x1008;
  CHECK(glowq_block_forward(&bad, 1, NULL, (void*)0x9000, 1 << 20, NULL) == GLOWQ_ERR_ALIGN);
  CHECK(glowq_group_forward(&u, 1, NULL, 0, NULL) == GLOWQ_ERR_WORKSPACE);
  CHECK(glowq_group_forward(&u, 1, (void*)0x9000, 16, NULL) == GLOWQ_ERR_WORKSPACE);
  CHECK(glowq_group_forward_static(&bad, 1, NULL) == GLOWQ_ERR_ALIGN);
  uint32_t word;
  CHECK(glowq_workspace_status(&u, 1, (void*)0x9000, 16, &word, NULL) == GLOWQ_ERR_WORKSPACE);
  {
    /* layer-wise mode: the modules become one-module units on the callee's stack */
    glowq_unit lw = make_unit(ms, 4, 256, 16, 128);
    lw.n_modules = GLOWQ_MAX_MODULES;
    const void* Bs[GLOWQ_MAX_MODULES];
    for (int i = 0; i < GLOWQ_MAX_MODULES; ++i) Bs[i] = (void*)(uintptr_t)(0x2000 + 0x100 * i);
    size_t solo = 0, all = 0;
    glowq_unit one = lw; one.n_modules = 1;
    CHECK(glowq_workspace_bytes(&one, 1, &solo) == GLOWQ_OK);
    CHECK(glowq_layerwise_workspace_bytes(&lw, 1, &all) == GLOWQ_OK && all == GLOWQ_MAX_MODULES * solo);
    CHECK(glowq_layerwise_forward(&lw, 1, Bs, (void*)0x9000, all - 16, NULL) == GLOWQ_ERR_WORKSPACE);
    Bs[GLOWQ_MAX_MODULES - 1] = NULL;
    CHECK(glowq_layerwise_forward(&lw, 1, Bs, (void*)0x9000, all, NULL) == GLOWQ_ERR_NULL);
    CHECK(glowq_layerwise_forward(&lw, 1, NULL, (void*)0x9000, all, NULL) == GLOWQ_ERR_NULL);
  }
  {
    /* the offline side and the microscaling variant: workspace planning over every size
       class, and rejection before anything is enqueued */
    static const int Kf[] = {128, 512, 3072, 8192};
    for (unsigned b = 0; b < sizeof Kf / sizeof *Kf; ++b)
      for (int r = 8; r <= GLOWQ_MAX_RANK; r += 24)
        for (int p = 0; p <= 24; p += 8)
          for (int nm = 1; nm <= GLOWQ_MAX_MODULES; nm += 7) {
            glowq_unit v = make_unit(ms, 1, Kf[b], 0, 128);
            v.n_modules = nm;
            long long rows = 0;
            for (int i = 0; i < nm; ++i) rows += ms[i].d_out;
            glowq_status want = (r > rows || r + p > Kf[b]) ? GLOWQ_ERR_SHAPE : GLOWQ_OK;
            CHECK(glowq_factorize_workspace_bytes(&v, r, p, &bytes) == want);
            if (want == GLOWQ_OK) CHECK(bytes % 256 == 0 && bytes >= (size_t)rows * Kf[b] * 8);
          }
    const float* Wp[1] = {(const float*)0x7000};
    void* Ap[1] = {(void*)0xD000};
    glowq_unit f = make_unit(&m, 1, 256, 0, 128);
    CHECK(glowq_factorize_workspace_bytes(&f, 16, 8, &bytes) == GLOWQ_OK);
    CHECK(glowq_factorize_unit(&f, Wp, NULL, 16, 8, 2, (const double*)0xB000, (void*)0xC000, bytes - 1, Ap,
                               (void*)0xE000, NULL, NULL) == GLOWQ_ERR_WORKSPACE);
    CHECK(glowq_factorize_unit(&f, Wp, NULL, 16, 8, 9, (const double*)0xB000, (void*)0xC000, bytes, Ap,
                               (void*)0xE000, NULL, NULL) == GLOWQ_ERR_UNSUPPORTED);
    CHECK(glowq_factorize_unit(&f, Wp, NULL, 16, 8, 2, NULL, (void*)0xC000, bytes, Ap, (void*)0xE000, NULL,
                               NULL) == GLOWQ_ERR_NULL);
    CHECK(glowq_quantize_rtn(NULL, 64, 256, 128, (uint32_t*)0x8000, (uint16_t*)0x9000, (uint16_t*)0xA000, NULL) ==
          GLOWQ_ERR_NULL);
    CHECK(glowq_quantize_rtn((const float*)0x7000, 64, 200, 128, (uint32_t*)0x8000, (uint16_t*)0x9000,
                             (uint16_t*)0xA000, NULL) == GLOWQ_ERR_SHAPE);
    for (unsigned a = 0; a < sizeof Ts / sizeof *Ts; ++a)
      for (unsigned b = 0; b < sizeof Ks / sizeof *Ks; ++b)
        for (int r = 0; r <= GLOWQ_MAX_RANK; r += 64) {
          glowq_unit v = make_unit(ms, Ts[a], Ks[b], r, 0);
          v.n_modules = GLOWQ_MAX_MODULES;
          CHECK(glowq_mx_workspace_bytes(&v, &bytes) == GLOWQ_OK && bytes % 256 == 0);
          CHECK(bytes >= (size_t)(Ts[a] > 16 ? Ts[a] : 16) * Ks[b]);
        }
    glowq_unit x = make_unit(&m, 4, 256, 16, 0);
    CHECK(glowq_mx_workspace_bytes(&x, &bytes) == GLOWQ_OK);
    CHECK(glowq_mx_group_forward(&x, 1, (void*)0xC000, bytes - 1, NULL) == GLOWQ_ERR_WORKSPACE);
    CHECK(glowq_mx_group_forward(&x, 1, (void*)0xC010, bytes, NULL) == GLOWQ_ERR_ALIGN);
    CHECK(glowq_mx_prepared_bytes(40, 256, &bytes) == GLOWQ_OK && bytes == 3 * 2 * 1088);
    CHECK(glowq_mx_prepare_weights(NULL, NULL, 64, 256, NULL, NULL) == GLOWQ_ERR_NULL);
    CHECK(glowq_mx_quantize_activations((void*)0x7000, 4, 250, GLOWQ_F16, (uint8_t*)0x8000, (uint8_t*)0x9000,
                                        NULL) == GLOWQ_ERR_SHAPE);
  }
  CHECK(glowq_prepared_bytes(40, 128, 128, &bytes) == GLOWQ_OK && bytes == 3 * 272 * 4);
  CHECK(glowq_prepared_bytes(40, 100, 128, &bytes) == GLOWQ_ERR_SHAPE);
  CHECK(glowq_prepare_weights(NULL, NULL, NULL, 64, 256, 64, NULL, NULL) == GLOWQ_ERR_NULL);
  for (int s = GLOWQ_ERR_HIP; s <= GLOWQ_OK; ++s) CHECK(strlen(glowq_status_string((glowq_status)s)) > 0);
}
#endif

int main(void) {
  static const int cases[][5] = {{1, 128, 8, 0, 128}, {3, 192, 24, 8, 64}, {5, 256, 40, 24, 128},
                                 {17, 384, 9, 16, 64}, {2, 64, 1, 8, 64}};
  for (unsigned c = 0; c < sizeof cases / sizeof *cases; ++c)
    for (int act = 0; act < 2; ++act)
      oracle_case(cases[c][0], cases[c][1], cases[c][2], cases[c][3], cases[c][4], act);
#ifdef WITH_GLOWQ_ABI
  abi_checks();
  printf("sanitizer driver: oracle and ABI host checks clean\n");
#else
  printf("sanitizer driver: oracle clean\n");
#endif
  return 0;
}
