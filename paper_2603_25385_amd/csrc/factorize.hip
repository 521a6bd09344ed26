// Shared factors of one unit's stacked quantisation error, computed on the GPU
// (paper Alg. 1 and App. A.3-A.4: randomised range finder with power steps on the
// covariance-aligned error, small SVD, balanced split, lift back).  Offline work, no part
// of the forward.  Everything is float64.
//
//   Ms     = E_cat Sigma_x^(1/2)            E_cat = [W_i - dequant(W_q,i)]_i stacked by rows
//   Y      = Ms Omega,  q times  Y <- Ms (Ms^T Y)
//   Q      = orth(Y)                        classical Gram-Schmidt, every column twice
//   Bs     = Q^T Ms = U~ S V^T              one-sided Jacobi on the rows of Bs
//   A      = Q U~_r S_r^(1/2),  B = S_r^(1/2) V_r^T Sigma_x^(-1/2)
//
// The algorithm in the paper first replaces the m x d stack by the d x d triangular factor
// of its thin QR, so that a dense SVD of the core is affordable.  With the operator form of
// the range finder (App. A.3: only products with M and M^T are needed) the products run on
// the stack itself here: Q_e M = E_cat Sigma_x^(1/2), so every quantity below is Q_e times
// (or equal to) its counterpart on the core and A, B come out the same; forming the Gram
// matrix or a Householder QR of the stack would cost m d^2 operations against
// (2q + 2) m d (r + p) for the products.
//
// The matrix products are float64 matrix-core contractions (16x16x4), one wave per output
// tile and K slice, partial results in slices that a second kernel adds in slice order, so
// results do not depend on timing.
#include "common.hpp"
#include "launch.hpp"
#include <algorithm>

namespace glowq {

typedef double double4_t __attribute__((ext_vector_type(4)));

constexpr int FZ_NT = 5;            // 16-column blocks per pass of a product (80 columns)
constexpr int FZ_TARGET_WAVES = 2048;

// ---------------------------------------------------------------------------------------
// the stack
// ---------------------------------------------------------------------------------------
__global__ void k_roots(const double* __restrict__ sigma, int d, double* root, double* inv_root) {
  const int k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= d) return;
  const double s = sigma[k];
  const double r = s > 0.0 ? sqrt(s) : 0.0;
  root[k] = r;
  inv_root[k] = r > 0.0 ? 1.0 / r : 0.0;      // (pseudo-inverse on a zero variance)
}

// Ms[row_off + o][k] = (W[o][k] - What[o][k]) * root[k], What the stored 16-bit weight.
// A block per tile record, lanes as in the record (row l & 15, channels 32 j + 8 (l >> 4)).
template <int ACT>
__global__ void __launch_bounds__(256) k_error_stack(const float* __restrict__ W, const void* prepared,
                                                     int d_out, int d_in, int G,
                                                     const double* __restrict__ root,
                                                     double* __restrict__ Ms, long long row_off) {
  PreparedView v = prepared_view(prepared, d_out, d_in, G);
  const int n_rec = v.rows16 * v.ktiles;
  const int j = threadIdx.x >> 6, lane = threadIdx.x & 63;
  for (int rec = (int)blockIdx.x; rec < n_rec; rec += (int)gridDim.x) {
    const int rb = rec / v.ktiles, kt = rec - rb * v.ktiles;
    const int row = rb * 16 + (lane & 15), k = kt * 128 + 32 * j + 8 * (lane >> 4);
    if (row >= d_out) continue;
    const uint32_t* r = tile_record(v, rb, kt);
    GroupConst<ACT> g;
    g.set(r[256 + 16 * ((k & 127) / G) + (row & 15)]);
    const u32x4_t dq = dequant_word<ACT>(r[lane * 4 + j], g);
    const float4_t* src = (const float4_t*)(W + (long long)row * d_in + k);
    const float4_t w0 = src[0], w1 = src[1];
    const float w[8] = {w0[0], w0[1], w0[2], w0[3], w1[0], w1[1], w1[2], w1[3]};
    double* dst = Ms + (row_off + row) * (long long)d_in + k;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t word = dq[i >> 1];
      const double wh = act16_value<ACT>((i & 1) ? (word >> 16) : (word & 0xffffu));
      double e = (double)w[i] - wh;
      if (root) e *= root[k + i];
      dst[i] = e;
    }
  }
}

// ---------------------------------------------------------------------------------------
// float64 products on the matrix cores.  v_mfma_f64_16x16x4: lane l holds A[l & 15][l >> 4],
// B[l >> 4][l & 15] and, in register v, D[(l >> 4) + 4 v][l & 15].
// One wave owns a tile of 16 RB rows x 16 NT columns over one K slice and writes it to
// slice ks of P ([KS][M][ldp]).  Operands come straight from global memory (the small one
// stays in the L2s); rows, columns and K past the edge are clamped on the load and dropped
// (zeroed, for K) afterwards.
// ---------------------------------------------------------------------------------------
struct GemmShape {
  int M, N, K;
  int n0;          // first column of this pass
  int kslice;      // channels of K per slice (multiple of 16)
  int n_slices;
  int row_tiles;   // ceil(M / (16 RB))
};

// C = A B, A [M][lda] and B [K][ldb] row-major.  Within a step of 16 channels lane group g
// owns channels 4g .. 4g + 3 (contiguous in a row of A); instruction t multiplies channel
// 4g + t of every group.
template <int RB, int NT>
__global__ void __launch_bounds__(256) k_gemm_nn(const double* __restrict__ A, long long lda,
                                                 const double* __restrict__ B, long long ldb,
                                                 double* __restrict__ P, long long ldp, GemmShape s) {
  const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int tile = wave % s.row_tiles, ks = wave / s.row_tiles;
  if (ks >= s.n_slices) return;
  const int l = threadIdx.x & 63, i = l & 15, g = l >> 4;
  const int kbeg = ks * s.kslice, kend = min(s.K, kbeg + s.kslice);
  double4_t acc[RB][NT];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[rb][nt] = double4_t{0.0, 0.0, 0.0, 0.0};
  const double* arow[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) arow[rb] = A + (long long)min(s.M - 1, tile * 16 * RB + rb * 16 + i) * lda;
  int bcol[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) bcol[nt] = min(s.N - 1, s.n0 + 16 * nt + i);
  for (int k0 = kbeg; k0 < kend; k0 += 16) {
    double a[RB][4], b[4][NT];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int kk = k0 + 4 * g + t, kc = min(kk, s.K - 1);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        const double v = arow[rb][kc];
        a[rb][t] = kk < kend ? v : 0.0;
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) b[t][nt] = B[(long long)kc * ldb + bcol[nt]];
    }
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
          acc[rb][nt] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[rb][t], b[t][nt], acc[rb][nt], 0, 0, 0);
  }
  double* Ps = P + (long long)ks * s.M * ldp;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = tile * 16 * RB + rb * 16 + g + 4 * v, col = s.n0 + 16 * nt + i;
        if (row < s.M && col < s.N) Ps[(long long)row * ldp + col] = acc[rb][nt][v];
      }
}

// C = A^T B, A [K][lda] (M columns) and B [K][ldb] (N columns) row-major: both operands are
// read along their rows.
template <int RB, int NT>
__global__ void __launch_bounds__(256) k_gemm_tn(const double* __restrict__ A, long long lda,
                                                 const double* __restrict__ B, long long ldb,
                                                 double* __restrict__ P, long long ldp, GemmShape s) {
  const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int tile = wave % s.row_tiles, ks = wave / s.row_tiles;
  if (ks >= s.n_slices) return;
  const int l = threadIdx.x & 63, i = l & 15, g = l >> 4;
  const int kbeg = ks * s.kslice, kend = min(s.K, kbeg + s.kslice);
  double4_t acc[RB][NT];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[rb][nt] = double4_t{0.0, 0.0, 0.0, 0.0};
  int acol[RB], bcol[NT];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) acol[rb] = min(s.M - 1, tile * 16 * RB + rb * 16 + i);
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) bcol[nt] = min(s.N - 1, s.n0 + 16 * nt + i);
  for (int k0 = kbeg; k0 < kend; k0 += 16) {
    double a[4][RB], b[4][NT];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int kk = k0 + 4 * t + g, kc = min(kk, s.K - 1);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        const double v = A[(long long)kc * lda + acol[rb]];
        a[t][rb] = kk < kend ? v : 0.0;
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) b[t][nt] = B[(long long)kc * ldb + bcol[nt]];
    }
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
          acc[rb][nt] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[t][rb], b[t][nt], acc[rb][nt], 0, 0, 0);
  }
  double* Ps = P + (long long)ks * s.M * ldp;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = tile * 16 * RB + rb * 16 + g + 4 * v, col = s.n0 + 16 * nt + i;
        if (row < s.M && col < s.N) Ps[(long long)row * ldp + col] = acc[rb][nt][v];
      }
}

// C[row][col] (or C[col][row] when transposed) = sum over slices, in slice order
__global__ void k_reduce_slices(const double* __restrict__ P, long long ldp, int n_slices, int M, int N,
                                double* __restrict__ C, long long ldc, int transposed) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)M * N) return;
  const int row = (int)(idx / N), col = (int)(idx - (long long)row * N);
  double sum = 0.0;
  for (int sl = 0; sl < n_slices; ++sl) sum += P[((long long)sl * M + row) * ldp + col];
  if (transposed) C[(long long)col * ldc + row] = sum;
  else C[(long long)row * ldc + col] = sum;
}

struct GemmPlan {
  int kslice, n_slices, row_tiles;
};

static GemmPlan plan_gemm(int M, int K, int RB) {
  GemmPlan p;
  p.row_tiles = (M + 16 * RB - 1) / (16 * RB);
  int want = (FZ_TARGET_WAVES + p.row_tiles - 1) / p.row_tiles;
  const int max_slices = (K + 15) / 16;
  if (want > max_slices) want = max_slices;
  if (want > 64) want = 64;
  if (want < 1) want = 1;
  p.kslice = (((K + want - 1) / want) + 15) / 16 * 16;
  p.n_slices = (K + p.kslice - 1) / p.kslice;
  return p;
}

constexpr int NN_RB = 2, TN_RB = 4;

static size_t gemm_slice_doubles(int M, int N, int K, int RB) {
  const GemmPlan p = plan_gemm(M, K, RB);
  return (size_t)p.n_slices * (size_t)M * (size_t)((N + 15) / 16 * 16);
}

template <bool TN, int NT>
static void launch_gemm_pass(const double* A, long long lda, const double* B, long long ldb, double* P,
                             long long ldp, const GemmShape& s, hipStream_t st) {
  const int waves = s.row_tiles * s.n_slices;
  dim3 grid((unsigned)((waves + 3) / 4)), block(256);
  if (TN) k_gemm_tn<TN_RB, NT><<<grid, block, 0, st>>>(A, lda, B, ldb, P, ldp, s);
  else k_gemm_nn<NN_RB, NT><<<grid, block, 0, st>>>(A, lda, B, ldb, P, ldp, s);
}

// C [M][N] = op(A) B through the slice buffer
template <bool TN>
static hipError_t gemm(const double* A, long long lda, const double* B, long long ldb, double* C,
                       long long ldc, bool c_transposed, int M, int N, int K, double* slices,
                       hipStream_t st) {
  const GemmPlan p = plan_gemm(M, K, TN ? TN_RB : NN_RB);
  const long long ldp = (N + 15) / 16 * 16;
  GemmShape s;
  s.M = M; s.N = N; s.K = K;
  s.kslice = p.kslice; s.n_slices = p.n_slices; s.row_tiles = p.row_tiles;
  for (int n0 = 0; n0 < N; n0 += 16 * FZ_NT) {
    s.n0 = n0;
    const int nt = (std::min(N - n0, 16 * FZ_NT) + 15) / 16;
    switch (nt) {
      case 1: launch_gemm_pass<TN, 1>(A, lda, B, ldb, slices, ldp, s, st); break;
      case 2: launch_gemm_pass<TN, 2>(A, lda, B, ldb, slices, ldp, s, st); break;
      case 3: launch_gemm_pass<TN, 3>(A, lda, B, ldb, slices, ldp, s, st); break;
      case 4: launch_gemm_pass<TN, 4>(A, lda, B, ldb, slices, ldp, s, st); break;
      default: launch_gemm_pass<TN, 5>(A, lda, B, ldb, slices, ldp, s, st); break;
    }
  }
  const long long n = (long long)M * N;
  k_reduce_slices<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st>>>(slices, ldp, p.n_slices, M, N, C,
                                                                          ldc, c_transposed ? 1 : 0);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Q = orth(Y): classical Gram-Schmidt, every column projected twice.  Y is [m][ld], l
// columns, l <= 256.  Workgroup b owns rows [b rpw, (b + 1) rpw), rpw <= 256, in every
// launch; sums over rows go through per-workgroup partials that every workgroup adds in the
// same order.  Three launches per column j:
//   phase 0: finish column j - 1 (scale by 1 / norm, or clear a column that the projections
//            took below the rank threshold); partial c1 = Q^T y_j, partial |y_j|^2
//   phase 1: y_j -= Q c1; partial c2 = Q^T y_j
//   phase 2: y_j -= Q c2; partial |y_j|^2
// and one more phase 0 with j = l that only finishes the last column.
// ---------------------------------------------------------------------------------------
struct CgsBuffers {
  double* c1;       // [n_groups][256]
  double* c2;       // [n_groups][256]
  double* norm;     // [n_groups]      |y_j|^2 after both projections
  double* norm0;    // [2][n_groups]   |y_j|^2 before, by parity of j
};

constexpr double FZ_RANK_TOL2 = 1e-24;      // a column whose norm^2 fell by this factor is dependent

__device__ inline double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  return v;
}

// sum of one value per thread over the block; every thread gets the result
__device__ inline double block_sum(double v, double* lds4) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) lds4[threadIdx.x >> 6] = v;
  __syncthreads();
  return lds4[0] + lds4[1] + lds4[2] + lds4[3];
}

// dot[t] = sum over the rows [r0, r1) of Y[k][t] * ycol[k - r0] for every column t < j, by all 256
// threads: the rows are dealt to 256 / CW thread groups of CW >= j columns, whose partial sums
// meet in `part` (256 doubles of LDS); thread t < j returns the sum, in group order
__device__ inline double cgs_dots(const double* __restrict__ Y, long long ld, int r0, int r1, int j,
                                  const double* ycol, double* part) {
  const int t = threadIdx.x;
  const int CW = j <= 64 ? 64 : (j <= 128 ? 128 : 256), n_sub = 256 / CW;
  const int col = t & (CW - 1), sub = t / CW;
  double dot = 0.0;
  if (col < j) {
#pragma unroll 8
    for (int k = r0 + sub; k < r1; k += n_sub) dot += Y[(long long)k * ld + col] * ycol[k - r0];
  }
  __syncthreads();
  part[t] = dot;
  __syncthreads();
  double sum = 0.0;
  if (t < j)
    for (int sgrp = 0; sgrp < n_sub; ++sgrp) sum += part[sgrp * CW + t];
  return sum;
}

__global__ void __launch_bounds__(256) k_cgs(double* __restrict__ Y, long long ld, int m, int l, int rpw,
                                             int n_groups, int j, int phase, CgsBuffers cb) {
  __shared__ double c[256];
  __shared__ double ycol[256];
  __shared__ double red[4];
  const int t = threadIdx.x, b = blockIdx.x;
  const int r0 = b * rpw, r1 = min(m, r0 + rpw);
  if (phase == 0) {
    if (j > 0) {
      // finish column j - 1 (every workgroup adds the partial norms in the same order)
      double n2 = 0.0, n0 = 0.0;
      for (int gq = t; gq < n_groups; gq += 256) {
        n2 += cb.norm[gq];
        n0 += cb.norm0[(size_t)((j - 1) & 1) * n_groups + gq];
      }
      n2 = block_sum(n2, red);
      n0 = block_sum(n0, red);
      const double scale = (n2 > FZ_RANK_TOL2 * n0 && n2 > 0.0) ? 1.0 / sqrt(n2) : 0.0;
      for (int k = r0 + t; k < r1; k += 256) Y[(long long)k * ld + (j - 1)] *= scale;
      __syncthreads();       // (the scaled column is read below, by other threads)
    }
    if (j >= l) return;
    for (int k = r0 + t; k < r1; k += 256) ycol[k - r0] = Y[(long long)k * ld + j];
    __syncthreads();
    double nn = 0.0;
    const double dot = cgs_dots(Y, ld, r0, r1, j, ycol, c);
    cb.c1[(size_t)b * 256 + t] = dot;
    for (int k = r0 + t; k < r1; k += 256) nn += ycol[k - r0] * ycol[k - r0];
    nn = block_sum(nn, red);
    if (t == 0) cb.norm0[(size_t)(j & 1) * n_groups + b] = nn;
    return;
  }
  // phases 1 and 2: coefficients, in workgroup order
  const double* part = phase == 1 ? cb.c1 : cb.c2;
  double ct = 0.0;
  if (t < j) {
#pragma unroll 16
    for (int gq = 0; gq < n_groups; ++gq) ct += part[(size_t)gq * 256 + t];
  }
  c[t] = ct;
  __syncthreads();
  // sixteen lanes per row: y_k -= sum_i Q[k][i] c[i]   (every lane runs the same number of
  // rounds, so that the shuffles below see whole waves)
  const int slot = t >> 4, sub = t & 15;
  for (int kb = r0; kb < r1; kb += 16) {
    const int k = kb + slot;
    double sum = 0.0;
    if (k < r1)
      for (int i = sub; i < j; i += 16) sum += Y[(long long)k * ld + i] * c[i];
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    if (sub == 0 && k < r1) {
      const double y = Y[(long long)k * ld + j] - sum;
      Y[(long long)k * ld + j] = y;
      ycol[k - r0] = y;
    }
  }
  __syncthreads();
  if (phase == 1) {
    const double dot = cgs_dots(Y, ld, r0, r1, j, ycol, c);     // (c is free again: barrier inside)
    cb.c2[(size_t)b * 256 + t] = dot;
  } else {
    double nn = 0.0;
    for (int k = r0 + t; k < r1; k += 256) nn += ycol[k - r0] * ycol[k - r0];
    nn = block_sum(nn, red);
    if (t == 0) cb.norm[b] = nn;
  }
}

// ---------------------------------------------------------------------------------------
// SVD of Bs [l][d] by one-sided Jacobi rotations of its rows (Hestenes): a rotation of rows
// (a, b) makes them orthogonal; at convergence row a is sigma_a v_a^T and the accumulated
// rotations, applied to the columns of Um, leave U~ in Um.  One launch per round of a round-robin schedule over n = l rounded up to even players
// (n / 2 disjoint pairs, a workgroup each); a sweep is n - 1 rounds.  counters[w] counts the
// rotations of sweep w; once a sweep made none, the launches of later sweeps return at once.
// ---------------------------------------------------------------------------------------
constexpr int FZ_MAX_SWEEPS = 16;
constexpr int FZ_POLISH_SWEEPS = 8;     // after the rotation by the Gram matrix's eigenvectors
constexpr double FZ_JACOBI_TOL2 = 1e-28;     // rotate while (a.b)^2 > tol^2 |a|^2 |b|^2, tol = 1e-14

constexpr int FZ_JT = 1024;       // threads of a Jacobi workgroup
constexpr int FZ_JC = 4;          // elements of each row a thread keeps in registers

__global__ void __launch_bounds__(FZ_JT) k_jacobi_round(double* __restrict__ Bs, long long ldb, int d,
                                                        double* __restrict__ Um, long long ldu, int l, int n,
                                                        int round, int sweep, int* counters) {
  __shared__ double red[3][FZ_JT / 64];
  if (sweep > 0 && counters[sweep - 1] == 0) return;
  const int k = blockIdx.x, t = threadIdx.x;
  int a, b;
  if (k == 0) { a = n - 1; b = round; }
  else { a = (round + k) % (n - 1); b = (round - k + (n - 1)) % (n - 1); }
  if (a >= l || b >= l) return;      // the odd player out
  double* ra = Bs + (long long)a * ldb;
  double* rb = Bs + (long long)b * ldb;
  double xa[FZ_JC], xb[FZ_JC];
  double aa = 0.0, bb = 0.0, ab = 0.0;
#pragma unroll
  for (int c = 0; c < FZ_JC; ++c) {
    const int i = t + c * FZ_JT;
    xa[c] = i < d ? ra[i] : 0.0;
    xb[c] = i < d ? rb[i] : 0.0;
    aa += xa[c] * xa[c]; bb += xb[c] * xb[c]; ab += xa[c] * xb[c];
  }
  for (int i = t + FZ_JC * FZ_JT; i < d; i += FZ_JT) {
    const double x = ra[i], y = rb[i];
    aa += x * x; bb += y * y; ab += x * y;
  }
  aa = wave_sum(aa); bb = wave_sum(bb); ab = wave_sum(ab);
  if ((t & 63) == 0) { red[0][t >> 6] = aa; red[1][t >> 6] = bb; red[2][t >> 6] = ab; }
  __syncthreads();
  aa = bb = ab = 0.0;
#pragma unroll
  for (int w = 0; w < FZ_JT / 64; ++w) { aa += red[0][w]; bb += red[1][w]; ab += red[2][w]; }
  if (!(ab * ab > FZ_JACOBI_TOL2 * aa * bb)) return;
  if (t == 0) atomicAdd(&counters[sweep], 1);
  const double zeta = (bb - aa) / (2.0 * ab);
  const double tt = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
  const double cs = 1.0 / sqrt(1.0 + tt * tt), sn = cs * tt;
#pragma unroll
  for (int c = 0; c < FZ_JC; ++c) {
    const int i = t + c * FZ_JT;
    if (i < d) {
      ra[i] = cs * xa[c] - sn * xb[c];
      rb[i] = sn * xa[c] + cs * xb[c];
    }
  }
  for (int i = t + FZ_JC * FZ_JT; i < d; i += FZ_JT) {
    const double x = ra[i], y = rb[i];
    ra[i] = cs * x - sn * y;
    rb[i] = sn * x + cs * y;
  }
  for (int i = t; i < l; i += FZ_JT) {
    double* u = Um + (long long)i * ldu;
    const double x = u[a], y = u[b];
    u[a] = cs * x - sn * y;
    u[b] = sn * x + cs * y;
  }
}

// Eigenvectors of the l x l Gram matrix T = Bs Bs^T by two-sided Jacobi rotations, one
// workgroup, T in LDS (l <= FZ_EIG_MAX): with Um = its eigenvectors, the rows of Um^T Bs
// are orthogonal up to the rounding of the Gram matrix, so that the one-sided rotations on
// the long rows that follow only polish (one or two sweeps instead of eight or nine).  The
// same rotation G = [[c, -s], [s, c]] on the pair (a, b) as above: T <- G T G^T, rows then
// columns, and the columns of Um.  Rounds pair the players as above; all pairs of a round
// are disjoint and are rotated together.
constexpr int FZ_EIG_MAX = 128;
constexpr int FZ_EIG_SWEEPS = 8;
constexpr int FZ_EIG_LDS_DOUBLES = 19 * 1024;     // 152 KiB: T, and Um beside it when both fit (l <= 97)
constexpr double FZ_EIG_TOL2 = 1e-20;             // rotate while (T_ab)^2 > tol^2 T_aa T_bb, tol = 1e-10 ...
constexpr double FZ_EIG_ABS = 1e-13;              // ... and |T_ab| is above the rounding of the largest entry

__global__ void __launch_bounds__(1024) k_gram_eigenvectors(const double* __restrict__ Tg, long long ldt, int l,
                                                            double* __restrict__ Um, long long ldu) {
  __shared__ double pool[FZ_EIG_LDS_DOUBLES];
  __shared__ double cs[FZ_EIG_MAX / 2], sn[FZ_EIG_MAX / 2];
  __shared__ int pa[FZ_EIG_MAX / 2], pb[FZ_EIG_MAX / 2];
  __shared__ int rotated;
  __shared__ double tmax;
  const int t = threadIdx.x, LD = l + 1;
  double* T = pool;
  const bool u_in_lds = 2 * l * LD <= FZ_EIG_LDS_DOUBLES;
  double* U = u_in_lds ? pool + l * LD : Um;           // (generic pointer: LDS or global)
  const long long LDU = u_in_lds ? LD : ldu;
  for (int idx = t; idx < l * l; idx += 1024) {
    const int i = idx / l, k = idx - i * l;
    T[i * LD + k] = Tg[(long long)i * ldt + k];
    U[(long long)i * LDU + k] = i == k ? 1.0 : 0.0;
  }
  __syncthreads();
  if (t == 0) {
    double mx = 0.0;
    for (int i = 0; i < l; ++i) mx = fmax(mx, T[i * LD + i]);
    tmax = mx;
  }
  const int n = (l + 1) & ~1, pairs = n / 2;
  for (int sweep = 0; sweep < FZ_EIG_SWEEPS; ++sweep) {
    __syncthreads();
    if (t == 0) rotated = 0;
    for (int round = 0; round < n - 1; ++round) {
      __syncthreads();
      if (t < pairs) {
        int a, b;
        if (t == 0) { a = n - 1; b = round; }
        else { a = (round + t) % (n - 1); b = (round - t + (n - 1)) % (n - 1); }
        double c = 1.0, s = 0.0;
        if (a < l && b < l) {
          const double aa = T[a * LD + a], bb = T[b * LD + b], ab = T[a * LD + b];
          if (ab * ab > FZ_EIG_TOL2 * aa * bb && fabs(ab) > FZ_EIG_ABS * tmax) {
            const double zeta = (bb - aa) / (2.0 * ab);
            const double tt = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
            c = 1.0 / sqrt(1.0 + tt * tt);
            s = c * tt;
            rotated = 1;
          }
        } else {
          a = b = -1;
        }
        pa[t] = a; pb[t] = b; cs[t] = c; sn[t] = s;
      }
      __syncthreads();
      // rows a, b of every pair
      for (int idx = t; idx < pairs * l; idx += 1024) {
        const int k = idx / l, i = idx - k * l, a = pa[k], b = pb[k];
        if (a < 0 || sn[k] == 0.0) continue;
        const double x = T[a * LD + i], y = T[b * LD + i];
        T[a * LD + i] = cs[k] * x - sn[k] * y;
        T[b * LD + i] = sn[k] * x + cs[k] * y;
      }
      __syncthreads();
      // columns a, b of every pair, of T and of the eigenvector matrix
      for (int idx = t; idx < pairs * l; idx += 1024) {
        const int k = idx / l, i = idx - k * l, a = pa[k], b = pb[k];
        if (a < 0 || sn[k] == 0.0) continue;
        const double x = T[i * LD + a], y = T[i * LD + b];
        T[i * LD + a] = cs[k] * x - sn[k] * y;
        T[i * LD + b] = sn[k] * x + cs[k] * y;
        double* u = U + (long long)i * LDU;
        const double ux = u[a], uy = u[b];
        u[a] = cs[k] * ux - sn[k] * uy;
        u[b] = sn[k] * ux + cs[k] * uy;
      }
    }
    __syncthreads();
    if (rotated == 0) break;
  }
  if (u_in_lds) {
    __syncthreads();
    for (int idx = t; idx < l * l; idx += 1024) {
      const int i = idx / l, k = idx - i * l;
      Um[(long long)i * ldu + k] = U[(long long)i * LDU + k];
    }
  }
}

__global__ void k_identity(double* U, long long ld, int l) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= l * l) return;
  const int a = idx / l, i = idx - a * l;
  U[(long long)a * ld + i] = a == i ? 1.0 : 0.0;
}

// sig2[a] = |row a of Bs|^2; one block per row
__global__ void __launch_bounds__(256) k_row_norms(const double* __restrict__ Bs, long long ldb, int d,
                                                   double* sig2) {
  __shared__ double red[4];
  const double* r = Bs + (long long)blockIdx.x * ldb;
  double s = 0.0;
  for (int i = threadIdx.x; i < d; i += 256) s += r[i] * r[i];
  s = block_sum(s, red);
  if (threadIdx.x == 0) sig2[blockIdx.x] = s;
}

// descending order of the singular values (equal values: lower row first); one block
__global__ void __launch_bounds__(256) k_sort_sigma(const double* sig2, int l, double* sigma_sorted, int* perm) {
  const int a = threadIdx.x;
  if (a >= l) return;
  const double s = sig2[a];
  int rank = 0;
  for (int b = 0; b < l; ++b) {
    const double o = sig2[b];
    rank += (o > s || (o == s && b < a)) ? 1 : 0;
  }
  sigma_sorted[rank] = sqrt(s);
  perm[rank] = a;
}

// P[i][jr] = U~[i][perm jr] sqrt(sigma_jr): the l x r matrix that takes Q to A (Alg. 1,
// lift and balance)
__global__ void k_build_lift(const double* __restrict__ Um, long long ldu, const double* sigma_sorted,
                             const int* perm, int l, int r, double* P, long long ldp) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= l * r) return;
  const int i = idx / r, jr = idx - i * r;
  P[(long long)i * ldp + jr] = Um[(long long)i * ldu + perm[jr]] * sqrt(sigma_sorted[jr]);
}

template <int ACT>
__global__ void k_store_A(const double* __restrict__ A64, long long lda, long long row_off, int d_out, int r,
                          uint16_t* __restrict__ A) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)d_out * r) return;
  const long long o = idx / r;
  const int j = (int)(idx - o * r);
  A[idx] = (uint16_t)act16_round<ACT>(A64[(row_off + o) * lda + j]);
}

// B[jr][k] = row perm jr of Bs / sqrt(sigma_jr) * Sigma_x^(-1/2)[k]
template <int ACT>
__global__ void k_store_B(const double* __restrict__ Bs, long long ldb, const double* sigma_sorted,
                          const int* perm, const double* __restrict__ inv_root, int r, int d,
                          uint16_t* __restrict__ B) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)r * d) return;
  const int jr = (int)(idx / d), k = (int)(idx - (long long)jr * d);
  const double s = sigma_sorted[jr];
  double v = s > 0.0 ? Bs[(long long)perm[jr] * ldb + k] / sqrt(s) : 0.0;
  if (inv_root) v *= inv_root[k];
  B[idx] = (uint16_t)act16_round<ACT>(v);
}

__global__ void k_copy_doubles(const double* src, double* dst, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
static size_t up256(size_t b) { return (b + 255) & ~(size_t)255; }

FactorizePlan plan_factorize(const glowq_unit& u, int r, int p) {
  FactorizePlan f;
  long long m = 0;
  for (int i = 0; i < u.n_modules; ++i) m += u.modules[i].d_out;
  f.m = m;
  f.d = u.d_in;
  f.l = r + p;
  f.l16 = (f.l + 15) / 16 * 16;
  f.r16 = (r + 15) / 16 * 16;
  f.n_groups = (int)((m + 255) / 256);                 // at most 256 rows per group ...
  if (f.n_groups < 64) f.n_groups = (int)(m < 64 ? m : 64);   // ... and few groups: their partial sums are added serially
  f.rpw = (int)((m + f.n_groups - 1) / f.n_groups);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += up256(bytes); return o; };
  f.off_ms = take((size_t)m * f.d * 8);
  f.off_y = take((size_t)m * f.l16 * 8);
  f.off_z = take((size_t)f.d * f.l16 * 8);
  f.off_bs = take((size_t)f.l * f.d * 8);
  f.off_ut = take((size_t)f.l * f.l16 * 8);
  f.off_gram = take((size_t)f.l * f.l16 * 8);
  f.off_lift = take((size_t)f.l * f.r16 * 8);
  f.off_a64 = take((size_t)m * f.r16 * 8);
  size_t sl = gemm_slice_doubles((int)m, f.l, f.d, NN_RB);                      // Y = Ms Omega, Y = Ms Z
  size_t s2 = gemm_slice_doubles(f.d, f.l, (int)m, TN_RB);                      // Z = Ms^T Y, Bs^T = Ms^T Q
  size_t s3 = gemm_slice_doubles((int)m, r, f.l, NN_RB);                        // A = Q P
  size_t s4 = gemm_slice_doubles(f.l, f.l, f.d, TN_RB);                         // Gram of Bs
  size_t s5 = gemm_slice_doubles(f.d, f.l, f.l, NN_RB);                         // rows = Um^T Bs
  for (size_t o : {s2, s3, s4, s5})
    if (o > sl) sl = o;
  f.off_slices = take(sl * 8);
  f.off_root = take((size_t)f.d * 8);
  f.off_inv_root = take((size_t)f.d * 8);
  f.off_c1 = take((size_t)f.n_groups * 256 * 8);
  f.off_c2 = take((size_t)f.n_groups * 256 * 8);
  f.off_norm = take((size_t)f.n_groups * 8);
  f.off_norm0 = take((size_t)2 * f.n_groups * 8);
  f.off_sig2 = take(256 * 8);
  f.off_sigma = take(256 * 8);
  f.off_perm = take(256 * 4);
  f.off_counters = take(FZ_MAX_SWEEPS * 4);
  f.bytes = off;
  return f;
}

hipError_t launch_factorize(const glowq_unit& u, const float* const* W_modules, const double* sigma_x,
                            int r, int p, int q, const double* Omega, char* ws, void* const* A_out,
                            void* B_out, double* sigma_out, hipStream_t st) {
  const FactorizePlan f = plan_factorize(u, r, p);
  const bool f16 = u.act_dtype == GLOWQ_F16;
  const int m = (int)f.m, d = f.d, l = f.l;
  double* Ms = (double*)(ws + f.off_ms);
  double* Y = (double*)(ws + f.off_y);
  double* Z = (double*)(ws + f.off_z);
  double* Bs = (double*)(ws + f.off_bs);
  double* Um = (double*)(ws + f.off_ut);
  double* gram = (double*)(ws + f.off_gram);
  double* lift = (double*)(ws + f.off_lift);
  double* A64 = (double*)(ws + f.off_a64);
  double* slices = (double*)(ws + f.off_slices);
  double* root = sigma_x ? (double*)(ws + f.off_root) : nullptr;
  double* inv_root = sigma_x ? (double*)(ws + f.off_inv_root) : nullptr;
  double* sig2 = (double*)(ws + f.off_sig2);
  double* sigma_sorted = (double*)(ws + f.off_sigma);
  int* perm = (int*)(ws + f.off_perm);
  int* counters = (int*)(ws + f.off_counters);
  CgsBuffers cb;
  cb.c1 = (double*)(ws + f.off_c1);
  cb.c2 = (double*)(ws + f.off_c2);
  cb.norm = (double*)(ws + f.off_norm);
  cb.norm0 = (double*)(ws + f.off_norm0);

  hipError_t err = launch_fill_zero(counters, FZ_MAX_SWEEPS * 4, st);
  if (err != hipSuccess) return err;
  if (sigma_x) k_roots<<<dim3((unsigned)((d + 255) / 256)), dim3(256), 0, st>>>(sigma_x, d, root, inv_root);
  // the stack, scaled by Sigma_x^(1/2) (Alg. 1, core construction)
  long long row_off = 0;
  for (int i = 0; i < u.n_modules; ++i) {
    const glowq_module& mod = u.modules[i];
    const long long recs = (long long)((mod.d_out + 15) / 16) * (d / 128);
    dim3 grid((unsigned)(recs < 4096 ? recs : 4096)), block(256);
    if (f16) k_error_stack<ACT_F16><<<grid, block, 0, st>>>(W_modules[i], mod.w_prepared, mod.d_out, d, u.group_size, root, Ms, row_off);
    else k_error_stack<ACT_BF16><<<grid, block, 0, st>>>(W_modules[i], mod.w_prepared, mod.d_out, d, u.group_size, root, Ms, row_off);
    row_off += mod.d_out;
  }
  // sketch and power steps (Alg. 1, range finding)
  err = gemm<false>(Ms, d, Omega, l, Y, f.l16, false, m, l, d, slices, st);
  for (int it = 0; it < q && err == hipSuccess; ++it) {
    err = gemm<true>(Ms, d, Y, f.l16, Z, f.l16, false, d, l, m, slices, st);
    if (err == hipSuccess) err = gemm<false>(Ms, d, Z, f.l16, Y, f.l16, false, m, l, d, slices, st);
  }
  if (err != hipSuccess) return err;
  // orthonormal basis of the range
  for (int j = 0; j <= l; ++j) {
    k_cgs<<<dim3((unsigned)f.n_groups), dim3(256), 0, st>>>(Y, f.l16, m, l, f.rpw, f.n_groups, j, 0, cb);
    if (j == l) break;
    if (j > 0) {
      k_cgs<<<dim3((unsigned)f.n_groups), dim3(256), 0, st>>>(Y, f.l16, m, l, f.rpw, f.n_groups, j, 1, cb);
      k_cgs<<<dim3((unsigned)f.n_groups), dim3(256), 0, st>>>(Y, f.l16, m, l, f.rpw, f.n_groups, j, 2, cb);
    } else {
      // the first column has nothing to be projected against: its norm is the one just taken
      k_cgs<<<dim3((unsigned)f.n_groups), dim3(256), 0, st>>>(Y, f.l16, m, l, f.rpw, f.n_groups, 0, 2, cb);
    }
  }
  // compressed matrix Bs = Q^T Ms and its SVD.  When the small Gram matrix fits one
  // workgroup's LDS its eigenvectors rotate the rows first, and the one-sided rotations on
  // the long rows only polish.
  int sweeps = FZ_MAX_SWEEPS;
  if (l <= FZ_EIG_MAX) {
    double* BsT = Z;                                                               // [d][l16]
    err = gemm<true>(Ms, d, Y, f.l16, BsT, f.l16, false, d, l, m, slices, st);     // Ms^T Q
    if (err == hipSuccess) err = gemm<true>(BsT, f.l16, BsT, f.l16, gram, f.l16, false, l, l, d, slices, st);
    if (err != hipSuccess) return err;
    k_gram_eigenvectors<<<dim3(1), dim3(1024), 0, st>>>(gram, f.l16, l, Um, f.l16);
    err = gemm<false>(BsT, f.l16, Um, f.l16, Bs, d, true, d, l, l, slices, st);    // (BsT Um)^T = Um^T Bs
    sweeps = FZ_POLISH_SWEEPS;
  } else {
    err = gemm<true>(Ms, d, Y, f.l16, Bs, d, true, d, l, m, slices, st);           // (Ms^T Q)^T
    k_identity<<<dim3((unsigned)((l * l + 255) / 256)), dim3(256), 0, st>>>(Um, f.l16, l);
  }
  if (err != hipSuccess) return err;
  const int n = (l + 1) & ~1;
  for (int sweep = 0; sweep < sweeps; ++sweep)
    for (int round = 0; round < n - 1; ++round)
      k_jacobi_round<<<dim3((unsigned)(n / 2)), dim3(FZ_JT), 0, st>>>(Bs, d, d, Um, f.l16, l, n, round, sweep, counters);
  k_row_norms<<<dim3((unsigned)l), dim3(256), 0, st>>>(Bs, d, d, sig2);
  k_sort_sigma<<<dim3(1), dim3(256), 0, st>>>(sig2, l, sigma_sorted, perm);
  // truncate, balance, lift
  k_build_lift<<<dim3((unsigned)((l * r + 255) / 256)), dim3(256), 0, st>>>(Um, f.l16, sigma_sorted, perm, l, r, lift, f.r16);
  err = gemm<false>(Y, f.l16, lift, f.r16, A64, f.r16, false, m, r, l, slices, st);
  if (err != hipSuccess) return err;
  row_off = 0;
  for (int i = 0; i < u.n_modules; ++i) {
    const glowq_module& mod = u.modules[i];
    const long long n_el = (long long)mod.d_out * r;
    dim3 grid((unsigned)((n_el + 255) / 256)), block(256);
    if (f16) k_store_A<ACT_F16><<<grid, block, 0, st>>>(A64, f.r16, row_off, mod.d_out, r, (uint16_t*)A_out[i]);
    else k_store_A<ACT_BF16><<<grid, block, 0, st>>>(A64, f.r16, row_off, mod.d_out, r, (uint16_t*)A_out[i]);
    row_off += mod.d_out;
  }
  {
    const long long n_el = (long long)r * d;
    dim3 grid((unsigned)((n_el + 255) / 256)), block(256);
    if (f16) k_store_B<ACT_F16><<<grid, block, 0, st>>>(Bs, d, sigma_sorted, perm, inv_root, r, d, (uint16_t*)B_out);
    else k_store_B<ACT_BF16><<<grid, block, 0, st>>>(Bs, d, sigma_sorted, perm, inv_root, r, d, (uint16_t*)B_out);
  }
  if (sigma_out) k_copy_doubles<<<dim3(1), dim3(256), 0, st>>>(sigma_sorted, sigma_out, l);
  return hipGetLastError();
}

}  // namespace glowq
