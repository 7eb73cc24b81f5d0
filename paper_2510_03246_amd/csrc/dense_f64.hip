// fp64 dense kernels for the ridge systems: blocked Cholesky, right-side triangular solves built from
// inverted 64x64 diagonal blocks plus rank-64 GEMM updates, and small cast / scatter helpers.
// The Gram systems can reach condition numbers ~1e4, so factor and solve stay in fp64 (the chip's
// vector fp64 rate equals its fp64 matrix rate, so these are plain FMA kernels staged through LDS).
#include "strp_internal.h"

namespace strp {

// ---------------------------------------------------------------------------------------------
// dgemm: 64x64 tile per 256-thread block, 4x4 micro-tile per thread, K staged 16 at a time
// ---------------------------------------------------------------------------------------------
constexpr int DT = 64, DK = 16;

__global__ __launch_bounds__(256) void dgemm_kernel(int M, int N, int K, double alpha, const double* A, long long rsa,
                                                    long long csa, const double* B, long long rsb, long long csb,
                                                    double beta, double* C, long long ldc, int lower) {
  const int m0 = blockIdx.y * DT, n0 = blockIdx.x * DT;
  if (lower && n0 > m0) return;
  __shared__ double As[DK][DT + 2];
  __shared__ double Bs[DK][DT + 2];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  double acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;

  for (int k0 = 0; k0 < K; k0 += DK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + 256 * i;
      int m, k;
      if (csa == 1) { m = e / DK; k = e % DK; } else { k = e / DT; m = e % DT; }
      double v = 0.0;
      if (m0 + m < M && k0 + k < K) v = A[(long long)(m0 + m) * rsa + (long long)(k0 + k) * csa];
      As[k][m] = v;
      int n, kb;
      if (csb == 1) { kb = e / DT; n = e % DT; } else { n = e / DK; kb = e % DK; }
      double w = 0.0;
      if (n0 + n < N && k0 + kb < K) w = B[(long long)(k0 + kb) * rsb + (long long)(n0 + n) * csb];
      Bs[kb][n] = w;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < DK; ++kk) {
      double a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fma(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      double* c = C + (long long)m * ldc + n;
      *c = (beta == 0.0) ? alpha * acc[i][j] : alpha * acc[i][j] + beta * (*c);
    }
  }
}

strp_status dgemm(strp_ctx* ctx, int M, int N, int K, double alpha, const double* A, long long rsa, long long csa,
                  const double* B, long long rsb, long long csb, double beta, double* C, long long ldc, int lower) {
  if (M <= 0 || N <= 0) return STRP_OK;
  dim3 grid((N + DT - 1) / DT, (M + DT - 1) / DT);
  hipLaunchKernelGGL(dgemm_kernel, grid, dim3(256), 0, ctx->stream, M, N, K, alpha, A, rsa, csa, B, rsb, csb, beta, C,
                     ldc, lower);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

// ---------------------------------------------------------------------------------------------
// Diagonal block: Cholesky of a jb x jb block (jb <= 64) in LDS and the inverse of its factor
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void potrf_diag_kernel(double* A, long long ld, int jb, double* invd, int32_t* status,
                                                         int block_row0) {
  __shared__ double S[NB][NB + 1];
  __shared__ double V[NB][NB + 1];
  __shared__ int bad;
  const int tid = threadIdx.x;
  if (tid == 0) bad = 0;
  for (int e = tid; e < NB * NB; e += 256) {
    const int i = e / NB, j = e % NB;
    S[i][j] = (i < jb && j <= i) ? A[(long long)i * ld + j] : 0.0;
    V[i][j] = 0.0;
  }
  __syncthreads();
  for (int j = 0; j < jb; ++j) {
    if (tid == 0) {
      const double dj = S[j][j];
      if (!(dj > 0.0)) {
        bad = 1;
        atomicCAS(status, 0, (int)STRP_ENOTPD);
        S[j][j] = 1.0;
      } else {
        S[j][j] = sqrt(dj);
      }
    }
    __syncthreads();
    const double piv = S[j][j];
    for (int i = j + 1 + tid; i < jb; i += 256) S[i][j] /= piv;
    __syncthreads();
    // trailing update of the lower triangle: S[i][k] -= S[i][j] * S[k][j], j < k <= i
    const int rem = jb - j - 1;
    for (int e = tid; e < rem * rem; e += 256) {
      const int i = j + 1 + e / rem, k = j + 1 + e % rem;
      if (k <= i) S[i][k] -= S[i][j] * S[k][j];
    }
    __syncthreads();
  }
  // inverse of the lower factor, one column per thread (forward substitution)
  if (tid < jb) {
    const int c = tid;
    for (int i = c; i < jb; ++i) {
      double acc = (i == c) ? 1.0 : 0.0;
      for (int k = c; k < i; ++k) acc -= S[i][k] * V[k][c];
      V[i][c] = acc / S[i][i];
    }
  }
  __syncthreads();
  for (int e = tid; e < NB * NB; e += 256) {
    const int i = e / NB, j = e % NB;
    invd[e] = V[i][j];
    if (i < jb && j < jb) A[(long long)i * ld + j] = (j <= i) ? S[i][j] : 0.0;
  }
  (void)block_row0;
}

// X[rows x jb] <- X * Mt, Mt[k][c] = trans ? Linv[c][k] : Linv[k][c]; one block per 64 rows
__global__ __launch_bounds__(256) void panel_mul_kernel(double* X, long long ldx, int rows, int jb, const double* invd,
                                                        int trans) {
  __shared__ double Xs[NB][NB + 1];
  __shared__ double Ms[NB][NB + 1];
  const int tid = threadIdx.x, r0 = blockIdx.x * NB;
  for (int e = tid; e < NB * NB; e += 256) {
    const int i = e / NB, j = e % NB;
    Xs[i][j] = (r0 + i < rows && j < jb) ? X[(long long)(r0 + i) * ldx + j] : 0.0;
    Ms[i][j] = trans ? invd[j * NB + i] : invd[e];
  }
  __syncthreads();
  const int tx = tid & 15, ty = tid >> 4;
  double acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;
  for (int k = 0; k < jb; ++k) {
    double a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = Xs[ty * 4 + i][k];
#pragma unroll
    for (int j = 0; j < 4; ++j) b[j] = Ms[k][tx * 4 + j];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fma(a[i], b[j], acc[i][j]);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = r0 + ty * 4 + i;
    if (r >= rows) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int c = tx * 4 + j;
      if (c < jb) X[(long long)r * ldx + c] = acc[i][j];
    }
  }
}

static strp_status panel_mul(strp_ctx* ctx, double* X, long long ldx, int rows, int jb, const double* invd, int trans) {
  if (rows <= 0) return STRP_OK;
  hipLaunchKernelGGL(panel_mul_kernel, dim3((rows + NB - 1) / NB), dim3(256), 0, ctx->stream, X, ldx, rows, jb, invd,
                     trans);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

strp_status chol_factor(strp_ctx* ctx, double* A, int n, long long ld, double* invd, int32_t* status) {
  ProfScope ps(ctx, "chol_factor_f64", (double)n * n * n / 3.0, 8.0 * (double)n * n);
  for (int j0 = 0; j0 < n; j0 += NB) {
    const int jb = (n - j0 < NB) ? (n - j0) : NB;
    double* Ajj = A + (long long)j0 * ld + j0;
    double* inv = invd + (long long)(j0 / NB) * NB * NB;
    hipLaunchKernelGGL(potrf_diag_kernel, dim3(1), dim3(256), 0, ctx->stream, Ajj, ld, jb, inv, status, j0);
    STRP_HIP(ctx, hipGetLastError());
    const int rest = n - j0 - jb;
    if (rest > 0) {
      double* A21 = A + (long long)(j0 + jb) * ld + j0;
      STRP_TRY(panel_mul(ctx, A21, ld, rest, jb, inv, 1));
      double* A22 = A + (long long)(j0 + jb) * ld + (j0 + jb);
      STRP_TRY(dgemm(ctx, rest, rest, jb, -1.0, A21, ld, 1, A21, 1, ld, 1.0, A22, ld, 1));
    }
  }
  return STRP_OK;
}

strp_status chol_solve_right(strp_ctx* ctx, const double* L, int n, long long ldl, const double* invd, double* X, int m,
                             long long ldx) {
  ProfScope ps(ctx, "chol_solve_f64", 2.0 * (double)m * n * n, 8.0 * ((double)n * n * 0.5 + 2.0 * (double)m * n));
  // V L^T = X  (column blocks ascending), then  X L = V  (descending); both in place.
  for (int j0 = 0; j0 < n; j0 += NB) {
    const int jb = (n - j0 < NB) ? (n - j0) : NB;
    const double* inv = invd + (long long)(j0 / NB) * NB * NB;
    STRP_TRY(panel_mul(ctx, X + j0, ldx, m, jb, inv, 1));
    const int j1 = j0 + jb, rest = n - j1;
    if (rest > 0)
      STRP_TRY(dgemm(ctx, m, rest, jb, -1.0, X + j0, ldx, 1, L + (long long)j1 * ldl + j0, 1, ldl, 1.0, X + j1, ldx, 0));
  }
  const int nblk = (n + NB - 1) / NB;
  for (int b = nblk - 1; b >= 0; --b) {
    const int j0 = b * NB;
    const int jb = (n - j0 < NB) ? (n - j0) : NB;
    const double* inv = invd + (long long)b * NB * NB;
    STRP_TRY(panel_mul(ctx, X + j0, ldx, m, jb, inv, 0));
    if (j0 > 0)
      STRP_TRY(dgemm(ctx, m, j0, jb, -1.0, X + j0, ldx, 1, L + (long long)j0 * ldl, ldl, 1, 1.0, X, ldx, 0));
  }
  return STRP_OK;
}

// ---------------------------------------------------------------------------------------------
// casts, scatter, fill
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void f32_to_f64_ridge_kernel(const float* Af, long long ldf, double* Ad, long long ld, int n,
                                                               double lam, const double* lam_dev) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= (long long)n * n) return;
  const int i = (int)(e / n), j = (int)(e % n);
  double v = (double)Af[(long long)i * ldf + j];
  if (i == j) v += lam_dev ? *lam_dev : lam;
  Ad[(long long)i * ld + j] = v;
}

strp_status f32_to_f64_ridge(strp_ctx* ctx, const float* Af, long long ldf, double* Ad, long long ld, int n, double lam,
                             const double* lam_dev) {
  const long long tot = (long long)n * n;
  hipLaunchKernelGGL(f32_to_f64_ridge_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, ctx->stream, Af, ldf,
                     Ad, ld, n, lam, lam_dev);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

__global__ __launch_bounds__(256) void cast_f64_f32_kernel(const double* src, long long lds, float* dst, long long ldd,
                                                           int rows, int cols) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= (long long)rows * ldd) return;
  const int i = (int)(e / ldd), j = (int)(e % ldd);
  dst[e] = j < cols ? (float)src[(long long)i * lds + j] : 0.0f;
}

strp_status cast_f64_f32(strp_ctx* ctx, const double* src, long long lds, float* dst, long long ldd, int rows, int cols) {
  const long long tot = (long long)rows * ldd;
  hipLaunchKernelGGL(cast_f64_f32_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, ctx->stream, src, lds, dst,
                     ldd, rows, cols);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t* p, long long words) {
  const long long stride = (long long)gridDim.x * 256;
  for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < words; e += stride) p[e] = 0u;
}

strp_status fill_zero(strp_ctx* ctx, void* ptr, size_t bytes) {
  if (bytes == 0) return STRP_OK;
  if (bytes % 4 != 0) return fail(ctx, STRP_EINVAL, "fill_zero: size not a multiple of 4");
  const long long words = (long long)(bytes / 4);
  long long blocks = (words + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, ctx->stream, (uint32_t*)ptr, words);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

// side FC2: sol [out x s] -> W[o][idx[c]];  side FC1: sol [s x in] -> W[idx[r]][c]
__global__ __launch_bounds__(256) void scatter_weights_kernel(const double* sol, long long lds, int side, const int32_t* idx,
                                                              int s, float* W, int out, int in) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (side == STRP_SIDE_FC2) {
    if (e >= (long long)out * s) return;
    const int o = (int)(e / s), c = (int)(e % s);
    W[(long long)o * in + idx[c]] = (float)sol[(long long)o * lds + c];
  } else {
    if (e >= (long long)s * in) return;
    const int r = (int)(e / in), c = (int)(e % in);
    W[(long long)idx[r] * in + c] = (float)sol[(long long)r * lds + c];
  }
}

strp_status scatter_weights(strp_ctx* ctx, const double* sol, long long lds, int side, const int32_t* idx, int s, float* W,
                            int out, int in) {
  STRP_TRY(fill_zero(ctx, W, sizeof(float) * (size_t)out * (size_t)in));
  const long long tot = side == STRP_SIDE_FC2 ? (long long)out * s : (long long)s * in;
  hipLaunchKernelGGL(scatter_weights_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, ctx->stream, sol, lds,
                     side, idx, s, W, out, in);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

}  // namespace strp
