// fp64 dense kernels for the ridge systems: blocked Cholesky, inversion of the triangular factor by
// recursive doubling, right-side solves as two triangular-aware GEMMs, and small cast / scatter helpers.
// The Gram systems reach condition numbers ~1e4, so factor and solve stay in fp64.  The GEMM runs on the
// fp64 matrix cores (v_mfma_f64_16x16x4_f64): same peak as the vector unit, far less LDS traffic per flop.
#include "cojob.h"
#include "strp_internal.h"

namespace strp {

typedef double doublex4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------------------------
// dgemm: C = alpha * A * B + beta * C, element strides for A(m,k) and B(k,n), C row-major.
//   block = 4 wavefronts (2x2), wavefront tile = WT x WT MFMA tiles of 16x16, K staged 16 at a time.
//   batch (grid.z): operand pointers advance by sa / sb / sc elements per batch entry and the batch
//   entry's M and K are clamped to lim_base - z * lim_step (ragged last block of a blocked algorithm).
//   tri restricts the K range of a tile to where a triangular operand is non-zero:
//     1: k < n0 + tile (B upper in (k, n)),  2: k >= n0 (B lower),  3: k >= m0 (A upper in (m, k)),
//     4: k < m0 + tile (A lower).
//   lower != 0 skips output tiles entirely above the diagonal.
// MFMA lane layout: A operand lane l = A[i = l % 16][k = l / 16], B operand lane l = B[k = l / 16][j = l % 16],
// result register r of lane l = D[i = 4 r + l / 16][j = l % 16].
// ---------------------------------------------------------------------------------------------
struct DgemmP {
  int M, N, K;
  double alpha, beta;
  const double* A; long long rsa, csa;
  const double* B; long long rsb, csb;
  double* C; long long ldc;
  int lower, tri;
  long long sa, sb, sc;
  int lim_base, lim_step;   // lim_step == 0: no clamping
  int clamp_k;              // clamp K like M (square ragged block)
  int own_x;                // blocks with blockIdx.x >= own_x are spare workgroups for the ride-along job (0: there are none)
};

template <int WT>
__global__ __launch_bounds__(256) void dgemm_kernel(const DgemmP p, const CoJob job) {
  constexpr int TS = 32 * WT;      // block tile (rows and columns)
  constexpr int DK = 16;
  constexpr int LD = TS + 4;
  // double-buffered operand tiles: one barrier per K tile
  __shared__ double As[2][DK][LD];
  __shared__ double Bs[2][DK][LD];
  if (p.own_x && (int)blockIdx.x >= p.own_x) {
    cojob_help(job);
    return;
  }
  const int z = blockIdx.z;
  int M = p.M, K = p.K;
  if (p.lim_step) {
    const int lim = p.lim_base - z * p.lim_step;
    M = M < lim ? M : lim;
    if (p.clamp_k) K = K < lim ? K : lim;
  }
  const int N = p.N;
  // blockIdx.x walks the rows of C; blockIdx.y walks column tiles in order of decreasing K range
  const int ntile = (p.tri == 1) ? (int)(gridDim.y - 1 - blockIdx.y) : (int)blockIdx.y;
  const int m0 = blockIdx.x * TS, n0 = ntile * TS;
  if (M <= 0 || m0 >= M) return;
  if (p.lower && n0 >= m0 + TS) return;
  const double* A = p.A + (long long)z * p.sa;
  const double* B = p.B + (long long)z * p.sb;
  double* C = p.C + (long long)z * p.sc;
  int kbeg = 0, kend = K;
  if (p.tri == 1) kend = (n0 + TS < K) ? n0 + TS : K;
  if (p.tri == 2) kbeg = n0;            // multiples of TS, hence of DK
  if (p.tri == 3) kbeg = m0;
  if (p.tri == 4) kend = (m0 + TS < K) ? m0 + TS : K;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  constexpr int EPT = TS * DK / 256;   // elements per thread per operand tile (8 or 4)
  doublex4 acc[WT][WT];
#pragma unroll
  for (int i = 0; i < WT; ++i)
#pragma unroll
    for (int j = 0; j < WT; ++j) acc[i][j] = doublex4{0.0, 0.0, 0.0, 0.0};

  double ra[EPT], rb[EPT];
  auto gload = [&](int k0) {
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
      const int e = tid + 256 * i;
      int m, k;
      if (p.csa == 1) { m = e / DK; k = e % DK; } else { k = e / TS; m = e % TS; }
      ra[i] = (m0 + m < M && k0 + k < kend) ? A[(long long)(m0 + m) * p.rsa + (long long)(k0 + k) * p.csa] : 0.0;
      int n, kb;
      if (p.csb == 1) { kb = e / TS; n = e % TS; } else { n = e / DK; kb = e % DK; }
      rb[i] = (n0 + n < N && k0 + kb < kend) ? B[(long long)(k0 + kb) * p.rsb + (long long)(n0 + n) * p.csb] : 0.0;
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
      const int e = tid + 256 * i;
      int m, k;
      if (p.csa == 1) { m = e / DK; k = e % DK; } else { k = e / TS; m = e % TS; }
      As[buf][k][m] = ra[i];
      int n, kb;
      if (p.csb == 1) { kb = e / TS; n = e % TS; } else { n = e / DK; kb = e % DK; }
      Bs[buf][kb][n] = rb[i];
    }
  };
  if (kbeg < kend) {
    gload(kbeg);
    sstore(0);
  }
  __syncthreads();
  int buf = 0;
  for (int k0 = kbeg; k0 < kend; k0 += DK) {
    const bool more = k0 + DK < kend;
    if (more) gload(k0 + DK);
#pragma unroll
    for (int ks = 0; ks < DK / 4; ++ks) {
      double af[WT], bf[WT];
      const int kk = ks * 4 + (lane >> 4);
#pragma unroll
      for (int i = 0; i < WT; ++i) af[i] = As[buf][kk][wm * 16 * WT + i * 16 + (lane & 15)];
#pragma unroll
      for (int j = 0; j < WT; ++j) bf[j] = Bs[buf][kk][wn * 16 * WT + j * 16 + (lane & 15)];
#pragma unroll
      for (int i = 0; i < WT; ++i)
#pragma unroll
        for (int j = 0; j < WT; ++j) acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    if (more) sstore(buf ^ 1);   // the other buffer: its readers finished before the previous barrier
    __syncthreads();
    buf ^= 1;
  }
#pragma unroll
  for (int i = 0; i < WT; ++i)
#pragma unroll
    for (int j = 0; j < WT; ++j) {
      const int n = n0 + wn * 16 * WT + j * 16 + (lane & 15);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int m = m0 + wm * 16 * WT + i * 16 + 4 * r + (lane >> 4);
        if (m < M && n < N) {
          double* c = C + (long long)m * p.ldc + n;
          const double v = p.alpha * acc[i][j][r];
          *c = (p.beta == 0.0) ? v : v + p.beta * (*c);
        }
      }
    }
}

// spare workgroups a short launch of the factorisation chain carries for the ride-along job: about as many units as
// HBM moves in the ~30 us such a launch takes (1024, 1536 and 2048 units per launch with 2, 3 and 4 per workgroup were
// timed on the benchmark's module: 1536 at 3 is the best by a little; the launches grow by about half of what they hide)
static int cojob_spare_blocks(const CoJob* cj, int own, int cap) {
  if (!cj || !cj->ticket || cj->take <= 0) return 0;
  int h = 1536 / cj->take;
  if (h > cap - own) h = cap - own;
  return h > 0 ? h : 0;
}

static strp_status dgemm_launch(strp_ctx* ctx, const DgemmP& pin, int batch, const CoJob* cj = nullptr) {
  DgemmP p = pin;
  if (p.M <= 0 || p.N <= 0 || batch <= 0) return STRP_OK;
  // 64 x 64 tiles throughout: a block is a serial chain of fp64 matrix-core instructions, the grids here are a few
  // thousand tiles at most, and with triangular K ranges small tiles balance far better (measured 20 % faster than
  // 128 x 128 tiles on the 4096 x 4915 solves)
  constexpr int ts = 64;
  dim3 grid((p.M + ts - 1) / ts, (p.N + ts - 1) / ts, batch);
  p.own_x = 0;
  CoJob job;
  memset(&job, 0, sizeof(job));
  const int own = (int)(grid.x * grid.y * grid.z);
  const int spare = cojob_spare_blocks(cj, own, 1024);   // four workgroups of this kernel fit a CU
  if (spare > 0) {
    job = *cj;
    p.own_x = (int)grid.x;
    grid.x += (unsigned)((spare + grid.y * grid.z - 1) / (grid.y * grid.z));
  }
  hipLaunchKernelGGL((dgemm_kernel<2>), grid, dim3(256), 0, ctx->stream, p, job);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

strp_status dgemm(strp_ctx* ctx, int M, int N, int K, double alpha, const double* A, long long rsa, long long csa,
                  const double* B, long long rsb, long long csb, double beta, double* C, long long ldc, int lower, int tri) {
  DgemmP p;
  memset(&p, 0, sizeof(p));
  p.M = M; p.N = N; p.K = K; p.alpha = alpha; p.beta = beta;
  p.A = A; p.rsa = rsa; p.csa = csa; p.B = B; p.rsb = rsb; p.csb = csb; p.C = C; p.ldc = ldc; p.lower = lower; p.tri = tri;
  return dgemm_launch(ctx, p, 1);
}

// ---------------------------------------------------------------------------------------------
// Diagonal block: Cholesky of a jb x jb block (jb <= 64) and the inverse of its factor
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ double rsqrt_f64(double d) {
  double y = __builtin_amdgcn_rsq(d);
  y = y * (1.5 - 0.5 * d * y * y);
  y = y * (1.5 - 0.5 * d * y * y);
  return y;
}

// Thread (ty, tx) of the 16x16 block keeps the 16 elements (ty + 16 ii, tx + 16 kk) of the working block AND of
// the inverse being built in registers for the whole factorisation.  Four columns are eliminated per barrier:
// the four columns of the block and rows j0..j0+3 of the inverse go through LDS (double buffered), every thread
// factors the 4 x 4 pivot block redundantly (A = Lu D Lu^T, Lu unit lower), eliminates the four panel entries of
// the eight row indices it needs (p_c(x) = P(x,c) - sum_{c'<c} p_c'(x) u_{c,c'}), and applies the rank-4 update
//   a_ik -= sum_c (p_c(i) / d_c) p_c(k)            (unpredicated: entries of finished columns are never re-read)
//   V_i. -= sum_c (p_c(i) / d_c) q_c(.)  for i > j0 + c,   q_c = row j0 + c of the inverse, eliminated likewise
// so that V ends as Lu^-1 and L^-1 = D^-1/2 Lu^-1.
struct PotrfShared {
  double colb[2][4][NB];
  double rowb[2][4][NB];
  double rsd[NB];          // d_j^-1/2
};

// On return (after its closing barrier): sh.rsd holds the inverse square roots of the pivots and v the unit-lower
// inverse (L^-1 = diag(rsd) v) at this thread's 16 positions.  The factor of the block itself is not formed: every
// consumer (panel multiplication, triangular inverse) works with the inverse.  report: this block raises ENOTPD.
__device__ __forceinline__ void potrf_block(const double* A, long long ld, int jb, PotrfShared& sh, double (&v)[4][4], int32_t* status,
                                            bool report) {
  auto& colb = sh.colb;
  auto& rowb = sh.rowb;
  auto& rsd = sh.rsd;
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  double a[4][4];
#pragma unroll
  for (int ii = 0; ii < 4; ++ii)
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int i = ty + 16 * ii, k = tx + 16 * kk;
      a[ii][kk] = (i < jb && k <= i) ? A[(long long)i * ld + k] : ((i == k) ? 1.0 : 0.0);
      v[ii][kk] = (i == k) ? 1.0 : 0.0;
    }
  // rounds j0 = 16 hi + lo16: the outer loop is unrolled so that the register rows and columns a round publishes
  // (index hi) are compile-time choices
#pragma unroll
  for (int hi = 0; hi < 4; ++hi)
#pragma unroll 1
  for (int lo16 = 0; lo16 < 16; lo16 += 4) {
    const int j0 = 16 * hi + lo16, buf = (j0 >> 2) & 1;
    if (tx >= lo16 && tx < lo16 + 4) {      // owners of columns j0 .. j0+3 publish them (rows ty + 16 ii)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        if (kk == hi) {
#pragma unroll
          for (int ii = 0; ii < 4; ++ii) colb[buf][tx - lo16][ty + 16 * ii] = a[ii][kk];
        }
    }
    if (ty >= lo16 && ty < lo16 + 4) {      // owners of rows j0 .. j0+3 of the inverse publish them
#pragma unroll
      for (int ii = 0; ii < 4; ++ii)
        if (ii == hi) {
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) rowb[buf][ty - lo16][tx + 16 * kk] = v[ii][kk];
        }
    }
    __syncthreads();
    // ---- 4 x 4 pivot block (every thread, redundantly) --------------------------------------------
    const double (*cb)[NB] = colb[buf];
    const double D00 = cb[0][j0], D10 = cb[0][j0 + 1], D20 = cb[0][j0 + 2], D30 = cb[0][j0 + 3];
    const double D11 = cb[1][j0 + 1], D21 = cb[1][j0 + 2], D31 = cb[1][j0 + 3];
    const double D22 = cb[2][j0 + 2], D32 = cb[2][j0 + 3], D33 = cb[3][j0 + 3];
    bool ok = true;
    double rs[4], id[4];
    ok = ok && D00 > 0.0;
    rs[0] = rsqrt_f64(D00 > 0.0 ? D00 : 1.0);
    id[0] = rs[0] * rs[0];
    const double u10 = D10 * id[0], u20 = D20 * id[0], u30 = D30 * id[0];
    const double E11 = D11 - D10 * u10, E21 = D21 - D20 * u10, E31 = D31 - D30 * u10;
    ok = ok && E11 > 0.0;
    rs[1] = rsqrt_f64(E11 > 0.0 ? E11 : 1.0);
    id[1] = rs[1] * rs[1];
    const double u21 = E21 * id[1], u31 = E31 * id[1];
    const double F22 = D22 - D20 * u20 - E21 * u21, F32 = D32 - D30 * u20 - E31 * u21;
    ok = ok && F22 > 0.0;
    rs[2] = rsqrt_f64(F22 > 0.0 ? F22 : 1.0);
    id[2] = rs[2] * rs[2];
    const double u32 = F32 * id[2];
    const double G33 = D33 - D30 * u30 - E31 * u31 - F32 * u32;
    ok = ok && G33 > 0.0;
    rs[3] = rsqrt_f64(G33 > 0.0 ? G33 : 1.0);
    id[3] = rs[3] * rs[3];
    if (tid == 0) {
#pragma unroll
      for (int c = 0; c < 4; ++c) rsd[j0 + c] = rs[c];
      if (report && !ok) {   // in a ragged block only the pivots inside jb count (the padding is the identity)
        const bool bad = j0 + 3 < jb || (0 < jb - j0 && !(D00 > 0.0)) || (1 < jb - j0 && !(E11 > 0.0)) || (2 < jb - j0 && !(F22 > 0.0));
        if (bad) atomicCAS(status, 0, (int)STRP_ENOTPD);
      }
    }
    // ---- eliminated panel entries of this thread's rows (pi) and columns (pk) --------------------------
    double pi[4][4], pk[4][4];   // [c][ii] and [c][kk]
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int xi = ty + 16 * q, xk = tx + 16 * q;
      pi[0][q] = cb[0][xi];
      pi[1][q] = cb[1][xi] - pi[0][q] * u10;
      pi[2][q] = cb[2][xi] - pi[0][q] * u20 - pi[1][q] * u21;
      pi[3][q] = cb[3][xi] - pi[0][q] * u30 - pi[1][q] * u31 - pi[2][q] * u32;
      pk[0][q] = cb[0][xk];
      pk[1][q] = cb[1][xk] - pk[0][q] * u10;
      pk[2][q] = cb[2][xk] - pk[0][q] * u20 - pk[1][q] * u21;
      pk[3][q] = cb[3][xk] - pk[0][q] * u30 - pk[1][q] * u31 - pk[2][q] * u32;
    }
    // rows j0 + c of the inverse, eliminated among themselves, at this thread's columns
    const double (*rb)[NB] = rowb[buf];
    double qk[4][4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int xk = tx + 16 * q;
      qk[0][q] = rb[0][xk];
      qk[1][q] = rb[1][xk] - u10 * qk[0][q];
      qk[2][q] = rb[2][xk] - u20 * qk[0][q] - u21 * qk[1][q];
      qk[3][q] = rb[3][xk] - u30 * qk[0][q] - u31 * qk[1][q] - u32 * qk[2][q];
    }
    // ---- rank-4 updates ------------------------------------------------------------------------
#pragma unroll
    for (int ii = 0; ii < 4; ++ii) {
      const int row = ty + 16 * ii;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const double m = pi[c][ii] * id[c];
        const double mv = row > j0 + c ? m : 0.0;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          a[ii][kk] = __builtin_fma(-m, pk[c][kk], a[ii][kk]);
          v[ii][kk] = __builtin_fma(-mv, qk[c][kk], v[ii][kk]);
        }
      }
    }
  }
  __syncthreads();
}

// One 64-column step of the factorisation in one launch.  Every block factors the (already updated) diagonal block
// itself -- the chip is idle during these steps, and a separate one-block launch would only add a kernel boundary to
// the critical path.  Block 0 stores the inverse of the block's factor; block b >= 1 multiplies rows [64 (b-1), +64)
// of the panel below the diagonal block by L^-T in place.  The diagonal block itself is only read (all blocks load
// it; nobody writes it), so blocks that start at different times cannot see each other's output.
// Blocks past `own` are spare workgroups for the ride-along job (cojob.h).
__global__ __launch_bounds__(256) void potrf_panel_kernel(double* Ajj, long long ld, int jb, int rest, double* invd, int32_t* status, int own,
                                                          const CoJob job) {
  __shared__ PotrfShared sh;
  __shared__ double Ms[NB][NB + 1];   // Ms[k][c] = Linv[c][k]
  __shared__ double Xs[NB][NB + 1];
  if ((int)blockIdx.x >= own) {
    cojob_help(job);
    return;
  }
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int b = blockIdx.x;
  double* X = Ajj + (long long)jb * ld;          // panel below the diagonal block
  const int r0 = (b - 1) * NB;
  // this block's panel rows, requested before the factorisation so that their latency hides behind it
  double xr[16];
  if (b > 0) {
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int e = tid + 256 * q, i = e >> 6, j = e & 63;
      xr[q] = (r0 + i < rest && j < jb) ? X[(long long)(r0 + i) * ld + j] : 0.0;
    }
  }
  double v[4][4];
  potrf_block(Ajj, ld, jb, sh, v, status, b == 0);
  if (b == 0) {
#pragma unroll
    for (int ii = 0; ii < 4; ++ii)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int i = ty + 16 * ii, k = tx + 16 * kk;
        const bool in = i < jb && k < jb;
        invd[i * NB + k] = (in && k <= i) ? v[ii][kk] * sh.rsd[i] : 0.0;
      }
    return;
  }
#pragma unroll
  for (int ii = 0; ii < 4; ++ii)
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int i = ty + 16 * ii, k = tx + 16 * kk;
      Ms[k][i] = (i < jb && k <= i) ? v[ii][kk] * sh.rsd[i] : 0.0;
    }
#pragma unroll
  for (int q = 0; q < 16; ++q) {
    const int e = tid + 256 * q;
    Xs[e >> 6][e & 63] = xr[q];
  }
  __syncthreads();
  double acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;
  for (int k = 0; k < jb; ++k) {
    double a[4], bb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = Xs[ty * 4 + i][k];
#pragma unroll
    for (int j = 0; j < 4; ++j) bb[j] = Ms[k][tx * 4 + j];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fma(a[i], bb[j], acc[i][j]);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = r0 + ty * 4 + i;
    if (r >= rest) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int c = tx * 4 + j;
      if (c < jb) X[(long long)r * ld + c] = acc[i][j];
    }
  }
}

// Two-level right-looking blocking: 64-column steps (diagonal block + panel) update only the rest of their
// 256-column outer panel; the trailing matrix is updated once per outer panel with K = 256, which quarters the
// read-modify-write traffic of the trailing matrix (a rank-64 update of a 4915 x 4915 matrix is memory bound).
strp_status chol_factor(strp_ctx* ctx, double* A, int n, long long ld, double* invd, int32_t* status) {
  ProfScope ps(ctx, "chol_factor_f64", (double)n * n * n / 3.0, 8.0 * (double)n * n);
  constexpr int NB2 = 4 * NB;
  const CoJob* cj = ctx->cojob;
  CoJob nojob;
  memset(&nojob, 0, sizeof(nojob));
  for (int J0 = 0; J0 < n; J0 += NB2) {
    const int Jend = (n - J0 < NB2) ? n : J0 + NB2;
    for (int j0 = J0; j0 < Jend; j0 += NB) {
      const int jb = (n - j0 < NB) ? (n - j0) : NB;
      double* Ajj = A + (long long)j0 * ld + j0;
      double* inv = invd + (long long)(j0 / NB) * NB * NB;
      const int rest = n - j0 - jb;
      const int own = 1 + (rest + NB - 1) / NB;
      const int spare = cojob_spare_blocks(cj, own, 512);   // two workgroups of this kernel fit a CU
      hipLaunchKernelGGL(potrf_panel_kernel, dim3(own + spare), dim3(256), 0, ctx->stream, Ajj, ld, jb, rest, inv, status, own, spare ? *cj : nojob);
      STRP_HIP(ctx, hipGetLastError());
      if (rest <= 0) continue;
      double* A21 = A + (long long)(j0 + jb) * ld + j0;
      const int pc = Jend - (j0 + jb);   // columns of the outer panel still to be factored
      if (pc > 0) {
        double* A22 = A + (long long)(j0 + jb) * ld + (j0 + jb);
        DgemmP u;
        memset(&u, 0, sizeof(u));
        u.M = rest; u.N = pc; u.K = jb; u.alpha = -1.0; u.beta = 1.0;
        u.A = A21; u.rsa = ld; u.csa = 1; u.B = A21; u.rsb = 1; u.csb = ld; u.C = A22; u.ldc = ld; u.lower = 1;
        STRP_TRY(dgemm_launch(ctx, u, 1, cj));
      }
    }
    const int rest2 = n - Jend;
    if (rest2 > 0) {
      const double* P = A + (long long)Jend * ld + J0;
      double* C = A + (long long)Jend * ld + Jend;
      STRP_TRY(dgemm(ctx, rest2, rest2, Jend - J0, -1.0, P, ld, 1, P, 1, ld, 1.0, C, ld, 1));
    }
  }
  return STRP_OK;
}

// Linv = L^-1 (lower triangular, n x n, leading dimension n) from the factor and its inverted 64-blocks.
// tmp: n x n fp64 scratch.  Doubling: for block size b = 64, 128, ...: V21 = -V22 (L21 V11) for every pair of
// adjacent diagonal blocks, all pairs of a level in one batched launch.
__global__ __launch_bounds__(256) void place_diag_blocks_kernel(const double* invd, int n, double* Linv) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= (long long)n * n) return;
  const int i = (int)(e / n), j = (int)(e % n);
  double v = 0.0;
  if ((i / NB) == (j / NB)) v = invd[(long long)(i / NB) * NB * NB + (i % NB) * NB + (j % NB)];
  Linv[e] = v;
}

strp_status tri_inverse(strp_ctx* ctx, const double* L, int n, long long ldl, const double* invd, double* Linv, double* tmp) {
  ProfScope ps(ctx, "tri_inverse_f64", (double)n * n * n / 3.0, 24.0 * (double)n * n);
  hipLaunchKernelGGL(place_diag_blocks_kernel, dim3((unsigned)(((long long)n * n + 255) / 256)), dim3(256), 0, ctx->stream, invd, n, Linv);
  STRP_HIP(ctx, hipGetLastError());
  for (int b = NB; b < n; b <<= 1) {
    const int pairs = (n - b + 2 * b - 1) / (2 * b);   // pairs whose second block is non-empty
    DgemmP p;
    memset(&p, 0, sizeof(p));
    // tmp21 = L21 V11
    p.M = b; p.N = b; p.K = b; p.alpha = 1.0; p.beta = 0.0;
    p.A = L + (long long)b * ldl; p.rsa = ldl; p.csa = 1;
    p.B = Linv; p.rsb = n; p.csb = 1;
    p.C = tmp + (long long)b * n; p.ldc = n;
    p.sa = 2LL * b * ldl + 2LL * b; p.sb = 2LL * b * n + 2LL * b; p.sc = p.sb;
    p.lim_base = n - b; p.lim_step = 2 * b; p.lower = 0;
    p.tri = 2;   // V11 is lower triangular
    STRP_TRY(dgemm_launch(ctx, p, pairs));
    // V21 = -V22 tmp21   (M and K both limited to the rows of the second block)
    p.alpha = -1.0;
    p.A = Linv + (long long)b * n + b; p.rsa = n; p.csa = 1; p.sa = p.sb;
    p.B = tmp + (long long)b * n; p.rsb = n; p.csb = 1;
    p.C = Linv + (long long)b * n; p.ldc = n;
    p.clamp_k = 1;
    p.tri = 4;   // V22 is lower triangular
    STRP_TRY(dgemm_launch(ctx, p, pairs));
  }
  return STRP_OK;
}

// X <- X (L L^T)^-1 = (X Linv^T) Linv for X [m x n] (leading dimension n); tmp: m x n scratch.
strp_status apply_inverse_right(strp_ctx* ctx, const double* Linv, int n, double* X, int m, double* tmp) {
  ProfScope ps(ctx, "chol_solve_f64", 2.0 * (double)m * n * n, 8.0 * ((double)n * n + 4.0 * (double)m * n));
  DgemmP p;
  memset(&p, 0, sizeof(p));
  p.M = m; p.N = n; p.K = n; p.alpha = 1.0; p.beta = 0.0;
  // tmp[m, j] = sum_{k <= j} X[m, k] Linv[j, k]
  p.A = X; p.rsa = n; p.csa = 1; p.B = Linv; p.rsb = 1; p.csb = n; p.C = tmp; p.ldc = n; p.tri = 1;
  STRP_TRY(dgemm_launch(ctx, p, 1));
  // X[m, j] = sum_{k >= j} tmp[m, k] Linv[k, j]
  p.A = tmp; p.B = Linv; p.rsb = n; p.csb = 1; p.C = X; p.tri = 2;
  return dgemm_launch(ctx, p, 1);
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
