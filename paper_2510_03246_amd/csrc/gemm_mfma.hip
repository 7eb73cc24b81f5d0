// MFMA GEMM family for gfx950 on 16-bit operand planes: v_mfma_f32_32x32x16_f16 matrix-core instructions,
// LDS-staged tiles, fp32 accumulation, 2x2 wavefronts per block.
//
// fp32 quantities (ADMM auxiliaries, refitted weights, targets) are kept for the matrix cores as TWO fp16
// planes, x*scale = hi + lo with hi = fp16(x*scale), lo = fp16(x*scale - hi) (fp16 subnormals are honoured by
// the f16 MFMA, so lo is exact to 2^-25 absolute).  A product of two split operands runs the three leading
// passes hi*hi + hi*lo + lo*hi into ONE fp32 accumulator (the dropped lo*lo term is ~2^-22 relative); a bf16
// input is exact in a single fp16 plane.  Planes are written once by the split kernels (split_planes.hip) or by
// a producing epilogue instead of being re-converted by every tile that reads them.
//
// Every operand uses one memory layout, chosen for the matrix cores and for HBM:
//   element (k, r)   k = contraction index, r = output row (P operand) or output column (Q operand)
//   offset(k, r) = (((r / 128) * KG + k / 8) * 128 + r % 128) * 8 + k % 8,   KG = ceil(K / 8)
// i.e. panels of 128 rows; inside a panel the 8 k-values a matrix-core lane needs are one 16-byte chunk, the 128
// chunks of a k-group are contiguous (a wavefront load is 1 KB contiguous, an LDS image needs no transpose and
// no padding), and walking k walks memory sequentially (one stream per panel, TLB- and DRAM-page-friendly).
// The kernel computes C[m, n] = sum_k P(k, m) Q(k, n); token-contraction products (Gram matrices, refit
// right-hand sides) use split-K partials, token-parallel products use the fused epilogues.
#include <stdlib.h>

#include "gemm_epilogue.h"

namespace strp {

// Tile shapes (WT = 32x32 MFMA tiles per wavefront per dimension):
//   WT = 2: 128x128 block (one panel per operand), K tile 64, two blocks per CU
//   WT = 4: 256x256 block (two panels per operand), K tile 32, one block per CU
template <int WT>
struct Tile {
  static constexpr int ROWS = 64 * WT;             // rows of P and columns of Q per block
  static constexpr int BK = WT == 2 ? 64 : 32;
  static constexpr int G = BK / 8;                 // k-groups per K tile
  static constexpr int PANS = ROWS / 128;
  static constexpr int NCH = ROWS * G / 256;       // 16-byte chunks per thread per plane per K tile (= 4)
  static constexpr int GSTEP = 256 / ROWS;         // k-groups covered by one pass of the block's threads (2 or 1)
};

// Operand tile loader: thread t owns row t % 128 of panel (t / 128) % PANS and k-groups g0 + GSTEP * i.
// Loads are unconditional (panel clamped to the last one, k-groups past the end read group 0 and are zeroed
// by select) and pointers advance by one K tile per iteration.
template <int NP, int WT>
struct PlaneLoader {
  static constexpr int NCH = Tile<WT>::NCH, BK = Tile<WT>::BK, ROWS = Tile<WT>::ROWS, GSTEP = Tile<WT>::GSTEP;
  const unsigned short* bp[NP];     // chunk (group of the next tile + g0, this thread's row)
  const unsigned short* safe[NP];   // same row, group 0
  uint4 r[NP][NCH];
  long long gnext;                  // absolute k-group of bp
  int lds_off;                      // element offset of chunk (g0, row) inside an LDS plane tile

  __device__ __forceinline__ void init(const PlaneOp& op, int row0, long long k0) {
    const int t = threadIdx.x;
    const int rr = t & 127;
    const int q = t >> 7;
    int pan = (row0 >> 7) + (Tile<WT>::PANS == 2 ? q : 0);
    pan = pan < op.npan ? pan : op.npan - 1;
    const int g0 = Tile<WT>::PANS == 2 ? 0 : q;
    gnext = (k0 >> 3) + g0;
    const long long base = ((long long)pan * op.kg * 128 + rr) * 8;
    bp[0] = op.hi + base + gnext * 1024;
    safe[0] = op.hi + base;
    if (NP == 2) {
      bp[NP - 1] = op.lo + base + gnext * 1024;
      safe[NP - 1] = op.lo + base;
    }
    lds_off = (g0 * ROWS + (Tile<WT>::PANS == 2 ? q * 128 : 0) + rr) * 8;
  }
  __device__ __forceinline__ void load(long long g_end) {
#pragma unroll
    for (int pl = 0; pl < NP; ++pl) {
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const bool valid = gnext + GSTEP * i < g_end;
        const unsigned short* src = valid ? bp[pl] + (long long)(GSTEP * i) * 1024 : safe[pl];
        const uint4 v = *(const uint4*)src;
        r[pl][i] = valid ? v : make_uint4(0, 0, 0, 0);
      }
      bp[pl] += (BK / 8) * 1024;
    }
    gnext += BK / 8;
  }
  __device__ __forceinline__ void store(unsigned short (*s)[ROWS * BK]) const {
#pragma unroll
    for (int pl = 0; pl < NP; ++pl)
#pragma unroll
      for (int i = 0; i < NCH; ++i) *(uint4*)(&s[pl][lds_off + GSTEP * i * ROWS * 8]) = r[pl][i];
  }
};

__device__ __forceinline__ floatx16 mma(uint4 a, uint4 b, floatx16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
}

template <int NPP, int NPQ, int WT>
__global__ __launch_bounds__(256, WT == 4 ? 1 : 2) void gemm_kernel(const GemmP p) {
  constexpr int ROWS = Tile<WT>::ROWS, BK = Tile<WT>::BK, KS = BK / 16;
  __shared__ __attribute__((aligned(16))) unsigned short sP[NPP][ROWS * BK];
  __shared__ __attribute__((aligned(16))) unsigned short sQ[NPQ][ROWS * BK];
  __shared__ double sred[4][2];
  __shared__ int srow[ROWS];   // gathered state row of each output row (AUPD / ZUPD)

  // ---- which tile, which K range ---------------------------------------------------------
  int tm, tn, split;
  if (!decode_tile(p, (int)blockIdx.x, (int)gridDim.x, tm, tn, split)) return;
  const int m0 = tm * ROWS, n0 = tn * ROWS;
  const long long k0 = (long long)split * p.kchunk;
  const long long k1 = (k0 + p.kchunk < p.K) ? (k0 + p.kchunk) : p.K;
  const long long g_end = (k1 + 7) >> 3;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid < ROWS) srow[tid] = (p.oidx && m0 + tid < p.M) ? p.oidx[m0 + tid] : 0;   // visible after the loop's barriers
  const int wm = wave >> 1, wn = wave & 1;
  constexpr int WROWS = 32 * WT;   // rows (and columns) of the output owned by one wavefront

  PlaneLoader<NPP, WT> lp;
  lp.init(p.P, m0, k0);
  PlaneLoader<NPQ, WT> lq;
  lq.init(p.Q, n0, k0);

  floatx16 acc[WT][WT];
#pragma unroll
  for (int i = 0; i < WT; ++i)
#pragma unroll
    for (int j = 0; j < WT; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  // fragment addresses of this lane inside an LDS tile [k-group][row][8]: lanes 0-31 take the even group of a
  // 16-deep step, lanes 32-63 the odd one; 32 consecutive rows are 512 contiguous bytes (no bank conflicts)
  const int offP = ((lane >> 5) * ROWS + wm * WROWS + (lane & 31)) * 8;
  const int offQ = ((lane >> 5) * ROWS + wn * WROWS + (lane & 31)) * 8;
  struct Frags { uint4 ph[WT], pl[WT], qh[WT], ql[WT]; };
  auto read_frags = [&](Frags& f, int ks) {
#pragma unroll
    for (int i = 0; i < WT; ++i) {
      const int off = offP + (2 * ks * ROWS + i * 32) * 8;
      f.ph[i] = *(const uint4*)(&sP[0][off]);
      if (NPP == 2) f.pl[i] = *(const uint4*)(&sP[NPP - 1][off]);
    }
#pragma unroll
    for (int j = 0; j < WT; ++j) {
      const int off = offQ + (2 * ks * ROWS + j * 32) * 8;
      f.qh[j] = *(const uint4*)(&sQ[0][off]);
      if (NPQ == 2) f.ql[j] = *(const uint4*)(&sQ[NPQ - 1][off]);
    }
  };
  auto run_mfma = [&](const Frags& f) {
    if (NPQ == 2) {
#pragma unroll
      for (int i = 0; i < WT; ++i)
#pragma unroll
        for (int j = 0; j < WT; ++j) acc[i][j] = mma(f.ph[i], f.ql[j], acc[i][j]);
    }
    if (NPP == 2) {
#pragma unroll
      for (int i = 0; i < WT; ++i)
#pragma unroll
        for (int j = 0; j < WT; ++j) acc[i][j] = mma(f.pl[i], f.qh[j], acc[i][j]);
    }
#pragma unroll
    for (int i = 0; i < WT; ++i)
#pragma unroll
      for (int j = 0; j < WT; ++j) acc[i][j] = mma(f.ph[i], f.qh[j], acc[i][j]);
  };

  if (k0 < k1) {
    lp.load(g_end);
    lq.load(g_end);
  }
  for (long long k = k0; k < k1; k += BK) {
    lp.store(sP);
    lq.store(sQ);
    __syncthreads();
    if (k + BK < k1) {  // next tile's global loads fly during the matrix work
      lp.load(g_end);
      lq.load(g_end);
    }
    // software pipeline over the 16-deep steps: fragments of step ks+1 are read while step ks multiplies
    Frags f[2];
    read_frags(f[0], 0);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      __builtin_amdgcn_sched_barrier(0);
      if (ks + 1 < KS) read_frags(f[(ks + 1) & 1], ks + 1);
      __builtin_amdgcn_sched_barrier(0);
      run_mfma(f[ks & 1]);
    }
    __syncthreads();
  }

  // ---- epilogue (one specialised, fully unrolled body per epilogue kind) -------------------------
  float unscale = 1.0f;
  if (p.P.scale) unscale /= *p.P.scale;
  if (p.Q.scale) unscale /= *p.Q.scale;
  double red0 = 0.0, red1 = 0.0;
  const int mbase = m0 + wm * WROWS + 4 * (lane >> 5), nbase = n0 + wn * WROWS + (lane & 31);
  switch (p.epi) {
    case EPI_PARTIAL: epilogue<EPI_PARTIAL, WT, WT>(p, acc, unscale, mbase, nbase, split, srow, m0, red0, red1); break;
    case EPI_STORE: epilogue<EPI_STORE, WT, WT>(p, acc, unscale, mbase, nbase, split, srow, m0, red0, red1); break;
    case EPI_INITZ: epilogue<EPI_INITZ, WT, WT>(p, acc, unscale, mbase, nbase, split, srow, m0, red0, red1); break;
    case EPI_RESID: epilogue<EPI_RESID, WT, WT>(p, acc, unscale, mbase, nbase, split, srow, m0, red0, red1); break;
    case EPI_AUPD: epilogue<EPI_AUPD, WT, WT>(p, acc, unscale, mbase, nbase, split, srow, m0, red0, red1); break;
    default: epilogue<EPI_ZUPD, WT, WT>(p, acc, unscale, mbase, nbase, split, srow, m0, red0, red1); break;
  }
  if (p.red) {
    red0 = wave_sum(red0);
    red1 = wave_sum(red1);
    if (lane == 0) {
      sred[wave][0] = red0;
      sred[wave][1] = red1;
    }
    __syncthreads();
    if (tid == 0) {
      p.red[2 * (long long)blockIdx.x + 0] = sred[0][0] + sred[1][0] + sred[2][0] + sred[3][0];
      p.red[2 * (long long)blockIdx.x + 1] = sred[0][1] + sred[1][1] + sred[2][1] + sred[3][1];
    }
  }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
void gemm_plan_tiles(GemmP& p, int want_splits) {
  {
    // 256x256 tiles with the LDS-DMA pipeline when they still give most CUs a block
    const long long t4m = (p.M + 255) / 256, t4n = (p.N + 255) / 256;
    const long long n4 = p.triangle ? t4m * (t4m + 1) / 2 : t4m * t4n;
    const bool big = p.M >= 256 && p.N >= 256 && n4 * (want_splits > 1 ? want_splits : 1) >= 192 && p.K >= 256;
    p.wt = (big && p.force_wt != 2) ? 4 : 2;
  }
  const int ROWS = 64 * p.wt, BK = p.wt == 2 ? 64 : 32;
  p.tilesM = (p.M + ROWS - 1) / ROWS;
  p.tilesN = (p.N + ROWS - 1) / ROWS;
  p.ntiles = p.triangle ? p.tilesM * (p.tilesM + 1) / 2 : p.tilesM * p.tilesN;
  if (p.triangle) {
    p.gridM = (p.tilesM + 1) / 2;
    p.gridN = 2 * p.gridM + 1;
  } else {
    p.gridM = p.tilesM;
    p.gridN = p.tilesN;
  }
  {
    // tile group: 32 tiles, shaped to the grid
    int gm = 4;
    while (gm > 1 && gm > p.gridM) gm >>= 1;
    int gn = 32 / gm;
    while (gn > 1 && gn / 2 >= p.gridN) { gn >>= 1; if (gm * 2 <= p.gridM) gm <<= 1; }
    p.gm = gm;
    p.gn = gn;
  }
  if (want_splits <= 1) {
    p.splits = 1;
    p.kchunk = ((p.K + BK - 1) / BK) * BK;
  } else {
    long long chunk = (p.K + want_splits - 1) / want_splits;
    chunk = ((chunk + BK - 1) / BK) * BK;
    p.kchunk = chunk;
    p.splits = (int)((p.K + chunk - 1) / chunk);
  }
}

int gemm_grid_blocks(const GemmP& p) { return p.gridM * p.gridN * p.splits; }

// zero the pad k-groups [g_first, kg) of a plane written by an epilogue (whose rows fill the groups below g_first)
__global__ __launch_bounds__(256) void zero_pad_group_kernel(unsigned short* hi, unsigned short* lo, long long kg, int g_first, int npan) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;   // 16-byte chunk index over npan x 128
  if (e >= (long long)npan * 128) return;
  for (long long g = g_first; g < kg; ++g) {
    const long long o = (((e >> 7) * kg + g) * 128 + (e & 127)) * 8;
    *(uint4*)(hi + o) = make_uint4(0, 0, 0, 0);
    if (lo) *(uint4*)(lo + o) = make_uint4(0, 0, 0, 0);
  }
}

void launch_gemm_dma(strp_ctx* ctx, const GemmP& p, int npp, int npq);   // gemm_dma.hip

template <int NPP, int NPQ>
static void launch_one(strp_ctx* ctx, const GemmP& p) {
  if (p.wt == 4)
    launch_gemm_dma(ctx, p, NPP, NPQ);
  else
    hipLaunchKernelGGL((gemm_kernel<NPP, NPQ, 2>), dim3(gemm_grid_blocks(p)), dim3(256), 0, ctx->stream, p);
}

strp_status launch_gemm(strp_ctx* ctx, GemmP& p) {
  if (p.M <= 0 || p.N <= 0 || p.K <= 0) return fail(ctx, STRP_EINVAL, "gemm: empty shape");
  if (p.ntiles <= 0 || p.splits <= 0 || (p.wt != 2 && p.wt != 4)) return fail(ctx, STRP_EINVAL, "gemm: tiles not planned");
  if (!p.P.hi || !p.Q.hi) return fail(ctx, STRP_EINVAL, "gemm: null operand plane");
  if (p.P.kg * 8 < p.K || p.Q.kg * 8 < p.K || (p.P.kg & 3) || (p.Q.kg & 3))
    return fail(ctx, STRP_EINVAL, "gemm: operand planes shorter than K or a group count that is not a multiple of four");
  if ((long long)p.P.npan * 128 < p.M || (long long)p.Q.npan * 128 < p.N) return fail(ctx, STRP_EINVAL, "gemm: operand planes narrower than the output");
  if (p.epi != EPI_PARTIAL && p.splits != 1) return fail(ctx, STRP_EINVAL, "gemm: fused epilogues do not split K");
  const int npp = p.P.lo ? 2 : 1, npq = p.Q.lo ? 2 : 1;
  static const char* const epi_names[] = {"partial", "store", "initz", "resid", "aupd", "zupd"};
  static char names[3][3][6][40];
  char* name = names[npp][npq][p.epi];
  if (!name[0]) snprintf(name, 40, "gemm_h%dx%d_%s", npp, npq, epi_names[p.epi]);
  const double mn = p.triangle ? 0.5 * (double)p.M * ((double)p.M + 1.0) : (double)p.M * (double)p.N;
  static const double out_words[] = {1.0, 1.0, 3.0, 2.0, 2.0, 2.0};
  double obytes = 4.0 * out_words[p.epi] * (double)p.M * (double)p.N * (p.epi == EPI_PARTIAL ? (double)p.splits : 1.0);
  if (p.epi == EPI_RESID) obytes *= 0.5;
  if (p.k8_hi) obytes += (p.k8_lo ? 4.0 : 2.0) * (double)p.M * (double)p.N;
  const double ibytes = p.triangle ? 2.0 * npp * (double)p.M * (double)p.K
                                   : 2.0 * npp * (double)p.M * (double)p.K + 2.0 * npq * (double)p.N * (double)p.K;
  ProfScope ps(ctx, name, 2.0 * mn * (double)p.K, ibytes + obytes);
  if (p.k8_hi && (p.M + 7) / 8 < p.k8_kg) {
    const int npan = (p.N + 127) / 128;
    hipLaunchKernelGGL(zero_pad_group_kernel, dim3((npan * 128 + 255) / 256), dim3(256), 0, ctx->stream, p.k8_hi, p.k8_lo, p.k8_kg,
                       (p.M + 7) / 8, npan);
  }
  switch (npp * 10 + npq) {
    case 11: launch_one<1, 1>(ctx, p); break;
    case 12: launch_one<1, 2>(ctx, p); break;
    case 21: launch_one<2, 1>(ctx, p); break;
    default: launch_one<2, 2>(ctx, p); break;
  }
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

// ---- split-K reduction -----------------------------------------------------------------------
// One block reduces a 64 x 64 output tile (thread = column tx, rows ty + 4 i): a wavefront load is 256 contiguous bytes
// of one row of one partial.  Symmetric products: only tiles on or below the diagonal are reduced; the strict lower
// part is also written transposed through LDS, so the upper half is a bit-exact mirror and the partials are read once,
// row-contiguously.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* part, int splits, int M, int N, int triangle,
                                                           float* outf, long long ldof, double* outd, long long ldod,
                                                           double* diag, int accumulate) {
  constexpr int TS = 64;
  __shared__ double tile[TS][TS + 1];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int n0 = blockIdx.x * TS, m0 = blockIdx.y * TS;
  if (triangle && n0 > m0) return;
  const long long MN = (long long)M * N;
  auto put = [&](int m, int n, double s) {
    if (outf) {
      float* o = outf + (long long)m * ldof + n;
      *o = accumulate ? (float)((double)*o + s) : (float)s;
    }
    if (outd) outd[(long long)m * ldod + n] = s;
    if (diag && m == n) diag[m] = s;
  };
  const int n = n0 + tx;
  double acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.0;
  {
    // rows and the column are clamped into range (results of clamped lanes are not stored): the 16 loads of a split
    // are then unconditional and all in flight together
    const int nc = n < N ? n : N - 1;
    long long ro[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int m = m0 + ty + 4 * i;
      ro[i] = (long long)(m < M ? m : M - 1) * N + nc;
    }
    for (int sp = 0; sp < splits; ++sp) {
      const float* src = part + (long long)sp * MN;
      float v[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] = src[ro[i]];
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] += (double)v[i];
    }
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int m = m0 + ty + 4 * i;
    if (m < M && n < N && (!triangle || n <= m)) put(m, n, acc[i]);
    tile[ty + 4 * i][tx] = acc[i];
  }
  if (!triangle) return;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int lo_m = m0 + tx, lo_n = n0 + ty + 4 * i;     // element (lo_m, lo_n) of the lower half, mirrored to (lo_n, lo_m)
    if (lo_n < lo_m && lo_m < M && lo_n < N) put(lo_n, lo_m, tile[tx][ty + 4 * i]);
  }
}

strp_status launch_splitk_reduce(strp_ctx* ctx, const float* part, int splits, int M, int N, int triangle,
                                 float* outf, long long ldof, double* outd, long long ldod, double* diag,
                                 int accumulate) {
  const long long tot = (long long)M * N;
  if (triangle && M != N) return fail(ctx, STRP_EINVAL, "split-K reduce: a symmetric product must be square");
  ProfScope ps(ctx, "splitk_reduce", 0.0, 4.0 * (double)tot * (double)splits * (triangle ? 0.5 : 1.0) + (outf ? 4.0 : 0.0) * tot + (outd ? 8.0 : 0.0) * tot);
  hipLaunchKernelGGL(splitk_reduce_kernel, dim3((N + 63) / 64, (M + 63) / 64), dim3(256), 0, ctx->stream, part,
                     splits, M, N, triangle, outf, ldof, outd, ldod, diag, accumulate);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

__global__ __launch_bounds__(256) void block_sum_kernel(const double* red, int nblocks, double* dst0, double* dst1,
                                                       double scale0, double scale1) {
  __shared__ double s[256][2];
  double a = 0.0, b = 0.0;
  for (int i = threadIdx.x; i < nblocks; i += 256) {
    a += red[2 * (long long)i];
    b += red[2 * (long long)i + 1];
  }
  s[threadIdx.x][0] = a;
  s[threadIdx.x][1] = b;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) {
      s[threadIdx.x][0] += s[threadIdx.x + o][0];
      s[threadIdx.x][1] += s[threadIdx.x + o][1];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    if (dst0) *dst0 = s[0][0] * scale0;
    if (dst1) *dst1 = s[0][1] * scale1;
  }
}

strp_status launch_block_sum(strp_ctx* ctx, const double* red, int nblocks, double* dst0, double* dst1,
                             double scale0, double scale1) {
  hipLaunchKernelGGL(block_sum_kernel, dim3(1), dim3(256), 0, ctx->stream, red, nblocks, dst0, dst1, scale0, scale1);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

}  // namespace strp
