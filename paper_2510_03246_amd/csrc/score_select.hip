// HBM-bound scoring reductions, the softmax sparsity allocation and the top-k structured select.
//   row_sums      : per-channel token sums (fp64 accumulation, one block per channel, float4 loads)
//   colnorm2      : squared column norms of the next linear layer
//   unit_scores   : WANDA / LEMMA / GAIN unit scores (+ group sums for heads) and the layer energy
//   alloc         : softmax allocation with clipping, rescale and largest-remainder prune counts
//   topk          : radix select on order-preserving keys, ballot/prefix compaction, ties -> lower index
#include "strp_internal.h"

namespace strp {

__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  return v;
}
__device__ __forceinline__ double wave_allsum_d(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ double wave_allmax_d(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float bf16lo(unsigned int w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16hi(unsigned int w) { return __builtin_bit_cast(float, w & 0xffff0000u); }

// ---------------------------------------------------------------------------------------------
// per-channel token sums: sums[0][r] = sum A^2, [1][r] = sum A*relu(Z0), [2][r] = sum Z0*Z, [3][r] = sum Z0^2
// ---------------------------------------------------------------------------------------------
template <bool A_BF16, bool FULL>
__global__ __launch_bounds__(256) void row_sums_kernel(const void* Av, const float* Z, const float* Z0, long long ld,
                                                       long long T, int rows, double* sums, int32_t* status) {
  const int r = blockIdx.x;
  const int tid = threadIdx.x;
  double g = 0.0, e = 0.0, u = 0.0, v = 0.0;
  const long long T8 = T & ~7LL;
  if (A_BF16 && !FULL) {
    const uint4* a8 = (const uint4*)((const unsigned short*)Av + (long long)r * ld);
    for (long long c = tid; c < T8 / 8; c += 256) {
      const uint4 w = a8[c];
      const unsigned int ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const double lo = (double)bf16lo(ww[q]), hi = (double)bf16hi(ww[q]);
        g = __builtin_fma(lo, lo, g);
        g = __builtin_fma(hi, hi, g);
      }
    }
    const unsigned short* as = (const unsigned short*)Av + (long long)r * ld;
    for (long long t = T8 + tid; t < T; t += 256) {
      const double x = (double)__builtin_bit_cast(float, (unsigned int)as[t] << 16);
      g = __builtin_fma(x, x, g);
    }
  } else {
    const float* a = (const float*)Av + (long long)r * ld;
    const float* z = FULL ? Z + (long long)r * ld : nullptr;
    const float* z0 = FULL ? Z0 + (long long)r * ld : nullptr;
    const float4* a4 = (const float4*)a;
    const float4* z4 = (const float4*)z;
    const float4* z04 = (const float4*)z0;
    const long long T4 = T & ~3LL;
    for (long long c = tid; c < T4 / 4; c += 256) {
      const float4 x = a4[c];
      const float xa[4] = {x.x, x.y, x.z, x.w};
      if (FULL) {
        const float4 y = z4[c], w = z04[c];
        const float ya[4] = {y.x, y.y, y.z, y.w}, wa[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const double xd = xa[q], zd = ya[q], z0d = wa[q];
          g = __builtin_fma(xd, xd, g);
          e = __builtin_fma(xd, fmax(z0d, 0.0), e);
          u = __builtin_fma(z0d, zd, u);
          v = __builtin_fma(z0d, z0d, v);
        }
      } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const double xd = xa[q];
          g = __builtin_fma(xd, xd, g);
        }
      }
    }
    for (long long t = T4 + tid; t < T; t += 256) {
      const double xd = a[t];
      g = __builtin_fma(xd, xd, g);
      if (FULL) {
        const double zd = z[t], z0d = z0[t];
        e = __builtin_fma(xd, fmax(z0d, 0.0), e);
        u = __builtin_fma(z0d, zd, u);
        v = __builtin_fma(z0d, z0d, v);
      }
    }
  }
  __shared__ double sh[4][4];
  g = wave_sum_d(g);
  if (FULL) {
    e = wave_sum_d(e);
    u = wave_sum_d(u);
    v = wave_sum_d(v);
  }
  const int lane = tid & 63, wave = tid >> 6;
  if (lane == 0) {
    sh[wave][0] = g;
    sh[wave][1] = e;
    sh[wave][2] = u;
    sh[wave][3] = v;
  }
  __syncthreads();
  if (tid < 4) {
    const double s = sh[0][tid] + sh[1][tid] + sh[2][tid] + sh[3][tid];
    if (tid == 0 || FULL) sums[(long long)tid * rows + r] = s;
    if (!(fabs(s) <= 1.79e308)) atomicCAS(status, 0, (int)STRP_ENONFINITE);
  }
}

strp_status launch_row_sums(strp_ctx* ctx, const void* A, int a_dtype, const float* Z, const float* Z0, long long ld,
                            long long T, int rows, int mode, double* sums) {
  const bool full = mode != STRP_SCORE_WANDA;
  if (full && a_dtype != STRP_F32) return fail(ctx, STRP_EINVAL, "score: LEMMA/GAIN need fp32 auxiliaries");
  dim3 grid(rows), block(256);
  const double es = a_dtype == STRP_BF16 ? 2.0 : 4.0;
  ProfScope ps(ctx, full ? "row_sums_full" : "row_sums_wanda", (full ? 8.0 : 2.0) * (double)rows * (double)T,
               (full ? 12.0 : es) * (double)rows * (double)T);
  if (full)
    hipLaunchKernelGGL((row_sums_kernel<false, true>), grid, block, 0, ctx->stream, A, Z, Z0, ld, T, rows, sums, ctx->status_dev);
  else if (a_dtype == STRP_BF16)
    hipLaunchKernelGGL((row_sums_kernel<true, false>), grid, block, 0, ctx->stream, A, Z, Z0, ld, T, rows, sums, ctx->status_dev);
  else
    hipLaunchKernelGGL((row_sums_kernel<false, false>), grid, block, 0, ctx->stream, A, Z, Z0, ld, T, rows, sums, ctx->status_dev);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

// Scoring sums of the kept rows from the strips the a- and z-update epilogues wrote: part[q][strip][m] (fp32, one value
// per output row m and 64-column strip) -> rowsums[qdst[q] * f + idx[m]] (fp64).  Two fixed-order levels: 16 chunks of
// strips per row, then the 16 chunk sums.
constexpr int RS_CHUNKS = 16;
__global__ __launch_bounds__(256) void rowsum_chunk_kernel(const float* part, int slots, int M, double* chunk_sums) {
  const int m = blockIdx.x * 256 + threadIdx.x;
  const int c = blockIdx.y, q = blockIdx.z;
  if (m >= M) return;
  const int per = (slots + RS_CHUNKS - 1) / RS_CHUNKS;
  const int s0 = c * per, s1 = (s0 + per < slots) ? s0 + per : slots;
  const float* src = part + (long long)q * slots * M + m;
  double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;   // four independent chains keep four loads in flight
  int sidx = s0;
  for (; sidx + 3 < s1; sidx += 4) {
    a0 += (double)src[(long long)sidx * M];
    a1 += (double)src[(long long)(sidx + 1) * M];
    a2 += (double)src[(long long)(sidx + 2) * M];
    a3 += (double)src[(long long)(sidx + 3) * M];
  }
  for (; sidx < s1; ++sidx) a0 += (double)src[(long long)sidx * M];
  chunk_sums[((long long)q * RS_CHUNKS + c) * M + m] = (a0 + a1) + (a2 + a3);
}
__global__ __launch_bounds__(256) void rowsum_final_kernel(const double* chunk_sums, int M, const int32_t* idx, double* rowsums, int f,
                                                           int qdst0, int qdst1, int32_t* status) {
  const int m = blockIdx.x * 256 + threadIdx.x;
  const int q = blockIdx.y;
  if (m >= M) return;
  double t = 0.0;
#pragma unroll
  for (int c = 0; c < RS_CHUNKS; ++c) t += chunk_sums[((long long)q * RS_CHUNKS + c) * M + m];
  rowsums[(long long)(q == 0 ? qdst0 : qdst1) * f + idx[m]] = t;
  if (!(fabs(t) <= 1.79e308)) atomicCAS(status, 0, (int)STRP_ENONFINITE);
}

size_t rowsum_scratch_bytes(int nq, int M) { return sizeof(double) * (size_t)nq * RS_CHUNKS * (size_t)M; }

strp_status launch_rowsum_reduce(strp_ctx* ctx, const float* part, int nq, int slots, int M, const int32_t* idx, double* rowsums, int f,
                                 int qdst0, int qdst1, double* chunk_sums) {
  if (nq <= 0 || M <= 0 || slots <= 0) return STRP_OK;
  ProfScope ps(ctx, "rowsum_reduce", 0.0, 4.0 * (double)nq * (double)slots * (double)M);
  hipLaunchKernelGGL(rowsum_chunk_kernel, dim3((M + 255) / 256, RS_CHUNKS, nq), dim3(256), 0, ctx->stream, part, slots, M, chunk_sums);
  hipLaunchKernelGGL(rowsum_final_kernel, dim3((M + 255) / 256, nq), dim3(256), 0, ctx->stream, (const double*)chunk_sums, M, idx, rowsums, f,
                     qdst0, qdst1, ctx->status_dev);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

// ---------------------------------------------------------------------------------------------
// squared column norms: block = 64 columns x 4 row lanes
// ---------------------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(256) void colnorm2_kernel(const void* Wv, int rows, int cols, long long ldw, double* n2) {
  const int c = blockIdx.x * 64 + (threadIdx.x & 63);
  const int rl = threadIdx.x >> 6;
  double acc = 0.0;
  if (c < cols) {
    for (int r = rl; r < rows; r += 4) {
      double x;
      if (BF16) {
        x = (double)__builtin_bit_cast(float, (unsigned int)((const unsigned short*)Wv)[(long long)r * ldw + c] << 16);
      } else {
        x = (double)((const float*)Wv)[(long long)r * ldw + c];
      }
      acc = __builtin_fma(x, x, acc);
    }
  }
  __shared__ double sh[4][64];
  sh[rl][threadIdx.x & 63] = acc;
  __syncthreads();
  if (rl == 0 && c < cols) n2[c] = sh[0][threadIdx.x] + sh[1][threadIdx.x] + sh[2][threadIdx.x] + sh[3][threadIdx.x];
}

strp_status launch_colnorm2(strp_ctx* ctx, const void* W, int w_dtype, int rows, int cols, long long ldw, double* n2) {
  dim3 grid((cols + 63) / 64), block(256);
  if (w_dtype == STRP_BF16)
    hipLaunchKernelGGL((colnorm2_kernel<true>), grid, block, 0, ctx->stream, W, rows, cols, ldw, n2);
  else
    hipLaunchKernelGGL((colnorm2_kernel<false>), grid, block, 0, ctx->stream, W, rows, cols, ldw, n2);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

// ---------------------------------------------------------------------------------------------
// unit scores + layer energy (single block, fixed summation order)
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void unit_scores_kernel(const double* sums, const double* n2, int n_channels, int group,
                                                          int mode, float* score, double* energy_out) {
  const int n = n_channels / group;
  const double* g = sums;
  const double* e = sums + (long long)n_channels;
  const double* u = sums + 2LL * n_channels;
  const double* v = sums + 3LL * n_channels;
  double esum = 0.0;
  for (int unit = threadIdx.x; unit < n; unit += 1024) {
    double sp = 0.0, sq = 0.0, sw = 0.0;
    for (int c = 0; c < group; ++c) {
      const int j = unit * group + c;
      const double w = n2[j] * g[j];
      sw += w;
      if (mode != STRP_SCORE_WANDA) {
        sp += u[j] + n2[j] * e[j];
        sq += v[j] + w;
      }
    }
    double sc;
    if (mode == STRP_SCORE_WANDA) sc = sw;
    else if (mode == STRP_SCORE_LEMMA) sc = sp / sq;
    else sc = 2.0 * sp - sq;
    score[unit] = (float)sc;
    esum += sc;
  }
  __shared__ double sh[16];
  esum = wave_sum_d(esum);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = esum;
  __syncthreads();
  if (threadIdx.x == 0 && energy_out) {
    double tot = 0.0;
    for (int w = 0; w < 16; ++w) tot += sh[w];
    *energy_out = tot / (double)n;
  }
}

strp_status launch_unit_scores(strp_ctx* ctx, const double* sums, const double* n2, int n_channels, int group, int mode,
                               float* score, double* energy_out) {
  hipLaunchKernelGGL(unit_scores_kernel, dim3(1), dim3(1024), 0, ctx->stream, sums, n2, n_channels, group, mode, score,
                     energy_out);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

// ---------------------------------------------------------------------------------------------
// softmax allocation: one wavefront, fp64, layers strided over lanes
// ---------------------------------------------------------------------------------------------
// ---------------------------------------------------------------------------------------------
// weight statistics of a parameter group (Alg. 2 step 1): sum |w|, sum w, sum w^2 over every entry of a list of
// matrices.  Block b keeps its own partial [3] (launches on one stream add to it in order: deterministic);
// weight_energy_kernel folds the partials into  scale (|W|_1 + cv Var(W) + c2 |W|_2)  and adds it to the energy.
// ---------------------------------------------------------------------------------------------
constexpr int WSTAT_BLOCKS = 256;

template <bool BF16>
__global__ __launch_bounds__(256) void weight_stats_kernel(const void* W, int rows, int cols, long long ld, double* partial) {
  double s1 = 0.0, s = 0.0, s2 = 0.0;
  const long long n = (long long)rows * cols;
  for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long long)WSTAT_BLOCKS * 256) {
    const long long r = e / cols, c = e - r * cols;
    float x;
    if (BF16) x = __builtin_bit_cast(float, (unsigned int)((const unsigned short*)W)[r * ld + c] << 16);
    else x = ((const float*)W)[r * ld + c];
    const double v = (double)x;
    s1 += fabs(v);
    s += v;
    s2 += v * v;
  }
  __shared__ double red[4][3];
  s1 = wave_allsum_d(s1);
  s = wave_allsum_d(s);
  s2 = wave_allsum_d(s2);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) { red[wave][0] = s1; red[wave][1] = s; red[wave][2] = s2; }
  __syncthreads();
  if (threadIdx.x < 3) {
    const int q = threadIdx.x;
    partial[3 * blockIdx.x + q] += red[0][q] + red[1][q] + red[2][q] + red[3][q];
  }
}

__global__ __launch_bounds__(64) void weight_energy_kernel(const double* partial, double count, double var_coef, double l2_coef,
                                                           double scale, double* energy) {
  double a[3] = {0.0, 0.0, 0.0};
  for (int b = threadIdx.x; b < WSTAT_BLOCKS; b += 64)
    for (int q = 0; q < 3; ++q) a[q] += partial[3 * b + q];
  for (int q = 0; q < 3; ++q) a[q] = wave_allsum_d(a[q]);
  if (threadIdx.x == 0) {
    const double mean = a[1] / count;
    const double var = a[2] / count - mean * mean;
    *energy += scale * (a[0] + var_coef * var + l2_coef * sqrt(a[2]));
  }
}

strp_status launch_weight_energy(strp_ctx* ctx, const strp_weight_ref* mats, int n_mats, double var_coef, double l2_coef, double scale,
                                 double* energy, double* partial /* [3 * WSTAT_BLOCKS] scratch */) {
  STRP_TRY(fill_zero(ctx, partial, sizeof(double) * 3 * WSTAT_BLOCKS));
  double count = 0.0;
  for (int i = 0; i < n_mats; ++i) {
    const strp_weight_ref& m = mats[i];
    if (m.dtype == STRP_BF16)
      hipLaunchKernelGGL((weight_stats_kernel<true>), dim3(WSTAT_BLOCKS), dim3(256), 0, ctx->stream, m.W, m.rows, m.cols, (long long)m.ld, partial);
    else
      hipLaunchKernelGGL((weight_stats_kernel<false>), dim3(WSTAT_BLOCKS), dim3(256), 0, ctx->stream, m.W, m.rows, m.cols, (long long)m.ld, partial);
    count += (double)m.rows * (double)m.cols;
  }
  hipLaunchKernelGGL(weight_energy_kernel, dim3(1), dim3(64), 0, ctx->stream, (const double*)partial, count, var_coef, l2_coef, scale, energy);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}
size_t weight_energy_scratch_bytes() { return sizeof(double) * 3 * WSTAT_BLOCKS; }

constexpr int ALLOC_MAXL = 1024;

// rule 0: r = rbar L w, clip, conditional rescale (Alg. 1);  rule 1: r = rbar L (1 - w) / sum(1 - w), clip (Alg. 2)
__global__ __launch_bounds__(64) void alloc_kernel(const double* I, int L, const int32_t* n_units, const int32_t* group_id,
                                                   double rbar, double temperature, double rmax, int rule, double* r_out,
                                                   int32_t* nprune_out) {
  __shared__ double r[ALLOC_MAXL];
  __shared__ double frac[ALLOC_MAXL];
  __shared__ int base[ALLOC_MAXL];
  __shared__ int member[ALLOC_MAXL];
  const int lane = threadIdx.x;
  for (int lead = 0; lead < L; ++lead) {
    const int gid = group_id ? group_id[lead] : 0;
    bool is_lead = true;
    if (group_id) {
      for (int j = 0; j < lead; ++j)
        if (group_id[j] == gid) { is_lead = false; break; }
    } else {
      is_lead = (lead == 0);
    }
    if (!is_lead) continue;                    // uniform across the wavefront
    int Lg = 0;
    if (lane == 0) {
      for (int j = 0; j < L; ++j)
        if (!group_id || group_id[j] == gid) member[Lg++] = j;
    }
    Lg = __shfl(Lg, 0, 64);
    __syncthreads();
    // scale by mean |I|, softmax of -I/T with the maximum subtracted
    double sabs = 0.0;
    for (int q = lane; q < Lg; q += 64) sabs += fabs(I[member[q]]);
    sabs = wave_allsum_d(sabs);
    const double scale = sabs / (double)Lg;
    double amax = -1.0e308;
    for (int q = lane; q < Lg; q += 64) {
      const double a = (scale > 0.0) ? -(I[member[q]] / scale) / temperature : 0.0;
      r[q] = a;
      amax = fmax(amax, a);
    }
    amax = wave_allmax_d(amax);
    double wsum = 0.0;
    for (int q = lane; q < Lg; q += 64) {
      const double w = exp(r[q] - amax);
      r[q] = w;
      wsum += w;
    }
    wsum = wave_allsum_d(wsum);
    int at_max = 0;
    double rsum = 0.0;
    for (int q = lane; q < Lg; q += 64) {
      const double w = r[q] / wsum;
      double rv = rbar * (double)Lg * w;
      if (rule == 1) rv = Lg > 1 ? rbar * (double)Lg * (1.0 - w) / (double)(Lg - 1) : rbar;   // sum(1 - w) = L - 1
      rv = fmin(fmax(rv, 0.0), rmax);
      r[q] = rv;
      at_max |= (rv == rmax);
      rsum += rv;
    }
    at_max = __any(at_max);
    rsum = wave_allsum_d(rsum);
    if (!at_max && rule == 0) {
      const double mu = rsum / (double)Lg;
      for (int q = lane; q < Lg; q += 64) r[q] = fmin(fmax(r[q] * (rbar / mu), 0.0), rmax);
    }
    // largest-remainder integer counts
    double xsum = 0.0;
    long long bsum = 0;
    for (int q = lane; q < Lg; q += 64) {
      const double x = r[q] * (double)n_units[member[q]];
      const double fl = floor(x);
      base[q] = (int)fl;
      frac[q] = x - fl;
      xsum += x;
      bsum += (long long)fl;
    }
    xsum = wave_allsum_d(xsum);
    bsum = (long long)wave_allsum_d((double)bsum);
    const int extra = (int)(rint(xsum) - (double)bsum);
    __syncthreads();
    for (int q = lane; q < Lg; q += 64) {
      int rank = 0;
      const double fq = frac[q];
      for (int j = 0; j < Lg; ++j) rank += (frac[j] > fq) || (frac[j] == fq && j < q);
      int b = base[q] + ((rank < extra) ? 1 : 0);
      const int nu = n_units[member[q]];
      b = b > nu - 1 ? nu - 1 : b;
      b = b < 0 ? 0 : b;
      r_out[member[q]] = r[q];
      nprune_out[member[q]] = b;
    }
    __syncthreads();
  }
}

strp_status launch_alloc(strp_ctx* ctx, const double* energies, int L, const int32_t* n_units, const int32_t* group_id,
                         double rbar, double temperature, double rmax, int rule, double* r_out, int32_t* nprune_out) {
  if (L <= 0 || L > ALLOC_MAXL) return fail(ctx, STRP_EINVAL, "alloc: L=%d outside [1, %d]", L, ALLOC_MAXL);
  hipLaunchKernelGGL(alloc_kernel, dim3(1), dim3(64), 0, ctx->stream, energies, L, n_units, group_id, rbar, temperature,
                     rmax, rule, r_out, nprune_out);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

// ---------------------------------------------------------------------------------------------
// top-k select: one block of 1024 threads; 4 radix passes of 8 bits find the k-th largest key, then an
// index-ordered compaction (ballot + popcount prefix) writes mask and ascending kept indices.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ unsigned int score_key(float x) {
  const unsigned int u = __builtin_bit_cast(unsigned int, x + 0.0f);   // -0 and +0 are one value: both map to +0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_score(unsigned int k) {
  const unsigned int u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
  return __builtin_bit_cast(float, u);
}

__global__ __launch_bounds__(1024) void topk_kernel(const float* score, int n, int k, int group, uint8_t* mask, int32_t* idx,
                                                    float* tau) {
  __shared__ unsigned int hist[256];
  __shared__ unsigned int sel_prefix, sel_krem;
  __shared__ int wave_tot[16][2];
  __shared__ int run_eq, run_kept;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  if (k <= 0 || k >= n) {  // degenerate: nothing or everything kept
    const int keep = k >= n;
    for (int i = tid; i < n; i += 1024) {
      mask[i] = (uint8_t)keep;
      if (keep)
        for (int c = 0; c < group; ++c) idx[(long long)i * group + c] = i * group + c;
    }
    if (tid == 0 && tau) {
      float t = __builtin_inff();
      if (keep) {
        t = score[0];
        for (int i = 1; i < n; ++i) t = fminf(t, score[i]);
      }
      *tau = t;
    }
    return;
  }

  unsigned int prefix = 0, pmask = 0;
  unsigned int krem = (unsigned int)k;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += 1024) {
      const unsigned int key = score_key(score[i]);
      if ((key & pmask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (tid < 64) {
      // the bucket d with  #(keys in buckets above d) < krem <= #(keys in buckets d and above): lane l owns buckets
      // 4 l .. 4 l + 3, a wavefront suffix scan gives the count above its group, exactly one (lane, bucket) matches
      unsigned int h[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) h[j] = hist[4 * tid + j];
      const unsigned int own = h[0] + h[1] + h[2] + h[3];
      unsigned int suf = own;   // inclusive suffix sum over lanes >= tid
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const unsigned int v = __shfl_down(suf, o, 64);
        if (tid + o < 64) suf += v;
      }
      unsigned int cum = suf - own;   // keys in the groups above this lane's
#pragma unroll
      for (int j = 3; j >= 0; --j) {
        if (cum < krem && cum + h[j] >= krem) {
          sel_prefix = prefix | ((unsigned int)(4 * tid + j) << shift);
          sel_krem = krem - cum;
        }
        cum += h[j];
      }
    }
    __syncthreads();
    prefix = sel_prefix;
    krem = sel_krem;
    pmask |= 255u << shift;
    __syncthreads();
  }
  // prefix is the k-th largest key; krem of the keys equal to it are kept (lowest indices first)
  if (tid == 0) {
    run_eq = 0;
    run_kept = 0;
    if (tau) *tau = key_score(prefix);
  }
  __syncthreads();
  for (int base = 0; base < n; base += 1024) {
    const int i = base + tid;
    unsigned int key = 0;
    const bool in = i < n;
    if (in) key = score_key(score[i]);
    const bool gt = in && key > prefix;
    const bool eq = in && key == prefix;
    const unsigned long long beq = __ballot(eq);
    const unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    const int eq_before = __popcll(beq & lt_mask);
    if (lane == 0) wave_tot[wave][0] = __popcll(beq);
    __syncthreads();
    int eq_off = run_eq;
    for (int w = 0; w < wave; ++w) eq_off += wave_tot[w][0];
    const bool keep = gt || (eq && (unsigned int)(eq_off + eq_before) < krem);
    const unsigned long long bk = __ballot(keep);
    const int k_before = __popcll(bk & lt_mask);
    if (lane == 0) wave_tot[wave][1] = __popcll(bk);
    __syncthreads();
    int k_off = run_kept;
    for (int w = 0; w < wave; ++w) k_off += wave_tot[w][1];
    if (in) {
      mask[i] = (uint8_t)keep;
      if (keep) {
        const long long pos = (long long)(k_off + k_before) * group;
        for (int c = 0; c < group; ++c) idx[pos + c] = i * group + c;
      }
    }
    __syncthreads();
    if (tid == 0) {
      int te = 0, tk = 0;
      for (int w = 0; w < 16; ++w) {
        te += wave_tot[w][0];
        tk += wave_tot[w][1];
      }
      run_eq += te;
      run_kept += tk;
    }
    __syncthreads();
  }
}

// One module's scores (n <= 16384, 0 < k < n): the 16 keys of a thread (elements tid + 1024 j) stay in registers.
// The k-th largest key is built bit by bit from the top (32 counting rounds: ballots + one barrier each; a radix
// histogram in LDS serialises on the few exponent buckets real scores fall into).  The index-ordered compaction
// takes two table scans instead of a barrier chain per 1024 elements: per (round j, wavefront) counts of the keys
// equal to the threshold, then of the kept keys, scanned in (j, wavefront) order = index order.
__device__ __forceinline__ int table_scan_256(int val, int* wtot, int tid) {
  // exclusive prefix of val over threads 0..255 (called by every thread of the block; others pass 0 and ignore)
  const int lane = tid & 63, wave = tid >> 6;
  int inc = val;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int v = __shfl_up(inc, o, 64);
    if (lane >= o) inc += v;
  }
  if (lane == 63 && wave < 4) wtot[wave] = inc;
  __syncthreads();
  int off = 0;
  for (int w = 0; w < wave && w < 4; ++w) off += wtot[w];
  __syncthreads();
  return off + inc - val;
}

__global__ __launch_bounds__(1024) void topk_small_kernel(const float* score, int n, int k, int group, uint8_t* mask, int32_t* idx,
                                                          float* tau) {
  __shared__ int wcnt[2][16];
  __shared__ int table[256];      // [round j][wavefront]
  __shared__ int wtot[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  unsigned int kreg[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const int i = tid + 1024 * j;
    kreg[j] = i < n ? score_key(score[i]) : 0u;   // a candidate always has a bit set, so padding is never counted
  }
  auto count_ge = [&](unsigned int cand, int buf) {
    int c = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) c += __popcll(__ballot(kreg[j] >= cand));
    if (lane == 0) wcnt[buf][wave] = c;
    __syncthreads();
    int tot = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) tot += wcnt[buf][w];
    return tot;
  };
  unsigned int v = 0;
  for (int b = 31; b >= 0; --b) {
    const unsigned int cand = v | (1u << b);
    if (count_ge(cand, b & 1) >= k) v = cand;
  }
  // v = k-th largest key.  Keys above it are kept, of the keys equal to it the krem with the lowest indices.
  int n_gt = 0;
  if (v != 0xffffffffu) n_gt = count_ge(v + 1u, 1);   // buffer 1: round b = 0 may still be read from buffer 0
  const int krem = k - n_gt;
  if (tid == 0 && tau) *tau = key_score(v);
  const unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  // counts of equal keys per (round, wavefront)
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const unsigned long long beq = __ballot(tid + 1024 * j < n && kreg[j] == v);
    if (lane == 0) table[j * 16 + wave] = __popcll(beq);
  }
  __syncthreads();
  const int eq_pref = table_scan_256(tid < 256 ? table[tid] : 0, wtot, tid);
  if (tid < 256) table[tid] = eq_pref;
  __syncthreads();
  unsigned int keepbits = 0;
  int kcnt[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const bool in = tid + 1024 * j < n;
    const bool eq = in && kreg[j] == v;
    const unsigned long long beq = __ballot(eq);
    const int rank = table[j * 16 + wave] + __popcll(beq & lt_mask);
    const bool keep = in && (kreg[j] > v || (eq && rank < krem));
    keepbits |= (unsigned int)keep << j;
    const unsigned long long bk = __ballot(keep);
    kcnt[j] = __popcll(bk & lt_mask);
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const unsigned long long bk = __ballot((keepbits >> j) & 1u);
    if (lane == 0) table[j * 16 + wave] = __popcll(bk);
  }
  __syncthreads();
  const int kp_pref = table_scan_256(tid < 256 ? table[tid] : 0, wtot, tid);
  if (tid < 256) table[tid] = kp_pref;
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const int i = tid + 1024 * j;
    if (i >= n) continue;
    const bool keep = (keepbits >> j) & 1u;
    mask[i] = (uint8_t)keep;
    if (keep) {
      const long long pos = (long long)(table[j * 16 + wave] + kcnt[j]) * group;
      for (int c = 0; c < group; ++c) idx[pos + c] = i * group + c;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// top-k select over a long score vector (all layers' scores at once for a global threshold, or a stress
// input): several blocks, two reads of the scores and one of the mask.
//   level 0 (top 11 key bits: sign, exponent, 2 mantissa bits), over the scores
//     hist    every block histograms its contiguous chunk (kept per block and summed)
//     pick    one block picks the bucket that holds the k-th largest key; keys above it are kept, below dropped
//     gather  every block re-reads its chunk, writes the mask of the decided keys and appends the keys of the
//             bucket (a few per cent of n: the bucket is a 2^(1/4)-wide value range) to a candidate list, in
//             index order (the per-block histograms give the offsets)
//   level 1 (next 11 bits), over the candidates: the same three steps; what survives is ~n / 10^5 keys
//   resolve   one block selects among those on the last 10 bits, ties to the lower index, completes the mask and
//             scans the per-block kept counts
//   compact   every block turns its part of the mask into ascending indices
// A vector of equal scores degenerates to candidate lists of length n and a single-block resolve: correct, slow.
// ---------------------------------------------------------------------------------------------
namespace big {
constexpr int BINS = 2048;          // 11 bits
constexpr int THREADS = 512;
constexpr int MAXBLOCKS = 1024;
constexpr int L1BLOCKS = 256;
struct State {
  unsigned int bucket;      // chosen digit at this level
  unsigned int krem;        // keys still to keep inside the bucket
  unsigned int ncand;       // keys in the bucket
  unsigned int pad;
};
}  // namespace big

struct BigLevel {
  unsigned int* bhist;      // [blocks][BINS]
  unsigned int* ghist;      // [BINS]
  big::State* state;        // this level's choice
  unsigned int* coff;       // [blocks] offset of the block's candidates in the output list
  unsigned int* cand_key;   // output list
  int* cand_idx;
  int blocks;
};

struct BigTopkPlan {
  int blocks0;
  long long chunk0;         // elements per block at level 0 (multiple of big::THREADS)
  BigLevel lv[2];
  unsigned int* gtcnt;      // [blocks0] keys above the level-0 bucket in the block's chunk
  unsigned int* kept_cand;  // [blocks0] kept candidates per level-0 chunk (levels 1 and 2)
  unsigned int* kpre;       // [blocks0] kept entries before the block's chunk
  int vec;                  // scores 16-byte aligned and mask 8-byte aligned: vector accesses allowed
};

static void big_plan(long long n, int* blocks, long long* chunk) {
  long long b = (n + 8 * big::THREADS - 1) / (8 * big::THREADS);
  if (b > big::MAXBLOCKS) b = big::MAXBLOCKS;
  if (b < 1) b = 1;
  long long c = (n + b - 1) / b;
  c = (c + big::THREADS - 1) / big::THREADS * big::THREADS;
  *blocks = (int)((n + c - 1) / c);
  *chunk = c;
}

size_t topk_scratch_bytes(int n) {
  if (n <= 65536) return 0;
  int blocks;
  long long chunk;
  big_plan(n, &blocks, &chunk);
  auto al = [](size_t b) { return (b + 255) & ~size_t(255); };
  return al((size_t)blocks * big::BINS * 4) + al((size_t)big::L1BLOCKS * big::BINS * 4) + 2 * al(big::BINS * 4) + 2 * al(sizeof(big::State)) +
         al((size_t)blocks * 4) + al((size_t)big::L1BLOCKS * 4) + 3 * al((size_t)blocks * 4) + 4 * al((size_t)n * 4) + 256;
}

// chunk of block blk at level LEVEL: level 0 splits [0, n) by plan.chunk0; level 1 splits the candidate list, whose
// length is a device value
template <int LEVEL>
__device__ __forceinline__ void level_range(const BigTopkPlan& pl, long long n, long long* beg, long long* end) {
  if (LEVEL == 0) {
    *beg = (long long)blockIdx.x * pl.chunk0;
    *end = *beg + pl.chunk0 < n ? *beg + pl.chunk0 : n;
  } else {
    const long long m = pl.lv[0].state->ncand;
    long long c = (m + gridDim.x - 1) / gridDim.x;
    c = (c + big::THREADS - 1) / big::THREADS * big::THREADS;
    *beg = (long long)blockIdx.x * c < m ? (long long)blockIdx.x * c : m;
    *end = *beg + c < m ? *beg + c : m;
  }
}
template <int LEVEL>
__device__ __forceinline__ unsigned int level_key(const BigTopkPlan& pl, const float* score, long long i) {
  return LEVEL == 0 ? score_key(score[i]) : pl.lv[0].cand_key[i];
}
template <int LEVEL>
__device__ __forceinline__ unsigned int level_digit(unsigned int key) {
  return LEVEL == 0 ? key >> 21 : (key >> 10) & 0x7ffu;
}

template <int LEVEL>
__global__ __launch_bounds__(big::THREADS) void topk_hist_kernel(const float* score, long long n, BigTopkPlan pl) {
  __shared__ unsigned int hist[big::BINS];
  for (int i = threadIdx.x; i < big::BINS; i += big::THREADS) hist[i] = 0;
  __syncthreads();
  long long beg, end;
  level_range<LEVEL>(pl, n, &beg, &end);
  if (LEVEL == 0 && pl.vec) {   // beg is a multiple of 512: float4 loads stay aligned
    const long long nv = (end - beg) >> 2;
    const float4* s4 = (const float4*)(score + beg);
    for (long long v = threadIdx.x; v < nv; v += big::THREADS) {
      const float4 x = s4[v];
      atomicAdd(&hist[score_key(x.x) >> 21], 1u);
      atomicAdd(&hist[score_key(x.y) >> 21], 1u);
      atomicAdd(&hist[score_key(x.z) >> 21], 1u);
      atomicAdd(&hist[score_key(x.w) >> 21], 1u);
    }
    for (long long i = beg + (nv << 2) + threadIdx.x; i < end; i += big::THREADS) atomicAdd(&hist[score_key(score[i]) >> 21], 1u);
  } else {
    for (long long i = beg + threadIdx.x; i < end; i += big::THREADS) atomicAdd(&hist[level_digit<LEVEL>(level_key<LEVEL>(pl, score, i))], 1u);
  }
  __syncthreads();
  const BigLevel& lv = pl.lv[LEVEL];
  for (int i = threadIdx.x; i < big::BINS; i += big::THREADS) {
    const unsigned int h = hist[i];
    lv.bhist[(long long)blockIdx.x * big::BINS + i] = h;
    if (h) atomicAdd(&lv.ghist[i], h);
  }
}

// One block: bucket choice at this level and the per-block candidate offsets.  The number to keep is k at level 0
// and what level 0 left to its bucket at level 1.
template <int LEVEL>
__global__ __launch_bounds__(1024) void topk_pick_kernel(long long k0, BigTopkPlan pl) {
  __shared__ unsigned long long suf[big::BINS];   // suf[d] = number of keys with digit >= d
  __shared__ unsigned int sb;
  __shared__ unsigned int scan[1024];
  const int tid = threadIdx.x;
  const BigLevel& lv = pl.lv[LEVEL];
  const unsigned long long k = LEVEL == 0 ? (unsigned long long)k0 : (unsigned long long)pl.lv[0].state->krem;
  suf[tid] = lv.ghist[tid];
  suf[tid + 1024] = lv.ghist[tid + 1024];
  if (tid == 0) sb = 0;
  __syncthreads();
  for (int o = 1; o < big::BINS; o <<= 1) {   // inclusive suffix scan, two bins per thread
    const unsigned long long v0 = tid + o < big::BINS ? suf[tid + o] : 0ull;
    const unsigned long long v1 = tid + 1024 + o < big::BINS ? suf[tid + 1024 + o] : 0ull;
    __syncthreads();
    suf[tid] += v0;
    suf[tid + 1024] += v1;
    __syncthreads();
  }
  // the bucket is the largest digit whose suffix count reaches k (digit 0 always does: k <= n)
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int d = tid + 1024 * h;
    const unsigned long long above = d + 1 < big::BINS ? suf[d + 1] : 0ull;
    if (suf[d] >= k && above < k) {
      sb = (unsigned int)d;
      lv.state->bucket = (unsigned int)d;
      lv.state->krem = (unsigned int)(k - above);
      lv.state->ncand = (unsigned int)(suf[d] - above);
    }
  }
  __syncthreads();
  const unsigned int b = sb;
  const unsigned int mine = tid < lv.blocks ? lv.bhist[(long long)tid * big::BINS + b] : 0u;
  scan[tid] = mine;
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {   // inclusive scan
    const unsigned int v = tid >= o ? scan[tid - o] : 0;
    __syncthreads();
    scan[tid] += v;
    __syncthreads();
  }
  if (tid < lv.blocks) lv.coff[tid] = scan[tid] - mine;
}

// position of a flagged thread among the flagged threads of the block, in thread order; *total = their number
__device__ __forceinline__ int block_rank(bool flag, int* wave_tot, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const unsigned long long bal = __ballot(flag);
  const unsigned long long lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  if (lane == 0) wave_tot[wave] = __popcll(bal);
  __syncthreads();
  int off = 0, tot = 0;
  const int nw = blockDim.x >> 6;
  for (int w = 0; w < nw; ++w) {
    const int c = wave_tot[w];
    if (w < wave) off += c;
    tot += c;
  }
  __syncthreads();
  *total = tot;
  return off + __popcll(bal & lt);
}

// exclusive prefix, in thread order, of a per-thread count over the block; *total = the block's sum
__device__ __forceinline__ int block_scan(int cnt, int* wave_tot, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = cnt;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int v = __shfl_up(inc, o, 64);
    if (lane >= o) inc += v;
  }
  if (lane == 63) wave_tot[wave] = inc;
  __syncthreads();
  int off = 0, tot = 0;
  const int nw = blockDim.x >> 6;
  for (int w = 0; w < nw; ++w) {
    const int c = wave_tot[w];
    if (w < wave) off += c;
    tot += c;
  }
  __syncthreads();
  *total = tot;
  return off + inc - cnt;
}

// kept candidates are counted per level-0 chunk (for the final compaction): LDS counters, flushed at the end
__device__ __forceinline__ void kept_flush(unsigned int* lds_cnt, unsigned int* global_cnt, int blocks0) {
  __syncthreads();
  for (int i = threadIdx.x; i < blocks0; i += blockDim.x) {
    const unsigned int c = lds_cnt[i];
    if (c) atomicAdd(&global_cnt[i], c);
  }
}

// Each thread takes EPT consecutive entries per round (index order is thread order), so a round costs one block
// scan for EPT * THREADS entries.
template <int LEVEL>
__global__ __launch_bounds__(big::THREADS) void topk_gather_kernel(const float* score, long long n, uint8_t* mask, BigTopkPlan pl) {
  constexpr int EPT = 8;
  __shared__ int wave_tot[16];
  __shared__ unsigned int kept_blk[big::MAXBLOCKS];
  const BigLevel& lv = pl.lv[LEVEL];
  const unsigned int b = lv.state->bucket;
  if (LEVEL == 1) {
    for (int i = threadIdx.x; i < big::MAXBLOCKS; i += big::THREADS) kept_blk[i] = 0;
    __syncthreads();
  }
  long long beg, end;
  level_range<LEVEL>(pl, n, &beg, &end);
  unsigned int run = lv.coff[blockIdx.x];
  unsigned int n_above = 0;   // level 0: this thread's keys above the bucket
  for (long long base = beg; base < end; base += (long long)EPT * big::THREADS) {
    const long long i0 = base + (long long)threadIdx.x * EPT;
    unsigned int key[EPT];
    int id[EPT];
    int cnt = 0;
    unsigned int isc = 0, above = 0;
    const bool whole = LEVEL == 0 && pl.vec && i0 + EPT <= end;   // i0 is a multiple of 8
    float xv[EPT];
    if (whole) {
      const float4 x0 = *(const float4*)(score + i0), x1 = *(const float4*)(score + i0 + 4);
      xv[0] = x0.x; xv[1] = x0.y; xv[2] = x0.z; xv[3] = x0.w;
      xv[4] = x1.x; xv[5] = x1.y; xv[6] = x1.z; xv[7] = x1.w;
    }
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      const long long i = i0 + e;
      const bool in = i < end;
      key[e] = whole ? score_key(xv[e]) : (in ? level_key<LEVEL>(pl, score, i) : 0u);
      id[e] = LEVEL == 0 ? (int)i : (in ? pl.lv[0].cand_idx[i] : 0);
      const unsigned int dgt = level_digit<LEVEL>(key[e]);
      if (in && dgt == b) { isc |= 1u << e; ++cnt; }
      if (in && dgt > b) above |= 1u << e;
    }
    int tot;
    unsigned int pos = run + (unsigned int)block_scan(cnt, wave_tot, &tot);
    if (LEVEL == 0) {
      n_above += (unsigned int)__popc(above);
      if (whole) {   // eight mask bytes in one store
        unsigned long long m8 = 0;
#pragma unroll
        for (int e = 0; e < EPT; ++e) m8 |= (unsigned long long)((above >> e) & 1u) << (8 * e);
        *(unsigned long long*)(mask + i0) = m8;
      }
    }
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      const long long i = i0 + e;
      if (LEVEL == 0) {
        if (!whole && i < end) mask[i] = (uint8_t)((above >> e) & 1u);
      } else if ((above >> e) & 1u) {
        mask[id[e]] = 1;
        atomicAdd(&kept_blk[(long long)id[e] / pl.chunk0], 1u);
      }
      if ((isc >> e) & 1u) {
        lv.cand_key[pos] = key[e];
        lv.cand_idx[pos] = id[e];
        ++pos;
      }
    }
    run += (unsigned int)tot;
  }
  if (LEVEL == 1) kept_flush(kept_blk, pl.kept_cand, pl.blocks0);
  if (LEVEL == 0) {
    int tot;
    (void)block_scan((int)n_above, wave_tot, &tot);
    if (threadIdx.x == 0) pl.gtcnt[blockIdx.x] = (unsigned int)tot;
  }
}

// One block: the krem largest of the level-1 candidates on their last 10 key bits, ties to the lower index (the
// list is in index order), then the exclusive scan of the per-chunk kept counts.
__global__ __launch_bounds__(1024) void topk_resolve_kernel(uint8_t* mask, float* tau, BigTopkPlan pl) {
  __shared__ unsigned int hist[1024];
  __shared__ unsigned int sel_low, sel_krem;
  __shared__ int wave_tot[16];
  __shared__ unsigned int kept_blk[big::MAXBLOCKS];
  const int tid = threadIdx.x;
  const BigLevel& lv = pl.lv[1];
  const unsigned int ncand = lv.state->ncand;
  hist[tid] = 0;
  kept_blk[tid] = 0;
  __syncthreads();
  for (unsigned int i = tid; i < ncand; i += 1024) atomicAdd(&hist[lv.cand_key[i] & 0x3ffu], 1u);
  __syncthreads();
  if (tid == 0) {
    const unsigned int krem = lv.state->krem;
    unsigned int cum = 0;
    int d = 1023;
    for (; d > 0; --d) {
      if (cum + hist[d] >= krem) break;
      cum += hist[d];
    }
    sel_low = (unsigned int)d;
    sel_krem = krem - cum;
    if (tau) *tau = key_score((pl.lv[0].state->bucket << 21) | (lv.state->bucket << 10) | (unsigned int)d);
  }
  __syncthreads();
  const unsigned int low = sel_low, krem = sel_krem;   // krem of the candidates equal to the threshold are kept
  unsigned int run_eq = 0;
  for (unsigned int base = 0; base < ncand; base += 1024) {
    const unsigned int i = base + tid;
    const bool in = i < ncand;
    unsigned int key = 0;
    int id = 0;
    if (in) {
      key = lv.cand_key[i] & 0x3ffu;
      id = lv.cand_idx[i];
    }
    const bool eq = in && key == low;
    int tot;
    const int r = block_rank(eq, wave_tot, &tot);
    const bool keep = in && (key > low || (eq && run_eq + (unsigned int)r < krem));
    if (keep) {
      mask[id] = 1;
      atomicAdd(&kept_blk[(long long)id / pl.chunk0], 1u);
    }
    run_eq += (unsigned int)tot;
  }
  __syncthreads();
  // exclusive scan of kept = above the level-0 bucket + kept candidates, per level-0 chunk (<= 1024 = one per thread)
  const unsigned int mine = tid < pl.blocks0 ? pl.gtcnt[tid] + pl.kept_cand[tid] + kept_blk[tid] : 0;
  __syncthreads();
  kept_blk[tid] = mine;
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {
    const unsigned int v = tid >= o ? kept_blk[tid - o] : 0;
    __syncthreads();
    kept_blk[tid] += v;
    __syncthreads();
  }
  if (tid < pl.blocks0) pl.kpre[tid] = kept_blk[tid] - mine;
}

__global__ __launch_bounds__(big::THREADS) void topk_compact_kernel(const uint8_t* mask, long long n, int32_t* idx, BigTopkPlan pl) {
  constexpr int EPT = 8;   // eight consecutive mask bytes per thread: chunk0 and every round start are multiples of 8
  __shared__ int wave_tot[16];
  const long long beg = (long long)blockIdx.x * pl.chunk0;
  const long long end = beg + pl.chunk0 < n ? beg + pl.chunk0 : n;
  unsigned int run = pl.kpre[blockIdx.x];
  for (long long base = beg; base < end; base += (long long)EPT * big::THREADS) {
    const long long i0 = base + (long long)threadIdx.x * EPT;
    unsigned int bits = 0;
    if (pl.vec && i0 + EPT <= end) {
      const unsigned long long m8 = *(const unsigned long long*)(mask + i0);
#pragma unroll
      for (int e = 0; e < EPT; ++e)
        if ((m8 >> (8 * e)) & 0xffull) bits |= 1u << e;
    } else {
#pragma unroll
      for (int e = 0; e < EPT; ++e)
        if (i0 + e < end && mask[i0 + e]) bits |= 1u << e;
    }
    int tot;
    unsigned int pos = run + (unsigned int)block_scan(__popc(bits), wave_tot, &tot);
#pragma unroll
    for (int e = 0; e < EPT; ++e)
      if ((bits >> e) & 1u) idx[pos++] = (int)(i0 + e);
    run += (unsigned int)tot;
  }
}

strp_status launch_topk(strp_ctx* ctx, const float* score, int n, int k, int group, uint8_t* mask, int32_t* idx, float* tau,
                        void* scratch, size_t scratch_bytes) {
  ProfScope ps(ctx, "topk", 0.0, 5.0 * (double)n + 4.0 * (double)k * group);
  const bool big_path = n > 65536 && group == 1 && k > 0 && k < n;
  if (!big_path) {
    if (n <= 16 * 1024 && k > 0 && k < n)
      hipLaunchKernelGGL(topk_small_kernel, dim3(1), dim3(1024), 0, ctx->stream, score, n, k, group, mask, idx, tau);
    else
      hipLaunchKernelGGL(topk_kernel, dim3(1), dim3(1024), 0, ctx->stream, score, n, k, group, mask, idx, tau);
    STRP_HIP(ctx, hipGetLastError());
    return STRP_OK;
  }
  if (!scratch || scratch_bytes < topk_scratch_bytes(n))
    return fail(ctx, STRP_ENOMEM, "top-k over %d scores needs %zu bytes of workspace", n, topk_scratch_bytes(n));
  BigTopkPlan pl;
  big_plan(n, &pl.blocks0, &pl.chunk0);
  pl.vec = (((uintptr_t)score & 15) == 0 && ((uintptr_t)mask & 7) == 0) ? 1 : 0;
  char* p = (char*)scratch;
  auto take = [&](size_t bytes) { char* q = p; p += (bytes + 255) & ~size_t(255); return q; };
  pl.lv[0].blocks = pl.blocks0;
  pl.lv[1].blocks = big::L1BLOCKS;
  pl.lv[0].bhist = (unsigned int*)take((size_t)pl.blocks0 * big::BINS * 4);
  pl.lv[1].bhist = (unsigned int*)take((size_t)big::L1BLOCKS * big::BINS * 4);
  // contiguous from here to kept_cand: cleared by one fill
  char* z0 = p;
  pl.lv[0].ghist = (unsigned int*)take(big::BINS * 4);
  pl.lv[1].ghist = (unsigned int*)take(big::BINS * 4);
  pl.lv[0].state = (big::State*)take(sizeof(big::State));
  pl.lv[1].state = (big::State*)take(sizeof(big::State));
  pl.kept_cand = (unsigned int*)take((size_t)pl.blocks0 * 4);
  const size_t zbytes = (size_t)(p - z0);
  pl.lv[0].coff = (unsigned int*)take((size_t)pl.blocks0 * 4);
  pl.lv[1].coff = (unsigned int*)take((size_t)big::L1BLOCKS * 4);
  pl.gtcnt = (unsigned int*)take((size_t)pl.blocks0 * 4);
  pl.kpre = (unsigned int*)take((size_t)pl.blocks0 * 4);
  for (int l = 0; l < 2; ++l) {
    pl.lv[l].cand_key = (unsigned int*)take((size_t)n * 4);
    pl.lv[l].cand_idx = (int*)take((size_t)n * 4);
  }
  STRP_TRY(fill_zero(ctx, z0, zbytes));
  const dim3 b0(pl.blocks0), b1(big::L1BLOCKS), th(big::THREADS);
  hipLaunchKernelGGL((topk_hist_kernel<0>), b0, th, 0, ctx->stream, score, (long long)n, pl);
  hipLaunchKernelGGL((topk_pick_kernel<0>), dim3(1), dim3(1024), 0, ctx->stream, (long long)k, pl);
  hipLaunchKernelGGL((topk_gather_kernel<0>), b0, th, 0, ctx->stream, score, (long long)n, mask, pl);
  hipLaunchKernelGGL((topk_hist_kernel<1>), b1, th, 0, ctx->stream, score, (long long)n, pl);
  hipLaunchKernelGGL((topk_pick_kernel<1>), dim3(1), dim3(1024), 0, ctx->stream, (long long)k, pl);
  hipLaunchKernelGGL((topk_gather_kernel<1>), b1, th, 0, ctx->stream, score, (long long)n, mask, pl);
  hipLaunchKernelGGL(topk_resolve_kernel, dim3(1), dim3(1024), 0, ctx->stream, mask, tau, pl);
  hipLaunchKernelGGL(topk_compact_kernel, b0, th, 0, ctx->stream, (const uint8_t*)mask, (long long)n, idx, pl);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

}  // namespace strp
