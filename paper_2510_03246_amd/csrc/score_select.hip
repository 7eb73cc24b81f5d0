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
constexpr int ALLOC_MAXL = 1024;

__global__ __launch_bounds__(64) void alloc_kernel(const double* I, int L, const int32_t* n_units, const int32_t* group_id,
                                                   double rbar, double temperature, double rmax, double* r_out,
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
      double rv = rbar * (double)Lg * (r[q] / wsum);
      rv = fmin(fmax(rv, 0.0), rmax);
      r[q] = rv;
      at_max |= (rv == rmax);
      rsum += rv;
    }
    at_max = __any(at_max);
    rsum = wave_allsum_d(rsum);
    if (!at_max) {
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
                         double rbar, double temperature, double rmax, double* r_out, int32_t* nprune_out) {
  if (L <= 0 || L > ALLOC_MAXL) return fail(ctx, STRP_EINVAL, "alloc: L=%d outside [1, %d]", L, ALLOC_MAXL);
  hipLaunchKernelGGL(alloc_kernel, dim3(1), dim3(64), 0, ctx->stream, energies, L, n_units, group_id, rbar, temperature,
                     rmax, r_out, nprune_out);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

// ---------------------------------------------------------------------------------------------
// top-k select: one block of 1024 threads; 4 radix passes of 8 bits find the k-th largest key, then an
// index-ordered compaction (ballot + popcount prefix) writes mask and ascending kept indices.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ unsigned int score_key(float x) {
  const unsigned int u = __builtin_bit_cast(unsigned int, x);
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
    if (tid == 0) {
      unsigned int cum = 0;
      int d = 255;
      for (; d > 0; --d) {
        if (cum + hist[d] >= krem) break;
        cum += hist[d];
      }
      sel_prefix = prefix | ((unsigned int)d << shift);
      sel_krem = krem - cum;
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

size_t topk_scratch_bytes(int n) { (void)n; return 0; }

strp_status launch_topk(strp_ctx* ctx, const float* score, int n, int k, int group, uint8_t* mask, int32_t* idx, float* tau,
                        void* scratch, size_t scratch_bytes) {
  (void)scratch;
  (void)scratch_bytes;
  ProfScope ps(ctx, "topk", 0.0, 5.0 * (double)n + 4.0 * (double)k * group);
  hipLaunchKernelGGL(topk_kernel, dim3(1), dim3(1024), 0, ctx->stream, score, n, k, group, mask, idx, tau);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

}  // namespace strp
