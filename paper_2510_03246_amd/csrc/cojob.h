// A streaming pass that rides along with other kernels.
//
// The factorisation chains of an ADMM iteration are some hundred short launches (a 64-column Cholesky step is a panel
// kernel of at most 77 workgroups and an update of a few hundred) that leave most of the chip idle, and kernels of two
// streams do not share the chip usefully on this hardware.  Workgroups of ONE launch do: so a pass that is bound by
// HBM and independent of the chain is cut into units, and the chain's kernels are launched with spare workgroups that
// take a few units each from a device counter and exit.  Whatever is left when the chain ends is drained by a kernel
// of its own.  No workgroup ever waits for another one: the counter only hands out unit numbers.
//
// The one pass built this way is the fused a/z update of the PRUNED rows (Appendix A.1 with W2[:, j] = 0, W1[j, :] = 0:
// A_j = relu(Z_j), then the z rule with z1 = 0), which touches only rows outside S and can therefore run at any time
// between the selection and the end of the iteration.  A unit is one segment of `seg_tokens` tokens of one pruned row;
// its six sums (two objective terms, four scoring sums) go to `partial` and are added per row, in segment order, by
// the finishing kernel, so the result does not depend on which workgroup took which unit.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace strp {

struct CoJob {
  unsigned int* ticket;    // next unit to hand out (device counter, zero when the job starts); null = no job
  unsigned int units;      // nrows * segs
  int take;                // units a spare workgroup takes before it exits
  const int32_t* rows;     // the pruned rows, ascending
  int nrows, segs;
  long long seg_tokens;    // tokens per unit (a multiple of 4)
  float* Z;
  float* A;
  const float* Z0;         // null: only sum A^2 is collected for the scores
  long long lda, T;
  float alpha, beta;
  double* partial;         // [units][6]: sum (A - relu Z)^2, Z^2, A^2, A relu(Z0), Z0 Z, Z0^2 over the unit
};

// Rows of pruned units (mask == 0): W2[:, j] = 0 and W1[j, :] = 0 decouple them.
//   phase 0 (a-update): A_j = relu(Z_j)
//   phase 1 (z-update): exact z rule with z1 = 0; accumulates (A - relu Z)^2 and (Z - 0)^2
//   phase 2: both in one pass over the row (A_j = relu(Z_j), then the z rule on the new A_j)
__device__ __forceinline__ void pruned_elem(float& zv, float& av, int phase, float alpha, float beta, int write, double& r0, double& r1) {
  if (phase != 1) av = __builtin_fmaxf(zv, 0.0f);
  if (phase != 0) {
    if (write) {
      const float z2 = beta * av / (alpha + beta);
      const float costm = beta * av * av;
      const float cp = __builtin_fmaxf(z2, 0.0f);
      const float costp = beta * (av - cp) * (av - cp) + alpha * cp * cp;
      zv = costm < costp ? 0.0f : cp;
    }
    const float ra = av - __builtin_fmaxf(zv, 0.0f);
    r0 += (double)ra * (double)ra;
    r1 += (double)zv * (double)zv;
  }
}

// One unit, by a workgroup of 256 threads (every thread must call it; ends with a barrier).
__device__ __forceinline__ void cojob_unit(const CoJob& job, unsigned int u) {
  __shared__ double cj_sh[4][6];
  const int tid = threadIdx.x;
  const unsigned int p = u / (unsigned int)job.segs, g = u - p * (unsigned int)job.segs;
  const long long row = job.rows[p];
  if (row < 0) {   // no such row (see pruned_list_kernel): the unit's sums are zero
    if (tid < 6) job.partial[(unsigned long long)u * 6 + tid] = 0.0;
    __syncthreads();
    return;
  }
  float* z = job.Z + row * job.lda;
  float* a = job.A + row * job.lda;
  const float* z0 = job.Z0 ? job.Z0 + row * job.lda : nullptr;
  const long long s0 = (long long)g * job.seg_tokens;
  const bool last = s0 + job.seg_tokens >= job.T;
  const long long v0 = s0 >> 2, v1 = last ? (job.T >> 2) : ((s0 + job.seg_tokens) >> 2);
  const float alpha = job.alpha, beta = job.beta;
  double r0 = 0.0, r1 = 0.0, sg = 0.0, se = 0.0, su = 0.0, sv = 0.0;
  auto sums = [&](float av, float zv, float w) {
    sg = __builtin_fma((double)av, (double)av, sg);
    if (z0) {
      const double z0d = w;
      se = __builtin_fma((double)av, fmax(z0d, 0.0), se);
      su = __builtin_fma(z0d, (double)zv, su);
      sv = __builtin_fma(z0d, z0d, sv);
    }
  };
  const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
  // eight independent 16-byte groups per thread and trip (one trip covers 8192 tokens), all loads of a trip issued
  // before its first store: a spare workgroup is one of only two or four on its CU, so the bytes in flight per
  // workgroup are what sets the rate
  constexpr int NG = 8;
  for (long long c = v0 + tid; c < v1; c += 256 * NG) {
    float4 zv[NG], w[NG];
#pragma unroll
    for (int q = 0; q < NG; ++q) {
      const long long cc = c + 256 * q < v1 ? c + 256 * q : c;
      zv[q] = ((const float4*)z)[cc];
      w[q] = z0 ? ((const float4*)z0)[cc] : zero4;
    }
#pragma unroll
    for (int q = 0; q < NG; ++q) {
      const long long cc = c + 256 * q;
      if (cc >= v1) break;
      float4 av = zero4;
      pruned_elem(zv[q].x, av.x, 2, alpha, beta, 1, r0, r1);
      pruned_elem(zv[q].y, av.y, 2, alpha, beta, 1, r0, r1);
      pruned_elem(zv[q].z, av.z, 2, alpha, beta, 1, r0, r1);
      pruned_elem(zv[q].w, av.w, 2, alpha, beta, 1, r0, r1);
      ((float4*)a)[cc] = av;
      ((float4*)z)[cc] = zv[q];
      sums(av.x, zv[q].x, w[q].x);
      sums(av.y, zv[q].y, w[q].y);
      sums(av.z, zv[q].z, w[q].z);
      sums(av.w, zv[q].w, w[q].w);
    }
  }
  if (last) {
    for (long long t = ((job.T >> 2) << 2) + tid; t < job.T; t += 256) {
      float zv = z[t], av = 0.0f;
      pruned_elem(zv, av, 2, alpha, beta, 1, r0, r1);
      a[t] = av;
      z[t] = zv;
      sums(av, zv, z0 ? z0[t] : 0.0f);
    }
  }
  for (int o = 32; o > 0; o >>= 1) {
    r0 += __shfl_down(r0, o, 64);
    r1 += __shfl_down(r1, o, 64);
    sg += __shfl_down(sg, o, 64);
    se += __shfl_down(se, o, 64);
    su += __shfl_down(su, o, 64);
    sv += __shfl_down(sv, o, 64);
  }
  if ((tid & 63) == 0) {
    double* w = cj_sh[tid >> 6];
    w[0] = r0; w[1] = r1; w[2] = sg; w[3] = se; w[4] = su; w[5] = sv;
  }
  __syncthreads();
  if (tid < 6) job.partial[(unsigned long long)u * 6 + tid] = cj_sh[0][tid] + cj_sh[1][tid] + cj_sh[2][tid] + cj_sh[3][tid];
  __syncthreads();
}

// A spare workgroup (256 threads, all of them call this) takes up to job.take units and returns.
__device__ __forceinline__ void cojob_help(const CoJob& job) {
  __shared__ unsigned int cj_u0;
  if (!job.ticket) return;
  if (threadIdx.x == 0) cj_u0 = atomicAdd(job.ticket, (unsigned int)job.take);
  __syncthreads();
  const unsigned int u0 = cj_u0;
  for (int i = 0; i < job.take; ++i) {
    if (u0 + i >= job.units) break;
    cojob_unit(job, u0 + i);
  }
}

}  // namespace strp
