// Shared device code of the MFMA GEMM kernels: fp16 split helpers and the fused epilogues.
#pragma once

#include "strp_internal.h"

namespace strp {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ unsigned short half_bits(float x) {
  _Float16 h = (_Float16)x;
  return __builtin_bit_cast(unsigned short, h);
}
__device__ __forceinline__ float clamp_half_range(float x) {
  return __builtin_fminf(__builtin_fmaxf(x, -65504.0f), 65504.0f);
}
__device__ __forceinline__ void split_half(float x, unsigned short& hi, unsigned short& lo) {
  x = clamp_half_range(x);
  _Float16 h = (_Float16)x;
  hi = __builtin_bit_cast(unsigned short, h);
  lo = half_bits(x - (float)h);
}
__device__ __forceinline__ unsigned int pack2(unsigned short a, unsigned short b) {
  return (unsigned int)a | ((unsigned int)b << 16);
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  return v;
}

// Epilogue of one 32x32 accumulator tile (passed by value so the accumulators never need an address).
// Register e of lane l is output row m_tile + 8 (e / 4) + (e % 4), column n  (m_tile, n include the lane's share).
template <int EPI>
__device__ __forceinline__ void epilogue_tile(const GemmP& p, const floatx16 a16, float unscale, int m_tile, int n, int split,
                                              double& red0, double& red1) {
  const float ab = p.alpha + p.beta;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int mq = m_tile + 8 * q;  // rows mq .. mq+3
    float outv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int m = mq + r;
      const float v = a16[4 * q + r] * unscale;
      outv[r] = 0.0f;
      if (m >= p.M || n >= p.N) continue;
      if (EPI == EPI_PARTIAL) {
        p.out[((long long)split * p.M + m) * p.N + n] = v;
      } else if (EPI == EPI_STORE) {
        p.out[(long long)m * p.ldo + n] = v;
        outv[r] = v;
      } else if (EPI == EPI_INITZ) {
        const long long o = (long long)m * p.lda + n;
        const float a = __builtin_fmaxf(v, 0.0f);
        p.Z0s[o] = v;
        p.Zs[o] = v;
        p.As[o] = a;
        outv[r] = a;
        red0 += (double)a * (double)a;
      } else if (EPI == EPI_RESID) {
        const float rr = p.Yin[(long long)m * p.ldy + n] - v;
        outv[r] = rr;
        red0 += (double)rr * (double)rr;
      } else if (EPI == EPI_AUPD) {
        const long long o = (long long)p.oidx[m] * p.lda + n;
        const float a = __builtin_fmaxf(p.Zs[o], 0.0f) + v;
        p.As[o] = a;
        outv[r] = a;
      } else {  // EPI_ZUPD
        const long long o = (long long)p.oidx[m] * p.lda + n;
        const float a = p.As[o];
        const float z1 = v;
        float z;
        if (p.write_out) {
          const float z2 = (p.beta * a + p.alpha * z1) / ab;
          const float cm = __builtin_fminf(z1, 0.0f);
          const float costm = p.beta * a * a + p.alpha * (cm - z1) * (cm - z1);
          const float cp = __builtin_fmaxf(z2, 0.0f);
          const float costp = p.beta * (a - cp) * (a - cp) + p.alpha * (cp - z1) * (cp - z1);
          z = costm < costp ? cm : cp;
          p.Zs[o] = z;
        } else {
          z = p.Zs[o];
        }
        const float ra = a - __builtin_fmaxf(z, 0.0f);
        const float rz = z - z1;
        red0 += (double)ra * (double)ra;
        red1 += (double)rz * (double)rz;
      }
    }
    // optional operand-plane copy of the produced tile (its rows are the contraction axis of the consumer):
    // this lane's four rows are half of one 16-byte chunk; rows past M inside the last chunk are written as zeros
    if ((EPI == EPI_STORE || EPI == EPI_INITZ || EPI == EPI_RESID || EPI == EPI_AUPD) && p.k8_hi && n < p.N && (mq & ~7) < p.M) {
      unsigned short h[4], l[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) split_half(outv[r], h[r], l[r]);
      const long long o = ((((long long)(n >> 7) * p.k8_kg + (mq >> 3)) << 7) + (n & 127)) * 8 + (mq & 7);
      *(uint2*)(p.k8_hi + o) = make_uint2(pack2(h[0], h[1]), pack2(h[2], h[3]));
      if (p.k8_lo) *(uint2*)(p.k8_lo + o) = make_uint2(pack2(l[0], l[1]), pack2(l[2], l[3]));
    }
  }
}

// Compile-time walk over the WTM x WTN tiles of a wavefront (constant indices keep the accumulators in registers).
template <int EPI, int WTM, int WTN, int IJ>
struct EpilogueWalk {
  static __device__ __forceinline__ void run(const GemmP& p, floatx16 (&acc)[WTM][WTN], float unscale, int mbase, int nbase, int split,
                                             double& red0, double& red1) {
    epilogue_tile<EPI>(p, acc[IJ / WTN][IJ % WTN], unscale, mbase + (IJ / WTN) * 32, nbase + (IJ % WTN) * 32, split, red0, red1);
    EpilogueWalk<EPI, WTM, WTN, IJ + 1>::run(p, acc, unscale, mbase, nbase, split, red0, red1);
  }
};
template <int EPI, int WTM, int WTN>
struct EpilogueWalk<EPI, WTM, WTN, WTM * WTN> {
  static __device__ __forceinline__ void run(const GemmP&, floatx16 (&)[WTM][WTN], float, int, int, int, double&, double&) {}
};
template <int EPI, int WTM, int WTN>
__device__ __forceinline__ void epilogue(const GemmP& p, floatx16 (&acc)[WTM][WTN], float unscale, int mbase, int nbase, int split,
                                         double& red0, double& red1) {
  EpilogueWalk<EPI, WTM, WTN, 0>::run(p, acc, unscale, mbase, nbase, split, red0, red1);
}

}  // namespace strp
