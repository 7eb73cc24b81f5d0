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

// Which output tile and K split a block works on.
//
// Blocks are dealt round-robin to the 8 XCDs (block b runs on XCD b % 8) and each XCD keeps 32 blocks of the
// pipelined kernel resident, starting the next of its blocks when one retires.  Each XCD has its own L2, so the
// 32 blocks resident on an XCD should share operand panels: the work list is ordered tile group by tile group
// (gm x gn tiles, all of one K split, then the next split of the same group), and XCD x takes entries
// [256 c + 32 x, 256 c + 32 x + 32) of it in its c-th round.  A group of gm x gn tiles streams gm + gn panels
// instead of 2 gm gn.
// Symmetric products compute the lower triangle of an n x n tile grid; it is folded into a rectangle of
// ceil(n/2) x (2 ceil(n/2) + 1) tiles (row r holds triangle row r + h followed by triangle row h - 1 - r) so that
// the same grouping applies.  Returns false for the padding cells of an odd n.
__device__ __forceinline__ bool decode_tile(const GemmP& p, int bid, int nblocks, int& tm, int& tn, int& split) {
  const int full = nblocks & ~255;
  int q = bid;
  if (bid < full) {
    const int x = bid & 7, j = bid >> 3;
    q = ((j >> 5) << 8) + (x << 5) + (j & 31);
  }
  const int TM = p.gridM, TN = p.gridN;
  const int row_items = p.gm * TN * p.splits;           // work items of a full row of groups
  const int gi = q / row_items;
  int r = q - gi * row_items;
  const int hm = (TM - gi * p.gm) < p.gm ? (TM - gi * p.gm) : p.gm;
  // rows of groups above the last one are full, the last one has hm tile rows
  const int col_items = hm * p.gn * p.splits;
  const int gj = r / col_items;
  r -= gj * col_items;
  const int hn = (TN - gj * p.gn) < p.gn ? (TN - gj * p.gn) : p.gn;
  split = r / (hm * hn);
  r -= split * hm * hn;
  const int cc = r / hm;
  int a = gi * p.gm + (r - cc * hm), b = gj * p.gn + cc;
  if (p.triangle) {
    const int h = TM;                                   // = ceil(tilesM / 2)
    if (b <= a + h) { a += h; }
    else { b -= a + h + 1; a = h - 1 - a; }
    if (a >= p.tilesM) return false;
  }
  tm = a; tn = b;
  return true;
}

// Epilogue of one 32x32 accumulator tile (passed by value so the accumulators never need an address).
// Register e of lane l is output row m_tile + 8 (e / 4) + (e % 4), column n  (m_tile, n include the lane's share).
// Three phases per tile - row offsets, then every load the tile needs, then arithmetic and stores - so that the
// loads of a tile are in flight together (interleaving them with the stores would serialise one memory round trip
// per element: the compiler cannot prove that the state tensors do not overlap).
template <int EPI>
__device__ __forceinline__ void epilogue_tile(const GemmP& p, const floatx16 a16, float unscale, int m_tile, int n, int split,
                                              const int* rowmap, int m_blk, double& red0, double& red1) {
  const float ab = p.alpha + p.beta;
  const bool ncol = n < p.N;
  long long off[16];     // element offset of (row, n) in the tensor this epilogue reads / writes
  float in0[16];         // RESID: Y, AUPD: Z, ZUPD: A
  float in1[16];         // ZUPD without write-back: Z
  constexpr bool GATHER = (EPI == EPI_AUPD || EPI == EPI_ZUPD);
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int m = m_tile + 8 * (e >> 2) + (e & 3);
    const bool ok = ncol && m < p.M;
    long long row = m;
    if (GATHER) row = ok ? (long long)rowmap[m - m_blk] : 0;   // the block's slice of oidx, staged in LDS by the kernel
    if (EPI == EPI_PARTIAL) off[e] = ((long long)split * p.M + m) * p.N + n;
    else if (EPI == EPI_STORE) off[e] = (long long)m * p.ldo + n;
    else if (EPI == EPI_RESID) off[e] = (long long)m * p.ldy + n;
    else off[e] = row * p.lda + n;
  }
  if (EPI == EPI_RESID || EPI == EPI_AUPD || EPI == EPI_ZUPD) {
    const float* src = EPI == EPI_RESID ? p.Yin : (EPI == EPI_AUPD ? p.Zs : p.As);
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int m = m_tile + 8 * (e >> 2) + (e & 3);
      const bool ok = ncol && m < p.M;
      in0[e] = ok ? src[off[e]] : 0.0f;
      if (EPI == EPI_ZUPD) in1[e] = (ok && !p.write_out) ? p.Zs[off[e]] : 0.0f;
    }
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int mq = m_tile + 8 * q;  // rows mq .. mq+3
    float outv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int e = 4 * q + r;
      const int m = mq + r;
      const float v = a16[e] * unscale;
      outv[r] = 0.0f;
      if (m >= p.M || !ncol) continue;
      if (EPI == EPI_PARTIAL) {
        p.out[off[e]] = v;
      } else if (EPI == EPI_STORE) {
        p.out[off[e]] = v;
        outv[r] = v;
      } else if (EPI == EPI_INITZ) {
        const float a = __builtin_fmaxf(v, 0.0f);
        p.Z0s[off[e]] = v;
        p.Zs[off[e]] = v;
        p.As[off[e]] = a;
        outv[r] = a;
        red0 += (double)a * (double)a;
      } else if (EPI == EPI_RESID) {
        const float rr = in0[e] - v;
        outv[r] = rr;
        red0 += (double)rr * (double)rr;
      } else if (EPI == EPI_AUPD) {
        const float a = __builtin_fmaxf(in0[e], 0.0f) + v;
        p.As[off[e]] = a;
        outv[r] = a;
      } else {  // EPI_ZUPD
        const float a = in0[e];
        const float z1 = v;
        float z;
        if (p.write_out) {
          const float z2 = (p.beta * a + p.alpha * z1) / ab;
          const float cm = __builtin_fminf(z1, 0.0f);
          const float costm = p.beta * a * a + p.alpha * (cm - z1) * (cm - z1);
          const float cp = __builtin_fmaxf(z2, 0.0f);
          const float costp = p.beta * (a - cp) * (a - cp) + p.alpha * (cp - z1) * (cp - z1);
          z = costm < costp ? cm : cp;
          p.Zs[off[e]] = z;
        } else {
          z = in1[e];
        }
        const float ra = a - __builtin_fmaxf(z, 0.0f);
        const float rz = z - z1;
        red0 += (double)ra * (double)ra;
        red1 += (double)rz * (double)rz;
      }
    }
    // optional operand-plane copy of the produced tile (its rows are the contraction axis of the consumer):
    // this lane's four rows are half of one 16-byte chunk; rows past M inside the last chunk are written as zeros
    if ((EPI == EPI_STORE || EPI == EPI_INITZ || EPI == EPI_RESID || EPI == EPI_AUPD) && p.k8_hi && ncol && (mq & ~7) < p.M) {
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
                                             const int* rowmap, int m_blk, double& red0, double& red1) {
    epilogue_tile<EPI>(p, acc[IJ / WTN][IJ % WTN], unscale, mbase + (IJ / WTN) * 32, nbase + (IJ % WTN) * 32, split, rowmap, m_blk,
                       red0, red1);
    EpilogueWalk<EPI, WTM, WTN, IJ + 1>::run(p, acc, unscale, mbase, nbase, split, rowmap, m_blk, red0, red1);
  }
};
template <int EPI, int WTM, int WTN>
struct EpilogueWalk<EPI, WTM, WTN, WTM * WTN> {
  static __device__ __forceinline__ void run(const GemmP&, floatx16 (&)[WTM][WTN], float, int, int, int, const int*, int, double&, double&) {}
};
template <int EPI, int WTM, int WTN>
__device__ __forceinline__ void epilogue(const GemmP& p, floatx16 (&acc)[WTM][WTN], float unscale, int mbase, int nbase, int split,
                                         const int* rowmap, int m_blk, double& red0, double& red1) {
  EpilogueWalk<EPI, WTM, WTN, 0>::run(p, acc, unscale, mbase, nbase, split, rowmap, m_blk, red0, red1);
}

}  // namespace strp
