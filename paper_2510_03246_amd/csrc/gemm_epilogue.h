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

// Epilogue of one 32 x 32 tile of outputs, 16 values per lane (passed by value so the accumulators never need an address).
// Register e of lane l is output row m_tile + tile_rowoff<LAYOUT>(e / 4) + (e % 4), column n (m_tile and n include the
// lane's share: lane % 32 selects the column, lane / 32 the row half).  LAYOUT 0 is the accumulator of one 32x32
// matrix-core instruction (row offsets 0, 8, 16, 24; the upper half wavefront 4 rows further down); LAYOUT 1 is what
// four 16x16 accumulators become after exchanging quarter wavefronts between horizontal neighbours (row offsets 0, 4,
// 16, 20; the upper half wavefront 8 rows further down), see EpilogueWalk16.
//
// Loads are branch-free and come first: rows and the column are clamped into range so that every address is
// valid, and the 16 loads of the tile are issued back to back.  (A predicated load costs a wait per element, and
// loads interleaved with the stores would serialise one memory round trip per element, since the compiler cannot
// prove that the state tensors do not overlap.)  Only the stores are predicated.  Offsets are recomputed where
// they are used rather than kept: 16 64-bit offsets next to 128 accumulators would spill.
// ZWRITE (EPI_ZUPD only): true = apply the z rule and store Z, false = only accumulate the objective sums.
// Row sums (AUPD / ZUPD with p.rs_out): rs0 / rs1 collect, per element position e of this lane, the scoring terms of the
// values just produced (AUPD: a^2 and, with p.rs_z0, a relu(z0); ZUPD: z0 z); they run over the column tiles of the
// wavefront and are reduced over the lanes by rowsum_flush.
template <int LAYOUT>
__device__ __forceinline__ constexpr int tile_rowoff(int q) {
  return LAYOUT == 0 ? 8 * q : 16 * (q >> 1) + 4 * (q & 1);
}

template <int EPI, bool ZWRITE, bool EDGE, int LAYOUT = 0>
__device__ __forceinline__ void epilogue_tile(const GemmP& p, const floatx16 a16, float unscale, int m_tile, int n, int split,
                                              const int* rowmap, int m_blk, double& red0, double& red1, float (&rs0)[16],
                                              float (&rs1)[16]) {
  constexpr bool GATHER = (EPI == EPI_AUPD || EPI == EPI_ZUPD);
  const bool rsum = GATHER && ZWRITE && p.rs_out != nullptr;
  const bool rs_z0 = rsum && p.rs_z0 != nullptr;
  const bool ncol = !EDGE || n < p.N;
  const int nc = ncol ? n : p.N - 1;
  int rowid[16];         // GATHER: state row of each element's output row (0 for rows past M)
  if (GATHER) {
#pragma unroll
    for (int e = 0; e < 16; ++e) rowid[e] = rowmap[m_tile + tile_rowoff<LAYOUT>(e >> 2) + (e & 3) - m_blk];   // slice of oidx staged in LDS
  }
  // 32 x 32 -> 64-bit products (one instruction each): rows, leading dimensions and columns all fit 32 bits
  auto offset = [&](int e) -> long long {
    const int m = m_tile + tile_rowoff<LAYOUT>(e >> 2) + (e & 3);
    const unsigned mc = (unsigned)((!EDGE || m < p.M) ? m : p.M - 1);
    unsigned long long o;
    if (EPI == EPI_PARTIAL) o = (unsigned long long)((unsigned)split * (unsigned)p.M + mc) * (unsigned)p.N + (unsigned)nc;
    else if (EPI == EPI_STORE) o = (unsigned long long)mc * (unsigned)p.ldo + (unsigned)nc;
    else if (EPI == EPI_RESID) o = (unsigned long long)mc * (unsigned)p.ldy + (unsigned)nc;
    else if (GATHER) o = (unsigned long long)(unsigned)rowid[e] * (unsigned)p.lda + (unsigned)nc;
    else o = (unsigned long long)mc * (unsigned)p.lda + (unsigned)nc;
    return (long long)o;
  };
  float in0[16];         // RESID: Y, AUPD: Z, ZUPD: A (ZWRITE) or A and, in in1, Z (!ZWRITE)
  float in1[16];
  if (EPI == EPI_RESID || EPI == EPI_AUPD || EPI == EPI_ZUPD) {
    const float* src = EPI == EPI_RESID ? p.Yin : (EPI == EPI_AUPD ? p.Zs : p.As);
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const long long o = offset(e);
      in0[e] = src[o];
      if (EPI == EPI_ZUPD && !ZWRITE) in1[e] = p.Zs[o];
    }
    if (GATHER && ZWRITE && rs_z0) {   // uniform over the grid: a scalar branch around 16 more loads
#pragma unroll
      for (int e = 0; e < 16; ++e) in1[e] = p.rs_z0[offset(e)];
    }
  }
  const float inv_ab = 1.0f / (p.alpha + p.beta);
  float s0 = 0.0f, s1 = 0.0f;   // this tile's share of the reduction sums (16 terms in fp32, then fp64)
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int mq = m_tile + tile_rowoff<LAYOUT>(q);  // rows mq .. mq+3
    float outv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int e = 4 * q + r;
      const bool ok = !EDGE || (ncol && (mq + r) < p.M);
      const float v = a16[e] * unscale;
      outv[r] = 0.0f;
      if (EPI == EPI_PARTIAL) {
        if (ok) p.out[offset(e)] = v;
      } else if (EPI == EPI_STORE) {
        if (ok) p.out[offset(e)] = v;
        outv[r] = ok ? v : 0.0f;
      } else if (EPI == EPI_INITZ) {
        const float a = __builtin_fmaxf(v, 0.0f);
        if (ok) {
          const long long o = offset(e);
          p.Z0s[o] = v;
          p.Zs[o] = v;
          p.As[o] = a;
        }
        outv[r] = ok ? a : 0.0f;
        s0 += ok ? a * a : 0.0f;
      } else if (EPI == EPI_RESID) {
        const float rr = ok ? in0[e] - v : 0.0f;
        outv[r] = rr;
        s0 += rr * rr;
      } else if (EPI == EPI_AUPD) {
        const float a = __builtin_fmaxf(in0[e], 0.0f) + v;
        if (ok) p.As[offset(e)] = a;
        outv[r] = ok ? a : 0.0f;
        if (rsum) rs0[e] += ok ? a * a : 0.0f;
        if (rs_z0) rs1[e] += ok ? a * __builtin_fmaxf(in1[e], 0.0f) : 0.0f;
      } else {  // EPI_ZUPD
        const float a = in0[e];
        const float z1 = v;
        float z;
        if (ZWRITE) {
          const float z2 = (p.beta * a + p.alpha * z1) * inv_ab;
          const float cm = __builtin_fminf(z1, 0.0f);
          const float costm = p.beta * a * a + p.alpha * (cm - z1) * (cm - z1);
          const float cp = __builtin_fmaxf(z2, 0.0f);
          const float costp = p.beta * (a - cp) * (a - cp) + p.alpha * (cp - z1) * (cp - z1);
          z = costm < costp ? cm : cp;
          if (ok) p.Zs[offset(e)] = z;
          if (rs_z0) rs0[e] += ok ? in1[e] * z : 0.0f;
        } else {
          z = in1[e];
        }
        const float ra = ok ? a - __builtin_fmaxf(z, 0.0f) : 0.0f;
        const float rz = ok ? z - z1 : 0.0f;
        s0 += ra * ra;
        s1 += rz * rz;
      }
    }
    // optional operand-plane copy of the produced tile (its rows are the contraction axis of the consumer):
    // this lane's four rows are half of one 16-byte chunk; rows past M inside the last chunk are written as zeros
    if ((EPI == EPI_STORE || EPI == EPI_INITZ || EPI == EPI_RESID) && p.k8_hi && ncol && (!EDGE || (mq & ~7) < p.M)) {
      unsigned short h[4], l[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) split_half(outv[r], h[r], l[r]);
      const long long o = ((((long long)(n >> 7) * p.k8_kg + (mq >> 3)) << 7) + (n & 127)) * 8 + (mq & 7);
      *(uint2*)(p.k8_hi + o) = make_uint2(pack2(h[0], h[1]), pack2(h[2], h[3]));
      if (p.k8_lo) *(uint2*)(p.k8_lo + o) = make_uint2(pack2(l[0], l[1]), pack2(l[2], l[3]));
    }
    __builtin_amdgcn_sched_barrier(0);   // bounds the live temporaries to one group of four rows
  }
  red0 += (double)s0;
  red1 += (double)s1;
}

// Sum rs[e] over the 32 lanes of each half wavefront (= the 32 columns of a tile; the caller has already added the
// wavefront's column tiles) and store one value per output row: p.rs_out[(q * slots + slot) * M + row], slot = the
// wavefront's strip of columns (64 in both kernels).  A halving butterfly: each exchange keeps half of the values a lane still holds, so
// 8 + 4 + 2 + 1 + 1 shuffles do what 16 five-step reductions would; a lane ends with position e = (lane / 2) % 16.
// A strip that lies wholly past column N (last block of a ragged N) has no slot and is dropped.
template <int LAYOUT>
__device__ __forceinline__ void rowsum_flush(const GemmP& p, const float (&rs)[16], int q, int m_tile, int slot) {
  const int l5 = threadIdx.x & 31;
  const bool b4 = l5 & 16, b3 = l5 & 8, b2 = l5 & 4, b1 = l5 & 2;
  float v8[8], v4[4], v2[2];
#pragma unroll
  for (int i = 0; i < 8; ++i) v8[i] = (b4 ? rs[8 + i] : rs[i]) + __shfl_xor(b4 ? rs[i] : rs[8 + i], 16, 64);
#pragma unroll
  for (int i = 0; i < 4; ++i) v4[i] = (b3 ? v8[4 + i] : v8[i]) + __shfl_xor(b3 ? v8[i] : v8[4 + i], 8, 64);
#pragma unroll
  for (int i = 0; i < 2; ++i) v2[i] = (b2 ? v4[2 + i] : v4[i]) + __shfl_xor(b2 ? v4[i] : v4[2 + i], 4, 64);
  float v1 = (b1 ? v2[1] : v2[0]) + __shfl_xor(b1 ? v2[0] : v2[1], 2, 64);
  v1 += __shfl_xor(v1, 1, 64);
  const int e = (l5 >> 1) & 15;
  const int row = m_tile + tile_rowoff<LAYOUT>(e >> 2) + (e & 3);
  if (!(l5 & 1) && row < p.M && slot < p.rs_slots) p.rs_out[((long long)q * p.rs_slots + slot) * p.M + row] = v1;
}

// Compile-time walk over the WTM x WTN tiles of a wavefront (constant indices keep the accumulators in registers).
// The scheduling barrier keeps the compiler from hoisting the next tile's loads and offsets over this tile.
template <int EPI, bool ZWRITE, int WTM, int WTN, int IJ>
struct EpilogueWalk {
  static __device__ __forceinline__ void run(const GemmP& p, floatx16 (&acc)[WTM][WTN], float unscale, int mbase, int nbase, int split,
                                             const int* rowmap, int m_blk, double& red0, double& red1, float (&rs0)[16],
                                             float (&rs1)[16]) {
    constexpr bool ROWSUMS = (EPI == EPI_AUPD || EPI == EPI_ZUPD) && ZWRITE;
    if (ROWSUMS && IJ % WTN == 0) {
#pragma unroll
      for (int e = 0; e < 16; ++e) rs0[e] = rs1[e] = 0.0f;
    }
    // interior tiles (the common case, decided per wavefront) skip every bounds predicate
    const int mt = mbase + (IJ / WTN) * 32, nt = nbase + (IJ % WTN) * 32;
    const bool edge = __builtin_amdgcn_readfirstlane(mt) + 32 > p.M || __builtin_amdgcn_readfirstlane(nt) + 32 > p.N;
    if (edge) epilogue_tile<EPI, ZWRITE, true>(p, acc[IJ / WTN][IJ % WTN], unscale, mt, nt, split, rowmap, m_blk, red0, red1, rs0, rs1);
    else epilogue_tile<EPI, ZWRITE, false>(p, acc[IJ / WTN][IJ % WTN], unscale, mt, nt, split, rowmap, m_blk, red0, red1, rs0, rs1);
    if (ROWSUMS && IJ % WTN == WTN - 1 && p.rs_out) {
      if (EPI == EPI_AUPD) {
        rowsum_flush<0>(p, rs0, 0, mt, nbase / (32 * WTN));
        if (p.rs_z0) rowsum_flush<0>(p, rs1, 1, mt, nbase / (32 * WTN));
      } else if (p.rs_z0) {
        rowsum_flush<0>(p, rs0, 0, mt, nbase / (32 * WTN));
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    EpilogueWalk<EPI, ZWRITE, WTM, WTN, IJ + 1>::run(p, acc, unscale, mbase, nbase, split, rowmap, m_blk, red0, red1, rs0, rs1);
  }
};
template <int EPI, bool ZWRITE, int WTM, int WTN>
struct EpilogueWalk<EPI, ZWRITE, WTM, WTN, WTM * WTN> {
  static __device__ __forceinline__ void run(const GemmP&, floatx16 (&)[WTM][WTN], float, int, int, int, const int*, int, double&,
                                             double&, float (&)[16], float (&)[16]) {}
};
template <int EPI, int WTM, int WTN>
__device__ __forceinline__ void epilogue(const GemmP& p, floatx16 (&acc)[WTM][WTN], float unscale, int mbase, int nbase, int split,
                                         const int* rowmap, int m_blk, double& red0, double& red1) {
  float rs0[16], rs1[16];
  if (EPI == EPI_ZUPD && !p.write_out)
    EpilogueWalk<EPI, false, WTM, WTN, 0>::run(p, acc, unscale, mbase, nbase, split, rowmap, m_blk, red0, red1, rs0, rs1);
  else
    EpilogueWalk<EPI, true, WTM, WTN, 0>::run(p, acc, unscale, mbase, nbase, split, rowmap, m_blk, red0, red1, rs0, rs1);
}

// ---- the same for accumulators of 16x16 matrix-core tiles -------------------------------------------------------------
// Lane l of a 16x16 tile holds rows 4 (l / 16) + r (r < 4) of column l % 16, so a store instruction would write 64-byte
// pieces of four rows.  v_permlane16_swap exchanges the odd quarter wavefronts of one register with the even ones of
// another: applied to the same register of two horizontally adjacent tiles it yields two registers in which lanes
// 0-31 hold 32 consecutive columns of one row and lanes 32-63 those of the row 8 further down -- 128-byte pieces, the
// column-per-lane arrangement of epilogue_tile.  Two such tile pairs stacked vertically are one 32 x 32 tile in LAYOUT 1.
typedef float floatx4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void quarter_swap(float a, float b, float& x, float& y) {
  const auto r = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned int, a), __builtin_bit_cast(unsigned int, b), false, false);
  x = __builtin_bit_cast(float, (unsigned int)r[0]);
  y = __builtin_bit_cast(float, (unsigned int)r[1]);
}

// acc[8][4]: the wavefront's 128 x 64 outputs as 8 x 4 tiles of 16 x 16.  IJ walks its 4 x 2 tiles of 32 x 32.
template <int EPI, bool ZWRITE, int IJ>
struct EpilogueWalk16 {
  static __device__ __forceinline__ void run(const GemmP& p, floatx4 (&acc)[8][4], float unscale, int mbase, int nbase, int split,
                                             const int* rowmap, int m_blk, double& red0, double& red1, float (&rs0)[16],
                                             float (&rs1)[16]) {
    constexpr bool ROWSUMS = (EPI == EPI_AUPD || EPI == EPI_ZUPD) && ZWRITE;
    constexpr int I = IJ / 2, J = IJ % 2;
    if (ROWSUMS && J == 0) {
#pragma unroll
      for (int e = 0; e < 16; ++e) rs0[e] = rs1[e] = 0.0f;
    }
    floatx16 a16;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float x, y;
      quarter_swap(acc[2 * I][2 * J][r], acc[2 * I][2 * J + 1][r], x, y);
      a16[r] = x;
      a16[4 + r] = y;
      quarter_swap(acc[2 * I + 1][2 * J][r], acc[2 * I + 1][2 * J + 1][r], x, y);
      a16[8 + r] = x;
      a16[12 + r] = y;
    }
    const int mt = mbase + 32 * I, nt = nbase + 32 * J;
    const bool edge = __builtin_amdgcn_readfirstlane(mt) + 32 > p.M || __builtin_amdgcn_readfirstlane(nt) + 32 > p.N;
    if (edge) epilogue_tile<EPI, ZWRITE, true, 1>(p, a16, unscale, mt, nt, split, rowmap, m_blk, red0, red1, rs0, rs1);
    else epilogue_tile<EPI, ZWRITE, false, 1>(p, a16, unscale, mt, nt, split, rowmap, m_blk, red0, red1, rs0, rs1);
    if (ROWSUMS && J == 1 && p.rs_out) {
      if (EPI == EPI_AUPD) {
        rowsum_flush<1>(p, rs0, 0, mt, nbase >> 6);
        if (p.rs_z0) rowsum_flush<1>(p, rs1, 1, mt, nbase >> 6);
      } else if (p.rs_z0) {
        rowsum_flush<1>(p, rs0, 0, mt, nbase >> 6);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    EpilogueWalk16<EPI, ZWRITE, IJ + 1>::run(p, acc, unscale, mbase, nbase, split, rowmap, m_blk, red0, red1, rs0, rs1);
  }
};
template <int EPI, bool ZWRITE>
struct EpilogueWalk16<EPI, ZWRITE, 8> {
  static __device__ __forceinline__ void run(const GemmP&, floatx4 (&)[8][4], float, int, int, int, const int*, int, double&, double&,
                                             float (&)[16], float (&)[16]) {}
};
// mbase = first row of the wavefront's tile + 8 (lane / 32), nbase = first column + lane % 32
template <int EPI>
__device__ __forceinline__ void epilogue16(const GemmP& p, floatx4 (&acc)[8][4], float unscale, int mbase, int nbase, int split,
                                           const int* rowmap, int m_blk, double& red0, double& red1) {
  float rs0[16], rs1[16];
  if (EPI == EPI_ZUPD && !p.write_out)
    EpilogueWalk16<EPI, false, 0>::run(p, acc, unscale, mbase, nbase, split, rowmap, m_blk, red0, red1, rs0, rs1);
  else
    EpilogueWalk16<EPI, true, 0>::run(p, acc, unscale, mbase, nbase, split, rowmap, m_blk, red0, red1, rs0, rs1);
}

}  // namespace strp
