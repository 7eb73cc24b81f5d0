// MFMA GEMM family for gfx950 on 16-bit operand planes: 128x128 block tiles, four wavefronts of 64x64,
// v_mfma_f32_32x32x16 matrix-core instructions, LDS-staged tiles, fp32 accumulation.
//
// fp32 quantities (ADMM auxiliaries, refitted weights, targets) are kept for the matrix cores as TWO
// fp16 planes, x*scale = hi + lo with hi = fp16(x*scale), lo = fp16(x*scale - hi) (fp16 subnormals are
// honoured by the f16 MFMA, so lo is exact to 2^-25 absolute).  A product of two split operands runs
// the three leading passes hi*hi + hi*lo + lo*hi into ONE fp32 accumulator (the dropped lo*lo term is
// ~2^-22 relative); a bf16 input is exact in a single fp16 plane.  The planes are written once by the
// split kernels below (or by a producing epilogue) instead of being re-converted by every tile that
// reads them.  Two memory forms share the MFMA core:
//   token-contraction ("NT"):  C[m,n] = sum_t P[m,t] Q[n,t]   both operands ROW planes [row][t]
//   token-parallel   ("NN"):  C[m,t] = sum_k P[m,k] Q[k,t]   Q is a K8 plane [(k/8)][t][8]: the eight
//                              k-values a matrix-core lane needs are one 16-byte chunk, and consecutive
//                              tokens are consecutive chunks (coalesced), so no transpose is needed.
#include "strp_internal.h"

namespace strp {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// Tile shapes (WT = 32x32 MFMA tiles per wavefront per dimension, 2x2 wavefronts per block):
//   WT = 2: 128x128 block, K tile 64, two blocks per CU   (small problems)
//   WT = 4: 256x256 block, K tile 32, one block per CU    (halves the L2->CU traffic per flop)
template <int WT>
struct Tile {
  static constexpr int BM = 64 * WT, BN = 64 * WT;
  static constexpr int BK = WT == 2 ? 64 : 32;
  static constexpr int LDK = BK + 8;               // LDS row pitch in 16-bit elements (conflict-free b128 reads)
  static constexpr int CPR = BK / 8;               // 16-byte chunks per row
  static constexpr int NCH = BM * CPR / 256;       // chunks per thread per plane per K tile (= 4)
  static constexpr int RSTEP = 256 / CPR;          // row distance between a thread's chunks (ROW loader)
  static constexpr int KGS = 256 / BN;             // k groups covered by one pass of the block (K8 loader)
};

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

// ROW plane tile: [128 rows][64 k]; thread owns rows (tid>>3) + 32 i and the 8-element chunk tid&7.
// Loads are unconditional (row clamped, k clamped to the last valid chunk) and zeroed by select, so the
// main loop carries no branches; pointers advance by one K tile per iteration.
template <int NP, int WT>
struct RowLoader {
  static constexpr int NCH = Tile<WT>::NCH, BK = Tile<WT>::BK, LDK = Tile<WT>::LDK, BM = Tile<WT>::BM;
  const unsigned short* rp[NP][NCH];   // points at (row, k + kc) of the tile to load next
  uint4 r[NP][NCH];
  int kc, row0;
  long long kk;                        // k + kc of the tile to load next

  __device__ __forceinline__ void init(const PlaneOp& op, int tile_row0, long long k0) {
    kc = (threadIdx.x % Tile<WT>::CPR) * 8;
    row0 = threadIdx.x / Tile<WT>::CPR;
    kk = k0 + kc;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int row = tile_row0 + row0 + Tile<WT>::RSTEP * i;
      row = row < op.rows ? row : op.rows - 1;
      rp[0][i] = op.hi + (long long)row * op.ld + kk;
      if (NP == 2) rp[NP - 1][i] = op.lo + (long long)row * op.ld + kk;
    }
  }
  __device__ __forceinline__ void load(long long k1) {
    const bool valid = kk < k1;
    const long long back = valid ? 0 : (kk - (k1 - 1)) ;   // step back into the row's valid range
#pragma unroll
    for (int pl = 0; pl < NP; ++pl)
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        uint4 v = *(const uint4*)(rp[pl][i] - ((back + 7) & ~7LL));
        r[pl][i] = valid ? v : make_uint4(0, 0, 0, 0);
        rp[pl][i] += BK;
      }
    if ((k1 & 7) && valid && kk + 8 > k1) {  // ragged end of the contraction: zero the elements past k1
      const int nvalid = (int)(k1 - kk);
#pragma unroll
      for (int pl = 0; pl < NP; ++pl)
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
          unsigned int w[4] = {r[pl][i].x, r[pl][i].y, r[pl][i].z, r[pl][i].w};
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (e >= nvalid) w[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
          r[pl][i] = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
    kk += BK;
  }
  __device__ __forceinline__ void store(unsigned short (*s)[BM * LDK]) const {
#pragma unroll
    for (int pl = 0; pl < NP; ++pl)
#pragma unroll
      for (int i = 0; i < NCH; ++i) *(uint4*)(&s[pl][(row0 + Tile<WT>::RSTEP * i) * LDK + kc]) = r[pl][i];
  }
};

// K8 plane tile: chunk (kg, n) of the tile is the 16 bytes at ((k/8 + kg) * ld + n0 + n) * 8 elements.
// Columns past N read column N-1 (their outputs are never stored); k groups past K read group 0 and are zeroed.
template <int NP, int WT>
struct K8Loader {
  static constexpr int NCH = Tile<WT>::NCH, BK = Tile<WT>::BK, LDK = Tile<WT>::LDK, BN = Tile<WT>::BN, KGS = Tile<WT>::KGS;
  const unsigned short* bp[NP];        // points at chunk (k/8 + kg0, ncol) of the tile to load next
  const unsigned short* safe[NP];
  uint4 r[NP][NCH];
  int n, kg0;
  long long kk, gstep;                 // k of this thread's first chunk in the next tile; elements per KGS groups

  __device__ __forceinline__ void init(const PlaneOp& op, int n0, int N, long long k0) {
    n = threadIdx.x % BN;
    kg0 = threadIdx.x / BN;
    long long ncol = (long long)n0 + n;
    ncol = ncol < N ? ncol : (long long)N - 1;
    kk = k0 + kg0 * 8;
    gstep = KGS * op.ld * 8;
    bp[0] = op.hi + ((kk >> 3) * op.ld + ncol) * 8;
    safe[0] = op.hi + ncol * 8;
    if (NP == 2) {
      bp[NP - 1] = op.lo + ((kk >> 3) * op.ld + ncol) * 8;
      safe[NP - 1] = op.lo + ncol * 8;
    }
  }
  __device__ __forceinline__ void load(long long k1) {
#pragma unroll
    for (int pl = 0; pl < NP; ++pl) {
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const bool valid = kk + 8 * KGS * i < k1;
        const unsigned short* src = valid ? bp[pl] + i * gstep : safe[pl];
        uint4 v = *(const uint4*)src;
        r[pl][i] = valid ? v : make_uint4(0, 0, 0, 0);
      }
      bp[pl] += NCH * gstep;
    }
    kk += BK;
  }
  __device__ __forceinline__ void store(unsigned short (*s)[BN * LDK]) const {
#pragma unroll
    for (int pl = 0; pl < NP; ++pl)
#pragma unroll
      for (int i = 0; i < NCH; ++i) *(uint4*)(&s[pl][n * LDK + (kg0 + KGS * i) * 8]) = r[pl][i];
  }
};

template <bool BF>
__device__ __forceinline__ floatx16 mma(uint4 a, uint4 b, floatx16 c) {
  if (BF) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
  }
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
        p.As[o] = __builtin_fmaxf(p.Zs[o], 0.0f) + v;
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
    // optional K8-plane copy of the produced tile (its rows are the k axis of the consumer):
    // this lane's four rows are half of one 16-byte chunk
    if ((EPI == EPI_STORE || EPI == EPI_INITZ || EPI == EPI_RESID) && p.k8_hi && n < p.N && mq < p.M) {
      unsigned short h[4], l[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) split_half(outv[r], h[r], l[r]);
      const long long o = ((long long)(mq >> 3) * p.k8_ld + n) * 8 + (mq & 7);
      *(uint2*)(p.k8_hi + o) = make_uint2(pack2(h[0], h[1]), pack2(h[2], h[3]));
      if (p.k8_lo) *(uint2*)(p.k8_lo + o) = make_uint2(pack2(l[0], l[1]), pack2(l[2], l[3]));
    }
  }
}

// Compile-time walk over the WT x WT tiles of a wavefront (constant indices keep the accumulators in registers).
template <int EPI, int WT, int IJ>
struct EpilogueWalk {
  static __device__ __forceinline__ void run(const GemmP& p, floatx16 (&acc)[WT][WT], float unscale, int mbase, int nbase, int split,
                                             double& red0, double& red1) {
    epilogue_tile<EPI>(p, acc[IJ / WT][IJ % WT], unscale, mbase + (IJ / WT) * 32, nbase + (IJ % WT) * 32, split, red0, red1);
    EpilogueWalk<EPI, WT, IJ + 1>::run(p, acc, unscale, mbase, nbase, split, red0, red1);
  }
};
template <int EPI, int WT>
struct EpilogueWalk<EPI, WT, WT * WT> {
  static __device__ __forceinline__ void run(const GemmP&, floatx16 (&)[WT][WT], float, int, int, int, double&, double&) {}
};
template <int EPI, int WT>
__device__ __forceinline__ void epilogue(const GemmP& p, floatx16 (&acc)[WT][WT], float unscale, int mbase, int nbase, int split,
                                         double& red0, double& red1) {
  EpilogueWalk<EPI, WT, 0>::run(p, acc, unscale, mbase, nbase, split, red0, red1);
}

template <int NPP, int NPQ, bool NN, bool BF, int WT>
__global__ __launch_bounds__(256, WT == 4 ? 1 : 2) void gemm_kernel(const GemmP p) {
  constexpr int BM = Tile<WT>::BM, BN = Tile<WT>::BN, BK = Tile<WT>::BK, LDK = Tile<WT>::LDK, KS = BK / 16;
  __shared__ __attribute__((aligned(16))) unsigned short sP[NPP][BM * LDK];
  __shared__ __attribute__((aligned(16))) unsigned short sQ[NPQ][BN * LDK];
  __shared__ double sred[4][2];

  // ---- which tile, which K range ---------------------------------------------------------
  int bid = blockIdx.x;
  const int split = bid / p.ntiles;
  int t = bid - split * p.ntiles;
  if ((p.ntiles & 7) == 0) t = (t & 7) * (p.ntiles >> 3) + (t >> 3);  // one XCD owns a contiguous tile range
  int tm, tn;
  if (p.triangle) {
    tm = (int)((__builtin_sqrtf(8.0f * (float)t + 1.0f) - 1.0f) * 0.5f);
    while ((tm + 1) * (tm + 2) / 2 <= t) ++tm;
    while (tm * (tm + 1) / 2 > t) --tm;
    tn = t - tm * (tm + 1) / 2;
  } else {
    const int G = WT == 4 ? 4 : 8;
    const int per_group = G * p.tilesN;
    const int grp = t / per_group;
    const int first_m = grp * G;
    const int gsz = (p.tilesM - first_m) < G ? (p.tilesM - first_m) : G;
    const int w = t - grp * per_group;
    tm = first_m + w % gsz;
    tn = w / gsz;
  }
  const int m0 = tm * BM, n0 = tn * BN;
  const long long k0 = (long long)split * p.kchunk;
  const long long k1 = (k0 + p.kchunk < p.K) ? (k0 + p.kchunk) : p.K;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  constexpr int WROWS = 32 * WT;   // rows (and columns) of the output owned by one wavefront

  RowLoader<NPP, WT> lp;
  lp.init(p.P, m0, k0);
  RowLoader<NPQ, WT> lq_row;
  K8Loader<NPQ, WT> lq_k8;
  if (NN) lq_k8.init(p.Q, n0, p.N, k0); else lq_row.init(p.Q, n0, k0);

  floatx16 acc[WT][WT];
#pragma unroll
  for (int i = 0; i < WT; ++i)
#pragma unroll
    for (int j = 0; j < WT; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  // fragment addresses of this lane inside a tile (k step added per use)
  const int offP = (wm * WROWS + (lane & 31)) * LDK + 8 * (lane >> 5);
  const int offQ = (wn * WROWS + (lane & 31)) * LDK + 8 * (lane >> 5);
  struct Frags { uint4 ph[WT], pl[WT], qh[WT], ql[WT]; };
  auto read_frags = [&](Frags& f, int ks) {
#pragma unroll
    for (int i = 0; i < WT; ++i) {
      const int off = offP + i * 32 * LDK + ks * 16;
      f.ph[i] = *(const uint4*)(&sP[0][off]);
      if (NPP == 2) f.pl[i] = *(const uint4*)(&sP[NPP - 1][off]);
    }
#pragma unroll
    for (int j = 0; j < WT; ++j) {
      const int off = offQ + j * 32 * LDK + ks * 16;
      f.qh[j] = *(const uint4*)(&sQ[0][off]);
      if (NPQ == 2) f.ql[j] = *(const uint4*)(&sQ[NPQ - 1][off]);
    }
  };
  auto run_mfma = [&](const Frags& f) {
    if (NPQ == 2) {
#pragma unroll
      for (int i = 0; i < WT; ++i)
#pragma unroll
        for (int j = 0; j < WT; ++j) acc[i][j] = mma<BF>(f.ph[i], f.ql[j], acc[i][j]);
    }
    if (NPP == 2) {
#pragma unroll
      for (int i = 0; i < WT; ++i)
#pragma unroll
        for (int j = 0; j < WT; ++j) acc[i][j] = mma<BF>(f.pl[i], f.qh[j], acc[i][j]);
    }
#pragma unroll
    for (int i = 0; i < WT; ++i)
#pragma unroll
      for (int j = 0; j < WT; ++j) acc[i][j] = mma<BF>(f.ph[i], f.qh[j], acc[i][j]);
  };

  if (k0 < k1) {
    lp.load(k1);
    if (NN) lq_k8.load(k1); else lq_row.load(k1);
  }
  for (long long k = k0; k < k1; k += BK) {
    lp.store(sP);
    if (NN) lq_k8.store(sQ); else lq_row.store(sQ);
    __syncthreads();
    if (k + BK < k1) {  // next tile's global loads fly during the matrix work
      lp.load(k1);
      if (NN) lq_k8.load(k1); else lq_row.load(k1);
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
    case EPI_PARTIAL: epilogue<EPI_PARTIAL, WT>(p, acc, unscale, mbase, nbase, split, red0, red1); break;
    case EPI_STORE: epilogue<EPI_STORE, WT>(p, acc, unscale, mbase, nbase, split, red0, red1); break;
    case EPI_INITZ: epilogue<EPI_INITZ, WT>(p, acc, unscale, mbase, nbase, split, red0, red1); break;
    case EPI_RESID: epilogue<EPI_RESID, WT>(p, acc, unscale, mbase, nbase, split, red0, red1); break;
    case EPI_AUPD: epilogue<EPI_AUPD, WT>(p, acc, unscale, mbase, nbase, split, red0, red1); break;
    default: epilogue<EPI_ZUPD, WT>(p, acc, unscale, mbase, nbase, split, red0, red1); break;
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
void gemm_plan_tiles(GemmP& p, bool nn, int want_splits) {
  // 256x256 tiles when they still give every CU a block; otherwise 128x128
  {
    const long long t4m = (p.M + 255) / 256, t4n = (p.N + 255) / 256;
    const long long n4 = p.triangle ? t4m * (t4m + 1) / 2 : t4m * t4n;
    p.wt = (p.force_wt == 4 && p.M >= 256 && p.N >= 256 && n4 * (want_splits > 1 ? want_splits : 1) >= 256) ? 4 : 2;
  }
  const int BM = 64 * p.wt, BN = 64 * p.wt, BK = p.wt == 2 ? 64 : 32;
  p.tilesM = (p.M + BM - 1) / BM;
  p.tilesN = (p.N + BN - 1) / BN;
  p.ntiles = p.triangle ? p.tilesM * (p.tilesM + 1) / 2 : p.tilesM * p.tilesN;
  if (nn || want_splits <= 1) {
    p.splits = 1;
    p.kchunk = ((p.K + BK - 1) / BK) * BK;
  } else {
    long long chunk = (p.K + want_splits - 1) / want_splits;
    chunk = ((chunk + BK - 1) / BK) * BK;
    p.kchunk = chunk;
    p.splits = (int)((p.K + chunk - 1) / chunk);
  }
}

int gemm_grid_blocks(const GemmP& p) { return p.ntiles * p.splits; }

template <int NPP, int NPQ, bool NN, bool BF>
static void launch_one(strp_ctx* ctx, const GemmP& p) {
  if (p.wt == 4)
    hipLaunchKernelGGL((gemm_kernel<NPP, NPQ, NN, BF, 4>), dim3(gemm_grid_blocks(p)), dim3(256), 0, ctx->stream, p);
  else
    hipLaunchKernelGGL((gemm_kernel<NPP, NPQ, NN, BF, 2>), dim3(gemm_grid_blocks(p)), dim3(256), 0, ctx->stream, p);
}

strp_status launch_gemm(strp_ctx* ctx, GemmP& p, bool nn, bool bf16) {
  if (p.M <= 0 || p.N <= 0 || p.K <= 0) return fail(ctx, STRP_EINVAL, "gemm: empty shape");
  if (p.ntiles <= 0 || p.splits <= 0 || (p.wt != 2 && p.wt != 4)) return fail(ctx, STRP_EINVAL, "gemm: tiles not planned");
  if (!p.P.hi || !p.Q.hi) return fail(ctx, STRP_EINVAL, "gemm: null operand plane");
  if ((p.M % 8) && p.k8_hi) return fail(ctx, STRP_EINVAL, "gemm: K8 output needs M %% 8 == 0");
  const int npp = p.P.lo ? 2 : 1, npq = p.Q.lo ? 2 : 1;
  if (bf16 && (npp != 1 || npq != 1 || nn)) return fail(ctx, STRP_EINVAL, "gemm: bf16 cores take single ROW planes only");
  static const char* const epi_names[] = {"partial", "store", "initz", "resid", "aupd", "zupd"};
  static char names[2][2][3][3][6][40];
  char* name = names[nn ? 1 : 0][bf16 ? 1 : 0][npp][npq][p.epi];
  if (!name[0]) snprintf(name, 40, "gemm_%s_%s%dx%d_%s", nn ? "nn" : "nt", bf16 ? "bf" : "h", npp, npq, epi_names[p.epi]);
  const double mn = p.triangle ? 0.5 * (double)p.M * ((double)p.M + 1.0) : (double)p.M * (double)p.N;
  static const double out_words[] = {1.0, 1.0, 3.0, 2.0, 2.0, 2.0};
  double obytes = 4.0 * out_words[p.epi] * (double)p.M * (double)p.N * (p.epi == EPI_PARTIAL ? (double)p.splits : 1.0);
  if (p.epi == EPI_RESID) obytes *= 0.5;
  if (p.k8_hi) obytes += (p.k8_lo ? 4.0 : 2.0) * (double)p.M * (double)p.N;
  const double ibytes = p.triangle ? 2.0 * npp * (double)p.M * (double)p.K
                                   : 2.0 * npp * (double)p.M * (double)p.K + 2.0 * npq * (double)p.N * (double)p.K;
  ProfScope ps(ctx, name, 2.0 * mn * (double)p.K, ibytes + obytes);
  const int key = (nn ? 100 : 0) + npp * 10 + npq;
  if (bf16) {
    launch_one<1, 1, false, true>(ctx, p);
  } else {
    switch (key) {
      case 11: launch_one<1, 1, false, false>(ctx, p); break;
      case 12: launch_one<1, 2, false, false>(ctx, p); break;
      case 21: launch_one<2, 1, false, false>(ctx, p); break;
      case 22: launch_one<2, 2, false, false>(ctx, p); break;
      case 111: launch_one<1, 1, true, false>(ctx, p); break;
      case 112: launch_one<1, 2, true, false>(ctx, p); break;
      case 121: launch_one<2, 1, true, false>(ctx, p); break;
      case 122: launch_one<2, 2, true, false>(ctx, p); break;
      default: return fail(ctx, STRP_EINVAL, "gemm: plane combination %d not built", key);
    }
  }
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

// ---- split-K reduction -----------------------------------------------------------------------
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* part, int splits, int M, int N, int triangle,
                                                           float* outf, long long ldof, double* outd, long long ldod,
                                                           double* diag, int accumulate) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= (long long)M * N) return;
  const int m = (int)(e / N), n = (int)(e % N);
  long long src = e;
  if (triangle && n > m) src = (long long)n * N + m;  // upper half mirrors the computed lower half (exact symmetry)
  double s = 0.0;
  for (int sp = 0; sp < splits; ++sp) s += (double)part[(long long)sp * M * N + src];
  if (outf) {
    float* o = outf + (long long)m * ldof + n;
    *o = accumulate ? (float)((double)*o + s) : (float)s;
  }
  if (outd) outd[(long long)m * ldod + n] = s;
  if (diag && m == n) diag[m] = s;
}

strp_status launch_splitk_reduce(strp_ctx* ctx, const float* part, int splits, int M, int N, int triangle,
                                 float* outf, long long ldof, double* outd, long long ldod, double* diag,
                                 int accumulate) {
  const long long tot = (long long)M * N;
  ProfScope ps(ctx, "splitk_reduce", 0.0, 4.0 * (double)tot * (double)splits + (outf ? 4.0 : 0.0) * tot + (outd ? 8.0 : 0.0) * tot);
  hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, ctx->stream, part,
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

// ---------------------------------------------------------------------------------------------
// split kernels: fp32 / bf16 / fp64 sources -> fp16 planes
// ---------------------------------------------------------------------------------------------
// Activations: a block converts one group of 8 (gathered) rows x 1024 tokens; each thread 8 rows x 4 tokens.
//   ROW planes  [rows8][ld_row]         (token-contiguous; padding columns zero up to ld_row)
//   K8  planes  [(rows8/8)][T][8]       (relu applied when relu_k8 != 0)
// Rows >= rows inside the last group are written as zeros.
template <bool SRC_BF16>
__global__ __launch_bounds__(256) void split_rows_kernel(const void* src, long long lds, const int* idx, int rows, long long T,
                                                         int relu_row, int relu_k8, unsigned short* row_hi, unsigned short* row_lo,
                                                         long long ld_row, unsigned short* k8_hi, unsigned short* k8_lo) {
  const int g = blockIdx.y;
  const long long t0 = ((long long)blockIdx.x * 256 + threadIdx.x) * 4;
  const long long cols = row_hi ? ld_row : T;
  if (t0 >= cols) return;
  float v[8][4];
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const int row = g * 8 + r;
    v[r][0] = v[r][1] = v[r][2] = v[r][3] = 0.0f;
    if (row < rows && t0 < T) {
      const long long srow = idx ? (long long)idx[row] : (long long)row;
      if (SRC_BF16) {
        const uint2 w = *(const uint2*)((const unsigned short*)src + srow * lds + t0);
        v[r][0] = __builtin_bit_cast(float, w.x << 16);
        v[r][1] = __builtin_bit_cast(float, w.x & 0xffff0000u);
        v[r][2] = __builtin_bit_cast(float, w.y << 16);
        v[r][3] = __builtin_bit_cast(float, w.y & 0xffff0000u);
      } else {
        const float4 w = *(const float4*)((const float*)src + srow * lds + t0);
        v[r][0] = w.x; v[r][1] = w.y; v[r][2] = w.z; v[r][3] = w.w;
      }
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (t0 + c >= T) v[r][c] = 0.0f;
    }
  }
  if (row_hi) {
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      unsigned short h[4], l[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) split_half(relu_row ? __builtin_fmaxf(v[r][c], 0.0f) : v[r][c], h[c], l[c]);
      const long long o = (long long)(g * 8 + r) * ld_row + t0;
      *(uint2*)(row_hi + o) = make_uint2(pack2(h[0], h[1]), pack2(h[2], h[3]));
      if (row_lo) *(uint2*)(row_lo + o) = make_uint2(pack2(l[0], l[1]), pack2(l[2], l[3]));
    }
  }
  if (k8_hi) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      if (t0 + c >= T) continue;
      unsigned short h[8], l[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) split_half(relu_k8 ? __builtin_fmaxf(v[r][c], 0.0f) : v[r][c], h[r], l[r]);
      const long long o = ((long long)g * T + t0 + c) * 8;
      *(uint4*)(k8_hi + o) = make_uint4(pack2(h[0], h[1]), pack2(h[2], h[3]), pack2(h[4], h[5]), pack2(h[6], h[7]));
      if (k8_lo) *(uint4*)(k8_lo + o) = make_uint4(pack2(l[0], l[1]), pack2(l[2], l[3]), pack2(l[4], l[5]), pack2(l[6], l[7]));
    }
  }
}

strp_status split_rows(strp_ctx* ctx, const void* src, int src_dtype, long long lds, const int* idx, int rows, long long T,
                       int relu_row, int relu_k8, unsigned short* row_hi, unsigned short* row_lo, long long ld_row,
                       unsigned short* k8_hi, unsigned short* k8_lo) {
  if (rows <= 0 || T <= 0) return fail(ctx, STRP_EINVAL, "split_rows: empty");
  if (row_hi && (ld_row < T || ld_row % 8)) return fail(ctx, STRP_EINVAL, "split_rows: bad plane pitch");
  const long long cols = row_hi ? ld_row : T;
  dim3 grid((unsigned)((cols + 1023) / 1024), (unsigned)((rows + 7) / 8));
  const double es = src_dtype == STRP_BF16 ? 2.0 : 4.0;
  const double wb = (row_hi ? 2.0 : 0.0) + (row_lo ? 2.0 : 0.0) + (k8_hi ? 2.0 : 0.0) + (k8_lo ? 2.0 : 0.0);
  ProfScope ps(ctx, "split_rows", 0.0, (es + wb) * (double)rows * (double)T);
  if (src_dtype == STRP_BF16)
    hipLaunchKernelGGL((split_rows_kernel<true>), grid, dim3(256), 0, ctx->stream, src, lds, idx, rows, T, relu_row, relu_k8,
                       row_hi, row_lo, ld_row, k8_hi, k8_lo);
  else
    hipLaunchKernelGGL((split_rows_kernel<false>), grid, dim3(256), 0, ctx->stream, src, lds, idx, rows, T, relu_row, relu_k8,
                       row_hi, row_lo, ld_row, k8_hi, k8_lo);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

// Small matrices (weights): ROW planes [rows][ldp] of src * scale, zero padded to ldp.  transpose != 0 reads src[c][r].
// scale_dev (device, may be null = 1) is a power of two chosen by weight_scale_kernel.
__device__ __forceinline__ double small_src(const double* s, long long i) { return s[i]; }
__device__ __forceinline__ double small_src(const float* s, long long i) { return (double)s[i]; }
__device__ __forceinline__ double small_src(const unsigned short* s, long long i) {
  return (double)__builtin_bit_cast(float, (unsigned int)s[i] << 16);
}

template <typename TS>
__global__ __launch_bounds__(256) void split_small_kernel(const TS* src, long long lds, int rows, int cols, int transpose,
                                                          const float* scale_dev, unsigned short* hi, unsigned short* lo, long long ldp) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= (long long)rows * ldp) return;
  const int r = (int)(e / ldp), c = (int)(e % ldp);
  double x = 0.0;
  if (c < cols) x = transpose ? small_src(src, (long long)c * lds + r) : small_src(src, (long long)r * lds + c);
  x *= scale_dev ? (double)*scale_dev : 1.0;
  x = fmin(fmax(x, -65504.0), 65504.0);
  const _Float16 h = (_Float16)x;
  hi[e] = __builtin_bit_cast(unsigned short, h);
  if (lo) {
    const _Float16 l = (_Float16)(x - (double)h);
    lo[e] = __builtin_bit_cast(unsigned short, l);
  }
}

strp_status split_small(strp_ctx* ctx, const void* src, int src_kind, long long lds, int rows, int cols, int transpose,
                        const float* scale_dev, unsigned short* hi, unsigned short* lo, long long ldp) {
  const long long tot = (long long)rows * ldp;
  dim3 grid((unsigned)((tot + 255) / 256)), block(256);
  if (src_kind == SRC_F64)
    hipLaunchKernelGGL((split_small_kernel<double>), grid, block, 0, ctx->stream, (const double*)src, lds, rows, cols, transpose, scale_dev, hi, lo, ldp);
  else if (src_kind == SRC_F32)
    hipLaunchKernelGGL((split_small_kernel<float>), grid, block, 0, ctx->stream, (const float*)src, lds, rows, cols, transpose, scale_dev, hi, lo, ldp);
  else
    hipLaunchKernelGGL((split_small_kernel<unsigned short>), grid, block, 0, ctx->stream, (const unsigned short*)src, lds, rows, cols, transpose, scale_dev, hi, lo, ldp);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

// scale = 2^e with max|x| * scale in [2^11, 2^12): keeps fp16 hi far from overflow and lo out of the subnormals.
// Pass 1: grid-wide max of |x| through an integer atomic on the float bits (order-preserving for x >= 0).
template <typename TS>
__global__ __launch_bounds__(256) void absmax_kernel(const TS* src, long long lds, int rows, int cols, unsigned int* slot) {
  float m = 0.0f;
  const long long n = (long long)rows * cols;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256) {
    const long long r = i / cols, c = i % cols;
    m = __builtin_fmaxf(m, __builtin_fabsf((float)small_src(src, r * lds + c)));
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = __builtin_fmaxf(m, __shfl_down(m, o, 64));
  if ((threadIdx.x & 63) == 0 && m > 0.0f) atomicMax(slot, __builtin_bit_cast(unsigned int, m));
}
// Pass 2: the slot (max bits) becomes the scale (float) in place.
__global__ void scale_from_max_kernel(unsigned int* slot) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  const float m = __builtin_bit_cast(float, *slot);
  float s = 1.0f;
  if (m > 0.0f && m < 3.0e38f) {
    int e;
    (void)frexpf(m, &e);        // m = q * 2^e, q in [0.5, 1)
    s = ldexpf(1.0f, 12 - e);   // m * s in [2^11, 2^12)
  }
  *slot = __builtin_bit_cast(unsigned int, s);
}

strp_status weight_scale(strp_ctx* ctx, const void* src, int src_kind, long long lds, int rows, int cols, float* scale_out) {
  STRP_TRY(fill_zero(ctx, scale_out, 4));
  unsigned int* slot = (unsigned int*)scale_out;
  long long blocks = ((long long)rows * cols + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  dim3 grid((unsigned)blocks), block(256);
  if (src_kind == SRC_F64)
    hipLaunchKernelGGL((absmax_kernel<double>), grid, block, 0, ctx->stream, (const double*)src, lds, rows, cols, slot);
  else if (src_kind == SRC_F32)
    hipLaunchKernelGGL((absmax_kernel<float>), grid, block, 0, ctx->stream, (const float*)src, lds, rows, cols, slot);
  else
    hipLaunchKernelGGL((absmax_kernel<unsigned short>), grid, block, 0, ctx->stream, (const unsigned short*)src, lds, rows, cols, slot);
  hipLaunchKernelGGL(scale_from_max_kernel, dim3(1), dim3(1), 0, ctx->stream, slot);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

}  // namespace strp
