// MFMA GEMM family for gfx950: 128x128 block tiles, four wavefronts of 64x64, 32x32x16 matrix-core
// instructions, LDS-staged 16-bit operand tiles, fp32 accumulation.
//
// fp32 operands (ADMM auxiliaries, refitted weights) are fed to the 16-bit matrix cores as a
// two-term fp16 split x = hi + lo/2048 (hi = fp16(x), lo = fp16((x - hi) * 2048)).  The products
// hi*hi go to one accumulator set, hi*lo + lo*hi to a second one that is folded in with weight
// 1/2048 in the epilogue; the dropped lo*lo term is ~2^-22 relative.  bf16 inputs are exact in one
// plane.  Two memory forms share the MFMA core:
//   token-contraction ("NT"):  C[m,n] = sum_t P[m,t] Q[n,t]   (Gram matrices, refit right-hand sides)
//   token-parallel   ("NN"):  C[m,t] = sum_k P[m,k] Q[k,t]   (forward products with fused ADMM updates)
#include "strp_internal.h"

namespace strp {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 32;
constexpr int LDK = BK + 8;  // LDS row pitch in 16-bit elements (80 bytes: conflict-free b128 reads)
constexpr float LO_SCALE = 2048.0f;

__host__ __device__ constexpr bool kind_is_f32(int k) { return k == OP_F32_1 || k == OP_F32_2; }
__host__ __device__ constexpr int kind_planes(int k) { return k == OP_F32_2 ? 2 : 1; }

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
  lo = half_bits((x - (float)h) * LO_SCALE);
}
__device__ __forceinline__ float bf16_bits_to_float(unsigned short b) {
  return __builtin_bit_cast(float, (unsigned int)b << 16);
}
__device__ __forceinline__ unsigned int pack2(unsigned short a, unsigned short b) {
  return (unsigned int)a | ((unsigned int)b << 16);
}

// ---------------------------------------------------------------------------------------------
// K-contiguous operand tile: [128 rows][BK] elements, each thread owns fixed rows and a fixed k chunk
// ---------------------------------------------------------------------------------------------
template <int KIND>
struct KcTile {
  static constexpr bool F32 = kind_is_f32(KIND);
  static constexpr int EW = F32 ? 4 : 8;            // elements per 16-byte chunk
  static constexpr int NCH = F32 ? 4 : 2;           // chunks per thread per tile
  static constexpr int CPR = BK / EW;               // chunks per row
  static constexpr int RSTEP = 256 / CPR;           // row stride between a thread's chunks
  const char* rp[NCH];                              // row base pointers (bytes)
  uint4 r[NCH];
  int kc;                                           // element offset of this thread's chunk in the tile
  int row0;

  __device__ __forceinline__ void init(const Operand& op, int tile_row0) {
    const int tid = threadIdx.x;
    kc = (tid % CPR) * EW;
    row0 = tid / CPR;
    const int es = F32 ? 4 : 2;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int row = tile_row0 + row0 + i * RSTEP;
      row = row < op.rows ? row : op.rows - 1;
      long long srow = op.idx ? (long long)op.idx[row] : (long long)row;
      rp[i] = (const char*)op.ptr + srow * op.ld * es;
    }
  }

  __device__ __forceinline__ void load(long long k, long long k1) {
    const int es = F32 ? 4 : 2;
    const long long kk = k + kc;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      if (kk < k1) {
        r[i] = *(const uint4*)(rp[i] + kk * es);
      } else {
        r[i] = make_uint4(0, 0, 0, 0);
      }
    }
    if (kk < k1 && kk + EW > k1) {  // ragged end of the contraction: zero the elements past k1
      const int valid = (int)(k1 - kk);
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        unsigned int w[4] = {r[i].x, r[i].y, r[i].z, r[i].w};
        if (F32) {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (e >= valid) w[e] = 0u;
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (e >= valid) w[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
        }
        r[i] = make_uint4(w[0], w[1], w[2], w[3]);
      }
    }
  }

  // s0: hi plane (or the only plane), s1: lo plane (OP_F32_2 only)
  __device__ __forceinline__ void store(unsigned short* s0, unsigned short* s1, int relu) const {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int row = row0 + i * RSTEP;
      unsigned short* d0 = s0 + row * LDK + kc;
      if (KIND == OP_BF16) {
        *(uint4*)d0 = r[i];
      } else if (KIND == OP_BF16_H) {
        unsigned int w[4] = {r[i].x, r[i].y, r[i].z, r[i].w};
        unsigned int o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float a = clamp_half_range(bf16_bits_to_float((unsigned short)(w[e] & 0xffffu)));
          float b = clamp_half_range(bf16_bits_to_float((unsigned short)(w[e] >> 16)));
          o[e] = pack2(half_bits(a), half_bits(b));
        }
        *(uint4*)d0 = make_uint4(o[0], o[1], o[2], o[3]);
      } else {
        float v[4] = {__builtin_bit_cast(float, r[i].x), __builtin_bit_cast(float, r[i].y),
                      __builtin_bit_cast(float, r[i].z), __builtin_bit_cast(float, r[i].w)};
        if (relu) {
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = __builtin_fmaxf(v[e], 0.0f);
        }
        if (KIND == OP_F32_1) {
          unsigned short h[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) h[e] = half_bits(clamp_half_range(v[e]));
          *(uint2*)d0 = make_uint2(pack2(h[0], h[1]), pack2(h[2], h[3]));
        } else {
          unsigned short h[4], l[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) split_half(v[e], h[e], l[e]);
          *(uint2*)d0 = make_uint2(pack2(h[0], h[1]), pack2(h[2], h[3]));
          *(uint2*)(s1 + row * LDK + kc) = make_uint2(pack2(l[0], l[1]), pack2(l[2], l[3]));
        }
      }
    }
  }
};

// ---------------------------------------------------------------------------------------------
// Token-parallel Q tile: source is [K rows][N contiguous]; each thread loads an 8(k) x 2(n) patch and
// writes it transposed, so the LDS image is the same [n][k] layout the token-contraction form uses.
// ---------------------------------------------------------------------------------------------
template <int KIND>
struct NnTile {
  static constexpr bool F32 = kind_is_f32(KIND);
  uint2 r[8];
  int ng, kg;
  long long ncol;   // global column of this thread's first element
  bool nvalid;

  __device__ __forceinline__ void init(const Operand& op, int n0, int N) {
    ng = threadIdx.x & 63;
    kg = threadIdx.x >> 6;
    ncol = (long long)n0 + 2 * ng;
    nvalid = ncol < N;
  }

  __device__ __forceinline__ void load(const Operand& op, long long k, long long k1) {
    const int es = F32 ? 4 : 2;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const long long kk = k + kg * 8 + i;
      if (kk < k1 && nvalid) {
        long long srow = op.idx ? (long long)op.idx[kk] : kk;
        const char* src = (const char*)op.ptr + (srow * op.ld + ncol) * es;
        if (F32) {
          r[i] = *(const uint2*)src;
        } else {
          r[i].x = *(const unsigned int*)src;
          r[i].y = 0;
        }
      } else {
        r[i] = make_uint2(0, 0);
      }
    }
  }

  __device__ __forceinline__ void store(unsigned short* s0, unsigned short* s1, int relu) const {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      unsigned short h[8], l[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (F32) {
          float v = __builtin_bit_cast(float, j == 0 ? r[i].x : r[i].y);
          if (relu) v = __builtin_fmaxf(v, 0.0f);
          if (KIND == OP_F32_2) {
            split_half(v, h[i], l[i]);
          } else {
            h[i] = half_bits(clamp_half_range(v));
          }
        } else {
          unsigned short b = (unsigned short)(j == 0 ? (r[i].x & 0xffffu) : (r[i].x >> 16));
          h[i] = (KIND == OP_BF16) ? b : half_bits(clamp_half_range(bf16_bits_to_float(b)));
        }
      }
      const int off = (2 * ng + j) * LDK + kg * 8;
      *(uint4*)(s0 + off) = make_uint4(pack2(h[0], h[1]), pack2(h[2], h[3]), pack2(h[4], h[5]), pack2(h[6], h[7]));
      if (KIND == OP_F32_2)
        *(uint4*)(s1 + off) = make_uint4(pack2(l[0], l[1]), pack2(l[2], l[3]), pack2(l[4], l[5]), pack2(l[6], l[7]));
    }
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

template <int KP, int KQ, bool NN>
__global__ __launch_bounds__(256) void gemm_kernel(const GemmP p) {
  constexpr int NPP = kind_planes(KP), NPQ = kind_planes(KQ);
  constexpr bool BF = (KP == OP_BF16);
  constexpr bool CROSS = (NPP == 2 || NPQ == 2);
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
    const int G = 8;
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

  KcTile<KP> lp;
  lp.init(p.P, m0);
  KcTile<KQ> lq_kc;
  NnTile<KQ> lq_nn;
  if (NN) {
    lq_nn.init(p.Q, n0, p.N);
  } else {
    lq_kc.init(p.Q, n0);
  }

  floatx16 acc[2][2], acx[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        acc[i][j][e] = 0.0f;
        acx[i][j][e] = 0.0f;
      }

  if (k0 < k1) {
    lp.load(k0, k1);
    if (NN) lq_nn.load(p.Q, k0, k1); else lq_kc.load(k0, k1);
  }
  for (long long k = k0; k < k1; k += BK) {
    lp.store(sP[0], sP[NPP - 1], p.P.relu);
    if (NN) lq_nn.store(sQ[0], sQ[NPQ - 1], p.Q.relu); else lq_kc.store(sQ[0], sQ[NPQ - 1], p.Q.relu);
    __syncthreads();
    if (k + BK < k1) {  // next tile's global loads fly during the matrix work
      lp.load(k + BK, k1);
      if (NN) lq_nn.load(p.Q, k + BK, k1); else lq_kc.load(k + BK, k1);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const int koff = ks * 16 + 8 * (lane >> 5);
      uint4 ph[2], pl[2], qh[2], ql[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int off = (wm * 64 + i * 32 + (lane & 31)) * LDK + koff;
        ph[i] = *(const uint4*)(&sP[0][off]);
        if (NPP == 2) pl[i] = *(const uint4*)(&sP[NPP - 1][off]);
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int off = (wn * 64 + j * 32 + (lane & 31)) * LDK + koff;
        qh[j] = *(const uint4*)(&sQ[0][off]);
        if (NPQ == 2) ql[j] = *(const uint4*)(&sQ[NPQ - 1][off]);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          acc[i][j] = mma<BF>(ph[i], qh[j], acc[i][j]);
          if (NPQ == 2) acx[i][j] = mma<BF>(ph[i], ql[j], acx[i][j]);
          if (NPP == 2) acx[i][j] = mma<BF>(pl[i], qh[j], acx[i][j]);
        }
    }
    __syncthreads();
  }

  // ---- epilogue -----------------------------------------------------------------------------
  double red0 = 0.0, red1 = 0.0;
  const float ab = p.alpha + p.beta;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = m0 + wm * 64 + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        const int n = n0 + wn * 64 + j * 32 + (lane & 31);
        if (m >= p.M || n >= p.N) continue;
        float v = acc[i][j][e];
        if (CROSS) v += acx[i][j][e] * (1.0f / LO_SCALE);
        switch (p.epi) {
          case EPI_PARTIAL:
            p.out[((long long)split * p.M + m) * p.N + n] = v;
            break;
          case EPI_STORE:
            p.out[(long long)m * p.ldo + n] = v;
            break;
          case EPI_INITZ: {
            const long long o = (long long)m * p.lda + n;
            const float a = __builtin_fmaxf(v, 0.0f);
            p.Z0s[o] = v;
            p.Zs[o] = v;
            p.As[o] = a;
            red0 += (double)a * (double)a;
          } break;
          case EPI_RESID: {
            const float r = p.Yin[(long long)m * p.ldy + n] - v;
            if (p.write_out) p.out[(long long)m * p.ldo + n] = r;
            red0 += (double)r * (double)r;
          } break;
          case EPI_AUPD: {
            const long long o = (long long)p.oidx[m] * p.lda + n;
            p.As[o] = __builtin_fmaxf(p.Zs[o], 0.0f) + v;
          } break;
          case EPI_ZUPD: {
            const long long o = (long long)p.oidx[m] * p.lda + n;
            const float a = p.As[o];
            const float z1 = v;
            const float z2 = (p.beta * a + p.alpha * z1) / ab;
            const float cm = __builtin_fminf(z1, 0.0f);
            const float costm = p.beta * a * a + p.alpha * (cm - z1) * (cm - z1);
            const float cp = __builtin_fmaxf(z2, 0.0f);
            const float costp = p.beta * (a - cp) * (a - cp) + p.alpha * (cp - z1) * (cp - z1);
            const float z = costm < costp ? cm : cp;
            p.Zs[o] = z;
            const float ra = a - __builtin_fmaxf(z, 0.0f);
            const float rz = z - z1;
            red0 += (double)ra * (double)ra;
            red1 += (double)rz * (double)rz;
          } break;
          default:
            break;
        }
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

template <int KP, int KQ, bool NN>
static void launch_one(strp_ctx* ctx, const GemmP& p) {
  hipLaunchKernelGGL((gemm_kernel<KP, KQ, NN>), dim3(gemm_grid_blocks(p)), dim3(256), 0, ctx->stream, p);
}

strp_status launch_gemm(strp_ctx* ctx, GemmP& p, int kp, int kq, bool nn) {
  if (p.M <= 0 || p.N <= 0 || p.K <= 0) return fail(ctx, STRP_EINVAL, "gemm: empty shape");
  if (p.ntiles <= 0 || p.splits <= 0) return fail(ctx, STRP_EINVAL, "gemm: tiles not planned");
  if ((kp == OP_BF16) != (kq == OP_BF16)) return fail(ctx, STRP_EINVAL, "gemm: bf16 cores need both operands bf16");
  const int key = (nn ? 100 : 0) + kp * 10 + kq;
  static const char* const epi_names[] = {"partial", "store", "initz", "resid", "aupd", "zupd"};
  static char names[2][4][4][6][40];
  char* name = names[nn ? 1 : 0][kp][kq][p.epi];
  if (!name[0]) snprintf(name, 40, "gemm_%s_p%d_q%d_%s", nn ? "nn" : "nt", kp, kq, epi_names[p.epi]);
  const double mn = p.triangle ? 0.5 * (double)p.M * ((double)p.M + 1.0) : (double)p.M * (double)p.N;
  const double esp = (kp == OP_BF16 || kp == OP_BF16_H) ? 2.0 : 4.0, esq = (kq == OP_BF16 || kq == OP_BF16_H) ? 2.0 : 4.0;
  static const double out_words[] = {1.0, 1.0, 3.0, 2.0, 2.0, 2.0};
  double obytes = 4.0 * out_words[p.epi] * (double)p.M * (double)p.N * (p.epi == EPI_PARTIAL ? (double)p.splits : 1.0);
  if (p.epi == EPI_RESID && !p.write_out) obytes *= 0.5;
  const double ibytes = p.triangle ? esp * (double)p.M * (double)p.K : esp * (double)p.M * (double)p.K + esq * (double)p.N * (double)p.K;
  ProfScope ps(ctx, name, 2.0 * mn * (double)p.K, ibytes + obytes);
  switch (key) {
    case 0: launch_one<OP_BF16, OP_BF16, false>(ctx, p); break;
    case 11: launch_one<OP_F32_1, OP_F32_1, false>(ctx, p); break;
    case 22: launch_one<OP_F32_2, OP_F32_2, false>(ctx, p); break;
    case 13: launch_one<OP_F32_1, OP_BF16_H, false>(ctx, p); break;
    case 23: launch_one<OP_F32_2, OP_BF16_H, false>(ctx, p); break;
    case 31: launch_one<OP_BF16_H, OP_F32_1, false>(ctx, p); break;
    case 32: launch_one<OP_BF16_H, OP_F32_2, false>(ctx, p); break;
    case 100: launch_one<OP_BF16, OP_BF16, true>(ctx, p); break;
    case 111: launch_one<OP_F32_1, OP_F32_1, true>(ctx, p); break;
    case 122: launch_one<OP_F32_2, OP_F32_2, true>(ctx, p); break;
    case 113: launch_one<OP_F32_1, OP_BF16_H, true>(ctx, p); break;
    case 123: launch_one<OP_F32_2, OP_BF16_H, true>(ctx, p); break;
    case 131: launch_one<OP_BF16_H, OP_F32_1, true>(ctx, p); break;
    case 132: launch_one<OP_BF16_H, OP_F32_2, true>(ctx, p); break;
    default:
      return fail(ctx, STRP_EINVAL, "gemm: operand kind combination %d/%d not built", kp, kq);
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

}  // namespace strp
