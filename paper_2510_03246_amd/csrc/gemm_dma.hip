// Pipelined MFMA GEMM for large problems: 256x256 block tile, eight wavefronts of 128x64, operand tiles
// brought from HBM/L2 straight into LDS by the global-load-to-LDS path (no staging registers), LDS stages of
// 16 contraction steps each, the stages behind the one being multiplied in flight.
//
// Why: with staging registers only one K tile can be in flight per CU (the accumulator registers of a
// 128x64 wavefront tile leave little room for more), and one tile in flight (64 KB per CU) at ~2 us of loaded
// memory latency caps the chip at ~9 TB/s of operand traffic.  LDS has room for two to four pairs of stages.
//
// The operand layout (see gemm_mfma.hip) makes every load one contiguous KB: a wavefront instruction
// moves the 64 chunks (16 B each) of 64 consecutive rows of one k-group, and the hardware writes lane l's
// chunk at LDS base + 16 l, which is exactly the [k-group][row][8] image the matrix-core fragments read.
//
// The loads are issued from inline assembly, so the compiler does not track them: completion is enforced
// here with explicit vmcnt waits (loads retire in order) followed by a workgroup barrier.
#include <stdlib.h>

#include "gemm_epilogue.h"

namespace strp {

namespace dma {
constexpr int ROWS = 256;          // rows of P / columns of Q per block
constexpr int PLANE_STAGE_BYTES = 2 * ROWS * 16;   // one plane of one operand in one stage (16 contraction steps = two k-groups): 8 KB
}  // namespace dma

// m0 is written here, so it is named as clobbered; the compiler treats m0 as a reserved register (it never keeps a
// value in it across statements) and warns about the listing, which is silenced for this one statement.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void lds_dma_16(const void* gptr, unsigned lds_addr) {
  // m0 = LDS byte address of lane 0's chunk; lane l lands at m0 + 16 l
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_addr), "v"(gptr) : "memory", "m0");
}
#pragma clang diagnostic pop

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt_lgkm0() {
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" : : "n"(N) : "memory");
}

// ---------------------------------------------------------------------------------------------------------------------
// The matrix-core instruction is v_mfma_f32_16x16x32_f16: each wavefront's 128 x 64 outputs are 8 x 4 tiles of
// 16 x 16, one instruction contracts 32 steps.  Measured on this chip with random fp16 operands fed from LDS in exactly
// this wavefront shape, the 16x16x32 instruction sustains 11 % more than the 32x32x16 one (the chip is power-limited
// while the matrix cores run; the smaller accumulator tile costs less energy per flop).
// Two consecutive 16-step stages form the 32 steps of one instruction (lanes 0-31 read their operand chunks from the
// first stage of the pair, lanes 32-63 from the second), so the pipeline advances by pairs: while pair p is multiplied,
// the next one to three pairs are in flight (LDS holds two pairs of four planes, three of three, four of two), and the
// slots of pair p are refilled as soon as every wavefront has its last fragment of the pair in registers.  The Q fragments of a pair stay in registers (double
// buffered across pairs), the P fragments stream through two register sets.
template <int NPP, int NPQ>
__global__ __launch_bounds__(512, 1) void gemm_dma_kernel(const GemmP p) {
  using namespace dma;
  constexpr int NW = 8;
  constexpr int NPL = NPP + NPQ;
  constexpr int STAGE_BYTES = NPL * PLANE_STAGE_BYTES;
  constexpr int LPW = 8 * NPL / NW;
  // pairs of stages LDS holds: two with four planes (128 KB), three with three (144 KB), four with two (128 KB)
  constexpr int NP = NPL == 4 ? 2 : (NPL == 3 ? 3 : 4);
  __shared__ __attribute__((aligned(1024))) unsigned char smem[2 * NP * STAGE_BYTES];
  __shared__ double sred[NW][2];
  __shared__ int srow[dma::ROWS];

  int tm, tn, split;
  if (!decode_tile(p, (int)blockIdx.x, (int)gridDim.x, tm, tn, split)) return;
  const int m0 = tm * ROWS, n0 = tn * ROWS;
  const long long k0 = (long long)split * p.kchunk;                 // a multiple of 32
  const long long k1 = (k0 + p.kchunk < p.K) ? (k0 + p.kchunk) : p.K;
  const int npairs = (int)((k1 - k0 + 31) / 32);                    // k-groups past k1 inside the last pair are zero padding
  const long long g0 = k0 >> 3;
  const long long g_last = ((k1 + 7) >> 3) - 1;

  const int tid = threadIdx.x, lane = tid & 63;
  int my_row = 0;
  if (p.oidx && tid < ROWS && m0 + tid < p.M) my_row = p.oidx[m0 + tid];
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;

  const unsigned short* gp[LPW];
  unsigned lds_off[LPW];
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    const int q = wave + NW * i;
    const int plane = q >> 3, g = (q >> 2) & 1, seg = q & 3;
    const bool isP = plane < NPP;
    const PlaneOp& op = isP ? p.P : p.Q;
    const int pl = isP ? plane : plane - NPP;
    const unsigned short* base = pl == 0 ? op.hi : op.lo;
    const int row0 = isP ? m0 : n0;
    int pan = (row0 >> 7) + (seg >> 1);
    pan = pan < op.npan ? pan : op.npan - 1;
    const int rr = (seg & 1) * 64 + lane;
    gp[i] = base + (((long long)pan * op.kg + g0 + g) * 128 + rr) * 8;
    lds_off[i] = (unsigned)(plane * PLANE_STAGE_BYTES + (g * ROWS + seg * 64) * 16);
  }
  // stage s = k-groups g0 + 2 s, g0 + 2 s + 1; the planes are padded to a multiple of four k-groups, so both stages of
  // the last pair exist in memory; stages past them re-read the last one (never multiplied)
  const long long last_stage = 2 * (long long)npairs - 1;
  auto issue_stage = [&](int s) {
    const long long sp = s < last_stage ? s : last_stage;
    const unsigned slot = lds_base + (unsigned)(s % (2 * NP)) * STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < LPW; ++i) lds_dma_16(gp[i] + sp * 2048, slot + lds_off[i]);
  };
  (void)g_last;

  floatx4 acc[8][4];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};

  // lane l reads the chunk of k-group l / 16 of the 32-deep step: groups 0, 1 in the pair's first stage, 2, 3 in its second
  const int kgl = lane >> 4;
  const int offP = (kgl >> 1) * STAGE_BYTES + ((kgl & 1) * ROWS + wm * 128 + (lane & 15)) * 16;
  const int offQ = (kgl >> 1) * STAGE_BYTES + NPP * PLANE_STAGE_BYTES + ((kgl & 1) * ROWS + wn * 64 + (lane & 15)) * 16;
  struct QF { uint4 h[4], l[4]; };
  struct PF { uint4 h, l; };
  auto read_q = [&](QF& f, int pr) {
    const unsigned char* st = smem + (pr % NP) * 2 * STAGE_BYTES;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      f.h[j] = *(const uint4*)(st + offQ + j * 256);
      if (NPQ == 2) f.l[j] = *(const uint4*)(st + PLANE_STAGE_BYTES + offQ + j * 256);
    }
  };
  auto read_p = [&](PF& f, int pr, int i) {
    const unsigned char* st = smem + (pr % NP) * 2 * STAGE_BYTES;
    f.h = *(const uint4*)(st + offP + i * 256);
    if (NPP == 2) f.l = *(const uint4*)(st + PLANE_STAGE_BYTES + offP + i * 256);
  };
  auto mma = [&](uint4 a, uint4 b, floatx4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
  };
  auto pass_hl = [&](floatx4 (&c)[4], const PF& a, const QF& b) {
    if (NPQ == 2) {
#pragma unroll
      for (int j = 0; j < 4; ++j) c[j] = mma(a.h, b.l[j], c[j]);
    }
  };
  auto pass_lh = [&](floatx4 (&c)[4], const PF& a, const QF& b) {
    if (NPP == 2) {
#pragma unroll
      for (int j = 0; j < 4; ++j) c[j] = mma(a.l, b.h[j], c[j]);
    }
  };
  auto pass_hh = [&](floatx4 (&c)[4], const PF& a, const QF& b) {
#pragma unroll
    for (int j = 0; j < 4; ++j) c[j] = mma(a.h, b.h[j], c[j]);
  };
  auto run_row = [&](floatx4 (&c)[4], const PF& a, const QF& b) {
    pass_hl(c, a, b);
    pass_lh(c, a, b);
    pass_hh(c, a, b);
  };
  // One pair: bc holds the pair's Q fragments, pa its first P fragment; on return bn / pa hold those of the next pair.
  PF pa, pb;
  // Instruction order: the fragment reads of row i + 1 are issued ahead of the matrix-core instructions of row i (a
  // scheduling barrier after each pair of reads keeps the compiler from sinking them to where they are needed).
  auto pair_step = [&](int pr, const QF& bc, QF& bn) {
#define STRP_ROW(i, cur, nxt)                \
    read_p(nxt, pr, (i) + 1);                \
    __builtin_amdgcn_sched_barrier(0);       \
    run_row(acc[i], cur, bc);                \
    __builtin_amdgcn_sched_barrier(0);
    STRP_ROW(0, pa, pb)
    STRP_ROW(1, pb, pa)
    STRP_ROW(2, pa, pb)
    STRP_ROW(3, pb, pa)
    STRP_ROW(4, pa, pb)
    STRP_ROW(5, pb, pa)
    STRP_ROW(6, pa, pb)
#undef STRP_ROW
    wait_vmcnt_lgkm0<(NP - 2) * 2 * LPW>();   // the next pair has landed; this wavefront's fragment reads of this pair are complete
    __syncthreads();               // ... and so for every wavefront: the pair's slots may be overwritten
    // the last row needs nothing from LDS: its matrix-core instructions go out first and run while the refill is
    // requested and the next pair's first fragments are read
    pass_hh(acc[7], pb, bc);
    __builtin_amdgcn_sched_barrier(0);
    issue_stage(2 * (pr + NP));
    issue_stage(2 * (pr + NP) + 1);
    __builtin_amdgcn_sched_barrier(0);
    pass_hl(acc[7], pb, bc);
    __builtin_amdgcn_sched_barrier(0);
    read_q(bn, pr + 1);            // past the last pair this reads slots that are never multiplied
    read_p(pa, pr + 1, 0);
    __builtin_amdgcn_sched_barrier(0);
    pass_lh(acc[7], pb, bc);
    __builtin_amdgcn_sched_barrier(0);
  };

#pragma unroll
  for (int q = 0; q < 2 * NP; ++q) issue_stage(q);
  QF q0, q1;
  wait_vmcnt<(NP - 1) * 2 * LPW>();   // the first pair has landed
  __syncthreads();
  read_q(q0, 0);
  read_p(pa, 0, 0);
  int pr = 0;
#pragma unroll 1
  for (; pr + 1 < npairs; pr += 2) {
    pair_step(pr, q0, q1);
    pair_step(pr + 1, q1, q0);
  }
  if (pr < npairs) pair_step(pr, q0, q1);
  wait_vmcnt<0>();
  if (tid < ROWS) srow[tid] = my_row;
  __syncthreads();

  float unscale = 1.0f;
  if (p.P.scale) unscale /= *p.P.scale;
  if (p.Q.scale) unscale /= *p.Q.scale;
  double red0 = 0.0, red1 = 0.0;
  const int mbase = m0 + wm * 128 + 8 * (lane >> 5), nbase = n0 + wn * 64 + (lane & 31);
  switch (p.epi) {
    case EPI_PARTIAL: epilogue16<EPI_PARTIAL>(p, acc, unscale, mbase, nbase, split, srow, m0, red0, red1); break;
    case EPI_STORE: epilogue16<EPI_STORE>(p, acc, unscale, mbase, nbase, split, srow, m0, red0, red1); break;
    case EPI_INITZ: epilogue16<EPI_INITZ>(p, acc, unscale, mbase, nbase, split, srow, m0, red0, red1); break;
    case EPI_RESID: epilogue16<EPI_RESID>(p, acc, unscale, mbase, nbase, split, srow, m0, red0, red1); break;
    case EPI_AUPD: epilogue16<EPI_AUPD>(p, acc, unscale, mbase, nbase, split, srow, m0, red0, red1); break;
    default: epilogue16<EPI_ZUPD>(p, acc, unscale, mbase, nbase, split, srow, m0, red0, red1); break;
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
      double r0 = 0.0, r1 = 0.0;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        r0 += sred[w][0];
        r1 += sred[w][1];
      }
      p.red[2 * (long long)blockIdx.x + 0] = r0;
      p.red[2 * (long long)blockIdx.x + 1] = r1;
    }
  }
}

void launch_gemm_dma(strp_ctx* ctx, const GemmP& p, int npp, int npq) {
  const dim3 grid(gemm_grid_blocks(p)), block(512);
  switch (npp * 10 + npq) {
    case 11: hipLaunchKernelGGL((gemm_dma_kernel<1, 1>), grid, block, 0, ctx->stream, p); break;
    case 12: hipLaunchKernelGGL((gemm_dma_kernel<1, 2>), grid, block, 0, ctx->stream, p); break;
    case 21: hipLaunchKernelGGL((gemm_dma_kernel<2, 1>), grid, block, 0, ctx->stream, p); break;
    default: hipLaunchKernelGGL((gemm_dma_kernel<2, 2>), grid, block, 0, ctx->stream, p); break;
  }
}


}  // namespace strp
