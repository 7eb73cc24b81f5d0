// Pipelined MFMA GEMM for large problems: 256x256 block tile, eight wavefronts of 128x64, operand tiles
// brought from HBM/L2 straight into LDS by the global-load-to-LDS path (no staging registers), four LDS
// stages of 16 contraction steps each, three stages in flight behind the one being multiplied.
//
// Why: with staging registers only one K tile can be in flight per CU (the 256 accumulator registers of a
// 128x128 wavefront tile leave no room for more), and one tile in flight (64 KB per CU) at ~2 us of loaded
// memory latency caps the chip at ~9 TB/s of operand traffic.  LDS has room for four stages.
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
constexpr int SK = 16;             // contraction steps per stage (two k-groups)
constexpr int NSTAGE = 4;
constexpr int PLANE_STAGE_BYTES = 2 * ROWS * 16;   // one plane of one operand in one stage: 8 KB
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

// NW = wavefronts per block: 4 (2x2, 128x128 each) or 8 (2x4, 128x64 each; two per SIMD give the memory
// system twice as many independent request streams).
template <int NPP, int NPQ, int NW>
__global__ __launch_bounds__(64 * NW, 1) void gemm_dma_kernel(const GemmP p) {
  using namespace dma;
  constexpr int NPL = NPP + NPQ;                       // planes per stage
  constexpr int STAGE_BYTES = NPL * PLANE_STAGE_BYTES;
  constexpr int LPW = 8 * NPL / NW;                    // load instructions per wavefront per stage
  constexpr int WTM = 4, WTN = NW == 8 ? 2 : 4;        // 32x32 MFMA tiles per wavefront
  __shared__ __attribute__((aligned(1024))) unsigned char smem[NSTAGE * STAGE_BYTES];
  __shared__ double sred[NW][2];
  __shared__ int srow[dma::ROWS];   // gathered state row of each output row (AUPD / ZUPD)

  // ---- which tile, which K range ---------------------------------------------------------
  int tm, tn, split;
  if (!decode_tile(p, (int)blockIdx.x, (int)gridDim.x, tm, tn, split)) return;
  const int m0 = tm * ROWS, n0 = tn * ROWS;
  const long long k0 = (long long)split * p.kchunk;
  const long long k1 = (k0 + p.kchunk < p.K) ? (k0 + p.kchunk) : p.K;
  const int nstages = (int)((k1 - k0 + SK - 1) / SK);
  const long long g0 = k0 >> 3;                       // first k-group of this block (even)
  const long long g_last = ((k1 + 7) >> 3) - 1;       // last k-group holding data; its pair partner is zero padding

  const int tid = threadIdx.x, lane = tid & 63;
  // fetched now, parked in LDS after the main loop: the epilogue never waits for an index load
  int my_row = 0;
  if (p.oidx && tid < ROWS && m0 + tid < p.M) my_row = p.oidx[m0 + tid];
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = NW == 8 ? wave >> 2 : wave >> 1, wn = NW == 8 ? wave & 3 : wave & 1;
  constexpr int WROWS = 32 * WTM, WCOLS = 32 * WTN;

  // ---- this wavefront's load instructions: q = wave + NW i, plane = q / 8, k-group = (q / 4) % 2, row segment = q % 4
  const unsigned short* gp[LPW];     // lane's source chunk for stage 0
  unsigned lds_off[LPW];             // byte offset of the instruction's 1 KB destination inside a stage
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
  // stage s reads k-groups g0 + 2 s and g0 + 2 s + 1; stages past the end re-read the last pair (never multiplied)
  const long long last_pair = (g_last - g0) >> 1;
  auto issue_stage = [&](int s) {
    const long long sp = s < last_pair ? s : last_pair;
    const unsigned slot = lds_base + (unsigned)(s & (NSTAGE - 1)) * STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < LPW; ++i) lds_dma_16(gp[i] + sp * 2048, slot + lds_off[i]);
  };

  floatx16 acc[WTM][WTN];
#pragma unroll
  for (int i = 0; i < WTM; ++i)
#pragma unroll
    for (int j = 0; j < WTN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  // fragment addresses: lanes 0-31 read k-group 0 of the stage, lanes 32-63 k-group 1; 32 consecutive rows = 512 B
  const int offP = ((lane >> 5) * ROWS + wm * WROWS + (lane & 31)) * 16;
  const int offQ = ((lane >> 5) * ROWS + wn * WCOLS + (lane & 31)) * 16;
  struct Frags { uint4 ph[WTM], pl[WTM], qh[WTN], ql[WTN]; };
  auto read_frags = [&](Frags& f, int s) {
    const unsigned char* st = smem + (s & (NSTAGE - 1)) * STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < WTM; ++i) {
      f.ph[i] = *(const uint4*)(st + offP + i * 512);
      if (NPP == 2) f.pl[i] = *(const uint4*)(st + PLANE_STAGE_BYTES + offP + i * 512);
    }
#pragma unroll
    for (int j = 0; j < WTN; ++j) {
      f.qh[j] = *(const uint4*)(st + NPP * PLANE_STAGE_BYTES + offQ + j * 512);
      if (NPQ == 2) f.ql[j] = *(const uint4*)(st + (NPP + 1) * PLANE_STAGE_BYTES + offQ + j * 512);
    }
  };
  auto mma1 = [&](uint4 a, uint4 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
  };
  auto run_mfma = [&](const Frags& f) {
    if (NPQ == 2) {
#pragma unroll
      for (int i = 0; i < WTM; ++i)
#pragma unroll
        for (int j = 0; j < WTN; ++j) acc[i][j] = mma1(f.ph[i], f.ql[j], acc[i][j]);
    }
    if (NPP == 2) {
#pragma unroll
      for (int i = 0; i < WTM; ++i)
#pragma unroll
        for (int j = 0; j < WTN; ++j) acc[i][j] = mma1(f.pl[i], f.qh[j], acc[i][j]);
    }
#pragma unroll
    for (int i = 0; i < WTM; ++i)
#pragma unroll
      for (int j = 0; j < WTN; ++j) acc[i][j] = mma1(f.ph[i], f.qh[j], acc[i][j]);
  };

  // Instruction order inside a half stage: the fragment reads of the next stage are issued in the shadow of the
  // matrix-core instructions of this one (one LDS read after each of the first MFMAs) instead of ahead of them.
  auto interleave = [&]() {
    constexpr int NRD = WTM * NPP + WTN * NPQ;   // ds_read_b128 per half stage
    constexpr int NMF = WTM * WTN * (NPP * NPQ == 4 ? 3 : NPP * NPQ);
#pragma unroll
    for (int i = 0; i < NRD; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one DS read
    }
    __builtin_amdgcn_sched_group_barrier(0x008, NMF - NRD, 0);
  };

  // ---- pipeline: stages 0..3 requested up front; iteration s multiplies stage s from registers while the
  // fragments of stage s+1 are read from LDS and stage s+4 is requested into the slot stage s just left.
  issue_stage(0);
  issue_stage(1);
  issue_stage(2);
  issue_stage(3);
  Frags fa, fb;
  wait_vmcnt<3 * LPW>();     // stage 0 has landed (three younger stages may still be in flight)
  __syncthreads();
  read_frags(fa, 0);
  int s = 0;
#pragma unroll 1
  for (; s + 1 < nstages; s += 2) {
    // -- even half: multiply stage s (fa), fetch fragments of stage s+1 into fb
    wait_vmcnt_lgkm0<2 * LPW>();   // stage s+1 has landed; this wavefront's fragment reads of stage s are complete
    __syncthreads();               // ... and so for every wavefront: the slot of stage s may be overwritten
    issue_stage(s + 4);            // into the slot of stage s
    read_frags(fb, s + 1);
    run_mfma(fa);
    interleave();
    __builtin_amdgcn_sched_barrier(0);
    // -- odd half
    wait_vmcnt_lgkm0<2 * LPW>();
    __syncthreads();
    issue_stage(s + 5);
    read_frags(fa, s + 2);         // past the last stage this reads a slot that is never multiplied
    run_mfma(fb);
    interleave();
    __builtin_amdgcn_sched_barrier(0);
  }
  if (s < nstages) run_mfma(fa);   // odd stage count: the last stage is already in registers
  wait_vmcnt<0>();           // nothing may still be writing LDS when the block ends or reuses it
  if (tid < ROWS) srow[tid] = my_row;
  __syncthreads();

  // ---- epilogue -------------------------------------------------------------------------------
  float unscale = 1.0f;
  if (p.P.scale) unscale /= *p.P.scale;
  if (p.Q.scale) unscale /= *p.Q.scale;
  double red0 = 0.0, red1 = 0.0;
  const int mbase = m0 + wm * WROWS + 4 * (lane >> 5), nbase = n0 + wn * WCOLS + (lane & 31);
  switch (p.epi) {
    case EPI_PARTIAL: epilogue<EPI_PARTIAL, WTM, WTN>(p, acc, unscale, mbase, nbase, split, srow, m0, red0, red1); break;
    case EPI_STORE: epilogue<EPI_STORE, WTM, WTN>(p, acc, unscale, mbase, nbase, split, srow, m0, red0, red1); break;
    case EPI_INITZ: epilogue<EPI_INITZ, WTM, WTN>(p, acc, unscale, mbase, nbase, split, srow, m0, red0, red1); break;
    case EPI_RESID: epilogue<EPI_RESID, WTM, WTN>(p, acc, unscale, mbase, nbase, split, srow, m0, red0, red1); break;
    case EPI_AUPD: epilogue<EPI_AUPD, WTM, WTN>(p, acc, unscale, mbase, nbase, split, srow, m0, red0, red1); break;
    default: epilogue<EPI_ZUPD, WTM, WTN>(p, acc, unscale, mbase, nbase, split, srow, m0, red0, red1); break;
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

template <int NW>
static void launch_dma_nw(strp_ctx* ctx, const GemmP& p, int npp, int npq) {
  const dim3 grid(gemm_grid_blocks(p)), block(64 * NW);
  switch (npp * 10 + npq) {
    case 11: hipLaunchKernelGGL((gemm_dma_kernel<1, 1, NW>), grid, block, 0, ctx->stream, p); break;
    case 12: hipLaunchKernelGGL((gemm_dma_kernel<1, 2, NW>), grid, block, 0, ctx->stream, p); break;
    case 21: hipLaunchKernelGGL((gemm_dma_kernel<2, 1, NW>), grid, block, 0, ctx->stream, p); break;
    default: hipLaunchKernelGGL((gemm_dma_kernel<2, 2, NW>), grid, block, 0, ctx->stream, p); break;
  }
}

void launch_gemm_dma(strp_ctx* ctx, const GemmP& p, int npp, int npq) { launch_dma_nw<8>(ctx, p, npp, npq); }

}  // namespace strp
