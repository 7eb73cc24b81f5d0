// Benchmark helper, built as its own shared library (libstrp_bench.so) and no part of libstrp.so or its ABI.
// Measurement aid: the sustained rate of the fp16 matrix-core instructions on this chip, so that the GEMM figures can be
// read against what the matrix cores deliver in practice and not only against the nominal 2.5 PFLOP/s.
//   kind 0: back-to-back v_mfma_f32_16x16x32_f16 on constant register operands (no LDS, no memory): the issue limit
//   kind 2: as kind 0 with random fp16 values in the operand registers (operand toggling is what the power
//           management reacts to)
//   kind 1: the pipelined GEMM's inner loop without its memory side: eight wavefronts per CU, each 8 x 4 tiles of
//           16 x 16, three passes per 32-deep step, operand fragments re-read from LDS every step, LDS filled with
//           random fp16 values
//   kind 3: kind 1 with v_mfma_f32_32x32x16_f16 (4 x 2 tiles of 32 x 32 per wavefront, 16-deep steps): same flops, same
//           LDS traffic; the comparison that made the GEMM use the 16x16x32 instruction
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace strp {

typedef _Float16 probe_half8 __attribute__((ext_vector_type(8)));
typedef float probe_floatx16 __attribute__((ext_vector_type(16)));
typedef float probe_floatx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned int probe_rnd(unsigned int& x) {   // two random halves of magnitude in [0.5, 2)
  x = x * 1664525u + 1013904223u;
  const unsigned int lo = (x & 0x83ffu) | 0x3800u, hi = ((x >> 16) & 0x83ffu) | 0x3800u;
  return lo | (hi << 16);
}

// 32 accumulators of 16 x 16: 8 P fragments x 4 Q fragments from registers
template <bool RANDOM>
__global__ __launch_bounds__(512, 1) void probe_mfma_reg_kernel(float* out, int iters, unsigned int seed) {
  probe_floatx4 acc[32];
#pragma unroll
  for (int i = 0; i < 32; ++i) acc[i] = probe_floatx4{0.0f, 0.0f, 0.0f, 0.0f};
  unsigned int x = seed + threadIdx.x * 2654435761u + blockIdx.x * 40503u;
  uint4 a[8], b[4];
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = RANDOM ? make_uint4(probe_rnd(x), probe_rnd(x), probe_rnd(x), probe_rnd(x)) : make_uint4(0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u);
#pragma unroll
  for (int i = 0; i < 4; ++i) b[i] = RANDOM ? make_uint4(probe_rnd(x), probe_rnd(x), probe_rnd(x), probe_rnd(x)) : make_uint4(0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i * 4 + j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(probe_half8, a[i]), __builtin_bit_cast(probe_half8, b[j]),
                                                                acc[i * 4 + j], 0, 0, 0);
  }
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 32; ++i)
#pragma unroll
    for (int e = 0; e < 4; ++e) s += acc[i][e];
  out[blockIdx.x * 512 + threadIdx.x] = s;
}

__device__ __forceinline__ void probe_fill(unsigned char* smem, unsigned int seed) {
  unsigned int x = seed + threadIdx.x * 2654435761u + blockIdx.x * 40503u;
  for (int i = threadIdx.x; i < 4 * 32768 / 4; i += 512) ((unsigned int*)smem)[i] = probe_rnd(x);
  __syncthreads();
}

// the pipelined GEMM's wavefront shape on 16x16x32: a 32-deep step is 4 planes x 16 KB
__global__ __launch_bounds__(512, 1) void probe_mfma_lds16_kernel(float* out, int iters, unsigned int seed) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[4 * 32768];
  probe_fill(smem, seed);
  probe_floatx4 acc[8][4];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = probe_floatx4{0.0f, 0.0f, 0.0f, 0.0f};
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 2, wn = wave & 3;
  const int offP = ((lane >> 4) * 256 + wm * 128 + (lane & 15)) * 16, offQ = ((lane >> 4) * 256 + wn * 64 + (lane & 15)) * 16;
  auto mm = [](uint4 p, uint4 q, probe_floatx4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(probe_half8, p), __builtin_bit_cast(probe_half8, q), c, 0, 0, 0);
  };
  for (int it = 0; it < iters; ++it) {
    const unsigned char* st = smem + (it & 1) * 65536;
    uint4 qh[4], ql[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      qh[j] = *(const uint4*)(st + 32768 + offQ + j * 256);
      ql[j] = *(const uint4*)(st + 49152 + offQ + j * 256);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint4 ph = *(const uint4*)(st + offP + i * 256), pl = *(const uint4*)(st + 16384 + offP + i * 256);
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = mm(ph, ql[j], acc[i][j]);
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = mm(pl, qh[j], acc[i][j]);
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = mm(ph, qh[j], acc[i][j]);
    }
  }
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) s += acc[i][j][e];
  out[blockIdx.x * 512 + threadIdx.x] = s;
}

// the same work on 32x32x16: a 16-deep step is 4 planes x 8 KB
__global__ __launch_bounds__(512, 1) void probe_mfma_lds32_kernel(float* out, int iters, unsigned int seed) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[4 * 32768];
  probe_fill(smem, seed);
  probe_floatx16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 2, wn = wave & 3;
  const int offP = ((lane >> 5) * 256 + wm * 128 + (lane & 31)) * 16, offQ = ((lane >> 5) * 256 + wn * 64 + (lane & 31)) * 16;
  auto mm = [](uint4 p, uint4 q, probe_floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(probe_half8, p), __builtin_bit_cast(probe_half8, q), c, 0, 0, 0);
  };
  for (int it = 0; it < iters; ++it) {
    const unsigned char* st = smem + (it & 3) * 32768;
    uint4 ph[4], pl[4], qh[2], ql[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      ph[i] = *(const uint4*)(st + offP + i * 512);
      pl[i] = *(const uint4*)(st + 8192 + offP + i * 512);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      qh[j] = *(const uint4*)(st + 16384 + offQ + j * 512);
      ql[j] = *(const uint4*)(st + 24576 + offQ + j * 512);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = mm(ph[i], ql[j], acc[i][j]);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = mm(pl[i], qh[j], acc[i][j]);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = mm(ph[i], qh[j], acc[i][j]);
  }
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) s += acc[i][j][e];
  out[blockIdx.x * 512 + threadIdx.x] = s;
}

}  // namespace strp

using namespace strp;

// hip_stream: the stream to run on; scratch: 512 KiB of device memory (256-byte aligned).  Returns 0, 1 (bad argument)
// or 5 (a HIP call failed).  Runs for about `milliseconds` twice, times the second run, synchronises the stream.
extern "C" int strp_bench_mfma_rate(void* hip_stream, void* scratch, size_t scratch_bytes, int32_t kind, double milliseconds,
                                    double* tflops_out) {
  if (!scratch || scratch_bytes < 256 * 512 * sizeof(float) || !tflops_out || kind < 0 || kind > 3 || !(milliseconds > 0.0) ||
      milliseconds > 2000.0)
    return 1;
  hipStream_t stream = (hipStream_t)hip_stream;
  float* out = (float*)scratch;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return 5;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return 5; }
  // flops per wavefront and loop trip: 32 x 16x16x32 (kinds 0, 2), 96 x 16x16x32 (kind 1), 24 x 32x32x16 (kind 3)
  const double flops_per_iter = kind == 1 ? 96.0 * 16384.0 : (kind == 3 ? 24.0 * 32768.0 : 32.0 * 16384.0);
  // two wavefronts per SIMD at ~13 ns per 32768 flops at full rate: size the run to the requested duration (long enough
  // for the power management to settle), then measure
  int iters = (int)(milliseconds * 1e-3 / (flops_per_iter / 32768.0 * 2.0 * 13.4e-9));
  if (iters < 1000) iters = 1000;
  float ms = 0.0f;
  bool ok = true;
  for (int rep = 0; rep < 2 && ok; ++rep) {   // the first run warms the clocks
    ok = ok && hipEventRecord(e0, stream) == hipSuccess;
    if (kind == 0)
      hipLaunchKernelGGL(probe_mfma_reg_kernel<false>, dim3(256), dim3(512), 0, stream, out, iters, 3u + rep);
    else if (kind == 2)
      hipLaunchKernelGGL(probe_mfma_reg_kernel<true>, dim3(256), dim3(512), 0, stream, out, iters, 5u + rep);
    else if (kind == 1)
      hipLaunchKernelGGL(probe_mfma_lds16_kernel, dim3(256), dim3(512), 0, stream, out, iters, 17u + rep);
    else
      hipLaunchKernelGGL(probe_mfma_lds32_kernel, dim3(256), dim3(512), 0, stream, out, iters, 17u + rep);
    ok = ok && hipEventRecord(e1, stream) == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
         hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (!ok || !(ms > 0.0f)) return 5;
  *tflops_out = 256.0 * 8.0 * (double)iters * flops_per_iter / ((double)ms * 1e-3) / 1e12;
  return 0;
}
