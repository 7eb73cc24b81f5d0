// Benchmark helper, built as its own shared library (libstrp_bench.so) and no part of libstrp.so or its ABI.
// Measurement aid: the sustained rate of v_mfma_f32_32x32x16_f16 on this chip, so that the GEMM figures can be read
// against what the matrix cores deliver in practice and not only against the nominal 2.5 PFLOP/s.
//   kind 0: back-to-back MFMA on constant register operands (no LDS, no memory): the instruction's issue limit
//   kind 2: as kind 0 with random fp16 values in the operand registers (operand toggling is what the power
//           management reacts to)
//   kind 1: the GEMM's inner loop without its memory side: eight wavefronts per CU, each 4 x 2 tiles, three passes
//           per 16-deep stage, operand fragments re-read from LDS every stage, LDS filled with random fp16 values
//           (operand toggling is what the power management reacts to)
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace strp {

typedef _Float16 probe_half8 __attribute__((ext_vector_type(8)));
typedef float probe_floatx16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(512, 1) void probe_mfma_reg_kernel(float* out, int iters) {
  probe_floatx16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.0f;
  probe_half8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (_Float16)(threadIdx.x * 1e-3f + e);
    b[e] = (_Float16)(1.0f + e * 0.25f);
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[i][e];
  out[blockIdx.x * 512 + threadIdx.x] = s;
}

__global__ __launch_bounds__(512, 1) void probe_mfma_rand_kernel(float* out, int iters, unsigned int seed) {
  probe_floatx16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.0f;
  unsigned int x = seed + threadIdx.x * 2654435761u + blockIdx.x * 40503u;
  auto rnd = [&]() {
    x = x * 1664525u + 1013904223u;
    const unsigned int lo = (x & 0x83ffu) | 0x3800u, hi = ((x >> 16) & 0x83ffu) | 0x3800u;
    return lo | (hi << 16);
  };
  uint4 a[4], b[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) a[i] = make_uint4(rnd(), rnd(), rnd(), rnd());
#pragma unroll
  for (int i = 0; i < 2; ++i) b[i] = make_uint4(rnd(), rnd(), rnd(), rnd());
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i * 2 + j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(probe_half8, a[i]), __builtin_bit_cast(probe_half8, b[j]),
                                                                acc[i * 2 + j], 0, 0, 0);
  }
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[i][e];
  out[blockIdx.x * 512 + threadIdx.x] = s;
}

__global__ __launch_bounds__(512, 1) void probe_mfma_lds_kernel(float* out, int iters, unsigned int seed) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[4 * 32768];
  unsigned int x = seed + threadIdx.x * 2654435761u + blockIdx.x * 40503u;
  for (int i = threadIdx.x; i < 4 * 32768 / 4; i += 512) {   // random halves of magnitude in [0.5, 2): nothing overflows
    x = x * 1664525u + 1013904223u;
    const unsigned int lo = (x & 0x83ffu) | 0x3800u, hi = ((x >> 16) & 0x83ffu) | 0x3800u;
    ((unsigned int*)smem)[i] = lo | (hi << 16);
  }
  __syncthreads();
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
  if (!scratch || scratch_bytes < 256 * 512 * sizeof(float) || !tflops_out || kind < 0 || kind > 2 || !(milliseconds > 0.0) ||
      milliseconds > 2000.0)
    return 1;
  hipStream_t stream = (hipStream_t)hip_stream;
  float* out = (float*)scratch;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return 5;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return 5; }
  const double flops_per_iter = kind == 1 ? 24.0 * 32768.0 : 8.0 * 32768.0;   // per wavefront
  // ~25 ns per MFMA pair of wavefronts at full rate: size the run to the requested duration (long enough for the
  // power management to settle), then measure
  int iters = (int)(milliseconds * 1e-3 / ((kind == 1 ? 24.0 : 8.0) * 2.0 * 13.4e-9));
  if (iters < 1000) iters = 1000;
  float ms = 0.0f;
  bool ok = true;
  for (int rep = 0; rep < 2 && ok; ++rep) {   // the first run warms the clocks
    ok = ok && hipEventRecord(e0, stream) == hipSuccess;
    if (kind == 0)
      hipLaunchKernelGGL(probe_mfma_reg_kernel, dim3(256), dim3(512), 0, stream, out, iters);
    else if (kind == 2)
      hipLaunchKernelGGL(probe_mfma_rand_kernel, dim3(256), dim3(512), 0, stream, out, iters, 5u + rep);
    else
      hipLaunchKernelGGL(probe_mfma_lds_kernel, dim3(256), dim3(512), 0, stream, out, iters, 17u + rep);
    ok = ok && hipEventRecord(e1, stream) == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
         hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (!ok || !(ms > 0.0f)) return 5;
  *tflops_out = 256.0 * 8.0 * (double)iters * flops_per_iter / ((double)ms * 1e-3) / 1e12;
  return 0;
}
