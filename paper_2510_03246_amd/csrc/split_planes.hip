// Split kernels: fp32 / bf16 / fp64 sources -> fp16 operand planes in the panel-major chunk layout
//   offset(k, r) = (((r / 128) * KG + k / 8) * 128 + r % 128) * 8 + k % 8
// (see gemm_mfma.hip).  All padding (rows up to a full panel, k up to a full group) is written as zero.
#include "strp_internal.h"

namespace strp {

__device__ __forceinline__ unsigned short sp_half_bits(float x) {
  _Float16 h = (_Float16)x;
  return __builtin_bit_cast(unsigned short, h);
}
__device__ __forceinline__ void sp_split_half(float x, unsigned short& hi, unsigned short& lo) {
  x = __builtin_fminf(__builtin_fmaxf(x, -65504.0f), 65504.0f);
  _Float16 h = (_Float16)x;
  hi = __builtin_bit_cast(unsigned short, h);
  lo = sp_half_bits(x - (float)h);
}
__device__ __forceinline__ unsigned int sp_pack2(unsigned short a, unsigned short b) {
  return (unsigned int)a | ((unsigned int)b << 16);
}

// Activations [rows x T] (optionally gathered by idx) -> planes.  Both kernels read the source row-contiguously
// and write whole contiguous kilobytes per wavefront store (a 16-byte chunk per lane, consecutive lanes =
// consecutive chunks): partial-line stores cost twice the HBM write traffic.
//   T-planes (contraction over tokens,   k = token,   r = channel row): [ceil(rows/128)][KG(T)][128][8]
//   C-planes (contraction over channels, k = channel, r = token):       [ceil(T/128)][KG(rows)][128][8]
template <bool SRC_BF16>
__device__ __forceinline__ void load4(const void* src, long long off, float (&v)[4]) {
  if (SRC_BF16) {
    const uint2 w = *(const uint2*)((const unsigned short*)src + off);
    v[0] = __builtin_bit_cast(float, w.x << 16);
    v[1] = __builtin_bit_cast(float, w.x & 0xffff0000u);
    v[2] = __builtin_bit_cast(float, w.y << 16);
    v[3] = __builtin_bit_cast(float, w.y & 0xffff0000u);
  } else {
    const float4 a = *(const float4*)((const float*)src + off);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
  }
}

// T-planes: one block = one 128-row panel x 64 tokens (8 k-groups).  Phase 1 reads 4-token pieces (16 lanes cover
// the 64 tokens of a row, a wavefront 4 rows) and drops the fp16 halves into an LDS image of the output
// ([k-group][row][8], k-groups padded by one chunk against bank conflicts); phase 2 copies the image out linearly:
// the block's output is one contiguous 16 KB run per plane.
// WITH_C: the same pass also writes the C-planes of the block's 128 rows x 64 tokens from the LDS image (a chunk = one
// token's 8 consecutive rows, gathered as 2-byte reads; a wavefront stores 64 consecutive tokens of one row group =
// 1 KB contiguous).  relu_c on top of an image without relu: relu(x) has the planes of x where hi is not negative
// and zero planes elsewhere (hi carries the sign of x, also when it rounds to zero).
template <bool SRC_BF16, bool WITH_C>
__global__ __launch_bounds__(256) void split_t_kernel(const void* src, long long lds, const int* idx, int rows, long long T,
                                                      int relu, unsigned short* t_hi, unsigned short* t_lo, long long TGa,
                                                      int relu_c, unsigned short* c_hi, unsigned short* c_lo, int KGc,
                                                      int32_t* status) {
  constexpr int GP = 128 * 16 + 16;   // bytes per k-group in LDS
  bool bad = false;                   // a value the fp16 planes cannot hold: NaN, Inf or |x| > 65504
  __shared__ __attribute__((aligned(16))) unsigned char sh[8 * GP];
  __shared__ __attribute__((aligned(16))) unsigned char sl[8 * GP];
  const int t = threadIdx.x, piece = t & 15, rsub = t >> 4;
  const int pan = blockIdx.y;
  const long long tg0 = (long long)blockIdx.x * 8;
  const long long tok = tg0 * 8 + piece * 4;
  float v[8][4];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = pan * 128 + rsub + 16 * i;
#pragma unroll
    for (int c = 0; c < 4; ++c) v[i][c] = 0.0f;
    if (row < rows && tok < T) {
      const long long srow = idx ? (long long)idx[row] : (long long)row;
      load4<SRC_BF16>(src, srow * lds + tok, v[i]);
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int rr = rsub + 16 * i;
    unsigned short h[4], l[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      float x = (tok + c < T) ? v[i][c] : 0.0f;
      bad |= !(__builtin_fabsf(x) <= 65504.0f);
      if (relu) x = __builtin_fmaxf(x, 0.0f);
      sp_split_half(x, h[c], l[c]);
    }
    const int o = (piece >> 1) * GP + rr * 16 + (piece & 1) * 8;
    *(uint2*)(sh + o) = make_uint2(sp_pack2(h[0], h[1]), sp_pack2(h[2], h[3]));
    if (t_lo) *(uint2*)(sl + o) = make_uint2(sp_pack2(l[0], l[1]), sp_pack2(l[2], l[3]));
  }
  if (bad) atomicCAS(status, 0, (int32_t)STRP_ENONFINITE);
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int c = t + 256 * j, g = c >> 7, rr = c & 127;
    if (tg0 + g >= TGa) continue;
    const long long o = (((long long)pan * TGa + tg0 + g) * 128 + rr) * 8;
    *(uint4*)(t_hi + o) = *(const uint4*)(sh + g * GP + rr * 16);
    if (t_lo) *(uint4*)(t_lo + o) = *(const uint4*)(sl + g * GP + rr * 16);
  }
  if (WITH_C) {
    const long long tok_c = tg0 * 8 + (t & 63);                  // this thread's token
    if (tok_c < (((T + 127) >> 7) << 7)) {                        // inside the last token panel
      const int tl = t & 63;
      const unsigned char* bh = sh + (tl >> 3) * GP + (tl & 7) * 2;
      const unsigned char* bl = sl + (tl >> 3) * GP + (tl & 7) * 2;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int g = (t >> 6) + 4 * j;                           // row group of the panel (8 rows)
        const int rg = pan * 16 + g;
        if (rg >= KGc) continue;
        unsigned short h[8], l[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
          h[r] = *(const unsigned short*)(bh + (g * 8 + r) * 16);
          l[r] = c_lo ? *(const unsigned short*)(bl + (g * 8 + r) * 16) : (unsigned short)0;
          if (relu_c && (h[r] & 0x8000u)) h[r] = l[r] = 0;
        }
        const long long o = (((tok_c >> 7) * KGc + rg) * 128 + (tok_c & 127)) * 8;
        *(uint4*)(c_hi + o) = make_uint4(sp_pack2(h[0], h[1]), sp_pack2(h[2], h[3]), sp_pack2(h[4], h[5]), sp_pack2(h[6], h[7]));
        if (c_lo) *(uint4*)(c_lo + o) = make_uint4(sp_pack2(l[0], l[1]), sp_pack2(l[2], l[3]), sp_pack2(l[4], l[5]), sp_pack2(l[6], l[7]));
      }
    }
  }
}

// C-planes: thread = token, a chunk is that token's 8 consecutive channels; one block covers 256 tokens x 32
// channels (4 k-groups).  Every load of a row is 1 KB contiguous per wavefront, every store 1 KB contiguous.
template <bool SRC_BF16>
__global__ __launch_bounds__(256) void split_c_kernel(const void* src, long long lds, const int* idx, int rows, long long T,
                                                      int relu, unsigned short* c_hi, unsigned short* c_lo, int KGa,
                                                      int32_t* status) {
  const long long tok = (long long)blockIdx.x * 256 + threadIdx.x;
  const int rg0 = blockIdx.y * 4;
  if (tok >= (((T + 127) >> 7) << 7)) return;   // past the last token panel
  bool bad = false;
  float v[4][8];
#pragma unroll
  for (int g = 0; g < 4; ++g)
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const int row = (rg0 + g) * 8 + r;
      float x = 0.0f;
      if (row < rows && tok < T) {
        const long long srow = idx ? (long long)idx[row] : (long long)row;
        if (SRC_BF16) x = __builtin_bit_cast(float, (unsigned int)((const unsigned short*)src)[srow * lds + tok] << 16);
        else x = ((const float*)src)[srow * lds + tok];
      }
      bad |= !(__builtin_fabsf(x) <= 65504.0f);
      v[g][r] = relu ? __builtin_fmaxf(x, 0.0f) : x;
    }
  if (bad) atomicCAS(status, 0, (int32_t)STRP_ENONFINITE);
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    if (rg0 + g >= KGa) continue;
    unsigned short h[8], l[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) sp_split_half(v[g][r], h[r], l[r]);
    const long long o = (((tok >> 7) * KGa + rg0 + g) * 128 + (tok & 127)) * 8;
    *(uint4*)(c_hi + o) = make_uint4(sp_pack2(h[0], h[1]), sp_pack2(h[2], h[3]), sp_pack2(h[4], h[5]), sp_pack2(h[6], h[7]));
    if (c_lo) *(uint4*)(c_lo + o) = make_uint4(sp_pack2(l[0], l[1]), sp_pack2(l[2], l[3]), sp_pack2(l[4], l[5]), sp_pack2(l[6], l[7]));
  }
}

strp_status split_act(strp_ctx* ctx, const void* src, int src_dtype, long long lds, const int* idx, int rows, long long T,
                      int relu_t, int relu_c, unsigned short* t_hi, unsigned short* t_lo, unsigned short* c_hi,
                      unsigned short* c_lo) {
  if (rows <= 0 || T <= 0) return fail(ctx, STRP_EINVAL, "split_act: empty");
  if (!ctx->status_dev) return fail(ctx, STRP_ENOMEM, "split_act: no workspace set");
  if (lds % 8 || lds < T) return fail(ctx, STRP_EINVAL, "split_act: source pitch must be a multiple of 8 and at least T");
  const double es = src_dtype == STRP_BF16 ? 2.0 : 4.0;
  const double wb = (t_hi ? 2.0 : 0.0) + (t_lo ? 2.0 : 0.0) + (c_hi ? 2.0 : 0.0) + (c_lo ? 2.0 : 0.0);
  const bool one_read = t_hi && c_hi && (relu_t == relu_c || !relu_t) && (t_lo != nullptr) == (c_lo != nullptr);
  ProfScope ps(ctx, "split_act", 0.0, (es * (one_read ? 1.0 : (t_hi ? 1.0 : 0.0) + (c_hi ? 1.0 : 0.0)) + wb) * (double)rows * (double)T);
  // both layouts of the same rows in one pass over the source when the C-planes can be derived from the T image
  const bool fused = t_hi && c_hi && (relu_t == relu_c || !relu_t) && (t_lo != nullptr) == (c_lo != nullptr);
  if (t_hi) {
    const long long TGa = plane_kg(T);
    const int KGc = (int)plane_kg(rows);
    const int rc = fused ? (relu_c && !relu_t) : 0;
    // fused: the blocks reach the end of the last 128-token panel, whose padding the C-planes hold as zeros
    const long long gx = fused ? 2 * ((T + 127) / 128) : (TGa + 7) / 8;
    dim3 grid((unsigned)gx, (unsigned)((rows + 127) / 128));
    if (fused && src_dtype == STRP_BF16)
      hipLaunchKernelGGL((split_t_kernel<true, true>), grid, dim3(256), 0, ctx->stream, src, lds, idx, rows, T, relu_t, t_hi, t_lo, TGa, rc, c_hi, c_lo, KGc, ctx->status_dev);
    else if (fused)
      hipLaunchKernelGGL((split_t_kernel<false, true>), grid, dim3(256), 0, ctx->stream, src, lds, idx, rows, T, relu_t, t_hi, t_lo, TGa, rc, c_hi, c_lo, KGc, ctx->status_dev);
    else if (src_dtype == STRP_BF16)
      hipLaunchKernelGGL((split_t_kernel<true, false>), grid, dim3(256), 0, ctx->stream, src, lds, idx, rows, T, relu_t, t_hi, t_lo, TGa, 0,
                         (unsigned short*)nullptr, (unsigned short*)nullptr, 0, ctx->status_dev);
    else
      hipLaunchKernelGGL((split_t_kernel<false, false>), grid, dim3(256), 0, ctx->stream, src, lds, idx, rows, T, relu_t, t_hi, t_lo, TGa, 0,
                         (unsigned short*)nullptr, (unsigned short*)nullptr, 0, ctx->status_dev);
    STRP_HIP(ctx, hipGetLastError());
  }
  if (c_hi && !fused) {
    const int KGa = (int)plane_kg(rows);
    dim3 grid((unsigned)(((T + 127) / 128 * 128 + 255) / 256), (unsigned)((KGa + 3) / 4));
    if (src_dtype == STRP_BF16)
      hipLaunchKernelGGL((split_c_kernel<true>), grid, dim3(256), 0, ctx->stream, src, lds, idx, rows, T, relu_c, c_hi, c_lo, KGa, ctx->status_dev);
    else
      hipLaunchKernelGGL((split_c_kernel<false>), grid, dim3(256), 0, ctx->stream, src, lds, idx, rows, T, relu_c, c_hi, c_lo, KGa, ctx->status_dev);
    STRP_HIP(ctx, hipGetLastError());
  }
  return STRP_OK;
}

__device__ __forceinline__ double small_src(const double* s, long long i) { return s[i]; }
__device__ __forceinline__ double small_src(const float* s, long long i) { return (double)s[i]; }
__device__ __forceinline__ double small_src(const unsigned short* s, long long i) {
  return (double)__builtin_bit_cast(float, (unsigned int)s[i] << 16);
}


// Small matrices (weights): planes of src * scale with k = column (contraction), r = row:
// [ceil(rows/128)][ceil(cols/8)][128][8], zero padded.  transpose != 0 reads src[c][r].
// scale_dev (device, may be null = 1) is a power of two chosen by weight_scale.
// transpose == 2: src is symmetric and only its lower triangle is valid (reads src[max(r,c)][min(r,c)]).
template <typename TS>
__global__ __launch_bounds__(256) void split_small_kernel(const TS* src, long long lds, int rows, int cols, int transpose,
                                                          const float* scale_dev, unsigned short* hi, unsigned short* lo) {
  const int KG = (int)((((cols + 7) >> 3) + 3) & ~3);   // = plane_kg(cols)
  const long long total = (long long)((rows + 127) >> 7) * KG * 1024;
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  const int j = (int)(e & 7);
  const int rr = (int)((e >> 3) & 127);
  const long long pg = e >> 10;
  const int g = (int)(pg % KG), pan = (int)(pg / KG);
  const int r = pan * 128 + rr, c = g * 8 + j;
  double x = 0.0;
  if (r < rows && c < cols) {
    if (transpose == 2) x = r >= c ? small_src(src, (long long)r * lds + c) : small_src(src, (long long)c * lds + r);
    else x = transpose ? small_src(src, (long long)c * lds + r) : small_src(src, (long long)r * lds + c);
  }
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
                        const float* scale_dev, unsigned short* hi, unsigned short* lo) {
  const long long tot = (long long)plane_elems(rows, cols);
  dim3 grid((unsigned)((tot + 255) / 256)), block(256);
  if (src_kind == SRC_F64)
    hipLaunchKernelGGL((split_small_kernel<double>), grid, block, 0, ctx->stream, (const double*)src, lds, rows, cols, transpose, scale_dev, hi, lo);
  else if (src_kind == SRC_F32)
    hipLaunchKernelGGL((split_small_kernel<float>), grid, block, 0, ctx->stream, (const float*)src, lds, rows, cols, transpose, scale_dev, hi, lo);
  else
    hipLaunchKernelGGL((split_small_kernel<unsigned short>), grid, block, 0, ctx->stream, (const unsigned short*)src, lds, rows, cols, transpose, scale_dev, hi, lo);
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

// scale = 2^e with max|x| * scale in [2^11, 2^12): keeps fp16 hi far from overflow and lo out of the subnormals.
// Pass 1: grid-wide max of |x| through an integer atomic on the float bits (order-preserving for x >= 0).
template <typename TS>
__global__ __launch_bounds__(256) void absmax_kernel(const TS* src, long long lds, int rows, int cols, unsigned int* slot) {
  float m = 0.0f;
  for (int r = blockIdx.x; r < rows; r += gridDim.x) {   // a block walks whole rows: no division per element
    const TS* row = src + (long long)r * lds;
    // eight independent loads per trip keep enough requests in flight for a latency-bound reduction
    int c = threadIdx.x;
    for (; c + 7 * 256 < cols; c += 8 * 256) {
      float v[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) v[q] = (float)small_src(row, c + 256 * q);
#pragma unroll
      for (int q = 0; q < 8; ++q) m = __builtin_fmaxf(m, __builtin_fabsf(v[q]));
    }
    for (; c < cols; c += 256) m = __builtin_fmaxf(m, __builtin_fabsf((float)small_src(row, c)));
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = __builtin_fmaxf(m, __shfl_down(m, o, 64));
  // one atomic per block: thousands of atomics on one address serialise in L2 and were the whole run time
  __shared__ float wm[4];
  if ((threadIdx.x & 63) == 0) wm[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    m = __builtin_fmaxf(__builtin_fmaxf(wm[0], wm[1]), __builtin_fmaxf(wm[2], wm[3]));
    if (m > 0.0f) atomicMax(slot, __builtin_bit_cast(unsigned int, m));
  }
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
  long long blocks = rows < 1024 ? rows : 1024;
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

// ---------------------------------------------------------------------------------------------
// One fp16 plane with k = channel, r = token  ->  the same values as a plane with k = token, r = channel.
// A block moves 128 tokens x 128 channels: both its source (16 k-groups of one token panel) and its destination
// (16 k-groups of one channel panel) are contiguous 32 KB runs; the 2-byte transposition happens in LDS.
// Tokens >= T are written as zero (they are contraction padding on the output side).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void plane_c_to_t_kernel(const unsigned short* src, unsigned short* dst, int C, long long T,
                                                           long long kg_src, long long kg_dst) {
  constexpr int GS = 1024 + 8;                    // elements per source k-group in LDS (+16 B against bank conflicts)
  __shared__ __attribute__((aligned(16))) unsigned short sm[16 * GS];
  const int tid = threadIdx.x;
  const long long pt = blockIdx.x;                // token panel
  const int pc = blockIdx.y;                      // channel panel
  // load: source k-groups 16 pc .. 16 pc + 15 (those below kg_src) of token panel pt
  for (int q = tid; q < 2048; q += 256) {
    const int g = q >> 7, piece = q & 127;        // 128 16-byte pieces (one token each) per k-group
    const long long cg = (long long)pc * 16 + g;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (cg < kg_src) v = *(const uint4*)(src + ((pt * kg_src + cg) * 128 + piece) * 8);
    *(uint4*)(sm + g * GS + piece * 8) = v;
  }
  __syncthreads();
  // store: destination k-groups 16 pt .. 16 pt + 15 (those below kg_dst) of channel panel pc
  for (int q = tid; q < 2048; q += 256) {
    const int tg = q >> 7, cl = q & 127;          // piece = channel cl, token group tg
    const long long tgg = pt * 16 + tg;
    if (tgg >= kg_dst) continue;
    const unsigned short* col = sm + (cl >> 3) * GS + (cl & 7);
    unsigned short e[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const long long t = tgg * 8 + j;
      e[j] = t < T ? col[(tg * 8 + j) * 8] : (unsigned short)0;
    }
    uint4 v;
    v.x = e[0] | ((unsigned)e[1] << 16);
    v.y = e[2] | ((unsigned)e[3] << 16);
    v.z = e[4] | ((unsigned)e[5] << 16);
    v.w = e[6] | ((unsigned)e[7] << 16);
    *(uint4*)(dst + (((long long)pc * kg_dst + tgg) * 128 + cl) * 8) = v;
  }
  (void)C;
}

strp_status plane_c_to_t(strp_ctx* ctx, const unsigned short* src, unsigned short* dst, int C, long long T) {
  ProfScope ps(ctx, "plane_c_to_t", 0.0, 4.0 * (double)C * (double)T);
  dim3 grid((unsigned)((T + 127) / 128), (unsigned)((C + 127) / 128));
  hipLaunchKernelGGL(plane_c_to_t_kernel, grid, dim3(256), 0, ctx->stream, src, dst, C, T, plane_kg(C), plane_kg(T));
  STRP_HIP(ctx, hipGetLastError());
  return STRP_OK;
}

}  // namespace strp
