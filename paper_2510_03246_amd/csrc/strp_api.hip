// C ABI of libstrp.so: argument validation, workspace carving and the per-module ADMM drivers.
#include <stdarg.h>

#include <cmath>
#include <new>
#include <string>
#include <vector>

#include "cojob.h"
#include "strp_internal.h"

struct Profiler {
  struct Rec { const char* name; double flops, bytes; hipEvent_t e0, e1; };
  bool on = false;
  std::vector<Rec> recs;
  std::vector<hipEvent_t> pool;
  hipEvent_t get() {
    if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
  void clear() {
    for (auto& r : recs) { pool.push_back(r.e0); pool.push_back(r.e1); }
    recs.clear();
  }
  ~Profiler() {
    clear();
    for (auto e : pool) if (e) (void)hipEventDestroy(e);
  }
};

// Scratch of strp_mask_topk_static (the entry point for callers that cannot allocate): per-block histograms, candidate
// lists and counters of the multi-block select, for up to STRP_TOPK_STATIC_MAX_N scores.  Every GPU the library runs on
// holds its own copy of the array until the process ends; in host code the array's name is only a handle for
// hipGetSymbolAddress, the device address is resolved once per device in strp_create and kept in g_topk_scratch.
constexpr size_t TOPK_STATIC_BYTES = 16 * (size_t)STRP_TOPK_STATIC_MAX_N + (8u << 20);
static __device__ __align__(256) unsigned char topk_static_scratch[TOPK_STATIC_BYTES];
constexpr int MAX_DEVICES = 64;
static void* g_topk_scratch[MAX_DEVICES];

namespace strp {

int prof_begin(strp_ctx* ctx, const char* name, double flops, double bytes) {
  Profiler* pr = ctx->prof;
  if (!pr || !pr->on) return -1;
  Profiler::Rec r{name, flops, bytes, pr->get(), pr->get()};
  if (!r.e0 || !r.e1) return -1;
  (void)hipEventRecord(r.e0, ctx->stream);
  pr->recs.push_back(r);
  return (int)pr->recs.size() - 1;
}
void prof_end(strp_ctx* ctx, int rec) {
  if (rec < 0) return;
  (void)hipEventRecord(ctx->prof->recs[rec].e1, ctx->stream);
}

strp_status fail(strp_ctx* ctx, strp_status st, const char* fmt, ...) {
  if (ctx) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
    va_end(ap);
  }
  return st;
}

static inline long long round_up(long long x, long long a) { return (x + a - 1) / a * a; }
static inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// ---- small kernels ------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void add_diag_kernel(double* A, long long ld, int n, double lam, const double* lam_dev) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) A[(long long)i * ld + i] += lam_dev ? *lam_dev : lam;
}

// out[0] = scale * sum(v[0..n)) (single block, fixed order)
__global__ __launch_bounds__(256) void vec_sum_kernel(const double* v, int n, double scale, double* out, double* raw) {
  __shared__ double s[256];
  double a = 0.0;
  for (int i = threadIdx.x; i < n; i += 256) a += v[i];
  s[threadIdx.x] = a;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) s[threadIdx.x] += s[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    if (raw) *raw = s[0];
    *out = s[0] * scale;
  }
}

// dst[r][c] (fp32, ld ldd, zero padded) = W[r][idx[c]]  (kept columns of fc2)
__global__ __launch_bounds__(256) void gather_cols_kernel(const float* W, int rows, int in, const int32_t* idx, int s, float* dst,
                                                          long long ldd) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= (long long)rows * ldd) return;
  const int r = (int)(e / ldd), c = (int)(e % ldd);
  dst[e] = c < s ? W[(long long)r * in + idx[c]] : 0.0f;
}
// dst[r][c] = W[idx[r]][c]  (kept rows of fc1)
__global__ __launch_bounds__(256) void gather_rows_kernel(const float* W, int in, const int32_t* idx, int s, float* dst, long long ldd) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= (long long)s * ldd) return;
  const int r = (int)(e / ldd), c = (int)(e % ldd);
  dst[e] = c < in ? W[(long long)idx[r] * in + c] : 0.0f;
}
// dst[c][r] (fp64, ld ldd) = src[r][c] (fp32, ld lds): r < rows, c < cols
__global__ __launch_bounds__(256) void transpose_f32_f64_kernel(const float* src, long long lds, int rows, int cols, double* dst,
                                                                long long ldd) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= (long long)rows * cols) return;
  const int c = (int)(e / rows), r = (int)(e % rows);
  dst[(long long)c * ldd + r] = (double)src[(long long)r * lds + c];
}

// The per-element rules of the pruned rows (pruned_elem) are in cojob.h.
// rowsums (phase 2 only, may be null): the scoring sums of the row's NEW state, [0][j] = sum A^2 and, when Z0 is
// given, [1][j] = sum A relu(Z0), [2][j] = sum Z0 Z, [3][j] = sum Z0^2, so that the next selection does not have
// to stream the pruned rows again.
__global__ __launch_bounds__(256) void pruned_rows_kernel(const uint8_t* mask, float* Z, float* A, long long lda, long long T, int phase,
                                                          float alpha, float beta, int write, double* red, const float* Z0,
                                                          double* rowsums, int rows) {
  const int j = blockIdx.x;
  double r0 = 0.0, r1 = 0.0;
  double sg = 0.0, se = 0.0, su = 0.0, sv = 0.0;
  const bool pruned = !mask[j];
  if (pruned) {
    float* z = Z + (long long)j * lda;
    float* a = A + (long long)j * lda;
    const float* z0 = Z0 ? Z0 + (long long)j * lda : nullptr;
    const long long T4 = T >> 2;
    // two independent 16-byte groups per thread and trip: all loads of a trip are issued before its first store
    auto body = [&](long long c, float4 zv, float4 av, float4 w) {
      pruned_elem(zv.x, av.x, phase, alpha, beta, write, r0, r1);
      pruned_elem(zv.y, av.y, phase, alpha, beta, write, r0, r1);
      pruned_elem(zv.z, av.z, phase, alpha, beta, write, r0, r1);
      pruned_elem(zv.w, av.w, phase, alpha, beta, write, r0, r1);
      if (phase != 1) ((float4*)a)[c] = av;
      if (phase != 0 && write) ((float4*)z)[c] = zv;
      if (rowsums) {
        const float aa[4] = {av.x, av.y, av.z, av.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) sg = __builtin_fma((double)aa[q], (double)aa[q], sg);
        if (z0) {
          const float wa[4] = {w.x, w.y, w.z, w.w}, za[4] = {zv.x, zv.y, zv.z, zv.w};
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const double z0d = wa[q];
            se = __builtin_fma((double)aa[q], fmax(z0d, 0.0), se);
            su = __builtin_fma(z0d, (double)za[q], su);
            sv = __builtin_fma(z0d, z0d, sv);
          }
        }
      }
    };
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
    long long c = threadIdx.x;
    for (; c + 256 < T4; c += 512) {
      const float4 zv0 = ((const float4*)z)[c], zv1 = ((const float4*)z)[c + 256];
      const float4 av0 = phase == 1 ? ((const float4*)a)[c] : zero4, av1 = phase == 1 ? ((const float4*)a)[c + 256] : zero4;
      const float4 w0 = z0 ? ((const float4*)z0)[c] : zero4, w1 = z0 ? ((const float4*)z0)[c + 256] : zero4;
      body(c, zv0, av0, w0);
      body(c + 256, zv1, av1, w1);
    }
    if (c < T4) body(c, ((const float4*)z)[c], phase == 1 ? ((const float4*)a)[c] : zero4, z0 ? ((const float4*)z0)[c] : zero4);
    for (long long t = T4 * 4 + threadIdx.x; t < T; t += 256) {
      float zv = z[t], av = phase == 1 ? a[t] : 0.0f;
      pruned_elem(zv, av, phase, alpha, beta, write, r0, r1);
      if (phase != 1) a[t] = av;
      if (phase != 0 && write) z[t] = zv;
      if (rowsums) {
        sg = __builtin_fma((double)av, (double)av, sg);
        if (z0) {
          const double z0d = z0[t];
          se = __builtin_fma((double)av, fmax(z0d, 0.0), se);
          su = __builtin_fma(z0d, (double)zv, su);
          sv = __builtin_fma(z0d, z0d, sv);
        }
      }
    }
  }
  if (red || rowsums) {
    __shared__ double sh[4][6];
    for (int o = 32; o > 0; o >>= 1) {
      r0 += __shfl_down(r0, o, 64);
      r1 += __shfl_down(r1, o, 64);
      if (rowsums) {
        sg += __shfl_down(sg, o, 64);
        se += __shfl_down(se, o, 64);
        su += __shfl_down(su, o, 64);
        sv += __shfl_down(sv, o, 64);
      }
    }
    if ((threadIdx.x & 63) == 0) {
      double* w = sh[threadIdx.x >> 6];
      w[0] = r0; w[1] = r1; w[2] = sg; w[3] = se; w[4] = su; w[5] = sv;
    }
    __syncthreads();
    if (threadIdx.x < 6) {
      const int q = threadIdx.x;
      const double t = sh[0][q] + sh[1][q] + sh[2][q] + sh[3][q];
      if (q < 2) {
        if (red) red[2 * (long long)j + q] = t;
      } else if (rowsums && pruned && (q == 2 || Z0)) {
        rowsums[(long long)(q - 2) * rows + j] = t;
      }
    }
  }
}

// ---- the fused a/z pass of the pruned rows as a ride-along job (cojob.h) ---------------------------------------------
// rows[0 .. f - s) = the rows with mask == 0, ascending (one block; f is a few ten thousand at most)
__global__ __launch_bounds__(1024) void pruned_list_kernel(const uint8_t* mask, int f, int32_t* rows) {
  __shared__ int scan[1024];
  const int tid = threadIdx.x;
  const int per = (f + 1023) / 1024;
  const int j0 = tid * per, j1 = (j0 + per < f) ? j0 + per : f;
  int cnt = 0;
  for (int j = j0; j < j1; ++j) cnt += mask[j] ? 0 : 1;
  scan[tid] = cnt;
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {
    const int v = tid >= o ? scan[tid - o] : 0;
    __syncthreads();
    scan[tid] += v;
    __syncthreads();
  }
  int pos = scan[tid] - cnt;
  for (int j = j0; j < j1; ++j)
    if (!mask[j]) rows[pos++] = j;
  // entries past the last pruned row name no row (a unit of such an entry does nothing): the job's row count comes
  // from the host's record of the kept count, which a caller-supplied mask need not match
  const int total = scan[1023];
  for (int j = total + tid; j < f; j += 1024) rows[j] = -1;
}

// takes units until none are left
__global__ __launch_bounds__(256) void cojob_drain_kernel(const CoJob job) {
  __shared__ unsigned int u0s;
  for (;;) {
    if (threadIdx.x == 0) u0s = atomicAdd(job.ticket, (unsigned int)job.take);
    __syncthreads();
    const unsigned int u0 = u0s;
    if (u0 >= job.units) return;
    for (int i = 0; i < job.take; ++i) {
      if (u0 + i >= job.units) break;
      cojob_unit(job, u0 + i);   // ends with a barrier: u0s may be rewritten afterwards
    }
  }
}

// per pruned row: the units' sums added in segment order -> red[2 j], red[2 j + 1] and the row's scoring sums
__global__ __launch_bounds__(256) void cojob_finish_kernel(const CoJob job, double* red, double* rowsums, int f) {
  const int p = blockIdx.x * 256 + threadIdx.x;
  if (p >= job.nrows) return;
  const int j = job.rows[p];
  double t[6] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
  const double* src = job.partial + (unsigned long long)p * job.segs * 6;
  for (int g = 0; g < job.segs; ++g)
#pragma unroll
    for (int q = 0; q < 6; ++q) t[q] += src[g * 6 + q];
  red[2 * (long long)j] = t[0];
  red[2 * (long long)j + 1] = t[1];
  if (rowsums) {
    rowsums[j] = t[2];
    if (job.Z0) {
      rowsums[(long long)f + j] = t[3];
      rowsums[2 * (long long)f + j] = t[4];
      rowsums[3 * (long long)f + j] = t[5];
    }
  }
}

// per-block sum of squares of an fp32 array -> red[block][0] (red[block][1] = 0)
__global__ __launch_bounds__(256) void sumsq_kernel(const float* x, long long n, double* red) {
  double a = 0.0;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256) a += (double)x[i] * (double)x[i];
  __shared__ double sh[4];
  for (int o = 32; o > 0; o >>= 1) a += __shfl_down(a, o, 64);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) {
    red[2 * (long long)blockIdx.x] = sh[0] + sh[1] + sh[2] + sh[3];
    red[2 * (long long)blockIdx.x + 1] = 0.0;
  }
}

// per-block partial of sum_i a[i] b[i] -> red[block][0] (red[block][1] = 0)
__global__ __launch_bounds__(256) void dot_f32_f64_kernel(const float* a, const double* b, long long n, double* red) {
  double acc = 0.0;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256) acc = __builtin_fma((double)a[i], b[i], acc);
  __shared__ double sh[4];
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_down(acc, o, 64);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    red[2 * (long long)blockIdx.x] = sh[0] + sh[1] + sh[2] + sh[3];
    red[2 * (long long)blockIdx.x + 1] = 0.0;
  }
}

// scalars[dst] = a * scalars[s0] + b * scalars[s1]   (one thread; keeps the objective assembly on device)
__global__ void axpby_scalar_kernel(double* sc, int dst, double a, int s0, double b, int s1) {
  if (threadIdx.x == 0 && blockIdx.x == 0) sc[dst] = a * sc[s0] + (s1 >= 0 ? b * sc[s1] : 0.0);
}

static unsigned blocks_for(long long n) { return (unsigned)((n + 255) / 256); }

// scalar slots of strp_module_state::scalars
// bits of strp_module_state::sums_cached: which token sums cv.rowsums holds for EVERY row of the current state
enum { SUMS_G = 1, SUMS_EU = 2, SUMS_V = 4 };
enum { SC_LAM1 = 0, SC_LAM2 = 1, SC_SUMA0 = 2, SC_TRH = 3, SC_T1 = 4, SC_T2 = 5, SC_T3 = 6, SC_T4 = 7, SC_T5 = 8,
       SC_TAU = 9, SC_ENERGY = 10, SC_TMP0 = 11, SC_TMP1 = 12, SC_TMP2 = 13, SC_TMP3 = 14, SC_W2SQ = 15, SC_W1SQ = 16, SC_COUNT = 32 };

static strp_status check_desc(strp_ctx* ctx, const strp_module_desc* d) {
  if (!d) return fail(ctx, STRP_EINVAL, "null module descriptor");
  if (d->d <= 0 || d->f <= 0 || d->T <= 0) return fail(ctx, STRP_EINVAL, "module: d, f, T must be positive");
  if (d->ldx < d->T || d->lda < d->T) return fail(ctx, STRP_EINVAL, "module: leading dimension below T");
  if (d->ldx % 8 || d->lda % 8 || d->d % 8 || d->f % 8) return fail(ctx, STRP_EINVAL, "module: d, f and leading dimensions must be multiples of 8");
  if ((d->x_dtype != STRP_BF16 && d->x_dtype != STRP_F32) || (d->w_dtype != STRP_BF16 && d->w_dtype != STRP_F32))
    return fail(ctx, STRP_EINVAL, "module: unknown dtype");
  if (d->k_max < 0 || d->k_max > d->f) return fail(ctx, STRP_EINVAL, "module: k_max outside [0, f]");
  return STRP_OK;
}

}  // namespace strp

using namespace strp;

extern "C" {

strp_status strp_create(strp_ctx** out, int device, void* hip_stream) {
  if (!out) return STRP_EINVAL;
  *out = nullptr;
  int count = 0;
  if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return STRP_EHIP;
  if (hipSetDevice(device) != hipSuccess) return STRP_EHIP;
  strp_ctx* c = new (std::nothrow) strp_ctx();
  if (!c) return STRP_ENOMEM;
  memset(c, 0, sizeof(*c));
  c->device = device;
  c->stream = (hipStream_t)hip_stream;
  c->precision = STRP_PREC_SPLIT;
  for (int i = 0; i < 8; ++i) c->prod_planes[i][0] = c->prod_planes[i][1] = 2;
  if (hipHostMalloc(&c->pinned, 4096, hipHostMallocDefault) != hipSuccess) {
    delete c;
    return STRP_EHIP;
  }
  // device address of this GPU's copy of the static select scratch (the device was made current above)
  if (device < MAX_DEVICES && !g_topk_scratch[device]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(topk_static_scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      (void)hipHostFree(c->pinned);
      delete c;
      return STRP_EHIP;
    }
    g_topk_scratch[device] = ptr;
  }
  *out = c;
  return STRP_OK;
}

strp_status strp_destroy(strp_ctx* ctx) {
  if (!ctx) return STRP_EINVAL;
  if (ctx->pinned) (void)hipHostFree(ctx->pinned);
  delete ctx->prof;
  delete ctx;
  return STRP_OK;
}

const char* strp_last_error(const strp_ctx* ctx) { return ctx ? ctx->err : "null context"; }

strp_status strp_set_precision(strp_ctx* ctx, strp_precision prec) {
  if (!ctx) return STRP_EINVAL;
  if (prec != STRP_PREC_FAST && prec != STRP_PREC_SPLIT) return fail(ctx, STRP_EINVAL, "unknown precision %d", (int)prec);
  ctx->precision = prec;
  return STRP_OK;
}

strp_status strp_set_product_planes(strp_ctx* ctx, strp_product product, int32_t planes_p, int32_t planes_q) {
  if (!ctx) return STRP_EINVAL;
  if (product < 0 || product >= STRP_PROD_COUNT || planes_p < 1 || planes_p > 2 || planes_q < 1 || planes_q > 2)
    return fail(ctx, STRP_EINVAL, "set_product_planes: product in [0, %d), planes 1 or 2", (int)STRP_PROD_COUNT);
  ctx->prod_planes[product][0] = (unsigned char)planes_p;
  ctx->prod_planes[product][1] = (unsigned char)planes_q;
  return STRP_OK;
}

strp_status strp_profile_enable(strp_ctx* ctx, int on) {
  if (!ctx) return STRP_EINVAL;
  if (!ctx->prof) ctx->prof = new (std::nothrow) Profiler();
  if (!ctx->prof) return fail(ctx, STRP_ENOMEM, "profile: host allocation failed");
  STRP_HIP(ctx, hipStreamSynchronize(ctx->stream));
  ctx->prof->clear();
  ctx->prof->on = on != 0;
  return STRP_OK;
}

strp_status strp_profile_read(strp_ctx* ctx, strp_profile_entry* out_host, int32_t max_entries, int32_t* n_out) {
  if (!ctx || !out_host || !n_out || max_entries <= 0) return ctx ? fail(ctx, STRP_EINVAL, "profile_read: bad argument") : STRP_EINVAL;
  *n_out = 0;
  if (!ctx->prof) return STRP_OK;
  STRP_HIP(ctx, hipStreamSynchronize(ctx->stream));
  int n = 0;
  for (auto& r : ctx->prof->recs) {
    float ms = 0.0f;
    if (hipEventElapsedTime(&ms, r.e0, r.e1) != hipSuccess) continue;
    int j = 0;
    for (; j < n; ++j)
      if (strncmp(out_host[j].name, r.name, sizeof(out_host[j].name)) == 0) break;
    if (j == n) {
      if (n == max_entries) continue;
      memset(&out_host[n], 0, sizeof(out_host[n]));
      strncpy(out_host[n].name, r.name, sizeof(out_host[n].name) - 1);
      ++n;
    }
    out_host[j].launches += 1;
    out_host[j].ms += ms;
    out_host[j].flops += r.flops;
    out_host[j].bytes += r.bytes;
  }
  *n_out = n;
  return STRP_OK;
}

strp_status strp_profile_launches(strp_ctx* ctx, strp_profile_entry* out_host, int32_t max_entries, int32_t* n_out) {
  if (!ctx || !out_host || !n_out || max_entries <= 0) return ctx ? fail(ctx, STRP_EINVAL, "profile_launches: bad argument") : STRP_EINVAL;
  *n_out = 0;
  if (!ctx->prof) return STRP_OK;
  STRP_HIP(ctx, hipStreamSynchronize(ctx->stream));
  int n = 0;
  for (auto& r : ctx->prof->recs) {
    if (n == max_entries) break;
    float ms = 0.0f;
    if (hipEventElapsedTime(&ms, r.e0, r.e1) != hipSuccess) ms = -1.0f;
    memset(&out_host[n], 0, sizeof(out_host[n]));
    strncpy(out_host[n].name, r.name, sizeof(out_host[n].name) - 1);
    out_host[n].launches = 1;
    out_host[n].ms = ms;
    out_host[n].flops = r.flops;
    out_host[n].bytes = r.bytes;
    ++n;
  }
  *n_out = n;
  return STRP_OK;
}

strp_status strp_set_workspace(strp_ctx* ctx, void* dev_ptr, size_t bytes) {
  if (!ctx) return STRP_EINVAL;
  if (!dev_ptr || bytes < 4096) return fail(ctx, STRP_EINVAL, "workspace: null or smaller than 4096 bytes");
  if ((uintptr_t)dev_ptr & 255u) return fail(ctx, STRP_EINVAL, "workspace: pointer not 256-byte aligned");
  ctx->ws = (char*)dev_ptr;
  ctx->ws_bytes = bytes;
  ctx->status_dev = (int32_t*)dev_ptr;
  return fill_zero(ctx, dev_ptr, 256);
}

strp_status strp_poll(strp_ctx* ctx) {
  if (!ctx) return STRP_EINVAL;
  if (!ctx->ws) return fail(ctx, STRP_ENOMEM, "no workspace set");
  STRP_HIP(ctx, hipMemcpyAsync(ctx->pinned, ctx->status_dev, sizeof(int32_t), hipMemcpyDeviceToHost, ctx->stream));
  STRP_HIP(ctx, hipStreamSynchronize(ctx->stream));
  const int32_t st = *(int32_t*)ctx->pinned;
  if (st != 0) {
    fail(ctx, (strp_status)st, "device status word = %d", st);
    STRP_TRY(fill_zero(ctx, ctx->status_dev, 256));
  }
  return (strp_status)st;
}

strp_status strp_score_alloc(strp_ctx* ctx, const strp_score_in* in, float* unit_score, double* energies, int32_t layer_idx,
                             int32_t L, const int32_t* n_units, const int32_t* group_id, double rbar, double temperature,
                             double rmax, double* r_out, int32_t* nprune_out) {
  if (!ctx) return STRP_EINVAL;
  if (!in || !unit_score || !energies) return fail(ctx, STRP_EINVAL, "score_alloc: null argument");
  if (!in->A || in->n_channels <= 0 || in->group <= 0 || in->T <= 0) return fail(ctx, STRP_EINVAL, "score_alloc: bad input block");
  if (in->n_channels % in->group) return fail(ctx, STRP_EINVAL, "score_alloc: n_channels %% group != 0");
  if (in->ld < in->T || in->ld % 8 || !aligned16(in->A)) return fail(ctx, STRP_EINVAL, "score_alloc: bad leading dimension or alignment");
  if (in->mode < STRP_SCORE_WANDA || in->mode > STRP_SCORE_GAIN) return fail(ctx, STRP_EINVAL, "score_alloc: unknown mode");
  if (in->mode != STRP_SCORE_WANDA && (!in->Z || !in->Z0)) return fail(ctx, STRP_EINVAL, "score_alloc: LEMMA/GAIN need Z and Z0");
  if (!in->n2 && !in->What) return fail(ctx, STRP_EINVAL, "score_alloc: need n2 or What");
  if (L <= 0 || layer_idx < 0 || layer_idx >= L) return fail(ctx, STRP_EINVAL, "score_alloc: layer_idx outside [0, L)");
  if (r_out && (!nprune_out || !n_units)) return fail(ctx, STRP_EINVAL, "score_alloc: allocation needs n_units and nprune_out");
  if (r_out && (!(temperature > 0.0) || !(rbar >= 0.0) || !(rmax > 0.0))) return fail(ctx, STRP_EINVAL, "score_alloc: bad rbar/temperature/rmax");
  if (!ctx->ws) return fail(ctx, STRP_ENOMEM, "score_alloc: no workspace set");
  Arena arena(ctx);
  STRP_TAKE(ctx, arena, sums, double, 4 * (size_t)in->n_channels);
  const double* n2 = in->n2;
  if (!n2) {
    STRP_TAKE(ctx, arena, n2buf, double, (size_t)in->n_channels);
    STRP_TRY(launch_colnorm2(ctx, in->What, in->w_dtype, in->w_rows, in->n_channels, in->ldw, n2buf));
    n2 = n2buf;
  }
  STRP_TRY(launch_row_sums(ctx, in->A, in->a_dtype, in->Z, in->Z0, in->ld, in->T, in->n_channels, in->mode, sums));
  STRP_TRY(launch_unit_scores(ctx, sums, n2, in->n_channels, in->group, in->mode, unit_score, energies + layer_idx));
  if (r_out) STRP_TRY(launch_alloc(ctx, energies, L, n_units, group_id, rbar, temperature, rmax, 0, r_out, nprune_out));
  return STRP_OK;
}

strp_status strp_mask_topk(strp_ctx* ctx, const float* score, int32_t n, int32_t k, int32_t group, uint8_t* mask, int32_t* idx,
                           float* tau) {
  if (!ctx) return STRP_EINVAL;
  if (!score || !mask || !idx) return fail(ctx, STRP_EINVAL, "mask_topk: null argument");
  if (n <= 0 || k < 0 || k > n || group <= 0) return fail(ctx, STRP_EINVAL, "mask_topk: need n > 0, 0 <= k <= n, group > 0");
  const size_t need = (group == 1 && k > 0 && k < n) ? topk_scratch_bytes(n) : 0;
  void* scratch = nullptr;
  if (need) {
    Arena arena(ctx);
    scratch = arena.take(need);
    if (!scratch) return fail(ctx, STRP_ENOMEM, "mask_topk: %d scores need %zu bytes of workspace (strp_topk_workspace_bytes)", n, need + 256);
  }
  return launch_topk(ctx, score, n, k, group, mask, idx, tau, scratch, need);
}

strp_status strp_weight_energy(strp_ctx* ctx, const strp_weight_ref* mats, int32_t n_mats, double var_coef, double l2_coef,
                               double scale, double* energy) {
  if (!ctx) return STRP_EINVAL;
  if (!mats || n_mats <= 0 || !energy) return fail(ctx, STRP_EINVAL, "weight_energy: null or empty matrix list");
  for (int i = 0; i < n_mats; ++i) {
    const strp_weight_ref& m = mats[i];
    if (!m.W || m.rows <= 0 || m.cols <= 0 || m.ld < m.cols) return fail(ctx, STRP_EINVAL, "weight_energy: bad matrix %d", i);
    if (m.dtype != STRP_BF16 && m.dtype != STRP_F32) return fail(ctx, STRP_EINVAL, "weight_energy: unknown dtype");
  }
  Arena arena(ctx);
  STRP_TAKE(ctx, arena, partial, double, weight_energy_scratch_bytes() / sizeof(double));
  return launch_weight_energy(ctx, mats, n_mats, var_coef, l2_coef, scale, energy, partial);
}

strp_status strp_alloc_inverse(strp_ctx* ctx, const double* energies, int32_t L, const int32_t* n_units, const int32_t* group_id,
                               double rbar, double temperature, double rmax, double* r_out, int32_t* nprune_out) {
  if (!ctx) return STRP_EINVAL;
  if (!energies || !n_units || !r_out || !nprune_out) return fail(ctx, STRP_EINVAL, "alloc_inverse: null argument");
  if (L <= 0) return fail(ctx, STRP_EINVAL, "alloc_inverse: L must be positive");
  if (!(temperature > 0.0) || !(rbar >= 0.0 && rbar <= 1.0) || !(rmax > 0.0 && rmax <= 1.0))
    return fail(ctx, STRP_EINVAL, "alloc_inverse: need temperature > 0, 0 <= rbar <= 1, 0 < rmax <= 1");
  return launch_alloc(ctx, energies, L, n_units, group_id, rbar, temperature, rmax, 1, r_out, nprune_out);
}

strp_status strp_alloc_softmax(strp_ctx* ctx, const double* energies, int32_t L, const int32_t* n_units, const int32_t* group_id,
                               double rbar, double temperature, double rmax, double* r_out, int32_t* nprune_out) {
  if (!ctx) return STRP_EINVAL;
  if (!energies || !n_units || !r_out || !nprune_out) return fail(ctx, STRP_EINVAL, "alloc_softmax: null argument");
  if (L <= 0) return fail(ctx, STRP_EINVAL, "alloc_softmax: L must be positive");
  if (!(temperature > 0.0) || !(rbar >= 0.0 && rbar <= 1.0) || !(rmax > 0.0 && rmax <= 1.0))
    return fail(ctx, STRP_EINVAL, "alloc_softmax: need temperature > 0, 0 <= rbar <= 1, 0 < rmax <= 1");
  return launch_alloc(ctx, energies, L, n_units, group_id, rbar, temperature, rmax, 0, r_out, nprune_out);
}

size_t strp_topk_workspace_bytes(int32_t n) { return n > 0 ? topk_scratch_bytes(n) + 512 : 0; }

strp_status strp_mask_topk_static(strp_ctx* ctx, const float* score, int32_t n, int32_t k, uint8_t* mask, int32_t* idx, float* tau) {
  if (!ctx) return STRP_EINVAL;
  if (!score || !mask || !idx) return fail(ctx, STRP_EINVAL, "mask_topk_static: null argument");
  if (n <= 0 || k < 0 || k > n) return fail(ctx, STRP_EINVAL, "mask_topk_static: need n > 0 and 0 <= k <= n");
  if (n > STRP_TOPK_STATIC_MAX_N)
    return fail(ctx, STRP_EINVAL, "mask_topk_static: %d scores exceed the static scratch (at most %d); use strp_mask_topk with a workspace",
                n, (int)STRP_TOPK_STATIC_MAX_N);
  const size_t need = (k > 0 && k < n) ? topk_scratch_bytes(n) : 0;
  if (need > TOPK_STATIC_BYTES) return fail(ctx, STRP_EINVAL, "mask_topk_static: %zu bytes of scratch needed, %zu held", need, TOPK_STATIC_BYTES);
  void* scratch = ctx->device < MAX_DEVICES ? g_topk_scratch[ctx->device] : nullptr;
  if (need && !scratch) return fail(ctx, STRP_ESTATE, "mask_topk_static: no static scratch resolved for device %d", ctx->device);
  // no timing records here: they would create HIP events
  Profiler* pr = ctx->prof;
  const bool was_on = pr && pr->on;
  if (pr) pr->on = false;
  const strp_status st = launch_topk(ctx, score, n, k, 1, mask, idx, tau, scratch, need);
  if (pr) pr->on = was_on;
  return st;
}

}  // extern "C"

namespace strp {

static inline int planes_for(int dtype, int prec) { return (dtype == STRP_F32 && prec == STRP_PREC_SPLIT) ? 2 : 1; }
// the operand as product `prod` of strp_admm_step is set to see it: without its lo plane when one plane was asked for
static inline PlaneOp operand_for(const strp_ctx* ctx, int prod, int side, const PlaneOp& op) {
  PlaneOp o = op;
  if (ctx->prod_planes[prod][side] < 2) o.lo = nullptr;
  return o;
}

// Planes of `rows` (optionally gathered) activation rows for a product that contracts over the tokens.
static strp_status make_t_planes(strp_ctx* ctx, Arena& arena, const void* src, int dtype, long long lds, const int* idx, int rows,
                                 long long T, int relu, int np, PlaneOp* out) {
  const size_t n = plane_elems(rows, T);
  STRP_TAKE(ctx, arena, hi, unsigned short, n);
  unsigned short* lo = nullptr;
  if (np == 2) {
    STRP_TAKE(ctx, arena, lo2, unsigned short, n);
    lo = lo2;
  }
  STRP_TRY(split_act(ctx, src, dtype, lds, idx, rows, T, relu, 0, hi, lo, nullptr, nullptr));
  *out = PlaneOp{hi, lo, plane_kg(T), (rows + 127) / 128, nullptr};
  return STRP_OK;
}

// Planes of `rows` (optionally gathered) activation rows for a product that contracts over those rows.
static strp_status make_c_planes(strp_ctx* ctx, Arena& arena, const void* src, int dtype, long long lds, const int* idx, int rows,
                                 long long T, int relu, int np, PlaneOp* out) {
  const size_t n = plane_elems(T, rows);
  STRP_TAKE(ctx, arena, hi, unsigned short, n);
  unsigned short* lo = nullptr;
  if (np == 2) {
    STRP_TAKE(ctx, arena, lo2, unsigned short, n);
    lo = lo2;
  }
  STRP_TRY(split_act(ctx, src, dtype, lds, idx, rows, T, 0, relu, nullptr, nullptr, hi, lo));
  *out = PlaneOp{hi, lo, plane_kg(rows), (int)((T + 127) / 128), nullptr};
  return STRP_OK;
}

// Planes of a small matrix (weights; k = column, r = row), scaled by a device-chosen power of two.
static strp_status make_weight_planes(strp_ctx* ctx, Arena& arena, const void* src, int src_kind, long long lds, int rows, int cols,
                                      int transpose, int np, PlaneOp* out) {
  const size_t n = plane_elems(rows, cols);
  STRP_TAKE(ctx, arena, scale, float, 64);
  STRP_TAKE(ctx, arena, hi, unsigned short, n);
  unsigned short* lo = nullptr;
  if (np == 2) {
    STRP_TAKE(ctx, arena, lo2, unsigned short, n);
    lo = lo2;
  }
  STRP_TRY(weight_scale(ctx, src, src_kind, lds, transpose ? cols : rows, transpose ? rows : cols, scale));
  STRP_TRY(split_small(ctx, src, src_kind, lds, rows, cols, transpose, scale, hi, lo));
  *out = PlaneOp{hi, lo, plane_kg(cols), (rows + 127) / 128, scale};
  return STRP_OK;
}

// number of K splits of a token-contraction product: enough blocks to fill the chip and fp32
// accumulation chains of at most 8192 tokens (partials are then summed in fp64)
static int plan_splits(int ntiles, long long K) {
  long long s_chain = (K + 8191) / 8192;
  long long s_fill = (1024 + ntiles - 1) / ntiles;
  long long s = s_chain > s_fill ? s_chain : s_fill;
  long long s_max = K / 256 > 1 ? K / 256 : 1;
  if (s > s_max) s = s_max;
  return (int)s;
}

// Tiles and K splits of a token-contraction product.  A grid of no more than two rounds of workgroups is a matter of
// how well its last round fills the chip: from the split count of plan_splits upwards (at most a quarter more: shorter
// chains, never longer ones) the one with the least rounds x chain length is taken (17 % on the Gram of a d = 768
// module).  Larger grids are left alone: measured, their run time does not follow the round count (workgroups do not run
// in lockstep, and more splits cost more prologues and partial sums).
static void plan_nt_product(GemmP& p) {
  gemm_plan_tiles(p, 1);
  const int s0 = plan_splits(p.ntiles, p.K);
  gemm_plan_tiles(p, s0);
  const long long slots0 = p.wt == 4 ? 256 : 512;   // workgroups the chip runs at a time (one or two per CU)
  if (s0 <= 1 || (long long)p.ntiles * p.splits > 2 * slots0) return;
  double best_cost = 0.0;
  int best = s0;
  for (int s = s0; s <= s0 + s0 / 4; ++s) {
    GemmP q = p;
    gemm_plan_tiles(q, s);
    const long long slots = q.wt == 4 ? 256 : 512;
    const long long blocks = (long long)q.ntiles * q.splits;
    const double cost = (double)((blocks + slots - 1) / slots) * (double)q.kchunk;
    if (s == s0 || cost < best_cost * 0.995) {
      best_cost = cost;
      best = s;
    }
  }
  gemm_plan_tiles(p, best);
}

static size_t nt_partial_elems(int M, int N, long long K, int triangle) {
  GemmP p;
  memset(&p, 0, sizeof(p));
  p.M = M; p.N = N; p.K = K; p.triangle = triangle;
  plan_nt_product(p);
  return (size_t)p.splits * (size_t)M * (size_t)N;
}

// C = P Q^T over K (ROW planes); partials in the arena (by value: released on return), fp64 reduction.
static strp_status nt_product(strp_ctx* ctx, Arena arena, const PlaneOp& P, const PlaneOp& Q, int M, int N, long long K, int triangle,
                              float* outf, long long ldof, double* outd, long long ldod, double* diag, int accumulate) {
  GemmP p;
  memset(&p, 0, sizeof(p));
  p.P = P; p.Q = Q; p.M = M; p.N = N; p.K = K; p.triangle = triangle;
  p.epi = EPI_PARTIAL;
  plan_nt_product(p);
  STRP_TAKE(ctx, arena, part, float, (size_t)p.splits * M * N);
  p.out = part;
  STRP_TRY(launch_gemm(ctx, p));
  return launch_splitk_reduce(ctx, part, p.splits, M, N, triangle, outf, ldof, outd, ldod, diag, accumulate);
}

// Solve Wsub (Gram + lam I) = R with R = Lhs Rhs^T over the tokens.  Returns the fp64 solution
// [m x n] (leading dimension n) in *sol_out; it lives in the arena passed by reference.
struct RefitIn {
  const float* Gram; long long ldg;       // fp32 Gram (used when sys_ready == 0)
  double* sys; int sys_ready;             // [n x n] fp64 scratch: 0 = empty, 1 = holds Gram + lam I
  double* Linv; int linv_ready;           // [n x n] fp64 inverse of the Cholesky factor (output, or input if linv_ready)
  double lam; const double* lam_dev;
  PlaneOp Lhs, Rhs;
  int m, n; long long T;
};

// Factor the system in `sys` (which must hold Gram + lam I) and leave the inverse of its Cholesky factor in Linv.
static strp_status factor_and_invert(strp_ctx* ctx, Arena arena, double* sys, int n, double* Linv) {
  const int nblk = (n + NB - 1) / NB;
  STRP_TAKE(ctx, arena, invd, double, (size_t)nblk * NB * NB);
  STRP_TAKE(ctx, arena, tmp, double, (size_t)n * n);
  STRP_TRY(chol_factor(ctx, sys, n, n, invd, ctx->status_dev));
  return tri_inverse(ctx, sys, n, n, invd, Linv, tmp);
}

static strp_status ridge_solve(strp_ctx* ctx, Arena& arena, const RefitIn& in, double** sol_out) {
  const int n = in.n, m = in.m;
  const bool factor = !in.linv_ready;
  if (factor) {
    if (in.sys_ready == 0) STRP_TRY(f32_to_f64_ridge(ctx, in.Gram, in.ldg, in.sys, n, n, in.lam, in.lam_dev));
    const size_t fbytes = (((size_t)((n + NB - 1) / NB) * NB * NB * 8 + 255) & ~size_t(255)) + (((size_t)n * n * 8 + 255) & ~size_t(255));
    STRP_TAKE(ctx, arena, fscratch, char, fbytes);
    STRP_TRY(factor_and_invert(ctx, Arena(fscratch, fbytes), in.sys, n, in.Linv));
  }
  STRP_TAKE(ctx, arena, R, double, (size_t)m * n);
  STRP_TAKE(ctx, arena, tmp, double, (size_t)m * n);
  STRP_TRY(nt_product(ctx, arena, in.Lhs, in.Rhs, m, n, in.T, 0, nullptr, 0, R, n, nullptr, 0));
  STRP_TRY(apply_inverse_right(ctx, in.Linv, n, R, m, tmp));
  *sol_out = R;
  return STRP_OK;
}

// Persistent per-module planes (caller-owned strp_module_state::cache), fixed at initialisation:
// Y as ROW planes, X as ROW planes and as K8 planes.
struct CacheView {
  int nx, ny;
  double* rowsums;     // [4][f] scoring sums of the pruned rows, valid as strp_module_state::sums_cached says
  PlaneOp Yt, Xt, Xc;   // Y and X for token-contraction products; X for the channel-contraction product W1 X
};
static size_t cache_layout(const strp_module_desc* desc, int prec, char* base, CacheView* v) {
  const long long d = desc->d, T = desc->T;
  const int nx = planes_for(desc->x_dtype, prec), ny = planes_for(STRP_F32, prec);
  size_t off = 256;
  double* rowsums = (double*)(base ? base + off : nullptr);
  off += ((size_t)desc->f * 4 * sizeof(double) + 255) & ~size_t(255);
  auto take = [&](size_t elems) {
    char* p = base ? base + off : nullptr;
    off += (elems * 2 + 255) & ~size_t(255);
    return (unsigned short*)p;
  };
  unsigned short* yh = take(plane_elems(d, T));
  unsigned short* yl = ny == 2 ? take(plane_elems(d, T)) : nullptr;
  unsigned short* xh = take(plane_elems(d, T));
  unsigned short* xl = nx == 2 ? take(plane_elems(d, T)) : nullptr;
  unsigned short* kh = take(plane_elems(T, d));
  unsigned short* kl = nx == 2 ? take(plane_elems(T, d)) : nullptr;
  if (v) {
    v->nx = nx; v->ny = ny;
    v->rowsums = rowsums;
    v->Yt = PlaneOp{yh, yl, plane_kg(T), (int)((d + 127) / 128), nullptr};
    v->Xt = PlaneOp{xh, xl, plane_kg(T), (int)((d + 127) / 128), nullptr};
    v->Xc = PlaneOp{kh, kl, plane_kg(d), (int)((T + 127) / 128), nullptr};
  }
  return off;
}

}  // namespace strp

extern "C" {

size_t strp_module_cache_bytes(const strp_module_desc* desc) {
  if (!desc || desc->d <= 0 || desc->f <= 0 || desc->T <= 0) return 0;
  return cache_layout(desc, STRP_PREC_SPLIT, nullptr, nullptr);
}

size_t strp_workspace_bytes(const strp_module_desc* desc) {
  if (!desc || desc->d <= 0 || desc->f <= 0 || desc->T <= 0) return 0;
  const size_t d = desc->d, f = desc->f;
  const size_t km = desc->k_max > 0 ? (size_t)desc->k_max : f;
  const size_t kp = (size_t)round_up((long long)km, 8);
  const long long T = desc->T;
  auto al = [](size_t bytes) { return (bytes + 255) & ~size_t(255); };
  const size_t nmax = km > d ? km : d;
  const size_t invd_max = ((nmax + NB - 1) / NB) * NB * NB * 8;
  const size_t tilesT = (size_t)((T + 127) / 128);
  const size_t red = al((((f + 127) / 128) * tilesT + f + 4096) * 16);
  // initialisation: weight planes, relu(Z0) planes, H partials
  size_t init = 256 + 2 * (al(256) + 2 * al(plane_elems(f, d) * 2)) + 2 * al(plane_elems(T, f) * 2) + red +
                al(nt_partial_elems((int)d, (int)d, T, 1) * 4) + al(d * 8) + al(invd_max) + 2 * al(d * d * 8);
  // one iteration: everything every stage carves (stages reuse the arena, so this is an upper bound)
  size_t part = 0;
  auto upd = [&](size_t e) { if (e > part) part = e; };
  upd(nt_partial_elems((int)km, (int)km, T, 1));
  upd(nt_partial_elems((int)d, (int)km, T, 0));
  upd(nt_partial_elems((int)km, (int)d, T, 0));
  upd(nt_partial_elems((int)d, (int)d, (long long)kp, 1));
  upd(nt_partial_elems((int)d, (int)d, T, 1));   // E E^T of the objective
  const size_t segs = (size_t)((T + 8191) / 8192);
  size_t step = 256 + al(4 * f * 8) + al(d * kp * 4) + al(km * d * 4) +
                /* the pruned rows' pass: its sums, the row list, the unit counter, the units' partial sums */
                al(2 * f * 8) + al(f * 4) + 256 + al(f * segs * 6 * 8) +
                (al(256) + 2 * al(plane_elems(d, km) * 2)) + 2 * (al(256) + 2 * al(plane_elems(km, d) * 2)) +
                al(part * 4) + 3 * al(nmax * nmax * 8) + 2 * al(invd_max) + al(d * km * 8) * 4 + 2 * al(d * d * 8) +
                2 * al(plane_elems(km, T) * 2) /* kept rows, token contraction */ +
                2 * al(plane_elems(T, km) * 2) /* kept rows, channel contraction */ +
                2 * al(plane_elems(T, d) * 2) /* E */ + red +
                al(plane_elems(d, T) * 2) + al(d * d * 8) + al(d * d * 4) /* objective: E by tokens, E E^T, M^-2 */ +
                /* the M-inverse chain keeps its block while the fc1 refit runs beside it */
                al(nt_partial_elems((int)d, (int)d, (long long)kp, 1) * 4) + al(d * d * 8) + al(invd_max) +
                2 * (al(256) + 2 * al(plane_elems(km, d) * 2)) + (al(256) + 2 * al(plane_elems(d, d) * 2)) + al(plane_elems(T, km) * 2) + 8192 +
                /* strip sums of the kept rows from the a- and z-update epilogues */
                al(2 * (size_t)((T + 63) / 64) * km * 4) + al((size_t)((T + 63) / 64) * km * 4) + al(rowsum_scratch_bytes(2, (int)km));
  return (init > step ? init : step) + (1 << 20);
}

strp_status strp_gram(strp_ctx* ctx, const void* A, strp_dtype dt, int32_t C, int64_t T, int64_t ldA, const int32_t* idx,
                      int32_t s, float* G, int32_t ldG, double* diag, int accumulate) {
  if (!ctx) return STRP_EINVAL;
  if (!A || !G) return fail(ctx, STRP_EINVAL, "gram: null A or G");
  if (dt != STRP_BF16 && dt != STRP_F32) return fail(ctx, STRP_EINVAL, "gram: unknown dtype");
  if (C <= 0 || s <= 0 || s > C || T <= 0) return fail(ctx, STRP_EINVAL, "gram: need 0 < s <= C and T > 0");
  if (!idx && s != C) return fail(ctx, STRP_EINVAL, "gram: idx == NULL requires s == C");
  if (ldA < T || ldA % 8 || ldG < s) return fail(ctx, STRP_EINVAL, "gram: bad leading dimension");
  if (!aligned16(A)) return fail(ctx, STRP_EINVAL, "gram: A not 16-byte aligned");
  if (!ctx->ws) return fail(ctx, STRP_ENOMEM, "gram: no workspace set");
  Arena arena(ctx);
  PlaneOp op;
  STRP_TRY(make_t_planes(ctx, arena, A, dt, ldA, idx, s, T, 0, planes_for(dt, ctx->precision), &op));
  return nt_product(ctx, arena, op, op, s, s, T, 1, G, ldG, nullptr, 0, diag, accumulate);
}

strp_status strp_refit(strp_ctx* ctx, strp_side side, const float* Gram, int32_t ldg, double lambda, double* chol, int chol_valid,
                       const void* Lhs, strp_dtype lhs_dtype, int64_t ld_lhs, const void* Rhs, strp_dtype rhs_dtype,
                       int64_t ld_rhs, int64_t T, const int32_t* idx, int32_t s, float* W, int32_t out, int32_t in) {
  if (!ctx) return STRP_EINVAL;
  if (side != STRP_SIDE_FC1 && side != STRP_SIDE_FC2) return fail(ctx, STRP_EINVAL, "refit: unknown side");
  if (!Lhs || !Rhs || !W || !idx) return fail(ctx, STRP_EINVAL, "refit: null argument");
  if (out <= 0 || in <= 0 || T <= 0 || s <= 0) return fail(ctx, STRP_EINVAL, "refit: non-positive size");
  if (side == STRP_SIDE_FC2 && s > in) return fail(ctx, STRP_EINVAL, "refit: s > in");
  if (side == STRP_SIDE_FC1 && s > out) return fail(ctx, STRP_EINVAL, "refit: s > out");
  if (ld_lhs < T || ld_rhs < T || ld_lhs % 8 || ld_rhs % 8) return fail(ctx, STRP_EINVAL, "refit: bad leading dimension");
  if (!aligned16(Lhs) || !aligned16(Rhs)) return fail(ctx, STRP_EINVAL, "refit: operands not 16-byte aligned");
  if (chol_valid && !chol) return fail(ctx, STRP_EINVAL, "refit: chol_valid without chol");
  if (!chol_valid && !Gram) return fail(ctx, STRP_EINVAL, "refit: need Gram or a valid factor");
  const int n = side == STRP_SIDE_FC2 ? s : in;
  const int m = side == STRP_SIDE_FC2 ? out : s;
  if (!chol_valid && ldg < n) return fail(ctx, STRP_EINVAL, "refit: ldg below the order of Gram");
  if (!(lambda >= 0.0)) return fail(ctx, STRP_EINVAL, "refit: negative lambda");
  if (!ctx->ws) return fail(ctx, STRP_ENOMEM, "refit: no workspace set");
  Arena arena(ctx);
  RefitIn ri;
  memset(&ri, 0, sizeof(ri));
  ri.Gram = Gram; ri.ldg = ldg; ri.lam = lambda; ri.lam_dev = nullptr;
  if (chol) {
    ri.Linv = chol;
  } else {
    STRP_TAKE(ctx, arena, Linv, double, (size_t)n * n);
    ri.Linv = Linv;
  }
  ri.linv_ready = chol_valid ? 1 : 0;
  if (!chol_valid) {
    STRP_TAKE(ctx, arena, sys, double, (size_t)n * n);
    ri.sys = sys;
  }
  const int prec = ctx->precision;
  if (side == STRP_SIDE_FC2) {
    STRP_TRY(make_t_planes(ctx, arena, Lhs, lhs_dtype, ld_lhs, nullptr, out, T, 0, planes_for(lhs_dtype, prec), &ri.Lhs));
    STRP_TRY(make_t_planes(ctx, arena, Rhs, rhs_dtype, ld_rhs, idx, s, T, 0, planes_for(rhs_dtype, prec), &ri.Rhs));
  } else {
    STRP_TRY(make_t_planes(ctx, arena, Lhs, lhs_dtype, ld_lhs, idx, s, T, 0, planes_for(lhs_dtype, prec), &ri.Lhs));
    STRP_TRY(make_t_planes(ctx, arena, Rhs, rhs_dtype, ld_rhs, nullptr, in, T, 0, planes_for(rhs_dtype, prec), &ri.Rhs));
  }
  ri.m = m; ri.n = n; ri.T = T;
  double* sol = nullptr;
  STRP_TRY(ridge_solve(ctx, arena, ri, &sol));
  return scatter_weights(ctx, sol, n, side, idx, s, W, out, in);
}

strp_status strp_module_init(strp_ctx* ctx, const strp_module_desc* desc, strp_module_state* st, const strp_params* params) {
  if (!ctx) return STRP_EINVAL;
  STRP_TRY(check_desc(ctx, desc));
  if (!st || !params) return fail(ctx, STRP_EINVAL, "module_init: null state or params");
  if (!st->X || !st->W1hat || !st->W2hat || !st->Z || !st->A || !st->Z0 || !st->Y || !st->W1 || !st->W2 || !st->H || !st->cholH ||
      !st->n2 || !st->score || !st->mask || !st->idx || !st->scalars || !st->cache)
    return fail(ctx, STRP_EINVAL, "module_init: null buffer in state");
  if (!aligned16(st->X) || !aligned16(st->W1hat) || !aligned16(st->W2hat) || !aligned16(st->Z) || !aligned16(st->A) ||
      !aligned16(st->Z0) || !aligned16(st->Y) || ((uintptr_t)st->cache & 255u))
    return fail(ctx, STRP_EINVAL, "module_init: buffers must be 16-byte aligned (cache: 256)");
  if (!(params->delta >= 0.0)) return fail(ctx, STRP_EINVAL, "module_init: negative delta");
  if (!ctx->ws) return fail(ctx, STRP_ENOMEM, "module_init: no workspace set");
  const int d = desc->d, f = desc->f;
  const long long T = desc->T, lda = desc->lda;
  const int prec = ctx->precision;
  const int npw = planes_for(desc->w_dtype, prec), npa = planes_for(STRP_F32, prec);
  const int wkind = desc->w_dtype == STRP_BF16 ? SRC_BF16 : SRC_F32;
  CacheView cv;
  cache_layout(desc, prec, (char*)st->cache, &cv);
  Arena arena(ctx);
  double* sc = st->scalars;
  STRP_TRY(fill_zero(ctx, sc, SC_COUNT * sizeof(double)));
  STRP_TRY(launch_colnorm2(ctx, st->W2hat, desc->w_dtype, d, f, f, st->n2));
  // X planes (persistent)
  STRP_TRY(split_act(ctx, st->X, desc->x_dtype, desc->ldx, nullptr, d, T, 0, 0, (unsigned short*)cv.Xt.hi, (unsigned short*)cv.Xt.lo,
                     (unsigned short*)cv.Xc.hi, (unsigned short*)cv.Xc.lo));
  {
    Arena a2 = arena;
    PlaneOp W1p, W2p, A0k8;
    STRP_TRY(make_weight_planes(ctx, a2, st->W1hat, wkind, d, f, d, 0, npw, &W1p));
    STRP_TRY(make_weight_planes(ctx, a2, st->W2hat, wkind, f, d, f, 0, npw, &W2p));
    STRP_TAKE(ctx, a2, a0h, unsigned short, plane_elems(T, f));
    unsigned short* a0l = nullptr;
    if (npa == 2) {
      STRP_TAKE(ctx, a2, a0l2, unsigned short, plane_elems(T, f));
      a0l = a0l2;
    }
    A0k8 = PlaneOp{a0h, a0l, plane_kg(f), (int)((T + 127) / 128), nullptr};
    {  // Z0 = W1hat X, Z = Z0, A = relu(Z0) (+ K8 planes of A), sum A^2
      GemmP p;
      memset(&p, 0, sizeof(p));
      p.P = W1p; p.Q = cv.Xc;
      p.M = f; p.N = (int)T; p.K = d;
      p.epi = EPI_INITZ; p.Zs = st->Z; p.As = st->A; p.Z0s = st->Z0; p.lda = lda;
      p.k8_hi = a0h; p.k8_lo = a0l; p.k8_kg = plane_kg(f);
      gemm_plan_tiles(p, 1);
      STRP_TAKE(ctx, a2, red, double, 2 * (size_t)gemm_grid_blocks(p));
      p.red = red;
      STRP_TRY(launch_gemm(ctx, p));
      STRP_TRY(launch_block_sum(ctx, red, gemm_grid_blocks(p), sc + SC_SUMA0, nullptr, 1.0, 1.0));
      hipLaunchKernelGGL(axpby_scalar_kernel, dim3(1), dim3(1), 0, ctx->stream, sc, (int)SC_LAM2, params->delta / (double)f, (int)SC_SUMA0, 0.0, -1);
    }
    {  // Y = W2hat A
      GemmP p;
      memset(&p, 0, sizeof(p));
      p.P = W2p; p.Q = A0k8;
      p.M = d; p.N = (int)T; p.K = f;
      p.epi = EPI_STORE; p.out = st->Y; p.ldo = lda;
      gemm_plan_tiles(p, 1);
      STRP_TRY(launch_gemm(ctx, p));
    }
  }
  STRP_TRY(split_act(ctx, st->Y, STRP_F32, lda, nullptr, d, T, 0, 0, (unsigned short*)cv.Yt.hi, (unsigned short*)cv.Yt.lo, nullptr,
                     nullptr));
  {  // H = X X^T (fp32 copy and fp64 system), lam1 = delta tr(H)/d, factor of H + lam1 I
    Arena a2 = arena;
    STRP_TAKE(ctx, a2, diag, double, (size_t)d);
    STRP_TAKE(ctx, a2, Hd, double, (size_t)d * d);
    STRP_TRY(nt_product(ctx, a2, cv.Xt, cv.Xt, d, d, T, 1, st->H, d, Hd, d, diag, 0));
    hipLaunchKernelGGL(vec_sum_kernel, dim3(1), dim3(256), 0, ctx->stream, diag, d, params->delta / (double)d, sc + SC_LAM1, sc + SC_TRH);
    hipLaunchKernelGGL(add_diag_kernel, dim3(blocks_for(d)), dim3(256), 0, ctx->stream, Hd, (long long)d, d, 0.0, sc + SC_LAM1);
    STRP_TRY(factor_and_invert(ctx, a2, Hd, d, st->cholH));
  }
  STRP_TRY(fill_zero(ctx, st->W1, sizeof(float) * (size_t)f * d));
  STRP_TRY(fill_zero(ctx, st->W2, sizeof(float) * (size_t)f * d));
  STRP_TRY(fill_zero(ctx, st->mask, (size_t)f));
  STRP_HIP(ctx, hipGetLastError());
  st->s = 0;
  st->iter = 0;
  st->sums_cached = 0;
  st->precision = 1 + prec;
  return STRP_OK;
}

strp_status strp_admm_step(strp_ctx* ctx, const strp_module_desc* desc, strp_module_state* st, const strp_params* params,
                           strp_report* report_host) {
  if (!ctx) return STRP_EINVAL;
  STRP_TRY(check_desc(ctx, desc));
  if (!st || !params) return fail(ctx, STRP_EINVAL, "admm_step: null state or params");
  if (!st->X || !st->W2hat || !st->Z || !st->A || !st->Z0 || !st->Y || !st->W1 || !st->W2 || !st->cholH || !st->n2 || !st->score ||
      !st->mask || !st->idx || !st->scalars || !st->cache)
    return fail(ctx, STRP_EINVAL, "admm_step: null buffer in state");
  const int d = desc->d, f = desc->f;
  const long long T = desc->T, lda = desc->lda;
  const int stages = params->stages ? params->stages : 63;
  const bool do_select = (stages & STRP_STAGE_SELECT) && (params->reselect || st->s == 0);
  if (do_select && (params->k <= 0 || params->k > f)) return fail(ctx, STRP_EINVAL, "admm_step: k outside [1, f]");
  if (desc->k_max > 0 && do_select && params->k > desc->k_max) return fail(ctx, STRP_EINVAL, "admm_step: k above desc.k_max");
  if (!do_select && st->s <= 0) return fail(ctx, STRP_ESTATE, "admm_step: no mask selected yet");
  if (!(params->alpha > 0.0) || !(params->beta > 0.0)) return fail(ctx, STRP_EINVAL, "admm_step: alpha, beta must be positive");
  if (params->mode < STRP_SCORE_WANDA || params->mode > STRP_SCORE_GAIN) return fail(ctx, STRP_EINVAL, "admm_step: unknown score mode");
  if (!ctx->ws) return fail(ctx, STRP_ENOMEM, "admm_step: no workspace set");
  const int prec = ctx->precision;
  // the plane cache was laid out and written under the precision of strp_module_init: another one would read other offsets
  if (st->precision == 0) return fail(ctx, STRP_ESTATE, "admm_step: strp_module_init has not run on this state");
  if (st->precision != 1 + prec)
    return fail(ctx, STRP_ESTATE, "admm_step: the context's precision (%d) differs from the one the module was initialised with (%d)",
                prec, st->precision - 1);
  const int npa = planes_for(STRP_F32, prec);
  CacheView cv;
  cache_layout(desc, prec, (char*)st->cache, &cv);
  double* sc = st->scalars;
  const float alpha = (float)params->alpha, beta = (float)params->beta;
  Arena arena(ctx);

  // ---- S2/S4: scores and top-k ---------------------------------------------------------
  // The token sums every score is built from live in the module cache (cv.rowsums, [4][f]): sum A^2, sum A relu(Z0),
  // sum Z0 Z, sum Z0^2.  A full iteration leaves them there for every row -- the pruned rows' from the pass that writes
  // those rows, the kept rows' from the epilogues of the a- and z-update products (sum Z0^2 never changes after it has
  // been streamed once) -- so that only a selection on a state the library did not produce streams the rows.
  const bool wanda = params->mode == STRP_SCORE_WANDA;
  if (do_select) {
    const bool have = (st->sums_cached & SUMS_G) && (wanda || ((st->sums_cached & SUMS_EU) && (st->sums_cached & SUMS_V)));
    if (!have) {
      STRP_TRY(launch_row_sums(ctx, st->A, STRP_F32, st->Z, st->Z0, lda, T, f, params->mode, cv.rowsums));
      st->sums_cached = wanda ? (st->sums_cached & SUMS_V) | SUMS_G : SUMS_G | SUMS_EU | SUMS_V;
    }
    STRP_TRY(launch_unit_scores(ctx, cv.rowsums, st->n2, f, 1, params->mode, st->score, sc + SC_ENERGY));
    STRP_TRY(launch_topk(ctx, st->score, f, params->k, 1, st->mask, st->idx, (float*)(sc + SC_TAU), nullptr, 0));
    st->s = params->k;
  }
  // the sums describe the state as it is now: void them before an update changes it (sum Z0^2 stays valid)
  if (stages & (STRP_STAGE_AUPD | STRP_STAGE_ZUPD)) st->sums_cached &= SUMS_V;
  const int s = st->s;
  const long long sp = round_up(s, 8);

  // ---- the pruned rows' fused a/z pass as a ride-along job ------------------------------------------------------
  // It touches only rows outside S, which nothing else in the step reads or writes, so it may run any time from
  // here to the end of the step: the factorisation chains of the fc2 refit and of the a-update carry spare
  // workgroups for it (chol_factor reads ctx->cojob), and what they leave is drained where the pass used to run.
  const bool fuse_pruned = (stages & STRP_STAGE_AUPD) && (stages & STRP_STAGE_ZUPD);
  struct CoJobGuard {
    strp_ctx* c;
    ~CoJobGuard() { c->cojob = nullptr; }
  } cojob_guard{ctx};
  CoJob pjob;
  memset(&pjob, 0, sizeof(pjob));
  double* red_pruned = nullptr;
  if (fuse_pruned) {
    STRP_TAKE(ctx, arena, rp, double, 2 * (size_t)f);
    red_pruned = rp;
    STRP_TRY(fill_zero(ctx, red_pruned, 2 * (size_t)f * sizeof(double)));
    if (s < f) {
      constexpr long long SEG = 8192;
      const int segs = (int)((T + SEG - 1) / SEG);
      STRP_TAKE(ctx, arena, prow, int32_t, (size_t)f);
      STRP_TAKE(ctx, arena, ticket, unsigned int, 64);
      STRP_TAKE(ctx, arena, partial, double, (size_t)(f - s) * segs * 6);
      STRP_TRY(fill_zero(ctx, ticket, 256));
      hipLaunchKernelGGL(pruned_list_kernel, dim3(1), dim3(1024), 0, ctx->stream, st->mask, f, prow);
      pjob.ticket = ticket;
      pjob.units = (unsigned int)(f - s) * (unsigned int)segs;
      pjob.take = 3;
      pjob.rows = prow; pjob.nrows = f - s; pjob.segs = segs; pjob.seg_tokens = SEG;
      pjob.Z = st->Z; pjob.A = st->A; pjob.Z0 = wanda ? nullptr : st->Z0;
      pjob.lda = lda; pjob.T = T; pjob.alpha = alpha; pjob.beta = beta; pjob.partial = partial;
      // a small pass (a module of a few hundred hidden units per kept one, or few tokens) is over before the chains
      // have taken their first steps and only lengthens those: it is left to the drain (measured on a d = 768 module:
      // 2 % slower with the ride, against 1-2 % faster from d = 2048 on)
      if (pjob.units >= 65536u) ctx->cojob = &pjob;
    }
  }
  // ---- S1/S5: Gram of the kept A rows, fc2 refit -------------------------------------------
  if (stages & STRP_STAGE_REFIT2) {
    Arena a2 = arena;
    STRP_TAKE(ctx, a2, Gd, double, (size_t)s * s);
    PlaneOp Arow;
    STRP_TRY(make_t_planes(ctx, a2, st->A, STRP_F32, lda, st->idx, s, T, 0, npa, &Arow));
    STRP_TRY(nt_product(ctx, a2, operand_for(ctx, STRP_PROD_GRAM, 0, Arow), operand_for(ctx, STRP_PROD_GRAM, 1, Arow), s, s, T, 1, nullptr,
                        0, Gd, s, nullptr, 0));
    hipLaunchKernelGGL(add_diag_kernel, dim3(blocks_for(s)), dim3(256), 0, ctx->stream, Gd, (long long)s, s, 0.0, sc + SC_LAM2);
    RefitIn ri;
    memset(&ri, 0, sizeof(ri));
    STRP_TAKE(ctx, a2, Ginv, double, (size_t)s * s);
    ri.sys = Gd; ri.sys_ready = 1; ri.Linv = Ginv; ri.linv_ready = 0;
    ri.Lhs = operand_for(ctx, STRP_PROD_RHS2, 0, cv.Yt);
    ri.Rhs = operand_for(ctx, STRP_PROD_RHS2, 1, Arow);
    ri.m = d; ri.n = s; ri.T = T;
    double* sol = nullptr;
    STRP_TRY(ridge_solve(ctx, a2, ri, &sol));
    STRP_TRY(scatter_weights(ctx, sol, s, STRP_SIDE_FC2, st->idx, s, st->W2, d, f));
  }
  // compact kept weights and their planes (shared by the stages below)
  PlaneOp W2Sp, W1Sp;
  memset(&W2Sp, 0, sizeof(W2Sp));
  memset(&W1Sp, 0, sizeof(W1Sp));
  float* W2S = nullptr;
  float* W1S = nullptr;
  if (stages & (STRP_STAGE_AUPD | STRP_STAGE_OBJ)) {
    STRP_TAKE(ctx, arena, w2s, float, (size_t)d * sp);
    W2S = w2s;
    hipLaunchKernelGGL(gather_cols_kernel, dim3(blocks_for((long long)d * sp)), dim3(256), 0, ctx->stream, st->W2, d, f, st->idx, s, W2S, sp);
    STRP_TRY(make_weight_planes(ctx, arena, W2S, SRC_F32, sp, d, s, 0, npa, &W2Sp));
  }
  // ---- a-update, part 1: B = W^T M^-1 with M = (beta/alpha) I + W W^T, W = W2[:, S] -------------------------
  // Needs only the refitted W2.  Its buffers come from the base arena and stay until the step ends.
  PlaneOp Bp;
  memset(&Bp, 0, sizeof(Bp));
  // First objective term when the a-update runs in the same call: the update solves its least-squares problem exactly, so
  //   Y - W A_S = E - W W^T M^-1 E = (M - W W^T) M^-1 E = (beta/alpha) M^-1 E,   E = Y - W relu(Z_S),
  // and |Y - W A_S|_F^2 = (beta/alpha)^2 <M^-2, E E^T>: a d x d Gram of E over the tokens (half the work of the product
  // W A_S) and two d x d matrices.  One fp16 plane of E is ample for a sum reported to 1e-3.
  const bool term1_identity = (stages & STRP_STAGE_AUPD) && (stages & STRP_STAGE_OBJ);
  float* M2f = nullptr;
  if (stages & STRP_STAGE_AUPD) {
    STRP_TAKE(ctx, arena, Md, double, (size_t)d * d);
    STRP_TAKE(ctx, arena, Linv, double, (size_t)d * d);
    STRP_TAKE(ctx, arena, Bf, float, (size_t)s * d);
    if (term1_identity) {
      STRP_TAKE(ctx, arena, m2, float, (size_t)d * d);
      M2f = m2;
    }
    const size_t al = 255;
    const size_t cbytes = ((nt_partial_elems(d, d, sp, 1) * 4 + al) & ~al) + (((size_t)((d + NB - 1) / NB) * NB * NB * 8 + al) & ~al) +
                          (((size_t)d * d * 8 + al) & ~al) + (512 + 2 * ((plane_elems(s, d) * 2 + al) & ~al)) +
                          (512 + 2 * ((plane_elems(d, d) * 2 + al) & ~al)) + 4096;
    STRP_TAKE(ctx, arena, cblock, char, cbytes);
    Arena a2(cblock, cbytes);
    STRP_TRY(nt_product(ctx, a2, W2Sp, W2Sp, d, d, sp, 1, nullptr, 0, Md, d, nullptr, 0));
    hipLaunchKernelGGL(add_diag_kernel, dim3(blocks_for(d)), dim3(256), 0, ctx->stream, Md, (long long)d, d, params->beta / params->alpha, (const double*)nullptr);
    STRP_TRY(factor_and_invert(ctx, a2, Md, d, Linv));
    // M is well conditioned (its spectrum lies in [beta/alpha, beta/alpha + |W|^2]): form M^-1 = Linv^T Linv
    // (lower half, fp64) and B = W^T M^-1 on the fp16-split matrix cores instead of a third fp64 solve
    STRP_TRY(fill_zero(ctx, Md, sizeof(double) * (size_t)d * d));
    STRP_TRY(dgemm(ctx, d, d, d, 1.0, Linv, 1, d, Linv, d, 1, 0.0, Md, d, 1, 3));
    {
      Arena a3 = a2;
      PlaneOp Wt, Mi;
      STRP_TRY(make_weight_planes(ctx, a3, W2S, SRC_F32, sp, s, d, 1, npa, &Wt));
      STRP_TRY(make_weight_planes(ctx, a3, Md, SRC_F64, d, d, d, 2, npa, &Mi));
      GemmP p;
      memset(&p, 0, sizeof(p));
      p.P = Wt; p.Q = Mi;
      p.M = s; p.N = d; p.K = d;
      p.epi = EPI_STORE; p.out = Bf; p.ldo = d;
      gemm_plan_tiles(p, 1);
      STRP_TRY(launch_gemm(ctx, p));
      if (term1_identity) {   // M^-2 for the first objective term (see the a-update below)
        GemmP q;
        memset(&q, 0, sizeof(q));
        q.P = Mi; q.Q = Mi;
        q.M = d; q.N = d; q.K = d;
        q.epi = EPI_STORE; q.out = M2f; q.ldo = d;
        gemm_plan_tiles(q, 1);
        STRP_TRY(launch_gemm(ctx, q));
      }
    }
    STRP_TRY(make_weight_planes(ctx, arena, Bf, SRC_F32, d, s, d, 0, npa, &Bp));
  }
  // Z_S is needed by tokens (fc1 refit) and, with relu, by channels (a-update): when both stages run, one pass over
  // the kept rows of Z writes both sets of planes; the second set stays in the base arena until the a-update.
  PlaneOp Zk8pre;
  memset(&Zk8pre, 0, sizeof(Zk8pre));
  const bool z_planes_once = (stages & STRP_STAGE_REFIT1) && (stages & STRP_STAGE_AUPD);
  if (z_planes_once) {
    STRP_TAKE(ctx, arena, zch, unsigned short, plane_elems(T, s));
    unsigned short* zcl = nullptr;
    if (npa == 2) {
      STRP_TAKE(ctx, arena, zcl2, unsigned short, plane_elems(T, s));
      zcl = zcl2;
    }
    Zk8pre = PlaneOp{zch, zcl, plane_kg(s), (int)((T + 127) / 128), nullptr};
  }
  // ---- S6: fc1 refit with the cached factor of H + lam1 I ------------------------------------
  if (stages & STRP_STAGE_REFIT1) {
    Arena a2 = arena;
    PlaneOp Zrow;
    if (z_planes_once) {
      STRP_TAKE(ctx, a2, zth, unsigned short, plane_elems(s, T));
      unsigned short* ztl = nullptr;
      if (npa == 2) {
        STRP_TAKE(ctx, a2, ztl2, unsigned short, plane_elems(s, T));
        ztl = ztl2;
      }
      STRP_TRY(split_act(ctx, st->Z, STRP_F32, lda, st->idx, s, T, 0, 1, zth, ztl, (unsigned short*)Zk8pre.hi, (unsigned short*)Zk8pre.lo));
      Zrow = PlaneOp{zth, ztl, plane_kg(T), (s + 127) / 128, nullptr};
    } else {
      STRP_TRY(make_t_planes(ctx, a2, st->Z, STRP_F32, lda, st->idx, s, T, 0, npa, &Zrow));
    }
    RefitIn ri;
    memset(&ri, 0, sizeof(ri));
    ri.Linv = st->cholH; ri.linv_ready = 1;
    ri.Lhs = operand_for(ctx, STRP_PROD_RHS1, 0, Zrow);
    ri.Rhs = operand_for(ctx, STRP_PROD_RHS1, 1, cv.Xt);
    ri.m = s; ri.n = d; ri.T = T;
    double* sol = nullptr;
    STRP_TRY(ridge_solve(ctx, a2, ri, &sol));
    STRP_TRY(scatter_weights(ctx, sol, d, STRP_SIDE_FC1, st->idx, s, st->W1, f, d));
  }
  if (stages & (STRP_STAGE_ZUPD | STRP_STAGE_OBJ)) {
    STRP_TAKE(ctx, arena, w1s, float, (size_t)s * d);
    W1S = w1s;
    hipLaunchKernelGGL(gather_rows_kernel, dim3(blocks_for((long long)s * d)), dim3(256), 0, ctx->stream, st->W1, d, st->idx, s, W1S, (long long)d);
    STRP_TRY(make_weight_planes(ctx, arena, W1S, SRC_F32, d, s, d, 0, npa, &W1Sp));
  }

  // scoring sums of the kept rows, collected by the two epilogues that write those rows (64-column strips, fp32)
  const int rs_slots = (int)((T + 63) / 64);
  float* rsA = nullptr;
  float* rsZ = nullptr;
  double* rs_chunks = nullptr;
  if (fuse_pruned) {
    STRP_TAKE(ctx, arena, rsa_, float, (size_t)(wanda ? 1 : 2) * rs_slots * s);
    STRP_TAKE(ctx, arena, rsc_, double, rowsum_scratch_bytes(2, s) / sizeof(double));
    rsA = rsa_;
    rs_chunks = rsc_;
    if (!wanda) {
      STRP_TAKE(ctx, arena, rsz_, float, (size_t)rs_slots * s);
      rsZ = rsz_;
    }
  }
  // ---- S7: a-update in residual (Woodbury) form ------------------------------------------------
  //   A_S = relu(Z_S) + W^T M^-1 (Y - W relu(Z_S)),  M = (beta/alpha) I + W W^T,  W = W2[:, S];  A_j = relu(Z_j) for pruned j
  if (stages & STRP_STAGE_AUPD) {
    Arena a2 = arena;
    PlaneOp Zk8 = Zk8pre;
    if (!z_planes_once) {
      STRP_TRY(make_c_planes(ctx, a2, st->Z, STRP_F32, lda, st->idx, s, T, 1, npa, &Zk8));
    }
    STRP_TAKE(ctx, a2, ekh, unsigned short, plane_elems(T, d));
    unsigned short* ekl = nullptr;
    if (npa == 2) {
      STRP_TAKE(ctx, a2, ekl2, unsigned short, plane_elems(T, d));
      ekl = ekl2;
    }
    {  // E = Y - W relu(Z_S), kept only as K8 planes
      GemmP p;
      memset(&p, 0, sizeof(p));
      p.P = operand_for(ctx, STRP_PROD_RESID, 0, W2Sp);
      p.Q = operand_for(ctx, STRP_PROD_RESID, 1, Zk8);
      p.M = d; p.N = (int)T; p.K = s;
      p.epi = EPI_RESID; p.Yin = st->Y; p.ldy = lda;
      p.k8_hi = ekh; p.k8_lo = ekl; p.k8_kg = plane_kg(d);
      gemm_plan_tiles(p, 1);
      STRP_TRY(launch_gemm(ctx, p));
    }
    if (term1_identity) {   // (alpha/T) |Y - W A_S|^2 = (alpha/T) (beta/alpha)^2 <M^-2, E E^T>
      Arena a3 = a2;
      STRP_TAKE(ctx, a3, eth, unsigned short, plane_elems(d, T));
      STRP_TAKE(ctx, a3, Sd, double, (size_t)d * d);
      STRP_TAKE(ctx, a3, red, double, 2 * 1024);
      STRP_TRY(plane_c_to_t(ctx, ekh, eth, d, T));
      const PlaneOp Et{eth, nullptr, plane_kg(T), (int)((d + 127) / 128), nullptr};
      STRP_TRY(nt_product(ctx, a3, Et, Et, d, d, T, 1, nullptr, 0, Sd, d, nullptr, 0));
      hipLaunchKernelGGL(dot_f32_f64_kernel, dim3(1024), dim3(256), 0, ctx->stream, M2f, Sd, (long long)d * d, red);
      const double c = params->beta / params->alpha;
      STRP_TRY(launch_block_sum(ctx, red, 1024, sc + SC_T1, nullptr, params->alpha / (double)T * c * c, 1.0));
    }
    {  // A_S = relu(Z_S) + B E
      GemmP p;
      memset(&p, 0, sizeof(p));
      p.P = operand_for(ctx, STRP_PROD_AUPD, 0, Bp);
      p.Q = operand_for(ctx, STRP_PROD_AUPD, 1, PlaneOp{ekh, ekl, plane_kg(d), (int)((T + 127) / 128), nullptr});
      p.M = s; p.N = (int)T; p.K = d;
      p.epi = EPI_AUPD; p.Zs = st->Z; p.As = st->A; p.lda = lda; p.oidx = st->idx;
      p.rs_out = rsA; p.rs_z0 = (rsA && !wanda) ? st->Z0 : nullptr; p.rs_slots = rs_slots;
      gemm_plan_tiles(p, 1);
      STRP_TRY(launch_gemm(ctx, p));
      if (rsA) STRP_TRY(launch_rowsum_reduce(ctx, rsA, wanda ? 1 : 2, rs_slots, s, st->idx, cv.rowsums, f, 0, 1, rs_chunks));
    }
    if (!fuse_pruned) {
      ProfScope ps(ctx, "pruned_rows_a", 0.0, 8.0 * (double)(f - s) * (double)T);
      hipLaunchKernelGGL(pruned_rows_kernel, dim3(f), dim3(256), 0, ctx->stream, st->mask, st->Z, st->A, lda, T, 0, alpha, beta, 1, (double*)nullptr,
                         (const float*)nullptr, (double*)nullptr, f);
    }
  }
  // ---- S8 (+ objective terms 2, 3): z-update fused on Z1 = W1 X --------------------------------
  const bool zupd = (stages & STRP_STAGE_ZUPD) != 0;
  if (zupd || (stages & STRP_STAGE_OBJ)) {
    Arena a2 = arena;
    GemmP p;
    memset(&p, 0, sizeof(p));
    p.P = operand_for(ctx, STRP_PROD_ZUPD, 0, W1Sp);
    p.Q = operand_for(ctx, STRP_PROD_ZUPD, 1, cv.Xc);
    p.M = s; p.N = (int)T; p.K = d;
    p.epi = EPI_ZUPD; p.Zs = st->Z; p.As = st->A; p.lda = lda; p.oidx = st->idx; p.alpha = alpha; p.beta = beta;
    p.write_out = zupd ? 1 : 0;
    p.rs_out = (zupd && rsZ) ? rsZ : nullptr; p.rs_z0 = p.rs_out ? st->Z0 : nullptr; p.rs_slots = rs_slots;
    gemm_plan_tiles(p, 1);
    const int nb = gemm_grid_blocks(p);
    STRP_TAKE(ctx, a2, red, double, 2 * (size_t)(nb > f ? nb : f));
    p.red = red;
    STRP_TRY(launch_gemm(ctx, p));
    STRP_TRY(launch_block_sum(ctx, red, nb, sc + SC_TMP0, sc + SC_TMP1, 1.0, 1.0));
    if (p.rs_out) STRP_TRY(launch_rowsum_reduce(ctx, rsZ, 1, rs_slots, s, st->idx, cv.rowsums, f, 2, 2, rs_chunks));
    if (fuse_pruned) {
      // what the factorisation chains' spare workgroups left of the pruned rows' pass, then the rows' sums
      ctx->cojob = nullptr;
      if (pjob.ticket) {
        {
          ProfScope ps(ctx, "pruned_rows_drain", 0.0, 0.0);
          CoJob dj = pjob;
          dj.take = 4;
          hipLaunchKernelGGL(cojob_drain_kernel, dim3(2048), dim3(256), 0, ctx->stream, dj);
        }
        hipLaunchKernelGGL(cojob_finish_kernel, dim3((pjob.nrows + 255) / 256), dim3(256), 0, ctx->stream, pjob, red_pruned, cv.rowsums, f);
      }
      // every row's sums are now in place: the kept rows' from the two epilogues, the pruned rows' from this pass
      // (which also rewrites their sum Z0^2; the kept rows' is only there if it was streamed before)
      st->sums_cached = (st->sums_cached & SUMS_V) | SUMS_G | (wanda ? 0 : SUMS_EU);
    } else {
      ProfScope ps(ctx, "pruned_rows_z", 0.0, 8.0 * (double)(f - s) * (double)T);
      hipLaunchKernelGGL(pruned_rows_kernel, dim3(f), dim3(256), 0, ctx->stream, st->mask, st->Z, st->A, lda, T, 1, alpha, beta,
                         zupd ? 1 : 0, red, (const float*)nullptr, (double*)nullptr, f);
    }
    STRP_TRY(launch_block_sum(ctx, fuse_pruned ? red_pruned : red, f, sc + SC_TMP2, sc + SC_TMP3, 1.0, 1.0));
    hipLaunchKernelGGL(axpby_scalar_kernel, dim3(1), dim3(1), 0, ctx->stream, sc, (int)SC_T2, params->beta / (double)T, (int)SC_TMP0, params->beta / (double)T, (int)SC_TMP2);
    hipLaunchKernelGGL(axpby_scalar_kernel, dim3(1), dim3(1), 0, ctx->stream, sc, (int)SC_T3, params->alpha / (double)T, (int)SC_TMP1, params->alpha / (double)T, (int)SC_TMP3);
  }
  // ---- S9: objective term 1 (one fp16 plane per operand is ample for a 1e-3 sum) and ridge terms ----
  if (stages & STRP_STAGE_OBJ) {
    Arena a2 = arena;
    STRP_TAKE(ctx, a2, red, double, 2 * 1024);
    if (!term1_identity) {   // A is whatever the caller left: the product itself
      Arena a3 = a2;
      PlaneOp Ak8;
      STRP_TRY(make_c_planes(ctx, a3, st->A, STRP_F32, lda, st->idx, s, T, 0, 1, &Ak8));
      GemmP p;
      memset(&p, 0, sizeof(p));
      p.P = W2Sp; p.P.lo = nullptr; p.Q = Ak8;
      p.M = d; p.N = (int)T; p.K = s;
      p.epi = EPI_RESID; p.Yin = st->Y; p.ldy = lda;
      gemm_plan_tiles(p, 1);
      const int nb = gemm_grid_blocks(p);
      STRP_TAKE(ctx, a3, redg, double, 2 * (size_t)nb);
      p.red = redg;
      STRP_TRY(launch_gemm(ctx, p));
      STRP_TRY(launch_block_sum(ctx, redg, nb, sc + SC_T1, nullptr, params->alpha / (double)T, 1.0));
    }
    hipLaunchKernelGGL(sumsq_kernel, dim3(1024), dim3(256), 0, ctx->stream, W2S, (long long)d * sp, red);
    STRP_TRY(launch_block_sum(ctx, red, 1024, sc + SC_W2SQ, nullptr, 1.0, 1.0));
    hipLaunchKernelGGL(sumsq_kernel, dim3(1024), dim3(256), 0, ctx->stream, W1S, (long long)s * d, red);
    STRP_TRY(launch_block_sum(ctx, red, 1024, sc + SC_W1SQ, nullptr, 1.0, 1.0));
  }
  STRP_HIP(ctx, hipGetLastError());
  st->iter += 1;

  if (report_host) {
    double* h = (double*)ctx->pinned;
    STRP_HIP(ctx, hipMemcpyAsync(h, sc, SC_COUNT * sizeof(double), hipMemcpyDeviceToHost, ctx->stream));
    STRP_HIP(ctx, hipMemcpyAsync(h + SC_COUNT, ctx->status_dev, sizeof(int32_t), hipMemcpyDeviceToHost, ctx->stream));
    STRP_HIP(ctx, hipStreamSynchronize(ctx->stream));
    memset(report_host, 0, sizeof(*report_host));
    report_host->lam1 = h[SC_LAM1];
    report_host->lam2 = h[SC_LAM2];
    report_host->terms[0] = h[SC_T1];
    report_host->terms[1] = h[SC_T2];
    report_host->terms[2] = h[SC_T3];
    report_host->terms[3] = params->alpha * h[SC_LAM2] * h[SC_W2SQ] / (double)T;
    report_host->terms[4] = params->alpha * h[SC_LAM1] * h[SC_W1SQ] / (double)T;
    report_host->J = report_host->terms[0] + report_host->terms[1] + report_host->terms[2];
    report_host->J_ridge = report_host->J + report_host->terms[3] + report_host->terms[4];
    report_host->tau = *(float*)(h + SC_TAU);
    report_host->s = s;
    report_host->status = *(int32_t*)(h + SC_COUNT);
    if (report_host->status != 0) {
      fail(ctx, (strp_status)report_host->status, "device status word = %d", report_host->status);
      STRP_TRY(fill_zero(ctx, ctx->status_dev, 256));
    }
  }
  return STRP_OK;
}

}  // extern "C"
