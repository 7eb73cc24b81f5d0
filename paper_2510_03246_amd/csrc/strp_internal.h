// Internal declarations shared by the HIP translation units of libstrp.so (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "strp.h"

namespace strp {
struct CoJob;
}

struct strp_ctx {
  int device;
  hipStream_t stream;
  char* ws;            // caller-owned device workspace
  size_t ws_bytes;
  int precision;       // strp_precision
  int32_t* status_dev; // first word of the workspace
  void* pinned;        // small pinned host buffer for report read-back
  char err[512];
  struct Profiler* prof;  // optional per-kernel event timing (host object)
  unsigned char prod_planes[8][2];  // fp16 planes (1 or 2) of the P and Q operand per strp_product of strp_admm_step
  // Set by strp_admm_step while a streaming job may ride along with the factorisation chains (see cojob.h); null
  // everywhere else.  chol_factor gives its short launches spare workgroups for it.
  const strp::CoJob* cojob;
};

struct Profiler;

namespace strp {

// ---- optional per-kernel timing with HIP events on the context's stream -----------------------
// prof_begin returns a record index (or -1 when profiling is off); prof_end closes it.
int prof_begin(strp_ctx* ctx, const char* name, double flops, double bytes);
void prof_end(strp_ctx* ctx, int rec);
struct ProfScope {
  strp_ctx* ctx;
  int rec;
  ProfScope(strp_ctx* c, const char* name, double flops, double bytes) : ctx(c), rec(prof_begin(c, name, flops, bytes)) {}
  ~ProfScope() { prof_end(ctx, rec); }
};

// ---- error helpers -------------------------------------------------------------------
strp_status fail(strp_ctx* ctx, strp_status st, const char* fmt, ...);
#define STRP_HIP(ctx, call)                                                              \
  do {                                                                                   \
    hipError_t e_ = (call);                                                              \
    if (e_ != hipSuccess)                                                                \
      return strp::fail((ctx), STRP_EHIP, "%s failed: %s", #call, hipGetErrorString(e_)); \
  } while (0)
#define STRP_TRY(expr)                  \
  do {                                  \
    strp_status s_ = (expr);            \
    if (s_ != STRP_OK) return s_;       \
  } while (0)

// ---- workspace bump arena (256-byte granules); the first granule holds the status word --
struct Arena {
  char* base;
  size_t off, cap;
  Arena() : base(nullptr), off(0), cap(0) {}
  explicit Arena(strp_ctx* ctx) : base(ctx->ws), off(256), cap(ctx->ws_bytes) {}
  Arena(void* block, size_t bytes) : base((char*)block), off(0), cap(bytes) {}   // sub-arena over a block taken elsewhere
  void* take(size_t bytes) {
    size_t b = (bytes + 255) & ~size_t(255);
    if (!base || off + b > cap) return nullptr;
    void* p = base + off;
    off += b;
    return p;
  }
};
#define STRP_TAKE(ctx, arena, var, type, count)                                                     \
  type* var = (type*)(arena).take(sizeof(type) * (size_t)(count));                                  \
  if (!var) return strp::fail((ctx), STRP_ENOMEM, "workspace too small for %s (%zu bytes more)",    \
                              #var, sizeof(type) * (size_t)(count))

// ---- MFMA GEMM family on 16-bit operand planes (gemm_mfma.hip, split_planes.hip) -----------------
// An operand as the matrix cores see it: one (hi) or two (hi, lo) fp16 planes in the panel-major chunk layout
//   offset(k, r) = (((r / 128) * kg + k / 8) * 128 + r % 128) * 8 + k % 8
// k = contraction index, r = output row (P) or output column (Q); npan panels of 128 rows, kg k-groups of 8
// (kg = plane_kg(K): a multiple of four, padding zero).
// scale (device, optional): the planes hold x * scale; the GEMM epilogue divides it out.
struct PlaneOp {
  const unsigned short* hi;
  const unsigned short* lo;
  long long kg;
  int npan;
  const float* scale;
};
// k-groups allocated for a contraction of length K: a multiple of four, the pad groups zero-filled (the pipelined
// kernel moves two k-groups per stage and multiplies four per matrix-core instruction, both without tail logic)
static inline long long plane_kg(long long K) { return (((K + 7) / 8) + 3) & ~3LL; }
static inline size_t plane_elems(long long rows, long long K) {
  return (size_t)((rows + 127) / 128) * (size_t)plane_kg(K) * 1024;
}

enum { EPI_PARTIAL = 0, EPI_STORE = 1, EPI_INITZ = 2, EPI_RESID = 3, EPI_AUPD = 4, EPI_ZUPD = 5 };
enum { SRC_F64 = 0, SRC_F32 = 1, SRC_BF16 = 2 };

struct GemmP {
  PlaneOp P, Q;        // C[m, n] = sum_k P(k, m) Q(k, n)
  int M, N;
  long long K;
  int force_wt;        // 2 forces the 128x128 register-staged kernel
  int wt;              // 32x32 MFMA tiles per wavefront per dimension: 2 (128x128 blocks) or 4 (256x256), set by gemm_plan_tiles
  int tilesM, tilesN, ntiles;
  int gridM, gridN;    // tile grid the blocks are laid over: tilesM x tilesN, or the folded triangle (see decode_tile)
  int gm, gn;          // tile group (gm x gn = tiles that are resident on one XCD together)
  int triangle;        // P == Q, only tiles with tn <= tm are computed
  int splits;
  long long kchunk;    // K range per split (multiple of the K tile)
  int epi;
  float* out;          // PARTIAL: [splits][M][N]; STORE: [M x ldo]
  long long ldo;
  const float* Yin;    // RESID: Y
  long long ldy;
  float* Zs;           // INITZ / AUPD / ZUPD state pointers, leading dimension lda
  float* As;
  float* Z0s;
  long long lda;
  const int* oidx;     // AUPD / ZUPD: output row m is state row oidx[m]
  float alpha, beta;
  double* red;         // per-block partial sums [gridDim.x][2] (INITZ, RESID, ZUPD)
  int write_out;       // ZUPD: 1 = update Z, 0 = only accumulate the objective sums
  unsigned short* k8_hi;  // optional operand planes of the produced values with k = output row, r = output column
  unsigned short* k8_lo;  //   (STORE: C, INITZ: relu(C), RESID: Y - C; not offered by AUPD / ZUPD); k8_kg = M / 8 groups, ceil(N/128) panels
  long long k8_kg;
  // AUPD / ZUPD, optional: scoring sums of the rows being written, one fp32 partial per output row and 64-column strip,
  //   rs_out[(q * rs_slots + strip) * M + m];  AUPD: q = 0 sum a^2, q = 1 sum a relu(z0) (iff rs_z0); ZUPD: q = 0 sum z0 z
  //   (iff rs_z0).  rs_z0 = the Z0 state tensor (leading dimension lda, rows gathered like Zs).  rs_slots = ceil(N / 64).
  float* rs_out;
  const float* rs_z0;
  int rs_slots;
};

strp_status launch_gemm(strp_ctx* ctx, GemmP& p);
int gemm_grid_blocks(const GemmP& p);
void gemm_plan_tiles(GemmP& p, int want_splits);

// Sum split-K partials in fp64; optional symmetric completion from the computed lower half.
// outf / outd (either may be null): [M x ldo]; accumulate adds to outf's previous content.
strp_status launch_splitk_reduce(strp_ctx* ctx, const float* part, int splits, int M, int N, int triangle,
                                 float* outf, long long ldof, double* outd, long long ldod, double* diag,
                                 int accumulate);
// Sum per-block fp64 partials red[nblocks][2] into dst[0], dst[1] (fixed order).
strp_status launch_block_sum(strp_ctx* ctx, const double* red, int nblocks, double* dst0, double* dst1,
                             double scale0, double scale1);

// fp32 / bf16 activation rows (optionally gathered by idx) -> fp16 planes; any output pair may be null.
//   t_* : contraction over tokens   (k = token,   r = row):   plane_elems(rows, T)
//   c_* : contraction over channels (k = row,     r = token): plane_elems(T, rows)
strp_status split_act(strp_ctx* ctx, const void* src, int src_dtype, long long lds, const int* idx, int rows, long long T,
                      int relu_t, int relu_c, unsigned short* t_hi, unsigned short* t_lo, unsigned short* c_hi,
                      unsigned short* c_lo);
// One fp16 plane of a [C x T] quantity with k = channel, r = token (plane_elems(T, C)) -> the plane with k = token,
// r = channel (plane_elems(C, T)); padding tokens zero.
strp_status plane_c_to_t(strp_ctx* ctx, const unsigned short* src, unsigned short* dst, int C, long long T);
// Small matrix (weights) -> planes with k = column, r = row: plane_elems(rows, cols); src_kind = SRC_*.
strp_status split_small(strp_ctx* ctx, const void* src, int src_kind, long long lds, int rows, int cols, int transpose,
                        const float* scale_dev, unsigned short* hi, unsigned short* lo);
// *scale_out = power of two that brings max|src| into [2^11, 2^12).
strp_status weight_scale(strp_ctx* ctx, const void* src, int src_kind, long long lds, int rows, int cols, float* scale_out);

// ---- fp64 dense kernels (dense_f64.hip) ---------------------------------------------------
constexpr int NB = 64;  // block order of the factorisation
// In-place lower Cholesky of the n x n fp64 matrix A (ld); the caller has added the ridge.  On return the blocks of A
// below the NB x NB diagonal blocks hold L; the diagonal blocks themselves are left as they were when their step
// began (never needed: invd has their inverses).  invd: [ceil(n/NB)][NB*NB] inverses of the diagonal blocks of L.
// status: device word.
strp_status chol_factor(strp_ctx* ctx, double* A, int n, long long ld, double* invd, int32_t* status);
// Linv [n x n, ld n] = L^-1 from the off-diagonal blocks of the factor and its inverted diagonal blocks; tmp: n x n scratch.
strp_status tri_inverse(strp_ctx* ctx, const double* L, int n, long long ldl, const double* invd, double* Linv, double* tmp);
// In place X <- X (L L^T)^-1 = (X Linv^T) Linv for X [m x n] (ld n); tmp: m x n scratch.
strp_status apply_inverse_right(strp_ctx* ctx, const double* Linv, int n, double* X, int m, double* tmp);
// C[M x N] = alpha * A * B + beta * C with arbitrary element strides; lower != 0 skips tiles above
// the diagonal; tri limits a tile's K range to the non-zero part of a triangular operand: 1: k < n0 + tile,
// 2: k >= n0 (B), 3: k >= m0, 4: k < m0 + tile (A).
strp_status dgemm(strp_ctx* ctx, int M, int N, int K, double alpha, const double* A, long long rsa,
                  long long csa, const double* B, long long rsb, long long csb, double beta, double* C,
                  long long ldc, int lower, int tri = 0);
// Ad[i*ld+j] = (double)Af[i*ldf+j] + (i==j ? lam (or *lam_dev if non-null) : 0)
strp_status f32_to_f64_ridge(strp_ctx* ctx, const float* Af, long long ldf, double* Ad, long long ld, int n,
                             double lam, const double* lam_dev);

// ---- reductions, scores, allocation, select (score_select.hip) ------------------------------
strp_status launch_row_sums(strp_ctx* ctx, const void* A, int a_dtype, const float* Z, const float* Z0,
                            long long ld, long long T, int rows, int mode, double* sums /*[4][rows]*/);
// part[nq][slots][M] fp32 strip sums written by the AUPD / ZUPD epilogues -> rowsums[qdst * f + idx[m]] (fp64);
// chunk_sums: rowsum_scratch_bytes(nq, M) bytes of scratch.
strp_status launch_rowsum_reduce(strp_ctx* ctx, const float* part, int nq, int slots, int M, const int32_t* idx, double* rowsums, int f,
                                 int qdst0, int qdst1, double* chunk_sums);
size_t rowsum_scratch_bytes(int nq, int M);
strp_status launch_colnorm2(strp_ctx* ctx, const void* W, int w_dtype, int rows, int cols, long long ldw,
                            double* n2);
strp_status launch_unit_scores(strp_ctx* ctx, const double* sums, const double* n2, int n_channels, int group,
                               int mode, float* score, double* energy_out);
strp_status launch_alloc(strp_ctx* ctx, const double* energies, int L, const int32_t* n_units,
                         const int32_t* group_id, double rbar, double temperature, double rmax, int rule, double* r_out,
                         int32_t* nprune_out);
strp_status launch_weight_energy(strp_ctx* ctx, const strp_weight_ref* mats, int n_mats, double var_coef, double l2_coef,
                                 double scale, double* energy, double* partial);
size_t weight_energy_scratch_bytes();
strp_status launch_topk(strp_ctx* ctx, const float* score, int n, int k, int group, uint8_t* mask, int32_t* idx,
                        float* tau, void* scratch, size_t scratch_bytes);
size_t topk_scratch_bytes(int n);

// ---- small elementwise helpers (dense_f64.hip) -----------------------------------------------
// dst (fp32, [rows x ldd]) = src (fp64, [rows x lds]) cast; pad columns [cols, ldd) zero-filled.
strp_status cast_f64_f32(strp_ctx* ctx, const double* src, long long lds, float* dst, long long ldd, int rows,
                         int cols);
// W[out x in] dense fp32: scatter compact solution rows/columns by idx, everything else zero.
strp_status scatter_weights(strp_ctx* ctx, const double* sol, long long lds, int side, const int32_t* idx,
                            int s, float* W, int out, int in);
strp_status fill_zero(strp_ctx* ctx, void* ptr, size_t bytes);

}  // namespace strp
