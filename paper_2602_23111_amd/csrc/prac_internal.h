// Internal declarations shared by the HIP translation units of libprac.
// Nothing here is part of the C ABI (see include/prac.h).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

#include <utility>
#include <vector>

#include "prac.h"

typedef unsigned short bf16_t;  // raw bf16 bit pattern
#define PRAC_MAX_DEVICES 64      // per-device tables (kernel attributes, the static scratch block's address)

struct prac_ctx {
  int device;
  hipStream_t stream;
  char* ws;           // device scratch, grown on demand
  size_t ws_bytes;
  char* static_scratch;  // this device's copy of the library's static scratch block (prac_weight_grad_static)
  int* d_flag;        // device-side numeric failure flag (0 = fine)
  int last_hip;       // last hipError_t that made a call fail
  int n_cu;
  int tune_splits;    // > 0: override the token-split count of C^T dY (tuning hook)
  int tune_one_launch;  // 1: the bf16 weight gradient as one launch instead of three (slabs, reduction, P T)
  int tune_tail;        // after the slabs of C^T dY: 0 built-in choice, 1 slab sum and P T as two launches, 2 as one
  int* d_sync;        // PRAC_SYNC_TILES x 3 counters of the one-launch weight gradient (zero between launches)
  int prof_kind;      // kernel kind bracketed by events (0: none), see prac_profile_select
  int prof_stride;    // every prof_stride-th launch of that kind carries the event pair
  int64_t prof_seen;  // launches of that kind since the selection
  hipEvent_t ev_start, ev_stop;  // set by ProfScope: the next PRAC_LAUNCH attaches them to its kernel
  std::vector<std::pair<hipEvent_t, hipEvent_t>> prof_pairs;  // recorded, not yet read
  std::vector<hipEvent_t> prof_pool;                          // idle events
};

// Brackets the launches issued during its lifetime with a HIP event pair on the ctx
// stream when the ctx is profiling this kernel kind.
struct ProfScope {
  prac_ctx* ctx;
  ProfScope(prac_ctx* c, int kind);
  ~ProfScope();
};

// Bump allocator over the ctx scratch for one API call.
struct WsPlan {
  size_t off = 0;
  size_t take(size_t bytes) {
    size_t o = off;
    off += (bytes + 255) & ~size_t(255);
    return o;
  }
};
int prac_ws_reserve(prac_ctx* ctx, size_t bytes);  // PRAC_OK / PRAC_ENOMEM / PRAC_EHIP

static inline int64_t round_up64(int64_t x, int64_t m) { return (x + m - 1) / m * m; }
// The streaming kernels address a row of a tile as a 32-bit byte offset from the tile's first row (at most 128
// rows of `pitch` 2-byte elements): row pitches up to this many elements keep it below 2^32.
constexpr int64_t PRAC_MAX_STREAM_PITCH = (int64_t)1 << 23;

// ---- bf16 MFMA GEMM ---------------------------------------------------------
// Out(M x N) = sum_k A(m,k) * B(k,n) over bf16 operands with fp32 accumulation.
// a_kc: A is stored M x K (K contiguous, lda) else K x M (M contiguous, lda).
// b_kc: B is stored N x K (K contiguous, ldb) else K x N (N contiguous, ldb).
struct GemmOperandB {
  const bf16_t* B;
  int64_t ldb;
  int N;
  void* out;  // out_bf16 ? bf16 : fp32, row-major M x N
  int64_t ldo;
};
struct GemmBf16Args {
  const bf16_t* A;
  int64_t lda;
  int M, K;
  bool a_kc, b_kc;
  GemmOperandB b0;     // columns of the first output
  GemmOperandB b1;     // optional second output sharing A (b1.B == nullptr: none)
  bool out_bf16;       // output element type (ignored when splits > 1)
  float beta;          // out = acc + beta * out (fp32 / bf16 out, splits == 1)
  int splits;          // > 1: split the K range, write fp32 slabs to `partial`
  float* partial;      // splits x M x N (b0 only), slab stride M*N
  int tile_hint;       // 0 auto
};
int launch_gemm_bf16(prac_ctx* ctx, const GemmBf16Args& a);

// ---- generic strided GEMM (fp32 / bf16 in, fp32 out) ----------------------------
// Out(m,n) = alpha * sum_k A(m,k) B(k,n) + beta * Out(m,n); element (m,k) of A at
// A[m*a_rs + k*a_cs], (k,n) of B at B[k*b_rs + n*b_cs]; accumulation in fp32 or
// fp64 (acc64).  k_stride > 1 visits k = 0, k_stride, 2 k_stride, ... (< K).
struct GemmGenArgs {
  const void* A;
  const void* B;
  prac_dtype adt, bdt;
  int64_t a_rs, a_cs, b_rs, b_cs;
  int M, N;
  int64_t K, k_stride;
  float* out;
  int64_t ldo;
  float alpha, beta;
  bool acc64;
  double* out64;  // when non-null the fp64 result is written here instead (ldo applies)
  int splits;     // > 1 with slabs != nullptr: split the reduction, then sum the slabs
  void* slabs;    // splits * M * N accumulators (fp64 if acc64 else fp32)
  size_t slab_bytes;  // size of `slabs`; a launch whose slabs would not fit is refused (PRAC_EINVAL)
};
int launch_gemm_generic(prac_ctx* ctx, const GemmGenArgs& a);

// ---- small helpers -------------------------------------------------------------
// out[i] = alpha * sum_s part[s*stride + i] + beta * out[i], i < n (fp32)
int launch_reduce_slabs(prac_ctx* ctx, const float* part, int splits, int64_t stride, float* out,
                        int64_t n, float alpha, float beta);
// out (N x M fp32, ld = ldo) = transpose of sum_s part[s][j][n], j < M
int launch_reduce_transpose_f32(prac_ctx* ctx, const float* part, int splits, int M, int N, float* out, int64_t ldo);
// fp32 matrix (rows x cols, ld) rows >= k_lo multiplied by s
int launch_scale_rows(prac_ctx* ctx, float* T, int rows, int cols, int64_t ld, int k_lo, float s);
int launch_philox(prac_ctx* ctx, uint64_t seed, uint32_t draw, uint32_t stream, void* out, int64_t n,
                  bool normal);
int launch_pack_basis(prac_ctx* ctx, const float* P, int64_t d, int64_t ldp, int c, bf16_t* Pt,
                      int64_t ldpt, bf16_t* Pn, int64_t ldpn);
int launch_cast_out(prac_ctx* ctx, const float* src, int64_t lds, void* dst, prac_dtype odt,
                    int64_t ldd, int rows, int cols, float beta);

// ---- kernels of the per-step path (ws_kernels.hip, hot_kernels.hip) -----------------
// Wfrag != nullptr: also Y (N x m, ldy) = X W, W in the fragment order of Pfrag with ncb_w column blocks
int launch_compress_ws(prac_ctx* ctx, const bf16_t* X, int64_t ldx, int N, int d, const bf16_t* Pfrag, int ncb,
                       int c, bf16_t* C, int64_t ldc, bool packed, const bf16_t* Wfrag, int ncb_w, int m,
                       bf16_t* Y, int64_t ldy);
// Xh (N x d, bf16) = C (N x c bf16, row-major with ldc or packed; c <= 256) Ps^T with Ps^T in fragment
// order [16][ncb][64][8] (pack_ptfrag_kernel); ncb a multiple of 8 covering d.
int launch_reconstruct_ws(prac_ctx* ctx, const bf16_t* C, int64_t ldc, bool packed, int N, int c, int d,
                          const bf16_t* Ptfrag, int ncb, bf16_t* Xh, int64_t ldxh);
// W (bf16; w_layout 0: d x m, 1: m x d; ldw) -> [nkb][ncb_w][64][8] fragment order, zero padded
int launch_pack_wfrag(prac_ctx* ctx, const bf16_t* W, int64_t ldw, int w_layout, int64_t d, int m, int nkb,
                      int ncb_w, bf16_t* out);
// token-split partial sums of C^T dY_h for n_out outputs that share C; slabs[h] is splits x c x m[h]
#define PRAC_CTDY_MAX_OUT 4
int launch_ctdy_ws(prac_ctx* ctx, const bf16_t* Cpk, int c, int N, int n_out, const bf16_t* const* dY,
                   const int64_t* lddy, const int* m, float* const* slabs, int splits);
// The whole weight gradient in one launch: partial slabs, their sum as T (bf16, fragment order, rows >= k_lo
// scaled) and dW_h = P T_h, the workgroups of a column tile meeting through `cnt` (PRAC_SYNC_INTS_PER_TILE
// ints per 128-column tile over all outputs, zero before and after the launch).  `splits` comes from
// wgrad_fused_splits (0: this shape runs as three launches).
#define PRAC_SYNC_TILES 4096
#define PRAC_SYNC_INTS_PER_TILE 8
#define PRAC_SYNC_BYTES ((size_t)PRAC_SYNC_TILES * PRAC_SYNC_INTS_PER_TILE * sizeof(int))
int wgrad_fused_splits(int n_cu, int c, int n_out, const int64_t* m, int64_t N, int tune_splits);
int launch_wgrad_fused(prac_ctx* ctx, const bf16_t* Cpk, int c, int N, int n_out, const bf16_t* const* dY,
                       const int64_t* lddy, const int* m, float* const* slabs, int splits, int k_lo, float scale_hi,
                       int nckb, const int* nmb, bf16_t* const* Tf, const bf16_t* Pa, int d, void* const* dW,
                       const int64_t* lddw, bool out_bf16, float beta, int* cnt);
int launch_pack_pfrag(prac_ctx* ctx, const float* P, int64_t d, int64_t ldp, int c, int nkb, int ncb, bf16_t* out);
int launch_unpack_c(prac_ctx* ctx, const bf16_t* Cpk, int N, int c, bf16_t* C, int64_t ldc);
int launch_pack_c(prac_ctx* ctx, const bf16_t* C, int64_t ldc, int N, int c, bf16_t* Cpk);

int launch_reduce_to_tfrag(prac_ctx* ctx, int n_out, const float* const* slabs, int splits, int c, const int* m, int k_lo,
                           float scale_hi, int nkb, const int* nmb, bf16_t* const* Tf);
int launch_pack_pafrag(prac_ctx* ctx, const float* P, int64_t d, int64_t ldp, int c, int nrb, int nkb, bf16_t* out);
// dW_h (d x m_h) = P T_h (+ beta dW_h) for n_out <= PRAC_CTDY_MAX_OUT outputs in one launch
int launch_pt(prac_ctx* ctx, const bf16_t* Pa, int n_out, const bf16_t* const* Tf, int d, const int* m, int nkb,
              const int* nmb, void* const* dW, const int64_t* lddw, bool out_bf16, float beta);

// dW_h (d x m_h) = P (scaled sum of the slabs of C^T dY_h) (+ beta dW_h) in one launch: the slab reduction and
// launch_pt without T passing through memory; same arithmetic in the same order, bit-identical results
bool sum_pt_eligible(int n_out, const int* m, int splits);  // shapes the one-launch form covers
int launch_sum_pt(prac_ctx* ctx, const bf16_t* Pa, int n_out, const float* const* slabs, int splits, int c, int k_lo,
                  float scale_hi, int nkb, int d, const int* m, void* const* dW, const int64_t* lddw, bool out_bf16,
                  float beta);

// P (d x c fp32, ldp) -> B operand of Xh = C Ps^T in fragment order [nkb][ncb][64][8] (bf16, zero padded):
// element (k = column of P, n = row of P) = P[n][k] * (k >= k_lo ? scale_hi : 1)
int launch_pack_ptfrag(prac_ctx* ctx, const float* P, int64_t d, int64_t ldp, int c, int k_lo, float scale_hi,
                       int nkb, int ncb, bf16_t* out);

// ---- basis fit -----------------------------------------------------------------
int fit_basis_device(prac_ctx* ctx, const void* X, prac_dtype xdt, int64_t N, int64_t d, int64_t ldx,
                     int k, int r, uint64_t seed, uint32_t draw, int refresh, const prac_fit_opts& o,
                     float* P, int64_t ldp);
size_t gram_scratch_bytes(int n_cu, const void* X, prac_dtype xdt, int64_t N, int64_t d,
                          int64_t ldx, int64_t row_stride, int64_t ldg);
// scratch of one prac_fit_basis call (X is only looked at for its alignment)
size_t fit_scratch_bytes(int n_cu, const void* X, prac_dtype xdt, int64_t N, int64_t d, int64_t ldx, int k, int r,
                         int refresh, const prac_fit_opts& o);
int64_t fit_slab_margin(int n_cu, prac_dtype xdt, int64_t N, int64_t d, int k, int r, int refresh,
                        const prac_fit_opts& o);
int gram_device(prac_ctx* ctx, const void* X, prac_dtype xdt, int64_t N, int64_t d, int64_t ldx,
                int64_t row_stride, float* G, int64_t ldg, char* scratch);

// Launch on the ctx stream; when a ProfScope is open, the kernel's own begin / end time
// stamps go into its event pair (so the measured time excludes launch gaps).
#define PRAC_LAUNCH(ctx, kern, grid, block, smem, ...)                                              \
  do {                                                                                             \
    if ((ctx)->ev_start) {                                                                         \
      hipExtLaunchKernelGGL(kern, grid, block, smem, (ctx)->stream, (ctx)->ev_start, (ctx)->ev_stop, 0, \
                            __VA_ARGS__);                                                          \
      (ctx)->ev_start = nullptr;                                                                   \
      (ctx)->ev_stop = nullptr;                                                                    \
    } else {                                                                                       \
      hipLaunchKernelGGL(kern, grid, block, smem, (ctx)->stream, __VA_ARGS__);                     \
    }                                                                                              \
  } while (0)

#define PRAC_HIP_TRY(ctx, expr)                 \
  do {                                          \
    hipError_t e__ = (expr);                    \
    if (e__ != hipSuccess) {                    \
      (ctx)->last_hip = (int)e__;               \
      return PRAC_EHIP;                         \
    }                                           \
  } while (0)
