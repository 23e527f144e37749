/*
 * prac.h - C ABI of the MI355X (gfx950) PRAC hot-path library.
 *
 * PRAC (Principal-Random subspace Activation Compression) keeps, for a linear
 * layer Y = X W, only the projection C = X P of the saved activation X
 * (N tokens x d features) onto a basis P = [Q1 | Q2] with orthonormal columns:
 * Q1 (d x k) spans the top-k right singular vectors of X, Q2 (d x r) is an
 * orthonormal basis of (I - Q1 Q1^T) S for a Gaussian S, and the random block
 * is weighted by the scaling factor s = (d - k) / r so that the reconstruction
 * X~ = C_1 Q1^T + s C_2 Q2^T is unbiased (Section 4.3, Eq. (S_o), Eq. (R),
 * Theorem 1).  The weight gradient is then X~^T dY (Lemma 1; Alg. 2).
 *
 * Symbols: the paper's n, r_1, r_2 and scaling factor k are d, k, r and
 * `scale` here; c = k + r.
 *
 * Conventions that hold for every entry point
 *   - Matrices are row-major with an explicit leading dimension (elements).
 *   - Unless marked [host], a pointer is a caller-owned DEVICE pointer valid on
 *     the ctx device.  The library never frees or keeps user buffers.
 *   - Work is enqueued on the ctx stream and the call returns without waiting,
 *     PROVIDED the ctx scratch block is large enough.  Scratch memory lives in
 *     the ctx; a call that needs more than the ctx holds waits for the device,
 *     frees the block and allocates a larger one (hipMalloc).  Callers that
 *     must not wait or allocate inside a hot call size the block up front:
 *     prac_workspace_bytes for every call shape they will issue, then one
 *     prac_reserve_workspace with the largest answer.  A ctx must not be used
 *     from two host threads at once.
 *   - Return value: PRAC_OK (0) or a negative prac_status.  Shape and argument
 *     errors are detected on the host BEFORE anything is enqueued and before
 *     the ctx is looked at, so they can be exercised without a GPU.
 *   - Size limits (PRAC_EINVAL beyond them): 1 <= N < 2^31 tokens,
 *     1 <= d, m <= 2^20 features.
 *   - bf16 fast paths need 16-byte aligned base pointers and leading
 *     dimensions that are multiples of 8 elements (and at most 2^23, times the
 *     row stride where one applies); otherwise a slower generic kernel runs
 *     (same results to rounding).  They read rows in whole 16-byte
 *     chunks: a matrix of R rows with leading dimension ld must own R * ld
 *     elements (the up to 7 elements after a row's last column may be read,
 *     never used, also in the last row); nothing outside those R * ld elements
 *     is ever read or written.
 */
#ifndef PRAC_H
#define PRAC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct prac_ctx prac_ctx;

typedef enum { PRAC_F32 = 0, PRAC_BF16 = 1 } prac_dtype;

typedef enum {
  PRAC_OK = 0,
  PRAC_EINVAL = -1,       /* bad shape, rank split, leading dimension, null pointer */
  PRAC_ENOMEM = -2,       /* device scratch allocation failed */
  PRAC_EHIP = -3,         /* a HIP runtime call failed (see prac_last_hip_error) */
  PRAC_ENUMERIC = -4,     /* non-finite Gram or orthonormalisation breakdown */
  PRAC_EUNSUPPORTED = -5, /* valid request this build has no kernel for */
  PRAC_ENOCTX = -6,       /* ctx is NULL (arguments themselves were valid) */
  PRAC_ETOOBIG = -7       /* prac_weight_grad_static: the call needs more scratch than the static block holds */
} prac_status;

/* refresh bits of prac_fit_basis: the two lazy-update branches of Alg. 1 */
enum { PRAC_REFRESH_PRINCIPAL = 1, PRAC_REFRESH_RANDOM = 2 };

/* Options of the principal-subspace iteration (the paper only says "SVD";
 * this library finds the same subspace by block power iteration on X^T X with
 * orthonormalisation and a final Rayleigh-Ritz step).  Zero / NULL = defaults. */
typedef struct {
  int iters;           /* power iterations; 0 -> 8 */
  int oversample;      /* extra block columns; <0 -> none, 0 -> min(k, d-k) */
  int64_t row_stride;  /* Gram over rows 0, stride, 2*stride, ...; 0 -> 1 */
  int warm_start;      /* 1: start the block from the Q1 already in P */
} prac_fit_opts;
/* Tracking refit: with warm_start = 1 and oversample < 0 (block width k), bf16 X that is
 * 16-byte aligned with ldx a multiple of 8, at least 256 rows in
 * the (sub)sample, d >= 128 and k <= 1024, no Gram matrix is formed: each of the `iters`
 * iterations is one subspace-iteration step Q1 <- orth(X^T (X Q1)) through the compress and
 * C^T dY kernels, without the Rayleigh-Ritz step (Q1 spans the tracked subspace; its columns
 * are not ordered by eigenvalue).  The lazy-update premise of Alg. 1 - the subspace drifts
 * slowly between refreshes - is what makes one or two such steps enough. */

/* ---- context ----------------------------------------------------------- */
/* Bind a context to HIP device `device` and to `hip_stream` (a hipStream_t;
 * NULL = the default stream).  *out is [host]. */
int prac_create(prac_ctx** out, int device, void* hip_stream);
int prac_destroy(prac_ctx* ctx);
int prac_set_stream(prac_ctx* ctx, void* hip_stream);
/* Block until the ctx stream is idle and return the first device-side
 * numeric failure recorded since the last call (PRAC_OK if none). */
int prac_sync_status(prac_ctx* ctx);
const char* prac_strerror(int status);          /* [host] static string */
int prac_last_hip_error(const prac_ctx* ctx);   /* last hipError_t seen */

/* ---- scratch sizing ------------------------------------------------------ */
/* The shape of one call, for prac_workspace_bytes.  Fields an entry point does not
 * take are ignored.  `generic` = 1 says that the call will run the strided kernels
 * (a base pointer that is not 16-byte aligned or a leading dimension that is not a
 * multiple of 8 elements; fp32 data always does). */
typedef enum {
  PRAC_OP_GRAM = 1,        /* prac_gram: dt, N, d, fit.row_stride */
  PRAC_OP_FIT_BASIS = 2,   /* prac_fit_basis: dt, N, d, k, r, refresh, fit */
  PRAC_OP_COMPRESS = 3,    /* prac_compress: dt, N, d, k + r, c_layout, have_p_lp */
  PRAC_OP_FUSED_FWD = 4,   /* prac_compress_fused_fwd: as compress, n_out = 1, m[0] */
  PRAC_OP_WEIGHT_GRAD = 5, /* prac_weight_grad(_shared): dt, odt, N, d, k, r, n_out, m[], c_layout, have_p_lp */
  PRAC_OP_RECONSTRUCT = 6  /* prac_reconstruct: dt, N, d, k, r, c_layout */
} prac_op;
#define PRAC_MAX_SHARED 4
typedef struct {
  int op;                      /* prac_op */
  int dt;                      /* prac_dtype of X / C / dY */
  int odt;                     /* prac_dtype of dW (weight gradient) */
  int64_t N, d;
  int k, r;
  int n_out;                   /* outputs that share C (weight gradient), 1 for the fused forward */
  int64_t m[PRAC_MAX_SHARED];  /* their widths */
  int c_layout;                /* prac_c_layout */
  int have_p_lp;               /* 1: the call hands over a packed basis P_lp */
  int generic;                 /* 1: unaligned operands, the strided kernels run */
  int refresh;                 /* fit: PRAC_REFRESH_* bits */
  prac_fit_opts fit;           /* fit / Gram: options as passed to the call */
} prac_call_shape;
/* Bytes of ctx scratch one call of that shape needs (0: none); (size_t)-1 for a shape
 * the entry point would reject.  [host]; ctx may be NULL (then the split counts are
 * planned for the 256 compute units of an MI355X).  The answer depends on the ctx's
 * tuning overrides (prac_set_tuning): query after setting them. */
size_t prac_workspace_bytes(const prac_ctx* ctx, const prac_call_shape* shape /* [host] */);
/* Grow the ctx scratch block to at least `bytes` now (waits for the device and
 * reallocates if it is smaller; never shrinks).  After it, no call whose
 * prac_workspace_bytes is <= bytes waits, frees or allocates. */
int prac_reserve_workspace(prac_ctx* ctx, size_t bytes);
/* Test hook [host]: bytes by which the fit's split-sum block exceeds the largest split
 * product prac_fit_basis issues for that shape (negative: the plan would be too small;
 * the launchers refuse such a product instead of writing past the block). */
int64_t prac_debug_fit_slab_margin(const prac_call_shape* shape /* [host] */);

/* ---- per-kernel timing hook (for benchmarks) ---------------------------- */
/* While a kind other than PRAC_KERNEL_NONE is selected, every launch of that
 * kernel is bracketed by a HIP event pair on the ctx stream.  prac_profile_read
 * waits for the stream, writes the summed duration [host, milliseconds] and the
 * number of launches [host] since the last read, and clears both. */
enum {
  PRAC_KERNEL_NONE = 0,
  PRAC_KERNEL_COMPRESS = 1,   /* C = X P */
  PRAC_KERNEL_CT_DY = 2,      /* token-split partial sums of C^T dY */
  PRAC_KERNEL_T_REDUCE = 3,   /* slab reduction + scaling factor + transpose */
  PRAC_KERNEL_P_T = 4,        /* dW = P T */
  PRAC_KERNEL_GRAM = 5,       /* X^T X partial sums */
  PRAC_KERNEL_FUSED_FWD = 6,  /* [Y | C] = X [W | P] */
  PRAC_KERNEL_RECONSTRUCT = 7, /* Xh = C Ps^T */
  PRAC_KERNEL_WEIGHT_GRAD = 8, /* the whole weight gradient in one launch (PRAC_TUNE_WGRAD_ONE_LAUNCH): partial
                                  sums of C^T dY, their sum T and dW = P T (kinds 2 - 4 then see no launch) */
  PRAC_KERNEL_SUM_P_T = 9      /* slab reduction + scaling factor and dW = P T as one launch (PRAC_TUNE_WGRAD_TAIL;
                                  kinds 3 and 4 then see no launch) */
};
int prac_profile_select(prac_ctx* ctx, int kind);
int prac_profile_read(prac_ctx* ctx, double* total_ms, int64_t* launches);
/* Same, launch by launch: the first min(cap, *launches) durations [host, milliseconds], in
 * launch order, go to each_ms (may be NULL when cap is 0). */
int prac_profile_read_each(prac_ctx* ctx, float* each_ms, int64_t cap, int64_t* launches);
/* Launch-shape override for sweeps: PRAC_TUNE_CTDY_SPLITS = number of token ranges
 * the C^T dY reduction is split into (1..64; 0 restores the built-in choice).
 * PRAC_TUNE_PROFILE_STRIDE = n (1..1024; 0 means 1): only every n-th launch of the selected
 * kernel kind, counted from the selection, carries the event pair (an event pair costs a few
 * microseconds of stream time, which a benchmark loop may not want on every step).
 * PRAC_TUNE_WGRAD_ONE_LAUNCH = 1: the bf16 weight gradient runs as one launch (the workgroups of a
 * column tile of T meet inside the kernel to sum their partial sums and to form dW = P T) instead of
 * three (partial sums, their reduction, P T); 0 restores the default.  Results are bit-identical; the
 * three launches are the faster of the two on an MI355X at every benchmarked shape.
 * PRAC_TUNE_WGRAD_TAIL: what follows the partial sums of C^T dY in the bf16 weight gradient.  2: their
 * reduction (with the scaling factor) and dW = P T run as one launch, T staying in LDS (for output widths
 * that are multiples of 4 and token-range counts that are multiples of 4; other shapes keep the two
 * launches); 1: as two launches with T (bf16, fragment order) in ctx scratch between them; 0 restores
 * the built-in choice (one launch for k + r > 256 and d <= 2048).  Results are bit-identical. */
enum { PRAC_TUNE_CTDY_SPLITS = 1, PRAC_TUNE_PROFILE_STRIDE = 2, PRAC_TUNE_WGRAD_ONE_LAUNCH = 3, PRAC_TUNE_WGRAD_TAIL = 4 };
int prac_set_tuning(prac_ctx* ctx, int key, int value);

/* ---- Gaussian draw (Eq. (S_o): S_ij ~ N(0,1) i.i.d.) -------------------- */
/* Counter-based Philox4x32-10.  Word i of stream (seed, draw, stream) is lane
 * i%4 of the block with counter (i/4 low, i/4 high, stream, draw) and key
 * (seed low, seed high); draw < 2^32.  uniforms: u = ((w >> 9) + 1/2) 2^-23;
 * normals by Box-Muller on consecutive pairs (cos first, then sin).
 * out: n elements.  stream 0 seeds the power-iteration block, 1 is S. */
int prac_philox_words(prac_ctx* ctx, uint64_t seed, uint64_t draw, uint32_t stream,
                      uint32_t* out, int64_t n);
int prac_philox_normal(prac_ctx* ctx, uint64_t seed, uint64_t draw, uint32_t stream,
                       float* out, int64_t n);

/* ---- Gram matrix (first step of "top-r_1 right singular vectors of X",
 *      Alg. 1 principal-subspace update) --------------------------------- */
/* G (d x d, fp32, ldg >= d) = Xs^T Xs over rows 0, row_stride, ... of X
 * (N x d, ldx >= d).  Both triangles are written. */
int prac_gram(prac_ctx* ctx, const void* X, prac_dtype xdt, int64_t N, int64_t d,
              int64_t ldx, int64_t row_stride, float* G, int64_t ldg);

/* ---- basis fit (Section 4.3 construction; Alg. 1, both update branches) -- */
/* Bytes of the packed low-precision copy of a d x c basis (see below). */
size_t prac_basis_lp_bytes(int64_t d, int c);
/* Build the packed bf16 copy P_lp of P (d x c fp32, ldp >= c) that the bf16
 * kernels read: P^T as c x round_up(d,64) bf16, P as d x round_up(c,64) bf16,
 * and P in MFMA fragment order both as a B operand (compress) and as an A
 * operand (dW = P T); all zero padded (the B-operand fragments to a multiple
 * of 256 rows), each part 256-byte aligned. */
int prac_pack_basis(prac_ctx* ctx, const float* P, int64_t d, int64_t ldp, int c,
                    void* P_lp);
/* Writes P = [Q1 | Q2] (d x (k+r) fp32, UNSCALED, ldp >= k+r), optionally its
 * packed copy P_lp (may be NULL) and *scale [host] = (d-k)/r (0 when r = 0).
 * refresh: PRAC_REFRESH_PRINCIPAL recomputes Q1 from X; if clear, Q1 is read
 * from the first k columns of P.  PRAC_REFRESH_RANDOM redraws Q2 from
 * (seed, draw); if clear, columns k.. of P are left as they are.
 * Needs 0 <= k, 0 <= r, 1 <= k+r <= d.  X may be NULL when Q1 is not
 * refreshed or k = 0.  A batch whose (sub)sampled rows are fewer than k has
 * rank below k: Q1 then holds the principal directions of those rows and an
 * orthonormal completion drawn from (seed, draw), generator stream 2, like Q2.
 * prac_sync_status reports PRAC_ENUMERIC afterwards if a factorisation met a
 * pivot that was not positive or a block did not come out orthonormal (data of
 * much lower rank than its row count can do that). */
int prac_fit_basis(prac_ctx* ctx, const void* X, prac_dtype xdt, int64_t N, int64_t d,
                   int64_t ldx, int k, int r, uint64_t seed, uint64_t draw, int refresh,
                   const prac_fit_opts* opts /* [host], may be NULL */, float* P,
                   int64_t ldp, void* P_lp, float* scale /* [host], may be NULL */);

/* ---- compression (Alg. 1 compression step, unscaled) ------------------- */
/* Storage of the compressed activation C (N x c).
 *   PRAC_C_ROWMAJOR  N x c row-major with leading dimension ldc >= c.
 *   PRAC_C_PACKED    bf16 only; the layout the weight-gradient kernel reads without
 *                    a transpose: blocks of 16 tokens x 32 columns, block (tb, cb) at
 *                    element offset ((tb * ceil(c/32) + cb) * 64 + lane) * 8 + e with
 *                    lane = 32 h + (column % 32) and token = 16 tb + (e < 4 ? 4 h + e
 *                    : 8 + 4 h + e - 4), h in {0,1}, e in 0..7.  The buffer holds
 *                    8 * ceil(N/128) token blocks (whole 128-token tiles); rows /
 *                    columns past N / c are stored as zeros; ldc is ignored.
 * prac_compressed_bytes gives the buffer size of either layout (0 on bad arguments). */
typedef enum { PRAC_C_ROWMAJOR = 0, PRAC_C_PACKED = 1 } prac_c_layout;
size_t prac_compressed_bytes(int64_t N, int c, prac_dtype dt, int c_layout, int64_t ldc);
/* Copy a packed C (bf16) into a row-major N x c bf16 matrix: a pure permutation. */
int prac_unpack_compressed(prac_ctx* ctx, const void* C_packed, int64_t N, int c, void* C,
                           int64_t ldc);

/* C (N x c, dtype of X, layout c_layout) = X (N x d, ldx >= d) * P (d x c).
 * P is the fp32 master (ldp >= c); P_lp its packed copy or NULL (then it is
 * packed into ctx scratch on every call).  fp32 X uses P directly and supports
 * the row-major layout only. */
int prac_compress(prac_ctx* ctx, const void* X, prac_dtype xdt, int64_t N, int64_t d,
                  int64_t ldx, const float* P, const void* P_lp, int64_t ldp, int c,
                  void* C, int64_t ldc, int c_layout);

/* The same C (equal to prac_compress's up to the order of the fp32 sums over d:
 * the two walk the k-tiles in different orders, so single elements may differ
 * in the last bit of the output type), plus the layer's forward output Y
 * (N x m, ldy >= m, dtype of X) in one pass over X.  W has X's dtype; w_layout 0: d x m row-major (Y = X W,
 * Lemma 1), 1: m x d row-major (Y = X W^T, the layout of Section 5.2). */
int prac_compress_fused_fwd(prac_ctx* ctx, const void* X, prac_dtype xdt, int64_t N,
                            int64_t d, int64_t ldx, const void* W, int64_t m, int64_t ldw,
                            int w_layout, const float* P, const void* P_lp, int64_t ldp,
                            int c, void* Y, int64_t ldy, void* C, int64_t ldc, int c_layout);

/* ---- weight gradient (Lemma 1; Alg. 2 backward) ------------------------- */
/* dW (d x m, lddw >= m, dtype odt) = beta * dW + X~^T dY with
 * X~ = C[:, :k] Q1^T + scale * C[:, k:] Q2^T, evaluated as
 * P * diag(1..1, scale..scale) * (C^T dY).
 * C (N x (k+r), layout c_layout) and dY (N x m, lddy) share dtype `dt`. */
int prac_weight_grad(prac_ctx* ctx, const void* C, const void* dY, prac_dtype dt, int64_t N,
                     int64_t m, int64_t ldc, int c_layout, int64_t lddy, const float* P,
                     const void* P_lp, int64_t d, int64_t ldp, int k, int r, float scale,
                     void* dW, prac_dtype odt, int64_t lddw, float beta);

/* For callers that cannot allocate device memory or wait for the device inside the call: code
 * under HIP graph capture, serving loops, harnesses that forbid hipMalloc.  The same weight
 * gradient as prac_weight_grad, same arguments, same kernels, same results bit for bit, with
 * every intermediate (the token-split partial sums of C^T dY, T in fragment order, the packed copies of
 * P and of a row-major C when they are not handed in) in a block of PRAC_STATIC_SCRATCH_BYTES that is
 * part of the library's code object: every GPU the library runs on holds its own copy until the
 * process ends.  The call never calls hipMalloc / hipFree or an allocating routine, never touches the
 * ctx scratch, and is not profiled (prac_profile_select is ignored for it).
 *   - PRAC_ETOOBIG when prac_workspace_bytes of the same call exceeds PRAC_STATIC_SCRATCH_BYTES
 *     (the headline shape N = 32768, d = m = 2048, k + r = 256 needs 34.6 MB); nothing is enqueued then.
 *   - All calls on one GPU share that GPU's block, which keeps the last call's contents: the
 *     kernels overwrite what they read, so nothing needs clearing between calls, but two calls that
 *     overlap in time on one GPU (two streams, two threads, two contexts) race.  Stream order on one
 *     stream is enough. */
#define PRAC_STATIC_SCRATCH_BYTES (48u << 20)
int prac_weight_grad_static(prac_ctx* ctx, const void* C, const void* dY, prac_dtype dt, int64_t N,
                            int64_t m, int64_t ldc, int c_layout, int64_t lddy, const float* P,
                            const void* P_lp, int64_t d, int64_t ldp, int k, int r, float scale,
                            void* dW, prac_dtype odt, int64_t lddw, float beta);

/* Several layers that read the same input share one compressed activation
 * (Section 5.1, "activation subspace sharing": the query / key / value or the
 * up / gate projections).  n_out (1..PRAC_MAX_SHARED) weight gradients
 * dW_h = beta * dW_h + X~^T dY_h from one C: the token-split partial sums of all
 * C^T dY_h are formed in one launch, so C is streamed once and the split can
 * be coarser than for one output alone.  dY, m, lddy, dW, lddw are [host] arrays
 * of n_out entries (dY[h], dW[h] device pointers; dW_h is d x m[h]); everything
 * else as in prac_weight_grad, which is this call with n_out = 1. */
int prac_weight_grad_shared(prac_ctx* ctx, const void* C, prac_dtype dt, int64_t N, int64_t ldc,
                            int c_layout, int n_out, const void* const* dY, const int64_t* m,
                            const int64_t* lddy, const float* P, const void* P_lp, int64_t d,
                            int64_t ldp, int k, int r, float scale, void* const* dW,
                            prac_dtype odt, const int64_t* lddw, float beta);

/* ---- reconstruction (Section 5.1 formula; Alg. 2 backward, first step) ------ */
/* Xh (N x d, ldxh >= d, dtype dt) = C[:, :k] Q1^T + scale * C[:, k:] Q2^T: the
 * unbiased estimate of the saved activation, for layers whose backward needs
 * the activation itself (normalisation and activation-function inputs,
 * Section 5.1 / Appendix B) rather than only X^T dY.
 * C (N x (k+r), layout c_layout, dtype dt); P is the fp32 master (d x (k+r),
 * ldp).  bf16 data runs on the matrix cores with a bf16 copy of P whose random
 * columns already carry `scale` (built in ctx scratch on every call); fp32
 * data is evaluated in fp32. */
int prac_reconstruct(prac_ctx* ctx, const void* C, prac_dtype dt, int64_t N, int64_t ldc,
                     int c_layout, const float* P, int64_t d, int64_t ldp, int k, int r,
                     float scale, void* Xh, int64_t ldxh);

#ifdef __cplusplus
}
#endif
#endif /* PRAC_H */
