// Basis fit: P = [Q1 | Q2] (Section 4.3 construction; Alg. 1, both refresh branches).
//
// Q1: the paper takes the top-r_1 right singular vectors of X "via SVD".  They are
// the dominant eigenvectors of G = X^T X, found here by block power iteration
// V <- orth(G V) on a block of b = k + oversample columns, followed by a
// Rayleigh-Ritz step (eigenvectors of the small matrix V^T G V, by one-sided Jacobi).
// Q2: S is drawn from the counter-based Gaussian generator, projected twice onto the
// complement of Q1 and orthonormalised.  orth() is Cholesky-QR with an fp64 Gram
// matrix, which yields the thin-QR factor with a positive-diagonal R, i.e. the
// same Q2 that Householder QR with sign normalisation gives.
#include <algorithm>

#include "prac_internal.h"

namespace {

// ---------------------------------------------------------------- Cholesky (upper)
// value of x in lane U of each row of 16 lanes
template <int U>
__device__ __forceinline__ double row_share64(double x) {
  const uint64_t b = (uint64_t)__double_as_longlong(x);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)b, 0x150 + U, 0xf, 0xf, false);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)(b >> 32), 0x150 + U, 0xf, 0xf, false);
  return __longlong_as_double((long long)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo));
}

template <int N, typename F>
__device__ __forceinline__ void chol_static_for(F&& f) {
  if constexpr (N > 0) {
    chol_static_for<N - 1>(f);
    f(std::integral_constant<int, N - 1>{});
  }
}

// In place on the row-major b x b fp64 matrix W (b <= 1024; the upper triangle is read, rows of R
// are written to it): W = R^T R.  `shift_rel` * max diag(W) is added to the diagonal first.
// Non-finite or non-positive pivots raise *flag and are replaced by a tiny positive number.
// One workgroup of 1024 threads.  Per panel of 16 rows: the rows go to LDS (columns padded to a
// multiple of 16 with the identity); one wave factors the 16 x 16 diagonal block in registers (a
// column per lane, pivots and multipliers broadcast with DPP, 1 / sqrt(pivot) by two Newton steps
// from v_rsq_f64); every thread then solves one column of the rest of the panel against that block;
// the finished rows go back to memory and the trailing matrix takes its rank-16 update as 16 x 16
// tiles on v_mfma_f64_16x16x4_f64, dealt to the 16 waves four at a time so that their loads overlap.
// 67 / 177 us at b = 128 / 256 (107 / 355 us for the vector-ALU version this replaces); per panel
// 2.8 us for the diagonal block, 2.3 us for the solve, 0.5 - 13 us for the update.
typedef double f64x4_t __attribute__((ext_vector_type(4)));
constexpr int CH_NB = 16;  // panel height = block size of the fp64 matrix instruction
constexpr int CH_TB = 4;   // trailing tiles a wave has in flight
constexpr int CH_MAX = 1024;
__global__ __launch_bounds__(1024) void chol_upper_kernel(double* W, int b, double shift_rel, int* flag) {
  extern __shared__ __align__(16) unsigned char chol_smem[];
  const int bpad = (b + CH_NB - 1) / CH_NB * CH_NB, ldp = bpad + 2;
  double* panel = reinterpret_cast<double*>(chol_smem);  // [CH_NB][ldp]
  __shared__ double s_red[16];
  __shared__ double s_dinv[CH_NB];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  double mx = 0.0;
  for (int i = tid; i < b; i += 1024) mx = fmax(mx, W[(int64_t)i * b + i]);
  for (int o = 32; o > 0; o >>= 1) mx = fmax(mx, __shfl_xor(mx, o));
  if (lane == 0) s_red[wave] = mx;
  __syncthreads();
  mx = 0.0;
  for (int w = 0; w < 16; ++w) mx = fmax(mx, s_red[w]);
  const double shift = shift_rel * mx;
  const double tiny = 1e-300 + 1e-30 * mx;
  const int fi = lane & 15, fk = lane >> 4;

  for (int j0 = 0; j0 < bpad; j0 += CH_NB) {
    const int wpad = bpad - j0;  // panel width, padded columns included
    // panel rows j0 .. j0+15, columns j0 .. bpad-1 (relative index c)
    for (int u = wave; u < CH_NB; u += 16)
      for (int c = lane; c < wpad; c += 64) {
        const bool real = j0 + u < b && j0 + c < b;
        double v = real ? (c >= u ? W[(int64_t)(j0 + u) * b + j0 + c] : 0.0) : (c == u ? 1.0 : 0.0);
        if (real && c == u) v += shift;
        panel[u * ldp + c] = v;
      }
    __syncthreads();
    // diagonal block: col[u] of lane c is element (u, c); the four rows of 16 lanes work alike
    if (wave == 0) {
      double col[CH_NB], dinv[CH_NB];
#pragma unroll
      for (int u = 0; u < CH_NB; ++u) col[u] = panel[u * ldp + fi];
      bool bad = false;
      chol_static_for<CH_NB>([&](auto tc) {
        constexpr int T = decltype(tc)::value;
        double p = row_share64<T>(col[T]);
        if (!(p > tiny) || !isfinite(p)) {
          bad = true;
          p = tiny;
        }
        double rs = __builtin_amdgcn_rsq(p);
        rs = rs * (1.5 - 0.5 * p * rs * rs);
        rs = rs * (1.5 - 0.5 * p * rs * rs);
        dinv[T] = rs;
        col[T] = fi == T ? p * rs : (fi > T ? col[T] * rs : 0.0);  // row T of R; the pivot becomes sqrt(p)
        chol_static_for<CH_NB - 1 - T>([&](auto uc) {
          constexpr int U = T + 1 + decltype(uc)::value;
          col[U] -= row_share64<U>(col[T]) * col[T];
        });
      });
      if (lane < CH_NB) {
#pragma unroll
        for (int u = 0; u < CH_NB; ++u) panel[u * ldp + fi] = fi >= u ? col[u] : 0.0;
      }
      if (lane == 0) {
#pragma unroll
        for (int u = 0; u < CH_NB; ++u) s_dinv[u] = dinv[u];
        if (bad) atomicOr(flag, 1);
      }
    }
    __syncthreads();
    // the rest of the panel: column c solves R11^T x = a by forward substitution
    for (int c = CH_NB + tid; c < wpad; c += 1024) {
      double x[CH_NB];
#pragma unroll
      for (int u = 0; u < CH_NB; ++u) {
        double s = panel[u * ldp + c];
#pragma unroll
        for (int t = 0; t < u; ++t) s -= panel[t * ldp + u] * x[t];
        x[u] = s * s_dinv[u];
      }
#pragma unroll
      for (int u = 0; u < CH_NB; ++u) panel[u * ldp + c] = x[u];
    }
    __syncthreads();
    // finished rows of R
    for (int u = wave; u < CH_NB; u += 16)
      if (j0 + u < b)
        for (int c = u + lane; c < wpad; c += 64)
          if (j0 + c < b) W[(int64_t)(j0 + u) * b + j0 + c] = panel[u * ldp + c];
    // trailing update, tile (I, J), I <= J, of the 16 x 16 blocks behind the panel:
    // W[i][c] -= sum_t R[t][i] R[t][c].  Lane (fi, fk) holds A(m = fi, k = fk), B(k = fk, n = fi);
    // its register v is D(m = 4 v + fk, n = fi).
    const int nb = wpad / CH_NB - 1;
    const int ntiles = nb * (nb + 1) / 2;
    for (int q0 = wave * CH_TB; q0 < ntiles; q0 += 16 * CH_TB) {
      f64x4_t acc[CH_TB];
      int ti[CH_TB], tj[CH_TB];
#pragma unroll
      for (int e = 0; e < CH_TB; ++e) {
        // tile number q -> (I, J): block row I holds nb - I tiles
        int q = q0 + e, I = 0;
        const bool live = q < ntiles;
        if (!live) q = 0;
        while (q >= nb - I) {
          q -= nb - I;
          ++I;
        }
        ti[e] = live ? I : -1;
        tj[e] = I + q;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int row = j0 + CH_NB * (I + 1) + 4 * v + fk, colg = j0 + CH_NB * (tj[e] + 1) + fi;
          acc[e][v] = (live && row < b && colg < b) ? W[(int64_t)row * b + colg] : 0.0;
        }
      }
#pragma unroll
      for (int e = 0; e < CH_TB; ++e) {
        if (ti[e] < 0) continue;  // uniform
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const double a = -panel[(4 * s + fk) * ldp + CH_NB * (ti[e] + 1) + fi];
          const double bb = panel[(4 * s + fk) * ldp + CH_NB * (tj[e] + 1) + fi];
          acc[e] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, bb, acc[e], 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int row = j0 + CH_NB * (ti[e] + 1) + 4 * v + fk, colg = j0 + CH_NB * (tj[e] + 1) + fi;
          if (row < b && colg < b) W[(int64_t)row * b + colg] = acc[e][v];
        }
      }
    }
    __syncthreads();
  }
}

// dst (rows x n, fp32) = src * R^-1 for the upper-triangular R (row-major n x n fp64, upper part):
// forward substitution along the columns, 16 rows per workgroup held in LDS, 16 threads per row
// (a row never spans two waves).  R is staged through LDS 16 rows at a time as fp32, with the
// reciprocal of the diagonal, so that the substitution loop never waits for global memory.
constexpr int TR_ROWS = 16, TR_CH = 16;
__global__ __launch_bounds__(256) void trsm_right_upper_kernel(const float* __restrict__ src, const double* __restrict__ R,
                                                               float* __restrict__ dst, int64_t rows, int n) {
  extern __shared__ __align__(16) unsigned char trsm_smem[];
  float* y = reinterpret_cast<float*>(trsm_smem);  // [TR_ROWS][n]
  float* rch = y + TR_ROWS * n;                    // [TR_CH][n]: rows t0 .. t0+15 of R, diagonal inverted
  const int tid = threadIdx.x, r = tid >> 4, cl = tid & 15;
  const int64_t row = (int64_t)blockIdx.x * TR_ROWS + r;
  const bool ok = row < rows;
  for (int c = cl; c < n; c += 16) y[r * n + c] = ok ? src[row * n + c] : 0.f;
  for (int t0 = 0; t0 < n; t0 += TR_CH) {
    const int nt = min(TR_CH, n - t0);
    __syncthreads();  // previous chunk fully used (and y loaded)
    for (int e = tid; e < nt * n; e += 256) {
      const int u = e / n, c = e % n;
      const double v = c >= t0 + u ? R[(int64_t)(t0 + u) * n + c] : 0.0;
      rch[u * n + c] = c == t0 + u ? (float)(1.0 / v) : (float)v;
    }
    __syncthreads();
    for (int u = 0; u < nt; ++u) {
      const int t = t0 + u;
      const float vt = y[r * n + t] * rch[u * n + t];
      __builtin_amdgcn_wave_barrier();
      if (cl == 0) y[r * n + t] = vt;
      for (int c = t + 1 + cl; c < n; c += 16) y[r * n + c] -= vt * rch[u * n + c];
      __syncthreads();
    }
  }
  if (ok)
    for (int c = cl; c < n; c += 16) dst[row * n + c] = y[r * n + c];
}

// value of x in lane U of each row of 16 lanes
template <int U>
__device__ __forceinline__ float row_share(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x150 + U, 0xf, 0xf, false));
}

// steps U .. 15 of chunk JC (columns 16 JC .. 16 JC + 15) of the register-resident triangular solve
// (see the kernel below)
template <int U, int JC, int NPT>
__device__ __forceinline__ void trsm_steps(float (&y)[NPT], const float* __restrict__ rch, int nt, int cl) {
  if constexpr (U < 16) {
    if (U < nt) {  // uniform
      // no per-element conditions: the staged rows are zero past column n, so every read and
      // multiply-add below is unconditional and the reads of a step are issued together
      const float* ru = rch + U * (16 * NPT);
      const float vt = row_share<U>(y[JC]) * ru[16 * JC + U];
      const float upd = y[JC] - vt * ru[16 * JC + cl];
      y[JC] = cl == U ? vt : (cl > U ? upd : y[JC]);
#pragma unroll
      for (int j = JC + 1; j < NPT; ++j) y[j] -= vt * ru[cl + 16 * j];
      trsm_steps<U + 1, JC, NPT>(y, rch, nt, cl);
    }
  }
}

// row t0 + r of R, columns cl, cl + 16, ... into registers (thread (r, cl) of the workgroup)
template <int NPT>
__device__ __forceinline__ void trsm_fetch(double (&nx)[NPT], const double* __restrict__ R, int n, int t0, int r, int cl) {
#pragma unroll
  for (int j = 0; j < NPT; ++j) {
    const int c = cl + 16 * j, t = t0 + r;
    nx[j] = (t < n && c < n && c >= t) ? R[(int64_t)t * n + c] : 0.0;
  }
}

// ... and from there into LDS as fp32, the diagonal inverted
template <int NPT>
__device__ __forceinline__ void trsm_stage(const double (&nx)[NPT], float* rch, int n, int t0, int r, int cl) {
#pragma unroll
  for (int j = 0; j < NPT; ++j) {
    const int c = cl + 16 * j;
    double v = nx[j];  // zero below the diagonal and past row / column n
    if (c == t0 + r) v = c < n ? 1.0 / v : 0.0;
    rch[r * (16 * NPT) + c] = (float)v;
  }
}

// chunks JC .. NPT-1: the 16 steps of chunk JC run while the rows of R for chunk JC + 1 are in flight
template <int JC, int NPT>
__device__ __forceinline__ void trsm_chunks(float (&y)[NPT], double (&nx)[NPT], float* rch, const double* __restrict__ R,
                                            int n, int r, int cl) {
  if constexpr (JC < NPT) {
    constexpr int t0 = 16 * JC;
    if (t0 < n) {  // uniform
      const int nt = min(16, n - t0);
      __syncthreads();  // previous chunk fully used
      trsm_stage<NPT>(nx, rch, n, t0, r, cl);
      __syncthreads();
      if (t0 + 16 < n) trsm_fetch<NPT>(nx, R, n, t0 + 16, r, cl);
      trsm_steps<0, JC, NPT>(y, rch, nt, cl);
      trsm_chunks<JC + 1, NPT>(y, nx, rch, R, n, r, cl);
    }
  }
}

// dst (rows x n, fp32) = src * R^-1 as above for n <= 16 NPT, with the rows of y in registers: 16
// threads per row, thread cl holds columns cl, cl + 16, ...  Step t multiplies column t by
// 1 / R[t][t] (a DPP row share broadcasts it to the row's 16 lanes) and subtracts it, times row t of
// R, from the columns to its right.  No barrier and no LDS round trip per step.  Chunks and steps
// are unrolled, so every register index and every broadcast lane is a constant.  R is staged
// through LDS 16 rows at a time as fp32 with the diagonal inverted (two barriers per chunk), the
// next chunk's rows being fetched while the current chunk's steps run.
template <int NPT>
__global__ __launch_bounds__(256) void trsm_right_upper_reg_kernel(const float* __restrict__ src,
                                                                   const double* __restrict__ R, float* __restrict__ dst,
                                                                   int64_t rows, int n) {
  extern __shared__ __align__(16) unsigned char trsm_smem[];
  float* rch = reinterpret_cast<float*>(trsm_smem);  // [TR_CH][16 NPT]: rows t0 .. t0+15 of R, diagonal inverted, zero padded
  const int tid = threadIdx.x, r = tid >> 4, cl = tid & 15;
  const int64_t row = (int64_t)blockIdx.x * TR_ROWS + r;
  const bool ok = row < rows;
  float y[NPT];
#pragma unroll
  for (int j = 0; j < NPT; ++j) {
    const int c = cl + 16 * j;
    y[j] = (ok && c < n) ? src[row * n + c] : 0.f;
  }
  double nx[NPT];
  trsm_fetch<NPT>(nx, R, n, 0, r, cl);
  trsm_chunks<0, NPT>(y, nx, rch, R, n, r, cl);
  if (ok) {
#pragma unroll
    for (int j = 0; j < NPT; ++j) {
      const int c = cl + 16 * j;
      if (c < n) dst[row * n + c] = y[j];
    }
  }
}

// ------------------------------------------------------- symmetric eigen (Jacobi)
// One-sided (Hestenes) Jacobi on the columns of the symmetric PSD matrix H, held
// row-major so that "column" p is the contiguous row p (H is symmetric).  Rotating
// column pairs until all are mutually orthogonal gives H J = B with B's columns
// lambda_i v_i, so the eigenvectors are the normalised columns and the eigenvalues
// their norms.
//
// Block version: the b columns are cut into blocks of nbk; a round-robin tournament
// over the blocks pairs them up, and one workgroup per pair loads its 2 nbk columns
// into LDS, orthogonalises them there with an inner tournament (all data movement
// of the rotations stays in LDS) and writes them back.  One launch per tournament
// step; `counts[sweep]` collects the number of rotations of a sweep, and the launches
// of sweep s+1 return at once when sweep s rotated nothing.

// Sum over the 64 lanes of a wave, result in every lane: four data-parallel-primitive steps
// inside each row of 16 lanes (no LDS traffic), then the four row sums through scalar registers.
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double x) {
  int lo = __double2loint(x), hi = __double2hiint(x);
  lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, 0xF, 0xF, true);
  hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, 0xF, 0xF, true);
  return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double readlane_f64(double x, int l) {
  return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(x), l),
                          __builtin_amdgcn_readlane(__double2loint(x), l));
}
__device__ __forceinline__ double wave_sum_f64(double v) {
  v += dpp_f64<0xB1>(v);   // quad_perm [1,0,3,2]
  v += dpp_f64<0x4E>(v);   // quad_perm [2,3,0,1]
  v += dpp_f64<0x141>(v);  // row_half_mirror
  v += dpp_f64<0x140>(v);  // row_mirror
  return (readlane_f64(v, 0) + readlane_f64(v, 16)) + (readlane_f64(v, 32) + readlane_f64(v, 48));
}

__device__ __forceinline__ void tournament_pair(int step, int i, int players_even, int& p, int& q) {
  const int n1 = players_even - 1;
  if (i == 0) {
    p = step % n1;
    q = players_even - 1;
  } else {
    p = (step + i) % n1;
    q = (step - i + n1) % n1;
  }
}

// H <- (H + H^T) / 2; block 0 also leaves the largest diagonal entry in *hmax (the scale against
// which the eigen-iteration decides that a column is numerically zero)
__global__ __launch_bounds__(1024) void symmetrize64_kernel(double* H, int b, double* hmax) {
  if (blockIdx.x == 0) {
    __shared__ double s_mx[16];
    double mx = 0.0;
    for (int i = threadIdx.x; i < b; i += 1024) mx = fmax(mx, fabs(H[(int64_t)i * b + i]));
    for (int o = 32; o > 0; o >>= 1) mx = fmax(mx, __shfl_xor(mx, o));
    if ((threadIdx.x & 63) == 0) s_mx[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
      for (int w = 1; w < 16; ++w) mx = fmax(mx, s_mx[w]);
      *hmax = mx;
    }
  }
  for (int e = blockIdx.x * 1024 + threadIdx.x; e < b * b; e += gridDim.x * 1024) {
    const int i = e / b, j = e % b;
    if (i < j) {
      const double m = 0.5 * (H[(int64_t)i * b + j] + H[(int64_t)j * b + i]);
      H[(int64_t)i * b + j] = m;
      H[(int64_t)j * b + i] = m;
    }
  }
}

__global__ __launch_bounds__(1024) void jacobi_block_kernel(double* H, int b, int nbk, int nblk_even, int step, int sweep,
                                                            int inner_sweeps, double tol, unsigned* counts,
                                                            const double* hmax) {
  extern __shared__ __align__(16) unsigned char jac_smem[];
  double* cols = reinterpret_cast<double*>(jac_smem);  // [2 nbk][b]
  __shared__ int s_rows[64];
  __shared__ double s_n2[64];
  __shared__ int s_rot;
  if (sweep > 0 && counts[sweep - 1] == 0) return;  // converged in the previous sweep
  const double floor2 = 1e-26 * *hmax * *hmax;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int bp, bq;
  tournament_pair(step, blockIdx.x, nblk_even, bp, bq);
  // global column indices of the local columns (blocks past the end are byes)
  int m = 0;
  if (tid == 0) {
    for (int blk = 0; blk < 2; ++blk) {
      const int base = (blk == 0 ? bp : bq) * nbk;
      for (int u = 0; u < nbk; ++u)
        if (base + u < b) s_rows[m++] = base + u;
    }
    s_rows[63] = m;  // nbk <= 31 columns per block keeps slot 63 free; see the host code
    s_rot = 0;
  }
  __syncthreads();
  m = s_rows[63];
  if (m < 2) return;
  for (int e = tid; e < m * b; e += 1024) cols[e] = H[(int64_t)s_rows[e / b] * b + e % b];
  __syncthreads();
  // squared norms of the local columns, kept up to date through the rotations (a rotation by
  // tan = tt moves tt * <p, q> from one squared norm to the other), so that a pair step needs
  // one inner product instead of three
  for (int p = wave; p < m; p += 16) {
    const double* hp = cols + p * b;
    double al = 0.0;
    for (int t = lane; t < b; t += 64) al += hp[t] * hp[t];
    al = wave_sum_f64(al);
    if (lane == 0) s_n2[p] = al;
  }
  __syncthreads();
  const int me = m + (m & 1);
  int rotated = 0;
  for (int isw = 0; isw < inner_sweeps; ++isw) {
    for (int s = 0; s < me - 1; ++s) {
      for (int i = wave; i < me / 2; i += 16) {
        int p, q;
        tournament_pair(s, i, me, p, q);
        if (p >= m || q >= m) continue;
        double* hp = cols + p * b;
        double* hq = cols + q * b;
        double ga = 0.0;
        for (int t = lane; t < b; t += 64) ga += hp[t] * hq[t];
        ga = wave_sum_f64(ga);
        const double al = s_n2[p], be2 = s_n2[q];
        // rotate when |ga| > tol sqrt(al be2), compared as squares.  A rotation that involves a
        // numerically zero column (an eigenvalue below 1e-13 of the largest: rank-deficient input)
        // is applied but does not count towards convergence: such a column is rounding noise and
        // its cosines never settle.
        if (ga * ga > tol * tol * al * be2 && fabs(ga) > 1e-300) {
          if (fmin(al, be2) > floor2) rotated = 1;
          // The angle may be approximate (the iteration corrects it), so tan comes from the
          // hardware reciprocal / square root estimates; (cs, sn) must be a rotation to full
          // precision, so cs = (1 + tt^2)^-1/2 gets Newton steps on top of its estimate.
          const double zeta = (be2 - al) * 0.5 * __builtin_amdgcn_rcp(ga);
          const double az = fabs(zeta);
          const double tt = copysign(__builtin_amdgcn_rcp(az + __builtin_amdgcn_sqrt(1.0 + az * az)), zeta);
          const double w = 1.0 + tt * tt;
          double cs = __builtin_amdgcn_rsq(w);
          cs = cs * (1.5 - 0.5 * w * cs * cs);
          cs = cs * (1.5 - 0.5 * w * cs * cs);
          const double sn = cs * tt;
          for (int t = lane; t < b; t += 64) {
            const double x = hp[t], y = hq[t];
            hp[t] = cs * x - sn * y;
            hq[t] = sn * x + cs * y;
          }
          if (lane == 0) {
            // exact for the rotation actually applied: |p'|^2 = cs^2 al - 2 cs sn ga + sn^2 be2
            s_n2[p] = cs * cs * al - 2.0 * cs * sn * ga + sn * sn * be2;
            s_n2[q] = sn * sn * al + 2.0 * cs * sn * ga + cs * cs * be2;
          }
        }
      }
      __syncthreads();
    }
  }
  if (rotated && lane == 0) atomicOr(&s_rot, 1);
  __syncthreads();
  if (s_rot) {
    for (int e = tid; e < m * b; e += 1024) H[(int64_t)s_rows[e / b] * b + e % b] = cols[e];
    if (tid == 0) atomicAdd(&counts[sweep], 1u);
  }
}

// eigenvalues = column norms; normalise the columns in place; raise flag bit 2 if the last
// sweep still rotated
__global__ __launch_bounds__(1024) void jacobi_finish_kernel(double* H, int b, double* lambda, const unsigned* counts,
                                                             int last_sweep, int* flag) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (blockIdx.x == 0 && tid == 0 && counts[last_sweep] != 0) atomicOr(flag, 2);
  for (int p = blockIdx.x * 16 + wave; p < b; p += gridDim.x * 16) {
    double* hp = H + (int64_t)p * b;
    double al = 0.0;
    for (int t = lane; t < b; t += 64) al += hp[t] * hp[t];
    for (int o = 32; o > 0; o >>= 1) al += __shfl_xor(al, o);
    const double nrm = sqrt(al);
    const double inv = nrm > 0.0 ? 1.0 / nrm : 0.0;
    for (int t = lane; t < b; t += 64) hp[t] *= inv;
    if (lane == 0) lambda[p] = nrm;
  }
}

__global__ void zero_u32_kernel(unsigned* p, int n) {
  for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = 0u;
}

// Z (b x k fp32, row-major) = the k eigenvectors with the largest eigenvalues, in
// descending order; eigenvector p is row p of Hn (normalised Jacobi output).
__global__ __launch_bounds__(1024) void select_top_kernel(const double* __restrict__ Hn, const double* __restrict__ lambda,
                                                          int b, int k, float* Z) {
  __shared__ int s_rank[1024];
  const int tid = threadIdx.x;
  if (tid < b) {
    const double me = lambda[tid];
    int rk = 0;
    for (int o = 0; o < b; ++o) {
      const double v = lambda[o];
      rk += (v > me) || (v == me && o < tid);
    }
    s_rank[tid] = rk;
  }
  __syncthreads();
  for (int p = 0; p < b; ++p) {
    const int rk = s_rank[p];
    if (rk < k)
      for (int t = tid; t < b; t += 1024) Z[(int64_t)t * k + rk] = (float)Hn[(int64_t)p * b + t];
  }
}

__global__ __launch_bounds__(256) void copy_cols_kernel(const float* __restrict__ src, int64_t lds, float* dst,
                                                        int64_t ldd, int64_t rows, int cols) {
  const int64_t total = rows * cols;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x)
    dst[(i / cols) * ldd + i % cols] = src[(i / cols) * lds + i % cols];
}

struct FitWs {
  size_t G, V, Y, W64, X64, Rinv, lam, Z, S, T, slabs, slab_bytes, gram, total;
  size_t trk_pf, trk_c, trk_slabs;  // tracking refit: V in fragment order, packed X V, slabs of (X V)^T X
  int trk_nkb, trk_ncb, trk_splits;
  int b;
  int kq;         // principal columns the iteration computes (see principal_rank); the other k - kq are drawn
  int splits_bb;  // split count of the b x b fp64 Gram products
  int splits_gv;  // split count of G V
};

int block_width(int64_t d, int k, const prac_fit_opts& o) {
  int p = o.oversample < 0 ? 0 : (o.oversample == 0 ? k : o.oversample);
  int64_t b = (int64_t)k + p;
  if (b > d) b = d;
  if (b > 1024) b = 1024;
  if (b < k) b = k;
  return (int)b;
}

// Tracking refit (warm start, block width k, bf16 X the streaming kernels accept): no Gram
// matrix is formed.  One step is V <- orth(X^T (X V)): the compress kernel forms X V, the C^T dY
// kernel with X in the place of dY forms (X V)^T X.
bool can_track(const void* X, prac_dtype xdt, int64_t rows, int64_t d, int64_t ldx, int k, const prac_fit_opts& o) {
  // ldx itself a multiple of 8 (not only the pitch ldx * row_stride of the sampled rows): the streaming kernels
  // read a row in whole 16-byte chunks, and the last chunk of the last row must lie inside that row's ldx elements
  return o.warm_start && o.oversample < 0 && o.iters >= 1 && k > 0 && k <= 1024 && xdt == PRAC_BF16 &&
         (reinterpret_cast<uintptr_t>(X) & 15) == 0 && ldx % 8 == 0 &&
         ldx * (o.row_stride > 0 ? o.row_stride : 1) <= PRAC_MAX_STREAM_PITCH && rows >= 256 && rows >= k &&
         rows < ((int64_t)1 << 31) && d >= 128;
}

// Principal directions the (sub)sampled rows can define: a batch of fewer rows than k has rank below k, and
// the columns of Q1 past that rank are an arbitrary orthonormal completion (any one is a valid set of "top-k right
// singular vectors").  They are drawn like Q2 - Gaussian, projected onto the complement, orthonormalised -
// instead of being left to the iteration, whose blocks would be rank deficient.
int principal_rank(int k, int64_t rows) { return rows < k ? (int)rows : k; }

FitWs plan_fit(int64_t d, int k, int r, const prac_fit_opts& o, int n_cu, bool need_g, size_t gram_bytes, bool track,
               int64_t rows) {
  FitWs w{};
  WsPlan p;
  const int kq = (need_g || track) ? principal_rank(k, rows) : k;
  const int fill = k - kq;  // columns of Q1 drawn at random
  int b = track ? k : (need_g ? block_width(d, kq, o) : 0);
  if (need_g && b > rows) b = (int)rows;  // kq <= rows: the block keeps at least kq columns
  const int rf = r > fill ? r : fill;     // widest random block
  const int bb = b > rf ? b : rf;         // widest panel that goes through orth()
  w.b = b;
  w.kq = kq;
  w.G = p.take(need_g ? (size_t)d * d * 4 : 0);
  w.V = p.take((size_t)d * bb * 4);
  w.Y = p.take((size_t)d * bb * 4);
  w.W64 = p.take((size_t)bb * bb * 8);
  w.X64 = p.take((size_t)bb * bb * 8);
  w.Rinv = p.take((size_t)bb * bb * 4);
  w.lam = p.take((size_t)bb * 8);
  w.Z = p.take((size_t)bb * (k > 0 ? k : 1) * 4);
  w.S = p.take((size_t)d * (rf > 0 ? rf : 1) * 4);
  w.T = p.take((size_t)(k > 0 ? k : 1) * (rf > 0 ? rf : 1) * 4);
  const int tiles = ((bb + 63) / 64) * ((bb + 63) / 64);
  int s = (2 * n_cu + tiles - 1) / tiles;
  if (s > d / 64) s = (int)(d / 64);
  if (s < 1) s = 1;
  if (s > 64) s = 64;
  w.splits_bb = s;
  // G V (d x b, fp32): split the sum over k until the tiles fill the chip
  const int tiles_gv = (int)((d + 63) / 64) * ((b + 63) / 64);
  int sg = need_g ? (n_cu + tiles_gv - 1) / tiles_gv : 1;
  if (sg > d / 256) sg = (int)(d / 256);
  if (sg < 1) sg = 1;
  if (sg > 16) sg = 16;
  w.splits_gv = sg;
  // the slab block serves every split product of the fit: the bb x bb panel Gram matrices (fp64), G V
  // (d x b, fp32) and Q1^T S (k x r, fp32; wider than a panel Gram when k > 2 r and Q1 is not refreshed)
  const size_t slab_bb = (size_t)s * bb * bb * 8, slab_gv = sg > 1 ? (size_t)sg * d * b * 4 : 0;
  const size_t slab_kr = (size_t)s * k * rf * 4;  // also the completion's Q1^T S (kq x fill)
  w.slab_bytes = std::max(slab_bb, std::max(slab_gv, slab_kr));
  w.slabs = p.take(w.slab_bytes);
  w.gram = p.take(gram_bytes);
  if (track) {
    w.trk_nkb = (int)(round_up64(d, 256) / 16);
    w.trk_ncb = (int)round_up64((k + 31) / 32, 8);
    const int tiles = (int)((d + 127) / 128) * ((k + 255) / 256);  // 256 x 128 tiles of (X Q1)^T X
    int sp = n_cu / tiles;
    if (sp > rows / 256) sp = (int)(rows / 256);
    if (sp < 1) sp = 1;
    if (sp > 64) sp = 64;
    w.trk_splits = sp;
    w.trk_pf = p.take((size_t)w.trk_nkb * w.trk_ncb * 64 * 8 * sizeof(bf16_t));
    w.trk_c = p.take((size_t)((rows + 127) / 128) * 8 * ((k + 31) / 32) * 64 * 8 * sizeof(bf16_t));
    w.trk_slabs = p.take((size_t)sp * k * d * sizeof(float));
  }
  w.total = p.off;
  return w;
}

// the two panel kernels keep up to 128 KB / 64 KB in LDS (n <= 1024)
int set_dyn_smem(prac_ctx* ctx) {
  static bool done_dev[PRAC_MAX_DEVICES] = {};  // the attribute is per device
  bool& done = done_dev[ctx->device % PRAC_MAX_DEVICES];
  if (!done) {
    PRAC_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(chol_upper_kernel),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, CH_NB * (CH_MAX + 2) * 8));
    PRAC_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(trsm_right_upper_kernel),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (TR_ROWS + TR_CH) * 1024 * 4));
    done = true;
  }
  return PRAC_OK;
}

__global__ __launch_bounds__(256) void f32_to_f64_kernel(const float* __restrict__ src, double* __restrict__ dst, int n) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) dst[i] = (double)src[i];
}

// W (n x n) <- 1.5 I - 0.5 W.  W is the Gram matrix of a block that should be close to orthonormal: an entry
// further than `limit` from the identity (or not finite) raises bit 1 of *flag - the step that follows squares
// the distance, so a block that far off does not come out orthonormal to fp32 rounding.
__global__ __launch_bounds__(256) void newton_schulz_factor_kernel(float* W, int n, float limit, int* flag) {
  bool off = false;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n * n; i += gridDim.x * blockDim.x) {
    const float id = i / n == i % n ? 1.f : 0.f;
    off = off || !(fabsf(W[i] - id) <= limit);
    W[i] = 1.5f * id - 0.5f * W[i];
  }
  if (off) atomicOr(flag, 1);
}

// M (n x n) = src^T src for a d x n block (ld = n): fp64 sums into W64, or fp32 sums on the matrix
// cores into M32 (enough for a block whose condition number is small)
int panel_gram(prac_ctx* ctx, const FitWs& w, const float* src, int64_t d, int n, double* W64, float* M32) {
  GemmGenArgs g{};
  g.A = src; g.B = src; g.adt = PRAC_F32; g.bdt = PRAC_F32;
  g.a_rs = 1; g.a_cs = n; g.b_rs = n; g.b_cs = 1;
  g.M = n; g.N = n; g.K = d; g.k_stride = 1;
  g.ldo = n; g.alpha = 1.f; g.beta = 0.f;
  g.splits = w.splits_bb; g.slabs = ctx->ws + w.slabs; g.slab_bytes = w.slab_bytes;
  if (W64) { g.out = nullptr; g.out64 = W64; g.acc64 = true; }
  else { g.out = M32; g.out64 = nullptr; g.acc64 = false; }
  return launch_gemm_generic(ctx, g);
}

// dst = src R^-1 with R^T R = src^T src (+ shift): one Cholesky-QR pass
int cholqr_pass(prac_ctx* ctx, const FitWs& w, const float* src, float* dst, int64_t d, int n, double shift, bool gram64) {
  double* W64 = reinterpret_cast<double*>(ctx->ws + w.W64);
  int rc;
  if (gram64) {
    rc = panel_gram(ctx, w, src, d, n, W64, nullptr);
    if (rc) return rc;
  } else {
    float* M32 = reinterpret_cast<float*>(ctx->ws + w.Rinv);
    rc = panel_gram(ctx, w, src, d, n, nullptr, M32);
    if (rc) return rc;
    hipLaunchKernelGGL(f32_to_f64_kernel, dim3((n * n + 255) / 256), dim3(256), 0, ctx->stream, M32, W64, n * n);
  }
  rc = set_dyn_smem(ctx);
  if (rc) return rc;
  if (n > CH_MAX) return PRAC_EUNSUPPORTED;
  hipLaunchKernelGGL(chol_upper_kernel, dim3(1), dim3(1024),
                     (size_t)CH_NB * (round_up64(n, CH_NB) + 2) * sizeof(double), ctx->stream, W64, n, shift, ctx->d_flag);
  const dim3 tgrid((unsigned)((d + TR_ROWS - 1) / TR_ROWS));
  if (n <= 128)
    hipLaunchKernelGGL(trsm_right_upper_reg_kernel<8>, tgrid, dim3(256), (size_t)TR_CH * 128 * sizeof(float), ctx->stream,
                       src, W64, dst, d, n);
  else if (n <= 256)
    hipLaunchKernelGGL(trsm_right_upper_reg_kernel<16>, tgrid, dim3(256), (size_t)TR_CH * 256 * sizeof(float), ctx->stream,
                       src, W64, dst, d, n);
  else if (n <= 512)
    hipLaunchKernelGGL(trsm_right_upper_reg_kernel<32>, tgrid, dim3(256), (size_t)TR_CH * 512 * sizeof(float), ctx->stream,
                       src, W64, dst, d, n);
  else
    hipLaunchKernelGGL(trsm_right_upper_kernel, tgrid, dim3(256), (size_t)(TR_ROWS + TR_CH) * n * sizeof(float),
                       ctx->stream, src, W64, dst, d, n);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

// dst = src (1.5 I - 0.5 src^T src): one Newton-Schulz step towards orthonormal columns.  For a block
// with ||src^T src - I|| = e the result has 0.75 e^2: the cheap second pass after a Cholesky-QR pass,
// made of two products and no factorisation.
int polish_pass(prac_ctx* ctx, const FitWs& w, const float* src, float* dst, int64_t d, int n, float limit) {
  float* M32 = reinterpret_cast<float*>(ctx->ws + w.Rinv);
  int rc = panel_gram(ctx, w, src, d, n, nullptr, M32);
  if (rc) return rc;
  hipLaunchKernelGGL(newton_schulz_factor_kernel, dim3((n * n + 255) / 256), dim3(256), 0, ctx->stream, M32, n, limit,
                     ctx->d_flag);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  GemmGenArgs g{};
  g.A = src; g.B = M32; g.adt = PRAC_F32; g.bdt = PRAC_F32;
  g.a_rs = n; g.a_cs = 1; g.b_rs = n; g.b_cs = 1;
  g.M = (int)d; g.N = n; g.K = n; g.k_stride = 1;
  g.out = dst; g.ldo = n; g.alpha = 1.f; g.beta = 0.f; g.acc64 = false; g.out64 = nullptr;
  return launch_gemm_generic(ctx, g);
}

// V (d x n, ld = n, fp32) <- orth(Y): `passes` rounds of Cholesky-QR (the first one shifted), then
// `polish` Newton-Schulz steps; ping-pongs between Y and V, result always ends in `V`.
// gram64_first = false: the first Gram matrix is summed in fp32 (well-conditioned blocks only).
int cholqr(prac_ctx* ctx, const FitWs& w, float* Y, float* V, int64_t d, int n, int passes, double first_shift,
           int polish = 0, bool gram64_first = true) {
  float* src = Y;
  float* dst = V;
  for (int pass = 0; pass < passes + polish; ++pass) {
    // Later passes work on a block that is orthonormal up to the first pass's error, except in
    // directions where the input was rank deficient: there the Gram matrix is zero up to rounding
    // (a few 1e-16), and the shift has to be safely above that for the pivot to stay positive.
    // the last Newton-Schulz step must start within 3e-3 of orthonormal to end below 1e-5 (0.75 e^2); earlier
    // ones may start anywhere inside the step's region of convergence
    int rc = pass < passes ? cholqr_pass(ctx, w, src, dst, d, n, pass == 0 ? first_shift : 1e-13, pass > 0 || gram64_first)
                           : polish_pass(ctx, w, src, dst, d, n, pass == passes + polish - 1 ? 3e-3f : 0.5f);
    if (rc) return rc;
    float* t = src; src = dst; dst = t;
  }
  // result is in `src` after the swap
  if (src != V) {
    hipLaunchKernelGGL(copy_cols_kernel, dim3(ctx->n_cu * 4), dim3(256), 0, ctx->stream, src, (int64_t)n, V,
                       (int64_t)n, d, n);
    PRAC_HIP_TRY(ctx, hipGetLastError());
  }
  return PRAC_OK;
}



// The scratch plan of one fit: which path runs (tracking / Gram-based) and where everything lives.
struct FitPlan {
  bool do_q1, do_q2, track;
  int64_t rows;
  FitWs L;
};
FitPlan make_fit_plan(int n_cu, const void* X, prac_dtype xdt, int64_t N, int64_t d, int64_t ldx, int k, int r,
                      int refresh, const prac_fit_opts& o) {
  FitPlan f{};
  f.do_q1 = (refresh & PRAC_REFRESH_PRINCIPAL) && k > 0;
  f.do_q2 = (refresh & PRAC_REFRESH_RANDOM) && r > 0;
  const int64_t stride = o.row_stride > 0 ? o.row_stride : 1;
  f.rows = (N + stride - 1) / stride;
  if (!f.do_q1 && !f.do_q2) return f;  // nothing to refresh: no scratch
  f.track = f.do_q1 && can_track(X, xdt, f.rows, d, ldx, k, o);
  const size_t gram_bytes = f.do_q1 && !f.track ? gram_scratch_bytes(n_cu, X, xdt, N, d, ldx, stride, d) : 0;
  f.L = plan_fit(d, k, r, o, n_cu, f.do_q1 && !f.track, gram_bytes, f.track, f.rows);
  return f;
}

}  // namespace

size_t fit_scratch_bytes(int n_cu, const void* X, prac_dtype xdt, int64_t N, int64_t d, int64_t ldx, int k, int r,
                         int refresh, const prac_fit_opts& o) {
  const FitPlan f = make_fit_plan(n_cu, X, xdt, N, d, ldx, k, r, refresh, o);
  return (f.do_q1 || f.do_q2) ? f.L.total : 0;
}

// Bytes by which the slab block of the plan exceeds the largest split product of the fit (negative:
// a product would not fit).  The products are listed here as fit_basis_device issues them.
int64_t fit_slab_margin(int n_cu, prac_dtype xdt, int64_t N, int64_t d, int k, int r, int refresh,
                        const prac_fit_opts& o) {
  const FitPlan f = make_fit_plan(n_cu, nullptr, xdt, N, d, d, k, r, refresh, o);
  const FitWs& L = f.L;
  if (!f.do_q1 && !f.do_q2) return 0;
  size_t need = 0;
  auto product = [&](int splits, int64_t M, int64_t Nn, size_t esz) {
    if (splits > 1) need = std::max(need, (size_t)splits * M * Nn * esz);
  };
  if (f.do_q1) {
    const int n = L.b;  // block width of the iteration (k when tracking)
    product(L.splits_bb, n, n, 8);                    // panel Gram matrices of orth(), Rayleigh-Ritz
    if (!f.track) product(L.splits_gv, d, n, 4);      // G V
    product(L.splits_bb, L.kq, L.kq, 8);              // tidy passes on Q1
    const int fill = k - L.kq;
    if (fill > 0) {
      product(L.splits_bb, L.kq, fill, 4);            // the completion's Q1^T S
      product(L.splits_bb, fill, fill, 8);            // and its panel Gram matrices
    }
  }
  if (f.do_q2) {
    if (k > 0) product(L.splits_bb, k, r, 4);         // Q1^T S
    product(L.splits_bb, r, r, 8);                    // panel Gram matrices of orth(S_o)
  }
  return (int64_t)L.slab_bytes - (int64_t)need;
}

int fit_basis_device(prac_ctx* ctx, const void* X, prac_dtype xdt, int64_t N, int64_t d, int64_t ldx, int k, int r,
                     uint64_t seed, uint32_t draw, int refresh, const prac_fit_opts& o, float* P, int64_t ldp) {
  const FitPlan plan = make_fit_plan(ctx->n_cu, X, xdt, N, d, ldx, k, r, refresh, o);
  const bool do_q1 = plan.do_q1, do_q2 = plan.do_q2, track = plan.track;
  if (!do_q1 && !do_q2) return PRAC_OK;
  if (k > 1024 || r > 1024) return PRAC_EUNSUPPORTED;  // single-workgroup panel kernels
  const int64_t stride = o.row_stride > 0 ? o.row_stride : 1;
  const int64_t rows = plan.rows;
  const FitWs& L = plan.L;
  int rc = prac_ws_reserve(ctx, L.total);
  if (rc) return rc;
  float* G = reinterpret_cast<float*>(ctx->ws + L.G);
  float* V = reinterpret_cast<float*>(ctx->ws + L.V);
  float* Y = reinterpret_cast<float*>(ctx->ws + L.Y);
  hipStream_t st = ctx->stream;

  if (track) {
    // V starts as the previous Q1.  The span is what matters (compression and the estimator are
    // invariant to a rotation inside Q1), so there is no Rayleigh-Ritz step: each iteration is one
    // subspace-iteration step on X^T X, orthonormalised by Cholesky-QR (two passes on the last).
    const bf16_t* Xb = reinterpret_cast<const bf16_t*>(X);
    const int64_t ld = ldx * stride;
    bf16_t* Pf = reinterpret_cast<bf16_t*>(ctx->ws + L.trk_pf);
    bf16_t* Cpk = reinterpret_cast<bf16_t*>(ctx->ws + L.trk_c);
    float* slabs = reinterpret_cast<float*>(ctx->ws + L.trk_slabs);
    const int dm = (int)d;
    for (int it = 0; it < o.iters; ++it) {
      rc = launch_pack_pfrag(ctx, it == 0 ? P : V, d, it == 0 ? ldp : (int64_t)k, k, L.trk_nkb, L.trk_ncb, Pf);
      if (rc) return rc;
      rc = launch_compress_ws(ctx, Xb, ld, (int)rows, dm, Pf, L.trk_ncb, k, Cpk, 0, true, nullptr, 0, 0, nullptr, 0);
      if (rc) return rc;
      rc = launch_ctdy_ws(ctx, Cpk, k, (int)rows, 1, &Xb, &ld, &dm, &slabs, L.trk_splits);
      if (rc) return rc;
      rc = launch_reduce_transpose_f32(ctx, slabs, L.trk_splits, k, dm, Y, k);
      if (rc) return rc;
      // One power step from an orthonormal block leaves a condition number of at most lambda_1 /
      // lambda_k, within reach of a Cholesky factor of the fp64 Gram matrix with a shift just above its
      // rounding (so that a rank-deficient batch still factors); the last
      // iteration then gets two Newton-Schulz steps in place of a second factorisation.
      rc = cholqr(ctx, L, Y, V, d, k, 1, 1e-14, it == o.iters - 1 ? 2 : 0);
      if (rc) return rc;
    }
    hipLaunchKernelGGL(copy_cols_kernel, dim3(ctx->n_cu * 4), dim3(256), 0, st, V, (int64_t)k, P, ldp, d, k);
    PRAC_HIP_TRY(ctx, hipGetLastError());
  } else if (do_q1) {
    const int b = L.b;
    const int k = L.kq;  // the columns this iteration computes: all of Q1 unless the batch has fewer rows than that
    rc = gram_device(ctx, X, xdt, N, d, ldx, o.row_stride, G, d, ctx->ws + L.gram);
    if (rc) return rc;

    // start block: Gaussian (stream 0); warm start puts the previous Q1 in front
    rc = launch_philox(ctx, seed, draw, 0u, Y, d * b, true);
    if (rc) return rc;
    if (o.warm_start) {
      hipLaunchKernelGGL(copy_cols_kernel, dim3(ctx->n_cu * 4), dim3(256), 0, st, P, ldp, Y, (int64_t)b, d, k);
      PRAC_HIP_TRY(ctx, hipGetLastError());
    }
    // The start block goes into the first product as it is: a Gaussian block and the previous
    // (orthonormal) Q1 are both well conditioned, and every product is orthonormalised anyway.
    for (int it = 0; it <= o.iters; ++it) {
      // Y = G V  (first round: V is the start block, still in Y's buffer, so the roles swap)
      GemmGenArgs g{};
      g.A = G; g.B = it == 0 ? Y : V; g.adt = PRAC_F32; g.bdt = PRAC_F32;
      g.a_rs = 1; g.a_cs = d; g.b_rs = b; g.b_cs = 1;  // G(m, k) read as G[k][m]: G is symmetric
      g.M = (int)d; g.N = b; g.K = d; g.k_stride = 1;
      g.splits = L.splits_gv; g.slabs = ctx->ws + L.slabs; g.slab_bytes = L.slab_bytes;
      g.out = it == 0 ? V : Y; g.ldo = b; g.alpha = 1.f; g.beta = 0.f; g.acc64 = false; g.out64 = nullptr;
      rc = launch_gemm_generic(ctx, g);
      if (rc) return rc;
      if (it == 0) {
        // product landed in V: move it to Y so that orth() below reads Y and writes V as always
        hipLaunchKernelGGL(copy_cols_kernel, dim3(ctx->n_cu * 4), dim3(256), 0, st, V, (int64_t)b, Y, (int64_t)b, d, b);
        PRAC_HIP_TRY(ctx, hipGetLastError());
      }
      if (it == o.iters) break;  // the last product feeds Rayleigh-Ritz
      // one shifted pass keeps the block well conditioned; the last iteration orthonormalises fully
      // (two passes: the second starts from a block whose condition number is already near one)
      rc = cholqr(ctx, L, Y, V, d, b, it == o.iters - 1 ? 2 : 1, 1e-11);
      if (rc) return rc;
    }
    // Rayleigh-Ritz: H = V^T (G V), eigenvectors of H, Q1 = V Z[:, :k]
    double* H = reinterpret_cast<double*>(ctx->ws + L.W64);
    double* lam = reinterpret_cast<double*>(ctx->ws + L.lam);
    float* Z = reinterpret_cast<float*>(ctx->ws + L.Z);
    {
      GemmGenArgs g{};
      g.A = V; g.B = Y; g.adt = PRAC_F32; g.bdt = PRAC_F32;
      g.a_rs = 1; g.a_cs = b; g.b_rs = b; g.b_cs = 1;
      g.M = b; g.N = b; g.K = d; g.k_stride = 1;
      g.out = nullptr; g.out64 = H; g.ldo = b; g.alpha = 1.f; g.beta = 0.f; g.acc64 = true;
      g.splits = L.splits_bb; g.slabs = ctx->ws + L.slabs; g.slab_bytes = L.slab_bytes;
      rc = launch_gemm_generic(ctx, g);
      if (rc) return rc;
    }
    {
      // block Jacobi: 2 nbk columns of length b (fp64) per workgroup in LDS, at most 128 KB
      // 16 columns per block: an inner tournament step then has at most 16 pairs, one per wave
      int nbk = 8192 / b;
      if (nbk > 16) nbk = 16;
      if (nbk < 1) nbk = 1;
      const int nblk = (b + nbk - 1) / nbk, nblk_even = nblk + (nblk & 1);
      constexpr int MAX_SWEEPS = 12;
      // columns count as orthogonal below this cosine: the Ritz vectors are re-orthonormalised in
      // fp32 afterwards, so anything far below fp32 rounding is spent effort
      constexpr double JACOBI_TOL = 1e-10;
      unsigned* counts = reinterpret_cast<unsigned*>(ctx->ws + L.X64);
      static bool smem_dev[PRAC_MAX_DEVICES] = {};
      bool& smem_set = smem_dev[ctx->device % PRAC_MAX_DEVICES];
      if (!smem_set) {
        PRAC_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(jacobi_block_kernel),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024));
        smem_set = true;
      }
      hipLaunchKernelGGL(zero_u32_kernel, dim3(1), dim3(64), 0, st, counts, MAX_SWEEPS);
      double* hmax = reinterpret_cast<double*>(counts + 16);
      hipLaunchKernelGGL(symmetrize64_kernel, dim3(16), dim3(1024), 0, st, H, b, hmax);
      const size_t smem = (size_t)2 * nbk * b * sizeof(double);
      if (nblk == 1) {
        // a single block: one workgroup orthogonalises everything in LDS
        hipLaunchKernelGGL(jacobi_block_kernel, dim3(1), dim3(1024), smem, st, H, b, nbk, 2, 0, 0, 30, JACOBI_TOL, counts, hmax);
        hipLaunchKernelGGL(jacobi_finish_kernel, dim3(16), dim3(1024), 0, st, H, b, lam, counts, MAX_SWEEPS - 1,
                           ctx->d_flag);
      } else {
        for (int sweep = 0; sweep < MAX_SWEEPS; ++sweep)
          for (int step = 0; step < nblk_even - 1; ++step)
            hipLaunchKernelGGL(jacobi_block_kernel, dim3(nblk_even / 2), dim3(1024), smem, st, H, b, nbk, nblk_even,
                               step, sweep, 1, JACOBI_TOL, counts, hmax);
        hipLaunchKernelGGL(jacobi_finish_kernel, dim3(16), dim3(1024), 0, st, H, b, lam, counts, MAX_SWEEPS - 1,
                           ctx->d_flag);
      }
    }
    hipLaunchKernelGGL(select_top_kernel, dim3(1), dim3(1024), 0, st, H, lam, b, k, Z);
    PRAC_HIP_TRY(ctx, hipGetLastError());
    {
      GemmGenArgs g{};
      g.A = V; g.B = Z; g.adt = PRAC_F32; g.bdt = PRAC_F32;
      g.a_rs = b; g.a_cs = 1; g.b_rs = k; g.b_cs = 1;
      g.M = (int)d; g.N = k; g.K = b; g.k_stride = 1;
      g.out = Y; g.ldo = k; g.alpha = 1.f; g.beta = 0.f; g.acc64 = false; g.out64 = nullptr;
      rc = launch_gemm_generic(ctx, g);
      if (rc) return rc;
    }
    // tidy the rounding of the last product (two Cholesky-QR passes and a Newton-Schulz step: with more
    // Ritz vectors asked for than the data has rank, the surplus ones are rounding noise, far from
    // orthogonal to each other, and one pass leaves 1e-4 or more), then store Q1 into P[:, :k]
    rc = cholqr(ctx, L, Y, V, d, k, 2, 1e-13, 1);
    if (rc) return rc;
    hipLaunchKernelGGL(copy_cols_kernel, dim3(ctx->n_cu * 4), dim3(256), 0, st, V, (int64_t)k, P, ldp, d, k);
    PRAC_HIP_TRY(ctx, hipGetLastError());
  }

  // P[:, kk : kk + rr] = orth((I - Q Q^T)^2 S) for Q = P[:, :kk] and the Gaussian d x rr block S of Philox
  // stream `stream`
  auto random_block = [&](int k, int r, uint32_t stream) -> int {
    float* S = reinterpret_cast<float*>(ctx->ws + L.S);
    float* T = reinterpret_cast<float*>(ctx->ws + L.T);
    int rc = launch_philox(ctx, seed, draw, stream, S, d * r, true);
    if (rc) return rc;
    if (k > 0) {
      for (int rep = 0; rep < 2; ++rep) {
        // T = Q^T S  (k x r), S -= Q T
        GemmGenArgs g{};
        g.A = P; g.B = S; g.adt = PRAC_F32; g.bdt = PRAC_F32;
        g.a_rs = 1; g.a_cs = ldp; g.b_rs = r; g.b_cs = 1;
        g.M = k; g.N = r; g.K = d; g.k_stride = 1;
        // fp32 sums on the matrix cores: the second projection removes what rounding left of the first
        g.out = T; g.ldo = r; g.alpha = 1.f; g.beta = 0.f; g.acc64 = false; g.out64 = nullptr;
        g.splits = L.splits_bb; g.slabs = ctx->ws + L.slabs; g.slab_bytes = L.slab_bytes;
        rc = launch_gemm_generic(ctx, g);
        if (rc) return rc;
        GemmGenArgs h{};
        h.A = P; h.B = T; h.adt = PRAC_F32; h.bdt = PRAC_F32;
        h.a_rs = ldp; h.a_cs = 1; h.b_rs = r; h.b_cs = 1;
        h.M = (int)d; h.N = r; h.K = k; h.k_stride = 1;
        h.out = S; h.ldo = r; h.alpha = -1.f; h.beta = 1.f; h.acc64 = false; h.out64 = nullptr;
        rc = launch_gemm_generic(ctx, h);
        if (rc) return rc;
      }
    }
    // a narrow projected Gaussian block is well conditioned (singular values within 1 +- sqrt(r/d) of
    // each other): fp32 sums are enough for its Gram matrix, and one Newton-Schulz step finishes it
    // (up to r = d/4, where the ratio of the extreme singular values reaches 3; wider blocks keep two
    // Cholesky-QR passes over fp64 Gram matrices)
    if ((int64_t)4 * r <= d - k) rc = cholqr(ctx, L, S, V, d, r, 1, 1e-13, 1, false);
    else rc = cholqr(ctx, L, S, V, d, r, 2, 1e-13);
    if (rc) return rc;
    hipLaunchKernelGGL(copy_cols_kernel, dim3(ctx->n_cu * 4), dim3(256), 0, st, V, (int64_t)r, P + k, ldp, d, r);
    PRAC_HIP_TRY(ctx, hipGetLastError());
    return PRAC_OK;
  };
  // the columns of Q1 that the batch's rows do not define (stream 2), then Q2 (stream 1) against all of Q1
  if (do_q1 && L.kq < k) {
    rc = random_block(L.kq, k - L.kq, 2u);
    if (rc) return rc;
  }
  if (do_q2) return random_block(k, r, 1u);
  return PRAC_OK;
}
