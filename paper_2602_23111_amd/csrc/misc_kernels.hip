// Small streaming kernels: the counter-based Gaussian generator, basis packing,
// split-reduction epilogues and element-wise helpers.
#include "prac_internal.h"

namespace {

__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// ---- Philox4x32-10 (Salmon et al., SC'11) ------------------------------------------
// Stream layout: word i of (seed, draw, stream) is output i%4 of the block whose counter
// is (i/4 low, i/4 high, stream, draw) under key (seed low, seed high).
struct U4 { uint32_t x, y, z, w; };

__device__ __forceinline__ U4 philox4x32_10(U4 c, uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c.x), lo0 = 0xD2511F53u * c.x;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c.z), lo1 = 0xCD9E8D57u * c.z;
    U4 n;
    n.x = hi1 ^ c.y ^ k0;
    n.y = lo1;
    n.z = hi0 ^ c.w ^ k1;
    n.w = lo0;
    c = n;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return c;
}

__device__ __forceinline__ float word_to_uniform(uint32_t w) {
  // ((w >> 9) + 1/2) * 2^-23: an odd multiple of 2^-24, exact in fp32, inside (0, 1)
  return ((float)(w >> 9) + 0.5f) * 1.1920928955078125e-07f;
}

__device__ __forceinline__ void box_muller(uint32_t wa, uint32_t wb, float& z0, float& z1) {
  const float rad = sqrtf(-2.0f * logf(word_to_uniform(wa)));
  float s, c;
  sincospif(2.0f * word_to_uniform(wb), &s, &c);
  z0 = rad * c;
  z1 = rad * s;
}

template <bool NORMAL>
__global__ __launch_bounds__(256) void philox_kernel(uint32_t seed_lo, uint32_t seed_hi, uint32_t draw,
                                                     uint32_t stream, void* out, int64_t n) {
  const int64_t nblk = (n + 3) / 4;
  for (int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; b < nblk; b += (int64_t)gridDim.x * blockDim.x) {
    U4 c;
    c.x = (uint32_t)(b & 0xFFFFFFFFu);
    c.y = (uint32_t)((uint64_t)b >> 32);
    c.z = stream;
    c.w = draw;
    const U4 x = philox4x32_10(c, seed_lo, seed_hi);
    const int64_t base = 4 * b;
    if (NORMAL) {
      float z[4];
      box_muller(x.x, x.y, z[0], z[1]);
      box_muller(x.z, x.w, z[2], z[3]);
      float* o = reinterpret_cast<float*>(out);
      if (base + 4 <= n) {
        *reinterpret_cast<float4*>(o + base) = make_float4(z[0], z[1], z[2], z[3]);
      } else {
        for (int e = 0; e < 4; ++e)
          if (base + e < n) o[base + e] = z[e];
      }
    } else {
      uint32_t* o = reinterpret_cast<uint32_t*>(out);
      const uint32_t w[4] = {x.x, x.y, x.z, x.w};
      if (base + 4 <= n) {
        *reinterpret_cast<uint4*>(o + base) = make_uint4(w[0], w[1], w[2], w[3]);
      } else {
        for (int e = 0; e < 4; ++e)
          if (base + e < n) o[base + e] = w[e];
      }
    }
  }
}

// ---- basis packing ---------------------------------------------------------------
// Pt (c x ldpt) = bf16(P^T), Pn (d x ldpn) = bf16(P); padding columns are zero.
__global__ __launch_bounds__(256) void pack_basis_kernel(const float* __restrict__ P, int64_t d, int64_t ldp, int c,
                                                         bf16_t* __restrict__ Pt, int64_t ldpt,
                                                         bf16_t* __restrict__ Pn, int64_t ldpn) {
  __shared__ float tile[32][33];
  const int i0 = blockIdx.y * 32, j0 = blockIdx.x * 32;  // i: feature (row of P), j: basis column
  const int tx = threadIdx.x % 32, ty = threadIdx.x / 32;  // 32 x 8
  for (int r = ty; r < 32; r += 8) {
    const int64_t i = i0 + r;
    const int j = j0 + tx;
    const float v = (i < d && j < c) ? P[i * ldp + j] : 0.f;
    tile[r][tx] = v;
    if (i < d && j < ldpn) Pn[i * ldpn + j] = f32_to_bf16(v);
  }
  __syncthreads();
  for (int r = ty; r < 32; r += 8) {
    const int j = j0 + r;
    const int64_t i = i0 + tx;
    if (j < c && i < ldpt) Pt[(int64_t)j * ldpt + i] = f32_to_bf16(tile[tx][r]);
  }
}

// ---- split reductions ------------------------------------------------------------
__global__ __launch_bounds__(256) void reduce_slabs_kernel(const float* __restrict__ part, int splits, int64_t stride,
                                                           float* __restrict__ out, int64_t n, float alpha,
                                                           float beta) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
    float s = 0.f;
#pragma unroll 8
    for (int z = 0; z < splits; ++z) s += part[z * stride + i];  // eight slabs in flight
    s *= alpha;
    out[i] = beta == 0.f ? s : s + beta * out[i];
  }
}

// part: splits x M x N fp32.  out[n][j] = sum_z part[z][j][n] (N x M, ld = ldo).  One workgroup per
// 16 (j) x 64 (n) patch: a thread sums four consecutive n of one row j over the slabs (16-byte loads,
// 256-byte runs per row and slab, eight slabs in flight), the patch is transposed through LDS and
// stored four consecutive j at a time.
__global__ __launch_bounds__(256) void reduce_transpose_f32_kernel(const float* __restrict__ part, int splits, int M,
                                                                   int N, float* __restrict__ out, int64_t ldo) {
  __shared__ float patch[16][65];
  const int j0 = blockIdx.y * 16, n0 = blockIdx.x * 64;
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  const int64_t slab = (int64_t)M * N;
  const bool vec_in = (N & 3) == 0 && (reinterpret_cast<uintptr_t>(part) & 15) == 0;
  {
    const int j = j0 + ty, n = n0 + 4 * tx;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (j < M && n < N) {
      const float* p = part + (int64_t)j * N + n;
      if (vec_in && n + 3 < N) {
#pragma unroll 8
        for (int z = 0; z < splits; ++z) {
          const float4 v = *reinterpret_cast<const float4*>(p + z * slab);
          s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
      } else {
        for (int z = 0; z < splits; ++z) {
          s.x += p[z * slab];
          if (n + 1 < N) s.y += p[z * slab + 1];
          if (n + 2 < N) s.z += p[z * slab + 2];
          if (n + 3 < N) s.w += p[z * slab + 3];
        }
      }
    }
    patch[ty][4 * tx + 0] = s.x;
    patch[ty][4 * tx + 1] = s.y;
    patch[ty][4 * tx + 2] = s.z;
    patch[ty][4 * tx + 3] = s.w;
  }
  __syncthreads();
  const bool vec_out = (ldo & 3) == 0 && (reinterpret_cast<uintptr_t>(out) & 15) == 0;
  const int nl = threadIdx.x / 4, jq = (threadIdx.x % 4) * 4;  // output row n0 + nl, columns j0 + jq .. + 3
  const int n = n0 + nl, j = j0 + jq;
  if (n < N && j < M) {
    float* o = out + (int64_t)n * ldo + j;
    const float x0 = patch[jq + 0][nl], x1 = patch[jq + 1][nl], x2 = patch[jq + 2][nl], x3 = patch[jq + 3][nl];
    if (vec_out && j + 3 < M) {
      *reinterpret_cast<float4*>(o) = make_float4(x0, x1, x2, x3);
    } else {
      o[0] = x0;
      if (j + 1 < M) o[1] = x1;
      if (j + 2 < M) o[2] = x2;
      if (j + 3 < M) o[3] = x3;
    }
  }
}

__global__ __launch_bounds__(256) void scale_rows_kernel(float* T, int rows, int cols, int64_t ld, int k_lo, float s) {
  const int64_t total = (int64_t)(rows - k_lo) * cols;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = k_lo + i / cols, c = i % cols;
    T[r * ld + c] *= s;
  }
}

template <bool OUT_BF16>
__global__ __launch_bounds__(256) void cast_out_kernel(const float* __restrict__ src, int64_t lds, void* dst,
                                                       int64_t ldd, int rows, int cols, float beta) {
  const int64_t total = (int64_t)rows * cols;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = i / cols, c = i % cols;
    const float v = src[r * lds + c];
    if (OUT_BF16) {
      bf16_t* q = reinterpret_cast<bf16_t*>(dst) + r * ldd + c;
      *q = f32_to_bf16(beta == 0.f ? v : v + beta * bf16_to_f32(*q));
    } else {
      float* q = reinterpret_cast<float*>(dst) + r * ldd + c;
      *q = beta == 0.f ? v : v + beta * *q;
    }
  }
}

inline int grid_for(int64_t n, int n_cu) {
  int64_t g = (n + 255) / 256;
  const int64_t cap = (int64_t)n_cu * 8;
  if (g > cap) g = cap;
  return g < 1 ? 1 : (int)g;
}

}  // namespace

int launch_philox(prac_ctx* ctx, uint64_t seed, uint32_t draw, uint32_t stream, void* out, int64_t n, bool normal) {
  if (n <= 0) return PRAC_OK;
  const int g = grid_for((n + 3) / 4, ctx->n_cu);
  const uint32_t lo = (uint32_t)(seed & 0xFFFFFFFFu), hi = (uint32_t)(seed >> 32);
  if (normal) hipLaunchKernelGGL(philox_kernel<true>, dim3(g), dim3(256), 0, ctx->stream, lo, hi, draw, stream, out, n);
  else hipLaunchKernelGGL(philox_kernel<false>, dim3(g), dim3(256), 0, ctx->stream, lo, hi, draw, stream, out, n);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

int launch_pack_basis(prac_ctx* ctx, const float* P, int64_t d, int64_t ldp, int c, bf16_t* Pt, int64_t ldpt,
                      bf16_t* Pn, int64_t ldpn) {
  // cover i < max(d, ldpt) and j < max(c, ldpn) so that the padding is written too
  const int64_t ni = ldpt > d ? ldpt : d, nj = ldpn > c ? ldpn : c;
  dim3 grid((unsigned)((nj + 31) / 32), (unsigned)((ni + 31) / 32));
  hipLaunchKernelGGL(pack_basis_kernel, grid, dim3(256), 0, ctx->stream, P, d, ldp, c, Pt, ldpt, Pn, ldpn);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

int launch_reduce_slabs(prac_ctx* ctx, const float* part, int splits, int64_t stride, float* out, int64_t n,
                        float alpha, float beta) {
  if (n <= 0) return PRAC_OK;
  hipLaunchKernelGGL(reduce_slabs_kernel, dim3(grid_for(n, ctx->n_cu)), dim3(256), 0, ctx->stream, part, splits,
                     stride, out, n, alpha, beta);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

int launch_reduce_transpose_f32(prac_ctx* ctx, const float* part, int splits, int M, int N, float* out, int64_t ldo) {
  dim3 grid((N + 63) / 64, (M + 15) / 16);
  hipLaunchKernelGGL(reduce_transpose_f32_kernel, grid, dim3(256), 0, ctx->stream, part, splits, M, N, out, ldo);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

int launch_scale_rows(prac_ctx* ctx, float* T, int rows, int cols, int64_t ld, int k_lo, float s) {
  if (rows <= k_lo || cols <= 0) return PRAC_OK;
  hipLaunchKernelGGL(scale_rows_kernel, dim3(grid_for((int64_t)(rows - k_lo) * cols, ctx->n_cu)), dim3(256), 0,
                     ctx->stream, T, rows, cols, ld, k_lo, s);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

int launch_cast_out(prac_ctx* ctx, const float* src, int64_t lds, void* dst, prac_dtype odt, int64_t ldd, int rows,
                    int cols, float beta) {
  const int g = grid_for((int64_t)rows * cols, ctx->n_cu);
  if (odt == PRAC_BF16)
    hipLaunchKernelGGL(cast_out_kernel<true>, dim3(g), dim3(256), 0, ctx->stream, src, lds, dst, ldd, rows, cols, beta);
  else
    hipLaunchKernelGGL(cast_out_kernel<false>, dim3(g), dim3(256), 0, ctx->stream, src, lds, dst, ldd, rows, cols, beta);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

