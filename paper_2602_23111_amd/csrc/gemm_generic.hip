// Strided GEMM on the vector ALUs: fp32 or bf16 operands with arbitrary element
// strides, fp32 or fp64 accumulation.  It serves the fp32 data path (where bf16 MFMA
// rounding is not allowed), unaligned bf16 inputs, and the small dense products of
// the basis fit (G V, Y R^-1, V Z, Q1 (Q1^T S)); products whose unit strides allow it run on
// the matrix cores instead (fp32 sums, or fp64 sums for the fit's Gram matrices).
#include "prac_internal.h"

namespace {

struct GArgs {
  const void* A;
  const void* B;
  int64_t a_rs, a_cs, b_rs, b_cs;
  int M, N;
  int64_t K, k_stride;
  float* out;
  double* out64;
  int64_t ldo;
  float alpha, beta;
  int splits;          // gridDim.z; > 1: raw partial sums go to `slabs`
  int64_t steps_per_split;
  void* slabs;         // splits x M x N of ACC
};

template <typename T>
__device__ __forceinline__ float ld_f32(const void* p, int64_t idx);
template <>
__device__ __forceinline__ float ld_f32<float>(const void* p, int64_t idx) {
  return reinterpret_cast<const float*>(p)[idx];
}
template <>
__device__ __forceinline__ float ld_f32<bf16_t>(const void* p, int64_t idx) {
  return __uint_as_float(((uint32_t) reinterpret_cast<const bf16_t*>(p)[idx]) << 16);
}

constexpr int TM = 64, TN = 64, TK = 16;

// 256 threads, 64 x 64 output tile, 4 x 4 per thread.  A_MFAST / B_NFAST pick the
// thread -> element map of the tile loads so that consecutive lanes walk the
// operand's unit-stride dimension.
template <typename TA, typename TB, typename ACC, bool A_MFAST, bool B_NFAST>
__global__ __launch_bounds__(256) void gemm_generic_kernel(GArgs a) {
  __shared__ float As[TK][TM + 4];
  __shared__ float Bs[TK][TN + 4];
  const int tid = threadIdx.x;
  const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
  const int tx = tid % 16, ty = tid / 16;
  ACC acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = (ACC)0;

  const int64_t nsteps_all = (a.K + a.k_stride - 1) / a.k_stride;  // visited k values
  const int64_t sbeg = (int64_t)blockIdx.z * a.steps_per_split;
  const int64_t nsteps = min(nsteps_all, sbeg + a.steps_per_split);
  for (int64_t s0 = sbeg; s0 < nsteps; s0 += TK) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int q = tid + p * 256;
      const int mm = A_MFAST ? q % TM : q / TK, kk = A_MFAST ? q / TM : q % TK;
      const int m = m0 + mm;
      const int64_t s = s0 + kk;
      As[kk][mm] = (m < a.M && s < nsteps) ? ld_f32<TA>(a.A, m * a.a_rs + s * a.k_stride * a.a_cs) : 0.f;
    }
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int q = tid + p * 256;
      const int nn = B_NFAST ? q % TN : q / TK, kk = B_NFAST ? q / TN : q % TK;
      const int n = n0 + nn;
      const int64_t s = s0 + kk;
      Bs[kk][nn] = (n < a.N && s < nsteps) ? ld_f32<TB>(a.B, s * a.k_stride * a.b_rs + n * a.b_cs) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      float av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) av[i] = As[kk][ty + 16 * i];
#pragma unroll
      for (int j = 0; j < 4; ++j) bv[j] = Bs[kk][tx + 16 * j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += (ACC)av[i] * (ACC)bv[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty + 16 * i, n = n0 + tx + 16 * j;
      if (m < a.M && n < a.N) {
        const int64_t o = (int64_t)m * a.ldo + n;
        if (a.splits > 1) {
          reinterpret_cast<ACC*>(a.slabs)[((int64_t)blockIdx.z * a.M + m) * a.N + n] = acc[i][j];
        } else if (a.out64) {
          a.out64[o] = (double)a.alpha * (double)acc[i][j] + (a.beta == 0.f ? 0.0 : (double)a.beta * a.out64[o]);
        } else {
          const float v = a.alpha * (float)acc[i][j];
          a.out[o] = a.beta == 0.f ? v : v + a.beta * a.out[o];
        }
      }
    }
}

// ---- fp32 on the matrix cores ------------------------------------------------------
// Same contract for fp32 operands with fp32 sums whose m (A) and n (B) strides are one
// element (the basis fit's G V with G read through its symmetry, and Q1 T): 64 x 64 tile per
// workgroup, one 32 x 32 block of v_mfma_f32_32x32x2_f32 per wave, k in steps of 32 through
// double-buffered LDS.  Lane l holds A(m = l % 32, k = l / 32) and B(k = l / 32, n = l % 32); rows
// are padded by 32 floats so that the two half-waves of a fragment read hit disjoint banks.
typedef float f32x16_t __attribute__((ext_vector_type(16)));
constexpr int FK = 32, FLD = 64 + 32;

// A_KFAST: A's k stride is one element instead (a tall row-major block times a small matrix: V M, V Z,
// Q1 T); a thread then fetches 8 consecutive k of one row, lanes along m as they are stored to LDS.
template <bool A_KFAST>
__global__ __launch_bounds__(256) void gemm_f32_mfma_kernel(GArgs a) {
  __shared__ float As[2][FK][FLD];
  __shared__ float Bs[2][FK][FLD];
  const float* __restrict__ A = reinterpret_cast<const float*>(a.A);
  const float* __restrict__ B = reinterpret_cast<const float*>(a.B);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int wm = (wave >> 1) * 32, wn = (wave & 1) * 32;
  const int64_t kbeg = (int64_t)blockIdx.z * a.steps_per_split;
  const int64_t kend = min(a.K, kbeg + a.steps_per_split);
  // tile loads: 8 elements per thread and operand, thread t -> k rows t / 64 + 4 p, column t % 64
  const int lc = tid & 63, lr = tid >> 6;
  float ra[8], rb[8];
  auto gload = [&](int64_t k0) {
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const int64_t k = k0 + lr + 4 * p;
      const bool kin = k < kend;
      if constexpr (A_KFAST) {
        const int64_t ka = k0 + 8 * lr + p;
        ra[p] = (ka < kend && m0 + lc < a.M) ? A[(int64_t)(m0 + lc) * a.a_rs + ka] : 0.f;
      } else {
        ra[p] = (kin && m0 + lc < a.M) ? A[k * a.a_cs + (m0 + lc)] : 0.f;
      }
      rb[p] = (kin && n0 + lc < a.N) ? B[k * a.b_rs + (n0 + lc)] : 0.f;
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      As[buf][A_KFAST ? 8 * lr + p : lr + 4 * p][lc] = ra[p];
      Bs[buf][lr + 4 * p][lc] = rb[p];
    }
  };
  f32x16_t acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  const int fi = lane & 31, fk = lane >> 5;
  if (kbeg < kend) {
    gload(kbeg);
    sstore(0);
    __syncthreads();
    int buf = 0;
    for (int64_t k0 = kbeg; k0 < kend; k0 += FK) {
      const bool more = k0 + FK < kend;
      if (more) gload(k0 + FK);
#pragma unroll
      for (int kk = 0; kk < FK; kk += 2)
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(As[buf][kk + fk][wm + fi], Bs[buf][kk + fk][wn + fi], acc, 0, 0, 0);
      if (more) sstore(buf ^ 1);  // last read by the MFMAs two steps ago, before the previous barrier
      __syncthreads();
      buf ^= 1;
    }
  }
  // register v of lane (fi, fk): row wm + 8 (v / 4) + 4 fk + v % 4, column wn + fi
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int m = m0 + wm + 8 * (v / 4) + 4 * fk + (v % 4), n = n0 + wn + fi;
    if (m < a.M && n < a.N) {
      const int64_t o = (int64_t)m * a.ldo + n;
      if (a.splits > 1) {
        reinterpret_cast<float*>(a.slabs)[((int64_t)blockIdx.z * a.M + m) * a.N + n] = acc[v];
      } else {
        const float x = a.alpha * acc[v];
        a.out[o] = a.beta == 0.f ? x : x + a.beta * a.out[o];
      }
    }
  }
}

// ---- fp64 sums on the matrix cores --------------------------------------------------
// Same contract again for fp32 operands with fp64 sums (the fit's n x n Gram matrices Y^T Y and
// V^T Y over panels of d rows): products of fp32 values are exact in fp64, the sums run on
// v_mfma_f64_16x16x4_f64.  64 x 64 tile per workgroup, a 32 x 32 block (2 x 2 MFMA blocks) per wave;
// operands go from global memory straight to registers, since a workgroup's share of k is a few
// dozen rows and all of its requests are in flight at once.  Lane l holds A(m = l % 16, k = l / 16)
// and B(k = l / 16, n = l % 16); register v of lane l is D(m = 4 v + l / 16, n = l % 16).
typedef double f64x4_t __attribute__((ext_vector_type(4)));
constexpr int DK = 32;  // k values per step: 8 MFMA steps of 4

__global__ __launch_bounds__(256) void gemm_f64_mfma_kernel(GArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int fi = lane & 15, fk = lane >> 4;
  const int m0 = blockIdx.y * 64 + (wave >> 1) * 32, n0 = blockIdx.x * 64 + (wave & 1) * 32;
  const int64_t kbeg = (int64_t)blockIdx.z * a.steps_per_split;
  const int64_t kend = min(a.K, kbeg + a.steps_per_split);
  const bool am[2] = {m0 + fi < a.M, m0 + 16 + fi < a.M}, bn[2] = {n0 + fi < a.N, n0 + 16 + fi < a.N};
  const float* __restrict__ Ap = reinterpret_cast<const float*>(a.A) + (m0 + fi);
  const float* __restrict__ Bp = reinterpret_cast<const float*>(a.B) + (n0 + fi);
  f64x4_t acc[2][2];
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[s][t][v] = 0.0;
  for (int64_t k0 = kbeg; k0 < kend; k0 += DK) {
    float ra[DK / 4][2], rb[DK / 4][2];
#pragma unroll
    for (int u = 0; u < DK / 4; ++u) {
      const int64_t k = k0 + 4 * u + fk;
      const bool kin = k < kend;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        ra[u][t] = (kin && am[t]) ? Ap[k * a.a_cs + 16 * t] : 0.f;
        rb[u][t] = (kin && bn[t]) ? Bp[k * a.b_rs + 16 * t] : 0.f;
      }
    }
#pragma unroll
    for (int u = 0; u < DK / 4; ++u)
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int t = 0; t < 2; ++t)
          acc[s][t] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)ra[u][s], (double)rb[u][t], acc[s][t], 0, 0, 0);
  }
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int m = m0 + 16 * s + 4 * v + fk, n = n0 + 16 * t + fi;
        if (m < a.M && n < a.N) {
          const int64_t o = (int64_t)m * a.ldo + n;
          if (a.splits > 1) {
            reinterpret_cast<double*>(a.slabs)[((int64_t)blockIdx.z * a.M + m) * a.N + n] = acc[s][t][v];
          } else if (a.out64) {
            a.out64[o] = (double)a.alpha * acc[s][t][v] + (a.beta == 0.f ? 0.0 : (double)a.beta * a.out64[o]);
          } else {
            const float x = a.alpha * (float)acc[s][t][v];
            a.out[o] = a.beta == 0.f ? x : x + a.beta * a.out[o];
          }
        }
      }
}

template <typename TA, typename TB, typename ACC>
void launch3(const GArgs& a, hipStream_t st) {
  dim3 grid((a.N + TN - 1) / TN, (a.M + TM - 1) / TM, a.splits), block(256);
  const bool a_mfast = a.a_rs == 1 || (a.a_cs != 1 && a.a_rs < a.a_cs);
  const bool b_nfast = a.b_cs == 1 || (a.b_rs != 1 && a.b_cs < a.b_rs);
  if (a_mfast && b_nfast) hipLaunchKernelGGL((gemm_generic_kernel<TA, TB, ACC, true, true>), grid, block, 0, st, a);
  else if (a_mfast) hipLaunchKernelGGL((gemm_generic_kernel<TA, TB, ACC, true, false>), grid, block, 0, st, a);
  else if (b_nfast) hipLaunchKernelGGL((gemm_generic_kernel<TA, TB, ACC, false, true>), grid, block, 0, st, a);
  else hipLaunchKernelGGL((gemm_generic_kernel<TA, TB, ACC, false, false>), grid, block, 0, st, a);
}

template <typename TA, typename TB>
void launch2(const GArgs& a, bool acc64, hipStream_t st) {
  if (acc64) launch3<TA, TB, double>(a, st);
  else launch3<TA, TB, float>(a, st);
}

// out = alpha * sum_z slab[z] + beta * out over an M x N matrix with leading dim ldo
template <typename ACC, typename OUT>
__global__ __launch_bounds__(256) void reduce_gen_kernel(const ACC* __restrict__ slabs, int splits, int M, int N,
                                                         OUT* out, int64_t ldo, float alpha, float beta) {
  const int64_t total = (int64_t)M * N;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    ACC s = (ACC)0;
#pragma unroll 8
    for (int z = 0; z < splits; ++z) s += slabs[z * total + i];  // eight slabs in flight
    const int64_t o = (i / N) * ldo + i % N;
    const OUT v = (OUT)alpha * (OUT)s;
    out[o] = beta == 0.f ? v : v + (OUT)beta * out[o];
  }
}

}  // namespace

int launch_gemm_generic(prac_ctx* ctx, const GemmGenArgs& g) {
  if (g.M <= 0 || g.N <= 0) return PRAC_OK;
  GArgs a;
  a.A = g.A; a.B = g.B;
  a.a_rs = g.a_rs; a.a_cs = g.a_cs; a.b_rs = g.b_rs; a.b_cs = g.b_cs;
  a.M = g.M; a.N = g.N; a.K = g.K; a.k_stride = g.k_stride < 1 ? 1 : g.k_stride;
  a.out = g.out; a.out64 = g.out64; a.ldo = g.ldo; a.alpha = g.alpha; a.beta = g.beta;
  const int64_t nsteps = (a.K + a.k_stride - 1) / a.k_stride;
  a.splits = (g.splits > 1 && g.slabs) ? g.splits : 1;
  if (a.splits > 1 && (size_t)a.splits * a.M * a.N * (g.acc64 ? sizeof(double) : sizeof(float)) > g.slab_bytes)
    return PRAC_EINVAL;  // the caller's plan is too small for this product: never write past it
  a.steps_per_split = ((nsteps + a.splits - 1) / a.splits + TK - 1) / TK * TK;
  if (a.steps_per_split < TK) a.steps_per_split = TK;
  a.slabs = g.slabs;
  const bool abf = g.adt == PRAC_BF16, bbf = g.bdt == PRAC_BF16;
  const bool mfma = !abf && !bbf && !g.acc64 && !g.out64 && (a.a_rs == 1 || a.a_cs == 1) && a.b_cs == 1 &&
                    a.k_stride == 1 && (int64_t)a.M * a.N >= 64 * 64 && a.K >= 64;
  const bool mfma64 = !abf && !bbf && g.acc64 && a.a_rs == 1 && a.b_cs == 1 && a.k_stride == 1;
  if (mfma) {
    a.steps_per_split = ((a.K + a.splits - 1) / a.splits + FK - 1) / FK * FK;
    const dim3 grid((a.N + 63) / 64, (a.M + 63) / 64, a.splits);
    if (a.a_rs == 1) hipLaunchKernelGGL(gemm_f32_mfma_kernel<false>, grid, dim3(256), 0, ctx->stream, a);
    else hipLaunchKernelGGL(gemm_f32_mfma_kernel<true>, grid, dim3(256), 0, ctx->stream, a);
  } else if (mfma64) {
    a.steps_per_split = ((a.K + a.splits - 1) / a.splits + 3) / 4 * 4;
    hipLaunchKernelGGL(gemm_f64_mfma_kernel, dim3((a.N + 63) / 64, (a.M + 63) / 64, a.splits), dim3(256), 0, ctx->stream,
                       a);
  } else if (abf && bbf) launch2<bf16_t, bf16_t>(a, g.acc64, ctx->stream);
  else if (abf) launch2<bf16_t, float>(a, g.acc64, ctx->stream);
  else if (bbf) launch2<float, bf16_t>(a, g.acc64, ctx->stream);
  else launch2<float, float>(a, g.acc64, ctx->stream);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  if (a.splits > 1) {
    const int64_t total = (int64_t)a.M * a.N;
    int64_t gr = (total + 255) / 256;
    if (gr > ctx->n_cu * 8) gr = ctx->n_cu * 8;
    if (g.acc64 && g.out64)
      hipLaunchKernelGGL((reduce_gen_kernel<double, double>), dim3((unsigned)gr), dim3(256), 0, ctx->stream,
                         reinterpret_cast<const double*>(a.slabs), a.splits, a.M, a.N, g.out64, a.ldo, a.alpha, a.beta);
    else if (g.acc64)
      hipLaunchKernelGGL((reduce_gen_kernel<double, float>), dim3((unsigned)gr), dim3(256), 0, ctx->stream,
                         reinterpret_cast<const double*>(a.slabs), a.splits, a.M, a.N, g.out, a.ldo, a.alpha, a.beta);
    else
      hipLaunchKernelGGL((reduce_gen_kernel<float, float>), dim3((unsigned)gr), dim3(256), 0, ctx->stream,
                         reinterpret_cast<const float*>(a.slabs), a.splits, a.M, a.N, g.out, a.ldo, a.alpha, a.beta);
    PRAC_HIP_TRY(ctx, hipGetLastError());
  }
  return PRAC_OK;
}
