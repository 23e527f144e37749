// Small kernels of the per-step path around the two streaming contractions (ws_kernels.hip):
// packing of P and C into MFMA fragment order, the slab reduction that turns the token-split
// partial sums of C^T dY into T (bf16, fragment order, random rows scaled), and dW = P T.
//
// Fragment order ("frag16x32"), used for P (B operand of compress), for the packed compressed
// activation C (A operand of C^T dY), for T and for P as an A operand: a block of 16 reduction
// indices x 32 rows/columns is 64 lanes x 8 bf16; lane = 32 h + j holds, for row/column j, the
// reduction indices listed by slot(h, e), e = 0..7.
//   P, T:  slot(h, e) = 8 h + e                         (k = 16 kb + 8 h + e)
//   C:     slot(h, e) = 4 h + e (e < 4), 8 + 4 h + e - 4 (e >= 4)   (token = 16 tb + slot)
// The C order is the order in which the 32x32 MFMA accumulator of compress holds its rows, so
// compress stores a packed block straight from its registers.  A wave fetches a whole 32x16
// operand block with one fully coalesced 1 KB load.
#include <algorithm>
#include <type_traits>

#include "frag_utils.h"

namespace {

// ------------------------------------------------------------- small helpers
// Pfrag[(kb * ncb + cb) * 64 + lane][e] = bf16(P[16 kb + 8 h + e][32 cb + j]), zero outside d x c
__global__ __launch_bounds__(256) void pack_pfrag_kernel(const float* __restrict__ P, int64_t d, int64_t ldp, int c,
                                                         int nkb, int ncb, bf16_t* __restrict__ out) {
  const int64_t total = (int64_t)nkb * ncb * 64;
  for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += (int64_t)gridDim.x * blockDim.x) {
    const int lane = (int)(g & 63), j = lane & 31, h = lane >> 5;
    const int64_t blk = g >> 6;
    const int cb = (int)(blk % ncb);
    const int64_t kb = blk / ncb;
    const int col = cb * 32 + j;
    uint32_t w[4];
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      float f0 = 0.f, f1 = 0.f;
      const int64_t k0 = kb * 16 + 8 * h + 2 * e2;
      if (col < c && k0 < d) f0 = P[k0 * ldp + col];
      if (col < c && k0 + 1 < d) f1 = P[(k0 + 1) * ldp + col];
      w[e2] = pack2(f0, f1);
    }
    reinterpret_cast<uint4*>(out)[g] = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// The same fragment order for a bf16 weight matrix (pure permutation, zero padded): element
// (k, n) of W is W[k * ldw + n] (w_layout 0, d x m) or W[n * ldw + k] (w_layout 1, m x d).
__global__ __launch_bounds__(256) void pack_wfrag_kernel(const bf16_t* __restrict__ W, int64_t ldw, int w_layout,
                                                         int64_t d, int m, int nkb, int ncb,
                                                         bf16_t* __restrict__ out) {
  const int64_t total = (int64_t)nkb * ncb * 64;
  for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += (int64_t)gridDim.x * blockDim.x) {
    const int lane = (int)(g & 63), j = lane & 31, h = lane >> 5;
    const int64_t blk = g >> 6;
    const int cb = (int)(blk % ncb);
    const int64_t kb = blk / ncb;
    const int col = cb * 32 + j;
    const int64_t k0 = kb * 16 + 8 * h;
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    if (col < m) {
      if (w_layout == 1 && k0 + 8 <= d && (ldw & 7) == 0 && (reinterpret_cast<uintptr_t>(W) & 15) == 0) {
        const uint4 v = *reinterpret_cast<const uint4*>(W + (int64_t)col * ldw + k0);
        w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int64_t kk = k0 + e;
          if (kk < d) {
            const uint32_t x = w_layout == 1 ? W[(int64_t)col * ldw + kk] : W[kk * ldw + col];
            w[e >> 1] |= x << (16 * (e & 1));
          }
        }
      }
    }
    reinterpret_cast<uint4*>(out)[g] = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// Fragment order of Ps^T for the reconstruction Xh = C Ps^T (Section 5.1): the sum runs over the
// columns of P, the output columns are the rows of P; the random columns carry the scaling factor.
__global__ __launch_bounds__(256) void pack_ptfrag_kernel(const float* __restrict__ P, int64_t d, int64_t ldp, int c,
                                                          int k_lo, float scale_hi, int nkb, int ncb,
                                                          bf16_t* __restrict__ out) {
  const int64_t total = (int64_t)nkb * ncb * 64;
  for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += (int64_t)gridDim.x * blockDim.x) {
    const int lane = (int)(g & 63), j = lane & 31, h = lane >> 5;
    const int64_t blk = g >> 6;
    const int cb = (int)(blk % ncb);
    const int64_t kb = blk / ncb;
    const int64_t row = (int64_t)cb * 32 + j;  // row of P = output column
    uint32_t w[4];
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      float f[2] = {0.f, 0.f};
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int64_t kk = kb * 16 + 8 * h + 2 * e2 + u;  // column of P
        if (row < d && kk < c) f[u] = P[row * ldp + kk] * (kk >= k_lo ? scale_hi : 1.f);
      }
      w[e2] = pack2(f[0], f[1]);
    }
    reinterpret_cast<uint4*>(out)[g] = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

__device__ __forceinline__ int c_slot(int h, int e) { return e < 4 ? 4 * h + e : 8 + 4 * h + (e - 4); }

// packed C -> row-major (bit-exact copy of the elements)
__global__ __launch_bounds__(256) void unpack_c_kernel(const bf16_t* __restrict__ Cpk, int N, int c, int ccb,
                                                       bf16_t* __restrict__ C, int64_t ldc) {
  const int64_t ntb = (N + 15) / 16, total = ntb * ccb * 64;
  for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += (int64_t)gridDim.x * blockDim.x) {
    const int lane = (int)(g & 63), j = lane & 31, h = lane >> 5;
    const int64_t blk = g >> 6;
    const int cb = (int)(blk % ccb);
    const int64_t tb = blk / ccb;
    const int col = cb * 32 + j;
    const uint4 v = reinterpret_cast<const uint4*>(Cpk)[g];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int64_t t = tb * 16 + c_slot(h, e);
      if (t < N && col < c) C[t * ldc + col] = (bf16_t)((w[e >> 1] >> (16 * (e & 1))) & 0xFFFFu);
    }
  }
}

// row-major C -> packed (padding rows / columns zero)
__global__ __launch_bounds__(256) void pack_c_kernel(const bf16_t* __restrict__ C, int64_t ldc, int N, int c, int ccb,
                                                     bf16_t* __restrict__ Cpk) {
  const int64_t ntb = (int64_t)((N + 127) / 128) * 8, total = ntb * ccb * 64;
  for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += (int64_t)gridDim.x * blockDim.x) {
    const int lane = (int)(g & 63), j = lane & 31, h = lane >> 5;
    const int64_t blk = g >> 6;
    const int cb = (int)(blk % ccb);
    const int64_t tb = blk / ccb;
    const int col = cb * 32 + j;
    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int64_t t = tb * 16 + c_slot(h, e);
      const uint32_t x = (t < N && col < c) ? C[t * ldc + col] : 0u;
      w[e >> 1] |= x << (16 * (e & 1));
    }
    reinterpret_cast<uint4*>(Cpk)[g] = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// ------------------------------------------------------------------- dW = P T
// T in fragment order, built by the slab reducer: Tf[(kb * nmb + nb) * 64 + lane][e] =
// bf16(w_k * sum_z slab[z][k][n]) with k = 16 kb + 8 h + e, n = 32 nb + j, lane = 32 h + j,
// w_k = 1 for k < k_lo and scale_hi above; zero where k >= c or n >= m.
// One workgroup per (k-block, pair of 32-column blocks): 256 threads sum a 16 x 64 patch of
// the slabs with one float4 per thread and slab (coalesced 256-byte rows), exchange it through
// LDS and 128 of them emit the two fragments.
struct ReduceTfArgs {
  int n_out, splits, c, k_lo, nkb;
  float scale_hi;
  const float* slabs[PRAC_CTDY_MAX_OUT];  // [splits][c][m_h]
  bf16_t* Tf[PRAC_CTDY_MAX_OUT];          // [nkb][nmb_h][64][8]
  int m[PRAC_CTDY_MAX_OUT];
  int nmb[PRAC_CTDY_MAX_OUT];
  int pair0[PRAC_CTDY_MAX_OUT + 1];       // first pair of column blocks of output h in the launch
};

__global__ __launch_bounds__(256) void reduce_to_tfrag_kernel(ReduceTfArgs a) {
  __shared__ float patch[16][68];
  const int bid = touch_kernel_args<sizeof(ReduceTfArgs)>(blockIdx.x);
  const int pairs = a.pair0[a.n_out];
  const int kb = bid / pairs, gp = bid % pairs;
  int h = 0;
#pragma unroll
  for (int q = 1; q < PRAC_CTDY_MAX_OUT; ++q)
    if (q < a.n_out && gp >= a.pair0[q]) h = q;
  const int np = gp - a.pair0[h];
  const float* __restrict__ slabs = a.slabs[h];
  const int m = a.m[h], nmb = a.nmb[h], c = a.c, splits = a.splits;
  const int tid = threadIdx.x;
  const int row = tid >> 4, col = (tid & 15) * 4;
  const int k = kb * 16 + row, n = np * 64 + col;
  const int64_t slab = (int64_t)c * m;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (k < c && n < m) {
    const float* p = slabs + (int64_t)k * m + n;
    if (n + 3 < m && (m & 3) == 0) {
#pragma unroll 8
      for (int z = 0; z < splits; ++z) {
        // read once
        const f32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p + z * slab));
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
      }
    } else {
      for (int z = 0; z < splits; ++z) {
        s.x += p[z * slab];
        if (n + 1 < m) s.y += p[z * slab + 1];
        if (n + 2 < m) s.z += p[z * slab + 2];
        if (n + 3 < m) s.w += p[z * slab + 3];
      }
    }
    const float w = k >= a.k_lo ? a.scale_hi : 1.f;
    s.x *= w; s.y *= w; s.z *= w; s.w *= w;
  }
  patch[row][col + 0] = s.x;
  patch[row][col + 1] = s.y;
  patch[row][col + 2] = s.z;
  patch[row][col + 3] = s.w;
  __syncthreads();
  if (tid < 128) {
    const int nbl = tid >> 6, lane = tid & 63, j = lane & 31, hh = lane >> 5;
    u32x4 o;
    o.x = pack2_hw(patch[8 * hh + 0][nbl * 32 + j], patch[8 * hh + 1][nbl * 32 + j]);
    o.y = pack2_hw(patch[8 * hh + 2][nbl * 32 + j], patch[8 * hh + 3][nbl * 32 + j]);
    o.z = pack2_hw(patch[8 * hh + 4][nbl * 32 + j], patch[8 * hh + 5][nbl * 32 + j]);
    o.w = pack2_hw(patch[8 * hh + 6][nbl * 32 + j], patch[8 * hh + 7][nbl * 32 + j]);
    reinterpret_cast<u32x4*>(a.Tf[h])[((int64_t)kb * nmb + np * 2 + nbl) * 64 + lane] = o;
  }
}

// P as an A operand in fragment order: Pa[(rb * nkb + kb) * 64 + lane][e] = bf16(P[32 rb + i][16 kb + 8 h + e]),
// lane = 32 h + i; zero outside d x c.
__global__ __launch_bounds__(256) void pack_pafrag_kernel(const float* __restrict__ P, int64_t d, int64_t ldp, int c,
                                                          int nrb, int nkb, bf16_t* __restrict__ out) {
  const int64_t total = (int64_t)nrb * nkb * 64;
  for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += (int64_t)gridDim.x * blockDim.x) {
    const int lane = (int)(g & 63), i = lane & 31, h = lane >> 5;
    const int64_t blk = g >> 6;
    const int kb = (int)(blk % nkb);
    const int64_t row = (blk / nkb) * 32 + i;
    float f[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int k = kb * 16 + 8 * h + e;
      f[e] = (row < d && k < c) ? P[row * ldp + k] : 0.f;
    }
    u32x4 o;
    o.x = pack2(f[0], f[1]);
    o.y = pack2(f[2], f[3]);
    o.z = pack2(f[4], f[5]);
    o.w = pack2(f[6], f[7]);
    reinterpret_cast<u32x4*>(out)[g] = o;
  }
}

struct PtArgs {
  const bf16_t* Pa;  // [nrb][nkb][64][8]
  int d, nkb;
  int tiles_m, tiles_n;  // tiles_n: 128-column tiles over all outputs
  int tiles_m_rb;        // 32-row blocks held by Pa
  float beta;
  // up to PRAC_CTDY_MAX_OUT products sharing P (layers reading the same input, Section 5.1):
  // output h owns the column tiles tile0[h] .. tile0[h+1]-1 of the launch
  int n_out;
  const bf16_t* Tf[PRAC_CTDY_MAX_OUT];  // [nkb][nmb_h][64][8]
  void* dW[PRAC_CTDY_MAX_OUT];
  int64_t lddw[PRAC_CTDY_MAX_OUT];
  int m[PRAC_CTDY_MAX_OUT];
  int nmb[PRAC_CTDY_MAX_OUT];
  int vec_ok[PRAC_CTDY_MAX_OUT];        // dW rows allow aligned 16-byte accesses
  int tile0[PRAC_CTDY_MAX_OUT + 1];
};

// which output a column tile of the launch belongs to
__device__ __forceinline__ int pt_output_of(const PtArgs& a, int tn) {
  int h = 0;
#pragma unroll
  for (int q = 1; q < PRAC_CTDY_MAX_OUT; ++q)
    if (q < a.n_out && tn >= a.tile0[q]) h = q;
  return h;
}

// dW (d x m) = P T, K = c (a few hundred): both operands are read in fragment order
// straight from L2, no LDS.  256 threads = 2 x 2 waves, a 128 x 128 tile per workgroup,
// 64 x 64 per wave; fragments are requested PT_PD k-blocks ahead (c = 256 is 16 k-blocks: one round
// of requests, one memory latency).
constexpr int PT_PD = 16;
constexpr int PT_TLD = 128 + 4;  // floats per row of the output staging tile
template <bool OUT_BF16>
__global__ __launch_bounds__(256) void pt_kernel(PtArgs a) {
  const int bid = touch_kernel_args<sizeof(PtArgs)>(blockIdx.x);
  const int total = a.tiles_m * a.tiles_n;
  const int per_xcd = (total + 7) / 8;
  const int xcd = bid & 7, slot = bid >> 3;
  const int logical = xcd * per_xcd + slot;
  if (slot >= per_xcd || logical >= total) return;
  const int tn_g = logical % a.tiles_n, tm = logical / a.tiles_n;
  const int h = pt_output_of(a, tn_g), tn = tn_g - a.tile0[h];
  const u32x4* __restrict__ Tf = reinterpret_cast<const u32x4*>(a.Tf[h]);
  void* const odW = a.dW[h];
  const int64_t olddw = a.lddw[h];
  const int om = a.m[h], onmb = a.nmb[h], ovec = a.vec_ok[h];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 31, lh = lane >> 5;
  const int rb0 = tm * 4 + (wave >> 1) * 2, nb0 = tn * 4 + (wave & 1) * 2;
  const u32x4* __restrict__ Pa = reinterpret_cast<const u32x4*>(a.Pa);

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  u32x4 fr[PT_PD][4];
  auto gload = [&](int kb, u32x4 (&r)[4]) {
    const int k = min(kb, a.nkb - 1);
    r[0] = Pa[((int64_t)rb0 * a.nkb + k) * 64 + lane];
    r[1] = Pa[((int64_t)(rb0 + 1) * a.nkb + k) * 64 + lane];
    r[2] = Tf[((int64_t)k * onmb + nb0) * 64 + lane];
    r[3] = Tf[((int64_t)k * onmb + nb0 + 1) * 64 + lane];
  };
  auto mfma4 = [&](const u32x4 (&r)[4]) {
    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(r[0]), as_frag(r[2]), acc[0][0], 0, 0, 0);
    acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(r[0]), as_frag(r[3]), acc[0][1], 0, 0, 0);
    acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(r[1]), as_frag(r[2]), acc[1][0], 0, 0, 0);
    acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(r[1]), as_frag(r[3]), acc[1][1], 0, 0, 0);
  };
#pragma unroll
  for (int t = 0; t < PT_PD; ++t) gload(t, fr[t]);
  int kb = 0;
  for (; kb + PT_PD <= a.nkb; kb += PT_PD) {
#pragma unroll
    for (int t = 0; t < PT_PD; ++t) {
      mfma4(fr[t]);
      if (kb + PT_PD + t < a.nkb) gload(kb + PT_PD + t, fr[t]);
    }
  }
#pragma unroll
  for (int t = 0; t < PT_PD; ++t)
    if (kb + t < a.nkb) mfma4(fr[t]);

  // The accumulators hold columns across lanes and rows across registers; the tile goes through
  // LDS (fp32, padded rows) so that the stores to dW are 16-byte chunks along rows.
  // block (i, j): register v of lane (li, lh) is row 32 (rb0 + i) + 8*(v/4) + 4 lh + v%4, column 32 (nb0 + j) + li
  extern __shared__ __align__(16) unsigned char pt_smem[];
  float* tile = reinterpret_cast<float*>(pt_smem);  // [128][PT_TLD]
  const int wr = wave >> 1, wc = wave & 1;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = (wr * 2 + i) * 32 + 8 * (v / 4) + 4 * lh + (v % 4);
        const int col = (wc * 2 + j) * 32 + li;
        tile[row * PT_TLD + col] = acc[i][j][v];
      }
  __syncthreads();
  const int row0 = tm * 128, col0 = tn * 128;
  if (OUT_BF16) {
    // 8 columns (16 bytes of bf16) per thread and step: 16 threads per row, 16 rows per step
    const int cr = tid >> 4, c8 = (tid & 15) * 8;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const int row = cr + 16 * p;
      const int grow = row0 + row, gcol = col0 + c8;
      if (grow >= a.d || gcol >= om) continue;
      const float4 lo = *reinterpret_cast<const float4*>(tile + row * PT_TLD + c8);
      const float4 hi = *reinterpret_cast<const float4*>(tile + row * PT_TLD + c8 + 4);
      float x[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      bf16_t* q = reinterpret_cast<bf16_t*>(odW) + (int64_t)grow * olddw + gcol;
      if (ovec && gcol + 8 <= om) {
        if (a.beta != 0.f) {
          const u32x4 old = *reinterpret_cast<const u32x4*>(q);
#pragma unroll
          for (int e = 0; e < 8; ++e)
            x[e] += a.beta * __uint_as_float(((e & 1) ? (old[e >> 1] >> 16) : (old[e >> 1] & 0xFFFFu)) << 16);
        }
        u32x4 o;
        o.x = pack2_hw(x[0], x[1]);
        o.y = pack2_hw(x[2], x[3]);
        o.z = pack2_hw(x[4], x[5]);
        o.w = pack2_hw(x[6], x[7]);
        stream_store(reinterpret_cast<u32x4*>(q), o);
      } else {
        for (int e = 0; e < 8 && gcol + e < om; ++e)
          q[e] = f32_to_bf16(a.beta == 0.f ? x[e] : x[e] + a.beta * __uint_as_float(((uint32_t)q[e]) << 16));
      }
    }
  } else {
    // 4 columns (16 bytes of fp32) per thread and step: 32 threads per row, 8 rows per step
    const int cr = tid >> 5, c4 = (tid & 31) * 4;
#pragma unroll
    for (int p = 0; p < 16; ++p) {
      const int row = cr + 8 * p;
      const int grow = row0 + row, gcol = col0 + c4;
      if (grow >= a.d || gcol >= om) continue;
      float4 x = *reinterpret_cast<const float4*>(tile + row * PT_TLD + c4);
      float* q = reinterpret_cast<float*>(odW) + (int64_t)grow * olddw + gcol;
      if (ovec && gcol + 4 <= om) {
        if (a.beta != 0.f) {
          const float4 old = *reinterpret_cast<const float4*>(q);
          x.x += a.beta * old.x; x.y += a.beta * old.y; x.z += a.beta * old.z; x.w += a.beta * old.w;
        }
        stream_store(reinterpret_cast<f32x4_t*>(q), f32x4_t{x.x, x.y, x.z, x.w});
      } else {
        const float xs[4] = {x.x, x.y, x.z, x.w};
        for (int e = 0; e < 4 && gcol + e < om; ++e) q[e] = a.beta == 0.f ? xs[e] : xs[e] + a.beta * q[e];
      }
    }
  }
}

// The same product for shapes with many tiles or a long K (c of several hundred, a wide or
// tall dW): operands go through LDS so that each fragment crosses L2 -> L1 once per workgroup
// instead of once per wave.  TM x 128 tile, 2 x 2 waves of (TM/2) x 64, K in chunks of
// PT2_KC k-blocks; the next chunk is fetched into registers while the current one is
// multiplied and written to the other LDS stage afterwards.  Fragments are stored in
// fragment order, so the copy is a straight 16 bytes per lane and every LDS access of a wave
// covers one contiguous 1 KB block.
constexpr int PT2_KC = 4;
constexpr int PT2_ELD = 64 + 4;  // floats per row of a wave's output staging tile (64 x 64)
template <int TM, bool OUT_BF16>
__global__ __launch_bounds__(256) void pt_tiled_kernel(PtArgs a) {
  constexpr int RB = TM / 32;  // 32-row blocks of the tile
  constexpr int RI = TM / 64;  // A fragments per wave and k-block
  constexpr int A_BYTES = RB * PT2_KC * 1024, B_BYTES = PT2_KC * 4 * 1024, STAGE = A_BYTES + B_BYTES;
  constexpr int A_LD = A_BYTES / 4096, B_LD = B_BYTES / 4096;  // 16-byte loads per thread and chunk
  extern __shared__ __align__(16) unsigned char pt_smem[];

  const int bid = touch_kernel_args<sizeof(PtArgs)>(blockIdx.x);
  const int total = a.tiles_m * a.tiles_n;
  const int per_xcd = (total + 7) / 8;
  const int xcd = bid & 7, slot = bid >> 3;
  const int logical = xcd * per_xcd + slot;
  if (slot >= per_xcd || logical >= total) return;
  const int tn_g = logical % a.tiles_n, tm = logical / a.tiles_n;
  const int h = pt_output_of(a, tn_g), tn = tn_g - a.tile0[h];
  const u32x4* __restrict__ Tf = reinterpret_cast<const u32x4*>(a.Tf[h]);
  void* const odW = a.dW[h];
  const int64_t olddw = a.lddw[h];
  const int om = a.m[h], onmb = a.nmb[h], ovec = a.vec_ok[h];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 31, lh = lane >> 5;
  const int wr = wave >> 1, wc = wave & 1;
  const u32x4* __restrict__ Pa = reinterpret_cast<const u32x4*>(a.Pa);
  const int nrb = a.tiles_m_rb;  // 32-row blocks Pa holds

  f32x16 acc[RI][2];
#pragma unroll
  for (int i = 0; i < RI; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // sweep s of A: row block s of the tile, its PT2_KC k-blocks (4 KB, contiguous in Pa); sweep s
  // of B: k-block s of the chunk, the tile's four column blocks (4 KB, contiguous in Tf).
  // k-blocks past the end re-read the last one and are not multiplied; row blocks past the
  // end re-read the last one and their rows are not stored.
  u32x4 ra[A_LD], rb[B_LD];
  const int sub = tid >> 6;  // which 1 KB block of a sweep this thread copies
  auto gload = [&](int kb0) {
#pragma unroll
    for (int s = 0; s < A_LD; ++s) {
      const int rbg = min(tm * RB + s, nrb - 1), kb = min(kb0 + sub, a.nkb - 1);
      ra[s] = Pa[((int64_t)rbg * a.nkb + kb) * 64 + lane];
    }
#pragma unroll
    for (int s = 0; s < B_LD; ++s) {
      const int kb = min(kb0 + s, a.nkb - 1);
      rb[s] = Tf[((int64_t)kb * onmb + tn * 4 + sub) * 64 + lane];
    }
  };
  auto sstore = [&](int stage) {
    unsigned char* st = pt_smem + stage * STAGE;
#pragma unroll
    for (int s = 0; s < A_LD; ++s) *reinterpret_cast<u32x4*>(st + s * 4096 + tid * 16) = ra[s];
#pragma unroll
    for (int s = 0; s < B_LD; ++s) *reinterpret_cast<u32x4*>(st + A_BYTES + s * 4096 + tid * 16) = rb[s];
  };

  gload(0);
  sstore(0);
  __syncthreads();
  int stage = 0;
  for (int kb0 = 0; kb0 < a.nkb; kb0 += PT2_KC) {
    const bool more = kb0 + PT2_KC < a.nkb;
    if (more) gload(kb0 + PT2_KC);
    const unsigned char* st = pt_smem + stage * STAGE;
    const int kbs = min(PT2_KC, a.nkb - kb0);
#pragma unroll
    for (int q = 0; q < PT2_KC; ++q) {
      if (q < kbs) {
        u32x4 fa[RI], fb[2];
#pragma unroll
        for (int i = 0; i < RI; ++i)
          fa[i] = *reinterpret_cast<const u32x4*>(st + ((wr * RI + i) * PT2_KC + q) * 1024 + lane * 16);
#pragma unroll
        for (int j = 0; j < 2; ++j)
          fb[j] = *reinterpret_cast<const u32x4*>(st + A_BYTES + (q * 4 + wc * 2 + j) * 1024 + lane * 16);
#pragma unroll
        for (int i = 0; i < RI; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(fa[i]), as_frag(fb[j]), acc[i][j], 0, 0, 0);
      }
    }
    if (more) sstore(stage ^ 1);
    stage ^= 1;
    __syncthreads();
  }

  // epilogue: each wave stages 64 x 64 of its tile at a time through its own LDS region (fp32, padded
  // rows) and stores 16-byte chunks along rows.  Block (i, j): register v of lane (li, lh) is row
  // 32 i + 8 (v / 4) + 4 lh + v % 4, column 32 j + li of the wave tile.
  float* tile = reinterpret_cast<float*>(pt_smem) + wave * (64 * PT2_ELD);
  const int er = lane >> 3, ec = (lane & 7) * 8;  // 8 lanes per row, 8 rows per step
#pragma unroll
  for (int p = 0; p < RI / 2; ++p) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          tile[(32 * i + 8 * (v / 4) + 4 * lh + (v % 4)) * PT2_ELD + 32 * j + li] = acc[2 * p + i][j][v];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int row = er + 8 * q;
      const int grow = tm * TM + wr * (TM / 2) + p * 64 + row, gcol = tn * 128 + wc * 64 + ec;
      const float4 lo = *reinterpret_cast<const float4*>(tile + row * PT2_ELD + ec);
      const float4 hi = *reinterpret_cast<const float4*>(tile + row * PT2_ELD + ec + 4);
      if (grow >= a.d || gcol >= om) continue;
      float x[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      if (OUT_BF16) {
        bf16_t* o = reinterpret_cast<bf16_t*>(odW) + (int64_t)grow * olddw + gcol;
        if (ovec && gcol + 8 <= om) {
          if (a.beta != 0.f) {
            const u32x4 old = *reinterpret_cast<const u32x4*>(o);
#pragma unroll
            for (int e = 0; e < 8; ++e)
              x[e] += a.beta * __uint_as_float(((e & 1) ? (old[e >> 1] >> 16) : (old[e >> 1] & 0xFFFFu)) << 16);
          }
          u32x4 w;
          w.x = pack2_hw(x[0], x[1]);
          w.y = pack2_hw(x[2], x[3]);
          w.z = pack2_hw(x[4], x[5]);
          w.w = pack2_hw(x[6], x[7]);
          stream_store(reinterpret_cast<u32x4*>(o), w);
        } else {
          for (int e = 0; e < 8 && gcol + e < om; ++e)
            o[e] = f32_to_bf16(a.beta == 0.f ? x[e] : x[e] + a.beta * __uint_as_float(((uint32_t)o[e]) << 16));
        }
      } else {
        float* o = reinterpret_cast<float*>(odW) + (int64_t)grow * olddw + gcol;
        if (ovec && gcol + 8 <= om) {
          if (a.beta != 0.f) {
            const float4 o0 = *reinterpret_cast<const float4*>(o), o1 = *reinterpret_cast<const float4*>(o + 4);
            x[0] += a.beta * o0.x; x[1] += a.beta * o0.y; x[2] += a.beta * o0.z; x[3] += a.beta * o0.w;
            x[4] += a.beta * o1.x; x[5] += a.beta * o1.y; x[6] += a.beta * o1.z; x[7] += a.beta * o1.w;
          }
          stream_store(reinterpret_cast<f32x4_t*>(o), f32x4_t{x[0], x[1], x[2], x[3]});
          stream_store(reinterpret_cast<f32x4_t*>(o + 4), f32x4_t{x[4], x[5], x[6], x[7]});
        } else {
          for (int e = 0; e < 8 && gcol + e < om; ++e) o[e] = a.beta == 0.f ? x[e] : x[e] + a.beta * o[e];
        }
      }
    }
  }
}

// ---------------------------------------------- dW = P (sum of the slabs), one launch
// The slab sum and dW = P T as one kernel, without T ever leaving the compute unit: a workgroup owns
// 32 columns of one output and a range of at most SP_RBW 32-row blocks of dW.  It sums the token-split
// partial slabs of its 32 columns of T (in slab order, rows >= k_lo weighted by the scaling factor,
// rounded to bf16: the same arithmetic in the same order as reduce_to_tfrag_kernel) into LDS in
// fragment order, 256 rows of T at a time, and multiplies: each of the 8 waves holds up to two
// 32 x 32 tiles of dW, the fragments of P come straight from L2 and are requested before the sum
// starts.  The workgroups that share a column block (the row ranges) sum the same slabs again; they
// sit next to each other on one XCD, so the slabs cross the fabric once and the repeats are L2 hits.
// What this buys over the two kernels: one launch, and no round trip of T through memory between them.
constexpr int SP_KC = 16;                   // k-blocks of T in LDS at a time
constexpr int SP_RBW = 16;                  // 32-row blocks of dW per workgroup at most
constexpr int SP_SLD = 36;                  // floats per row of a wave's 32 x 32 output staging tile
constexpr int SP_T_BYTES = SP_KC * 1024;
constexpr int SP_SMEM = SP_T_BYTES + 8 * 32 * SP_SLD * 4;
constexpr int SP_ZB = 4;                    // slabs requested together

struct SumPtArgs {
  int n_out, splits, c, k_lo, nkb;
  float scale_hi, beta;
  const bf16_t* Pa;  // [nrb_pa][nkb][64][8]
  int d, nrb_pa;
  int row_parts, rb_per_part;
  int cblks;         // 32-column blocks over all outputs
  const float* slabs[PRAC_CTDY_MAX_OUT];  // [splits][c][m_h]
  void* dW[PRAC_CTDY_MAX_OUT];
  int64_t lddw[PRAC_CTDY_MAX_OUT];
  int m[PRAC_CTDY_MAX_OUT];
  int vec_ok[PRAC_CTDY_MAX_OUT];
  int cblk0[PRAC_CTDY_MAX_OUT + 1];       // first column block of output h in the launch
};

template <bool OUT_BF16>
__global__ __launch_bounds__(512) void sum_pt_kernel(SumPtArgs a) {
  extern __shared__ __align__(16) unsigned char sp_smem[];
  const int bid = touch_kernel_args<sizeof(SumPtArgs)>(blockIdx.x);
  const int total = a.cblks * a.row_parts;
  const int per_xcd = (total + 7) / 8;
  const int xcd = bid & 7, slot = bid >> 3;
  const int logical = xcd * per_xcd + slot;
  if (slot >= per_xcd || logical >= total) return;
  const int cbg = logical / a.row_parts, rp = logical % a.row_parts;
  int h = 0;
#pragma unroll
  for (int q = 1; q < PRAC_CTDY_MAX_OUT; ++q)
    if (q < a.n_out && cbg >= a.cblk0[q]) h = q;
  const int n0 = (cbg - a.cblk0[h]) * 32;
  const float* __restrict__ slabs = a.slabs[h];
  const int mh = a.m[h], c = a.c, splits = a.splits, nkb = a.nkb;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 31, lh = lane >> 5;
  const int nrb = (a.d + 31) / 32;
  const int rb_end = min((rp + 1) * a.rb_per_part, nrb);
  const int rbA = rp * a.rb_per_part + wave, rbB = rbA + 8;
  const bool hasA = rbA < rb_end, hasB = rbB < rb_end;  // wave-uniform
  const u32x4* __restrict__ PaA = reinterpret_cast<const u32x4*>(a.Pa) + (int64_t)min(rbA, a.nrb_pa - 1) * nkb * 64 + lane;
  const u32x4* __restrict__ PaB = reinterpret_cast<const u32x4*>(a.Pa) + (int64_t)min(rbB, a.nrb_pa - 1) * nkb * 64 + lane;

  f32x16 accA, accB;
#pragma unroll
  for (int v = 0; v < 16; ++v) accA[v] = accB[v] = 0.f;

  // summing: thread (pr, col4) takes rows 2 pr, 2 pr + 1 (+ 128) of the chunk and 4 columns
  const int pr = tid >> 3, col4 = (tid & 7) * 4, n = n0 + col4;
  const int64_t slab = (int64_t)c * mh;
  const int nchunks = (nkb + SP_KC - 1) / SP_KC;
#pragma nounroll
  for (int ch = 0; ch < nchunks; ++ch) {
    const int kb0 = ch * SP_KC;
    // the fragments of P do not depend on T: the first tile's are requested before the sum starts, the
    // second tile's once the sum's registers are free
    u32x4 fa[SP_KC];
#pragma unroll
    for (int q = 0; q < SP_KC; ++q) fa[q] = PaA[(int64_t)min(kb0 + q, nkb - 1) * 64];
    if (ch > 0) __syncthreads();  // the previous chunk of T has been multiplied
    // rows kl, kl + 1 of the chunk, 4 columns: into fragment order (row 16 kb + 8 hh + e of T, column j ->
    // lane 32 hh + j, element e; the two rows are the elements e, e + 1, e even, of one 32-bit word)
    auto put = [&](int q2, float4 s0, float4 s1) {
      const int kl = 128 * q2 + 2 * pr, k = kb0 * 16 + kl;
      if (k >= c || n >= mh) s0 = make_float4(0.f, 0.f, 0.f, 0.f);
      if (k + 1 >= c || n >= mh) s1 = make_float4(0.f, 0.f, 0.f, 0.f);
      const float w0 = k >= a.k_lo ? a.scale_hi : 1.f, w1 = k + 1 >= a.k_lo ? a.scale_hi : 1.f;
      unsigned char* t = sp_smem + (kl >> 4) * 1024 + (((kl >> 3) & 1) * 32 + col4) * 16 + ((kl & 7) >> 1) * 4;
      *reinterpret_cast<uint32_t*>(t) = pack2_hw(s0.x * w0, s1.x * w1);
      *reinterpret_cast<uint32_t*>(t + 16) = pack2_hw(s0.y * w0, s1.y * w1);
      *reinterpret_cast<uint32_t*>(t + 32) = pack2_hw(s0.z * w0, s1.z * w1);
      *reinterpret_cast<uint32_t*>(t + 48) = pack2_hw(s0.w * w0, s1.w * w1);
    };
    {
      // SP_ZB slabs of a row pair per batch, the next batch requested before this one is summed, so that
      // the memory round trips of a thread's 4 x splits loads overlap (the launcher sends only column
      // counts that are multiples of 4 and slab counts that are multiples of SP_ZB here).  Threads whose
      // rows or columns lie outside T read a valid element instead and store zeros.
      const int nzf = splits / SP_ZB, nb = 2 * nzf;
      const int k0 = kb0 * 16 + 2 * pr, k1 = k0 + 128;
      const float* const pb0 = slabs + (int64_t)min(k0, c - 1) * mh + min(n, mh - 4);
      const float* const pb1 = slabs + (int64_t)min(k1, c - 1) * mh + min(n, mh - 4);
      const int64_t st0 = k0 + 1 < c ? mh : 0, st1 = k1 + 1 < c ? mh : 0;
      auto issue = [&](int b, float4 (&v0)[SP_ZB], float4 (&v1)[SP_ZB]) {
        const bool hi = b >= nzf;
        const float* p0 = (hi ? pb1 : pb0) + (int64_t)((hi ? b - nzf : b) * SP_ZB) * slab;
        const float* p1 = p0 + (hi ? st1 : st0);
#pragma unroll
        for (int z = 0; z < SP_ZB; ++z) {
          v0[z] = *reinterpret_cast<const float4*>(p0 + z * slab);
          v1[z] = *reinterpret_cast<const float4*>(p1 + z * slab);
        }
      };
      float4 s0 = make_float4(0.f, 0.f, 0.f, 0.f), s1 = s0;
      auto add = [&](int b, const float4 (&v0)[SP_ZB], const float4 (&v1)[SP_ZB]) {
#pragma unroll
        for (int z = 0; z < SP_ZB; ++z) {
          s0.x += v0[z].x; s0.y += v0[z].y; s0.z += v0[z].z; s0.w += v0[z].w;
          s1.x += v1[z].x; s1.y += v1[z].y; s1.z += v1[z].z; s1.w += v1[z].w;
        }
        if (b == nzf - 1 || b == nb - 1) {  // the row pair's last batch
          put(b >= nzf ? 1 : 0, s0, s1);
          s0 = make_float4(0.f, 0.f, 0.f, 0.f);
          s1 = s0;
        }
      };
      float4 va0[SP_ZB], va1[SP_ZB], vb0[SP_ZB], vb1[SP_ZB];
      issue(0, va0, va1);
#pragma nounroll
      for (int b = 0; b < nb; b += 2) {
        issue(b + 1, vb0, vb1);
        add(b, va0, va1);
        issue(min(b + 2, nb - 1), va0, va1);  // past the end: the last batch again, not summed
        add(b + 1, vb0, vb1);
      }
    }
    __syncthreads();
    {
      u32x4 fb[SP_KC];
      if (hasB) {
#pragma unroll
        for (int q = 0; q < SP_KC; ++q) fb[q] = PaB[(int64_t)min(kb0 + q, nkb - 1) * 64];
      }
      // all SP_KC k-blocks of the chunk, also past the last row of T: those fragments of T are zeros
      // (put), the fragments of P repeat the last k-block
      if (hasA) {
#pragma unroll
        for (int q = 0; q < SP_KC; ++q)
          accA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              as_frag(fa[q]), as_frag(*reinterpret_cast<const u32x4*>(sp_smem + q * 1024 + lane * 16)), accA, 0, 0, 0);
      }
      if (hasB) {
#pragma unroll
        for (int q = 0; q < SP_KC; ++q)
          accB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              as_frag(fb[q]), as_frag(*reinterpret_cast<const u32x4*>(sp_smem + q * 1024 + lane * 16)), accB, 0, 0, 0);
      }
    }
  }

  // register v of lane (li, lh) is row 8 (v / 4) + 4 lh + v % 4, column li of the tile: through this
  // wave's own LDS tile, so that the stores are 16 bytes per lane along rows
  float* stage = reinterpret_cast<float*>(sp_smem + SP_T_BYTES) + wave * (32 * SP_SLD);
  void* const odW = a.dW[h];
  const int64_t olddw = a.lddw[h];
  const int ovec = a.vec_ok[h];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    if (!(t == 0 ? hasA : hasB)) continue;
    const f32x16& acc = t == 0 ? accA : accB;
    const int row0 = (t == 0 ? rbA : rbB) * 32;
#pragma unroll
    for (int v = 0; v < 16; ++v) stage[(8 * (v / 4) + 4 * lh + (v % 4)) * SP_SLD + li] = acc[v];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if (OUT_BF16) {
      const int er = lane >> 2, ec = (lane & 3) * 8;  // 4 lanes per row (16 bytes each), 16 rows per pass
#pragma unroll
      for (int p = 0; p < 2; ++p) {
        const int row = er + 16 * p, grow = row0 + row, gcol = n0 + ec;
        const float4 lo = *reinterpret_cast<const float4*>(stage + row * SP_SLD + ec);
        const float4 hi = *reinterpret_cast<const float4*>(stage + row * SP_SLD + ec + 4);
        if (grow >= a.d || gcol >= mh) continue;
        float x[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
        bf16_t* o = reinterpret_cast<bf16_t*>(odW) + (int64_t)grow * olddw + gcol;
        if (ovec && gcol + 8 <= mh) {
          if (a.beta != 0.f) {
            const u32x4 old = *reinterpret_cast<const u32x4*>(o);
#pragma unroll
            for (int e = 0; e < 8; ++e)
              x[e] += a.beta * __uint_as_float(((e & 1) ? (old[e >> 1] >> 16) : (old[e >> 1] & 0xFFFFu)) << 16);
          }
          u32x4 w;
          w.x = pack2_hw(x[0], x[1]);
          w.y = pack2_hw(x[2], x[3]);
          w.z = pack2_hw(x[4], x[5]);
          w.w = pack2_hw(x[6], x[7]);
          stream_store(reinterpret_cast<u32x4*>(o), w);
        } else {
          for (int e = 0; e < 8 && gcol + e < mh; ++e)
            o[e] = f32_to_bf16(a.beta == 0.f ? x[e] : x[e] + a.beta * __uint_as_float(((uint32_t)o[e]) << 16));
        }
      }
    } else {
      const int er = lane >> 3, ec = (lane & 7) * 4;  // 8 lanes per row (16 bytes each), 8 rows per pass
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const int row = er + 8 * p, grow = row0 + row, gcol = n0 + ec;
        float4 x = *reinterpret_cast<const float4*>(stage + row * SP_SLD + ec);
        if (grow >= a.d || gcol >= mh) continue;
        float* o = reinterpret_cast<float*>(odW) + (int64_t)grow * olddw + gcol;
        if (ovec && gcol + 4 <= mh) {
          if (a.beta != 0.f) {
            const float4 old = *reinterpret_cast<const float4*>(o);
            x.x += a.beta * old.x; x.y += a.beta * old.y; x.z += a.beta * old.z; x.w += a.beta * old.w;
          }
          stream_store(reinterpret_cast<f32x4_t*>(o), f32x4_t{x.x, x.y, x.z, x.w});
        } else {
          const float xs[4] = {x.x, x.y, x.z, x.w};
          for (int e = 0; e < 4 && gcol + e < mh; ++e) o[e] = a.beta == 0.f ? xs[e] : xs[e] + a.beta * o[e];
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
}

inline int grid_for(int64_t n, int n_cu) {
  int64_t g = (n + 255) / 256;
  const int64_t cap = (int64_t)n_cu * 8;
  if (g > cap) g = cap;
  return g < 1 ? 1 : (int)g;
}

template <typename K>
int set_smem(prac_ctx* ctx, K kern, size_t bytes, bool& done) {
  if (!done) {
    PRAC_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    done = true;
  }
  return PRAC_OK;
}

}  // namespace

int launch_pack_pfrag(prac_ctx* ctx, const float* P, int64_t d, int64_t ldp, int c, int nkb, int ncb, bf16_t* out) {
  hipLaunchKernelGGL(pack_pfrag_kernel, dim3(grid_for((int64_t)nkb * ncb * 64, ctx->n_cu)), dim3(256), 0, ctx->stream,
                     P, d, ldp, c, nkb, ncb, out);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

int launch_pack_wfrag(prac_ctx* ctx, const bf16_t* W, int64_t ldw, int w_layout, int64_t d, int m, int nkb,
                      int ncb_w, bf16_t* out) {
  hipLaunchKernelGGL(pack_wfrag_kernel, dim3(grid_for((int64_t)nkb * ncb_w * 64, ctx->n_cu)), dim3(256), 0,
                     ctx->stream, W, ldw, w_layout, d, m, nkb, ncb_w, out);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

int launch_pack_ptfrag(prac_ctx* ctx, const float* P, int64_t d, int64_t ldp, int c, int k_lo, float scale_hi,
                       int nkb, int ncb, bf16_t* out) {
  hipLaunchKernelGGL(pack_ptfrag_kernel, dim3(grid_for((int64_t)nkb * ncb * 64, ctx->n_cu)), dim3(256), 0, ctx->stream,
                     P, d, ldp, c, k_lo, scale_hi, nkb, ncb, out);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

int launch_unpack_c(prac_ctx* ctx, const bf16_t* Cpk, int N, int c, bf16_t* C, int64_t ldc) {
  const int ccb = (c + 31) / 32;
  hipLaunchKernelGGL(unpack_c_kernel, dim3(grid_for((int64_t)((N + 15) / 16) * ccb * 64, ctx->n_cu)), dim3(256), 0,
                     ctx->stream, Cpk, N, c, ccb, C, ldc);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

int launch_pack_c(prac_ctx* ctx, const bf16_t* C, int64_t ldc, int N, int c, bf16_t* Cpk) {
  const int ccb = (c + 31) / 32;
  hipLaunchKernelGGL(pack_c_kernel, dim3(grid_for((int64_t)((N + 127) / 128) * 8 * ccb * 64, ctx->n_cu)), dim3(256), 0,
                     ctx->stream, C, ldc, N, c, ccb, Cpk);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

int launch_reduce_to_tfrag(prac_ctx* ctx, int n_out, const float* const* slabs, int splits, int c, const int* m, int k_lo,
                           float scale_hi, int nkb, const int* nmb, bf16_t* const* Tf) {
  if (n_out < 1 || n_out > PRAC_CTDY_MAX_OUT) return PRAC_EINVAL;
  ReduceTfArgs a{};
  a.n_out = n_out; a.splits = splits; a.c = c; a.k_lo = k_lo; a.nkb = nkb; a.scale_hi = scale_hi;
  int pairs = 0;
  for (int h = 0; h < n_out; ++h) {
    a.slabs[h] = slabs[h]; a.Tf[h] = Tf[h]; a.m[h] = m[h]; a.nmb[h] = nmb[h];
    a.pair0[h] = pairs;
    pairs += nmb[h] / 2;
  }
  for (int h = n_out; h <= PRAC_CTDY_MAX_OUT; ++h) a.pair0[h] = pairs;
  PRAC_LAUNCH(ctx, reduce_to_tfrag_kernel, dim3(nkb * pairs), dim3(256), 0, a);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

int launch_pack_pafrag(prac_ctx* ctx, const float* P, int64_t d, int64_t ldp, int c, int nrb, int nkb, bf16_t* out) {
  hipLaunchKernelGGL(pack_pafrag_kernel, dim3(grid_for((int64_t)nrb * nkb * 64, ctx->n_cu)), dim3(256), 0, ctx->stream,
                     P, d, ldp, c, nrb, nkb, out);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

int launch_pt(prac_ctx* ctx, const bf16_t* Pa, int n_out, const bf16_t* const* Tf, int d, const int* m, int nkb,
              const int* nmb, void* const* dW, const int64_t* lddw, bool out_bf16, float beta) {
  if (n_out < 1 || n_out > PRAC_CTDY_MAX_OUT) return PRAC_EINVAL;
  PtArgs a{};
  a.Pa = Pa; a.d = d; a.nkb = nkb; a.beta = beta; a.n_out = n_out;
  a.tiles_m_rb = ((d + 127) / 128) * 4;
  int tiles = 0;
  for (int h = 0; h < n_out; ++h) {
    a.Tf[h] = Tf[h]; a.dW[h] = dW[h]; a.lddw[h] = lddw[h]; a.m[h] = m[h]; a.nmb[h] = nmb[h];
    a.vec_ok[h] = (reinterpret_cast<uintptr_t>(dW[h]) % 16 == 0 && lddw[h] % (out_bf16 ? 8 : 4) == 0) ? 1 : 0;
    a.tile0[h] = tiles;
    tiles += (m[h] + 127) / 128;
  }
  for (int h = n_out; h <= PRAC_CTDY_MAX_OUT; ++h) a.tile0[h] = tiles;
  a.tiles_n = tiles;
  // the direct kernel for a single round of short products, the LDS-staged one otherwise (measured:
  // 21 against 26 us at d = 2048, m = 5461, c = 256; 95 against 117 us at d = 4096, m = 11008, c = 512)
  a.tiles_m = (d + 127) / 128;
  const int total = a.tiles_m * a.tiles_n;
  const bool tiled = total > ctx->n_cu || nkb > PT_PD;
  const dim3 grid(((total + 7) / 8) * 8), block(256);
  const size_t smem = !tiled ? (size_t)128 * PT_TLD * sizeof(float)
                             : std::max((size_t)2 * (128 / 32 + 4) * PT2_KC * 1024, (size_t)4 * 64 * PT2_ELD * sizeof(float));
  static bool done_dev[PRAC_MAX_DEVICES][4] = {};  // the attribute is per device
  bool* done = done_dev[ctx->device % PRAC_MAX_DEVICES];
  const int idx = (tiled ? 2 : 0) + (out_bf16 ? 1 : 0);
#define PRAC_PT_CASE(I, KERN)                          \
  case I: {                                            \
    constexpr auto kern = KERN;                        \
    int rc = set_smem(ctx, kern, smem, done[I]);       \
    if (rc) return rc;                                 \
    PRAC_LAUNCH(ctx, kern, grid, block, smem, a);      \
    break;                                             \
  }
  switch (idx) {
    PRAC_PT_CASE(0, pt_kernel<false>)
    PRAC_PT_CASE(1, pt_kernel<true>)
    PRAC_PT_CASE(2, (pt_tiled_kernel<128, false>))
    PRAC_PT_CASE(3, (pt_tiled_kernel<128, true>))
  }
#undef PRAC_PT_CASE
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

// Row ranges of the one-launch slab sum + P T: at most SP_RBW 32-row blocks per workgroup; more, smaller
// ranges when the launch would otherwise leave compute units idle (the repeated slab sums are cheap then).
int sum_pt_row_parts(int n_cu, int d, int n_out, const int* m) {
  const int nrb = (d + 31) / 32;
  int cblks = 0;
  for (int h = 0; h < n_out; ++h) cblks += (m[h] + 31) / 32;
  int parts = (nrb + SP_RBW - 1) / SP_RBW;
  const int fill = n_cu / (cblks > 0 ? cblks : 1);
  if (fill > parts) parts = fill < nrb ? fill : nrb;
  return parts;
}

// The one-launch form covers column counts that are multiples of 4 (16-byte slab loads) and slab counts that
// are multiples of SP_ZB (whole batches); everything else runs as the two launches.
bool sum_pt_eligible(int n_out, const int* m, int splits) {
  if (n_out < 1 || n_out > PRAC_CTDY_MAX_OUT || splits < SP_ZB || splits % SP_ZB != 0) return false;
  for (int h = 0; h < n_out; ++h)
    if (m[h] < 4 || (m[h] & 3) != 0) return false;
  return true;
}

int launch_sum_pt(prac_ctx* ctx, const bf16_t* Pa, int n_out, const float* const* slabs, int splits, int c, int k_lo,
                  float scale_hi, int nkb, int d, const int* m, void* const* dW, const int64_t* lddw, bool out_bf16,
                  float beta) {
  if (!sum_pt_eligible(n_out, m, splits)) return PRAC_EINVAL;
  SumPtArgs a{};
  a.n_out = n_out; a.splits = splits; a.c = c; a.k_lo = k_lo; a.nkb = nkb; a.scale_hi = scale_hi; a.beta = beta;
  a.Pa = Pa; a.d = d; a.nrb_pa = ((d + 127) / 128) * 4;
  const int nrb = (d + 31) / 32;
  const int parts = sum_pt_row_parts(ctx->n_cu, d, n_out, m);
  a.rb_per_part = (nrb + parts - 1) / parts;
  a.row_parts = (nrb + a.rb_per_part - 1) / a.rb_per_part;
  if (a.rb_per_part > SP_RBW) return PRAC_EINVAL;
  int cblks = 0;
  for (int h = 0; h < n_out; ++h) {
    a.slabs[h] = slabs[h]; a.dW[h] = dW[h]; a.lddw[h] = lddw[h]; a.m[h] = m[h];
    a.vec_ok[h] = (reinterpret_cast<uintptr_t>(dW[h]) % 16 == 0 && lddw[h] % (out_bf16 ? 8 : 4) == 0) ? 1 : 0;
    a.cblk0[h] = cblks;
    cblks += (m[h] + 31) / 32;
  }
  for (int h = n_out; h <= PRAC_CTDY_MAX_OUT; ++h) a.cblk0[h] = cblks;
  a.cblks = cblks;
  const int64_t total = (int64_t)cblks * a.row_parts;
  if (total > (1 << 28)) return PRAC_EINVAL;
  const dim3 grid((unsigned)(((total + 7) / 8) * 8)), block(512);
  static bool done_dev[PRAC_MAX_DEVICES][2] = {};
  bool* done = done_dev[ctx->device % PRAC_MAX_DEVICES];
  if (out_bf16) {
    int rc = set_smem(ctx, sum_pt_kernel<true>, (size_t)SP_SMEM, done[1]);
    if (rc) return rc;
    PRAC_LAUNCH(ctx, sum_pt_kernel<true>, grid, block, (size_t)SP_SMEM, a);
  } else {
    int rc = set_smem(ctx, sum_pt_kernel<false>, (size_t)SP_SMEM, done[0]);
    if (rc) return rc;
    PRAC_LAUNCH(ctx, sum_pt_kernel<false>, grid, block, (size_t)SP_SMEM, a);
  }
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

