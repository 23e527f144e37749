// The two streaming contractions of the per-step path, specialised for gfx950.
//
//   compress   C = X P          (Alg. 1 compression step)     compress_panel_kernel
//   C^T dY     token-split partial sums of T = C^T dY (Lemma 1, reassociated)  ctdy_kernel
//
// Both are HBM-bound at PRAC's ranks (c = k + r << d), so the design goal is to read the
// big operand (X, dY) exactly once, keep LDS traffic below the MFMA time and keep many
// bytes in flight.  The small operand never goes through LDS: it is stored in HBM in
// MFMA fragment order, so a wave fetches a whole 32x16 operand block with one fully
// coalesced 1 KB load.
//
// Fragment order ("frag16x32"), used for P (B operand of compress) and for the packed
// compressed activation C (A operand of C^T dY): a block of 16 reduction indices x 32
// rows/columns is 64 lanes x 8 bf16; lane = 32 h + j holds, for row/column j, the
// reduction indices listed by slot(h, e), e = 0..7.
//   P:  slot(h, e) = 8 h + e                         (k = 16 kb + 8 h + e)
//   C:  slot(h, e) = 4 h + e (e < 4), 8 + 4 h + e - 4 (e >= 4)   (token = 16 tb + slot)
// The C order is the order in which the 32x32 MFMA accumulator of compress holds its
// rows, so compress stores a packed block straight from its registers.
#include "prac_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

__device__ __forceinline__ uint4 load_chunk(const bf16_t* p, int n_valid) {
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  if (n_valid >= 8) {
    v = *reinterpret_cast<const uint4*>(p);
  } else if (n_valid > 0) {
    bf16_t t[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) t[e] = e < n_valid ? p[e] : (bf16_t)0;
    v.x = t[0] | ((uint32_t)t[1] << 16);
    v.y = t[2] | ((uint32_t)t[3] << 16);
    v.z = t[4] | ((uint32_t)t[5] << 16);
    v.w = t[6] | ((uint32_t)t[7] << 16);
  }
  return v;
}

__device__ __forceinline__ bf16x8 as_frag(uint4 v) {
  union {
    uint4 u;
    bf16x8 f;
  } c;
  c.u = v;
  return c.f;
}

// ------------------------------------------------------------------ compress
struct CompressArgs {
  const bf16_t* X;
  int64_t ldx;
  int N, d;
  const bf16_t* Pfrag;  // [d64/16][ncb][64][8]
  int ncb;              // 32-column blocks in the padded basis (multiple of 4*FN)
  int c;
  bf16_t* C;            // row-major (ldc) or packed [Npad/16][ccb][64][8]
  int64_t ldc;
  int ccb;              // 32-column blocks of packed C = ceil(c / 32)
  int packed;
  int tiles_m;
  int col_groups;       // column groups of 4*FN blocks
};

constexpr int CP_BM = 128, CP_BK = 64, CP_LD = CP_BK + 8, CP_STAGES = 3;

// 256 threads = 4 waves.  The workgroup owns 128 token rows; wave w owns the 32*FN
// columns [32 FN w, 32 FN (w+1)) of its column group and all 128 rows.  X tiles go
// global -> registers -> LDS (3-stage ring, loads issued two tiles ahead); P fragments
// go global -> registers one tile ahead.
template <int FN>
__global__ __launch_bounds__(256) void compress_panel_kernel(CompressArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);
  constexpr int STAGE = CP_BM * CP_LD;
  constexpr int A_CH = CP_BM * (CP_BK / 8) / 256;  // 4 chunks of 16 B per thread and tile
  constexpr int KK = CP_BK / 16;

  // XCD-aware order: consecutive logical tiles (same rows, next column group) on one XCD
  const int total = a.tiles_m * a.col_groups;
  const int per_xcd = (total + 7) / 8;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int logical = xcd * per_xcd + slot;
  if (slot >= per_xcd || logical >= total) return;
  const int cg = logical % a.col_groups, tm = logical / a.col_groups;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 31, lh = lane >> 5;
  const int m0 = tm * CP_BM;
  const int cb0 = cg * 4 * FN + wave * FN;  // first 32-column block of this wave
  const int nk = (a.d + CP_BK - 1) / CP_BK;
  const bf16_t* __restrict__ X = a.X;
  const uint4* __restrict__ Pf = reinterpret_cast<const uint4*>(a.Pfrag);

  f32x16 acc[4][FN];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  uint4 ra[2][A_CH];
  uint4 rb[2][KK * FN];

  auto gload_a = [&](int kt, uint4 (&r)[A_CH]) {
    const int k0 = kt * CP_BK;
#pragma unroll
    for (int p = 0; p < A_CH; ++p) {
      const int q = tid + p * 256, row = q >> 3, cc = (q & 7) * 8;
      const int m = m0 + row, k = k0 + cc;
      r[p] = load_chunk(X + (int64_t)m * a.ldx + k, m < a.N ? a.d - k : 0);
    }
  };
  auto sstore_a = [&](int stage, const uint4 (&r)[A_CH]) {
    bf16_t* s = smem + stage * STAGE;
#pragma unroll
    for (int p = 0; p < A_CH; ++p) {
      const int q = tid + p * 256, row = q >> 3, cc = (q & 7) * 8;
      *reinterpret_cast<uint4*>(s + row * CP_LD + cc) = r[p];
    }
  };
  auto gload_b = [&](int kt, uint4 (&r)[KK * FN]) {
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
#pragma unroll
      for (int j = 0; j < FN; ++j)
        r[kk * FN + j] = Pf[((int64_t)(kt * KK + kk) * a.ncb + cb0 + j) * 64 + lane];
  };
  auto compute = [&](int stage, const uint4 (&b)[KK * FN]) {
    const bf16_t* s = smem + stage * STAGE;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      bf16x8 fa[4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        fa[i] = *reinterpret_cast<const bf16x8*>(s + (i * 32 + li) * CP_LD + kk * 16 + lh * 8);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], as_frag(b[kk * FN + j]), acc[i][j], 0, 0, 0);
    }
  };

  // prologue: tile 0 into LDS stage 0, tile 1 (A) in registers, B of tile 0 in registers
  gload_a(0, ra[0]);
  gload_b(0, rb[0]);
  if (nk > 1) gload_a(1, ra[1]);
  sstore_a(0, ra[0]);
  __syncthreads();

  // steady state at iteration kt: stage kt%3 holds tile kt; ra[(kt+1)&1] holds tile kt+1
  for (int kt = 0; kt < nk; kt += 2) {
    // even half: kt
    if (kt + 1 < nk) sstore_a((kt + 1) % CP_STAGES, ra[1]);
    if (kt + 2 < nk) gload_a(kt + 2, ra[0]);
    if (kt + 1 < nk) gload_b(kt + 1, rb[1]);
    compute(kt % CP_STAGES, rb[0]);
    __syncthreads();
    // odd half: kt + 1
    if (kt + 1 < nk) {
      if (kt + 2 < nk) sstore_a((kt + 2) % CP_STAGES, ra[0]);
      if (kt + 3 < nk) gload_a(kt + 3, ra[1]);
      if (kt + 2 < nk) gload_b(kt + 2, rb[0]);
      compute((kt + 1) % CP_STAGES, rb[1]);
      __syncthreads();
    }
  }

  // epilogue: block (i, j) register v of lane (li, lh) is token row 8*(v/4) + 4*lh + v%4
  // of row block i, column li of column block cb0 + j.
  if (a.packed) {
    // registers v = 8 tb .. 8 tb + 7 are exactly the 8 slots of the 16-token block tb
    uint4* Cp = reinterpret_cast<uint4*>(a.C);
    const int ntb = (a.N + 15) / 16;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
          const int gtb = (m0 + i * 32) / 16 + tb, cb = cb0 + j;
          if (gtb < ntb && cb < a.ccb) {
            uint4 o;
            o.x = pack2(acc[i][j][8 * tb + 0], acc[i][j][8 * tb + 1]);
            o.y = pack2(acc[i][j][8 * tb + 2], acc[i][j][8 * tb + 3]);
            o.z = pack2(acc[i][j][8 * tb + 4], acc[i][j][8 * tb + 5]);
            o.w = pack2(acc[i][j][8 * tb + 6], acc[i][j][8 * tb + 7]);
            Cp[((int64_t)gtb * a.ccb + cb) * 64 + lane] = o;
          }
        }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int m = m0 + i * 32 + 8 * (v / 4) + 4 * lh + (v % 4);
          const int n = (cb0 + j) * 32 + li;
          if (m < a.N && n < a.c) a.C[(int64_t)m * a.ldc + n] = f32_to_bf16(acc[i][j][v]);
        }
  }
}

// -------------------------------------------------------------------- C^T dY
struct CtdyArgs {
  const bf16_t* Cpk;   // packed compressed activation [ntb][ccb][64][8]
  int ccb;             // 32-column blocks of C
  int c;
  const bf16_t* dY;
  int64_t lddy;
  int N, m;
  float* slabs;        // [splits][c][m]
  int splits;
  int tok_per_split;   // multiple of CT_BK
  int tiles_n;         // column tiles of 128 over m
  int row_groups;      // groups of 8 column blocks (256 rows of T) over c
};

constexpr int CT_BN = 128, CT_BK = 64, CT_LD = CT_BN + 8, CT_STAGES = 3;

// 256 threads = 4 waves.  The workgroup owns 256 rows of T (columns of C) x 128 columns
// (of dY) for one token range; wave w owns rows [64 w, 64 w + 64).  C fragments come
// straight from the packed layout; dY tiles are staged in LDS as they lie in memory
// ([token][column]) and turned into fragments by an in-register 8 x 4 transpose.
__global__ __launch_bounds__(256) void ctdy_kernel(CtdyArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);
  constexpr int STAGE = CT_BK * CT_LD;
  constexpr int B_CH = CT_BK * (CT_BN / 8) / 256;  // 4
  constexpr int KK = CT_BK / 16;

  const int per_split = a.tiles_n * a.row_groups;
  const int total = per_split * a.splits;
  const int per_xcd = (total + 7) / 8;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int logical = xcd * per_xcd + slot;
  if (slot >= per_xcd || logical >= total) return;
  const int tn = logical % a.tiles_n;
  const int rg = (logical / a.tiles_n) % a.row_groups;
  const int split = logical / per_split;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 31, lh = lane >> 5;
  const int n0 = tn * CT_BN;
  const int cb0 = rg * 8 + wave * 2;
  const int tok_beg = split * a.tok_per_split;
  const int tok_end = min(a.N, tok_beg + a.tok_per_split);
  const int nk = (tok_end - tok_beg + CT_BK - 1) / CT_BK;
  const int ntb = (a.N + 15) / 16;
  const uint4* __restrict__ Cp = reinterpret_cast<const uint4*>(a.Cpk);
  const bf16_t* __restrict__ dY = a.dY;

  f32x16 acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  uint4 rb[2][B_CH];
  uint4 rafr[2][KK * 2];

  auto gload_b = [&](int kt, uint4 (&r)[B_CH]) {
    const int t0 = tok_beg + kt * CT_BK;
#pragma unroll
    for (int p = 0; p < B_CH; ++p) {
      const int q = tid + p * 256, row = q >> 4, cc = (q & 15) * 8;
      const int t = t0 + row, n = n0 + cc;
      r[p] = load_chunk(dY + (int64_t)t * a.lddy + n, t < tok_end ? a.m - n : 0);
    }
  };
  auto sstore_b = [&](int stage, const uint4 (&r)[B_CH]) {
    bf16_t* s = smem + stage * STAGE;
#pragma unroll
    for (int p = 0; p < B_CH; ++p) {
      const int q = tid + p * 256, row = q >> 4, cc = (q & 15) * 8;
      *reinterpret_cast<uint4*>(s + row * CT_LD + cc) = r[p];
    }
  };
  auto gload_a = [&](int kt, uint4 (&r)[KK * 2]) {
    const int tb0 = (tok_beg + kt * CT_BK) / 16;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int tb = tb0 + kk, cb = cb0 + i;
        // token blocks past the split's end hold other splits' tokens: they must not count
        const bool ok = tb < ntb && tb * 16 < tok_end && cb < a.ccb;
        r[kk * 2 + i] = ok ? Cp[((int64_t)tb * a.ccb + cb) * 64 + lane] : make_uint4(0u, 0u, 0u, 0u);
      }
  };
  auto compute = [&](int stage, const uint4 (&fa)[KK * 2]) {
    const bf16_t* s = smem + stage * STAGE;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      // token rows of this lane's 8 slots: 4 lh + e (e < 4), 8 + 4 lh + e - 4 (e >= 4)
      union {
        uint2 p;
        bf16_t s4[4];
      } v[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int row = kk * 16 + (e < 4 ? 4 * lh + e : 8 + 4 * lh + (e - 4));
        v[e].p = *reinterpret_cast<const uint2*>(s + row * CT_LD + 4 * li);
      }
      bf16x8 fb[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        union {
          bf16x8 f;
          bf16_t s8[8];
        } o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o.s8[e] = v[e].s4[j];
        fb[j] = o.f;
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(fa[kk * 2 + i]), fb[j], acc[i][j], 0, 0, 0);
    }
  };

  if (nk > 0) {
    gload_b(0, rb[0]);
    gload_a(0, rafr[0]);
    if (nk > 1) gload_b(1, rb[1]);
    sstore_b(0, rb[0]);
  }
  __syncthreads();
  for (int kt = 0; kt < nk; kt += 2) {
    if (kt + 1 < nk) sstore_b((kt + 1) % CT_STAGES, rb[1]);
    if (kt + 2 < nk) gload_b(kt + 2, rb[0]);
    if (kt + 1 < nk) gload_a(kt + 1, rafr[1]);
    compute(kt % CT_STAGES, rafr[0]);
    __syncthreads();
    if (kt + 1 < nk) {
      if (kt + 2 < nk) sstore_b((kt + 2) % CT_STAGES, rb[0]);
      if (kt + 3 < nk) gload_b(kt + 3, rb[1]);
      if (kt + 2 < nk) gload_a(kt + 2, rafr[0]);
      compute((kt + 1) % CT_STAGES, rafr[1]);
      __syncthreads();
    }
  }

  // epilogue: T row = 32 (cb0 + i) + 8*(v/4) + 4*lh + v%4, columns n0 + 4 li .. + 3
  float* out = a.slabs + (int64_t)split * a.c * a.m;
  const int n = n0 + 4 * li;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = (cb0 + i) * 32 + 8 * (v / 4) + 4 * lh + (v % 4);
      if (row < a.c) {
        float* o = out + (int64_t)row * a.m + n;
        if (n + 3 < a.m && (a.m & 3) == 0) {
          *reinterpret_cast<float4*>(o) = make_float4(acc[i][0][v], acc[i][1][v], acc[i][2][v], acc[i][3][v]);
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (n + j < a.m) o[j] = acc[i][j][v];
        }
      }
    }
}

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
  const int64_t ntb = (N + 15) / 16, total = ntb * ccb * 64;
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

// T (c x ldt bf16, row-major) = w_j * sum_z slab[z][j][n]; w_j = 1 (j < k_lo) or scale_hi.
// Four columns per thread; columns m..ldt-1 are zeroed.
__global__ __launch_bounds__(256) void reduce_scale_bf16_kernel(const float* __restrict__ slabs, int splits, int c,
                                                                int m, int k_lo, float scale_hi,
                                                                bf16_t* __restrict__ T, int64_t ldt) {
  const int64_t quads = ldt / 4, total = (int64_t)c * quads, slab = (int64_t)c * m;
  for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += (int64_t)gridDim.x * blockDim.x) {
    const int64_t j = g / quads, n = (g % quads) * 4;
    float s[4] = {0.f, 0.f, 0.f, 0.f};
    const float* p = slabs + j * m + n;
    if (n + 3 < m && (m & 3) == 0) {
#pragma unroll 4
      for (int z = 0; z < splits; ++z) {
        const float4 v = *reinterpret_cast<const float4*>(p + z * slab);
        s[0] += v.x; s[1] += v.y; s[2] += v.z; s[3] += v.w;
      }
    } else {
      for (int z = 0; z < splits; ++z)
        for (int e = 0; e < 4; ++e)
          if (n + e < m) s[e] += p[z * slab + e];
    }
    const float w = j >= k_lo ? scale_hi : 1.f;
    uint2 o;
    o.x = pack2(s[0] * w, s[1] * w);
    o.y = pack2(s[2] * w, s[3] * w);
    *reinterpret_cast<uint2*>(T + j * ldt + n) = o;
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

int launch_compress_panel(prac_ctx* ctx, const bf16_t* X, int64_t ldx, int N, int d, const bf16_t* Pfrag, int ncb,
                          int c, bf16_t* C, int64_t ldc, bool packed) {
  CompressArgs a;
  a.X = X; a.ldx = ldx; a.N = N; a.d = d; a.Pfrag = Pfrag; a.ncb = ncb; a.c = c;
  a.C = C; a.ldc = ldc; a.ccb = (c + 31) / 32; a.packed = packed ? 1 : 0;
  a.tiles_m = (N + CP_BM - 1) / CP_BM;
  const int FN = (c <= 128) ? 1 : 2;
  a.col_groups = (a.ccb + 4 * FN - 1) / (4 * FN);
  if (a.col_groups * 4 * FN > ncb) return PRAC_EINVAL;  // packed basis narrower than the launch assumes
  const size_t smem = (size_t)CP_STAGES * CP_BM * CP_LD * sizeof(bf16_t);
  const int total = a.tiles_m * a.col_groups;
  const dim3 grid(((total + 7) / 8) * 8), block(256);
  static bool s1 = false, s2 = false;
  if (FN == 1) {
    int rc = set_smem(ctx, compress_panel_kernel<1>, smem, s1);
    if (rc) return rc;
    hipLaunchKernelGGL(compress_panel_kernel<1>, grid, block, smem, ctx->stream, a);
  } else {
    int rc = set_smem(ctx, compress_panel_kernel<2>, smem, s2);
    if (rc) return rc;
    hipLaunchKernelGGL(compress_panel_kernel<2>, grid, block, smem, ctx->stream, a);
  }
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

int launch_ctdy(prac_ctx* ctx, const bf16_t* Cpk, int c, const bf16_t* dY, int64_t lddy, int N, int m, float* slabs,
                int splits) {
  CtdyArgs a;
  a.Cpk = Cpk; a.ccb = (c + 31) / 32; a.c = c; a.dY = dY; a.lddy = lddy; a.N = N; a.m = m;
  a.slabs = slabs; a.splits = splits;
  const int ktiles = (N + CT_BK - 1) / CT_BK;
  a.tok_per_split = ((ktiles + splits - 1) / splits) * CT_BK;
  a.tiles_n = (m + CT_BN - 1) / CT_BN;
  a.row_groups = (a.ccb + 7) / 8;
  const size_t smem = (size_t)CT_STAGES * CT_BK * CT_LD * sizeof(bf16_t);
  const int total = a.tiles_n * a.row_groups * splits;
  static bool s = false;
  int rc = set_smem(ctx, ctdy_kernel, smem, s);
  if (rc) return rc;
  hipLaunchKernelGGL(ctdy_kernel, dim3(((total + 7) / 8) * 8), dim3(256), smem, ctx->stream, a);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

int launch_pack_pfrag(prac_ctx* ctx, const float* P, int64_t d, int64_t ldp, int c, int nkb, int ncb, bf16_t* out) {
  hipLaunchKernelGGL(pack_pfrag_kernel, dim3(grid_for((int64_t)nkb * ncb * 64, ctx->n_cu)), dim3(256), 0, ctx->stream,
                     P, d, ldp, c, nkb, ncb, out);
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
  hipLaunchKernelGGL(pack_c_kernel, dim3(grid_for((int64_t)((N + 15) / 16) * ccb * 64, ctx->n_cu)), dim3(256), 0,
                     ctx->stream, C, ldc, N, c, ccb, Cpk);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

int launch_reduce_scale_bf16(prac_ctx* ctx, const float* slabs, int splits, int c, int m, int k_lo, float scale_hi,
                             bf16_t* T, int64_t ldt) {
  hipLaunchKernelGGL(reduce_scale_bf16_kernel, dim3(grid_for((int64_t)c * (ldt / 4), ctx->n_cu)), dim3(256), 0,
                     ctx->stream, slabs, splits, c, m, k_lo, scale_hi, T, ldt);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}
