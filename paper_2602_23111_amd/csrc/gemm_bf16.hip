// bf16 MFMA GEMM for gfx950 with fp32 accumulation.
//
// One kernel template serves the dense contractions of the PRAC path:
//   compress        C  = X P            A = X  (K contiguous), B = P^T (K contiguous)
//   fused forward   [Y|C] = X [W|P]     two B operands sharing the A row panel
//   C^T dY          T  = C^T dY         A = C, B = dY, both with the reduction index
//                                       (tokens) as the slow dimension, split over tokens
//   Gram            G  = X^T X          same shape of problem as C^T dY
//   P T             dW = P T            A = P (K contiguous), B = T^T (K contiguous)
//
// A workgroup owns a BM x BN output tile and walks K in steps of BK through a
// double-buffered LDS stage; each wave owns a (BM/WGM) x (BN/WGN) sub-tile built
// from 32x32x16 MFMA blocks.  Operands whose reduction index is the slow (strided)
// dimension are staged in LDS as they lie in memory and turned into MFMA fragments
// by an in-register 8 x F transpose; this permutes the rows a lane owns inside the
// wave tile, which the epilogue undoes when it computes output coordinates.
#include "prac_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

struct KArgs {
  const bf16_t* A;
  int64_t lda;
  int M, K;
  const bf16_t* B0;
  int64_t ldb0;
  int N0;
  void* out0;
  int64_t ldo0;
  const bf16_t* B1;
  int64_t ldb1;
  int N1;
  void* out1;
  int64_t ldo1;
  int nb0, nb1;      // column blocks of each output
  int tiles_m;
  int splits;
  int k_per_split;   // multiple of BK
  int wg_per_xcd;    // ceil(total workgroups / 8)
  int total_wg;
  int out_bf16;
  float beta;
  float* partial;    // splits > 1
};

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// 8 consecutive bf16 starting at p; only the first n_valid (0..8) may be touched.
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

template <int F>
struct Pack;
template <>
struct Pack<1> { typedef uint16_t type; };
template <>
struct Pack<2> { typedef uint32_t type; };
template <>
struct Pack<4> { typedef uint2 type; };
template <>
struct Pack<8> { typedef uint4 type; };

// Fragments of an operand staged K-major ([k][row], row contiguous, leading dim ld).
// Lane (i = lane%32, h = lane/32) reads F consecutive rows f*i .. f*i+F-1 of the wave
// tile from the 8 k-rows krow .. krow+7 and transposes: fragment j holds, for tile row
// F*i + j, the 8 k values.
template <int F>
__device__ __forceinline__ void frags_kmajor(const bf16_t* tile, int ld, int row0, int krow, int i,
                                             bf16x8 (&out)[F]) {
  typedef typename Pack<F>::type P;
  union {
    P p;
    bf16_t s[F];
  } v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e].p = *reinterpret_cast<const P*>(tile + (krow + e) * ld + row0 + F * i);
#pragma unroll
  for (int j = 0; j < F; ++j) {
    union {
      bf16x8 f;
      bf16_t s[8];
    } o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o.s[e] = v[e].s[j];
    out[j] = o.f;
  }
}

template <int BM, int BN, int BK, int WGM, int WGN, bool A_KC, bool B_KC>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_bf16_kernel(KArgs a) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int FM = WM / 32, FN = WN / 32;
  constexpr int A_ROWS = A_KC ? BM : BK, A_LD = (A_KC ? BK : BM) + 8;
  constexpr int B_ROWS = B_KC ? BN : BK, B_LD = (B_KC ? BK : BN) + 8;
  constexpr int A_CPR = (A_KC ? BK : BM) / 8, B_CPR = (B_KC ? BK : BN) / 8;  // 16-byte chunks per staged row
  constexpr int A_CH = A_ROWS * A_CPR / NT, B_CH = B_ROWS * B_CPR / NT;
  static_assert(A_ROWS * A_CPR % NT == 0 && B_ROWS * B_CPR % NT == 0, "tile / thread mismatch");
  static_assert(FM >= 1 && FN >= 1 && BK % 16 == 0, "bad wave tile");
  static_assert(A_KC || FM == 1 || FM == 2 || FM == 4 || FM == 8, "K-major A needs FM in {1,2,4,8}");
  static_assert(B_KC || FN == 1 || FN == 2 || FN == 4 || FN == 8, "K-major B needs FN in {1,2,4,8}");

  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);
  constexpr int A_STAGE = A_ROWS * A_LD, B_STAGE = B_ROWS * B_LD;
  bf16_t* As[2] = {smem, smem + A_STAGE};
  bf16_t* Bs[2] = {smem + 2 * A_STAGE, smem + 2 * A_STAGE + B_STAGE};

  // Workgroup -> (split, tile row, tile column).  Dispatch hands consecutive workgroup
  // ids to the 8 XCDs round-robin; give each XCD one contiguous run of logical tiles so
  // that tiles sharing an A panel (and a split's slab) meet in the same L2.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int logical = xcd * a.wg_per_xcd + slot;
  if (slot >= a.wg_per_xcd || logical >= a.total_wg) return;
  const int nb = a.nb0 + a.nb1;
  const int tn = logical % nb;
  const int tm = (logical / nb) % a.tiles_m;
  const int split = logical / (nb * a.tiles_m);

  const bool second = tn >= a.nb0;
  const bf16_t* __restrict__ Bp = second ? a.B1 : a.B0;
  const int64_t ldb = second ? a.ldb1 : a.ldb0;
  const int N = second ? a.N1 : a.N0;
  const int n0 = (second ? tn - a.nb0 : tn) * BN;
  const int m0 = tm * BM;
  const int kbeg = split * a.k_per_split;
  const int kend = min(a.K, kbeg + a.k_per_split);
  const int nk = (kend - kbeg + BK - 1) / BK;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 31, lh = lane >> 5;
  const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
  const bf16_t* __restrict__ Ap = a.A;

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  uint4 ra[A_CH], rb[B_CH];

  auto gload = [&](int k0) {
#pragma unroll
    for (int p = 0; p < A_CH; ++p) {
      const int q = tid + p * NT, r = q / A_CPR, cc = (q % A_CPR) * 8;
      if (A_KC) {
        const int m = m0 + r, k = k0 + cc;
        ra[p] = load_chunk(Ap + (int64_t)m * a.lda + k, m < a.M ? kend - k : 0);
      } else {
        const int k = k0 + r, m = m0 + cc;
        ra[p] = load_chunk(Ap + (int64_t)k * a.lda + m, k < kend ? a.M - m : 0);
      }
    }
#pragma unroll
    for (int p = 0; p < B_CH; ++p) {
      const int q = tid + p * NT, r = q / B_CPR, cc = (q % B_CPR) * 8;
      if (B_KC) {
        const int n = n0 + r, k = k0 + cc;
        rb[p] = load_chunk(Bp + (int64_t)n * ldb + k, n < N ? kend - k : 0);
      } else {
        const int k = k0 + r, n = n0 + cc;
        rb[p] = load_chunk(Bp + (int64_t)k * ldb + n, k < kend ? N - n : 0);
      }
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int p = 0; p < A_CH; ++p) {
      const int q = tid + p * NT, r = q / A_CPR, cc = (q % A_CPR) * 8;
      *reinterpret_cast<uint4*>(As[buf] + r * A_LD + cc) = ra[p];
    }
#pragma unroll
    for (int p = 0; p < B_CH; ++p) {
      const int q = tid + p * NT, r = q / B_CPR, cc = (q % B_CPR) * 8;
      *reinterpret_cast<uint4*>(Bs[buf] + r * B_LD + cc) = rb[p];
    }
  };

  if (nk > 0) {
    gload(kbeg);
    sstore(0);
  }
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) gload(kbeg + (kt + 1) * BK);
    const bf16_t* At = As[buf];
    const bf16_t* Bt = Bs[buf];
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 fa[FM], fb[FN];
      if (A_KC) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
          fa[i] = *reinterpret_cast<const bf16x8*>(At + (wm0 + i * 32 + li) * A_LD + kk * 16 + lh * 8);
      } else {
        frags_kmajor<FM>(At, A_LD, wm0, kk * 16 + lh * 8, li, fa);
      }
      if (B_KC) {
#pragma unroll
        for (int j = 0; j < FN; ++j)
          fb[j] = *reinterpret_cast<const bf16x8*>(Bt + (wn0 + j * 32 + li) * B_LD + kk * 16 + lh * 8);
      } else {
        frags_kmajor<FN>(Bt, B_LD, wn0, kk * 16 + lh * 8, li, fb);
      }
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) sstore(buf ^ 1);
    __syncthreads();
  }

  // Epilogue.  Block (i, j), register v of lane (li, lh) is the element at block row
  // 8*(v/4) + 4*lh + v%4, block column li.
  const bool partial = a.splits > 1;
  void* outp = second ? a.out1 : a.out0;
  const int64_t ldo = partial ? (int64_t)a.N0 : (second ? a.ldo1 : a.ldo0);
  float* pout = partial ? a.partial + (int64_t)split * a.M * a.N0 : nullptr;
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int ri = 8 * (v / 4) + 4 * lh + (v % 4);
        const int m = m0 + (A_KC ? wm0 + i * 32 + ri : wm0 + FM * ri + i);
        const int n = n0 + (B_KC ? wn0 + j * 32 + li : wn0 + FN * li + j);
        if (m < a.M && n < N) {
          const int64_t o = (int64_t)m * ldo + n;
          const float val = acc[i][j][v];
          if (partial) {
            pout[o] = val;
          } else if (a.out_bf16) {
            bf16_t* q = reinterpret_cast<bf16_t*>(outp) + o;
            *q = f32_to_bf16(a.beta == 0.f ? val : val + a.beta * bf16_to_f32(*q));
          } else {
            float* q = reinterpret_cast<float*>(outp) + o;
            *q = a.beta == 0.f ? val : val + a.beta * *q;
          }
        }
      }
}

template <int BM, int BN, int BK, int WGM, int WGN, bool A_KC, bool B_KC>
int launch_cfg(prac_ctx* ctx, const GemmBf16Args& g) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int A_ROWS = A_KC ? BM : BK, A_LD = (A_KC ? BK : BM) + 8;
  constexpr int B_ROWS = B_KC ? BN : BK, B_LD = (B_KC ? BK : BN) + 8;
  constexpr size_t SMEM = 2 * (size_t)(A_ROWS * A_LD + B_ROWS * B_LD) * sizeof(bf16_t);
  KArgs a;
  a.A = g.A; a.lda = g.lda; a.M = g.M; a.K = g.K;
  a.B0 = g.b0.B; a.ldb0 = g.b0.ldb; a.N0 = g.b0.N; a.out0 = g.b0.out; a.ldo0 = g.b0.ldo;
  a.B1 = g.b1.B; a.ldb1 = g.b1.ldb; a.N1 = g.b1.B ? g.b1.N : 0; a.out1 = g.b1.out; a.ldo1 = g.b1.ldo;
  a.nb0 = (a.N0 + BN - 1) / BN;
  a.nb1 = a.B1 ? (a.N1 + BN - 1) / BN : 0;
  a.tiles_m = (a.M + BM - 1) / BM;
  a.splits = g.splits < 1 ? 1 : g.splits;
  const int ktiles = (a.K + BK - 1) / BK;
  a.k_per_split = ((ktiles + a.splits - 1) / a.splits) * BK;
  a.total_wg = (a.nb0 + a.nb1) * a.tiles_m * a.splits;
  a.wg_per_xcd = (a.total_wg + 7) / 8;
  a.beta = g.beta;
  a.partial = g.partial;
  a.out_bf16 = g.out_bf16 ? 1 : 0;
  auto kern = gemm_bf16_kernel<BM, BN, BK, WGM, WGN, A_KC, B_KC>;
  static bool attr_dev[PRAC_MAX_DEVICES] = {};  // per device; one ctx per host thread at a time, benign if raced
  bool& attr_set = attr_dev[ctx->device % PRAC_MAX_DEVICES];
  if (!attr_set) {
    PRAC_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)SMEM));
    attr_set = true;
  }
  PRAC_LAUNCH(ctx, kern, dim3(a.wg_per_xcd * 8), dim3(NT), SMEM, a);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

}  // namespace

// Tile choice.  Row-panel kernels (tile_hint 1) give one workgroup all columns of a
// narrow output so the streamed operand is read once; square tiles serve the rest.
int launch_gemm_bf16(prac_ctx* ctx, const GemmBf16Args& g) {
  if (g.splits > 1 && (g.b1.B != nullptr || g.partial == nullptr)) return PRAC_EINVAL;
  const int hint = g.tile_hint;
  if (g.a_kc && g.b_kc) {
    if (hint == 1) return launch_cfg<128, 256, 64, 2, 2, true, true>(ctx, g);
    return launch_cfg<128, 128, 64, 2, 2, true, true>(ctx, g);
  }
  if (!g.a_kc && !g.b_kc) {
    if (hint == 1) return launch_cfg<256, 128, 32, 2, 2, false, false>(ctx, g);
    return launch_cfg<128, 128, 32, 2, 2, false, false>(ctx, g);
  }
  if (g.a_kc && !g.b_kc) return launch_cfg<128, 128, 32, 2, 2, true, false>(ctx, g);
  return PRAC_EUNSUPPORTED;
}
