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
//
// All loads in the main loops are unconditional (addresses clamped into the operand,
// invalid elements masked to zero afterwards) and the loops run whole groups of bodies
// without branches: the compiler can then count exactly how many younger loads follow
// the one it waits for, which is what keeps several tiles in flight.
#include <type_traits>

#include "frag_utils.h"

namespace {

// ------------------------------------------------------------------ compress
struct CompressArgs {
  const bf16_t* X;
  int64_t ldx;
  int N, d;
  const bf16_t* Pfrag;  // [nkb][ncb][64][8], nkb = round_up(d,128)/16
  int ncb;              // 32-column blocks in the padded basis (multiple of 8)
  int c;
  bf16_t* C;            // row-major (ldc) or packed [ceil(N/16)][ccb][64][8]
  int64_t ldc;
  int ccb;              // 32-column blocks of packed C = ceil(c / 32)
  int packed;
  int tiles_m;
  int col_groups;       // column groups of 4*FN blocks
};

constexpr int CP_BM = 128, CP_BK = 128, CP_LD = CP_BK + 8, CP_STAGES = 2;
constexpr int CP_HK = 4;  // 16-row k-blocks per half tile (P fragments are fetched per half tile)

// 256 threads = 4 waves.  The workgroup owns 128 token rows; wave w owns the 32*FN
// columns [32 FN w, 32 FN (w+1)) of its column group and all 128 rows.
//   X tiles (128 x 128) go global -> registers -> LDS (two stages); tile kt+3 is requested
//   while tile kt is multiplied, 256 contiguous bytes per row and request.
//   P fragments go global (L2) -> registers, half a tile (64 k) at a time, three register
//   sets, each requested one tile ahead of its use.
//   Loads return in issue order, so P requests are always issued ahead of the far-ahead X
//   request of the same body: waiting for P never waits for HBM data requested just now.
//   LDS fragment reads are double-buffered one k-block ahead of the MFMAs that use them,
//   and the LDS store / global requests of the next tiles are issued behind the first MFMA
//   block so that their issue cycles hide under matrix-core time.
template <int FN, int VAR = 0>
__global__ __launch_bounds__(256) void compress_panel_kernel(CompressArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);
  constexpr int STAGE = CP_BM * CP_LD;
  constexpr int A_CH = CP_BM * (CP_BK / 8) / 256;  // 8 chunks of 16 B per thread and tile
  constexpr int KK = CP_BK / 16;                   // 8

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
  const int nh = 2 * nk;
  const u32x4* __restrict__ Pf = reinterpret_cast<const u32x4*>(a.Pfrag);

  // per-thread chunk coordinates: chunk p covers row (tid>>4) + 16 p, columns (tid&15)*8 ..
  const int crow = tid >> 4, ccol = (tid & 15) * 8;
  const int last_chunk = ((a.d - 1) / 8) * 8;  // start of the last (possibly partial) chunk of a row
  // Addresses are a uniform 64-bit base (scalar registers) plus a 32-bit per-thread byte offset,
  // so that a load needs one offset register instead of a 64-bit pointer per chunk.
  const char* xbase = reinterpret_cast<const char*>(a.X + (int64_t)m0 * a.ldx);
  uint32_t roff[A_CH];  // byte offset of this thread's row of chunk p (row clamped into the matrix)
#pragma unroll
  for (int p = 0; p < A_CH; ++p)
    roff[p] = (uint32_t)(min(m0 + crow + 16 * p, a.N - 1) - m0) * (uint32_t)a.ldx * 2u;
  const char* pbase = reinterpret_cast<const char*>(Pf);
  const uint32_t boff = (uint32_t)(cb0 * 64 + lane) * 16u;  // this lane's slot in a row of P blocks
  const int64_t brow = (int64_t)a.ncb * 1024;               // bytes per 16-row k-block of P fragments

  f32x16 acc[4][FN];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  u32x4 ra[2][A_CH];
  u32x4 rb[2][CP_HK * FN];

  // tile / half-tile indices are clamped to the last one: past-the-end prefetches re-read it
  // (from L2) and are never used, which keeps the loop free of conditional loads
  auto gload_a = [&](int kt, u32x4 (&r)[A_CH]) {
    const uint32_t kb = (uint32_t)min(min(kt, nk - 1) * CP_BK + ccol, last_chunk) * 2u;
#pragma unroll
    for (int p = 0; p < A_CH; ++p) r[p] = *reinterpret_cast<const u32x4*>(xbase + (roff[p] + kb));
  };
  // chunks [p0, p0 + 4) of tile kt into LDS.  Only the last tile of a d that is not a multiple
  // of 128 needs its tail columns zeroed (MASK); rows past N are never stored, so they may
  // hold anything finite or not.
  auto sstore_a = [&](int kt, int stage, const u32x4 (&r)[A_CH], auto first, auto mask) {
    constexpr bool MASK = decltype(mask)::value;
    constexpr int p0 = decltype(first)::value;
    bf16_t* s = smem + stage * STAGE;
    const int nv = a.d - (kt * CP_BK + ccol);
#pragma unroll
    for (int p = p0; p < p0 + 4; ++p)
      *reinterpret_cast<u32x4*>(s + (crow + 16 * p) * CP_LD + ccol) = MASK ? keep_first(r[p], nv) : r[p];
  };
  auto gload_b = [&](int hb, u32x4 (&r)[CP_HK * FN]) {
    const char* hbase = pbase + (int64_t)min(hb, nh - 1) * CP_HK * brow;  // uniform
#pragma unroll
    for (int kk = 0; kk < CP_HK; ++kk)
#pragma unroll
      for (int j = 0; j < FN; ++j)
        r[kk * FN + j] = *reinterpret_cast<const u32x4*>(hbase + kk * brow + j * 1024 + boff);
  };
  auto frag_load = [&](int stage, int kk, bf16x8 (&f)[4]) {
    const bf16_t* s = smem + stage * STAGE;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      f[i] = *reinterpret_cast<const bf16x8*>(s + (i * 32 + li) * CP_LD + kk * 16 + lh * 8);
  };
  auto mfma_block = [&](const bf16x8 (&f)[4], const u32x4* b) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i], as_frag(b[j]), acc[i][j], 0, 0, 0);
  };

  const bool tail_mask = (a.d % CP_BK) != 0;  // the last tile has columns past d

  // prologue: P half 0 and X tiles 0, 1 on their way; tile 0 into LDS; tile 2 requested
  gload_b(0, rb[0]);
  gload_a(0, ra[0]);
  gload_a(1, ra[1]);
  if (nk == 1 && tail_mask) {
    sstore_a(0, 0, ra[0], std::integral_constant<int, 0>{}, std::true_type{});
    sstore_a(0, 0, ra[0], std::integral_constant<int, 4>{}, std::true_type{});
  } else {
    sstore_a(0, 0, ra[0], std::integral_constant<int, 0>{}, std::false_type{});
    sstore_a(0, 0, ra[0], std::integral_constant<int, 4>{}, std::false_type{});
  }
  gload_a(2, ra[0]);
  __syncthreads();

  // body kt (PH = kt % 2): LDS stage kt%2 holds X tile kt; ra[(kt+1)%2] holds tile kt+1 and
  // ra[kt%2] awaits tile kt+2; rb[0] / rb[1] hold the first / second P half of tile kt (rb[1]
  // may still be in flight at the top).
  // A wave issues in order and the matrix core accepts one MFMA every ~32 cycles, so
  // everything else (LDS reads of the next k-block, the LDS store of tile kt+1, the global
  // requests) is spread between the MFMAs by the scheduling-group pipeline at the end.
  // Request order inside a body: second P half of tile kt+1 is not needed before the next
  // body, so per body the order is  P(2nd half, tile kt) .. P(1st half, tile kt+1), X(kt+3):
  // the X request is the youngest, and no wait for P ever has to wait for it.
  auto body = [&](int kt, auto ph, auto mask) {
    constexpr int PH = decltype(ph)::value;
    constexpr int S = PH % 2, SA = (PH + 1) % 2;
    constexpr int NMF = 4 * FN;  // MFMAs per k-block
    bf16x8 fa[2][4];
    if (!(VAR & 1)) frag_load(S, 0, fa[0]);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      if (!(VAR & 1) && kk + 1 < KK) frag_load(S, kk + 1, fa[(kk + 1) & 1]);
      if (kk == 0 && !(VAR & 2)) gload_b(2 * kt + 1, rb[1]);
      if (kk == 1 && !(VAR & 8)) sstore_a(kt + 1, SA, ra[SA], std::integral_constant<int, 0>{}, mask);
      if (kk == 2 && !(VAR & 8)) sstore_a(kt + 1, SA, ra[SA], std::integral_constant<int, 4>{}, mask);
      if (kk == 4 && !(VAR & 2)) gload_b(2 * kt + 2, rb[0]);
      if (kk == ((VAR & 64) ? 3 : 5) && !(VAR & 4)) gload_a(kt + 3, ra[SA]);
      if (!(VAR & 1)) mfma_block(fa[kk & 1], kk < CP_HK ? &rb[0][kk * FN] : &rb[1][(kk - CP_HK) * FN]);
    }
    if (VAR == 0 || VAR == 64) {
      // pipeline: 4 LDS reads for the first k-block, then per MFMA one LDS read (while the
      // next k-block still has some) and one of this k-block's extra operations
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
      for (int kk = 0; kk < KK; ++kk)
#pragma unroll
        for (int mi = 0; mi < NMF; ++mi) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          if (kk + 1 < KK && mi < 4) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          if ((kk == 0 || kk == 4) && mi < CP_HK * FN) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
          if ((kk == 1 || kk == 2) && mi < 4) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
          if (kk == ((VAR & 64) ? 3 : 5) && mi < A_CH) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
    }
    if (!(VAR & 16)) __syncthreads();
  };
  int kt = 0;
  const int nfull = tail_mask ? nk - 2 : nk;  // bodies that never store a masked tile
  for (; kt + 2 <= nfull; kt += 2) {
    body(kt, std::integral_constant<int, 0>{}, std::false_type{});
    body(kt + 1, std::integral_constant<int, 1>{}, std::false_type{});
  }
  // remaining bodies; body kt stores tile kt+1, so only body nk-2 stores the (masked) last tile
  for (; kt < nk; ++kt) {
    const bool m = tail_mask && kt == nk - 2;
    if (kt % 2 == 0) {
      if (m) body(kt, std::integral_constant<int, 0>{}, std::true_type{});
      else body(kt, std::integral_constant<int, 0>{}, std::false_type{});
    } else {
      if (m) body(kt, std::integral_constant<int, 1>{}, std::true_type{});
      else body(kt, std::integral_constant<int, 1>{}, std::false_type{});
    }
  }

  // epilogue: block (i, j) register v of lane (li, lh) is token row 8*(v/4) + 4*lh + v%4
  // of row block i, column li of column block cb0 + j.
  if (a.packed) {
    // registers v = 8 tb .. 8 tb + 7 are exactly the 8 slots of the 16-token block tb
    u32x4* Cp = reinterpret_cast<u32x4*>(a.C);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
          // every token block of the 128-row tile is written: packed C is padded to whole tiles
          const int gtb = (m0 + i * 32) / 16 + tb, cb = cb0 + j;
          if (cb < a.ccb) {
            // slot e of this lane is token 16 gtb + (e < 4 ? 4 lh + e : 8 + 4 lh + e - 4);
            // tokens past N (their X rows were not masked) are stored as zeros
            float x[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const int tok = gtb * 16 + (e < 4 ? 4 * lh + e : 8 + 4 * lh + (e - 4));
              x[e] = tok < a.N ? acc[i][j][8 * tb + e] : 0.f;
            }
            u32x4 o;
            o.x = pack2(x[0], x[1]);
            o.y = pack2(x[2], x[3]);
            o.z = pack2(x[4], x[5]);
            o.w = pack2(x[6], x[7]);
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

constexpr int CT_BN = 128, CT_BK = 128, CT_LD = CT_BN + 8, CT_STAGES = 2;
constexpr int CT_HK = 4;  // 16-token blocks per half tile (C fragments are fetched per half tile)

// 256 threads = 4 waves.  The workgroup owns 256 rows of T (columns of C) x 128 columns
// (of dY) for one token range; wave w owns rows [64 w, 64 w + 64).  C fragments come
// straight from the packed layout (global -> registers, half a tile at a time); dY tiles
// (128 tokens x 128 columns) go global -> registers -> LDS as they lie in memory
// ([token][column]) and are turned into fragments by an in-register 8 x 4 transpose.
// Same request order and scheduling-group pipeline as the compress kernel.
// No masking is needed: splits are whole 128-token tiles, token rows past N are read from
// the last valid row of dY and meet the zero padding of packed C (stored for whole tiles);
// columns past m or c only reach outputs that are never stored.
__global__ __launch_bounds__(256) void ctdy_kernel(CtdyArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);
  constexpr int STAGE = CT_BK * CT_LD;
  constexpr int B_CH = CT_BK * (CT_BN / 8) / 256;  // 8 chunks of 16 B per thread and tile
  constexpr int KK = CT_BK / 16;                   // 8

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
  const int nk = tok_end > tok_beg ? (tok_end - tok_beg + CT_BK - 1) / CT_BK : 0;
  const int ntb = ((a.N + 127) / 128) * 8;  // token blocks of packed C, padded to whole 128-token tiles

  f32x16 acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  if (nk > 0) {
    // chunk p of a dY tile: token row (tid>>4) + 16 p, columns n0 + (tid&15)*8 ..
    const int brow = tid >> 4, bcol = (tid & 15) * 8;
    const int last_chunk = ((a.m - 1) / 8) * 8;
    const char* ybase = reinterpret_cast<const char*>(a.dY) + (int64_t)min(n0 + bcol, last_chunk) * 2;
    const int ok_a0 = cb0 < a.ccb, ok_a1 = cb0 + 1 < a.ccb;
    const char* cbase = reinterpret_cast<const char*>(a.Cpk);
    const uint32_t aoff0 = (uint32_t)((ok_a0 ? cb0 : 0) * 64 + lane) * 16u;
    const uint32_t aoff1 = (uint32_t)((ok_a1 ? cb0 + 1 : 0) * 64 + lane) * 16u;
    const int64_t tbrow = (int64_t)a.ccb * 1024;  // bytes per 16-token block of packed C
    const int nh = 2 * nk;

    // register sets are flat arrays indexed with compile-time constants only (a set index
    // that reaches a lambda as a run-time value would push the whole array into scratch)
    u32x4 rb[2 * B_CH];
    u32x4 rafr[2 * CT_HK * 2];

    auto gload_b = [&](int kt, auto set) {
      constexpr int o = decltype(set)::value * B_CH;
      const int t0 = tok_beg + min(kt, nk - 1) * CT_BK + brow;
#pragma unroll
      for (int p = 0; p < B_CH; ++p)
        rb[o + p] = *reinterpret_cast<const u32x4*>(ybase + (int64_t)min(t0 + 16 * p, a.N - 1) * a.lddy * 2);
    };
    auto sstore_b = [&](int stage, auto set, auto first) {
      constexpr int o = decltype(set)::value * B_CH, p0 = decltype(first)::value;
      bf16_t* s = smem + stage * STAGE;
#pragma unroll
      for (int p = p0; p < p0 + 4; ++p) *reinterpret_cast<u32x4*>(s + (brow + 16 * p) * CT_LD + bcol) = rb[o + p];
    };
    // C fragments of half tile hb (4 token blocks), unmasked (see mfma_block)
    auto gload_a = [&](int hb, auto set) {
      constexpr int o = decltype(set)::value * CT_HK * 2;
      const int tb0 = tok_beg / 16 + min(hb, nh - 1) * CT_HK;
#pragma unroll
      for (int kk = 0; kk < CT_HK; ++kk) {
        const char* base = cbase + (int64_t)min(tb0 + kk, ntb - 1) * tbrow;  // uniform
        rafr[o + kk * 2 + 0] = *reinterpret_cast<const u32x4*>(base + aoff0);
        rafr[o + kk * 2 + 1] = *reinterpret_cast<const u32x4*>(base + aoff1);
      }
    };
    // raw LDS rows of k-block kk for this lane: token rows 4 lh + e (e < 4), 8 + 4 lh + e - 4
    auto raw_load = [&](int stage, int kk, u32x2 (&v)[8]) {
      const bf16_t* s = smem + stage * STAGE;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int row = kk * 16 + (e < 4 ? 4 * lh + e : 8 + 4 * lh + (e - 4));
        v[e] = *reinterpret_cast<const u32x2*>(s + row * CT_LD + 4 * li);
      }
    };
    auto mfma_block = [&](const u32x2 (&v)[8], const u32x4& a0, const u32x4& a1) {
      const bf16x8 fa0 = as_frag(a0), fa1 = as_frag(a1);
      // 8 x 4 transpose, one byte-permute per 32-bit word: fragment j takes 16-bit element j
      // of each of the 8 rows (selectors 0-3 address the second operand, 4-7 the first)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        u32x4 o;
        uint32_t w[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
          const uint32_t lo = j < 2 ? v[2 * e2].x : v[2 * e2].y;
          const uint32_t hi = j < 2 ? v[2 * e2 + 1].x : v[2 * e2 + 1].y;
          w[e2] = __builtin_amdgcn_perm(hi, lo, (j & 1) ? 0x07060302u : 0x05040100u);
        }
        o.x = w[0]; o.y = w[1]; o.z = w[2]; o.w = w[3];
        const bf16x8 fb = as_frag(o);
        acc[0][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa0, fb, acc[0][j], 0, 0, 0);
        acc[1][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa1, fb, acc[1][j], 0, 0, 0);
      }
    };

    // prologue: C half 0 and dY tiles 0, 1 on their way; tile 0 into LDS; tile 2 requested
    gload_a(0, std::integral_constant<int, 0>{});
    gload_b(0, std::integral_constant<int, 0>{});
    gload_b(1, std::integral_constant<int, 1>{});
    sstore_b(0, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    sstore_b(0, std::integral_constant<int, 0>{}, std::integral_constant<int, 4>{});
    gload_b(2, std::integral_constant<int, 0>{});
    __syncthreads();

    // body kt (PH = kt % 2): LDS stage kt%2 holds dY tile kt; rb[(kt+1)%2] holds tile kt+1 and
    // rb[kt%2] awaits tile kt+2; rafr[0] / rafr[1] hold the first / second C half of tile kt.
    auto body = [&](int kt, auto ph) {
      constexpr int PH = decltype(ph)::value;
      constexpr int S = PH % 2, SB = (PH + 1) % 2;
      u32x2 raw[2][8];
      raw_load(S, 0, raw[0]);
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        if (kk + 1 < KK) raw_load(S, kk + 1, raw[(kk + 1) & 1]);
        if (kk == 0) gload_a(2 * kt + 1, std::integral_constant<int, 1>{});
        if (kk == 1) sstore_b(SB, std::integral_constant<int, SB>{}, std::integral_constant<int, 0>{});
        if (kk == 2) sstore_b(SB, std::integral_constant<int, SB>{}, std::integral_constant<int, 4>{});
        if (kk == 4) gload_a(2 * kt + 2, std::integral_constant<int, 0>{});
        if (kk == 5) gload_b(kt + 3, std::integral_constant<int, SB>{});
        mfma_block(raw[kk & 1], rafr[kk * 2], rafr[kk * 2 + 1]);
      }
      // pipeline: the first k-block's LDS reads, then per pair of MFMAs the four permutes that
      // build their B fragment, one LDS read of the next k-block and this k-block's extras
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
      for (int kk = 0; kk < KK; ++kk)
#pragma unroll
        for (int pr = 0; pr < 4; ++pr) {
          __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          if (kk + 1 < KK) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          if (kk == 0 || kk == 4 || kk == 5) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
          if (kk == 1 || kk == 2) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          if (kk == 0 || kk == 4 || kk == 5) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
      __syncthreads();
    };
    int kt = 0;
    for (; kt + 2 <= nk; kt += 2) {
      body(kt, std::integral_constant<int, 0>{});
      body(kt + 1, std::integral_constant<int, 1>{});
    }
    if (kt < nk) body(kt, std::integral_constant<int, 0>{});
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

// ------------------------------------------------------------------- dW = P T
// T in fragment order, built by the slab reducer: Tf[(kb * nmb + nb) * 64 + lane][e] =
// bf16(w_k * sum_z slab[z][k][n]) with k = 16 kb + 8 h + e, n = 32 nb + j, lane = 32 h + j,
// w_k = 1 for k < k_lo and scale_hi above; zero where k >= c or n >= m.
// One workgroup per (k-block, pair of 32-column blocks): 256 threads sum a 16 x 64 patch of
// the slabs with one float4 per thread and slab (coalesced 256-byte rows), exchange it through
// LDS and 128 of them emit the two fragments.
__global__ __launch_bounds__(256) void reduce_to_tfrag_kernel(const float* __restrict__ slabs, int splits, int c, int m,
                                                              int k_lo, float scale_hi, int nkb, int nmb,
                                                              bf16_t* __restrict__ Tf) {
  __shared__ float patch[16][68];
  const int pairs = nmb / 2;
  const int kb = blockIdx.x / pairs, np = blockIdx.x % pairs;
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
        const float4 v = *reinterpret_cast<const float4*>(p + z * slab);
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
    const float w = k >= k_lo ? scale_hi : 1.f;
    s.x *= w; s.y *= w; s.z *= w; s.w *= w;
  }
  patch[row][col + 0] = s.x;
  patch[row][col + 1] = s.y;
  patch[row][col + 2] = s.z;
  patch[row][col + 3] = s.w;
  __syncthreads();
  if (tid < 128) {
    const int nbl = tid >> 6, lane = tid & 63, j = lane & 31, h = lane >> 5;
    u32x4 o;
    o.x = pack2(patch[8 * h + 0][nbl * 32 + j], patch[8 * h + 1][nbl * 32 + j]);
    o.y = pack2(patch[8 * h + 2][nbl * 32 + j], patch[8 * h + 3][nbl * 32 + j]);
    o.z = pack2(patch[8 * h + 4][nbl * 32 + j], patch[8 * h + 5][nbl * 32 + j]);
    o.w = pack2(patch[8 * h + 6][nbl * 32 + j], patch[8 * h + 7][nbl * 32 + j]);
    reinterpret_cast<u32x4*>(Tf)[((int64_t)kb * nmb + np * 2 + nbl) * 64 + lane] = o;
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
  const bf16_t* Tf;  // [nkb][nmb][64][8]
  void* dW;
  int64_t lddw;
  int d, m, nkb, nmb;
  int tiles_m, tiles_n;
  float beta;
  int vec_ok;  // dW rows allow aligned 16-byte accesses
};

// dW (d x m) = P T, K = c (a few hundred): both operands are read in fragment order
// straight from L2, no LDS.  256 threads = 2 x 2 waves, a 128 x 128 tile per workgroup,
// 64 x 64 per wave; fragments are requested PT_PD k-blocks ahead.
constexpr int PT_PD = 8;
constexpr int PT_TLD = 128 + 4;  // floats per row of the output staging tile
template <bool OUT_BF16>
__global__ __launch_bounds__(256) void pt_kernel(PtArgs a) {
  const int total = a.tiles_m * a.tiles_n;
  const int per_xcd = (total + 7) / 8;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int logical = xcd * per_xcd + slot;
  if (slot >= per_xcd || logical >= total) return;
  const int tn = logical % a.tiles_n, tm = logical / a.tiles_n;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 31, lh = lane >> 5;
  const int rb0 = tm * 4 + (wave >> 1) * 2, nb0 = tn * 4 + (wave & 1) * 2;
  const u32x4* __restrict__ Pa = reinterpret_cast<const u32x4*>(a.Pa);
  const u32x4* __restrict__ Tf = reinterpret_cast<const u32x4*>(a.Tf);

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
    r[2] = Tf[((int64_t)k * a.nmb + nb0) * 64 + lane];
    r[3] = Tf[((int64_t)k * a.nmb + nb0 + 1) * 64 + lane];
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
      gload(kb + PT_PD + t, fr[t]);
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
      if (grow >= a.d || gcol >= a.m) continue;
      const float4 lo = *reinterpret_cast<const float4*>(tile + row * PT_TLD + c8);
      const float4 hi = *reinterpret_cast<const float4*>(tile + row * PT_TLD + c8 + 4);
      float x[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      bf16_t* q = reinterpret_cast<bf16_t*>(a.dW) + (int64_t)grow * a.lddw + gcol;
      if (a.vec_ok && gcol + 8 <= a.m) {
        if (a.beta != 0.f) {
          const u32x4 old = *reinterpret_cast<const u32x4*>(q);
#pragma unroll
          for (int e = 0; e < 8; ++e)
            x[e] += a.beta * __uint_as_float(((e & 1) ? (old[e >> 1] >> 16) : (old[e >> 1] & 0xFFFFu)) << 16);
        }
        u32x4 o;
        o.x = pack2(x[0], x[1]);
        o.y = pack2(x[2], x[3]);
        o.z = pack2(x[4], x[5]);
        o.w = pack2(x[6], x[7]);
        *reinterpret_cast<u32x4*>(q) = o;
      } else {
        for (int e = 0; e < 8 && gcol + e < a.m; ++e)
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
      if (grow >= a.d || gcol >= a.m) continue;
      float4 x = *reinterpret_cast<const float4*>(tile + row * PT_TLD + c4);
      float* q = reinterpret_cast<float*>(a.dW) + (int64_t)grow * a.lddw + gcol;
      if (a.vec_ok && gcol + 4 <= a.m) {
        if (a.beta != 0.f) {
          const float4 old = *reinterpret_cast<const float4*>(q);
          x.x += a.beta * old.x; x.y += a.beta * old.y; x.z += a.beta * old.z; x.w += a.beta * old.w;
        }
        *reinterpret_cast<float4*>(q) = x;
      } else {
        const float xs[4] = {x.x, x.y, x.z, x.w};
        for (int e = 0; e < 4 && gcol + e < a.m; ++e) q[e] = a.beta == 0.f ? xs[e] : xs[e] + a.beta * q[e];
      }
    }
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
    PRAC_LAUNCH(ctx, compress_panel_kernel<1>, grid, block, smem, a);
  } else {
    int rc = set_smem(ctx, compress_panel_kernel<2>, smem, s2);
    if (rc) return rc;
    PRAC_LAUNCH(ctx, compress_panel_kernel<2>, grid, block, smem, a);
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
  PRAC_LAUNCH(ctx, ctdy_kernel, dim3(((total + 7) / 8) * 8), dim3(256), smem, a);
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
  hipLaunchKernelGGL(pack_c_kernel, dim3(grid_for((int64_t)((N + 127) / 128) * 8 * ccb * 64, ctx->n_cu)), dim3(256), 0,
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

int launch_reduce_to_tfrag(prac_ctx* ctx, const float* slabs, int splits, int c, int m, int k_lo, float scale_hi,
                           int nkb, int nmb, bf16_t* Tf) {
  PRAC_LAUNCH(ctx, reduce_to_tfrag_kernel, dim3(nkb * (nmb / 2)), dim3(256), 0, slabs, splits, c, m, k_lo, scale_hi, nkb,
              nmb, Tf);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

int launch_pack_pafrag(prac_ctx* ctx, const float* P, int64_t d, int64_t ldp, int c, int nrb, int nkb, bf16_t* out) {
  hipLaunchKernelGGL(pack_pafrag_kernel, dim3(grid_for((int64_t)nrb * nkb * 64, ctx->n_cu)), dim3(256), 0, ctx->stream,
                     P, d, ldp, c, nrb, nkb, out);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

int launch_pt(prac_ctx* ctx, const bf16_t* Pa, const bf16_t* Tf, int d, int m, int nkb, int nmb, void* dW,
              int64_t lddw, bool out_bf16, float beta) {
  PtArgs a;
  a.Pa = Pa; a.Tf = Tf; a.dW = dW; a.lddw = lddw; a.d = d; a.m = m; a.nkb = nkb; a.nmb = nmb;
  a.tiles_m = (d + 127) / 128; a.tiles_n = (m + 127) / 128; a.beta = beta;
  const int total = a.tiles_m * a.tiles_n;
  const dim3 grid(((total + 7) / 8) * 8), block(256);
  a.vec_ok = (reinterpret_cast<uintptr_t>(dW) % 16 == 0 && lddw % (out_bf16 ? 8 : 4) == 0) ? 1 : 0;
  const size_t smem = (size_t)128 * PT_TLD * sizeof(float);
  static bool sb = false, sf = false;
  if (out_bf16) {
    int rc = set_smem(ctx, pt_kernel<true>, smem, sb);
    if (rc) return rc;
    PRAC_LAUNCH(ctx, pt_kernel<true>, grid, block, smem, a);
  } else {
    int rc = set_smem(ctx, pt_kernel<false>, smem, sf);
    if (rc) return rc;
    PRAC_LAUNCH(ctx, pt_kernel<false>, grid, block, smem, a);
  }
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}
