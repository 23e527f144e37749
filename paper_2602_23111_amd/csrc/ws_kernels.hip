// Wave-specialised streaming contractions for gfx950.
//
//   compress        C = X P          (Alg. 1 compression step)          compress_ws_kernel
//   reconstruction  X~ = C Ps^T      (Section 5.1; Alg. 2 backward)       reconstruct_ws_kernel
//   weight gradient T = C^T dY       (Lemma 1, reassociated)              ctdy_ws_kernel
//
// A workgroup is 8 waves: 4 matrix waves and 4 loader waves, one of each per SIMD.
//   loader waves   stream the big operand (X) HBM -> registers -> LDS in ordinary
//                  compiler-scheduled code;
//   matrix waves   read A fragments from LDS, fetch their private B fragments (P in MFMA
//                  fragment order, L2-resident) straight into registers and issue MFMAs.
// The matrix waves' inner step (one 16-deep k-block: 4 LDS fragment reads for the next
// k-block interleaved with this k-block's MFMAs) is a fixed instruction sequence in inline
// assembly: with one matrix wave per SIMD nothing else can fill a stall, so the order of
// LDS reads and MFMAs is set by hand rather than left to the scheduler.  The LDS reads are
// invisible to the compiler; every such block therefore ends with its own wait for them.
//
// A k-tile is 128 rows x 256 k: every row contributes a 512-byte run.  HBM delivers runs of
// 512 bytes about a quarter faster than runs of 256 (measured with a plain reader over the
// same panel shape), which is why the tile is deep rather than the ring long.  LDS holds
// two tiles (rows padded to 528 bytes): tile kt is multiplied while tile kt+1 is written
// and tile kt+2 is in flight to the loaders' registers.  One barrier per tile, placed in
// the matrix waves between k-blocks 14 and 15: everything before it has finished reading
// tile kt's stage (which the loaders overwrite next with tile kt+2), and k-block 15 already
// prefetches from tile kt+1, complete since the loaders reached the same barrier.
//
// The same kernel forms the layer's forward output Y = X W in the same launch (not in the
// paper; forward of Lemma 1): W is handed over in the fragment order of P, and the column
// groups of Y come before those of C in the grid.  Workgroups of one row tile sit next to
// each other on one XCD, so X comes from HBM once and from that XCD's L2 afterwards.
#include <algorithm>
#include <type_traits>

#include "frag_utils.h"

namespace {

// f(integral_constant<int, 0>{}), ..., f(integral_constant<int, N - 1>{})
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (N > 0) {
    static_for<N - 1>(f);
    f(std::integral_constant<int, N - 1>{});
  }
}

// Development builds only (-DPRAC_WS_TIMESTAMPS): thread 0 of every workgroup writes wall-clock stamps.
#ifdef PRAC_WS_TIMESTAMPS
#define PRAC_STAMP(a, i) \
  do { if ((a).stamps && threadIdx.x == 0) (a).stamps[(long long)blockIdx.x * 8 + (i)] = wall_clock64(); } while (0)
long long* g_ws_stamps = nullptr;
#else
#define PRAC_STAMP(a, i) do { } while (0)
#endif

struct CompressWsArgs {
#ifdef PRAC_WS_TIMESTAMPS
  long long* stamps;
#endif
  const bf16_t* X;
  int64_t ldx;
  int N, d;
  const bf16_t* Pfrag;  // [nkb][ncb][64][8], nkb = round_up(d,256)/16, zero outside d x c
  int ncb;              // 32-column blocks in the padded basis
  int c;
  bf16_t* C;            // row-major (ldc) or packed [ceil(N/128)*8][ccb][64][8]
  int64_t ldc;
  int ccb;              // 32-column blocks of packed C = ceil(c / 32)
  int packed;
  int tiles_m;
  int col_groups;       // column groups of 4*FN blocks (forward output first, then C)
  // fused forward Y = X W: the first w_groups column groups multiply by W instead of P
  const bf16_t* Wfrag;  // [nkb][ncb_w][64][8], same fragment order as Pfrag; nullptr: no forward output
  int ncb_w;            // 32-column blocks in the padded W (multiple of 4*FN)
  int w_groups;
  int m;                // columns of Y
  bf16_t* Y;            // row-major N x m
  int64_t ldy;
};

constexpr int WS_BM = 128, WS_BK = 256, WS_LD = WS_BK + 8;
constexpr int WS_STAGE = WS_BM * WS_LD * 2;  // bytes per LDS stage (67584)
constexpr int WS_STAGES = 2;
constexpr int WS_RB = 32 * WS_LD * 2;        // bytes between 32-row blocks of a stage (16896)
constexpr int WS_KB = WS_BK / 16;            // k-blocks per tile
constexpr int WS_NCH = 4, WS_NIF = 2;        // chunks per tile, chunks in flight

// One k-block of a 128 x 64 wave tile: acc[2 i + j] += fa[i] * b_j, while the four A fragments
// at byte offsets O + i * WS_RB from `lds` are read into fn.  The block also issues the two
// 1 KB requests that refill another slot of the P ring (n0, n1 <- fragments at `src` + lane
// offset `voff`, and 1 KB further); the address is an SGPR pair plus one VGPR, so no vector
// arithmetic sits between the blocks.  The requests come first in the block, before the LDS
// reads: a vector-memory request placed between two LDS reads stalls the wave's in-order issue
// and with it the MFMAs behind it (measured: 29 against 20 us for the 128 k-blocks of a workgroup).
// The compiler cannot see these loads.  The block therefore starts with its own wait: all
// but the VM youngest requests of this wave have arrived (the ring's distance times the
// requests per block; b0 / b1 were requested that long ago), and n0 / n1 may only be read
// by a later block, after that block's wait.
template <int O, int VM>
__device__ __forceinline__ void kblock2(f32x16 (&acc)[8], const u32x4 (&fa)[4], u32x4 (&fn)[4], const u32x4& b0,
                                        const u32x4& b1, unsigned lds, u32x4& n0, u32x4& n1, uint32_t voff,
                                        const char* src) {
  asm volatile(
      "s_waitcnt vmcnt(%27)\n"
      "global_load_dwordx4 %12, %21, %22\n"
      "global_load_dwordx4 %13, %21, %22 offset:1024\n"
      "ds_read_b128 %8, %20 offset:%23\n"
      "v_mfma_f32_32x32x16_bf16 %0, %14, %18, %0\n"
      "ds_read_b128 %9, %20 offset:%24\n"
      "v_mfma_f32_32x32x16_bf16 %1, %14, %19, %1\n"
      "ds_read_b128 %10, %20 offset:%25\n"
      "v_mfma_f32_32x32x16_bf16 %2, %15, %18, %2\n"
      "ds_read_b128 %11, %20 offset:%26\n"
      "v_mfma_f32_32x32x16_bf16 %3, %15, %19, %3\n"
      "v_mfma_f32_32x32x16_bf16 %4, %16, %18, %4\n"
      "v_mfma_f32_32x32x16_bf16 %5, %16, %19, %5\n"
      "v_mfma_f32_32x32x16_bf16 %6, %17, %18, %6\n"
      "v_mfma_f32_32x32x16_bf16 %7, %17, %19, %7\n"
      "s_waitcnt lgkmcnt(0)\n"
      : "+a"(acc[0]), "+a"(acc[1]), "+a"(acc[2]), "+a"(acc[3]), "+a"(acc[4]), "+a"(acc[5]), "+a"(acc[6]),
        "+a"(acc[7]), "=&v"(fn[0]), "=&v"(fn[1]), "=&v"(fn[2]), "=&v"(fn[3]), "=&v"(n0), "=&v"(n1)
      : "v"(fa[0]), "v"(fa[1]), "v"(fa[2]), "v"(fa[3]), "v"(b0), "v"(b1), "v"(lds), "v"(voff), "s"(src), "n"(O),
        "n"(O + WS_RB), "n"(O + 2 * WS_RB), "n"(O + 3 * WS_RB), "n"(VM)
      : "memory");
}

// Same for a 128 x 32 wave tile: acc[i] += fa[i] * b, one refill request.
template <int O, int VM>
__device__ __forceinline__ void kblock1(f32x16 (&acc)[4], const u32x4 (&fa)[4], u32x4 (&fn)[4], const u32x4& b,
                                        unsigned lds, u32x4& n0, uint32_t voff, const char* src) {
  asm volatile(
      "s_waitcnt vmcnt(%21)\n"
      "global_load_dwordx4 %8, %15, %16\n"
      "ds_read_b128 %4, %14 offset:%17\n"
      "ds_read_b128 %5, %14 offset:%18\n"
      "v_mfma_f32_32x32x16_bf16 %0, %9, %13, %0\n"
      "ds_read_b128 %6, %14 offset:%19\n"
      "ds_read_b128 %7, %14 offset:%20\n"
      "v_mfma_f32_32x32x16_bf16 %1, %10, %13, %1\n"
      "v_mfma_f32_32x32x16_bf16 %2, %11, %13, %2\n"
      "v_mfma_f32_32x32x16_bf16 %3, %12, %13, %3\n"
      "s_waitcnt lgkmcnt(0)\n"
      : "+a"(acc[0]), "+a"(acc[1]), "+a"(acc[2]), "+a"(acc[3]), "=&v"(fn[0]), "=&v"(fn[1]), "=&v"(fn[2]),
        "=&v"(fn[3]), "=&v"(n0)
      : "v"(fa[0]), "v"(fa[1]), "v"(fa[2]), "v"(fa[3]), "v"(b), "v"(lds), "v"(voff), "s"(src), "n"(O),
        "n"(O + WS_RB), "n"(O + 2 * WS_RB), "n"(O + 3 * WS_RB), "n"(VM)
      : "memory");
}

// One 1 KB ring request outside the k-blocks (the first fills): n <- 16 bytes at src + voff (+ OFF).
// Issued in assembly like the blocks' own requests, so that the compiler keeps no count of
// outstanding loads for the ring at all (its own waits would drain the ring once per tile).
template <int OFF>
__device__ __forceinline__ void ring_request(u32x4& n, uint32_t voff, const char* src) {
  asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3\n" : "=&v"(n) : "v"(voff), "s"(src), "n"(OFF) : "memory");
}

__device__ __forceinline__ void frag_read4(u32x4 (&f)[4], unsigned lds) {
  asm volatile(
      "ds_read_b128 %0, %4\n"
      "ds_read_b128 %1, %4 offset:%5\n"
      "ds_read_b128 %2, %4 offset:%6\n"
      "ds_read_b128 %3, %4 offset:%7\n"
      "s_waitcnt lgkmcnt(0)\n"
      : "=&v"(f[0]), "=&v"(f[1]), "=&v"(f[2]), "=&v"(f[3])
      : "v"(lds), "n"(WS_RB), "n"(2 * WS_RB), "n"(3 * WS_RB)
      : "memory");
}

// The compiler does not see the MFMAs inside the blocks above, so it cannot know that the
// accumulators may still be in the matrix pipeline: drain it before they are read.  The ring's
// last requests are still in flight as well, and nothing reads their results: without the ring
// among the operands here the compiler would treat those registers as free from the moment of
// the request and hand them to other values, which the late data would then overwrite.
template <int NACC, int NR>
__device__ __forceinline__ void drain_mfma(f32x16 (&acc)[NACC], u32x4 (&ring)[8][NR]) {
  asm volatile("s_waitcnt vmcnt(0)\n" : "+v"(ring[0][0]), "+v"(ring[1][0]), "+v"(ring[2][0]), "+v"(ring[3][0]),
               "+v"(ring[4][0]), "+v"(ring[5][0]), "+v"(ring[6][0]), "+v"(ring[7][0])
               :
               : "memory");
  if constexpr (NR == 2)
    asm volatile("" : "+v"(ring[0][1]), "+v"(ring[1][1]), "+v"(ring[2][1]), "+v"(ring[3][1]), "+v"(ring[4][1]),
                 "+v"(ring[5][1]), "+v"(ring[6][1]), "+v"(ring[7][1])
                 :
                 : "memory");
  if constexpr (NACC == 8) {
    asm volatile("s_nop 15\ns_nop 15\ns_nop 15\ns_nop 15\n"
                 : "+a"(acc[0]), "+a"(acc[1]), "+a"(acc[2]), "+a"(acc[3]), "+a"(acc[4]), "+a"(acc[5]), "+a"(acc[6]),
                   "+a"(acc[7])
                 :
                 : "memory");
  } else {
    asm volatile("s_nop 15\ns_nop 15\ns_nop 15\ns_nop 15\n"
                 : "+a"(acc[0]), "+a"(acc[1]), "+a"(acc[2]), "+a"(acc[3])
                 :
                 : "memory");
  }
}

template <int FN, int NCH, int NIF>
__global__ __launch_bounds__(512) void compress_ws_kernel(CompressWsArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const int bid = touch_kernel_args<sizeof(CompressWsArgs)>(blockIdx.x);

  // XCD-aware order: consecutive logical tiles (same rows, next column group) on one XCD
  const int total = a.tiles_m * a.col_groups;
  const int per_xcd = (total + 7) / 8;
  const int xcd = bid & 7, slot = bid >> 3;
  const int logical = xcd * per_xcd + slot;
  if (slot >= per_xcd || logical >= total) return;
  const int cg = logical % a.col_groups, tm = logical / a.col_groups;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  PRAC_STAMP(a, 0);
  const int m0 = tm * WS_BM;
  const int nk = (a.d + WS_BK - 1) / WS_BK;
  // Step kt of this workgroup works on k-tile act(kt): the sum over k may run in any order, and
  // workgroups that start at different tiles neither ask L2 for the same lines of P at once nor
  // all pull on the same memory channels (their row panels have the same alignment).
  // (not with a forward output: there workgroups of different row tiles share W through L2 and
  // should ask for it in the same order)
  const int rot = a.Wfrag ? 0 : tm % nk;
  auto act = [&](int kt) {
    const int t = min(kt, nk - 1) + rot;
    return t >= nk ? t - nk : t;
  };

  if (wave >= 4) {
    // ------------------------------------------------------------ loader waves
    const int lt = tid - 256;
    const int crow = lt >> 5, ccol = (lt & 31) * 8;  // chunk q: row crow + 8 q, columns ccol .. ccol + 7
    const int last_chunk = ((a.d - 1) / 8) * 8;      // start of the last (possibly partial) chunk of a row
    const char* xbase = reinterpret_cast<const char*>(a.X + (int64_t)m0 * a.ldx);
    uint32_t roff[16];  // byte offset of the row of chunk q (rows past N re-read the last row; never stored to C)
#pragma unroll
    for (int q = 0; q < 16; ++q) roff[q] = (uint32_t)(min(m0 + crow + 8 * q, a.N - 1) - m0) * (uint32_t)a.ldx * 2u;
    const uint32_t soff = (uint32_t)(crow * WS_LD + ccol) * 2u;

    // The tile is fetched in NCH chunks of 128 / NCH rows, one chunk per barrier interval, with
    // NIF chunks in flight: the vector L1 returns data in request order, so the matrix waves'
    // P loads wait behind every X request issued before them.  Requests for X issued in one burst
    // per tile stall the matrix waves for the length of that burst; spread evenly they delay each
    // P load by about one memory latency, which the P ring covers.
    constexpr int CR = 16 / NCH;  // 16-byte loads per thread and chunk
    u32x4 ra[16];                 // chunk g lives in ra[(g % NCH) * CR ...]
    // Requests past the last tile stay in the instruction stream (the loop has no load-free tail
    // version) but all go to one chunk of this thread's first row, which the caches already hold.  Like
    // every other request it is clamped to the row's last chunk: with d < 256 the thread's own column
    // lies past the end of the row, and in the last row of X past the end of the buffer.
    const uint32_t dead_off = roff[0] + (uint32_t)min(ccol, last_chunk) * 2u;
    auto cload = [&](int g, auto qc) {
      constexpr int Q = decltype(qc)::value;  // g % NCH
      const int kt = g / NCH;
      const uint32_t kb = (uint32_t)min(act(kt) * WS_BK + ccol, last_chunk) * 2u;
      const bool live = kt < nk;
#pragma unroll
      for (int j = 0; j < CR; ++j)
        ra[Q * CR + j] = __builtin_nontemporal_load(
            reinterpret_cast<const u32x4*>(xbase + (live ? roff[Q * CR + j] + kb : dead_off)));
    };
    // chunk g -> stage (g / NCH) % 2; columns past d are zeroed (only the last tile has any)
    auto cstore = [&](int g, auto qc) {
      constexpr int Q = decltype(qc)::value;
      const int kt = g / NCH;
      unsigned char* s = smem_raw + (kt & 1) * WS_STAGE + soff;
      const int nv = a.d - (act(kt) * WS_BK + ccol);
      if (nv >= 8) {
#pragma unroll
        for (int j = 0; j < CR; ++j) *reinterpret_cast<u32x4*>(s + (Q * CR + j) * (8 * WS_LD * 2)) = ra[Q * CR + j];
      } else {
#pragma unroll
        for (int j = 0; j < CR; ++j)
          *reinterpret_cast<u32x4*>(s + (Q * CR + j) * (8 * WS_LD * 2)) = keep_first(ra[Q * CR + j], nv);
      }
    };
#define PRAC_IC(v) std::integral_constant<int, (v)> {}
    // tile 0 at once, then the first NIF chunks of tile 1
    static_for<NCH>([&](auto q) { cload(decltype(q)::value, q); });
    static_for<NCH>([&](auto q) { cstore(decltype(q)::value, q); });
    static_for<NIF>([&](auto q) { cload(NCH + decltype(q)::value, q); });
    __syncthreads();  // tile 0 is in LDS
    for (int kt = 0; kt < nk; ++kt) {
      // interval q of tile kt: chunk q of tile kt+1 -> LDS (its stage was last read for tile kt-1, before
      // the previous tile's last barrier), then chunk q + NIF of tile kt+1 is requested
      static_for<NCH>([&](auto q) {
        constexpr int Q = decltype(q)::value;
        const int g = (kt + 1) * NCH + Q;
        if (kt + 1 < nk) cstore(g, q);
        cload(g + NIF, PRAC_IC((Q + NIF) % NCH));
        __syncthreads();
      });
    }
#undef PRAC_IC
    return;
  }

  // -------------------------------------------------------------- matrix waves
  const int lane = tid & 63, li = lane & 31, lh = lane >> 5;
  const bool fwd = cg < a.w_groups;  // this workgroup's columns belong to Y
  const int cb0 = (fwd ? cg : cg - a.w_groups) * 4 * FN + wave * FN;  // first 32-column block of this wave
  const char* pbase = reinterpret_cast<const char*>(fwd ? a.Wfrag : a.Pfrag);
  const uint32_t boff = (uint32_t)(cb0 * 64 + lane) * 16u;     // this lane's slot in a row of blocks
  const int64_t brow = (int64_t)(fwd ? a.ncb_w : a.ncb) * 1024;  // bytes per 16-row k-block of fragments

  constexpr int NACC = 4 * FN;
  f32x16 acc[NACC];
#pragma unroll
  for (int i = 0; i < NACC; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

  // Ring of eight k-blocks' P fragments.  Block j multiplies with slot j % 8 and requests k-block
  // j + 7 into slot (j + 7) % 8, the slot block j - 1 has just used: seven k-blocks of distance.
  // `preq` is the address of the next k-block to request: it walks down a tile's 16 k-blocks
  // and jumps to the next tile's base after the tile's last one.
  u32x4 rb[8][FN];
  auto tile_base = [&](int kt) {
    // past the last tile: tile 0's fragments again (valid memory, an L2 hit, never used)
    return pbase + (kt < nk ? (int64_t)act(kt) * WS_KB * brow : (int64_t)0);  // uniform
  };
  const char* preq = tile_base(0);
  const char* next_base = tile_base(1);
#pragma unroll
  for (int kk = 0; kk < 7; ++kk) {
    ring_request<0>(rb[kk][0], boff, preq);
    if constexpr (FN == 2) ring_request<1024>(rb[kk][FN - 1], boff, preq);
    preq += brow;
  }
  constexpr int VM = 6 * FN;  // requests younger than the ones a block is about to use
  auto kblock = [&](auto oc, const u32x4 (&fcur)[4], u32x4 (&fnext)[4], auto kkc, unsigned lds) {
    constexpr int O = decltype(oc)::value, KK = decltype(kkc)::value;
    if constexpr (FN == 2)
      kblock2<O, VM>(acc, fcur, fnext, rb[KK & 7][0], rb[KK & 7][1], lds, rb[(KK + 7) & 7][0], rb[(KK + 7) & 7][1],
                     boff, preq);
    else
      kblock1<O, VM>(acc, fcur, fnext, rb[KK & 7][0], lds, rb[(KK + 7) & 7][0], boff, preq);
    // the next request is k-block KK + 8 of this tile, or the next tile's first one
    if constexpr (KK == 8) preq = next_base;
    else preq += brow;
  };
#define PRAC_IC(v) std::integral_constant<int, (v)> {}

  // LDS byte address of this lane's A fragment of row block 0, k-block 0, stage 0:
  // row li, 16-byte half lh of the k-block
  const unsigned lds0 =
      (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem_raw + (unsigned)(li * WS_LD * 2 + lh * 16);
  u32x4 fa[4], fb[4];
  __builtin_amdgcn_s_barrier();  // tile 0 is in LDS
  PRAC_STAMP(a, 1);
  frag_read4(fa, lds0);
  for (int kt = 0; kt < nk; ++kt) {
    const unsigned cur = lds0 + (unsigned)(kt & 1) * WS_STAGE;
    const unsigned nxt = lds0 + (unsigned)((kt + 1) & 1) * WS_STAGE;
    // k-block j multiplies while the fragments of k-block j+1 are read; its P slot is then refilled.
    // Barriers: one per chunk interval of the loaders; the last one of a tile sits before k-block 15,
    // whose fragment reads are the first from the next stage.
    static_for<WS_KB>([&](auto jc) {
      constexpr int J = decltype(jc)::value;
      constexpr int IV = WS_KB / NCH;  // k-blocks per barrier interval
      if constexpr (J == WS_KB - 1) __builtin_amdgcn_s_barrier();
      if constexpr (J % 2 == 0) kblock(PRAC_IC(32 * ((J + 1) % WS_KB)), fa, fb, jc, J == WS_KB - 1 ? nxt : cur);
      else kblock(PRAC_IC(32 * ((J + 1) % WS_KB)), fb, fa, jc, J == WS_KB - 1 ? nxt : cur);
      if constexpr (J % IV == IV - 1 && J != WS_KB - 1) __builtin_amdgcn_s_barrier();
    });
    next_base = tile_base(kt + 2);
    // Drain inside the loop: at the loop's exit the compiler may move accumulators between
    // registers (it has no idea that matrix instructions are still writing them), and such
    // moves must find the pipeline empty.
    if (kt == nk - 1) drain_mfma<NACC, FN>(acc, rb);
  }
#undef PRAC_IC

  // epilogue: block (i, j) = acc[i * FN + j]; register v of lane (li, lh) is token row
  // 8*(v/4) + 4*lh + v%4 of row block i, column li of column block cb0 + j.
  PRAC_STAMP(a, 2);
  if (a.packed && !fwd) {
    // registers v = 8 tb .. 8 tb + 7 are exactly the 8 slots of the 16-token block tb
    u32x4* Cp = reinterpret_cast<u32x4*>(a.C);
    if (m0 + WS_BM <= a.N && cb0 + FN <= a.ccb) {
      // every token row and column block of the wave's tile is inside C: no masks, one base address
      // (the epilogue is bound by the number of vector instructions issued: 8 register reads and 4
      // conversions per store here against 45 instructions with the per-element checks below)
      u32x4* base = Cp + ((int64_t)(m0 / 16) * a.ccb + cb0) * 64 + lane;
      const int64_t tbs = (int64_t)a.ccb * 64;  // 16-token blocks are ccb * 64 slots apart
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
          asm volatile("" : "+a"(acc[i * FN + j]) : : "memory");  // one block at a time leaves the accumulators
#pragma unroll
          for (int tb = 0; tb < 2; ++tb) {
            const f32x16& t = acc[i * FN + j];
            u32x4 o;
            o.x = pack2_hw(t[8 * tb + 0], t[8 * tb + 1]);
            o.y = pack2_hw(t[8 * tb + 2], t[8 * tb + 3]);
            o.z = pack2_hw(t[8 * tb + 4], t[8 * tb + 5]);
            o.w = pack2_hw(t[8 * tb + 6], t[8 * tb + 7]);
            stream_store(base + (2 * i + tb) * tbs + j * 64, o);
          }
        }
    } else
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        // one block at a time leaves the accumulator registers (keeps the copies short-lived)
        asm volatile("" : "+a"(acc[i * FN + j]) : : "memory");
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
          // every token block of the 128-row tile is written: packed C is padded to whole tiles
          const int gtb = (m0 + i * 32) / 16 + tb, cb = cb0 + j;
          if (cb < a.ccb) {
            // slot e of this lane is token 16 gtb + (e < 4 ? 4 lh + e : 8 + 4 lh + e - 4);
            // tokens past N (computed from a repeated row) are stored as zeros
            float x[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const int tok = gtb * 16 + (e < 4 ? 4 * lh + e : 8 + 4 * lh + (e - 4));
              x[e] = tok < a.N ? acc[i * FN + j][8 * tb + e] : 0.f;
            }
            u32x4 o;
            o.x = pack2_hw(x[0], x[1]);
            o.y = pack2_hw(x[2], x[3]);
            o.z = pack2_hw(x[4], x[5]);
            o.w = pack2_hw(x[6], x[7]);
            stream_store(&Cp[((int64_t)gtb * a.ccb + cb) * 64 + lane], o);
          }
        }
      }
  } else {
    // Row-major output: the wave's 128 x (32 FN) tile goes through LDS (the X stages are free
    // once every matrix wave has left the loop) so that global stores are 16 bytes per lane
    // along a row.  LDS tile: [128][32 FN] bf16, rows padded by 16 bytes.
    constexpr int TW = 32 * FN, TLD = TW * 2 + 16;
    bf16_t* out = fwd ? a.Y : a.C;
    const int64_t ldo = fwd ? a.ldy : a.ldc;
    const int ncols = fwd ? a.m : a.c;
    __builtin_amdgcn_s_barrier();  // the loader waves have exited; they no longer count
    unsigned char* tile = smem_raw + wave * (128 * TLD);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        asm volatile("" : "+a"(acc[i * FN + j]) : : "memory");
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = i * 32 + 8 * (v / 4) + 4 * lh + (v % 4);
          *reinterpret_cast<bf16_t*>(tile + row * TLD + (j * 32 + li) * 2) =
              (bf16_t)(pack2_hw(acc[i * FN + j][v], 0.f) & 0xFFFFu);
        }
      }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    constexpr int CPR = TW / 8;  // 16-byte chunks per row
    const int n0 = cb0 * 32;
    const bool vec_ok = (ldo % 8 == 0) && ((reinterpret_cast<uintptr_t>(out) & 15) == 0);
#pragma unroll
    for (int it = 0; it < 128 * CPR / 64; ++it) {
      const int q = it * 64 + lane, row = q / CPR, ch = q % CPR;
      const int mrow = m0 + row, n = n0 + ch * 8;
      if (mrow < a.N && n < ncols) {
        const u32x4 val = *reinterpret_cast<const u32x4*>(tile + row * TLD + ch * 16);
        bf16_t* o = out + (int64_t)mrow * ldo + n;
        if (vec_ok && n + 8 <= ncols) {
          *reinterpret_cast<u32x4*>(o) = val;
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (n + e < ncols) o[e] = (bf16_t)((val[e >> 1] >> (16 * (e & 1))) & 0xFFFFu);
        }
      }
    }
  }
#ifdef PRAC_WS_TIMESTAMPS
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  PRAC_STAMP(a, 3);
#endif
}

// ------------------------------------------------------------------ reconstruction
// X~ = C Ps^T (Section 5.1; first step of the backward pass in Alg. 2) for c <= 256: the K dimension
// is one k-tile.  A workgroup owns 128 token rows: its C tile is put into LDS once, then the
// matrix waves walk over the column groups (256 columns of X~ each, 64 per wave) with the same
// k-blocks as the compress kernel, Ps^T streaming through the fragment ring.  The MFMA operands
// are swapped (the fragment of Ps^T is the A operand), so that a lane ends up with four
// consecutive columns of one token row per accumulator quad: after each group the matrix waves
// write their tile as bf16 into an LDS staging tile (8 bytes per lane and store), and the other
// four waves - idle once C is in LDS - read it back along rows and store 16 bytes per lane to
// HBM, with their own memory counter, while the matrix waves multiply the next group.
struct ReconWsArgs {
  const bf16_t* C;       // row-major N x c, or packed [ceil(N/128)*8][ccb][64][8] (see CtdyWsArgs)
  int64_t ldc;
  int packed, ccb;
  int N, c, d;
  const bf16_t* Ptfrag;  // [16][ncb][64][8]: fragments of Ps^T (k-block over c, 32-column block over d)
  int ncb;               // multiple of 8
  bf16_t* Xh;            // row-major N x d
  int64_t ldxh;
  int tiles_m;
  int groups;            // ceil(d / 256)
};

// kblock2 with the operand roles swapped: acc[2 i + j] += b_j (as A) * fa[i] (as B).  ZERO: the
// accumulators start from zero instead of their old contents (first k-block of a column group).
template <int O, int VM, bool ZERO>
__device__ __forceinline__ void kblock2t(f32x16 (&acc)[8], const u32x4 (&fa)[4], u32x4 (&fn)[4], const u32x4& b0,
                                         const u32x4& b1, unsigned lds, u32x4& n0, u32x4& n1, uint32_t voff,
                                         const char* src) {
  if constexpr (ZERO) {
    asm volatile(
        "s_waitcnt vmcnt(%27)\n"
        "global_load_dwordx4 %12, %21, %22\n"
        "global_load_dwordx4 %13, %21, %22 offset:1024\n"
        "ds_read_b128 %8, %20 offset:%23\n"
        "v_mfma_f32_32x32x16_bf16 %0, %18, %14, 0\n"
        "ds_read_b128 %9, %20 offset:%24\n"
        "v_mfma_f32_32x32x16_bf16 %1, %19, %14, 0\n"
        "ds_read_b128 %10, %20 offset:%25\n"
        "v_mfma_f32_32x32x16_bf16 %2, %18, %15, 0\n"
        "ds_read_b128 %11, %20 offset:%26\n"
        "v_mfma_f32_32x32x16_bf16 %3, %19, %15, 0\n"
        "v_mfma_f32_32x32x16_bf16 %4, %18, %16, 0\n"
        "v_mfma_f32_32x32x16_bf16 %5, %19, %16, 0\n"
        "v_mfma_f32_32x32x16_bf16 %6, %18, %17, 0\n"
        "v_mfma_f32_32x32x16_bf16 %7, %19, %17, 0\n"
        "s_waitcnt lgkmcnt(0)\n"
        : "=&a"(acc[0]), "=&a"(acc[1]), "=&a"(acc[2]), "=&a"(acc[3]), "=&a"(acc[4]), "=&a"(acc[5]), "=&a"(acc[6]),
          "=&a"(acc[7]), "=&v"(fn[0]), "=&v"(fn[1]), "=&v"(fn[2]), "=&v"(fn[3]), "=&v"(n0), "=&v"(n1)
        : "v"(fa[0]), "v"(fa[1]), "v"(fa[2]), "v"(fa[3]), "v"(b0), "v"(b1), "v"(lds), "v"(voff), "s"(src), "n"(O),
          "n"(O + WS_RB), "n"(O + 2 * WS_RB), "n"(O + 3 * WS_RB), "n"(VM)
        : "memory");
  } else {
    asm volatile(
        "s_waitcnt vmcnt(%27)\n"
        "global_load_dwordx4 %12, %21, %22\n"
        "global_load_dwordx4 %13, %21, %22 offset:1024\n"
        "ds_read_b128 %8, %20 offset:%23\n"
        "v_mfma_f32_32x32x16_bf16 %0, %18, %14, %0\n"
        "ds_read_b128 %9, %20 offset:%24\n"
        "v_mfma_f32_32x32x16_bf16 %1, %19, %14, %1\n"
        "ds_read_b128 %10, %20 offset:%25\n"
        "v_mfma_f32_32x32x16_bf16 %2, %18, %15, %2\n"
        "ds_read_b128 %11, %20 offset:%26\n"
        "v_mfma_f32_32x32x16_bf16 %3, %19, %15, %3\n"
        "v_mfma_f32_32x32x16_bf16 %4, %18, %16, %4\n"
        "v_mfma_f32_32x32x16_bf16 %5, %19, %16, %5\n"
        "v_mfma_f32_32x32x16_bf16 %6, %18, %17, %6\n"
        "v_mfma_f32_32x32x16_bf16 %7, %19, %17, %7\n"
        "s_waitcnt lgkmcnt(0)\n"
        : "+a"(acc[0]), "+a"(acc[1]), "+a"(acc[2]), "+a"(acc[3]), "+a"(acc[4]), "+a"(acc[5]), "+a"(acc[6]),
          "+a"(acc[7]), "=&v"(fn[0]), "=&v"(fn[1]), "=&v"(fn[2]), "=&v"(fn[3]), "=&v"(n0), "=&v"(n1)
        : "v"(fa[0]), "v"(fa[1]), "v"(fa[2]), "v"(fa[3]), "v"(b0), "v"(b1), "v"(lds), "v"(voff), "s"(src), "n"(O),
          "n"(O + WS_RB), "n"(O + 2 * WS_RB), "n"(O + 3 * WS_RB), "n"(VM)
        : "memory");
  }
}

constexpr int RW_OLD = 512 + 16;              // bytes per token row of the output staging tile
constexpr int RW_OUT = WS_STAGE;              // it follows the C stage in LDS
constexpr int RW_SMEM = WS_STAGE + WS_BM * RW_OLD;

__global__ __launch_bounds__(512) void reconstruct_ws_kernel(ReconWsArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const int bid = touch_kernel_args<sizeof(ReconWsArgs)>(blockIdx.x);
  const int per_xcd = (a.tiles_m + 7) / 8;
  const int xcd = bid & 7, slot = bid >> 3;
  const int tm = xcd * per_xcd + slot;
  if (slot >= per_xcd || tm >= a.tiles_m) return;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m0 = tm * WS_BM;
  const int G = a.groups;

  if (wave >= 4) {
    // ------------------------------------------------ loader, then store waves
    const int lt = tid - 256;
    const int crow = lt >> 5, ccol = (lt & 31) * 8;  // row crow + 8 q, 16-byte chunk at column ccol
    if (a.packed) {
      // Packed C holds, per lane slot, 8 tokens of one column; the tile needs 8 columns of one token per
      // 16 bytes.  A thread takes 8 x 8 patches: 8 consecutive column slots (128 contiguous bytes),
      // transposed in registers as the C^T dY loader does for dY.  Patch p of the tile's 512:
      // column octet o = p & 3, token half h = (p >> 2) & 1, column block cb = (p >> 3) & 7, token block tb = p >> 6.
      const u32x4* Cp = reinterpret_cast<const u32x4*>(a.C);
#pragma unroll
      for (int pp = 0; pp < 2; ++pp) {
        const int p = lt + 256 * pp;
        const int o = p & 3, h = (p >> 2) & 1, cb = (p >> 3) & 7, tb = p >> 6;
        u32x4 rr[8];
        const bool live = cb < a.ccb;  // column blocks past c are zero in the tile
        const int64_t base = ((int64_t)((m0 >> 4) + tb) * a.ccb + (live ? cb : 0)) * 64 + h * 32 + 8 * o;
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) rr[jj] = Cp[base + jj];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          // token slot e of the patch: 16-bit element e of each of the 8 column slots
          uint32_t w[4];
#pragma unroll
          for (int e2 = 0; e2 < 4; ++e2) {
            const uint32_t lo = rr[2 * e2][e >> 1], hi = rr[2 * e2 + 1][e >> 1];
            w[e2] = __builtin_amdgcn_perm(hi, lo, (e & 1) ? 0x07060302u : 0x05040100u);
          }
          const int row = 16 * tb + (e < 4 ? 4 * h + e : 8 + 4 * h + (e - 4));
          u32x4 v = {w[0], w[1], w[2], w[3]};
          if (!live) v = u32x4{0u, 0u, 0u, 0u};
          *reinterpret_cast<u32x4*>(smem_raw + (row * WS_LD + 32 * cb + 8 * o) * 2) = v;
        }
      }
    } else {
      const char* cbase = reinterpret_cast<const char*>(a.C + (int64_t)m0 * a.ldc);
      const int last_chunk = ((a.c - 1) / 8) * 8;
      const int nv = a.c - ccol;  // valid columns of this thread's chunk (<= 0: none)
      u32x4 rc[16];
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int row = min(m0 + crow + 8 * q, a.N - 1) - m0;  // rows past N repeat the last one, never stored
        rc[q] = *reinterpret_cast<const u32x4*>(cbase + ((int64_t)row * a.ldc + min(ccol, last_chunk)) * 2);
      }
      unsigned char* st = smem_raw + (crow * WS_LD + ccol) * 2;
#pragma unroll
      for (int q = 0; q < 16; ++q)
        *reinterpret_cast<u32x4*>(st + q * (8 * WS_LD * 2)) = nv >= 8 ? rc[q] : keep_first(rc[q], nv > 0 ? nv : 0);
    }
    __syncthreads();  // the C tile is in LDS
    // From here on plain barriers (no memory fence: a fence would wait for this wave's own stores
    // to HBM); LDS traffic is ordered by explicit waits, and the empty statements keep the
    // compiler from moving memory accesses across them.
    __builtin_amdgcn_s_barrier();  // staging tile free (first group)
    const bool vec_ok = (a.ldxh % 8 == 0) && ((reinterpret_cast<uintptr_t>(a.Xh) & 15) == 0);
    for (int g = 0; g < G; ++g) {
      __builtin_amdgcn_s_barrier();  // staging tile holds group g
      asm volatile("" ::: "memory");
      u32x4 ro[16];
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        ro[q] = *reinterpret_cast<const u32x4*>(smem_raw + RW_OUT + (crow + 8 * q) * RW_OLD + ccol * 2);
        // rows 8 .. 15 (mod 16) are staged with the 8-byte halves of every 16 bytes swapped (see the writers)
        if (q & 1) ro[q] = u32x4{ro[q].z, ro[q].w, ro[q].x, ro[q].y};
      }
      const int n = g * 256 + ccol;
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int mrow = m0 + crow + 8 * q;
        if (mrow < a.N && n < a.d) {
          bf16_t* o = a.Xh + (int64_t)mrow * a.ldxh + n;
          if (vec_ok && n + 8 <= a.d) {
            *reinterpret_cast<u32x4*>(o) = ro[q];  // (plain: the streaming hint costs this kernel 8 us of its 46)
          } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
              if (n + e < a.d) o[e] = (bf16_t)((ro[q][e >> 1] >> (16 * (e & 1))) & 0xFFFFu);
          }
        }
      }
      // the stores above have read their registers, hence the LDS reads are complete
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      if (g + 1 < G) __builtin_amdgcn_s_barrier();  // staging tile free again
    }
    return;
  }

  // -------------------------------------------------------------- matrix waves
  const int lane = tid & 63, li = lane & 31, lh = lane >> 5;
  const char* pbase = reinterpret_cast<const char*>(a.Ptfrag);
  const uint32_t boff = (uint32_t)(wave * 2 * 64 + lane) * 16u;  // this wave's two column blocks of a group
  const int64_t brow = (int64_t)a.ncb * 1024;                    // bytes per k-block of fragments
  f32x16 acc[8];
  // ring as in the compress kernel; a "tile" is a column group, 8 blocks (8 KB) further along each k-block row
  u32x4 rb[8][2];
  auto group_base = [&](int g) { return pbase + (g < G ? (int64_t)g * 8192 : (int64_t)0); };  // uniform
  const char* preq = group_base(0);
  const char* next_base = group_base(1);
#pragma unroll
  for (int kk = 0; kk < 7; ++kk) {
    ring_request<0>(rb[kk][0], boff, preq);
    ring_request<1024>(rb[kk][1], boff, preq);
    preq += brow;
  }
  constexpr int VM = 12;
#define PRAC_IC(v) std::integral_constant<int, (v)> {}
  auto kblock = [&](auto oc, const u32x4 (&fcur)[4], u32x4 (&fnext)[4], auto kkc, unsigned lds) {
    constexpr int O = decltype(oc)::value, KK = decltype(kkc)::value;
    kblock2t<O, VM, KK == 0>(acc, fcur, fnext, rb[KK & 7][0], rb[KK & 7][1], lds, rb[(KK + 7) & 7][0],
                             rb[(KK + 7) & 7][1], boff, preq);
    if constexpr (KK == 8) preq = next_base;
    else preq += brow;
  };
  const unsigned lds0 =
      (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem_raw + (unsigned)(li * WS_LD * 2 + lh * 16);
  u32x4 fa[4], fb[4];
  __builtin_amdgcn_s_barrier();  // the C tile is in LDS
  frag_read4(fa, lds0);
  // staging address of this lane: token row li (+ 32 i), columns 64 wave (+ 32 j + 8 q) + 4 lh .. + 3
  // (a row is 528 bytes: lanes li and li + 8 of an 8-byte store would meet in the same banks, so
  // rows 8 .. 15 of every 16 swap the two 8-byte halves of each 16 bytes)
  unsigned char* const orow = smem_raw + RW_OUT + li * RW_OLD + (((wave * 64 + 4 * lh) * 2) ^ (((li >> 3) & 1) << 3));
  for (int g = 0; g < G; ++g) {
    static_for<WS_KB>([&](auto jc) {
      constexpr int J = decltype(jc)::value;
      // the fragments read during k-block 15 are those of k-block 0 again: the next group's first
      if constexpr (J % 2 == 0) kblock(PRAC_IC(32 * ((J + 1) % WS_KB)), fa, fb, jc, lds0);
      else kblock(PRAC_IC(32 * ((J + 1) % WS_KB)), fb, fa, jc, lds0);
    });
    next_base = group_base(g + 2);
    // The matrix pipeline and the ring are drained before compiler-scheduled code runs (see the
    // compress kernel): the code below needs registers, and the compiler may only move or spill
    // ring registers whose requests have landed.  The ring then holds the next group's first
    // seven k-blocks, so the matrix pipeline restarts at once after the tile is staged.
    drain_mfma<8, 2>(acc, rb);
    __builtin_amdgcn_s_barrier();  // staging tile free
    asm volatile("" ::: "memory");
    // block (i, j) = acc[2 i + j]: register v of lane (li, lh) is token row 32 i + li, column
    // 32 j + 8 (v / 4) + 4 lh + v % 4 of the wave's 64
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        // one block at a time leaves the accumulator registers (keeps the copies short-lived)
        asm volatile("" : "+a"(acc[2 * i + j]) : : "memory");
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          uint2 w;
          w.x = pack2_hw(acc[2 * i + j][4 * q], acc[2 * i + j][4 * q + 1]);
          w.y = pack2_hw(acc[2 * i + j][4 * q + 2], acc[2 * i + j][4 * q + 3]);
          *reinterpret_cast<uint2*>(orow + i * 32 * RW_OLD + (j * 32 + q * 8) * 2) = w;
        }
      }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();  // staging tile holds group g
  }
#undef PRAC_IC
}

// ----------------------------------------------------------------------- C^T dY
// Token-split partial sums of T = C^T dY (Lemma 1, reassociated), same workgroup shape:
//   loader waves   stream dY tiles (128 tokens x 128 columns), transpose each 8 x 8 patch in
//                  registers and store the tile into LDS already in MFMA fragment order;
//   matrix waves   read those B fragments from LDS (shared by all four waves), fetch their own
//                  A fragments (packed C, L2-resident) straight into registers, issue MFMAs.
// LDS stage: [k-block 0..7][column block 0..3][64 lanes][16 bytes].  Column block nb holds the
// tile's columns 4 j + nb (j = 0..31), so that a lane's four accumulators of one row are four
// consecutive columns of T.  Lane slot (j, h) sits at 16-byte slot h*32 + (j ^ ((j >> 3) & 1)) of its
// 1 KB block.  A 16-byte LDS access is served eight lanes at a time (8 x 16 bytes = the 32 banks):
// eight consecutive lanes of a fragment read (j = 8 g .. 8 g + 7) get the eight slots of one
// 128-byte line, and eight consecutive loader lanes, which write every other column slot
// (j = 2 cc + u), get eight slots that differ modulo 8 - neither has a bank conflict.
// Element e of lane half h is token 16 kb + (e < 4 ? 4 h + e : 8 + 4 h + e - 4), the slot order of
// packed C, so both operands list the tokens of a k-block in the same order.
struct CtdyWsArgs {
  const bf16_t* Cpk;   // packed compressed activation [ntb][ccb][64][8]
  int ccb;             // 32-column blocks of C
  int c;
  int N;
  // up to PRAC_CTDY_MAX_OUT gradients dY_h (N x m_h) that share C (layers reading the same input,
  // Section 5.1): output h owns the column tiles tile0[h] .. tile0[h+1]-1 of the launch
  int n_out;
  const bf16_t* dY[PRAC_CTDY_MAX_OUT];
  int64_t lddy[PRAC_CTDY_MAX_OUT];
  int m[PRAC_CTDY_MAX_OUT];
  int tile0[PRAC_CTDY_MAX_OUT + 1];
  float* slabs[PRAC_CTDY_MAX_OUT];  // [splits][c][m_h] each
  int splits;
  int tok_per_split;   // multiple of 128
  int tiles_n;         // column tiles of 128 over all outputs
  int row_groups;      // groups of 8 column blocks (256 rows of T) over c
  int groups_per_xcd;  // MODE > 0: column tiles per XCD
  // ---- whole weight gradient in this launch (MODE > 0): the workgroups of one column tile sum their
  // partial slabs into T (bf16, fragment order, random rows scaled) and form dW = P T for that tile
  int* cnt;            // 3 counters per column tile, zero before the launch, zero again after it
  int* fail;           // set to 4 if a wait between workgroups gave up (bits 1 and 2 belong to the basis fit)
  int nckb;            // 16-row k-blocks of T = ceil(c / 16)
  int k_lo;            // rows >= k_lo of T carry scale_hi
  float scale_hi;
  bf16_t* Tf[PRAC_CTDY_MAX_OUT];   // [nckb][nmb_h][64][8]
  int nmb[PRAC_CTDY_MAX_OUT];
  const bf16_t* Pa;    // P as an A operand in fragment order [nrb][nckb][64][8]
  int d;
  void* dW[PRAC_CTDY_MAX_OUT];
  int64_t lddw[PRAC_CTDY_MAX_OUT];
  int vec_ok[PRAC_CTDY_MAX_OUT];   // dW rows allow aligned 16-byte accesses
  float beta;
#ifdef PRAC_WS_TIMESTAMPS
  long long* stamps;   // development builds only: 8 wall-clock stamps per workgroup
#endif
};


constexpr int CW_BK = 128, CW_BN = 128;
constexpr int CW_STAGE = 8 * 4 * 1024;  // bytes per LDS stage
constexpr int CW_STAGES = 3;

// One k-block of a 64 x 128 wave tile: acc[4 i + j] += a_i * f_j, while the four B fragments at
// byte offsets O + 1024 nb from `lds` are read into fn.  Like the compress kernel's blocks it
// issues the two requests that refill another slot of the ring of C fragments (n0 <- src + v0,
// n1 <- src + v1) and starts with its own wait for the fragments it multiplies.
template <int O, int VM>
__device__ __forceinline__ void kblock_ct(f32x16 (&acc)[8], const u32x4 (&fc)[4], u32x4 (&fn)[4], const u32x4& a0,
                                          const u32x4& a1, unsigned lds, u32x4& n0, u32x4& n1, uint32_t v0,
                                          uint32_t v1, const char* src) {
  asm volatile(
      "s_waitcnt vmcnt(%28)\n"
      "global_load_dwordx4 %12, %21, %23\n"
      "global_load_dwordx4 %13, %22, %23\n"
      "ds_read_b128 %8, %20 offset:%24\n"
      "v_mfma_f32_32x32x16_bf16 %0, %18, %14, %0\n"
      "ds_read_b128 %9, %20 offset:%25\n"
      "v_mfma_f32_32x32x16_bf16 %4, %19, %14, %4\n"
      "ds_read_b128 %10, %20 offset:%26\n"
      "v_mfma_f32_32x32x16_bf16 %1, %18, %15, %1\n"
      "ds_read_b128 %11, %20 offset:%27\n"
      "v_mfma_f32_32x32x16_bf16 %5, %19, %15, %5\n"
      "v_mfma_f32_32x32x16_bf16 %2, %18, %16, %2\n"
      "v_mfma_f32_32x32x16_bf16 %6, %19, %16, %6\n"
      "v_mfma_f32_32x32x16_bf16 %3, %18, %17, %3\n"
      "v_mfma_f32_32x32x16_bf16 %7, %19, %17, %7\n"
      "s_waitcnt lgkmcnt(0)\n"
      : "+a"(acc[0]), "+a"(acc[1]), "+a"(acc[2]), "+a"(acc[3]), "+a"(acc[4]), "+a"(acc[5]), "+a"(acc[6]),
        "+a"(acc[7]), "=&v"(fn[0]), "=&v"(fn[1]), "=&v"(fn[2]), "=&v"(fn[3]), "=&v"(n0), "=&v"(n1)
      : "v"(fc[0]), "v"(fc[1]), "v"(fc[2]), "v"(fc[3]), "v"(a0), "v"(a1), "v"(lds), "v"(v0), "v"(v1), "s"(src), "n"(O),
        "n"(O + 1024), "n"(O + 2048), "n"(O + 3072), "n"(VM)
      : "memory");
}

__device__ __forceinline__ void frag_read4_ct(u32x4 (&f)[4], unsigned lds) {
  asm volatile(
      "ds_read_b128 %0, %4\n"
      "ds_read_b128 %1, %4 offset:1024\n"
      "ds_read_b128 %2, %4 offset:2048\n"
      "ds_read_b128 %3, %4 offset:3072\n"
      "s_waitcnt lgkmcnt(0)\n"
      : "=&v"(f[0]), "=&v"(f[1]), "=&v"(f[2]), "=&v"(f[3])
      : "v"(lds)
      : "memory");
}

__device__ __forceinline__ int c_slot_tok(int h, int e) { return e < 4 ? 4 * h + e : 8 + 4 * h + (e - 4); }
__device__ __forceinline__ int frag_slot(int j, int h) { return h * 32 + (j ^ ((j >> 3) & 1)); }


// ---- second half of the weight gradient, inside the same launch --------------------------------
// The `members` workgroups that hold partial sums of one 128-column tile of T meet twice: once all
// partial slabs are written, each of them sums a share of the tile's 16-row k-blocks over the slabs
// (in slab order, so the result does not depend on who arrives when), scales the random rows and
// writes them as bf16 in fragment order; once all of T's tile is written, each of them forms a share
// of the 128-row tiles of dW[:, tile] = P T[:, tile].
//
// The members of a tile have neighbouring slots on one XCD (workgroup i of a launch runs on XCD i mod 8),
// so what they hand to each other stays in that XCD's L2, which is coherent for its compute units:
// ordinary stores, a wait for their acknowledgement, a counter, ordinary loads.  That placement is
// not promised by anything, so it is checked: at the first meeting every member adds the number of
// the XCD it runs on (hardware register XCC_ID) and its square into the tile's counter word; all
// members read the same final word and all are on one XCD exactly when n * sum(x^2) == (sum x)^2.  If
// they are not, the tile takes the slow route: one thread per member writes its XCD's dirty lines back
// (a cache-wide operation, tens of microseconds when many workgroups do it), the members meet again,
// and the loads bypass the caches.
//
// The host launches at most one workgroup per compute unit of an XCD, so all members are resident and
// the waits end; a wait that does not (a device shared with something that never finishes) gives up
// after about a second, sets *fail and lets the workgroup run on to its exit, so the grid always drains.
constexpr int WG_SPIN_LIMIT = 1 << 22;
constexpr int WG_PATCH_LD = 128 + 4;            // floats per row of the 16 x 128 reduction patch
constexpr int WG_T_BYTES = 16 * 4 * 1024;       // one chunk of T in LDS: 16 k-blocks x 4 column blocks
constexpr int WG_STAGE_LD = 64 + 4;             // floats per row of a wave's 32 x 64 output staging tile
constexpr int WG_SMEM = WG_T_BYTES + 8 * 32 * WG_STAGE_LD * 4 + 16;  // + the flag of the first meeting
constexpr int WG_CNT_INTS = 8;                  // counters per column tile: [0:1] first meeting (64 bit), [2] its
                                                // repeat on the slow route, [3] second meeting, [4] leavers
constexpr int BUF_FLAGS = 0x00020000;  // raw buffer descriptor, 32-bit data format
constexpr int DEV_SCOPE = 16;          // cache policy bit sc1 of the raw buffer builtins: device scope
constexpr int HWREG_XCC_ID = 20 | (0 << 6) | (3 << 11);  // s_getreg operand: register 20, bits 3:0

__device__ __forceinline__ __amdgpu_buffer_rsrc_t dev_buffer(const void* base, size_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)(bytes > 0xFFFFFFFFu ? 0xFFFFFFFFu : bytes),
                                           BUF_FLAGS);
}
// 16 / 4 bytes through the XCD's caches (`local`) or past them
__device__ __forceinline__ u32x4 tail_load16(__amdgpu_buffer_rsrc_t r, uint32_t off, bool local) {
  return local ? __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0) : __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, DEV_SCOPE);
}
__device__ __forceinline__ float tail_load4(__amdgpu_buffer_rsrc_t r, uint32_t off, bool local) {
  return __uint_as_float(local ? __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, 0)
                               : __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, DEV_SCOPE));
}

__device__ __forceinline__ void spin_until(int* cnt, int members, int* fail) {
  int spins = 0;
  while (__hip_atomic_load(cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < members) {
    __builtin_amdgcn_s_sleep(2);
    if (++spins > WG_SPIN_LIMIT) {
      __hip_atomic_store(fail, 4, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      break;
    }
  }
}

// First meeting: every member's slab is written.  Returns whether all members share one XCD.
__device__ __forceinline__ bool group_meet_first(int* cnt, int members, int* fail, int* lds_flag) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's stores are acknowledged by L2
  __syncthreads();
  if (threadIdx.x == 0) {
    int local = 1;
    if (members > 1) {
      unsigned long long* c64 = reinterpret_cast<unsigned long long*>(cnt);
      const unsigned long long x = (unsigned long long)(__builtin_amdgcn_s_getreg(HWREG_XCC_ID) & 15);
      __hip_atomic_fetch_add(c64, 1ull + (x << 16) + ((x * x) << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      unsigned long long w;
      int spins = 0;
      while (((w = __hip_atomic_load(c64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) & 0xFFFFull) <
             (unsigned long long)members) {
        __builtin_amdgcn_s_sleep(2);
        if (++spins > WG_SPIN_LIMIT) {
          __hip_atomic_store(fail, 4, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          break;
        }
      }
      const unsigned long long n = w & 0xFFFFull, sx = (w >> 16) & 0xFFFFull, sxx = w >> 32;
      local = (n * sxx == sx * sx) ? 1 : 0;
      if (!local) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");  // this XCD's dirty lines go to memory
        __hip_atomic_fetch_add(cnt + 2, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        spin_until(cnt + 2, members, fail);
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      }
    }
    *lds_flag = local;
  }
  __syncthreads();
  return *lds_flag != 0;
}

// Second meeting: every member's share of T is written.
__device__ __forceinline__ void group_meet_second(int* cnt, int members, int* fail, bool local) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (members > 1 && threadIdx.x == 0) {
    if (!local) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    __hip_atomic_fetch_add(cnt + 3, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    spin_until(cnt + 3, members, fail);
    if (!local) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    // the last member past this meeting leaves the counters as the next launch expects them
    if (__hip_atomic_fetch_add(cnt + 4, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == members - 1) {
#pragma unroll
      for (int i = 0; i < 5; ++i) __hip_atomic_store(cnt + i, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  __syncthreads();
}

template <bool OUT_BF16>
__device__ __forceinline__ void wgrad_tail(const CtdyWsArgs& a, unsigned char* smem, int tn, int h, int n0, int member,
                                           int members) {
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  int* cnt = a.cnt + WG_CNT_INTS * tn;
  const int mh = a.m[h], nmb = a.nmb[h], nb0 = n0 >> 5, nckb = a.nckb;
  const __amdgpu_buffer_rsrc_t rt = dev_buffer(a.Tf[h], (size_t)nckb * nmb * 1024);  // T_h, 1 KB per block

  PRAC_STAMP(a, 1);
  // every partial slab of this column tile is written
  const bool local = group_meet_first(cnt, members, a.fail, reinterpret_cast<int*>(smem + WG_SMEM - 16));
  PRAC_STAMP(a, 2);

  {  // T[16 kb .. 16 kb + 15, n0 .. n0 + 127] for this member's k-blocks
    const uint32_t slab = (uint32_t)a.c * (uint32_t)mh * 4u;  // bytes per slab (all slabs together stay below 4 GB)
    const __amdgpu_buffer_rsrc_t rs = dev_buffer(a.slabs[h], (size_t)slab * a.splits);
    float* patch = reinterpret_cast<float*>(smem);
    const int row = tid >> 5, col = (tid & 31) * 4;
    for (int kb = member; kb < nckb; kb += members) {
      const int k = kb * 16 + row, n = n0 + col;
      float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
      if (k < a.c && n < mh) {
        const uint32_t off = ((uint32_t)k * (uint32_t)mh + (uint32_t)n) * 4u;
        if (n + 3 < mh && (mh & 3) == 0) {
          // 16 slabs requested at once (one round trip), summed in slab order
          for (int z0 = 0; z0 < a.splits; z0 += 16) {
            u32x4 v[16];
#pragma unroll
            for (int z = 0; z < 16; ++z) v[z] = tail_load16(rs, off + (uint32_t)min(z0 + z, a.splits - 1) * slab, local);
#pragma unroll
            for (int z = 0; z < 16; ++z)
              if (z0 + z < a.splits) {
                sum.x += __uint_as_float(v[z].x); sum.y += __uint_as_float(v[z].y);
                sum.z += __uint_as_float(v[z].z); sum.w += __uint_as_float(v[z].w);
              }
          }
        } else {
          for (int z = 0; z < a.splits; ++z) {
            const uint32_t o = off + (uint32_t)z * slab;
            sum.x += tail_load4(rs, o, local);
            if (n + 1 < mh) sum.y += tail_load4(rs, o + 4, local);
            if (n + 2 < mh) sum.z += tail_load4(rs, o + 8, local);
            if (n + 3 < mh) sum.w += tail_load4(rs, o + 12, local);
          }
        }
        const float w = k >= a.k_lo ? a.scale_hi : 1.f;
        sum.x *= w; sum.y *= w; sum.z *= w; sum.w *= w;
      }
      *reinterpret_cast<float4*>(patch + row * WG_PATCH_LD + col) = sum;
      __syncthreads();
      if (tid < 256) {
        const int j = lane & 31, hh = lane >> 5;
        const float* q = patch + (8 * hh) * WG_PATCH_LD + wave * 32 + j;
        u32x4 o;
        o.x = pack2_hw(q[0], q[WG_PATCH_LD]);
        o.y = pack2_hw(q[2 * WG_PATCH_LD], q[3 * WG_PATCH_LD]);
        o.z = pack2_hw(q[4 * WG_PATCH_LD], q[5 * WG_PATCH_LD]);
        o.w = pack2_hw(q[6 * WG_PATCH_LD], q[7 * WG_PATCH_LD]);
        __builtin_amdgcn_raw_buffer_store_b128(o, rt, (uint32_t)(((kb * nmb + nb0 + wave) * 64 + lane) * 16), 0, 0);
      }
      __syncthreads();
    }
  }

  // the P fragments of this member's first dW tile do not depend on T: requested before the meeting
  const int tiles_m = (a.d + 127) / 128;
  const int wr = wave >> 1, wc = wave & 1;
  const u32x4* __restrict__ Pa = reinterpret_cast<const u32x4*>(a.Pa);
  u32x4 fa0[16];
  {
    const int64_t rb = (int64_t)min(member, tiles_m - 1) * 4 + wr;
#pragma unroll
    for (int q = 0; q < 16; ++q) fa0[q] = Pa[(rb * nckb + min(q, nckb - 1)) * 64 + lane];
  }
  PRAC_STAMP(a, 3);
  group_meet_second(cnt, members, a.fail, local);  // all of T[:, tile] is written
  PRAC_STAMP(a, 4);

  // dW[128 tm .. , n0 .. n0 + 127] = P[rows] T[:, tile]: 8 waves as 4 (row blocks) x 2 (column halves), each
  // 32 x 64.  T comes through LDS in chunks of 16 k-blocks (all of it when c <= 256), P straight from L2.
  const int nchunks = (nckb + 15) / 16;
  const int li = lane & 31, lh = lane >> 5;
  float* stage = reinterpret_cast<float*>(smem + WG_T_BYTES) + wave * (32 * WG_STAGE_LD);
  void* const odW = a.dW[h];
  const int64_t olddw = a.lddw[h];
  const int ovec = a.vec_ok[h];
  bool t_in_lds = false;
  for (int tm = member; tm < tiles_m; tm += members) {
    f32x16 acc0, acc1;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc0[v] = acc1[v] = 0.f;
    const int64_t rb = (int64_t)tm * 4 + wr;
    for (int ch = 0; ch < nchunks; ++ch) {
      const int kb0 = ch * 16, kbs = min(16, nckb - kb0);
      u32x4 fa[16];
      if (tm == member && ch == 0) {
#pragma unroll
        for (int q = 0; q < 16; ++q) fa[q] = fa0[q];
      } else {
#pragma unroll
        for (int q = 0; q < 16; ++q) fa[q] = Pa[(rb * nckb + min(kb0 + q, nckb - 1)) * 64 + lane];
      }
      if (!(nchunks == 1 && t_in_lds)) {
        __syncthreads();  // the previous chunk has been read
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int u = tid + 512 * i, blk = u >> 6, kbl = blk >> 2, nb = blk & 3;
          if (kbl < kbs)
            *reinterpret_cast<u32x4*>(smem + u * 16) =
                tail_load16(rt, (uint32_t)((((kb0 + kbl) * nmb + nb0 + nb) * 64 + (u & 63)) * 16), local);
        }
        __syncthreads();
        t_in_lds = true;
      }
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        if (q < kbs) {
          const u32x4 b0 = *reinterpret_cast<const u32x4*>(smem + (q * 4 + wc * 2) * 1024 + lane * 16);
          const u32x4 b1 = *reinterpret_cast<const u32x4*>(smem + (q * 4 + wc * 2 + 1) * 1024 + lane * 16);
          acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(fa[q]), as_frag(b0), acc0, 0, 0, 0);
          acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(fa[q]), as_frag(b1), acc1, 0, 0, 0);
        }
      }
    }
    // register v of lane (li, lh): row 8 (v / 4) + 4 lh + v % 4 of the wave's 32, column li (acc0) / 32 + li (acc1)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = 8 * (v / 4) + 4 * lh + (v % 4);
      stage[row * WG_STAGE_LD + li] = acc0[v];
      stage[row * WG_STAGE_LD + 32 + li] = acc1[v];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int row0 = tm * 128 + wr * 32, col0 = n0 + wc * 64;
    if (OUT_BF16) {
      const int er = lane >> 3, ec = (lane & 7) * 8;  // 8 lanes per row (16 bytes each), 8 rows per pass
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const int row = er + 8 * p, grow = row0 + row, gcol = col0 + ec;
        const float4 lo = *reinterpret_cast<const float4*>(stage + row * WG_STAGE_LD + ec);
        const float4 hi = *reinterpret_cast<const float4*>(stage + row * WG_STAGE_LD + ec + 4);
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
      const int er = lane >> 4, ec = (lane & 15) * 4;  // 16 lanes per row (16 bytes each), 4 rows per pass
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        const int row = er + 4 * p, grow = row0 + row, gcol = col0 + ec;
        float4 x = *reinterpret_cast<const float4*>(stage + row * WG_STAGE_LD + ec);
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

// MODE 0: partial slabs only; 1 / 2: the whole weight gradient (dW in fp32 / bf16)
template <int MODE>
__global__ __launch_bounds__(512) void ctdy_ws_kernel(CtdyWsArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const int bid = touch_kernel_args<(MODE == 0 ? offsetof(CtdyWsArgs, cnt) : sizeof(CtdyWsArgs))>(blockIdx.x);

  int tn, rg, split;
  if constexpr (MODE == 0) {
    const int per_split = a.tiles_n * a.row_groups;
    const int total = per_split * a.splits;
    const int per_xcd = (total + 7) / 8;
    const int xcd = bid & 7, slot = bid >> 3;
    const int logical = xcd * per_xcd + slot;
    if (slot >= per_xcd || logical >= total) return;
    tn = logical % a.tiles_n;
    rg = (logical / a.tiles_n) % a.row_groups;
    split = logical / per_split;
  } else {
    // the workgroups of a column tile (its token ranges and row groups) take neighbouring slots of one XCD
    const int members = a.splits * a.row_groups;
    const int per_xcd = a.groups_per_xcd * members;
    const int xcd = bid & 7, slot = bid >> 3;
    tn = xcd * a.groups_per_xcd + slot / members;
    if (slot >= per_xcd || tn >= a.tiles_n) return;
    const int member = slot % members;
    rg = member % a.row_groups;
    split = member / a.row_groups;
  }

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  PRAC_STAMP(a, 0);
  // which output this column tile belongs to
  int h = 0;
#pragma unroll
  for (int q = 1; q < PRAC_CTDY_MAX_OUT; ++q)
    if (q < a.n_out && tn >= a.tile0[q]) h = q;
  const bf16_t* const dYh = a.dY[h];
  const int64_t lddyh = a.lddy[h];
  const int mh = a.m[h];
  const int n0 = (tn - a.tile0[h]) * CW_BN;
  const int tok_beg = split * a.tok_per_split;
  const int tok_end = min(a.N, tok_beg + a.tok_per_split);
  const int nk = tok_end > tok_beg ? (tok_end - tok_beg + CW_BK - 1) / CW_BK : 0;
  // All workgroups of a split walk its tiles in the same order: they then ask for the same blocks
  // of packed C at about the same time, which keeps those blocks in L2 between uses.

  if (wave >= 4) {
    // ------------------------------------------------------------ loader waves
    if (nk > 0) {
    const int lt = tid - 256;
    const int cc = lt & 15, tg = lt >> 4, kb = tg >> 1, h = tg & 1;
    const int last_chunk = ((mh - 1) / 8) * 8;
    const char* ycol = reinterpret_cast<const char*>(dYh) + (int64_t)min(n0 + 8 * cc, last_chunk) * 2;
    const uint32_t rowb = (uint32_t)lddyh * 2u;
    // LDS byte offsets of the two lane slots this thread fills (columns 8 cc + j: j < 4 and j >= 4)
    const uint32_t sA = (uint32_t)(kb * 4096 + frag_slot(2 * cc, h) * 16);
    const uint32_t sB = (uint32_t)(kb * 4096 + frag_slot(2 * cc + 1, h) * 16);

    u32x4 ry[8], rz[8];
    // rows past N re-read the last row (finite data) and meet the zero padding of packed C
    auto gload = [&](int kt, u32x4 (&rr)[8]) {
      const bool live = kt < nk;
      const int t0 = tok_beg + min(kt, nk - 1) * CW_BK;
      const char* base = ycol + (int64_t)t0 * lddyh * 2;  // uniform part + this thread's column
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int row = min(16 * kb + c_slot_tok(h, e), a.N - 1 - t0);
        rr[e] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + (live ? (uint32_t)row * rowb : 0u)));
      }
    };
    auto sstore = [&](int stage, const u32x4 (&rr)[8]) {
      unsigned char* s = smem_raw + stage * CW_STAGE;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        // column j of the 8 x 8 patch: 16-bit element j of each of the 8 token rows
        u32x4 o;
        uint32_t w[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
          const uint32_t lo = rr[2 * e2][j >> 1], hi = rr[2 * e2 + 1][j >> 1];
          w[e2] = __builtin_amdgcn_perm(hi, lo, (j & 1) ? 0x07060302u : 0x05040100u);
        }
        o.x = w[0]; o.y = w[1]; o.z = w[2]; o.w = w[3];
        *reinterpret_cast<u32x4*>(s + ((j & 3) * 1024 + (j < 4 ? sA : sB))) = o;
      }
    };
    // the first two tiles are requested together; afterwards one tile is in flight per loader thread and two
    // more are complete in LDS
    gload(0, ry);
    gload(1, rz);
    sstore(0, ry);
    gload(2, ry);
    // The matrix waves start as soon as tile 0 is in LDS: at a kernel's start all workgroups ask for their
    // first tiles at once, and what holds the first multiplication back is the time HBM needs to deliver
    // them (8 MB per tile over the 256 workgroups of the headline shape).  Tile 1 is first read at k-block 7
    // of tile 0, behind the loop's first barrier, and is stored before that barrier.
    __syncthreads();  // tile 0 is in LDS
    if (nk > 1) sstore(1, rz);
    int stage = 2;
    for (int kt = 0; kt < nk; ++kt) {
      if (kt + 2 < nk) sstore(stage, ry);
      stage = stage == CW_STAGES - 1 ? 0 : stage + 1;
      gload(kt + 3, ry);
      __syncthreads();
    }
    }
    if constexpr (MODE == 0) return;
  } else {
  // -------------------------------------------------------------- matrix waves
  const int lane = tid & 63, li = lane & 31, lh = lane >> 5;
  const int cb0 = rg * 8 + wave * 2;  // this wave's two 32-row blocks of T (column blocks of C)
  f32x16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

  if (nk > 0) {
    const int ntb = ((a.N + 127) / 128) * 8;  // token blocks of packed C, padded to whole 128-token tiles
    const char* cbase = reinterpret_cast<const char*>(a.Cpk);
    // column blocks past the end re-read block 0; their rows of T are never stored
    const uint32_t aoff0 = (uint32_t)((cb0 < a.ccb ? cb0 : 0) * 64 + lane) * 16u;
    const uint32_t aoff1 = (uint32_t)((cb0 + 1 < a.ccb ? cb0 + 1 : 0) * 64 + lane) * 16u;
    const int64_t tbrow = (int64_t)a.ccb * 1024;  // bytes per 16-token block of packed C

    // Ring of eight k-blocks' C fragments (16 tokens each): block j multiplies with slot j % 8 and
    // requests token block j + 7 into the slot block j - 1 has just used.  Token blocks follow each
    // other in memory, so the request address just advances; it stops at the last token block of
    // packed C (requests past the split's end are never used).
    u32x4 rc[8][2];
    const char* creq = cbase + (int64_t)(tok_beg / 16) * tbrow;  // uniform
    const char* const clast = cbase + (int64_t)(ntb - 1) * tbrow;
    auto advance = [&]() {
      creq += tbrow;
      if (creq > clast) creq = clast;
    };
#pragma unroll
    for (int kk = 0; kk < 7; ++kk) {
      ring_request<0>(rc[kk][0], aoff0, creq);
      ring_request<0>(rc[kk][1], aoff1, creq);
      advance();
    }
    constexpr int VM = 12;  // requests younger than the ones a block is about to use
#define PRAC_IC(v) std::integral_constant<int, (v)> {}
    auto kblock = [&](auto oc, const u32x4 (&fcur)[4], u32x4 (&fnext)[4], auto kkc, unsigned lds) {
      constexpr int O = decltype(oc)::value, KK = decltype(kkc)::value;
      kblock_ct<O, VM>(acc, fcur, fnext, rc[KK][0], rc[KK][1], lds, rc[(KK + 7) & 7][0], rc[(KK + 7) & 7][1], aoff0,
                       aoff1, creq);
      advance();
    };

    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem_raw +
                          (unsigned)(frag_slot(li, lh) * 16);
    u32x4 fa[4], fb[4];
    __builtin_amdgcn_s_barrier();  // tile 0 is in LDS
    frag_read4_ct(fa, lds0);
    int stage = 0;
    for (int kt = 0; kt < nk; ++kt) {
      const unsigned cur = lds0 + (unsigned)stage * CW_STAGE;
      stage = stage == CW_STAGES - 1 ? 0 : stage + 1;
      const unsigned nxt = lds0 + (unsigned)stage * CW_STAGE;
      kblock(PRAC_IC(4096 * 1), fa, fb, PRAC_IC(0), cur);
      kblock(PRAC_IC(4096 * 2), fb, fa, PRAC_IC(1), cur);
      kblock(PRAC_IC(4096 * 3), fa, fb, PRAC_IC(2), cur);
      kblock(PRAC_IC(4096 * 4), fb, fa, PRAC_IC(3), cur);
      kblock(PRAC_IC(4096 * 5), fa, fb, PRAC_IC(4), cur);
      kblock(PRAC_IC(4096 * 6), fb, fa, PRAC_IC(5), cur);
      kblock(PRAC_IC(4096 * 7), fa, fb, PRAC_IC(6), cur);
      __builtin_amdgcn_s_barrier();
      kblock(PRAC_IC(0), fb, fa, PRAC_IC(7), nxt);
      if (kt == nk - 1) drain_mfma<8, 2>(acc, rc);  // inside the loop, see the compress kernel
    }
#undef PRAC_IC
  }

  // epilogue: acc[4 i + j], register v of lane (li, lh): T row 32 (cb0 + i) + 8*(v/4) + 4*lh + v%4,
  // column n0 + 4 li + j
  PRAC_STAMP(a, 6);
  float* out = a.slabs[h] + (int64_t)split * a.c * mh;
  const int n = n0 + 4 * li;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    asm volatile("" : "+a"(acc[4 * i]), "+a"(acc[4 * i + 1]), "+a"(acc[4 * i + 2]), "+a"(acc[4 * i + 3]) : : "memory");
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = (cb0 + i) * 32 + 8 * (v / 4) + 4 * lh + (v % 4);
      if (row < a.c) {
        float* o = out + (int64_t)row * mh + n;
        if (n + 3 < mh && (mh & 3) == 0) {
          *reinterpret_cast<float4*>(o) =
              make_float4(acc[4 * i][v], acc[4 * i + 1][v], acc[4 * i + 2][v], acc[4 * i + 3][v]);
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (n + j < mh) o[j] = acc[4 * i + j][v];
        }
      }
    }
  }
  }
  if constexpr (MODE != 0) {
    // all eight waves: the slabs of this column tile -> T -> dW (see wgrad_tail)
    const int members = a.splits * a.row_groups;
    wgrad_tail<MODE == 2>(a, smem_raw, tn, h, n0, split * a.row_groups + rg, members);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    PRAC_STAMP(a, 5);
  }
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

int launch_compress_ws(prac_ctx* ctx, const bf16_t* X, int64_t ldx, int N, int d, const bf16_t* Pfrag, int ncb, int c,
                       bf16_t* C, int64_t ldc, bool packed, const bf16_t* Wfrag, int ncb_w, int m, bf16_t* Y,
                       int64_t ldy) {
  if (ldx > PRAC_MAX_STREAM_PITCH) return PRAC_EINVAL;  // callers route wider pitches to the strided kernels
  CompressWsArgs a;
#ifdef PRAC_WS_TIMESTAMPS
  a.stamps = g_ws_stamps;
#endif
  a.X = X; a.ldx = ldx; a.N = N; a.d = d; a.Pfrag = Pfrag; a.ncb = ncb; a.c = c;
  a.C = C; a.ldc = ldc; a.ccb = (c + 31) / 32; a.packed = packed ? 1 : 0;
  a.tiles_m = (N + WS_BM - 1) / WS_BM;
  // with a forward output the wide (64-column) wave tile is used throughout; without one the narrow
  // tile also serves launches whose wide tiles would leave half of the CUs idle (few token rows):
  // twice the workgroups, each with half the multiplications, X reaching the second of a pair from L2
  const int wide_groups = (a.ccb + 7) / 8;
  const int FN = (!Wfrag && (c <= 128 || (int64_t)a.tiles_m * wide_groups * 2 <= ctx->n_cu)) ? 1 : 2;
  // Pfrag == nullptr (only with a forward output): no C part, the launch is a plain Y = X W
  const int p_groups = Pfrag ? (a.ccb + 4 * FN - 1) / (4 * FN) : 0;
  if (p_groups * 4 * FN > ncb || (!Pfrag && !Wfrag)) return PRAC_EINVAL;  // packed basis narrower than assumed
  a.Wfrag = Wfrag; a.ncb_w = ncb_w; a.m = m; a.Y = Y; a.ldy = ldy;
  a.w_groups = Wfrag ? ((m + 31) / 32 + 4 * FN - 1) / (4 * FN) : 0;
  if (a.w_groups * 4 * FN > ncb_w) return PRAC_EINVAL;
  a.col_groups = a.w_groups + p_groups;
  const size_t smem = (size_t)WS_STAGES * WS_STAGE;
  const int total = a.tiles_m * a.col_groups;
  const dim3 grid(((total + 7) / 8) * 8), block(512);
  static bool f1[PRAC_MAX_DEVICES] = {}, f2[PRAC_MAX_DEVICES] = {};  // the attribute is per device
  bool &s1 = f1[ctx->device % PRAC_MAX_DEVICES], &s2 = f2[ctx->device % PRAC_MAX_DEVICES];
  constexpr auto kern1 = compress_ws_kernel<1, WS_NCH, WS_NIF>;
  constexpr auto kern2 = compress_ws_kernel<2, WS_NCH, WS_NIF>;
  if (FN == 1) {
    int rc = set_smem(ctx, kern1, smem, s1);
    if (rc) return rc;
    PRAC_LAUNCH(ctx, kern1, grid, block, smem, a);
  } else {
    int rc = set_smem(ctx, kern2, smem, s2);
    if (rc) return rc;
    PRAC_LAUNCH(ctx, kern2, grid, block, smem, a);
  }
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

int launch_reconstruct_ws(prac_ctx* ctx, const bf16_t* C, int64_t ldc, bool packed, int N, int c, int d,
                          const bf16_t* Ptfrag, int ncb, bf16_t* Xh, int64_t ldxh) {
  if (c < 1 || c > WS_BK || ncb % 8 != 0 || (int64_t)ncb * 32 < d) return PRAC_EINVAL;
  ReconWsArgs a;
  a.C = C; a.ldc = ldc; a.packed = packed ? 1 : 0; a.ccb = (c + 31) / 32; a.N = N; a.c = c; a.d = d; a.Ptfrag = Ptfrag; a.ncb = ncb; a.Xh = Xh; a.ldxh = ldxh;
  a.tiles_m = (N + WS_BM - 1) / WS_BM;
  a.groups = (d + 255) / 256;
  static bool f[PRAC_MAX_DEVICES] = {};
  int rc = set_smem(ctx, reconstruct_ws_kernel, (size_t)RW_SMEM, f[ctx->device % PRAC_MAX_DEVICES]);
  if (rc) return rc;
  PRAC_LAUNCH(ctx, reconstruct_ws_kernel, dim3(((a.tiles_m + 7) / 8) * 8), dim3(512), (size_t)RW_SMEM, a);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

namespace {
void fill_ctdy_args(CtdyWsArgs& a, const bf16_t* Cpk, int c, int N, int n_out, const bf16_t* const* dY, const int64_t* lddy,
                    const int* m, float* const* slabs, int splits) {
  a.Cpk = Cpk; a.ccb = (c + 31) / 32; a.c = c; a.N = N; a.n_out = n_out; a.splits = splits;
  int tiles = 0;
  for (int h = 0; h < n_out; ++h) {
    a.dY[h] = dY[h]; a.lddy[h] = lddy[h]; a.m[h] = m[h]; a.slabs[h] = slabs[h];
    a.tile0[h] = tiles;
    tiles += (m[h] + CW_BN - 1) / CW_BN;
  }
  for (int h = n_out; h <= PRAC_CTDY_MAX_OUT; ++h) a.tile0[h] = tiles;
  const int ktiles = (N + CW_BK - 1) / CW_BK;
  a.tok_per_split = ((ktiles + splits - 1) / splits) * CW_BK;
  a.tiles_n = tiles;
  a.row_groups = (a.ccb + 7) / 8;
}
}  // namespace

int launch_ctdy_ws(prac_ctx* ctx, const bf16_t* Cpk, int c, int N, int n_out, const bf16_t* const* dY,
                   const int64_t* lddy, const int* m, float* const* slabs, int splits) {
  if (n_out < 1 || n_out > PRAC_CTDY_MAX_OUT) return PRAC_EINVAL;
  for (int h = 0; h < n_out; ++h)
    if (lddy[h] > PRAC_MAX_STREAM_PITCH) return PRAC_EINVAL;
  CtdyWsArgs a{};
  fill_ctdy_args(a, Cpk, c, N, n_out, dY, lddy, m, slabs, splits);
  const size_t smem = (size_t)CW_STAGES * CW_STAGE;
  const int total = a.tiles_n * a.row_groups * splits;
  static bool f[PRAC_MAX_DEVICES] = {};
  int rc = set_smem(ctx, ctdy_ws_kernel<0>, smem, f[ctx->device % PRAC_MAX_DEVICES]);
  if (rc) return rc;
  PRAC_LAUNCH(ctx, ctdy_ws_kernel<0>, dim3(((total + 7) / 8) * 8), dim3(512), smem, a);
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

// Token ranges per column tile for the one-launch weight gradient, or 0 where it cannot run: the
// workgroups of a column tile (token ranges x row groups) wait for each other, so all of them must be
// resident - at most one workgroup per compute unit, with the tiles dealt to the 8 XCDs in equal numbers.
int wgrad_fused_splits(int n_cu, int c, int n_out, const int64_t* m, int64_t N, int tune_splits) {
  int64_t tiles = 0;
  for (int h = 0; h < n_out; ++h) tiles += (m[h] + CW_BN - 1) / CW_BN;
  if (tiles > PRAC_SYNC_TILES) return 0;
  const int row_groups = ((c + 31) / 32 + 7) / 8;
  const int64_t gpx = (tiles + 7) / 8;           // column tiles per XCD
  const int cu_per_xcd = n_cu / 8;
  if (gpx * row_groups > cu_per_xcd) return row_groups == 1 ? 1 : 0;  // single-member groups never wait
  int splits = (int)(cu_per_xcd / (gpx * row_groups));
  if (tune_splits > 0) {
    if (tune_splits > splits) return 0;          // the override does not fit: three launches
    splits = tune_splits;
  }
  if (splits > N / 256) splits = (int)(N / 256);
  if (splits > 64) splits = 64;
  return splits < 1 ? 1 : splits;
}

int launch_wgrad_fused(prac_ctx* ctx, const bf16_t* Cpk, int c, int N, int n_out, const bf16_t* const* dY,
                       const int64_t* lddy, const int* m, float* const* slabs, int splits, int k_lo, float scale_hi,
                       int nckb, const int* nmb, bf16_t* const* Tf, const bf16_t* Pa, int d, void* const* dW,
                       const int64_t* lddw, bool out_bf16, float beta, int* cnt) {
  if (n_out < 1 || n_out > PRAC_CTDY_MAX_OUT) return PRAC_EINVAL;
  CtdyWsArgs a{};
  fill_ctdy_args(a, Cpk, c, N, n_out, dY, lddy, m, slabs, splits);
  a.groups_per_xcd = (a.tiles_n + 7) / 8;
  const int per_xcd = a.groups_per_xcd * splits * a.row_groups;
  // refuse a launch whose waiting workgroups might not all be resident
  if (a.tiles_n > PRAC_SYNC_TILES || (splits * a.row_groups > 1 && per_xcd > ctx->n_cu / 8)) return PRAC_EINVAL;
#ifdef PRAC_WS_TIMESTAMPS
  a.stamps = g_ws_stamps;
#endif
  a.cnt = cnt; a.fail = ctx->d_flag; a.nckb = nckb; a.k_lo = k_lo; a.scale_hi = scale_hi; a.Pa = Pa; a.d = d; a.beta = beta;
  for (int h = 0; h < n_out; ++h) {
    a.Tf[h] = Tf[h]; a.nmb[h] = nmb[h]; a.dW[h] = dW[h]; a.lddw[h] = lddw[h];
    a.vec_ok[h] = (reinterpret_cast<uintptr_t>(dW[h]) % 16 == 0 && lddw[h] % (out_bf16 ? 8 : 4) == 0) ? 1 : 0;
  }
  const size_t smem = std::max((size_t)CW_STAGES * CW_STAGE, (size_t)WG_SMEM);
  static bool f1[PRAC_MAX_DEVICES] = {}, f2[PRAC_MAX_DEVICES] = {};
  bool &s1 = f1[ctx->device % PRAC_MAX_DEVICES], &s2 = f2[ctx->device % PRAC_MAX_DEVICES];
  const dim3 grid(8 * per_xcd), block(512);
  if (out_bf16) {
    int rc = set_smem(ctx, ctdy_ws_kernel<2>, smem, s2);
    if (rc) return rc;
    PRAC_LAUNCH(ctx, ctdy_ws_kernel<2>, grid, block, smem, a);
  } else {
    int rc = set_smem(ctx, ctdy_ws_kernel<1>, smem, s1);
    if (rc) return rc;
    PRAC_LAUNCH(ctx, ctdy_ws_kernel<1>, grid, block, smem, a);
  }
  PRAC_HIP_TRY(ctx, hipGetLastError());
  return PRAC_OK;
}

#ifdef PRAC_WS_TIMESTAMPS
extern "C" void prac_debug_set_stamps(void* p) { g_ws_stamps = reinterpret_cast<long long*>(p); }
#endif
