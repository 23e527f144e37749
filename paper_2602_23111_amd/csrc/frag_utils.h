// Device-side helpers shared by the streaming kernels: MFMA fragment types, bf16 rounding
// and 16-byte chunk masking.
#pragma once

#include "prac_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
// 16-byte register value: a native vector (assignments of HIP's u32x4 struct lower to
// memcpy, which keeps whole register sets in scratch memory)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

static __device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  // round to nearest even; NaN keeps its payload's top bits and is made quiet (branch-free)
  const uint32_t u = __float_as_uint(f);
  const uint32_t rounded = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
  const uint32_t quiet = (u >> 16) | 0x40u;
  return (bf16_t)((u & 0x7fffffffu) > 0x7f800000u ? quiet : rounded);
}
static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

// Two fp32 -> packed bf16 with the hardware conversion of gfx950 (v_cvt_pk_bf16_f32: round to
// nearest even, NaN stays NaN); `lo` lands in the low half.
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
static __device__ __forceinline__ uint32_t pack2_hw(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  union {
    bf16x2_t b;
    uint32_t u;
  } c;
  c.b = __builtin_convertvector(v, bf16x2_t);
  return c.u;
}

// Keep the first n (0..8) bf16 of a 16-byte chunk, zero the rest.
static __device__ __forceinline__ u32x4 keep_first(u32x4 v, int n) {
  v.x &= (n > 0 ? 0x0000FFFFu : 0u) | (n > 1 ? 0xFFFF0000u : 0u);
  v.y &= (n > 2 ? 0x0000FFFFu : 0u) | (n > 3 ? 0xFFFF0000u : 0u);
  v.z &= (n > 4 ? 0x0000FFFFu : 0u) | (n > 5 ? 0xFFFF0000u : 0u);
  v.w &= (n > 6 ? 0x0000FFFFu : 0u) | (n > 7 ? 0xFFFF0000u : 0u);
  return v;
}

// Output a kernel does not read again is stored with the non-temporal hint: it streams out to memory
// instead of staying dirty in L2 until the write-back at the kernel's end, behind which the kernel's
// completion waits (measured at N = 32768, d = m = 2048: 2 us per step for the 17 MB of C, 1 us for dW;
// the 134 MB of the reconstruction are the opposite case, 54 against 46 us, and keep plain stores).
// Inputs that are read once (X, dY, the partial sums) are loaded with the same hint, which keeps the
// operand every workgroup shares (P, C) in L2.
template <typename V>
static __device__ __forceinline__ void stream_store(V* dst, V v) {
  __builtin_nontemporal_store(v, dst);
}

static __device__ __forceinline__ bf16x8 as_frag(u32x4 v) {
  union {
    u32x4 u;
    bf16x8 f;
  } c;
  c.u = v;
  return c.f;
}

// A kernel's arguments sit in memory no cache holds yet when its first waves start, and the compiler
// fetches them where they are first used: a few dependent rounds of scalar loads, each to another
// 64-byte line, each a full memory round trip before the first byte of data can be requested.  This
// asks for one word of every line of the first BYTES argument bytes at once and waits for them: one
// round trip, after which the compiler's own loads hit the scalar cache.  The workgroup index is handed
// through, so that everything computed from it (all of a kernel's set-up) is ordered after the wait.
template <int BYTES>
static __device__ __forceinline__ int touch_kernel_args(int block_index) {
  const auto ka = __builtin_amdgcn_kernarg_segment_ptr();
  uint32_t t0, t1, t2, t3, t4, t5;
  static_assert(BYTES > 0 && BYTES <= 384, "six lines at most");
  constexpr int L1 = BYTES > 64 ? 64 : 0, L2 = BYTES > 128 ? 128 : 0, L3 = BYTES > 192 ? 192 : 0,
                L4 = BYTES > 256 ? 256 : 0, L5 = BYTES > 320 ? 320 : 0;
  asm volatile(
      "s_load_dword %0, %7, 0x0\n"
      "s_load_dword %1, %7, %8\n"
      "s_load_dword %2, %7, %9\n"
      "s_load_dword %3, %7, %10\n"
      "s_load_dword %4, %7, %11\n"
      "s_load_dword %5, %7, %12\n"
      "s_waitcnt lgkmcnt(0)\n"
      : "=&s"(t0), "=&s"(t1), "=&s"(t2), "=&s"(t3), "=&s"(t4), "=&s"(t5), "+s"(block_index)
      : "s"(ka), "n"(L1), "n"(L2), "n"(L3), "n"(L4), "n"(L5)
      : "memory");
  return block_index;
}

