// Small device helpers shared by the two matrix-core prefix kernels.
#pragma once

#include "common.h"

namespace specext {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float floatx2;
typedef __attribute__((ext_vector_type(4))) float floatx4;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef __attribute__((ext_vector_type(4))) short shortx4;
typedef __attribute__((ext_vector_type(8))) short shortx8;
typedef __attribute__((ext_vector_type(4))) uint32_t uintx4;
typedef __attribute__((ext_vector_type(2))) uint32_t uintx2;
typedef __attribute__((ext_vector_type(2))) _Float16 halfx2;
typedef __attribute__((address_space(3))) shortx4 lds_shortx4;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(3))) uintx4 lds_uintx4;

// The running reference of a row only moves when a tile's max exceeds it by more
// than this many powers of two, so exp2(s - ref) stays below 2^kLazyLog2.
constexpr float kLazyLog2 = 10.f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Lanes l and l+32 exchange through v_permlane32_swap (no LDS access, so no wait on
// the LDS queue): of the two results one holds the lower half's values in both halves,
// the other the upper half's.
__device__ __forceinline__ float halves_sum(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float halves_max(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// 8 consecutive accumulator values -> 8 bf16 (round to nearest even)
__device__ __forceinline__ bf16x8 pack8(const floatx16& v, int first) {
  bf16x8 out;
#pragma unroll
  for (int e = 0; e < 8; e += 2) {
    floatx2 f = {v[first + e], v[first + e + 1]};
    bf16x2 b = __builtin_convertvector(f, bf16x2);
    out[e] = b[0];
    out[e + 1] = b[1];
  }
  return out;
}

// One direct global->LDS load: every lane moves 16 bytes from (base + voff) to LDS
// byte (lds_dst + 16 * lane).  Issued through inline assembly on purpose: the
// compiler then does not know that LDS is written and leaves the waiting to the
// caller's explicit s_waitcnt instead of draining the whole load queue (and with it
// the prefetch of later tiles) before the next LDS read.  s_nop covers the
// wait state the hardware wants between a scalar write of M0 and its use here.
__device__ __forceinline__ void load_to_lds_16(unsigned lds_dst, unsigned voff, const unsigned char* base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_dst), "v"(voff), "s"(base) : "memory", "m0");
}
// The same with the streaming hint (the line is the first to leave the caches again), for bytes that are read once:
// the K/V stream of the verification prefix kernel runs 4 % faster with it (measured against no hint and against the
// device- and system-scope bits, alone and combined with it).
__device__ __forceinline__ void load_to_lds_16_stream(unsigned lds_dst, unsigned voff, const unsigned char* base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
               :: "s"(lds_dst), "v"(voff), "s"(base) : "memory", "m0");
}

// s_waitcnt vmcnt(n) for a run-time even n in [0, 24]
__device__ __forceinline__ void wait_vmcnt_even(int n) {
  switch (n >> 1) {
    case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    case 1: asm volatile("s_waitcnt vmcnt(2)" ::: "memory"); break;
    case 2: asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); break;
    case 3: asm volatile("s_waitcnt vmcnt(6)" ::: "memory"); break;
    case 4: asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); break;
    case 5: asm volatile("s_waitcnt vmcnt(10)" ::: "memory"); break;
    case 6: asm volatile("s_waitcnt vmcnt(12)" ::: "memory"); break;
    case 7: asm volatile("s_waitcnt vmcnt(14)" ::: "memory"); break;
    case 8: asm volatile("s_waitcnt vmcnt(16)" ::: "memory"); break;
    case 9: asm volatile("s_waitcnt vmcnt(18)" ::: "memory"); break;
    case 10: asm volatile("s_waitcnt vmcnt(20)" ::: "memory"); break;
    case 11: asm volatile("s_waitcnt vmcnt(22)" ::: "memory"); break;
    default: asm volatile("s_waitcnt vmcnt(24)" ::: "memory"); break;
  }
}

// 16 bytes written / read at device scope (two 8-byte relaxed atomics: the accesses go to
// the point where the compute units of all XCDs agree, past the per-XCD L2 caches, so a
// workgroup on another XCD reads what was written without cache write-backs or invalidations)
__device__ __forceinline__ void store_device_scope_16(void* dst, const uintx4 v) {
  uint64_t* d = static_cast<uint64_t*>(dst);
  __hip_atomic_store(d, static_cast<uint64_t>(v[0]) | (static_cast<uint64_t>(v[1]) << 32), __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(d + 1, static_cast<uint64_t>(v[2]) | (static_cast<uint64_t>(v[3]) << 32), __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uintx4 load_device_scope_16(const void* src) {
  const uint64_t* s = static_cast<const uint64_t*>(src);
  const uint64_t a = __hip_atomic_load(s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const uint64_t b = __hip_atomic_load(s + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return uintx4{static_cast<uint32_t>(a), static_cast<uint32_t>(a >> 32), static_cast<uint32_t>(b),
                static_cast<uint32_t>(b >> 32)};
}
__device__ __forceinline__ void store_device_scope_8(void* dst, const floatx2 v) {
  __hip_atomic_store(static_cast<uint64_t*>(dst),
                     static_cast<uint64_t>(__float_as_uint(v[0])) | (static_cast<uint64_t>(__float_as_uint(v[1])) << 32),
                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ floatx2 load_device_scope_8(const void* src) {
  const uint64_t a = __hip_atomic_load(static_cast<const uint64_t*>(src), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return floatx2{__uint_as_float(static_cast<uint32_t>(a)), __uint_as_float(static_cast<uint32_t>(a >> 32))};
}

// workgroup barrier that the compiler may not move LDS accesses across
__device__ __forceinline__ void lds_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

}  // namespace specext
