// Small device-side helpers shared by the gfx950 kernels: vector types, LDS address-space casts, buffer descriptors,
// the asynchronous global -> LDS copy and explicit wait counters.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tbp {

typedef __bf16 bf16_t;
typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))
#define LDS_AS __attribute__((address_space(3)))
typedef LDS_AS unsigned char lds_u8;

constexpr unsigned kOob = 0x80000000u;     // byte offset beyond every descriptor: the access delivers zero / is dropped

// Buffer descriptor of a window of `bytes` bytes (at most 2 GiB - 1) starting at p, held in scalar registers
// (readfirstlane makes the workgroup-uniform address provably uniform for the compiler).
__device__ __forceinline__ u32x4 make_desc(const void* p, uint32_t bytes = 0x7fffffffu) {
  const uint64_t a = reinterpret_cast<uint64_t>(p);
  u32x4 d;
  d[0] = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)a);
  d[1] = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
  d[2] = (uint32_t)__builtin_amdgcn_readfirstlane(bytes);
  d[3] = 0x00020000u;
  return d;
}

// The same window as a resource value for the compiler's buffer load / store builtins (register destinations: the
// compiler tracks those with its own wait counters).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes = 0x7fffffffu) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// Asynchronous global -> LDS copy of 16 bytes per lane: lane i's data lands at lds_base + 16*i (lds_base is
// wave-uniform and goes through M0).  The copy is tracked by the vector-memory counter only; it is written as
// inline assembly so that the compiler's wait insertion does not drain every copy in flight before each LDS read.
__device__ __forceinline__ void dma16(uint32_t lds_base, u32x4 desc, uint32_t voff) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :: "s"(lds_base), "v"(voff), "s"(desc) : "memory");
}

// The same with 4 bytes per lane: lane i's dword lands at lds_base + 4*i.
__device__ __forceinline__ void dma4(uint32_t lds_base, u32x4 desc, uint32_t voff) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dword %1, %2, 0 offen lds"
               :: "s"(lds_base), "v"(voff), "s"(desc) : "memory");
}

// Store of 8 bytes per lane that the compiler does not track: a workgroup barrier after it then does not wait for the
// write to be acknowledged (the compiler's barrier waits for every vector-memory operation it knows to be in flight).
// For data that nobody reads before the kernel ends.  soff is wave-uniform.
__device__ __forceinline__ void store8_async(u32x2 data, u32x4 desc, uint32_t voff, uint32_t soff) {
  asm volatile("buffer_store_dwordx2 %0, %1, %2, %3 offen" :: "v"(data), "v"(voff), "s"(desc), "s"(soff) : "memory");
}

// The same with 16 bytes per lane.
__device__ __forceinline__ void store16_async(u32x4 data, u32x4 desc, uint32_t voff, uint32_t soff) {
  asm volatile("buffer_store_dwordx4 %0, %1, %2, %3 offen" :: "v"(data), "v"(voff), "s"(desc), "s"(soff) : "memory");
}

template <int N> __device__ __forceinline__ void wait_vmem() {   // at most N vector-memory operations outstanding
  __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

}  // namespace tbp
