// Hand-placed LDS traffic for the software-pipelined kernels.
//
// The kernels stream tiles from global memory straight into LDS (global_load_lds, no staging
// registers) several tiles ahead.  The compiler cannot tell which LDS bytes an in-flight
// global-to-LDS load will write, so before any LDS read it can see it waits for ALL of them,
// which would serialise the prefetch.  The reads of streamed tiles are therefore issued through
// inline assembly and the waits are placed by hand:
//   * vm_wait<N>()      : at most N of this wavefront's global(-to-LDS) loads still in flight
//   * lds_read_*<OFF>() : issue an LDS read (result NOT yet valid)
//   * lgkm_wait<N>(x..) : at most N LDS reads still in flight; the operands are tied to the wait so
//                         no consumer of those registers can be scheduled above it
// Every statement carries a "memory" clobber so global-to-LDS loads and barriers keep their
// program order relative to it.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "tmla_mfma.hpp"

namespace tmla {

typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) char* lds_char_ptr;
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef __attribute__((address_space(1))) const void* glb_void_ptr;

// compile-time unrolled loop: f(std::integral_constant<int, 0>{}), ..., f(<N-1>)
template <int... I, typename F>
__device__ inline void static_for_impl(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ inline void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

// 32-bit LDS byte address of a pointer into shared memory
__device__ inline uint32_t lds_addr(const void* p) {
  return (uint32_t)(uintptr_t)(lds_char_ptr)(p);
}

template <int OFF>
__device__ inline bf16x8 lds_read_b128(uint32_t addr) {
  bf16x8 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return v;
}
// transposing 64-bit read (four 16-bit elements gathered across 16 lanes)
template <int OFF>
__device__ inline short4v lds_read_tr16_b64(uint32_t addr) {
  short4v v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return v;
}

// LDS writes and a float4 read for small exchange buffers next to the streamed tiles (same
// reason for assembly: a compiler-visible LDS access would wait for every transfer in flight)
__device__ inline void lds_write_b32(uint32_t addr, float v) {
  asm volatile("ds_write_b32 %0, %1" ::"v"(addr), "v"(v) : "memory");
}
template <int OFF>
__device__ inline void lds_write_b128(uint32_t addr, bf16x8 v) {
  asm volatile("ds_write_b128 %0, %1 offset:%2" ::"v"(addr), "v"(v), "n"(OFF) : "memory");
}
__device__ inline f32x4 lds_read_f32x4(uint32_t addr) {
  f32x4 v;
  asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr) : "memory");
  return v;
}

template <int N>
__device__ inline void vm_wait() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
template <int N>
__device__ inline void lgkm_wait() {
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
}
template <int N, typename A>
__device__ inline void lgkm_wait(A& a) {
  asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a) : "n"(N) : "memory");
}
template <int N, typename A, typename B>
__device__ inline void lgkm_wait(A& a, B& b) {
  asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N) : "memory");
}
template <int N, typename A, typename B, typename C, typename D>
__device__ inline void lgkm_wait(A& a, B& b, C& c, D& d) {
  asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N) : "memory");
}

// workgroup barrier without the memory fence __syncthreads() implies (the fence would drain the
// prefetched global-to-LDS loads); callers wait for exactly what they need first
__device__ inline void raw_barrier() {
  asm volatile("s_barrier" ::: "memory");
}

// 64 lanes x 16 bytes from per-lane global addresses to 1 KiB of LDS at the wave-uniform `dst`
__device__ inline void dma16(const void* src, void* dst) {
  __builtin_amdgcn_global_load_lds((glb_void_ptr)src, (lds_void_ptr)(lds_char_ptr)dst, 16, 0, 0);
}
// The same for data that one workgroup reads once (a request's own cache rows, the expanded
// prefix of a head): the non-temporal hint keeps the stream from displacing what the caches
// hold.  Measured on MI355X: the HBM-bound kernels stream 11-13 % faster with it (5.8 instead of
// 5.1 TB/s).  Data that every request reads again -- the latent prefix in absorb_only mode,
// the absorbed queries -- keeps the default policy: streamed, the absorb_only pass over a
// 16384-token prefix shared by 512 requests was 30 % slower.
#ifndef TMLA_STREAM_AUX
#define TMLA_STREAM_AUX 2   // aux bit 1 = nt
#endif
__device__ inline void dma16_stream(const void* src, void* dst) {
  __builtin_amdgcn_global_load_lds((glb_void_ptr)src, (lds_void_ptr)(lds_char_ptr)dst, 16, 0,
                                   TMLA_STREAM_AUX);
}

#ifndef TMLA_STREAM_POLICY
#define TMLA_STREAM_POLICY " nt"   // assembly spelling of the non-temporal hint
#endif
// The same (streaming) transfer with the address split into a wave-uniform base (in scalar registers) and a
// 32-bit per-lane offset: no 64-bit vector additions per transfer.  `lds` + `lds2` = wave-uniform
// LDS byte address (two terms so that the sum lands in M0 directly).  The statement sets M0 behind the compiler's back, which is safe only in kernels that
// issue every global-to-LDS transfer through it and use nothing else that reads M0.
template <bool STREAM = true>
__device__ inline void dma16_scalar_base(uint32_t lane_off, const void* base, uint32_t lds,
                                         uint32_t lds2 = 0) {
  // wave-uniform by contract; made explicit so that both live in scalar registers
  const uint64_t u = (uint64_t)base;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
  base = (const void*)(((uint64_t)hi << 32) | lo);
  lds = __builtin_amdgcn_readfirstlane(lds);
  lds2 = __builtin_amdgcn_readfirstlane(lds2);
  if constexpr (STREAM)
    asm volatile("s_add_u32 m0, %2, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" TMLA_STREAM_POLICY
                 ::"v"(lane_off), "s"(base), "s"(lds), "s"(lds2) : "memory", "scc");
  else
    asm volatile("s_add_u32 m0, %2, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 ::"v"(lane_off), "s"(base), "s"(lds), "s"(lds2) : "memory", "scc");
}

// Scalar (SMEM) load of one int from a wave-uniform address.  A vector load here would have to be
// waited for with vmcnt(0), draining the tile prefetch; the scalar cache is only read.
__device__ inline int scalar_load_i32(const int32_t* p) {
  // the address is wave-uniform by contract; make that explicit so it lives in scalar registers
  const uint64_t u = (uint64_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
  p = (const int32_t*)(((uint64_t)hi << 32) | lo);
  int v;
  asm volatile("s_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(p) : "memory");
  return v;
}

__device__ inline bf16x8 join_tr(short4v lo, short4v hi) {
  const short8v both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, both);
}

}  // namespace tmla
