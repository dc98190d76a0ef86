// Device-side helpers of the gfx950 kernels: 16-bit float conversion, vector
// memory access, wave-uniform values.
#pragma once

#include <hip/hip_runtime.h>

#include "kvc_common.h"

namespace kvc {

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Stores of the restored cache and of the frames are written once and not read
// again by these kernels, and loads of frames / KV are read once: both carry the
// non-temporal hint so they do not displace the small reused data (per-channel
// scale/min, block table) from L2.
#ifndef KVC_NT_LOAD
#define KVC_NT_LOAD 1
#endif
#ifndef KVC_NT_STORE
#define KVC_NT_STORE 1
#endif

// Every pointer the kernels see is device global memory; saying so lets the
// compiler emit global_* instead of flat_* accesses for pointers it loaded from
// memory (the per-layer cache bases).
#define KVC_GLOBAL __attribute__((address_space(1)))
// Read-only for the whole kernel (block table, cache base pointers, scale/min on
// the restore side): loads at wave-uniform addresses become scalar loads.
#define KVC_CONST __attribute__((address_space(4)))

template <typename T>
__device__ __forceinline__ const KVC_CONST T* as_const(const T* p) {
  return (const KVC_CONST T*)p;
}

template <typename V>
__device__ __forceinline__ V stream_load(const void* p) {
#if KVC_NT_LOAD
  return __builtin_nontemporal_load((const KVC_GLOBAL V*)p);
#else
  return *(const KVC_GLOBAL V*)p;
#endif
}

template <typename V>
__device__ __forceinline__ void stream_store(void* p, V v) {
#if KVC_NT_STORE
  __builtin_nontemporal_store(v, (KVC_GLOBAL V*)p);
#else
  *(KVC_GLOBAL V*)p = v;
#endif
}

__device__ __forceinline__ uint32_t wave_uniform(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }

// Two binary32 values -> one dword of two fp16 / bf16 values, each rounded to
// nearest even (the default conversion mode).  Built as a 2-vector so the
// compiler can write the two halves of the dword directly.
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

template <int DT>
__device__ __forceinline__ uint32_t narrow_pair(float lo, float hi);
template <>
__device__ __forceinline__ uint32_t narrow_pair<KVC_F16>(float lo, float hi) {
  const f16x2 v = {(_Float16)lo, (_Float16)hi};
  return __builtin_bit_cast(uint32_t, v);
}
template <>
__device__ __forceinline__ uint32_t narrow_pair<KVC_BF16>(float lo, float hi) {
  const bf16x2 v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, v);
}

// fp16 / bf16 bits -> binary32 (exact).
template <int DT>
__device__ __forceinline__ float widen_bits(uint32_t b);
template <>
__device__ __forceinline__ float widen_bits<KVC_F16>(uint32_t b) {
  return (float)__builtin_bit_cast(_Float16, (unsigned short)b);
}
template <>
__device__ __forceinline__ float widen_bits<KVC_BF16>(uint32_t b) {
  return __builtin_bit_cast(float, b << 16);
}

// The two 16-bit values of one dword.
template <int DT>
__device__ __forceinline__ void widen_pair(uint32_t w, float& lo, float& hi) {
  lo = widen_bits<DT>(w & 0xffffu);
  hi = widen_bits<DT>(w >> 16);
}

}  // namespace kvc
