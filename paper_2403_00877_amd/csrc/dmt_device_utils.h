// Small device helpers: 16-byte chunk decode / encode for the three element
// types, round-to-nearest-even float -> 16-bit conversions.
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dmt.h"

namespace dmt {

template <int DT> struct EltBytes { static constexpr int value = (DT == DMT_F32) ? 4 : 2; };
// elements in one 16-byte chunk
template <int DT> struct ChunkElems { static constexpr int value = 16 / EltBytes<DT>::value; };

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;   // NaN stays NaN
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;         // ties to even
}

__device__ __forceinline__ uint32_t f32_to_f16_bits(float x) {
  return (uint32_t)__half_as_ushort(__float2half_rn(x));
}

__device__ __forceinline__ float f16_bits_to_f32(uint32_t h) {
  return __half2float(__ushort_as_half((unsigned short)h));
}

template <int DT> __device__ __forceinline__ uint32_t pack2(float a, float b);
template <> __device__ __forceinline__ uint32_t pack2<DMT_F16>(float a, float b) {
  return f32_to_f16_bits(a) | (f32_to_f16_bits(b) << 16);
}
template <> __device__ __forceinline__ uint32_t pack2<DMT_BF16>(float a, float b) {
  return f32_to_bf16_bits(a) | (f32_to_bf16_bits(b) << 16);
}

template <int DT> __device__ __forceinline__ void unpack2(uint32_t u, float& a, float& b);
template <> __device__ __forceinline__ void unpack2<DMT_F16>(uint32_t u, float& a, float& b) {
  a = f16_bits_to_f32(u & 0xffffu);
  b = f16_bits_to_f32(u >> 16);
}
template <> __device__ __forceinline__ void unpack2<DMT_BF16>(uint32_t u, float& a, float& b) {
  a = bf16_lo(u);
  b = bf16_hi(u);
}

// acc += the elements of one 16-byte chunk, as float32.
template <int DT>
__device__ __forceinline__ void accumulate_chunk(float (&acc)[ChunkElems<DT>::value], uint4 v) {
  if constexpr (DT == DMT_F32) {
    acc[0] += __uint_as_float(v.x);
    acc[1] += __uint_as_float(v.y);
    acc[2] += __uint_as_float(v.z);
    acc[3] += __uint_as_float(v.w);
  } else {
    float a, b;
    unpack2<DT>(v.x, a, b); acc[0] += a; acc[1] += b;
    unpack2<DT>(v.y, a, b); acc[2] += a; acc[3] += b;
    unpack2<DT>(v.z, a, b); acc[4] += a; acc[5] += b;
    unpack2<DT>(v.w, a, b); acc[6] += a; acc[7] += b;
  }
}

template <int DT>
__device__ __forceinline__ void decode_chunk(float (&x)[ChunkElems<DT>::value], uint4 v) {
#pragma unroll
  for (int q = 0; q < ChunkElems<DT>::value; ++q) x[q] = 0.f;
  accumulate_chunk<DT>(x, v);
}

// Store N floats (N = 4 or 8) as OD elements starting at element offset `off`
// of `base`.  `off` is a multiple of N.
template <int OD, int N>
__device__ __forceinline__ void store_chunk(void* base, int64_t off, const float (&a)[N]) {
  if constexpr (OD == DMT_F32) {
    float4* o = (float4*)((float*)base + off);
    o[0] = make_float4(a[0], a[1], a[2], a[3]);
    if constexpr (N == 8) o[1] = make_float4(a[4], a[5], a[6], a[7]);
  } else {
    uint16_t* o = (uint16_t*)base + off;
    if constexpr (N == 8) {
      *(uint4*)o = make_uint4(pack2<OD>(a[0], a[1]), pack2<OD>(a[2], a[3]),
                              pack2<OD>(a[4], a[5]), pack2<OD>(a[6], a[7]));
    } else {
      *(uint2*)o = make_uint2(pack2<OD>(a[0], a[1]), pack2<OD>(a[2], a[3]));
    }
  }
}

// Loads / stores that tell the caches the line will not be reused (streaming
// row traffic must not evict data that is gathered repeatedly).
typedef float dmt_f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int dmt_u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int dmt_u32x4 __attribute__((ext_vector_type(4)));

// Table rows, states and the other tensors the kernels stream live in global memory.  A
// pointer that was read from a descriptor in memory or rebuilt from an integer has lost that
// fact and would be accessed with flat instructions (which also occupy the LDS path): these
// casts give it back.
#define DMT_GLOBAL __attribute__((address_space(1)))

__device__ __forceinline__ float4 nt_load(const float4* p) {
  const dmt_f32x4 v = __builtin_nontemporal_load((const DMT_GLOBAL dmt_f32x4*)p);
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void nt_store(float4 v, float4* p) {
  dmt_f32x4 t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, (DMT_GLOBAL dmt_f32x4*)p);
}
__device__ __forceinline__ uint2 nt_load(const uint2* p) {
  const dmt_u32x2 v = __builtin_nontemporal_load((const DMT_GLOBAL dmt_u32x2*)p);
  return make_uint2(v.x, v.y);
}
__device__ __forceinline__ void nt_store(uint2 v, uint2* p) {
  dmt_u32x2 t = {v.x, v.y};
  __builtin_nontemporal_store(t, (DMT_GLOBAL dmt_u32x2*)p);
}
__device__ __forceinline__ uint4 nt_load(const uint4* p) {
  const dmt_u32x4 v = __builtin_nontemporal_load((const DMT_GLOBAL dmt_u32x4*)p);
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void nt_store(uint4 v, uint4* p) {
  dmt_u32x4 t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, (DMT_GLOBAL dmt_u32x4*)p);
}

__device__ __forceinline__ float nt_load(const float* p) {
  return __builtin_nontemporal_load((const DMT_GLOBAL float*)p);
}
__device__ __forceinline__ void nt_store(float v, float* p) {
  __builtin_nontemporal_store(v, (DMT_GLOBAL float*)p);
}

// Plain loads / stores of global memory through a pointer of unknown address space.
typedef float dmt_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float4 gload(const float4* p) {
  const dmt_f32x4 v = *(const DMT_GLOBAL dmt_f32x4*)p;
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void gstore(float4 v, float4* p) {
  dmt_f32x4 t = {v.x, v.y, v.z, v.w};
  *(DMT_GLOBAL dmt_f32x4*)p = t;
}
__device__ __forceinline__ float2 gload(const float2* p) {
  const dmt_f32x2 v = *(const DMT_GLOBAL dmt_f32x2*)p;
  return make_float2(v.x, v.y);
}
__device__ __forceinline__ void gstore(float2 v, float2* p) {
  dmt_f32x2 t = {v.x, v.y};
  *(DMT_GLOBAL dmt_f32x2*)p = t;
}
__device__ __forceinline__ uint4 gload(const uint4* p) {
  const dmt_u32x4 v = *(const DMT_GLOBAL dmt_u32x4*)p;
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint2 gload(const uint2* p) {
  const dmt_u32x2 v = *(const DMT_GLOBAL dmt_u32x2*)p;
  return make_uint2(v.x, v.y);
}
__device__ __forceinline__ void gstore(uint2 v, uint2* p) {
  dmt_u32x2 t = {v.x, v.y};
  *(DMT_GLOBAL dmt_u32x2*)p = t;
}
__device__ __forceinline__ float gload(const float* p) { return *(const DMT_GLOBAL float*)p; }
__device__ __forceinline__ void gstore(float v, float* p) { *(DMT_GLOBAL float*)p = v; }
__device__ __forceinline__ uint32_t gload(const uint32_t* p) { return *(const DMT_GLOBAL uint32_t*)p; }
__device__ __forceinline__ void gstore(uint32_t v, uint32_t* p) { *(DMT_GLOBAL uint32_t*)p = v; }
__device__ __forceinline__ uint16_t gload(const uint16_t* p) { return *(const DMT_GLOBAL uint16_t*)p; }
__device__ __forceinline__ void gstore(uint16_t v, uint16_t* p) { *(DMT_GLOBAL uint16_t*)p = v; }

}  // namespace dmt

namespace dmt {

// Inclusive prefix sum over the 64 lanes of a wave.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    uint32_t t = __shfl_up(v, o);
    if (lane >= o) v += t;
  }
  return v;
}

// Exclusive prefix sum over a block of NW waves (NW*64 threads); `total`
// receives the block sum in every thread.  `smem` holds NW + 1 words.  Ends with
// a barrier, so `smem` may be reused right after.
template <int NW>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* smem,
                                                         uint32_t& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t incl = wave_inclusive_scan(v);
  if (lane == 63) smem[wave] = incl;
  __syncthreads();
  uint32_t before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    const uint32_t s = smem[w];
    if (w < wave) before += s;
    all += s;
  }
  __syncthreads();
  total = all;
  return before + incl - v;
}

}  // namespace dmt
