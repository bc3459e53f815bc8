// Device-side helpers shared by the HIP kernels of this library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace taw {

typedef __bf16 bf16_t;
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

// ---- V storage elements moved as one vector; kept packed in registers, unpacked on use -------
// load_nt / store_nt: non-temporal accesses for data streamed through once
// pin(): the compiler must treat the packed value as new from here on, so nothing unpacked from it before stays live
template <typename T, int V> struct Vec;
template <> struct Vec<float, 4> {
  f32x4_t raw;
  __device__ __forceinline__ void load(const float* p) { raw = *reinterpret_cast<const f32x4_t*>(p); }
  __device__ __forceinline__ void store(float* p) const { *reinterpret_cast<f32x4_t*>(p) = raw; }
  __device__ __forceinline__ void load_nt(const float* p) { raw = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p)); }
  __device__ __forceinline__ void store_nt(float* p) const { __builtin_nontemporal_store(raw, reinterpret_cast<f32x4_t*>(p)); }
  __device__ __forceinline__ float get(int i) const { return raw[i]; }
  __device__ __forceinline__ void set(int i, float x) { raw[i] = x; }
  __device__ __forceinline__ void pin() { asm volatile("" : "+v"(raw)); }
};
template <> struct Vec<float, 1> {
  float raw;
  __device__ __forceinline__ void load(const float* p) { raw = *p; }
  __device__ __forceinline__ void store(float* p) const { *p = raw; }
  __device__ __forceinline__ void load_nt(const float* p) { raw = __builtin_nontemporal_load(p); }
  __device__ __forceinline__ void store_nt(float* p) const { __builtin_nontemporal_store(raw, p); }
  __device__ __forceinline__ float get(int) const { return raw; }
  __device__ __forceinline__ void set(int, float x) { raw = x; }
  __device__ __forceinline__ void pin() { asm volatile("" : "+v"(raw)); }
};
template <> struct Vec<bf16_t, 8> {
  bf16x8_t raw;
  __device__ __forceinline__ void load(const bf16_t* p) { raw = *reinterpret_cast<const bf16x8_t*>(p); }
  __device__ __forceinline__ void store(bf16_t* p) const { *reinterpret_cast<bf16x8_t*>(p) = raw; }
  __device__ __forceinline__ void load_nt(const bf16_t* p) { raw = __builtin_nontemporal_load(reinterpret_cast<const bf16x8_t*>(p)); }
  __device__ __forceinline__ void store_nt(bf16_t* p) const { __builtin_nontemporal_store(raw, reinterpret_cast<bf16x8_t*>(p)); }
  __device__ __forceinline__ float get(int i) const { return (float)raw[i]; }
  __device__ __forceinline__ void set(int i, float x) { raw[i] = (bf16_t)x; }
  __device__ __forceinline__ void pin() { asm volatile("" : "+v"(raw)); }
};
template <> struct Vec<bf16_t, 1> {
  bf16_t raw;
  __device__ __forceinline__ void load(const bf16_t* p) { raw = *p; }
  __device__ __forceinline__ void store(bf16_t* p) const { *p = raw; }
  __device__ __forceinline__ void load_nt(const bf16_t* p) { raw = __builtin_nontemporal_load(p); }
  __device__ __forceinline__ void store_nt(bf16_t* p) const { __builtin_nontemporal_store(raw, p); }
  __device__ __forceinline__ float get(int) const { return (float)raw; }
  __device__ __forceinline__ void set(int, float x) { raw = (bf16_t)x; }
  __device__ __forceinline__ void pin() { asm volatile("" : "+v"(raw)); }
};

template <typename T> struct VecWidth;
template <> struct VecWidth<float> { static constexpr int value = 4; };
template <> struct VecWidth<bf16_t> { static constexpr int value = 8; };

// ---- wavefront reductions (64 lanes, xor butterfly: every lane ends with the result) ----------
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}

}  // namespace taw
